"""Pins of the oracle's T5-style decoder forward (arch 1; CPU only).

The paper names the FLAN-T5 family as reviewers (Section 5.1) and fixes nothing else, so the forward
is pinned to what the architecture's own definition and the mathematics fix: hand-computed bucket
values of the relative-position bias (identity below 16, logarithmic spacing up to 128), library
routines on a whole sequence, closed forms of degenerate weights that isolate the sign and direction
of the bias, the cross-attention and the gated activation, and the cache invariants.
"""
import math

import numpy as np
import torch
import torch.nn.functional as F

import csd_inputs as I
from oracle import csd_oracle as O

SHAPE = I.ModelShape("t5pin", 1, "fp32", 2, 32, 4, 8, 48, 40, rms_eps=1e-6, enc_len=9)
EPS = float(np.float32(SHAPE.rms_eps))


def _weights(shape=SHAPE, seed=13, std=0.3, **override):
    w = I.make_weights(shape, seed, std=std)
    names = I.weight_names(shape)
    for i, t in enumerate(w):
        if t.ndim == 1:       # non-trivial gains so that a dropped gain is visible
            w[i] = (1.0 + 0.1 * I.normal(t.shape, 1.0, seed, 900 + i)).contiguous()
        if names[i] == "rel_bias":   # a bias large enough to matter
            w[i] = I.normal(t.shape, 1.0, seed, 777).contiguous()
    for key, val in override.items():
        for i, n in enumerate(names):
            if n.endswith(key):
                w[i] = torch.full_like(w[i], val) if not torch.is_tensor(val) else val.clone()
    return w


def test_bucket_values_fixed_by_the_definition():
    # exact buckets for distances below 16
    assert [O.rel_bucket(n) for n in range(16)] == list(range(16))
    # 16 + floor(16 * log8(n / 16)), worked by hand: log8(17/16) = 0.029, log8(2) = 1/3, log8(4) = 2/3,
    # log8(127/16) = 0.9962, log8(8) = 1 (capped to the last bucket)
    by_hand = {16: 16, 17: 16, 18: 16, 19: 17, 31: 21, 32: 21, 33: 21, 34: 21, 63: 26, 64: 26, 90: 29, 91: 29,
               127: 31, 128: 31, 129: 31, 5000: 31}
    assert {n: O.rel_bucket(n) for n in by_hand} == by_hand
    b = [O.rel_bucket(n) for n in range(300)]
    assert all(x <= y for x, y in zip(b, b[1:])) and sorted(set(b)) == list(range(32))
    # bucket edges from the inverse of the definition: bucket 16 + j starts at ceil(16 * 8^(j/16))
    for j in range(1, 16):
        edge = math.ceil(16 * 8 ** (j / 16) - 1e-9)
        assert O.rel_bucket(edge) == 16 + j and O.rel_bucket(edge - 1) == 16 + j - 1


def _torch_forward(shape, w, tokens, enc):
    """Whole-sequence forward without a cache from library routines, fp64."""
    names = I.weight_names(shape)
    W = {n: t.double() for n, t in zip(names, w)}
    T, H, dh, d = len(tokens), shape.n_heads, shape.head_dim, shape.d_model
    h = W["embed"][torch.tensor(tokens)]
    encd = torch.as_tensor(enc, dtype=torch.float64)
    dist = torch.arange(T)[:, None] - torch.arange(T)[None, :]            # query - key
    bucket = torch.tensor([[O.rel_bucket(int(n)) if n >= 0 else 0 for n in row] for row in dist])
    bias = W["rel_bias"][bucket].permute(2, 0, 1)                          # [H][T][T]
    causal = torch.full((T, T), float("-inf"), dtype=torch.float64).triu(1)
    for l in range(shape.n_layers):
        a = F.rms_norm(h, (d,), W[f"l{l}.self_norm"], EPS)
        q = (a @ W[f"l{l}.wq"]).view(T, H, dh).transpose(0, 1)
        k = (a @ W[f"l{l}.wk"]).view(T, H, dh).transpose(0, 1)
        v = (a @ W[f"l{l}.wv"]).view(T, H, dh).transpose(0, 1)
        o = F.scaled_dot_product_attention(q, k, v, attn_mask=bias + causal, scale=1.0)
        h = h + o.transpose(0, 1).reshape(T, H * dh) @ W[f"l{l}.wo"]
        a = F.rms_norm(h, (d,), W[f"l{l}.cross_norm"], EPS)
        q = (a @ W[f"l{l}.cq"]).view(T, H, dh).transpose(0, 1)
        k = (encd @ W[f"l{l}.ck"]).view(-1, H, dh).transpose(0, 1)
        v = (encd @ W[f"l{l}.cv"]).view(-1, H, dh).transpose(0, 1)
        o = F.scaled_dot_product_attention(q, k, v, scale=1.0)
        h = h + o.transpose(0, 1).reshape(T, H * dh) @ W[f"l{l}.co"]
        a = F.rms_norm(h, (d,), W[f"l{l}.ffn_norm"], EPS)
        h = h + (F.gelu(a @ W[f"l{l}.w0"], approximate="tanh") * (a @ W[f"l{l}.w1"])) @ W[f"l{l}.w_out"]
    a = F.rms_norm(h, (d,), W["final_norm"], EPS)
    return (a @ W["lm_head"]).numpy()


def _oracle_run(shape, w, tokens, enc, chunk):
    m = O.Model(shape, w, max_batch=1, max_seq=len(tokens) + 4, max_block=chunk)
    m.cross_kv_init(enc[None])
    outs = []
    for pos in range(0, len(tokens), chunk):
        blk = tokens[pos:pos + chunk]
        outs.append(m.verify_block(np.array([blk], np.int32), np.array([pos], np.int32))[0])
    return np.concatenate(outs, axis=0)


def test_matches_library_routines_whole_sequence():
    w = _weights()
    tokens = I.token_ids(27, SHAPE.vocab, 5, 1).tolist()     # distances up to 26: exact and logarithmic buckets
    enc = I.encoder_output(SHAPE, 1, 5)[0].numpy()
    ref = _torch_forward(SHAPE, w, tokens, enc)
    got = _oracle_run(SHAPE, w, tokens, enc, chunk=27)
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-9)


def test_block_equals_incremental_and_chunked_prefill():
    w = _weights()
    tokens = I.token_ids(21, SHAPE.vocab, 6, 1).tolist()
    enc = I.encoder_output(SHAPE, 1, 6)[0].numpy()
    whole = _oracle_run(SHAPE, w, tokens, enc, chunk=21)
    for chunk in (1, 4, 8):
        np.testing.assert_allclose(_oracle_run(SHAPE, w, tokens, enc, chunk), whole, rtol=1e-9, atol=1e-9)


def test_closed_form_all_sublayers_silenced():
    # wo = co = w_out = 0: the residual stream stays the embedding
    w = _weights(wo=0.0, co=0.0, w_out=0.0)
    names = I.weight_names(SHAPE)
    W = {n: t.double().numpy() for n, t in zip(names, w)}
    tokens = [3, 9, 9, 1]
    enc = I.encoder_output(SHAPE, 1, 1)[0].numpy()
    got = _oracle_run(SHAPE, w, tokens, enc, chunk=4)
    e = W["embed"][tokens]
    a = e / np.sqrt((e * e).mean(-1, keepdims=True) + EPS) * W["final_norm"]
    np.testing.assert_allclose(got, a @ W["lm_head"], rtol=1e-10, atol=1e-10)


def test_closed_form_bias_selects_the_distance():
    """A bias table that is 0 in one bucket and -1e9 elsewhere makes every row attend exactly the key at
    that distance (rows with no such key: the nearest allowed... so only rows that have one are checked):
    pins the sign of the bias, which side the distance is measured from and that it is added before the
    softmax.  Cross-attention and the FFN are silenced; one layer."""
    shape = I.ModelShape("t5one", 1, "fp32", 1, 32, 4, 8, 48, 40, rms_eps=1e-6, enc_len=5)
    for dist in (0, 1, 3):
        bias = torch.full((32, shape.n_heads), -1e9)
        bias[dist] = 0.0
        w = _weights(shape, co=0.0, w_out=0.0, rel_bias=bias)
        names = I.weight_names(shape)
        W = {n: t.double().numpy() for n, t in zip(names, w)}
        tokens = I.token_ids(9, shape.vocab, 8, 2).tolist()
        enc = I.encoder_output(shape, 1, 2)[0].numpy()
        got = _oracle_run(shape, w, tokens, enc, chunk=9)
        e = W["embed"][tokens]
        a = e / np.sqrt((e * e).mean(-1, keepdims=True) + EPS) * W["l0.self_norm"]
        v = a @ W["l0.wv"]
        for i in range(dist, len(tokens)):
            h = e[i] + v[i - dist] @ W["l0.wo"]
            x = h / np.sqrt((h * h).mean() + EPS) * W["final_norm"]
            np.testing.assert_allclose(got[i], x @ W["lm_head"], rtol=1e-8, atol=1e-8)


def test_closed_form_cross_attention_over_identical_encoder_rows():
    """All encoder rows equal: whatever the queries are, cross-attention returns that row's value
    projection.  Self-attention and the FFN are silenced; one layer."""
    shape = I.ModelShape("t5one", 1, "fp32", 1, 32, 4, 8, 48, 40, rms_eps=1e-6, enc_len=5)
    w = _weights(shape, wo=0.0, w_out=0.0)
    names = I.weight_names(shape)
    W = {n: t.double().numpy() for n, t in zip(names, w)}
    row = I.normal((shape.d_model,), 1.0, 3, 5).numpy()
    enc = np.tile(row, (shape.enc_len, 1))
    tokens = [4, 4, 17, 2]
    got = _oracle_run(shape, w, tokens, enc, chunk=4)
    e = W["embed"][tokens]
    h = e + (row.astype(np.float64) @ W["l0.cv"]) @ W["l0.co"]
    a = h / np.sqrt((h * h).mean(-1, keepdims=True) + EPS) * W["final_norm"]
    np.testing.assert_allclose(got, a @ W["lm_head"], rtol=1e-9, atol=1e-9)


def test_cross_attention_is_not_masked_and_ignores_encoder_row_order_only_jointly():
    """Permuting the encoder rows permutes keys and values together: the output must not change
    (no positional term, no mask on the encoder side)."""
    w = _weights()
    tokens = I.token_ids(6, SHAPE.vocab, 9, 1).tolist()
    enc = I.encoder_output(SHAPE, 1, 9)[0].numpy()
    a = _oracle_run(SHAPE, w, tokens, enc, chunk=6)
    b = _oracle_run(SHAPE, w, tokens, enc[::-1].copy(), chunk=6)
    np.testing.assert_allclose(a, b, rtol=1e-9, atol=1e-9)


def test_bf16_configuration_stores_cross_keys_and_values_in_bf16():
    shape = I.ModelShape("t5bf", 1, "bf16", 1, 32, 4, 8, 48, 40, rms_eps=1e-6, enc_len=5)
    w = I.make_weights(shape, 4, std=0.3)
    m = O.Model(shape, w, max_batch=1, max_seq=8, max_block=4)
    enc = I.encoder_output(shape, 1, 4).numpy()
    m.cross_kv_init(enc)
    hd = shape.n_heads * shape.head_dim
    self_elems = 2 * shape.n_layers * 1 * 8 * hd
    cross = m.kv[self_elems:self_elems + shape.enc_len * hd].reshape(shape.enc_len, hd)
    names = I.weight_names(shape)
    ck = w[names.index("l0.ck")].double()
    want = (torch.as_tensor(enc[0], dtype=torch.float64) @ ck).float().bfloat16().double().numpy()
    np.testing.assert_array_equal(cross, want)
