"""Pins of the oracle's review forward (CPU only).

The paper fixes nothing about the decoder beyond naming model families (Section 5.1), so the
forward is pinned to library routines, closed forms of degenerate weights and invariants:
a mistake in the mask, the scale, the rotary pairing, a residual or a transposed weight
fails at least one of them.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import csd_inputs as I
from oracle import csd_oracle as O

SHAPE = I.ModelShape("pin", 0, "fp32", 2, 32, 4, 8, 48, 40)
EPS = float(np.float32(SHAPE.rms_eps))   # the model configuration carries eps as an fp32


def _weights(shape=SHAPE, seed=11, std=0.3, **override):
    w = I.make_weights(shape, seed, std=std)
    # non-trivial norm gains so that a dropped gain is visible
    for i, t in enumerate(w):
        if t.ndim == 1:
            w[i] = (1.0 + 0.1 * I.normal(t.shape, 1.0, seed, 900 + i)).contiguous()
    names = I.weight_names(shape)
    for key, val in override.items():
        for i, n in enumerate(names):
            if n.endswith(key):
                w[i] = torch.full_like(w[i], val)
    return w


def _torch_forward(shape, w, tokens, kv_bf16=False):
    """Whole-sequence forward without a cache, from library routines, in fp64.  With kv_bf16 the
    keys and values pass through the library's bf16 conversion, as a bf16 cache stores them."""
    names = I.weight_names(shape)
    W = {n: t.double() for n, t in zip(names, w)}
    T = len(tokens)
    H, dh = shape.n_heads, shape.head_dim
    h = W["embed"][torch.tensor(tokens)]
    pos = torch.arange(T, dtype=torch.float64)
    inv = shape.rope_theta ** (-torch.arange(0, dh, 2, dtype=torch.float64) / dh)
    ang = torch.polar(torch.ones(T, dh // 2, dtype=torch.float64), pos[:, None] * inv[None, :])

    def rot(x):      # x [T][H][dh]; rotation as a complex multiply on (x_j, x_{j+dh/2})
        z = torch.complex(x[..., : dh // 2], x[..., dh // 2:]) * ang[:, None, :]
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(shape.n_layers):
        a = F.rms_norm(h, (shape.d_model,), W[f"l{l}.attn_norm"], EPS)
        q = rot((a @ W[f"l{l}.wq"]).view(T, H, dh)).transpose(0, 1)
        k = rot((a @ W[f"l{l}.wk"]).view(T, H, dh)).transpose(0, 1)
        v = (a @ W[f"l{l}.wv"]).view(T, H, dh).transpose(0, 1)
        if kv_bf16:
            k, v = k.float().bfloat16().double(), v.float().bfloat16().double()
        o = F.scaled_dot_product_attention(q, k, v, is_causal=True).transpose(0, 1).reshape(T, H * dh)
        h = h + o @ W[f"l{l}.wo"]
        a = F.rms_norm(h, (shape.d_model,), W[f"l{l}.ffn_norm"], EPS)
        h = h + (F.silu(a @ W[f"l{l}.w_gate"]) * (a @ W[f"l{l}.w_up"])) @ W[f"l{l}.w_down"]
    a = F.rms_norm(h, (shape.d_model,), W["final_norm"], EPS)
    return (a @ W["lm_head"]).numpy()


def _oracle_full(shape, w, tokens, chunk):
    m = O.Model(shape, w, max_batch=1, max_seq=len(tokens) + 4, max_block=chunk)
    outs = []
    for pos in range(0, len(tokens), chunk):
        blk = tokens[pos:pos + chunk]
        outs.append(m.verify_block(np.array([blk], np.int32), np.array([pos], np.int32))[0])
    return np.concatenate(outs, axis=0), m


def test_matches_library_routines_whole_sequence():
    w = _weights()
    tokens = I.token_ids(23, SHAPE.vocab, 3, 1).tolist()
    ref = _torch_forward(SHAPE, w, tokens)
    got, _ = _oracle_full(SHAPE, w, tokens, chunk=23)
    np.testing.assert_allclose(got, ref, rtol=1e-10, atol=1e-10)


def test_bf16_configuration_widens_weights_exactly_and_stores_kv_as_bf16():
    """bf16 configurations: the weights are bf16 values widened exactly, and the KV cache holds
    bf16 values (the configuration's storage type), everything else stays fp64.  The reference
    rounds K and V with the library's conversion; a cache left unrounded differs visibly."""
    shape = I.ModelShape("pinb", 0, "bf16", 2, 32, 4, 8, 48, 40)
    w = _weights(shape)
    w = [t.to(torch.bfloat16) if t.ndim == 2 else t for t in w]
    tokens = I.token_ids(9, shape.vocab, 4, 1).tolist()
    ref = _torch_forward(shape, [t.float() for t in w], tokens, kv_bf16=True)
    got, m = _oracle_full(shape, w, tokens, chunk=4)
    np.testing.assert_allclose(got, ref, rtol=1e-9, atol=1e-9)
    unrounded = _torch_forward(shape, [t.float() for t in w], tokens, kv_bf16=False)
    assert np.abs(unrounded - ref).max() > 1e-5
    K, V = m.kv_read(1, 0, 0, 9)
    assert np.array_equal(K, torch.tensor(K).float().bfloat16().double().numpy())
    assert np.array_equal(V, torch.tensor(V).float().bfloat16().double().numpy())


def test_round_to_bf16_ties_to_even_and_is_not_double_rounded():
    """kv_write rounds fp32 inputs to the cache type: exact ties go to the even significand."""
    shape = I.ModelShape("pinb", 0, "bf16", 1, 32, 4, 8, 48, 40)
    m = O.Model(shape, [t.to(torch.bfloat16) if t.ndim == 2 else t for t in _weights(shape)],
                max_batch=1, max_seq=8, max_block=4)
    vals = np.zeros((1, 32), np.float32)
    vals[0, :6] = [1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, -(1.0 + 2.0 ** -8), 3.1415926, 1e-30]
    m.kv_write(0, 0, 0, vals, vals)
    K, _ = m.kv_read(0, 0, 0, 1)
    want = torch.tensor(vals).bfloat16().double().numpy()
    assert np.array_equal(K, want)
    assert K[0, 0] == 1.0 and K[0, 1] == 1.0 + 2.0 ** -6 and K[0, 2] == 1.0 + 2.0 ** -7


@pytest.mark.parametrize("chunk", [1, 4, 7])
def test_block_equals_incremental_and_cache_equals_no_cache(chunk):
    """Reviewing a block in one run equals feeding its tokens one at a time, and a cached
    prefix gives the same logits as a forward over prefix + block from an empty cache."""
    w = _weights()
    tokens = I.token_ids(19, SHAPE.vocab, 5, 1).tolist()
    whole, _ = _oracle_full(SHAPE, w, tokens, chunk=19)
    parts, _ = _oracle_full(SHAPE, w, tokens, chunk=chunk)
    np.testing.assert_allclose(parts, whole, rtol=1e-11, atol=1e-12)


def test_stale_cache_rows_are_overwritten():
    """Rows past the committed length are rewritten by the next block: reviewing a rejected
    draft first must not change the result of the next review."""
    w = _weights()
    tokens = I.token_ids(12, SHAPE.vocab, 6, 1).tolist()
    clean, _ = _oracle_full(SHAPE, w, tokens, chunk=12)
    m = O.Model(SHAPE, w, max_batch=1, max_seq=32, max_block=8)
    m.verify_block(np.array([tokens[:6]], np.int32), np.array([0], np.int32))
    m.verify_block(np.array([[1, 2, 3, 4, 5]], np.int32), np.array([6], np.int32))   # rejected drafts
    got = m.verify_block(np.array([tokens[6:]], np.int32), np.array([6], np.int32))[0]
    np.testing.assert_allclose(got, clean[6:], rtol=1e-12, atol=1e-13)


def test_closed_form_no_mixing_layers():
    """With W_o = 0 and W_down = 0 the residual stream is the embedding, so
    logits = rmsnorm(E[token]) * g_final @ W_lm, whatever the position."""
    w = _weights(wo=0.0, w_down=0.0)
    names = I.weight_names(SHAPE)
    W = {n: t.double().numpy() for n, t in zip(names, w)}
    tokens = [3, 17, 3, 39]
    got, _ = _oracle_full(SHAPE, w, tokens, chunk=4)
    for i, t in enumerate(tokens):
        x = W["embed"][t]
        a = x / np.sqrt(np.mean(x * x) + EPS) * W["final_norm"]
        np.testing.assert_allclose(got[i], a @ W["lm_head"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(got[0], got[2], rtol=0, atol=0)


def test_closed_form_uniform_attention_is_causal_mean():
    """One layer, W_q = 0: all scores are equal, so attention returns the mean of the value
    rows over exactly the visible positions 0..i; checks the mask and the V/W_o path."""
    shape = I.ModelShape("pin1", 0, "fp32", 1, 32, 4, 8, 48, 40)
    w = _weights(shape, wq=0.0, w_down=0.0)
    names = I.weight_names(shape)
    W = {n: t.double().numpy() for n, t in zip(names, w)}
    tokens = I.token_ids(7, shape.vocab, 8, 1).tolist()
    got, _ = _oracle_full(shape, w, tokens, chunk=3)

    def norm(x, g):
        return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + EPS) * g

    h = W["embed"][tokens]
    v = norm(h, W["l0.attn_norm"]) @ W["l0.wv"]
    mean_v = np.cumsum(v, axis=0) / np.arange(1, len(tokens) + 1)[:, None]
    h = h + mean_v @ W["l0.wo"]
    ref = norm(h, W["final_norm"]) @ W["lm_head"]
    np.testing.assert_allclose(got, ref, rtol=1e-11, atol=1e-12)


def test_single_token_attention_returns_its_own_value():
    """t = 0, m = 1: softmax over one key is 1, so the layer output has a closed form that
    does not involve q, k or the rotary embedding at all."""
    shape = I.ModelShape("pin1", 0, "fp32", 1, 32, 4, 8, 48, 40)
    w = _weights(shape)
    names = I.weight_names(shape)
    W = {n: t.double().numpy() for n, t in zip(names, w)}
    got, _ = _oracle_full(shape, w, [5], chunk=1)

    def norm(x, g):
        return x / np.sqrt(np.mean(x * x) + EPS) * g

    h = W["embed"][5]
    h = h + (norm(h, W["l0.attn_norm"]) @ W["l0.wv"]) @ W["l0.wo"]
    a = norm(h, W["l0.ffn_norm"])
    g = a @ W["l0.w_gate"]
    h = h + ((g / (1 + np.exp(-g))) * (a @ W["l0.w_up"])) @ W["l0.w_down"]
    np.testing.assert_allclose(got[0], norm(h, W["final_norm"]) @ W["lm_head"], rtol=1e-12, atol=1e-13)


def test_rope_is_a_rotation_with_relative_phase():
    rng = np.random.default_rng(0)
    dh = 16
    q, k = rng.normal(size=dh), rng.normal(size=dh)
    # norm preserving, identity at position 0
    np.testing.assert_allclose(O.rope(q, 0), q, atol=0)
    np.testing.assert_allclose(np.linalg.norm(O.rope(q, 37)), np.linalg.norm(q), rtol=1e-14)
    # q.k depends on the position difference only
    a = O.rope(q, 9) @ O.rope(k, 4)
    b = O.rope(q, 105) @ O.rope(k, 100)
    np.testing.assert_allclose(a, b, rtol=1e-12)
    # pair (j, j+dh/2) turns by pos * theta^(-2j/dh): check one pair against cos/sin
    e = np.zeros(dh)
    e[3] = 1.0
    r = O.rope(e, 5, theta=10000.0)
    ang = 5 * 10000.0 ** (-2 * 3 / dh)
    np.testing.assert_allclose([r[3], r[3 + dh // 2]], [np.cos(ang), np.sin(ang)], rtol=1e-14)
    assert np.count_nonzero(r) == 2


def test_rmsnorm_and_softmax_against_library():
    rng = np.random.default_rng(1)
    x = rng.normal(size=50)
    g = rng.normal(size=50).astype(np.float32)
    ref = F.rms_norm(torch.tensor(x), (50,), torch.tensor(g).double(), 1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), ref, rtol=1e-13)
    lg = rng.normal(size=33) * 5
    np.testing.assert_allclose(O.softmax(lg, 0.7), torch.softmax(torch.tensor(lg) / 0.7, 0).numpy(), rtol=1e-13)
    assert abs(O.softmax(lg).sum() - 1) < 1e-14


def test_equal_tokens_without_position_signal_give_equal_rows():
    """All tokens equal and W_q = W_k = 0: no row can tell its position, so all rows agree."""
    w = _weights(wq=0.0, wk=0.0)
    got, _ = _oracle_full(SHAPE, w, [7] * 6, chunk=6)
    for i in range(1, 6):
        np.testing.assert_allclose(got[i], got[0], rtol=1e-12, atol=1e-13)


def test_batch_rows_are_independent():
    w = _weights()
    t0 = I.token_ids(8, SHAPE.vocab, 9, 1).tolist()
    t1 = I.token_ids(8, SHAPE.vocab, 9, 2).tolist()
    m = O.Model(SHAPE, w, max_batch=2, max_seq=16, max_block=8)
    both = m.verify_block(np.array([t0, t1], np.int32), np.array([0, 0], np.int32))
    one, _ = _oracle_full(SHAPE, w, t1, chunk=8)
    np.testing.assert_allclose(both[1], one, rtol=0, atol=0)


def test_kv_write_read_roundtrip_and_use():
    """A cache filled through kv_write behaves like one filled by the forward itself."""
    w = _weights()
    tokens = I.token_ids(10, SHAPE.vocab, 10, 1).tolist()
    whole, m0 = _oracle_full(SHAPE, w, tokens, chunk=10)
    m1 = O.Model(SHAPE, w, max_batch=1, max_seq=14, max_block=10)
    for l in range(SHAPE.n_layers):
        K, V = m0.kv_read(l, 0, 0, 6)
        m1.kv_write(l, 0, 0, K, V)   # through fp32: tolerance below
    got = m1.verify_block(np.array([tokens[6:]], np.int32), np.array([6], np.int32))[0]
    np.testing.assert_allclose(got, whole[6:], rtol=1e-5, atol=1e-6)
