"""GPU parity of the review forward through the C ABI against the CPU oracle.

Tolerances are the ones the task states: |gpu - oracle| <= 1e-4 (+1e-4 relative) for the fp32
configuration and <= 1e-2 + 2e-2 |oracle| for bf16 configurations, element by element on
logits; token decisions are compared through csd_accept on identical probabilities elsewhere.
"""
import os

import numpy as np
import pytest
import torch

import csd_inputs as I
from gpu_util import import_synthetic_kv, make_pair, prefill_both, tol_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2312_11462_amd as P
    P.lib()


def _dev(x, dtype=torch.int32):
    return torch.as_tensor(np.asarray(x), dtype=dtype).cuda()


def _check_block(gm, om, block, cache_len, rtol, atol, what, trace_tol=None):
    block = np.asarray(block, np.int32)
    B, m = block.shape
    L, d = gm.shape.n_layers, gm.shape.d_model
    tr = torch.zeros((L + 1, B * m, d), dtype=torch.float32, device="cuda")
    gm.set_trace(tr)
    lg, pr = gm.verify_block(_dev(block), _dev(cache_len), want_probs=True)
    gm.set_trace(None)
    ref, refp, otr = om.verify_block(block, cache_len, want_probs=True, trace=True)
    if trace_tol is not None:      # residual stream of sequence 0 after the embedding and after every layer
        g = tr.cpu().numpy()[:, :m, :].astype(np.float64)
        for l in range(L + 1):
            rel = np.linalg.norm(g[l] - otr[l]) / np.linalg.norm(otr[l])
            assert rel < trace_tol, f"{what}: residual stream after layer {l}: relative error {rel}"
    ok, err = tol_ok(lg.cpu().numpy().astype(np.float64), ref, rtol, atol)
    assert ok, f"{what}: logits max abs err {err}"
    okp, errp = tol_ok(pr.cpu().numpy().astype(np.float64), refp, 5 * rtol, 1e-6)
    assert okp, f"{what}: probs max abs err {errp}"
    return err


def test_tiny_fp32_config_prefix_then_block():
    """Configuration 1: tiny fp32 decoder, 32-token prefix in the cache, k = 4 drafts."""
    wl = I.WORKLOADS["tiny"]
    shape, seed = wl["shape"], wl["seed"]
    gm, om = make_pair(shape, seed, 1, 64, 8)
    prefix = I.token_ids(33, shape.vocab, seed, 1)
    prefill_both(gm, om, prefix[:32][None], 8)
    from oracle import csd_oracle as O
    table = O.bigram_fit(prefix.numpy(), shape.vocab, I.default_next_table(shape.vocab, seed).numpy())
    draft, _ = O.bigram_draft(prefix.numpy(), [33], table, 4)
    block = np.concatenate([prefix[-1:].numpy(), draft[0]])[None]
    err = _check_block(gm, om, block, [32], 1e-4, 1e-4, "tiny", 1e-5)
    # the cache rows written by the block and by the prefill agree with the oracle's
    for l in range(shape.n_layers):
        K, V = gm.kv_read(l, 0, 0, 37)
        Ko, Vo = om.kv_read(l, 0, 0, 37)
        assert np.abs(K.cpu().numpy() - Ko).max() < 1e-4 and np.abs(V.cpu().numpy() - Vo).max() < 1e-4
    print("tiny max err", err)


def test_fp32_ragged_shapes_batch_and_block_vs_incremental():
    """Odd sizes on the generic path: d, F, V not multiples of the tile sizes; batch of 3 with
    different cache lengths; and the block result equals one-row-at-a-time on the GPU itself."""
    shape = I.ModelShape("odd", 0, "fp32", 2, 48, 3, 16, 100, 301)
    gm, om = make_pair(shape, 5, 3, 80, 7, std=0.1)
    toks = I.token_ids(3 * 40, shape.vocab, 5, 1).reshape(3, 40)
    prefill_both(gm, om, toks[:, :21], 7)
    # ragged: sequence b keeps only 21 - 3b rows committed
    cl = [21, 18, 15]
    block = np.stack([toks[b, cl[b]:cl[b] + 6].numpy() for b in range(3)])
    _check_block(gm, om, block, cl, 1e-4, 1e-4, "ragged batch")
    one = []
    for i in range(6):
        lg = gm.verify_block(_dev(block[:, i:i + 1].copy()), _dev([c + i for c in cl]))
        one.append(lg.cpu().numpy())
    whole = gm.verify_block(_dev(block), _dev(cl)).cpu().numpy()
    assert np.abs(np.concatenate(one, axis=1) - whole).max() < 1e-4


BF = I.ModelShape("bf_small", 0, "bf16", 2, 256, 4, 64, 512, 1024)
BF128 = I.ModelShape("bf_dh128", 0, "bf16", 2, 256, 2, 128, 512, 1024)


@pytest.mark.parametrize("gemm,attn,path", [("generic", "generic", "multikernel"), ("mfma", "generic", "multikernel"),
                                            ("mfma", "mfma", "multikernel"), ("mfma", "mfma", "default")])
@pytest.mark.parametrize("shape", [BF, BF128], ids=["dh64", "dh128"])
def test_bf16_paths_small_model(shape, gemm, attn, path):
    """Several key chunks and a ragged tail (prefix 200 = 128 + 72 keys; 5 and 13 block rows);
    every forward implementation against the oracle: generic kernels, the per-operation MFMA
    kernels, and the forward with the epilogues inside its GEMM kernels (the default for blocks of up to
    32 rows: the 10-row block with one row tile, the 26-row block with two)."""
    os.environ["CSD_GEMM"], os.environ["CSD_ATTN"], os.environ["CSD_PATH"] = gemm, attn, path
    try:
        gm, om = make_pair(shape, 7, 2, 300, 16, std=0.05)
    finally:
        del os.environ["CSD_GEMM"], os.environ["CSD_ATTN"], os.environ["CSD_PATH"]
    assert gm.path(2, 5) == (1 if path == "default" else 0) and gm.path(2, 13) == (1 if path == "default" else 0)
    toks = I.token_ids(2 * 260, shape.vocab, 7, 1).reshape(2, 260)
    prefill_both(gm, om, toks[:, :200], 16)
    e1 = _check_block(gm, om, toks[:, 200:205].numpy(), [200, 200], 2e-2, 1e-2, f"{gemm}/{attn} m=5", 5e-3)
    e2 = _check_block(gm, om, toks[:, 190:203].numpy(), [190, 187], 2e-2, 1e-2, f"{gemm}/{attn} m=13 ragged", 5e-3)
    print(shape.name, gemm, attn, path, "max err", e1, e2)


def test_many_calls_in_a_row_give_the_same_logits():
    """400 back-to-back calls on a small model (the attention kernel's arrival counters must be back at zero
    after every launch): every call returns the first call's logits, and those match the oracle."""
    gm, om = make_pair(BF, 11, 1, 128, 8, std=0.05)
    assert gm.path(1, 5) == 1
    toks = I.token_ids(64, BF.vocab, 11, 1).reshape(1, 64)
    prefill_both(gm, om, toks[:, :40], 8)
    _check_block(gm, om, toks[:, 40:45].numpy(), [40], 2e-2, 1e-2, "first call")
    block, clen = _dev(toks[:, 40:45].numpy()), _dev([40])
    first = gm.verify_block(block, clen).clone()
    for _ in range(400):
        assert torch.equal(gm.verify_block(block, clen), first)


def test_bf16_block_of_17_rows_two_row_tiles():
    gm, om = make_pair(BF, 9, 1, 200, 17, std=0.05)
    toks = I.token_ids(160, BF.vocab, 9, 1).reshape(1, 160)
    prefill_both(gm, om, toks[:, :130], 17)
    _check_block(gm, om, toks[:, 130:147].numpy(), [130], 2e-2, 1e-2, "m=17")


WIDE = I.ModelShape("bf_wide_blocks", 0, "bf16", 2, 256, 4, 64, 576, 1040)


@pytest.mark.parametrize("B,m", [(4, 5), (4, 9), (4, 13), (4, 17), (8, 12), (8, 14), (8, 16), (8, 17), (10, 16), (12, 17)])
def test_bf16_blocks_of_2_to_13_row_tiles_workgroup_tiled_gemms(B, m):
    """B * m = 20 ... 204 rows: two row tiles on the forward with in-kernel epilogues, every row-tile count of the
    row-split GEMM (33 to 144 rows: 3 to 9 row tiles, two or three per compute wave), and two blocks that go in row
    chunks of 128 (160 rows = 128 + 32, the rest on the GEMM that shares activations through LDS; 204 = 128 + 76);
    the FFN width (18 k-steps) leaves ragged chunk tails and the vocabulary (65 column tiles) a ragged last workgroup."""
    gm, om = make_pair(WIDE, 17, B, 96, 17, std=0.05)
    assert gm.path(B, m) == (1 if B * m <= 32 else 0)
    toks = I.token_ids(B * 64, WIDE.vocab, 17, 1).reshape(B, 64)
    prefill_both(gm, om, toks[:, :32], 16)
    cl = [32 - (b % 3) for b in range(B)]                  # ragged cache lengths
    blocks = np.stack([toks[b, cl[b]:cl[b] + m].numpy() for b in range(B)])
    err = _check_block(gm, om, blocks, cl, 2e-2, 1e-2, f"B={B} m={m}")
    print("rows", B * m, "max err", err)
    # the K-split partial sums are reduced in a fixed order: a second run gives the same bits
    a = gm.verify_block(_dev(blocks), _dev(cl)).cpu().numpy().copy()
    b = gm.verify_block(_dev(blocks), _dev(cl)).cpu().numpy()
    assert np.array_equal(a, b)


@pytest.mark.parametrize("path", [None, "multikernel"])
def test_draft160m_config_synthetic_cache(path):
    """Configuration 2: 160M-shaped bf16 model, 512 cached rows (seeded stand-in K/V, since the
    oracle needs minutes to prefill them), k = 8 drafts from the Max-Gram model; on the default forward
    and on the per-operation kernels."""
    wl = I.WORKLOADS["draft160m"]
    shape, seed = wl["shape"], wl["seed"]
    if path:
        os.environ["CSD_PATH"] = path
    try:
        gm, om = make_pair(shape, seed, 1, 640, 16)
    finally:
        os.environ.pop("CSD_PATH", None)
    assert gm.path(1, 9) == (0 if path else 1)
    import_synthetic_kv(gm, om, shape, 512, seed)
    import paper_2312_11462_amd as P
    prefix = I.repeat_stream(513, shape.vocab, seed, 1)
    table = P.bigram_fit(prefix.cuda(), shape.vocab, I.default_next_table(shape.vocab, seed).cuda())
    draft, _ = P.bigram_draft(prefix.cuda(), _dev([513]), table, 8)
    block = torch.cat([prefix[-1:].cuda(), draft[0]])[None].cpu().numpy()
    err = _check_block(gm, om, block, [512], 2e-2, 1e-2, "160M", 5e-3)
    print("160M max err", err)


def test_run_to_run_determinism():
    gm, _ = make_pair(BF, 11, 2, 300, 16, std=0.05)
    toks = I.token_ids(2 * 150, BF.vocab, 11, 1).reshape(2, 150)
    cl = _dev([0, 0])
    outs = []
    for _ in range(2):
        for pos in range(0, 144, 16):
            lg = gm.verify_block(toks[:, pos:pos + 16].contiguous().cuda(), cl + pos)
        outs.append(lg.cpu().numpy().copy())
    assert np.array_equal(outs[0], outs[1])


@pytest.mark.parametrize("shape", [BF, I.ModelShape("odd", 0, "fp32", 2, 48, 3, 16, 100, 301)], ids=["bf16_V1024", "fp32_V301"])
def test_verify_accept_equals_the_two_calls(shape):
    """csd_verify_accept (every row normalised, tested and its replacement drawn in one launch, probabilities
    written only on request) decides exactly as csd_verify_block + csd_accept on the written probabilities, and as
    the oracle's accept rule on those probabilities (Section 2, Section 3.1), for one-hot and dense draft
    distributions, several lenience values and temperatures, in both modes; the probabilities it writes on request
    are those of csd_verify_block bit for bit.  The second shape has a vocabulary that is not a multiple of 4."""
    import paper_2312_11462_amd as P
    from oracle import csd_oracle as O
    BF = shape
    gm, _ = make_pair(BF, 13, 2, 128, 8, std=0.05 if shape.dtype == "bf16" else 0.1)
    toks = I.token_ids(2 * 70, BF.vocab, 13, 1).reshape(2, 70)
    for pos in range(0, 64, 8):
        gm.verify_block(toks[:, pos:pos + 8].contiguous().cuda(), _dev([pos, pos]))
    block = toks[:, 64:70].contiguous().cuda()
    cl = _dev([64, 64])
    draft = block[:, 1:].contiguous()
    n_checked = 0
    for case, (mode, dense, lenience, temperature) in enumerate(
            [(0, False, 1.0, 1.0), (1, False, 1.0, 1.0), (0, True, 1.0, 1.0), (0, True, 3.0, 0.7), (0, True, 1.0, 1.6),
             (1, True, 2.0, 1.0), (0, True, 1.5, 1.0)]):
        u_acc = I.uniforms(10, 13, 20 + case).reshape(2, 5).contiguous().cuda()
        u_s = I.uniforms(2, 13, 40 + case).cuda()
        lg, pr = gm.verify_block(block, cl, want_probs=True, temperature=temperature)
        q = None
        if dense:      # a draft distribution close to the reviewer's, so that acceptance really depends on u
            noise = torch.from_numpy(np.random.default_rng(case).normal(0, 0.5, (2, 5, BF.vocab)).astype(np.float32)).cuda()
            q = pr[:, :5] * torch.exp(noise)
            q = (q / q.sum(-1, keepdim=True)).contiguous()
        uses_probs = mode == 0 or lenience > 1.0
        a = P.accept(pr if uses_probs else lg, q, draft, u_acc, u_s, lenience=lenience, mode=mode)
        b = gm.verify_accept(block, cl, u_acc, u_s, q=q, temperature=temperature, lenience=lenience, mode=mode)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]), (case, a, b)
        o = O.accept((pr if uses_probs else lg).cpu().numpy(), None if q is None else q.cpu().numpy(), draft.cpu().numpy(),
                     u_acc.cpu().numpy(), u_s.cpu().numpy(), lenience, mode)
        assert np.array_equal(o[0], b[0].cpu().numpy()) and np.array_equal(o[1], b[1].cpu().numpy()), (case, o, b)
        pr2 = torch.empty_like(pr)
        c = gm.verify_accept(block, cl, u_acc, u_s, q=q, temperature=temperature, lenience=lenience, mode=mode, probs=pr2)
        assert torch.equal(c[0], b[0]) and torch.equal(c[1], b[1]) and torch.equal(pr2, pr), case
        n_checked += int(b[0].sum())
    assert n_checked > 10          # drafts were kept, so later rows and their statistics took part


@pytest.mark.parametrize("B,m", [(1, 1), (3, 1), (3, 16), (5, 12)])
def test_verify_accept_block_shapes_one_row_to_sixteen(B, m):
    """The fused call at the edges of its launch shape: no drafts at all (m = 1: only the extra token is drawn), full
    16-row blocks, several sequences with ragged cache lengths; decisions equal csd_verify_block + csd_accept and the
    oracle's rule on the same probabilities, in both modes, one-hot and dense drafts."""
    import paper_2312_11462_amd as P
    from oracle import csd_oracle as O
    gm, _ = make_pair(BF, 21, B, 128, 16, std=0.05)
    toks = I.token_ids(B * 100, BF.vocab, 21, 1).reshape(B, 100)
    for pos in range(0, 64, 16):
        gm.verify_block(toks[:, pos:pos + 16].contiguous().cuda(), _dev([pos] * B))
    cl_host = [64 - 3 * b for b in range(B)]
    block = torch.stack([toks[b, cl_host[b]:cl_host[b] + m] for b in range(B)]).contiguous().cuda()
    cl = _dev(cl_host)
    k = m - 1
    draft = block[:, 1:].contiguous()
    for case, (mode, dense) in enumerate([(0, False), (0, True), (1, False)]):
        u_acc = I.uniforms(B * max(k, 1), 21, 60 + case).reshape(B, max(k, 1))[:, :k].contiguous().cuda()
        u_s = I.uniforms(B, 21, 80 + case).cuda()
        lg, pr = gm.verify_block(block, cl, want_probs=True)
        q = None
        if dense and k > 0:
            noise = torch.from_numpy(np.random.default_rng(case).normal(0, 0.5, (B, k, BF.vocab)).astype(np.float32)).cuda()
            q = pr[:, :k] * torch.exp(noise)
            q = (q / q.sum(-1, keepdim=True)).contiguous()
        src = pr if mode == 0 else lg
        a = P.accept(src, q, draft, u_acc, u_s, mode=mode)
        b = gm.verify_accept(block, cl, u_acc, u_s, q=q, mode=mode)
        assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1]), (case, a, b)
        o = O.accept(src.cpu().numpy(), None if q is None else q.cpu().numpy(), draft.cpu().numpy().reshape(B, k),
                     u_acc.cpu().numpy().reshape(B, k), u_s.cpu().numpy(), 1.0, mode)
        assert np.array_equal(o[0], b[0].cpu().numpy()) and np.array_equal(o[1], b[1].cpu().numpy()), (case, o, b)


def test_argument_errors_enqueue_nothing():
    import paper_2312_11462_amd as P
    gm, _ = make_pair(I.TINY, 1, 1, 64, 8)
    with pytest.raises(P.CsdError):
        gm.verify_block(_dev(np.zeros((1, 9))), _dev([0]))          # m > max_block
    with pytest.raises(P.CsdError):
        gm.verify_block(_dev(np.zeros((2, 4))), _dev([0, 0]))       # B > max_batch
    with pytest.raises(P.CsdError):
        gm.kv_write(0, 0, 60, torch.zeros((8, 64)).cuda(), torch.zeros((8, 64)).cuda())
