"""GPU parity of the T5-style decoder reviewer (arch 1, the encoder-decoder family of Section 5.1;
benchmark configuration 4) against the CPU oracle: fp32 on the generic kernels, bf16 on every
GEMM / attention kernel combination with a prefix long enough that look-back distances pass 128
(the last bias bucket), and the configuration's full shape with seeded stand-in self-attention
cache rows (the oracle cannot prefill 256 rows of a 24-layer 4096-wide model in test time)."""
import os

import numpy as np
import pytest
import torch

import csd_inputs as I
from gpu_util import import_synthetic_kv, make_pair, prefill_both, tol_ok

pytestmark = pytest.mark.gpu


def _dev(a, dtype=torch.int32):
    return torch.as_tensor(np.asarray(a), dtype=dtype).cuda()


def _cross_init(gm, om, shape, B, seed):
    enc = I.encoder_output(shape, B, seed)
    gm.cross_kv_init(enc.cuda())
    om.cross_kv_init(enc.numpy())


def _check(gm, om, block, cache_len, rtol, atol, what):
    lg = gm.verify_block(_dev(block), _dev(cache_len))
    ref = om.verify_block(np.asarray(block), np.asarray(cache_len))
    ok, err = tol_ok(lg.cpu().numpy().astype(np.float64), ref, rtol, atol)
    assert ok, f"{what}: max abs err {err}"
    return err


def test_t5_tiny_fp32_generic_kernels():
    shape = I.T5_TINY
    gm, om = make_pair(shape, 21, 2, 64, 8, std=0.1)
    _cross_init(gm, om, shape, 2, 21)
    toks = I.token_ids(2 * 40, shape.vocab, 21, 1).reshape(2, 40)
    prefill_both(gm, om, toks[:, :24], 8)
    e1 = _check(gm, om, toks[:, 24:29].numpy(), [24, 24], 1e-4, 1e-4, "t5 tiny m=5")
    e2 = _check(gm, om, toks[:, 20:27].numpy(), [20, 17], 1e-4, 1e-4, "t5 tiny ragged m=7")
    print("t5 tiny max err", e1, e2)


BF_T5 = I.ModelShape("t5_bf_small", 1, "bf16", 2, 256, 4, 64, 512, 1024, rms_eps=1e-6, enc_len=96)


@pytest.mark.parametrize("gemm,attn,path", [("generic", "generic", "multikernel"), ("mfma", "generic", "multikernel"),
                                            ("mfma", "mfma", "multikernel"), ("mfma", "mfma", "default")])
def test_t5_bf16_small_every_kernel_combination(gemm, attn, path):
    """Prefix of 200 rows: distances beyond 128 share the last bias bucket; 96 encoder rows are not a
    multiple of the 128-key attention chunk; 5 and 13 block rows (one and two row tiles), the second call ragged.
    The last combination is the forward with the epilogues inside its GEMM kernels (the default)."""
    os.environ["CSD_GEMM"], os.environ["CSD_ATTN"], os.environ["CSD_PATH"] = gemm, attn, path
    try:
        gm, om = make_pair(BF_T5, 23, 2, 300, 16, std=0.05)
    finally:
        del os.environ["CSD_GEMM"], os.environ["CSD_ATTN"], os.environ["CSD_PATH"]
    assert gm.path(2, 5) == (1 if path == "default" else 0)
    _cross_init(gm, om, BF_T5, 2, 23)
    toks = I.token_ids(2 * 260, BF_T5.vocab, 23, 1).reshape(2, 260)
    prefill_both(gm, om, toks[:, :200], 16)
    e1 = _check(gm, om, toks[:, 200:205].numpy(), [200, 200], 2e-2, 1e-2, f"t5 {gemm}/{attn} m=5")
    e2 = _check(gm, om, toks[:, 190:203].numpy(), [190, 187], 2e-2, 1e-2, f"t5 {gemm}/{attn} m=13 ragged")
    print("t5 bf16", gemm, attn, "max err", e1, e2)


@pytest.mark.parametrize("B,m", [(3, 13), (3, 17)])
def test_t5_bf16_blocks_of_39_and_51_rows_row_split_gemm(B, m):
    """More than 32 rows: the per-operation kernels with the GEMM that splits the rows over its waves (two row
    tiles per wave, the fourth wave without rows), the cross-attention over 96 encoder rows and, at 17 rows per
    sequence, a second row tile in both attentions; ragged cache lengths."""
    gm, om = make_pair(BF_T5, 29, B, 300, 17, std=0.05)
    assert gm.path(B, m) == 0
    _cross_init(gm, om, BF_T5, B, 29)
    toks = I.token_ids(B * 260, BF_T5.vocab, 29, 1).reshape(B, 260)
    prefill_both(gm, om, toks[:, :160], 16)
    cl = [160 - 3 * b for b in range(B)]
    block = np.stack([toks[b, cl[b]:cl[b] + m].numpy() for b in range(B)])
    err = _check(gm, om, block, cl, 2e-2, 1e-2, f"t5 B={B} m={m}")
    print("t5 bf16 rows", B * m, "max err", err)


def test_t5xxl_decoder_shape_block_of_k4_against_oracle():
    """Configuration 4 at full size: 24 layers, d_model 4096, 64 heads of 64, gated-GELU FFN 10240, vocab
    32128, 512 encoder rows projected by csd_cross_kv_init on both sides, 256 seeded cache rows, k = 4."""
    from oracle import csd_oracle as O
    import paper_2312_11462_amd as P
    wl = I.WORKLOADS["t5xxl"]
    shape, seed, t, k = wl["shape"], wl["seed"], wl["prefix"], wl["k"]
    w = I.make_weights(shape, seed, device="cuda")
    gm = P.Model(shape, w, max_batch=1, max_seq=t + 64, max_block=8)
    assert gm.path(1, k + 1) == 1      # the forward with in-kernel epilogues, as bench.py times it
    host = [x.cpu() for x in w]
    del w
    torch.cuda.empty_cache()
    om = O.Model(shape, host, max_batch=1, max_seq=t + 64, max_block=8)
    print("T5-XXL-decoder-shaped pair ready; oracle threads", O.threads(), flush=True)
    enc = I.encoder_output(shape, 1, seed)
    gm.cross_kv_init(enc.cuda())
    torch.cuda.synchronize()
    print("gpu cross K/V ready; oracle projecting", flush=True)
    om.cross_kv_init(enc.numpy())
    print("oracle cross K/V ready", flush=True)
    import_synthetic_kv(gm, om, shape, t, seed)
    block = I.token_ids(k + 1, shape.vocab, seed, 5)[None].contiguous()
    L, d, m = shape.n_layers, shape.d_model, k + 1
    tr = torch.zeros((L + 1, m, d), dtype=torch.float32, device="cuda")
    gm.set_trace(tr)
    lg = gm.verify_block(block.cuda(), _dev([t]))
    gm.set_trace(None)
    torch.cuda.synchronize()
    print("gpu forward done; oracle running", flush=True)
    ref, otr = om.verify_block(block.numpy(), [t], trace=True)
    ok, err = tol_ok(lg[0].cpu().numpy().astype(np.float64), ref[0], 2e-2, 1e-2)
    g = tr.cpu().numpy().astype(np.float64)
    rel = max(np.linalg.norm(g[l] - otr[l]) / np.linalg.norm(otr[l]) for l in range(L + 1))
    print(f"t5xxl: max |dlogit| {err:.3e}, worst residual-stream relative error {rel:.3e}", flush=True)
    assert ok, f"logits max abs err {err}"
    assert rel < 5e-3
