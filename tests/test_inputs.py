"""The seeded input generator: reproducible bits, sane moments (CPU only)."""
import numpy as np
import torch

import csd_inputs as I


def test_vectorised_stream_is_the_scalar_splitmix64_sequence():
    base = I.stream_base(5, 7)
    got = [v & ((1 << 64) - 1) for v in I.raw_bits(6, 5, 7).tolist()]
    want = [I.splitmix64_scalar((base + (i + 1) * 0x9E3779B97F4A7C15) & ((1 << 64) - 1)) for i in range(6)]
    assert got == want
    # published first output of splitmix64 seeded with 0
    assert I.splitmix64_scalar(0x9E3779B97F4A7C15) == 0xE220A8397B1DCDAF


def test_chunking_and_offsets_do_not_change_values():
    a = I.raw_bits(100, 3, 4)
    b = torch.cat([I.raw_bits(40, 3, 4), I.raw_bits(60, 3, 4, offset=40)])
    assert torch.equal(a, b)


def test_moments_and_ranges():
    w = I.normal((512, 512), 0.02, 1, 2)
    assert abs(w.std().item() - 0.02) < 2e-4 and abs(w.mean().item()) < 2e-4
    u = I.uniforms(10000, 1, 3)
    assert u.min() >= 0 and u.max() < 1 and abs(u.mean().item() - 0.5) < 0.02
    assert torch.equal(u * 2 ** 24, torch.floor(u * 2 ** 24))
    t = I.token_ids(10000, 512, 1, 4)
    assert t.min() >= 0 and t.max() < 512 and len(torch.unique(t)) > 400


def test_weights_shapes_and_dtypes():
    w = I.make_weights(I.TINY, 1)
    assert len(w) == I.TINY.n_weights() == len(I.weight_names(I.TINY))
    assert w[0].shape == (512, 64) and w[-1].shape == (64, 512) and w[1].dtype == torch.float32
    shp = I.ModelShape("b", 0, "bf16", 1, 32, 2, 16, 64, 100)
    wb = I.make_weights(shp, 1)
    assert wb[0].dtype == torch.bfloat16 and wb[1].dtype == torch.float32
    assert I.TARGET_7B.streamed_params() == 6_607_077_376


def test_repeat_stream_has_repeats():
    s = I.repeat_stream(500, 32000, 3, 1).numpy()
    assert len(s) == 500 and s.min() >= 0 and s.max() < 32000
    bigrams = set(zip(s[:-1], s[1:]))
    assert len(bigrams) < 0.9 * 499


def test_t5_recipe_keeps_unscaled_scores_of_order_one():
    """arch 1 has no 1/sqrt(head_dim) in its scores (the family folds it into the query projection's initialisation), so
    the recipe draws the query projections with std 0.02/sqrt(head_dim).  For unit-variance normalised rows the
    score of a (query, key) pair has std  s_q * s_k * d * sqrt(head_dim): measured here on a one-layer shape of
    width 1024, and evaluated for the T5-XXL-decoder shape with and without the smaller query std (13 against 1.6:
    with 13 a random-init softmax is near one-hot and rounding differences double per layer)."""
    shp = I.ModelShape("t5probe", 1, "fp32", 1, 1024, 16, 64, 64, 64, rms_eps=1e-6, enc_len=8)
    w = dict(zip(I.weight_names(shp), I.make_weights(shp, 3)))
    x = I.normal((256, 1024), 1.0, 3, 77)
    H, dh = shp.n_heads, shp.head_dim
    q = (x @ w["l0.wq"]).reshape(256, H, dh)
    k = (x @ w["l0.wk"]).reshape(256, H, dh)
    s = torch.einsum("ihd,jhd->hij", q, k)
    want = (0.02 / dh ** 0.5) * 0.02 * 1024 * dh ** 0.5
    off_diag = s[:, ~torch.eye(256, dtype=torch.bool)]
    assert abs(off_diag.std().item() / want - 1.0) < 0.05, (off_diag.std().item(), want)
    assert abs(w["l0.cq"].std().item() - 0.02 / 8) < 1e-4 and abs(w["l0.wk"].std().item() - 0.02) < 2e-4
    xxl = I.WORKLOADS["t5xxl"]["shape"]
    full = lambda s_q: s_q * 0.02 * xxl.d_model * xxl.head_dim ** 0.5
    assert 12.5 < full(0.02) < 13.5 and 1.5 < full(0.02 / xxl.head_dim ** 0.5) < 1.8
