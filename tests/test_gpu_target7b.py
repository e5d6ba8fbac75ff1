"""Full-size GPU parity: the 7B-shaped bf16 target at the benchmark's launch configuration
(batch 1, 1024 cached rows, block of k = 5 drafts) and at the batch-8 / 2048-row configuration,
against the CPU oracle on the same seeded weights and the same seeded stand-in cache rows
(a real prefill of 1024+ rows is hours of oracle time).  The oracle computes one sequence of
the batch; sequences are independent, so any one of them is a fair sample."""
import os

import numpy as np
import pytest
import torch

import csd_inputs as I
from gpu_util import tol_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def big():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2312_11462_amd as P
    from oracle import csd_oracle as O
    wl = I.WORKLOADS["target7b"]
    shape, seed = wl["shape"], wl["seed"]
    w = I.make_weights(shape, seed, device="cuda")
    gm = P.Model(shape, w, max_batch=8, max_seq=2048 + 64, max_block=17)
    host = [x.cpu() for x in w]
    del w
    torch.cuda.empty_cache()
    om = O.Model(shape, host, max_batch=1, max_seq=2048 + 64, max_block=17)
    print("7B-shaped pair ready; oracle threads", O.threads(), flush=True)
    return P, O, gm, om, shape, seed


def _fill(gm, om, shape, seed, n_rows, B, oracle_b):
    for l in range(shape.n_layers):
        for b in range(B):
            K, V = I.synthetic_kv(shape, n_rows, seed, l, b, device="cuda")
            gm.kv_write(l, b, 0, K, V)
            if b == oracle_b:
                om.kv_write(l, 0, 0, K.cpu().numpy(), V.cpu().numpy())
    torch.cuda.synchronize()


def _compare(gm, om, block, cache_len, oracle_b, what):
    B, m = block.shape
    L, d = gm.shape.n_layers, gm.shape.d_model
    tr = torch.zeros((L + 1, B * m, d), dtype=torch.float32, device="cuda")
    gm.set_trace(tr)
    lg, pr = gm.verify_block(block.cuda(), torch.tensor(cache_len, dtype=torch.int32).cuda(), want_probs=True)
    gm.set_trace(None)
    torch.cuda.synchronize()
    print(what, "gpu done; oracle running", flush=True)
    ref, otr = om.verify_block(block[oracle_b:oracle_b + 1].numpy(), [cache_len[oracle_b]], trace=True)
    got = lg[oracle_b].cpu().numpy().astype(np.float64)
    ok, err = tol_ok(got, ref[0], 2e-2, 1e-2)
    g = tr.cpu().numpy()[:, oracle_b * m:(oracle_b + 1) * m, :].astype(np.float64)
    rel = max(np.linalg.norm(g[l] - otr[l]) / np.linalg.norm(otr[l]) for l in range(L + 1))
    print(f"{what}: max |dlogit| {err:.3e}, worst residual-stream relative error {rel:.3e}", flush=True)
    assert ok, f"{what}: logits max abs err {err}"
    assert rel < 5e-3
    return lg, pr, ref


def test_target7b_batch1_prefix1024_k5(big):
    """The benchmark configuration itself: the block mixes 2 stand-in neural drafts and 3 Max-Gram
    drafts; logits of all 6 rows x 32000 entries are compared, then the accept decision."""
    P, O, gm, om, shape, seed = big
    t, k = 1024, 5
    _fill(gm, om, shape, seed, t, 1, 0)
    ctx = torch.zeros(t + 64, dtype=torch.int32)
    ctx[:t + 1] = I.repeat_stream(t + 1, shape.vocab, seed, 10)
    ctx[t + 1:t + 3] = I.token_ids(2, shape.vocab, seed, 99)
    table = P.bigram_fit(ctx[:t + 1].cuda(), shape.vocab, I.default_next_table(shape.vocab, seed).cuda())
    tail, mlen = P.bigram_draft(ctx.cuda(), torch.tensor([t + 3], dtype=torch.int32).cuda(), table, 3)
    otab = O.bigram_fit(ctx[:t + 1].numpy(), shape.vocab, I.default_next_table(shape.vocab, seed).numpy())
    otail, omlen = O.bigram_draft(ctx.numpy(), [t + 3], otab, 3)
    assert np.array_equal(tail.cpu().numpy(), otail) and int(mlen[0]) == int(omlen[0])
    block = torch.cat([ctx[t:t + 3], tail[0].cpu()])[None].contiguous()
    lg, pr, ref = _compare(gm, om, block, [t], 0, "7B b1 t1024 k5")
    # accept on identical probabilities must agree bit for bit; on each side's own probabilities the
    # decisions are reported (they can differ only within the logit tolerance of a threshold)
    u_acc = I.uniforms(k, seed, 7)[None].contiguous()
    u_s = I.uniforms(1, seed, 8)
    drafts = block[:, 1:].contiguous()
    gn, gt = P.accept(pr, None, drafts.cuda(), u_acc.cuda(), u_s.cuda())
    on, ot = O.accept(pr.cpu().numpy(), None, drafts.numpy(), u_acc.numpy(), u_s.numpy())
    assert int(gn[0]) == int(on[0]) and int(gt[0]) == int(ot[0])
    # end to end (each side on its own probabilities): decisions may differ only where the oracle's margin is inside
    # what the logit tolerance allows.  A logit error e changes a probability by at most a factor e^(2e); with the
    # stated tolerance at these logits (|l| < 1) that is about 6 %; the draw's threshold can move by as much of the
    # total weight.  Decisions with a larger margin must agree; the others are counted.
    on2, ot2, tests, draw = O.accept_margins(O.probs_f32(ref), None, drafts.numpy(), u_acc.numpy(), u_s.numpy())
    tol = float(np.expm1(2 * (1e-2 + 2e-2 * np.abs(ref).max())))
    inside = sum(1 for _, mg in tests if mg <= tol) + (1 if draw <= tol else 0)
    print(f"accept on gpu probs: {int(gn[0])} {int(gt[0])}  on oracle probs: {on2} {ot2}; decisions within the "
          f"tolerance's reach ({tol:.3f}): {inside} of {len(tests) + 1}", flush=True)
    if all(mg > tol for _, mg in tests):
        assert int(gn[0]) == on2
        if draw > tol:
            assert int(gt[0]) == ot2
    # greedy: arg-max tokens of all rows agree unless the oracle's top-2 gap is inside the tolerance
    gam = lg[0].argmax(-1).cpu().numpy()
    for i in range(k + 1):
        top2 = np.sort(ref[0, i])[-2:]
        if top2[1] - top2[0] > 2 * (1e-2 + 2e-2 * abs(top2[1])):
            assert gam[i] == int(np.argmax(ref[0, i]))
    # 30 more calls: the same logits every time
    assert gm.path(1, k + 1) == 1
    cl = torch.tensor([t], dtype=torch.int32).cuda()
    for _ in range(30):
        assert torch.equal(gm.verify_block(block.cuda(), cl), lg)


@pytest.mark.parametrize("k,oracle_b", [(1, 5), (4, 3), (16, 6)])
def test_target7b_batch8_prefix2048(big, k, oracle_b):
    """Batch of 8 independent sequences with 2048 cached rows each: 16 block rows on the forward with the
    epilogues inside its GEMM kernels, 40 and 136 rows on the per-operation kernels with the GEMM that shares
    activations through LDS (40 rows) and the row-split GEMM (136 rows); one sampled sequence is checked
    against the oracle."""
    P, O, gm, om, shape, seed = big
    assert gm.path(8, k + 1) == (1 if 8 * (k + 1) <= 32 else 0)
    t, B, m = 2048, 8, k + 1
    _fill(gm, om, shape, seed, t, B, oracle_b)
    block = I.token_ids(B * m, shape.vocab, seed, 200 + k).reshape(B, m).contiguous()
    _compare(gm, om, block, [t] * B, oracle_b, f"7B b8 t2048 k{k} seq{oracle_b}")


def test_two_level_step_of_configuration_3_with_device_resident_control(big):
    """Configuration 3 as one step of Algorithm 1 at full size, K = [[2, 3], [0, 8]], greedy rule: the 160M-shaped
    level reviews Max-Gram drafts until two of its tokens exist, Max-Gram adds three, the 7B-shaped target reviews;
    one chain of enqueues with device-resident control.  The kept tokens equal the oracle driver's for the same
    seeded weights and stand-in caches (1024 rows in both models)."""
    P, O, gm, om, shape, seed = big
    from oracle import cascade as OC
    from paper_2312_11462_amd.cascade import Level, ResidentCascade
    t = 1024
    dwl = I.WORKLOADS["draft160m"]
    dshape, dseed = dwl["shape"], dwl["seed"]
    dw = I.make_weights(dshape, dseed, device="cuda")
    gd = P.Model(dshape, dw, max_batch=1, max_seq=t + 64, max_block=16)
    od = O.Model(dshape, [x.cpu() for x in dw], max_batch=1, max_seq=t + 64, max_block=16)
    del dw
    _fill(gm, om, shape, seed, t, 1, 0)
    _fill(gd, od, dshape, dseed, t, 1, 0)
    prompt = I.repeat_stream(t + 1, shape.vocab, seed, 10)
    table = P.bigram_fit(prompt.cuda(), shape.vocab, I.default_next_table(shape.vocab, seed).cuda())
    K = [[2, 3], [0, 8]]
    rc = ResidentCascade([Level(gm, 16), Level(gd, 16)], table, K, t + 64, mode=1)
    rc.ctx[0, :t + 1] = prompt.cuda()
    rc.ctx_len.fill_(t + 1)
    rc.cache_len[0].fill_(t)
    rc.cache_len[1].fill_(t)
    rc.step()
    got = rc.tokens()
    assert [int(s.item()) for s in rc.status] == [0, 0]
    print("device-resident two-level step: kept", got[t + 1:], "accepted by target / draft level:",
          int(rc.n_acc[0].item()), int(rc.n_acc[1].item()), flush=True)
    ot, odl = OC.Level(om, 16), OC.Level(od, 16)
    ot.cached = odl.cached = t
    toks, _ = OC._step([ot, odl], table.cpu().numpy(), prompt.tolist(), K, 1.0, 1, None, True, 0)
    assert got[t + 1:] == toks


def test_target7b_block_over_rows_the_gpu_prefilled_itself(big):
    """The cached prefix of the benchmark configuration with its last 64 rows written by the GPU's own review
    forward (four 16-row blocks on top of 960 stand-in rows, the oracle doing the same on its side): the 6-row
    block is then compared as above, so the rows that the path itself appends at full size are part of what is
    checked, not only rows imported through csd_kv_write."""
    P, O, gm, om, shape, seed = big
    t0, extra, k = 960, 64, 5
    _fill(gm, om, shape, seed, t0, 1, 0)
    toks = I.token_ids(extra + k + 1, shape.vocab, seed, 321)
    for pos in range(0, extra, 16):
        blk = toks[pos:pos + 16][None].contiguous()
        gm.verify_block(blk.cuda(), torch.tensor([t0 + pos], dtype=torch.int32).cuda())
        om.verify_block(blk.numpy(), [t0 + pos])
        print("prefilled rows", t0 + pos, "..", t0 + pos + 16, flush=True)
    # the rows both sides appended agree (bf16 values of nearly equal fp32 numbers: a rounding step at most)
    Kg, Vg = gm.kv_read(shape.n_layers - 1, 0, t0, extra)
    Ko, Vo = om.kv_read(shape.n_layers - 1, 0, t0, extra)
    assert np.abs(Kg.cpu().numpy() - Ko).max() < 2e-2 * np.abs(Ko).max()
    assert np.abs(Vg.cpu().numpy() - Vo).max() < 2e-2 * np.abs(Vo).max()
    block = toks[extra:][None].contiguous()
    _compare(gm, om, block, [t0 + extra], 0, "7B b1, 64 of 1024 cached rows from the GPU's own prefill, k5")


def test_target7b_tree_of_17_rows_appendix_b_shape(big):
    """A tree block at the full shape (Section 5.1, Appendix B: eight children per lead node): root + 2 levels x 8
    children = 17 rows over the 1024-row cache.  All 17 x 32000 logits against the oracle's tree forward; the walk on
    the GPU's probabilities equals the oracle's walk on the same probabilities; after the commit of a two-row path the
    next plain block's logits match the oracle, which committed the same path."""
    P, O, gm, om, shape, seed = big
    t = 1024
    _fill(gm, om, shape, seed, t, 1, 0)
    parent = np.array([[-1] + [0] * 8 + [1] * 8], np.int32)
    tokens = I.token_ids(17, shape.vocab, seed, 555)[None].contiguous()
    cl = torch.tensor([t], dtype=torch.int32).cuda()
    assert gm.path(1, 17) == 1          # two row tiles on the forward with in-kernel epilogues
    lg, pr = gm.verify_tree(tokens.cuda(), torch.from_numpy(parent).cuda(), cl, want_probs=True)
    torch.cuda.synchronize()
    print("tree: gpu done; oracle running", flush=True)
    ref = om.verify_tree(tokens.numpy(), parent, [t])
    ok, err = tol_ok(lg.cpu().numpy().astype(np.float64), ref, 2e-2, 1e-2)
    print(f"7B tree of 17 rows: max |dlogit| {err:.3e}", flush=True)
    assert ok, err
    for mode in (0, 1):
        u = I.uniforms(17, seed, 777 + mode).reshape(1, 17)
        src = pr if mode == 0 else lg
        n, path, nxt = P.tree_accept(src, tokens.cuda(), torch.from_numpy(parent).cuda(), u.cuda(), mode=mode)
        on, opath, onxt = O.tree_accept(src.cpu().numpy(), tokens.numpy(), parent, u.numpy(), mode=mode)
        assert int(n.item()) == int(on[0]) and int(nxt.item()) == int(onxt[0])
    # keep the lead child and one of its children, as a review that accepted two candidates would
    path = torch.full((1, 17), -1, dtype=torch.int32)
    path[0, :2] = torch.tensor([1, 12], dtype=torch.int32)
    gm.tree_commit(cl, path.cuda(), torch.tensor([2], dtype=torch.int32).cuda())
    om.tree_commit(0, t, [1, 12])
    nxt_block = I.token_ids(6, shape.vocab, seed, 556)[None].contiguous()
    _compare(gm, om, nxt_block, [t + 3], 0, "7B b1, plain block after a tree commit")
