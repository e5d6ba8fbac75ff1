#!/usr/bin/env python3
"""Benchmark of one verify+accept step of Cascade Speculative Drafting on one MI355X.

A step is one pass of the whole hot path over one batch of synthetic input, all resident in HBM:
Max-Gram draft of the block's tail -> review forward of the 7B-shaped target over the k+1 block
rows against a 1024-row KV cache -> softmax -> accept / resample.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload target7b|t5xxl|draft160m|tiny]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0
# HBM bytes per launch of the dominant kernel, from rocprofv3 counter runs of this same command
# (FETCH_SIZE and WRITE_SIZE, each scaled by what the counter reads for a copy of known size); the
# summaries and the commands are under profiles/.  Keyed by (workload, forward path).
TRAFFIC_BYTES_PER_LAUNCH = {("target7b", 1): 104_085_000}
# Average duration of the same launches in the rocprofv3 kernel trace of this command (the HIP events that
# bench.py puts around every launch add about 1.5 us each): profiles/, same key.
TRACE_LAUNCH_US = {("target7b", 1): 21.47}


def algorithmic_bytes(shape, B, t, m):
    """Bytes one step must move: every streamed weight once, the visible K/V rows once (for an arch-1
    reviewer also the projected encoder rows), the new K/V rows, the gathered embedding rows and the
    logits written once for the caller."""
    d, L, V = shape.d_model, shape.n_layers, shape.vocab
    hd = shape.n_heads * shape.head_dim
    esz = 2 if shape.dtype == "bf16" else 4
    weights = shape.streamed_params() * esz
    kv_read = L * B * 2 * (t + m + shape.enc_len) * hd * esz
    kv_write = L * B * 2 * m * hd * esz
    return dict(weights=weights, total=weights + kv_read + kv_write + B * m * d * esz + 4 * B * m * V)


def algorithmic_flops(shape, B, t, m):
    L = shape.n_layers
    hd = shape.n_heads * shape.head_dim
    return 2 * shape.streamed_params() * B * m + L * B * 4 * (t + m + shape.enc_len) * hd * m


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--settle-ms", type=float, default=1000.0,
                    help="before the warm-up steps, run untimed steps for this long (part of the setup): the step time of a "
                         "chip that comes from idle settles only after some tenths of a second of load (3.19 ms for 200 steps "
                         "right after 20 warm-up steps, 3.12 after a second of load); 0 = none")
    ap.add_argument("--workload", default="target7b")
    ap.add_argument("--k", type=int, default=None, help="drafts per sequence instead of the workload's (configuration 5 sweeps it)")
    ap.add_argument("--prof-steps", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-peaks", action="store_true",
                    help="skip the peaks measured on the box (a streaming read, a copy, a loop of matrix instructions)")
    ap.add_argument("--cascade-steps", type=int, default=20, metavar="N",
                    help="workload target7b: also time N whole two-level cascade steps of configuration 3 "
                         "(the 160M-shaped draft level's reviews + the timed step); 0 = skip")
    ap.add_argument("--tree-steps", type=int, default=10, metavar="N",
                    help="workload target7b: also time N reviews of a tree block of Appendix B's shape (a lead chain of 4 "
                         "with 8 children per lead node = 33 rows: forward, walk, commit); 0 = skip")
    ap.add_argument("--eager", action="store_true", help="time plain launches instead of replays of the captured step")
    ap.add_argument("--mode", default="sample", choices=["sample", "greedy"])
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="N",
                    help="after the benchmark, launch N plain 1 GiB copies (kernel k_copy_calib) so that a "
                         "rocprofv3 counter run of this command also reads the counters for known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (sequences are independent, "
              "so N GPUs would each run this same step on their own share); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import csd_inputs as I
    import paper_2312_11462_amd as P

    P.lib()                                   # fail loudly when the HIP library is missing
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    wl = I.WORKLOADS[args.workload]
    shape, B, t, k, seed = wl["shape"], wl["B"], wl["prefix"], wl["k"], wl["seed"]
    if args.k is not None:
        k = args.k
    target_mix = wl.get("draft") == "target_mix"
    m = k + 1
    n_from_draft_model = 2 if args.workload in ("target7b", "t5xxl") else 0     # horizontal cascade: 2 neural drafts, tail from Max-Gram
    k_tail = k - n_from_draft_model

    # ---- setup (untimed): weights, model, cache, context, tables
    t0 = time.time()
    w = I.make_weights(shape, seed, device="cuda")
    # (the two-level step of configuration 3 reviews up to 16 rows: 1 + up to 10 tokens of the draft level + the tail)
    model = P.Model(shape, w, max_batch=B, max_seq=t + 64, max_block=16 if args.workload == "target7b" else max(m, 8))
    enc = None
    if shape.arch == 1:      # encoder-decoder reviewer: the encoder output is projected once per prompt (setup)
        enc = I.encoder_output(shape, B, seed, device="cuda")
        model.cross_kv_init(enc)
    host_w = None
    if not args.no_cpu_baseline:
        host_w = [x.cpu() for x in w]
    tree_model = None
    if args.workload == "target7b" and args.tree_steps > 0:      # a model of its own: blocks of up to 33 rows
        tree_model = P.Model(shape, w, max_batch=1, max_seq=t + 64, max_block=33)
    del w
    torch.cuda.empty_cache()
    for l in range(shape.n_layers):
        for b in range(B):
            K, V = I.synthetic_kv(shape, t, seed, l, b, device="cuda")
            model.kv_write(l, b, 0, K, V)
    stride = t + 64
    ctx = torch.zeros((B, stride), dtype=torch.int32)
    for b in range(B):
        ctx[b, :t + 1] = I.repeat_stream(t + 1, shape.vocab, seed, 10 + b)
    # the first drafts of the block stand in for the neural draft level's tokens
    neural = I.token_ids(B * max(1, n_from_draft_model), shape.vocab, seed, 99).reshape(B, -1)[:, :n_from_draft_model]
    ctx[:, t + 1:t + 1 + n_from_draft_model] = neural
    ctx_len = torch.full((B,), t + 1 + n_from_draft_model, dtype=torch.int32)
    ctx, ctx_len = ctx.cuda(), ctx_len.cuda()
    table = I.default_next_table(shape.vocab, seed).cuda()
    for b in range(B):
        P.bigram_fit(ctx[b, :t + 1].contiguous(), shape.vocab, table)
    block = torch.zeros((B, m), dtype=torch.int32, device="cuda")
    block[:, :1 + n_from_draft_model] = ctx[:, t:t + 1 + n_from_draft_model]
    tail = torch.zeros((B, k_tail), dtype=torch.int32, device="cuda")
    cache_len = torch.full((B,), t, dtype=torch.int32, device="cuda")
    u_acc = I.uniforms(B * k, seed, 7).reshape(B, k).contiguous().cuda()
    u_samp = I.uniforms(B, seed, 8).cuda()
    onehot = torch.ones(k, dtype=torch.uint8, device="cuda")
    n_acc = torch.zeros(B, dtype=torch.int32, device="cuda")
    nxt = torch.zeros(B, dtype=torch.int32, device="cuda")
    mode = 0 if args.mode == "sample" else 1
    q_draft = None
    if target_mix:
        # Drafts sampled from the reviewer's own next-token distributions perturbed by seeded noise:
        # q_i = softmax(logits_i + sigma * g_i), x_i ~ q_i, with sigma set (by bisection at the first position)
        # so that the expected acceptance sum_x min(p_i(x), q_i(x)) is the workload's.  k one-row forwards
        # at setup; they leave exactly the cache rows the timed block rewrites.
        V = shape.vocab
        q_draft = torch.empty((B, k, V), dtype=torch.float32, device="cuda")
        u_draft = I.uniforms(B * k, seed, 9).reshape(B, k).to(torch.float64).cuda()
        sigma = None
        for i in range(k):
            lg = model.verify_block(block[:, i:i + 1].contiguous(), cache_len + i)[:, 0, :]
            p_i = torch.softmax(lg, dim=-1)
            g_i = I.normal((B, V), 1.0, seed, 100 + i, device="cuda")
            if sigma is None:
                lo, hi = 0.0, 16.0
                for _ in range(40):
                    mid = 0.5 * (lo + hi)
                    acc = torch.minimum(p_i, torch.softmax(lg + mid * g_i, dim=-1)).sum(-1).mean().item()
                    lo, hi = (mid, hi) if acc > wl["acceptance"] else (lo, mid)
                sigma = 0.5 * (lo + hi)
            q_i = torch.softmax(lg + sigma * g_i, dim=-1)
            q_draft[:, i, :] = q_i
            cdf = torch.cumsum(q_i.to(torch.float64), dim=-1)
            x_i = torch.searchsorted(cdf, (u_draft[:, i] * cdf[:, -1])[:, None], right=True)[:, 0].clamp_(max=V - 1)
            block[:, i + 1] = x_i.to(torch.int32)
        onehot = None
    torch.cuda.synchronize()
    setup_s = time.time() - t0

    def step():
        if target_mix:   # the drafts and their distributions are inputs of this configuration
            model.verify_accept(block, cache_len, u_acc, u_samp, q=q_draft, q_onehot=None, mode=mode,
                                n_accepted=n_acc, next_token=nxt)
            return
        if B == 1:       # the draft lands directly in the block's tail
            P.bigram_draft(ctx, ctx_len, table, k_tail, want_match_len=False, out=block[:, 1 + n_from_draft_model:])
        else:
            P.bigram_draft(ctx, ctx_len, table, k_tail, want_match_len=False, out=tail)
            block[:, 1 + n_from_draft_model:] = tail
        model.verify_accept(block, cache_len, u_acc, u_samp, q=None, q_onehot=onehot, mode=mode,
                            n_accepted=n_acc, next_token=nxt)

    if args.settle_ms > 0:
        t_settle = time.perf_counter()
        while (time.perf_counter() - t_settle) * 1e3 < args.settle_ms:
            for _ in range(10):
                step()
            torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The timed step is launched the way a serving loop on this hardware would launch it: captured once in a HIP graph
    # (draft, forward and review: the same kernels on the same buffers; the library allocates nothing per call and
    # clears its counters with kernels, so its calls can be captured as they are) and replayed.  --eager times plain
    # launches instead; the other figure is reported beside `value` either way.
    graph = None
    if not args.eager:
        try:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                step()
            for _ in range(3):
                graph.replay()
            torch.cuda.synchronize()
        except Exception as e:      # noqa: BLE001  (a capture failure must not take the benchmark line with it)
            print("graph capture failed, timing eager launches:", e, file=sys.stderr)
            graph = None
    run = graph.replay if graph is not None else step

    def timed(fn, n):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(n):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / n, e0.elapsed_time(e1) / n

    ms_per_step, gpu_ms_per_step = timed(run, args.steps)
    wall = ms_per_step * args.steps / 1e3
    other_ms = timed(step if graph is not None else run, min(args.steps, 50))[1]    # eager launches when `value` is the graph's
    eager_ms_per_step = other_ms if graph is not None else gpu_ms_per_step
    # the same step timed one at a time (an event pair per step, each waited for): the median
    n_single = min(args.steps, 50)
    singles = []
    for _ in range(n_single):
        a, b_ = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        run()
        b_.record()
        b_.synchronize()
        singles.append(a.elapsed_time(b_))
    median_single_ms = sorted(singles)[len(singles) // 2] if singles else None
    emitted = float((n_acc + 1).sum().item())

    # ---- per-kernel timing with HIP events on the launch stream (separate loop: the events perturb the step)
    model.prof_enable(True)
    cls_ms, cls_n = [0.0, 0.0, 0.0], [0, 0, 0]
    for _ in range(args.prof_steps):
        step()
        torch.cuda.synchronize()
        for c in range(3):
            ms, n = model.prof_read(c, reset=(c == 2))
            cls_ms[c] += ms
            cls_n[c] += n
    model.prof_enable(False)
    ab = algorithmic_bytes(shape, B, t, m)
    fl = algorithmic_flops(shape, B, t, m)
    gemm_ms_step = cls_ms[0] / max(1, args.prof_steps)
    gemm_launches_step = cls_n[0] / max(1, args.prof_steps)
    path = model.path(B, m)
    # the dominant kernel: the weight-streaming GEMM.  One launch streams one matrix; the per-launch figures are
    # the step's weights over the step's GEMM launches.
    kernel = ("kc_gemm (GEMMs that own whole output tiles and hold their epilogues)" if path == 1 else
              ("k_gemm_rs" if B * m > 32 else "k_gemm_ws") + " (split-K GEMMs with epilogue kernels)") + \
             ": all weight-streaming GEMM launches of a step"
    launch_bytes = ab["weights"]
    achieved = launch_bytes / 1e9 / (gemm_ms_step / 1e3) if gemm_ms_step > 0 else 0.0
    roofline = {
        "bound": "hbm", "kernel": kernel,
        "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
        "bytes_per_launch": round(launch_bytes / max(1.0, gemm_launches_step)),
        "avg_launch_us": round(1e3 * gemm_ms_step / max(1.0, gemm_launches_step), 2),
        "launches_per_step": gemm_launches_step,
        "step_frac": round(ab["total"] / 1e9 / (gpu_ms_per_step / 1e3) / HBM_PEAK_GBS, 4),
        "mfma_frac": round(fl / 1e12 / (gpu_ms_per_step / 1e3) / MFMA_BF16_PEAK_TFLOPS, 5),
        "class_ms_per_step": {"gemm": round(gemm_ms_step, 4),
                              "attention": round(cls_ms[1] / max(1, args.prof_steps), 4),
                              "other": round(cls_ms[2] / max(1, args.prof_steps), 4)},
    }
    if TRAFFIC_BYTES_PER_LAUNCH.get((args.workload, path)):
        roofline["traffic"] = TRAFFIC_BYTES_PER_LAUNCH[(args.workload, path)]
    if TRACE_LAUNCH_US.get((args.workload, path)) and gemm_launches_step > 0:
        us = TRACE_LAUNCH_US[(args.workload, path)]
        roofline["trace_avg_launch_us"] = us
        roofline["trace_frac"] = round(roofline["bytes_per_launch"] / 1e3 / us / HBM_PEAK_GBS, 4)
    roofline["note"] = ("frac: GEMM launches only, weights only, timed live with HIP events around every launch; "
                        "trace_frac: the same with the launch duration of the committed rocprofv3 kernel trace; "
                        "step_frac: all algorithmic bytes of the step over the whole step's time")

    # ---- a review over a tree of drafts (extra, timed apart from `value`): Section 5.1 / Appendix B's shape, a lead chain
    # of 4 (1 token of the draft level + 3 of Max-Gram in the paper's K matrix) with 8 candidates per lead node
    tree = None
    if tree_model is not None:
        for l in range(shape.n_layers):
            K, V = I.synthetic_kv(shape, t, seed, l, 0, device="cuda")
            tree_model.kv_write(l, 0, 0, K, V)
        depth, kids = 4, 8
        par, lead = [-1], 0
        for _ in range(depth):
            first = len(par)
            par += [lead] * kids
            lead = first
        rows = len(par)
        t_parent = torch.tensor([par], dtype=torch.int32).cuda()
        t_tokens = I.token_ids(rows, shape.vocab, seed, 4242).reshape(1, rows).contiguous().cuda()
        t_tokens[0, 0] = ctx[0, t]
        t_u = I.uniforms(rows, seed, 4243).reshape(1, rows).contiguous().cuda()
        t_cl = cache_len[:1].clone()
        t_lg = torch.empty((1, rows, shape.vocab), dtype=torch.float32, device="cuda")
        t_pr = torch.empty_like(t_lg)

        def tree_step():
            tree_model.verify_tree(t_tokens, t_parent, t_cl, want_probs=(mode == 0), logits=t_lg, probs=t_pr if mode == 0 else None)
            n_, path_, _ = P.tree_accept(t_pr if mode == 0 else t_lg, t_tokens, t_parent, t_u, mode=mode)
            tree_model.tree_commit(t_cl, path_, n_)

        for _ in range(3):
            tree_step()
        torch.cuda.synchronize()
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record()
        for _ in range(args.tree_steps):
            tree_step()
        c1.record()
        torch.cuda.synchronize()
        tree = {"ms": round(c0.elapsed_time(c1) / args.tree_steps, 4), "steps": args.tree_steps, "rows": rows,
                "what": f"csd_verify_tree + csd_tree_accept + csd_tree_commit over a tree block of {rows} rows (lead chain of "
                        f"{depth}, {kids} candidates per lead node, seeded random candidates), batch 1, {t}-row cache"}
        del tree_model
        torch.cuda.empty_cache()

    # ---- configuration 3 as a whole (extra, timed apart from `value`): one step of Algorithm 1 with K = [[2, k_tail],
    # [0, dk]] and device-resident control: the 160M-shaped level reviews Max-Gram drafts until two of its tokens
    # exist (worst case two reviews, the second gated on the device), Max-Gram adds the tail, the target reviews the
    # block against the draft level's own distributions; and, beside it, plain speculative decoding with the same
    # two models (k one-row draft forwards, then the target's review).  No host synchronisation inside either.
    cascade = None
    if args.workload == "target7b" and args.cascade_steps > 0:
        from paper_2312_11462_amd.cascade import Level, ResidentCascade
        from paper_2312_11462_amd import ewif
        dwl = I.WORKLOADS["draft160m"]
        dshape, dseed, dk = dwl["shape"], dwl["seed"], dwl["k"]
        dw = I.make_weights(dshape, dseed, device="cuda")
        draft = P.Model(dshape, dw, max_batch=1, max_seq=t + 64, max_block=16)
        del dw
        for l in range(dshape.n_layers):
            K, V = I.synthetic_kv(dshape, t, dseed, l, 0, device="cuda")
            draft.kv_write(l, 0, 0, K, V)
        levels = [Level(model, 16), Level(draft, 16)]

        def timed_chain(Kmat):
            rc = ResidentCascade(levels, table, Kmat, stride, mode=mode)
            rc.ctx[0, :t + 1] = ctx[0, :t + 1]
            for i in range(2):
                rc.u_acc[i].copy_(I.uniforms(stride, seed, 20 + i)[None])
                rc.u_samp[i].copy_(I.uniforms(stride, seed, 30 + i)[None])

            def one():
                rc.ctx_len.fill_(t + 1)                 # every timed step starts from the same state
                rc.cache_len[0].fill_(t)
                rc.cache_len[1].fill_(t)
                rc.step()
            for _ in range(3):
                one()
            torch.cuda.synchronize()

            def timed_loop(fn):
                c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                c0.record()
                for _ in range(args.cascade_steps):
                    fn()
                c1.record()
                torch.cuda.synchronize()
                return c0.elapsed_time(c1) / args.cascade_steps
            eager_ms = timed_loop(one)
            # the step holds no host synchronisation, so it is captured as it is, like the main step (--eager: not)
            graph_ms = None
            if not args.eager:
                try:
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g):
                        one()
                    for _ in range(3):
                        g.replay()
                    torch.cuda.synchronize()
                    graph_ms = timed_loop(g.replay)
                except Exception as e:      # noqa: BLE001
                    print("cascade step: graph capture failed, eager launches only:", e, file=sys.stderr)
            bad = [int(x.item()) for x in rc.status if int(x.item()) not in (0, 1)]
            if bad:
                raise SystemExit("bench.py: a device-resident review did not fit its launch shape")
            return (graph_ms if graph_ms is not None else eager_ms), int(rc.ctx_len.item()) - (t + 1), eager_ms, graph_ms is not None

        csd_ms, csd_emitted, csd_eager_ms, csd_graph = timed_chain([[n_from_draft_model, k_tail], [0, dk]])
        sd_ms, sd_emitted, sd_eager_ms, sd_graph = timed_chain([[k, 0], [0, 0]])
        # tokens per target review under Section 4's i.i.d. acceptance model at synthetic rates (random-init models
        # accept next to nothing, so the measured step times are combined with assumed rates; the rates are inputs)
        a_td, a_dm, a_tm = 0.6, 0.4, 0.3     # target keeps a draft-model token / draft model keeps a Max-Gram token / target keeps a Max-Gram token
        import numpy as _np
        rs = _np.random.RandomState(1)
        tot = 0
        trials = 20000
        for _ in range(trials):
            from_d = 0
            while from_d < n_from_draft_model:           # vertical cascade: the draft level's reviews of dk Max-Gram drafts
                kept = 0
                while kept < dk and rs.rand() < a_dm:
                    kept += 1
                from_d += kept + 1
            # the tokens a draft-level review kept are Max-Gram tokens (rate a_tm for the target), its own one per review has rate a_td
            n_kept = 0
            alive = True
            rem = from_d
            while alive and rem > 0:
                rate = a_td                               # conservative: treat every handed-up token at the draft model's rate
                if rs.rand() < rate:
                    n_kept += 1
                    rem -= 1
                else:
                    alive = False
            for _j in range(k_tail):
                if alive and rs.rand() < a_tm:
                    n_kept += 1
                else:
                    alive = False
            tot += n_kept + 1
        csd_tokens = tot / trials
        sd_tokens = ewif.expected_tokens(a_td, k)
        cascade = {"ms": round(csd_ms, 4), "steps": args.cascade_steps,
                   "launch": "hip graph replay" if csd_graph else "eager", "eager_ms": round(csd_eager_ms, 4),
                   "what": f"one step of Algorithm 1, K = [[{n_from_draft_model}, {k_tail}], [0, {dk}]]: the {dshape.name} model "
                           f"reviews {dk} Max-Gram drafts (twice when its first review yields one token; gated on the device), "
                           f"Max-Gram adds {k_tail}, the target reviews up to 16 rows against the draft level's own rows; "
                           "device-resident control, no host synchronisation",
                   "emitted_tokens_this_input": csd_emitted,
                   "sd_vs_csd": {"sd_ms": round(sd_ms, 4), "sd_what": f"plain speculative decoding: {k} one-row forwards of the "
                                 f"{dshape.name} model, then the target's review",
                                 "csd_ms": round(csd_ms, 4), "sd_eager_ms": round(sd_eager_ms, 4),
                                 "sd_launch": "hip graph replay" if sd_graph else "eager",
                                 "assumed_acceptance": {"target_vs_draft_model": a_td, "draft_model_vs_maxgram": a_dm,
                                                        "target_vs_maxgram": a_tm},
                                 "tokens_per_review_sd": round(sd_tokens, 3), "tokens_per_review_csd": round(csd_tokens, 3),
                                 "tokens_per_s_sd": round(sd_tokens / (sd_ms / 1e3), 1),
                                 "tokens_per_s_csd": round(csd_tokens / (csd_ms / 1e3), 1),
                                 "note": "step times measured here; tokens per review from Section 4's i.i.d. model at the "
                                         "assumed rates (Theorem 4.1 for SD, a simulation of the same model for the cascade)"}}
        del draft
        torch.cuda.empty_cache()

    # ---- what plain kernels reach on this machine (context for the fractions of the published peaks)
    peaks = None
    if not args.no_peaks:
        def timed(fn, reps):
            for _ in range(2):
                fn()
            torch.cuda.synchronize()
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(reps):
                fn()
            b.record()
            torch.cuda.synchronize()
            return a.elapsed_time(b) / 1e3 / reps
        sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")        # 1 GiB
        dst = torch.empty_like(src)
        nbytes = src.numel() * 4
        t_read = timed(lambda: P.debug_read(src, sink), 5)
        t_copy = timed(lambda: P.debug_copy(dst, src), 5)
        iters = 20000
        t_mfma = timed(lambda: P.debug_mfma(iters, sink), 3)
        peaks = {"hbm_read_GBs": round(nbytes / 1e9 / t_read, 1), "hbm_copy_GBs": round(2 * nbytes / 1e9 / t_copy, 1),
                 "mfma_bf16_dense_TFLOPs": round(4096 * iters * 8 * 16384 / 1e12 / t_mfma, 1),
                 "what": "1 GiB streaming read (16-byte loads, 2048 workgroups); 1 GiB copy, read + write counted; "
                         "4096 waves x 8 independent chains of 16x16x32 bf16 matrix instructions on registers"}
        del src, dst, sink
        torch.cuda.empty_cache()

    if args.copy_calibration > 0:
        src = torch.full((1 << 28,), 1.0, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(args.copy_calibration):
            P.debug_copy(dst, src)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU baseline: the oracle as it stands, one whole step on the host cores
    cpu = None
    if host_w is not None:
        import numpy as np

        from oracle import csd_oracle as O
        om = O.Model(shape, host_w, max_batch=1, max_seq=t + 64, max_block=max(m, 8))
        if shape.arch == 1:
            om.cross_kv_init(enc[:1].cpu().numpy())          # setup, not part of the timed step
        for l in range(shape.n_layers):
            K, V = I.synthetic_kv(shape, t, seed, l, 0, device="cuda")
            om.kv_write(l, 0, 0, K.cpu().numpy(), V.cpu().numpy())
        hctx = ctx[:1].cpu().numpy()
        htab = table.cpu().numpy()
        hq = q_draft[:1].cpu().numpy() if target_mix else None
        c0 = time.perf_counter()
        hb = block[:1].cpu().numpy().copy()
        if not target_mix:
            d, _ = O.bigram_draft(hctx, ctx_len[:1].cpu().numpy(), htab, k_tail)
            hb[:, 1 + n_from_draft_model:] = d
        lg = om.verify_block(hb, [t])
        pr = O.probs_f32(lg)
        on, ot = O.accept(pr, hq, hb[:, 1:], u_acc[:1].cpu().numpy(), u_samp[:1].cpu().numpy(), 1.0, mode)
        cpu_s = time.perf_counter() - c0
        # in-run parity of sequence 0 (untimed): the forward within the logit tolerance, and the accept
        # decision bit-identical when both sides are given the same distributions (the GPU's)
        g_lg, g_pr = model.verify_block(block[:1].contiguous(), cache_len[:1].contiguous(), want_probs=True)
        torch.cuda.synchronize()
        dl = float(np.abs(g_lg[0].cpu().numpy().astype(np.float64) - lg[0]).max())
        gn, gt = O.accept((g_lg if mode == 1 else g_pr).cpu().numpy(), hq, hb[:, 1:], u_acc[:1].cpu().numpy(), u_samp[:1].cpu().numpy(), 1.0, mode)
        cpu = {"value": round(k / cpu_s, 3), "unit": "verified tokens/s", "cores": O.threads(), "kind": "oracle",
               "sample": f"one whole step of sequence 0 (k={k} drafts, {t}-row cache): {cpu_s:.2f} s",
               "max_abs_dlogit_vs_gpu": round(dl, 6),
               "accept_identical_on_same_probs": bool(int(gn[0]) == int(n_acc[0].item()) and int(gt[0]) == int(nxt[0].item()))}
        del on, ot

    out = {
        "metric": "verified tokens/s per verify+accept step, 7B-shaped bf16; % HBM/MFMA roofline" if args.workload.startswith("target7b")
                  else f"verified tokens/s per verify+accept step, {shape.name}; % HBM/MFMA roofline",
        "value": round(B * k / (wall / args.steps), 2), "unit": "verified tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "gpu_ms_per_step": round(gpu_ms_per_step, 4),
        "median_ms_single_step": None if median_single_ms is None else round(median_single_ms, 4),
        "launch": "hip graph replay" if graph is not None else "eager", "settle_ms": args.settle_ms,
        "eager_ms_per_step": round(eager_ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: {shape.n_layers} layers, d_model {shape.d_model}, batch {B}, "
                               f"{t}-row KV cache" + (f", {shape.enc_len} encoder rows" if shape.arch == 1 else "") +
                               (f", block of k={k} drafts sampled from the reviewer's noise-perturbed distributions "
                                f"(expected acceptance {wl['acceptance']})" if target_mix else
                                f", block of k={k} drafts ({n_from_draft_model} stand-ins for the neural "
                                f"draft level + {k_tail} from Max-Gram)") + f", mode {args.mode}",
                   "batch": B, "prefix": t, "k": k},
        "emitted_tokens_per_s": round(emitted / (wall / args.steps), 2),
        "accepted_drafts_per_sequence": round(float(n_acc.float().mean().item()), 3),
        "setup_s": round(setup_s, 1),
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if cascade is not None:
        out["cascade_step"] = cascade
    if tree is not None:
        out["tree_step"] = tree
    if peaks is not None:
        out["measured_peaks"] = peaks
    print(json.dumps(out))


if __name__ == "__main__":
    main()
