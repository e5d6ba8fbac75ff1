"""The hot path under HIP graph capture: one step (Max-Gram draft into the block, review forward, review) is captured
once and replayed; every replay must give what the same calls give eagerly on the same inputs, also after the inputs
in the captured buffers changed and with eager work of the same model between the replays.  The library allocates
nothing per call, clears its counters with kernels (not memsets) and launches on the caller's stream, which is what
capture needs; csd_verify_accept_static is the entry point meant for it."""
import numpy as np
import pytest
import torch

import csd_inputs as I

pytestmark = pytest.mark.gpu

SHAPE = I.ModelShape("graph_bf", 0, "bf16", 3, 256, 4, 64, 512, 1024)


@pytest.mark.parametrize("static", [False, True], ids=["model_scratch", "static_scratch"])
def test_captured_step_replays_to_the_eager_result(static):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2312_11462_amd as P
    seed, t, k = 77, 96, 5
    w = I.make_weights(SHAPE, seed, device="cuda", std=0.05)
    gm = P.Model(SHAPE, w, max_batch=1, max_seq=160, max_block=8)
    assert gm.path(1, k + 1) == 1
    toks = I.repeat_stream(t + 1, SHAPE.vocab, seed, 3)
    for pos in range(0, t, 8):
        gm.verify_block(toks[None, pos:pos + 8].contiguous().cuda(), torch.tensor([pos], dtype=torch.int32).cuda())
    ctx = torch.zeros((1, 160), dtype=torch.int32, device="cuda")
    ctx[0, :t + 1] = toks.cuda()
    ctx_len = torch.tensor([t + 1], dtype=torch.int32, device="cuda")
    table = P.bigram_fit(ctx[0, :t + 1], SHAPE.vocab, I.default_next_table(SHAPE.vocab, seed).cuda())
    block = torch.zeros((1, k + 1), dtype=torch.int32, device="cuda")
    block[0, 0] = toks[t]
    cl = torch.tensor([t], dtype=torch.int32, device="cuda")
    u_acc = I.uniforms(k, seed, 1).reshape(1, k).contiguous().cuda()
    u_s = I.uniforms(1, seed, 2).cuda()
    n = torch.zeros(1, dtype=torch.int32, device="cuda")
    x = torch.zeros(1, dtype=torch.int32, device="cuda")
    lg = torch.zeros((1, k + 1, SHAPE.vocab), dtype=torch.float32, device="cuda")
    onehot = torch.ones(k, dtype=torch.uint8, device="cuda")

    def step():
        P.bigram_draft(ctx, ctx_len, table, k, want_match_len=False, out=block[:, 1:])
        gm.verify_accept(block, cl, u_acc, u_s, q=None, q_onehot=onehot, logits=lg, n_accepted=n, next_token=x, static=static)

    def eager():
        step()
        torch.cuda.synchronize()
        return lg.clone(), n.clone(), x.clone(), block.clone()

    want0 = eager()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    inputs = [(u_s.clone(), ctx[0, t].clone())]
    inputs.append((I.uniforms(1, seed, 9).cuda(), ((ctx[0, t] + 5) % SHAPE.vocab).clone()))
    inputs.append((I.uniforms(1, seed, 10).cuda(), ((ctx[0, t] + 11) % SHAPE.vocab).clone()))
    for rep, (us_new, last_tok) in enumerate(inputs):
        u_s.copy_(us_new)                      # new contents in the captured buffers: another uniform, another last token
        ctx[0, t] = last_tok
        block[0, 0] = last_tok
        want = eager()
        lg.zero_(); n.fill_(-7); x.fill_(-7); block[0, 1:] = -1
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(lg, want[0]) and torch.equal(n, want[1]) and torch.equal(x, want[2]) and torch.equal(block, want[3]), rep
        # eager work of the same model between replays (it uses the same scratch and counters)
        # (it rewrites cache rows 8..15 with the values they already hold: same tokens, same positions)
        gm.verify_block(toks[None, 8:16].contiguous().cuda(), torch.tensor([8], dtype=torch.int32).cuda())
    torch.cuda.synchronize()
    assert not torch.equal(want0[0], lg)       # the last replay saw other inputs than the first eager run
