"""GPU parity of the integer paths through the C ABI: Max-Gram / bigram draft and the
accept / resample step must match the oracle bit for bit on the same seeded inputs."""
import numpy as np
import pytest
import torch

import csd_inputs as I

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def P():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2312_11462_amd as P
    P.lib()
    return P


def _O():
    from oracle import csd_oracle as O
    return O


def test_bigram_draft_matches_oracle(P):
    O = _O()
    for V, n_max, seed in [(3, 40, 1), (5, 300, 2), (300, 700, 3), (32000, 2048, 4)]:
        B, stride = 7, n_max
        ctx = torch.zeros((B, stride), dtype=torch.int32)
        lens = []
        for b in range(B):
            n = max(1, (n_max * (b + 1)) // B - (b % 3))
            s = I.repeat_stream(n, V, seed, b) if V > 5 else I.token_ids(n, V, seed, b)
            ctx[b, :n] = s
            lens.append(n)
        lens[0] = 1                                   # degenerate: single token -> fallback
        table = I.default_next_table(V, seed)
        for k, cap in [(1, 0), (6, 0), (10, 0), (10, 3), (0, 0)]:
            want, wlen = O.bigram_draft(ctx.numpy(), lens, table.numpy(), k, cap)
            got, glen = P.bigram_draft(ctx.cuda(), torch.tensor(lens, dtype=torch.int32).cuda(), table.cuda(), k, cap)
            assert np.array_equal(got.cpu().numpy(), want), (V, k, cap)
            assert np.array_equal(glen.cpu().numpy(), wlen), (V, k, cap)


def test_maxgram_with_separate_haystack_matches_oracle(P):
    """Appendix A's own signature: the needle's longest suffix inside a haystack of its own (the prompt /
    encoder ids), several sequences with ragged lengths, empty haystack, needle longer than the haystack,
    match cap, k = 0."""
    O = _O()
    for V, hs, ns, seed in [(3, 30, 12, 1), (5, 200, 40, 2), (300, 700, 300, 3), (32000, 2048, 600, 4)]:
        B = 6
        hay = torch.zeros((B, hs), dtype=torch.int32)
        ned = torch.zeros((B, ns), dtype=torch.int32)
        hl, nl = [], []
        for b in range(B):
            n = (hs * (b + 1)) // B
            src = I.repeat_stream(n + ns, V, seed, b) if V > 5 else I.token_ids(n + ns, V, seed, b)
            hay[b, :n] = src[:n]
            # the needle: a stretch that recurs in the haystack, followed by a few fresh tokens
            m = max(1, ns - b)
            ned[b, :m] = torch.cat([src[max(0, n // 2 - m):n // 2], src[n:n + ns]])[:m] if n >= 2 else src[:m]
            hl.append(n)
            nl.append(m)
        hl[0] = 0                                      # degenerate: nothing to search -> bigram chain
        table = I.default_next_table(V, seed)
        for k, cap in [(1, 0), (6, 0), (10, 3), (0, 0)]:
            want = O.maxgram_draft(hay.numpy(), hl, ned.numpy(), nl, table.numpy(), k, cap)
            got = P.maxgram_draft(hay.cuda(), torch.tensor(hl, dtype=torch.int32).cuda(), ned.cuda(),
                                  torch.tensor(nl, dtype=torch.int32).cuda(), table.cuda(), k, cap)
            for g, w, name in zip(got, want, ("tokens", "match length", "copied")):
                assert np.array_equal(g.cpu().numpy(), w), (V, k, cap, name)


def test_bigram_fit_matches_oracle(P):
    O = _O()
    for V, n, seed in [(8, 50, 1), (64, 1000, 2), (32000, 2048, 3), (32000, 8192, 4), (10, 2, 5), (10, 1, 6)]:
        s = I.repeat_stream(n, V, seed, 9) if n > 4 else I.token_ids(n, V, seed, 9)
        default = I.default_next_table(V, seed)
        want = O.bigram_fit(s.numpy(), V, default.numpy())
        got = P.bigram_fit(s.cuda(), V, default.cuda().clone())
        assert np.array_equal(got.cpu().numpy(), want), (V, n)


def _rand_dist(shape, seed, stream, sharp):
    x = I.normal(shape, sharp, seed, stream)
    return torch.softmax(x.double(), dim=-1).float().contiguous()


@pytest.mark.parametrize("V,B,k", [(7, 64, 3), (1000, 16, 5), (32000, 8, 16), (32000, 1, 5), (32128, 3, 1), (5, 9, 0)])
def test_accept_matches_oracle_bit_exact(P, V, B, k):
    O = _O()
    seed = 1000 + V + k
    p = _rand_dist((B, k + 1, V), seed, 1, 2.0)
    q = _rand_dist((B, max(k, 1), V), seed, 2, 2.0)[:, :k].contiguous()
    # drafts drawn from q so that acceptance is neither rare nor certain
    u = I.uniforms(B * max(k, 1), seed, 3).reshape(B, max(k, 1))[:, :k]
    draft = (torch.cumsum(q.double(), -1) <= u[..., None].double()).sum(-1).clamp(max=V - 1).int().contiguous()
    u_acc = I.uniforms(B * max(k, 1), seed, 4).reshape(B, max(k, 1))[:, :k].contiguous()
    u_s = I.uniforms(B, seed, 5)
    onehot = (I.token_ids(max(k, 1), 2, seed, 6)[:k]).to(torch.uint8)
    cases = [dict(q=q, lenience=1.0, mode=0, oh=None), dict(q=None, lenience=1.0, mode=0, oh=None),
             dict(q=q, lenience=2.5, mode=0, oh=None), dict(q=q, lenience=1.0, mode=0, oh=onehot),
             dict(q=None, lenience=1.0, mode=1, oh=None), dict(q=q, lenience=3.0, mode=1, oh=onehot)]
    for c in cases:
        if k == 0 and c["q"] is not None:
            continue
        qn = None if c["q"] is None else c["q"].numpy()
        ohn = None if c["oh"] is None else c["oh"].numpy()
        wn, wt = O.accept(p.numpy(), qn, draft.numpy(), u_acc.numpy(), u_s.numpy(), c["lenience"], c["mode"], ohn)
        gn, gt = P.accept(p.cuda(), None if c["q"] is None else c["q"].cuda(), draft.cuda(), u_acc.cuda(), u_s.cuda(),
                          c["lenience"], c["mode"], None if c["oh"] is None else c["oh"].cuda())
        assert np.array_equal(gn.cpu().numpy(), wn), c
        assert np.array_equal(gt.cpu().numpy(), wt), c


def test_accept_greedy_on_logits_with_ties(P):
    O = _O()
    V, B, k = 515, 6, 4
    lg = torch.round(I.normal((B, k + 1, V), 3.0, 5, 1))        # integers: many exact ties
    draft = lg[:, :k].argmax(-1).int()                           # torch picks some arg-max; only the first must pass
    draft[2, 1] = 3
    wn, wt = O.accept(lg.numpy(), None, draft.numpy(), np.zeros((B, k), np.float32), np.zeros(B, np.float32), 1.0, 1)
    gn, gt = P.accept(lg.cuda(), None, draft.cuda(), torch.zeros((B, k)).cuda(), torch.zeros(B).cuda(), 1.0, 1)
    assert np.array_equal(gn.cpu().numpy(), wn) and np.array_equal(gt.cpu().numpy(), wt)


def test_identical_draft_accepts_all_and_errors_are_reported(P):
    V, B, k = 1000, 4, 6
    p = _rand_dist((B, k + 1, V), 77, 1, 1.0)
    draft = I.token_ids(B * k, V, 77, 2).reshape(B, k).contiguous()
    u = torch.full((B, k), 1 - 2.0 ** -24)
    gn, _ = P.accept(p.cuda(), p[:, :k].contiguous().cuda(), draft.cuda(), u.cuda(), torch.zeros(B).cuda())
    assert (gn.cpu().numpy() == k).all()
    with pytest.raises(P.CsdError):
        P.accept(p.cuda(), None, draft.cuda(), u.cuda(), torch.zeros(B).cuda(), lenience=0.5)


def test_accept_long_blocks_odd_vocab_and_invalid_draft_ids(P):
    """More drafts than one wave of acceptance tests (k = 70) and a vocabulary that is not a multiple of 4
    (rows are not 16-byte aligned), against the oracle; then draft ids outside the vocabulary, which the
    kernel's bounds check turns into a rejection at that position (the oracle refuses such input)."""
    O = _O()
    V, B, k = 1001, 3, 70
    seed = 4242
    p = _rand_dist((B, k + 1, V), seed, 1, 3.0)
    draft = p[:, :k].argmax(-1).int().contiguous()          # likely accepted: long accepted prefixes
    u_acc = (I.uniforms(B * k, seed, 4).reshape(B, k) * 0.05).contiguous()
    u_s = I.uniforms(B, seed, 5)
    for mode, lenience in [(0, 1.0), (0, 2.0), (1, 1.0)]:
        wn, wt = O.accept(p.numpy(), None, draft.numpy(), u_acc.numpy(), u_s.numpy(), lenience, mode)
        gn, gt = P.accept(p.cuda(), None, draft.cuda(), u_acc.cuda(), u_s.cuda(), lenience, mode)
        assert np.array_equal(gn.cpu().numpy(), wn) and np.array_equal(gt.cpu().numpy(), wt), (mode, lenience)
    assert wn.max() > 64                                       # the second batch of 64 acceptance tests was reached
    bad = draft.clone()
    bad[1, 66] = V + 5
    bad[2, 0] = -1
    gn, gt = P.accept(p.cuda(), None, bad.cuda(), torch.zeros((B, k)).cuda(), u_s.cuda(), 1.0, 0)
    gn, gt = gn.cpu().numpy(), gt.cpu().numpy()
    assert gn[1] == 66 and gn[2] == 0 and (0 <= gt).all() and (gt < V).all()


def test_out_of_range_draft_is_a_rejection_drawn_from_the_reviewers_row(P):
    """A draft id outside [0, V) cannot be validated on the host.  The kernel treats it as a rejection at that
    position and draws the replacement from the reviewer's row there, with or without dense draft rows: the
    same outcome as the oracle gives for the block cut before that position (the draw of the extra token
    from that row with the same uniform)."""
    O = _O()
    B, k, V, seed = 3, 5, 300, 31
    p = _rand_dist((B, k + 1, V), seed, 1, 3.0)
    q = _rand_dist((B, k, V), seed, 2, 3.0)
    draft = p[:, :k, :].argmax(-1).to(torch.int32)            # likely accepted drafts
    u_acc = torch.zeros((B, k), dtype=torch.float32)           # u = 0: every valid draft with p > 0 is accepted
    u_s = I.uniforms(B, seed, 3)
    for bad_pos, bad_id in [(0, -1), (2, V), (4, 1 << 30)]:
        d = draft.clone()
        d[:, bad_pos] = bad_id
        for dense in (False, True):
            gn, gt = P.accept(p.cuda(), q.cuda() if dense else None, d.cuda(), u_acc.cuda(), u_s.cuda())
            on, ot = O.accept(p[:, :bad_pos + 1].numpy(), q[:, :bad_pos].numpy() if dense else None, d[:, :bad_pos].numpy(),
                              u_acc[:, :bad_pos].numpy(), u_s.numpy())
            assert np.array_equal(gn.cpu().numpy(), on) and (on == bad_pos).all()
            assert np.array_equal(gt.cpu().numpy(), ot)
