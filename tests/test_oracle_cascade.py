"""Pin: greedy cascaded decoding emits exactly the target's own greedy tokens (Sections 3.1
and 5.1: temperature 0, no lenience when the target reviews), for vertical + horizontal
cascades of several depths, with and without lenience between draft levels (CPU only)."""
import numpy as np
import pytest

import csd_inputs as I
from oracle import csd_oracle as O
from oracle.cascade import Level, autoregressive, cascade_generate

TARGET = I.ModelShape("t", 0, "fp32", 2, 64, 4, 16, 256, 512)
DRAFT1 = I.ModelShape("d1", 0, "fp32", 1, 32, 2, 16, 64, 512)
DRAFT2 = I.ModelShape("d2", 0, "fp32", 1, 16, 2, 8, 32, 512)


def _level(shape, seed, std=0.02):
    w = I.make_weights(shape, seed, std=std)
    lv = Level(O.Model(shape, w, max_batch=1, max_seq=160, max_block=16), 16)
    lv._keep = w
    return lv


@pytest.mark.parametrize("K,lenience,n_drafts", [
    ([[4]], 1.0, 0),                       # Max-Gram alone drafts for the target
    ([[2, 6], [0, 6]], 1.0, 1),            # the decoder-only setting's shape (Appendix B)
    ([[2, 6], [0, 6]], 3.0, 1),
    ([[2, 2, 4], [0, 1, 3], [0, 0, 3]], 2.0, 2),
])
def test_greedy_cascade_equals_target_greedy(K, lenience, n_drafts):
    prompt = I.token_ids(24, 512, 21, 1).tolist()
    prompt = prompt[:12] + prompt[:12]          # a repeated phrase so Max-Gram has matches
    table = O.bigram_fit(np.array(prompt, np.int32), 512, I.default_next_table(512, 1).numpy())
    # std 0.2: logits far enough apart that fp64 arg-max is stable between block shapes
    target = _level(TARGET, 1, std=0.2)
    want = autoregressive(target, prompt, 40)
    levels = [target] + [_level(s, 2 + i, std=0.2) for i, s in enumerate((DRAFT1, DRAFT2)[:n_drafts])]
    got, steps = cascade_generate(levels, table, prompt, 40, K, lenience=lenience, mode=1)
    assert got == want
    assert steps <= 40


def test_draft_identical_to_target_accepts_everything():
    """k drafts from a model identical to the target are all kept (q = p, Section 2)."""
    prompt = I.token_ids(10, 512, 22, 1).tolist()
    table = I.default_next_table(512, 1).numpy()
    target = _level(TARGET, 1, std=0.2)
    twin = _level(TARGET, 1, std=0.2)
    want = autoregressive(target, prompt, 24)
    got, steps = cascade_generate([target, twin], table, prompt, 24, [[3, 0], [0, 1]], mode=1)
    assert got == want
    # every target step keeps the twin's drafts (>= 3) and adds one token
    assert steps <= 24 // 4 + 1


def test_sampling_cascade_runs_and_is_reproducible():
    prompt = I.token_ids(16, 512, 23, 1).tolist()
    table = I.default_next_table(512, 1).numpy()
    levels = [_level(TARGET, 1, std=0.2), _level(DRAFT1, 2, std=0.2)]
    outs = []
    for _ in range(2):
        u = iter(I.uniforms(4000, 5, 5).tolist())
        outs.append(cascade_generate(levels, table, prompt, 20, [[2, 4], [0, 4]], mode=0, uniforms=u)[0])
    assert outs[0] == outs[1] and len(outs[0]) == 20


class _FixedLevel:
    """A "model" whose next-token distribution does not depend on the context: what the i.i.d. acceptance
    assumption of Section 4 describes.  Same interface as Level (rows_from, cached)."""

    def __init__(self, p):
        self.logits = np.log(np.asarray(p, np.float64))
        self.cached = 0

    def rows_from(self, seq, first_row):
        return np.tile(self.logits, (len(seq) - first_row, 1))


def _uniform_stream(seed):
    rs = np.random.RandomState(seed)
    while True:
        for u in rs.randint(0, 1 << 24, size=4096):
            yield float(u) / float(1 << 24)


def _alpha(p, q):
    """Acceptance rate of drafts from q under reviewer p (Section 2): sum_x min(p(x), q(x))."""
    return float(np.minimum(p.astype(np.float64), q.astype(np.float64)).sum())


P_T = [0.40, 0.25, 0.15, 0.12, 0.08]
P_1 = [0.30, 0.30, 0.20, 0.10, 0.10]     # close to the target
P_2 = [0.05, 0.15, 0.10, 0.20, 0.50]     # far from it


def test_sampling_horizontal_cascade_tokens_per_review_match_theorem_4_3():
    """Horizontal cascade, sampling: the first 3 drafts come from a model with acceptance alpha_1, the next 2
    from one with alpha_2 (each drafted one token at a time: no drafts below them).  Theorem 4.3: a review
    emits sum_{i=0..k} prod_{j<=i} alpha_j tokens on average.  And whatever the drafts, the emitted tokens
    follow the target's own distribution (Section 2)."""
    levels = [_FixedLevel(P_T), _FixedLevel(P_1), _FixedLevel(P_2)]
    pt, p1, p2 = (O.probs_f32(lv.logits[None])[0] for lv in levels)
    a1, a2 = _alpha(pt, p1), _alpha(pt, p2)
    alphas = [a1, a1, a1, a2, a2]
    want = sum(float(np.prod(alphas[:i])) for i in range(6))
    n_new = 60000
    table = np.zeros(5, np.int32)
    got, steps = cascade_generate(levels, table, [0, 1, 2], n_new, [[3, 2, 0], [0, 0, 0], [0, 0, 0]], mode=0,
                                  uniforms=_uniform_stream(11))
    mean = n_new / steps
    # a review emits between 1 and 6 tokens: its standard deviation is below 2
    assert abs(mean - want) < 4 * 2.0 / np.sqrt(steps), (mean, want)
    # a swapped or dropped alpha would move the mean by far more than that
    wrong = sum(float(np.prod(([a2] * 3 + [a1] * 2)[:i])) for i in range(6))
    assert abs(wrong - want) > 20 * 2.0 / np.sqrt(steps)
    counts = np.bincount(got, minlength=5).astype(np.float64)
    chi2 = float(((counts - n_new * pt) ** 2 / (n_new * pt)).sum())
    assert chi2 < 18.47, chi2            # 4 degrees of freedom, p = 0.001


def test_sampling_vertical_cascade_emits_target_distribution_and_expected_length():
    """Vertical cascade, sampling: level 1 reviews blocks of 3 drafts of level 2 (Theorem 4.1's length law
    with alpha' between them) until at least 4 of its tokens exist, then the target reviews them.  The
    emitted tokens follow the target's distribution, and the mean tokens per target review is
    E[(1 - alpha^(N+1)) / (1 - alpha)] with N the block length, computed here from Theorem 4.1's law by
    running the renewal "steps until >= 4 tokens" exactly."""
    levels = [_FixedLevel(P_T), _FixedLevel(P_1), _FixedLevel(P_2)]
    pt, p1, p2 = (O.probs_f32(lv.logits[None])[0] for lv in levels)
    a, ap = _alpha(pt, p1), _alpha(p1, p2)
    k2, k1 = 3, 4
    # Theorem 4.1: a step of level 1 emits i tokens with probability alpha'^(i-1) (1 - alpha') for i <= k2, alpha'^k2 for k2 + 1
    law = {i: ap ** (i - 1) * (1 - ap) for i in range(1, k2 + 1)}
    law[k2 + 1] = ap ** k2
    dist = {0: 1.0}                      # tokens so far -> probability, while fewer than k1
    final = {}
    while dist:
        nxt = {}
        for n, pr in dist.items():
            for i, pi in law.items():
                tgt = final if n + i >= k1 else nxt
                tgt[n + i] = tgt.get(n + i, 0.0) + pr * pi
        dist = nxt
    assert abs(sum(final.values()) - 1.0) < 1e-12
    want = sum(pr * (1 - a ** (n + 1)) / (1 - a) for n, pr in final.items())
    n_new = 60000
    got, steps = cascade_generate(levels, np.zeros(5, np.int32), [0, 1, 2], n_new,
                                  [[k1, 0, 0], [0, k2, 0], [0, 0, 0]], lenience=1.0, mode=0,
                                  uniforms=_uniform_stream(12))
    mean = n_new / steps
    assert abs(mean - want) < 4 * 2.5 / np.sqrt(steps), (mean, want)
    counts = np.bincount(got, minlength=5).astype(np.float64)
    chi2 = float(((counts - n_new * pt) ** 2 / (n_new * pt)).sum())
    assert chi2 < 18.47, chi2
