"""Pins of the oracle's Max-Gram / bigram draft (CPU only): the worked cases of
tests/golden/maxgram_cases.txt (Appendix A's matching rule), brute force on tiny alphabets,
and the invariants of Section 3.3."""
import os

import numpy as np
import pytest

import csd_inputs as I
from oracle import csd_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "maxgram_cases.txt")


def _cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        hay, needle, k, exp, mlen, _ = [c.strip() for c in line.split("|")]
        out.append(([int(x) for x in hay.split()], [int(x) for x in needle.split()], int(k),
                    [int(x) for x in exp.split()], int(mlen)))
    return out


@pytest.mark.parametrize("hay,needle,k,exp,mlen", _cases())
def test_worked_cases(hay, needle, k, exp, mlen):
    ctx = hay + [99] + needle
    table = (np.arange(100, dtype=np.int32) + 1) % 100
    out, got_len = O.bigram_draft(np.array(ctx, np.int32), [len(ctx)], table, k)
    assert out[0].tolist() == exp
    assert got_len[0] == mlen


def _brute(s, k, table):
    """Independent definition: among all proper occurrences of suffixes of s inside s, take the
    longest, then the left-most; emit one token; repeat on the extended sequence."""
    s = list(s)
    out = []
    for _ in range(k):
        n = len(s)
        best = (0, None)
        for r in range(n - 1, 0, -1):               # suffix length, longest first
            suf = s[n - r:]
            hits = [st for st in range(0, n - r) if s[st:st + r] == suf]   # start < n-r: not the suffix itself
            if hits:
                best = (r, hits[0] + r - 1)         # end index of the left-most occurrence
                break
        if best[1] is None:
            if out:
                raise AssertionError("a match can not disappear once found")
            cur = s[-1]                             # no occurrence at all: the bigram model drafts the block
            for _ in range(k):
                cur = int(table[cur])
                out.append(cur)
            return out
        else:
            tok = s[best[1] + 1]
        out.append(tok)
        s.append(tok)
    return out


@pytest.mark.parametrize("alphabet,length", [(2, 9), (3, 12), (3, 30), (5, 40)])
def test_brute_force_on_tiny_alphabets(alphabet, length):
    """One pass with the self-extending continuation equals re-matching after every token."""
    table = I.default_next_table(alphabet, 5).numpy()
    for trial in range(60):
        n = 1 + (trial * 7) % length
        s = I.token_ids(n, alphabet, 100 + alphabet, trial).numpy()
        k = 1 + trial % 6
        out, mlen = O.bigram_draft(s, [n], table, k)
        assert out[0].tolist() == _brute(s.tolist(), k, table), (s.tolist(), k)


def test_invariants_on_repeat_stream():
    V = 300
    s = I.repeat_stream(400, V, 3, 1).numpy()
    table = I.default_next_table(V, 9).numpy()
    for n in range(2, 400, 13):
        out, mlen = O.bigram_draft(s[:n], [n], table, 6)
        seen_before = s[n - 1] in s[:n - 1]
        assert (mlen[0] > 0) == bool(seen_before)
        if mlen[0] == 0:
            assert out[0, 0] == table[s[n - 1]] and out[0, 1] == table[out[0, 0]]
        else:
            ext = s[:n].tolist() + out[0].tolist()
            # the draft continues an earlier occurrence of the matched suffix
            L = mlen[0]
            starts = [st for st in range(0, n - L) if ext[st:st + L] == ext[n - L:n]]
            assert starts and ext[starts[0] + L:starts[0] + L + 6] == out[0].tolist()
            # and no longer suffix occurs earlier
            if n - L - 1 >= 0 and L + 1 <= n - 1:
                suf = ext[n - L - 1:n]
                assert not any(ext[st:st + L + 1] == suf for st in range(0, n - L - 1))


def test_match_cap_and_batching():
    s = np.array([1, 2, 3, 4, 9, 2, 3, 4, 8, 1, 2, 3, 4], np.int32)
    table = np.zeros(10, np.int32)
    out, mlen = O.bigram_draft(s, [13], table, 2)
    assert (out[0].tolist(), mlen[0]) == ([9, 2], 4)
    out, mlen = O.bigram_draft(s, [13], table, 2, max_match=3)      # capped: both occurrences tie, left-most wins
    assert (out[0].tolist(), mlen[0]) == ([9, 2], 3)
    ctx = np.zeros((2, 16), np.int32)
    ctx[0, :13] = s
    ctx[1, :5] = [4, 4, 5, 6, 4]
    out, mlen = O.bigram_draft(ctx, [13, 5], table, 3)
    assert out.tolist() == [[9, 2, 3], [4, 5, 6]] and mlen.tolist() == [4, 1]


def test_bigram_fit():
    V = 8
    base = np.full(V, 7, np.int32)
    s = np.array([1, 2, 1, 3, 1, 3, 1, 2, 5], np.int32)
    t = O.bigram_fit(s, V, base)
    # (1,2) x2 and (1,3) x2: the pair seen latest (1,2 at index 6) wins; 5 has no successor
    assert t.tolist() == [7, 2, 5, 1, 7, 7, 7, 7]
    s = np.array([1, 2, 1, 2, 1, 3], np.int32)
    assert O.bigram_fit(s, V, base)[1] == 2       # majority beats recency
    # agreement with a dense count matrix on random streams
    for trial in range(20):
        s = I.token_ids(50, V, 31, trial).numpy()
        cnt = np.zeros((V, V), int)
        last = np.full((V, V), -1)
        for i in range(len(s) - 1):
            cnt[s[i], s[i + 1]] += 1
            last[s[i], s[i + 1]] = i
        want = base.copy()
        for a in range(V):
            if cnt[a].sum():
                m = cnt[a].max()
                cands = [b for b in range(V) if cnt[a, b] == m]
                want[a] = max(cands, key=lambda b: last[a, b])
        assert O.bigram_fit(s, V, base).tolist() == want.tolist()


def test_fit_on_prefix_makes_fallback_fire_only_for_unseen_tokens():
    """A table fitted on the same sequence has an entry for token a exactly when Max-Gram finds a
    match of length >= 1, so the fallback only ever reads the caller's default entries."""
    V = 50
    s = I.token_ids(60, V, 77, 1).numpy()
    default = I.default_next_table(V, 4).numpy()
    table = O.bigram_fit(s, V, default)
    for n in range(2, 60):
        out, mlen = O.bigram_draft(s[:n], [n], O.bigram_fit(s[:n], V, default), 1)
        if mlen[0] == 0:
            assert out[0, 0] == default[s[n - 1]]
    assert table.shape == (V,)


# ---------------------------------------------------------------- separate haystack (Appendix A's signature)

ENC_GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "maxgram_encoder_cases.txt")


def _enc_cases():
    out = []
    for line in open(ENC_GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        hay, needle, k, exp, mlen = [c.strip() for c in line.split("|")]
        exp_t = None if exp == "None" else ([] if exp == "-" else [int(x) for x in exp.split()])
        out.append(([int(x) for x in hay.split()], [int(x) for x in needle.split()], int(k), exp_t, int(mlen)))
    return out


@pytest.mark.parametrize("hay,needle,k,exp,mlen", _enc_cases())
def test_encoder_side_worked_cases(hay, needle, k, exp, mlen):
    table = (np.arange(100, dtype=np.int32) + 1) % 100
    out, got_len, n_copied = O.maxgram_draft(hay, [len(hay)], needle, [len(needle)], table, k)
    assert got_len[0] == mlen
    want = [] if exp is None else exp
    assert n_copied[0] == len(want) and out[0, :len(want)].tolist() == want
    # what is not copied chains the bigram table from the last token so far
    cur = want[-1] if want else needle[-1]
    for j in range(len(want), k):
        cur = (cur + 1) % 100
        assert out[0, j] == cur


def _enc_brute(hay, needle):
    """Independent definition: the largest r such that needle[-r:] occurs in hay, and the smallest start."""
    for r in range(min(len(needle), len(hay)), 0, -1):
        suf = needle[-r:]
        for st in range(0, len(hay) - r + 1):
            if hay[st:st + r] == suf:
                return r, st + r - 1
    return 0, -1


def test_encoder_side_brute_force_small_alphabet():
    rng = np.random.default_rng(7)
    table = np.array([2, 0, 1], np.int32)
    for _ in range(400):
        hay = rng.integers(0, 3, size=int(rng.integers(0, 12))).tolist()
        needle = rng.integers(0, 3, size=int(rng.integers(1, 9))).tolist()
        k = int(rng.integers(0, 6))
        hp = hay + [0] * (12 - len(hay))
        out, mlen, ncp = O.maxgram_draft(np.array(hp, np.int32), [len(hay)], needle, [len(needle)], table, k)
        r, e = _enc_brute(hay, needle)
        assert mlen[0] == r
        copied = hay[e + 1:e + 1 + k] if r else []
        assert ncp[0] == len(copied) and out[0, :len(copied)].tolist() == copied
        cur = copied[-1] if copied else needle[-1]
        for j in range(len(copied), k):
            cur = int(table[cur])
            assert out[0, j] == cur


def test_encoder_side_match_cap_and_reduction_to_self_search():
    # with the cap the match length saturates but the left-most rule still holds
    hay = [1, 2, 3, 9, 1, 2, 3]
    out, mlen, ncp = O.maxgram_draft(hay, [7], [1, 2, 3], [3], np.zeros(10, np.int32), 2, max_match=2)
    assert mlen[0] == 2 and out[0].tolist() == [9, 1]
    # a context searched in itself without its last position is the decoder-only form
    s = I.repeat_stream(200, 50, 3, 1).numpy()
    table = I.default_next_table(50, 3).numpy()
    a, la = O.bigram_draft(s, [200], table, 4)
    b, lb, nb = O.maxgram_draft(s[:199], [199], s, [200], table, 4)
    assert la[0] == lb[0]
    assert a[0, :nb[0]].tolist() == b[0, :nb[0]].tolist()
