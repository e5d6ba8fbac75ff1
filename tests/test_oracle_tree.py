"""Pins of the oracle's tree review (CPU only): Section 5.1 combines the cascade with tree attention, Appendix B
gives the lead node eight children; the paper says no more, so the functions are pinned to what defines them:

  * a row of a tree block sees exactly its own root-to-node path, so its logits are those of the library
    whole-sequence forward over prefix + path (a wrong mask, a position taken from the storage slot instead of
    the depth, or a K/V row stored in the wrong slot fails this);
  * a chain-shaped tree is the plain block;
  * after the kept path's rows are moved, the cache is that of the kept sequence;
  * greedy decoding through trees of arbitrary content emits the reviewer's own greedy continuation (Sections 3.1,
    5.1: the output is not altered);
  * in sampling mode the emitted tokens follow the reviewer's law whatever the tree holds (exact counts over
    uniform grids).
"""
import numpy as np
import pytest
import torch

import csd_inputs as I
from oracle import csd_oracle as O
from test_oracle_forward import SHAPE, _torch_forward, _weights


def _random_tree(m, rng, max_children=3):
    parent = [-1]
    for i in range(1, m):
        cands = [j for j in range(i) if sum(1 for p in parent if p == j) < max_children]
        parent.append(int(rng.choice(cands)))
    return np.array(parent, np.int32)


def _path_to(parent, i):
    out = []
    while i > 0:
        out.append(i)
        i = parent[i]
    return out[::-1]


def test_every_row_of_a_tree_block_sees_its_own_path_library_forward():
    w = _weights()
    om = O.Model(SHAPE, w, max_batch=1, max_seq=40, max_block=16)
    rng = np.random.default_rng(3)
    prefix = rng.integers(0, SHAPE.vocab, 6).astype(np.int32)
    om.verify_block(prefix[None, :5], [0])                       # rows 0..4 cached; the block starts at prefix[5]
    m = 11
    parent = _random_tree(m, rng)
    assert len(set(_path_len for _path_len in map(lambda i: len(_path_to(parent, i)), range(m)))) > 2   # real branching
    tokens = np.concatenate([prefix[5:], rng.integers(0, SHAPE.vocab, m - 1)]).astype(np.int32)
    lg = om.verify_tree(tokens[None], parent[None], [5])[0]
    for i in range(m):
        seq = list(prefix) + [int(tokens[j]) for j in _path_to(parent, i)]
        ref = np.asarray(_torch_forward(SHAPE, w, seq))[-1]
        assert np.abs(lg[i] - ref).max() < 1e-9, i


def test_a_chain_shaped_tree_is_the_plain_block():
    w = _weights()
    a = O.Model(SHAPE, w, max_batch=2, max_seq=32, max_block=8)
    b = O.Model(SHAPE, w, max_batch=2, max_seq=32, max_block=8)
    rng = np.random.default_rng(5)
    toks = rng.integers(0, SHAPE.vocab, (2, 12)).astype(np.int32)
    for mdl in (a, b):
        mdl.verify_block(toks[:, :6], [0, 0])
    chain = np.tile(np.arange(-1, 5, dtype=np.int32), (2, 1))
    x = a.verify_block(toks[:, 6:12], [6, 6])
    y = b.verify_tree(toks[:, 6:12], chain, [6, 6])
    assert np.array_equal(x, y) and np.array_equal(a.kv, b.kv)


def test_parents_must_come_before_their_children():
    om = O.Model(SHAPE, _weights(), max_batch=1, max_seq=32, max_block=8)
    toks = np.zeros((1, 4), np.int32)
    for bad in ([0, 0, 1, 2], [-1, 1, 0, 0], [-1, 0, 3, 1], [-1, -1, 0, 0]):
        with pytest.raises(Exception):
            om.verify_tree(toks, np.array([bad], np.int32), [0])


def test_after_the_commit_the_cache_is_that_of_the_kept_sequence():
    w = _weights()
    om = O.Model(SHAPE, w, max_batch=1, max_seq=40, max_block=16)
    rng = np.random.default_rng(9)
    prefix = rng.integers(0, SHAPE.vocab, 5).astype(np.int32)
    om.verify_block(prefix[None, :4], [0])
    parent = np.array([-1, 0, 0, 1, 1, 2, 4, 4, 6], np.int32)
    tokens = np.concatenate([prefix[4:], rng.integers(0, SHAPE.vocab, 8)]).astype(np.int32)
    om.verify_tree(tokens[None], parent[None], [4])
    path = [1, 4, 6, 8]                                          # a chain below row 0
    om.tree_commit(0, 4, path)
    kept = list(prefix) + [int(tokens[j]) for j in path]
    nxt = rng.integers(0, SHAPE.vocab, 3).astype(np.int32)
    lg = om.verify_block(nxt[None], [len(kept)])[0]             # rows 0 .. len(kept)-1 must now be the kept sequence
    ref = np.asarray(_torch_forward(SHAPE, w, kept + [int(t) for t in nxt]))[-3:]
    assert np.abs(lg - ref).max() < 1e-9
    with pytest.raises(Exception):
        om.tree_commit(0, 4, [2, 1])                             # not increasing
    with pytest.raises(Exception):
        om.tree_commit(0, 4, [0])                                # row 0 is not below row 0


SMALL = I.ModelShape("tree_small", 0, "fp32", 2, 32, 4, 8, 48, 12)


def test_greedy_decoding_through_arbitrary_trees_is_the_reviewers_greedy_continuation():
    """Trees of random shape and random candidate tokens over a 12-token vocabulary (so that candidates often hit):
    whatever they hold, walk + commit emit exactly the reviewer's own greedy tokens, several per review on average."""
    w = I.make_weights(SMALL, 4, std=0.4)
    ref_model = O.Model(SMALL, w, max_batch=1, max_seq=96, max_block=16)
    prompt = [3, 7, 1, 0, 5]
    seq = list(prompt)                                           # plain greedy, one token at a time
    ref_model.verify_block(np.array([seq[:-1]], np.int32), [0])
    for _ in range(40):
        lg = ref_model.verify_block(np.array([[seq[-1]]], np.int32), [len(seq) - 1])[0]
        seq.append(int(np.argmax(lg[-1])))
    want = seq[len(prompt):]

    om = O.Model(SMALL, w, max_batch=1, max_seq=96, max_block=16)
    rng = np.random.default_rng(1)
    got = list(prompt)
    om.verify_block(np.array([got[:-1]], np.int32), [0])
    reviews, kept_total = 0, 0
    while len(got) - len(prompt) < 40:
        m = int(rng.integers(2, 14))
        parent = _random_tree(m, rng, max_children=6)
        tokens = np.concatenate([[got[-1]], rng.integers(0, SMALL.vocab, m - 1)]).astype(np.int32)
        t = len(got) - 1
        lg = om.verify_tree(tokens[None], parent[None], [t])
        n, path, nxt = O.tree_accept(lg.astype(np.float32), tokens[None], parent[None], np.zeros((1, m), np.float32), mode=1)
        n = int(n[0])
        om.tree_commit(0, t, path[0, :n])
        got += [int(tokens[j]) for j in path[0, :n]] + [int(nxt[0])]
        reviews += 1
        kept_total += n
    assert got[len(prompt):len(prompt) + 40] == want[:40]
    assert kept_total > 5 and reviews < 40                       # candidates were really kept along the way


def _laws(V, seed, rows):
    rng = np.random.default_rng(seed)
    p = rng.random((rows, V)).astype(np.float32) ** 2
    p[:, 0] = 0.0                                                # a token the reviewer never emits
    return (p / p.sum(-1, keepdims=True)).astype(np.float32)


def test_sampling_walk_emits_the_reviewers_law_whatever_the_tree_holds():
    """V = 6; row 0 has children carrying tokens {1, 2, 2, 0}: token 2 twice (the lower row wins), token 0 never drawn.
    Exact counts over a grid of the two uniforms: the first emitted token follows p_0; given a kept child the second
    follows that child's row; a first token without a child ends the review."""
    V, m = 6, 7
    p = _laws(V, 2, m)
    tokens = np.array([[9 % V, 1, 2, 2, 0, 4, 5]], np.int32)     # rows 5, 6 hang below row 2
    parent = np.array([[-1, 0, 0, 0, 0, 2, 2]], np.int32)
    G = 1 << 9
    first = np.zeros(V)
    second = np.zeros((m, V))
    ended = np.zeros(V)
    for a in range(G):
        for b in range(0, G, 8):
            u = np.zeros((1, m), np.float32)
            u[0, 0], u[0, 1] = (a + 0.5) / G, (b + 0.5) / G
            n, path, nxt = O.tree_accept(p[None], tokens, parent, u, mode=0)
            n = int(n[0])
            t1 = int(tokens[0, path[0, 0]]) if n >= 1 else int(nxt[0])
            first[t1] += 1
            if n == 0:
                ended[t1] += 1
            elif n == 1:
                assert path[0, 0] in (1, 2)                      # never row 3 (same token as row 2) or row 4 (token 0)
                second[path[0, 0], int(nxt[0])] += 1
            else:                                                # row 2's child kept as well: the second token is 4 or 5
                assert n == 2 and path[0, 0] == 2
                second[2, int(tokens[0, path[0, 1]])] += 1
    total = G * (G // 8)
    assert np.abs(first / total - p[0]).max() < 2.5 / G
    for t in (3, 4, 5):                                          # no child carries these: the review ends with them
        assert ended[t] == first[t]
    for row, t in ((1, 1), (2, 2)):
        got = second[row] / second[row].sum()
        assert np.abs(got - p[row]).max() < 8 * 8 / G, (row, got, p[row])


def test_walk_reduces_to_the_chain_rule_with_onehot_drafts_in_law():
    """A chain with one candidate per position: P(kept >= j) = prod p_i(x_i), the law of Section 2's rule for one-hot
    drafts (accept with probability p(x)); the uniforms are used differently, so the comparison is in law."""
    V, k = 5, 3
    p = _laws(V, 7, k + 1)
    p[:, 0] = 0.05
    p = (p / p.sum(-1, keepdims=True)).astype(np.float32)
    draft = np.array([2, 4, 1], np.int32)
    tokens = np.concatenate([[0], draft])[None].astype(np.int32)
    parent = np.arange(-1, k, dtype=np.int32)[None]
    G = 64
    kept = np.zeros(k + 1)
    for a in range(G):
        for b in range(G):
            for c in range(G):
                u = np.array([[(a + .5) / G, (b + .5) / G, (c + .5) / G, 0.5]], np.float32)
                n, _, _ = O.tree_accept(p[None], tokens, parent, u, mode=0)
                kept[int(n[0])] += 1
    want_ge = np.cumprod([p[i, draft[i]] for i in range(k)])
    got_ge = np.array([kept[j:].sum() for j in range(1, k + 1)]) / G ** 3
    assert np.abs(got_ge - want_ge).max() < 3.0 / G
