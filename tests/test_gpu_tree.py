"""GPU parity of the tree review (csd_verify_tree, csd_tree_accept, csd_tree_commit) against the CPU oracle
(Section 5.1: the cascade combined with tree attention; Appendix B: eight children per lead node).

Logits within the tolerances of the plain block; kept rows, accepted lengths and tokens bit-exact on identical
probabilities; after the commit the cache must be that of the kept sequence (checked through the logits of the next
plain block)."""
import os

import numpy as np
import pytest
import torch

import csd_inputs as I
from gpu_util import make_pair, prefill_both, tol_ok

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import paper_2312_11462_amd as P
    P.lib()


def _dev(x, dtype=torch.int32):
    return torch.as_tensor(np.asarray(x), dtype=dtype).cuda()


def _random_tree(m, rng, max_children=3):
    parent = [-1]
    for i in range(1, m):
        cands = [j for j in range(i) if sum(1 for p in parent if p == j) < max_children]
        parent.append(int(rng.choice(cands)))
    return np.array(parent, np.int32)


def _caterpillar(depth, children):
    """Appendix B's shape: a lead chain whose every node has `children` children, the first of which leads on."""
    parent = [-1]
    lead = 0
    for _ in range(depth):
        first = len(parent)
        parent += [lead] * children
        lead = first
    return np.array(parent, np.int32)


FP = I.ModelShape("tree_fp32", 0, "fp32", 2, 48, 3, 16, 100, 301)
BF = I.ModelShape("tree_bf", 0, "bf16", 2, 256, 4, 64, 512, 1024)
BF128 = I.ModelShape("tree_bf_dh128", 0, "bf16", 2, 256, 2, 128, 512, 1024)


def _check_tree(gm, om, tokens, parent, cl, rtol, atol, what):
    lg, pr = gm.verify_tree(_dev(tokens), _dev(parent), _dev(cl), want_probs=True)
    ref, refp = om.verify_tree(tokens, parent, cl, want_probs=True)
    ok, err = tol_ok(lg.cpu().numpy().astype(np.float64), ref, rtol, atol)
    assert ok, f"{what}: logits max abs err {err}"
    okp, errp = tol_ok(pr.cpu().numpy().astype(np.float64), refp, 5 * rtol, 1e-6)
    assert okp, f"{what}: probs max abs err {errp}"
    return err


def test_fp32_generic_kernels_two_sequences_ragged():
    gm, om = make_pair(FP, 5, 2, 96, 16, std=0.1)
    toks = I.token_ids(2 * 40, FP.vocab, 5, 1).reshape(2, 40)
    prefill_both(gm, om, toks[:, :20], 10)
    rng = np.random.default_rng(2)
    cl = [20, 17]
    m = 13
    parent = np.stack([_random_tree(m, rng), _caterpillar(3, 4)])
    tokens = np.stack([np.concatenate([[toks[b, cl[b]]], rng.integers(0, FP.vocab, m - 1)]) for b in range(2)]).astype(np.int32)
    _check_tree(gm, om, tokens, parent, cl, 1e-4, 1e-4, "fp32 tree")
    # a chain-shaped tree gives what the plain block gives
    chain = np.tile(np.arange(-1, m - 1, dtype=np.int32), (2, 1))
    a = gm.verify_tree(_dev(tokens), _dev(chain), _dev(cl)).cpu().numpy()
    b = gm.verify_block(_dev(tokens), _dev(cl)).cpu().numpy()
    assert np.array_equal(a, b)


@pytest.mark.parametrize("shape", [BF, BF128], ids=["dh64", "dh128"])
@pytest.mark.parametrize("path", ["default", "multikernel"])
def test_bf16_small_trees_on_both_forwards(shape, path):
    """Blocks of 12 and 16 rows over 200 cached rows (two key chunks and a ragged tail): the forward for small blocks
    (its attention kernel masks by ancestors) and the per-operation kernels."""
    os.environ["CSD_PATH"] = path
    try:
        gm, om = make_pair(shape, 7, 1, 300, 16, std=0.05)
    finally:
        del os.environ["CSD_PATH"]
    assert gm.path(1, 12) == (1 if path == "default" else 0)
    toks = I.token_ids(260, shape.vocab, 7, 1).reshape(1, 260)
    prefill_both(gm, om, toks[:, :200], 16)
    rng = np.random.default_rng(4)
    for m, parent in ((12, _random_tree(12, rng)), (16, _caterpillar(3, 5))):
        tokens = np.concatenate([[toks[0, 200]], rng.integers(0, shape.vocab, m - 1)]).astype(np.int32)[None]
        err = _check_tree(gm, om, tokens, parent[None], [200], 2e-2, 1e-2, f"{shape.name} {path} m={m}")
        print(shape.name, path, m, "max err", err)


def test_bf16_tree_of_41_rows_three_row_tiles_batch_of_two():
    """Appendix B's tree at depth 5: 1 + 5 x 8 = 41 rows per sequence, 82 rows in the GEMMs (the tall-block form),
    three 16-row tiles per sequence in the attention; different cache lengths."""
    gm, om = make_pair(BF, 9, 2, 256, 41, std=0.05)
    assert gm.path(2, 41) == 0
    toks = I.token_ids(2 * 160, BF.vocab, 9, 1).reshape(2, 160)
    prefill_both(gm, om, toks[:, :144], 36)
    rng = np.random.default_rng(6)
    cl = [144, 131]
    parent = np.stack([_caterpillar(5, 8), _random_tree(41, rng, max_children=8)])
    tokens = np.stack([np.concatenate([[toks[b, cl[b]]], rng.integers(0, BF.vocab, 40)]) for b in range(2)]).astype(np.int32)
    err = _check_tree(gm, om, tokens, parent, cl, 2e-2, 1e-2, "41-row trees")
    print("41 rows max err", err)


@pytest.mark.parametrize("V,m,B", [(40, 9, 3), (1000, 33, 2), (32000, 41, 2), (301, 64, 1)])
@pytest.mark.parametrize("mode", [0, 1])
def test_tree_accept_bit_exact(V, m, B, mode):
    """Random trees whose candidates are made to hit often: children carry the reviewer's most likely tokens of the
    parent row, with duplicates among siblings; kept rows, lengths and tokens equal the oracle's."""
    import paper_2312_11462_amd as P
    from oracle import csd_oracle as O
    rng = np.random.default_rng(V + m)
    p = rng.random((B, m, V)).astype(np.float32) ** 8
    p /= p.sum(-1, keepdims=True)
    heavy = rng.integers(0, V, (B, m, 3))
    for b in range(B):
        for i in range(m):
            p[b, i, heavy[b, i]] += 0.5                     # three tokens that carry most of the mass
    p /= p.sum(-1, keepdims=True)
    p = p.astype(np.float32)
    parent = np.stack([_random_tree(m, rng, max_children=5) for _ in range(B)])
    tokens = np.zeros((B, m), np.int32)
    for b in range(B):
        for i in range(1, m):
            top = np.argsort(-p[b, parent[b, i]])[:3]
            tokens[b, i] = int(rng.choice(top))
    total = 0
    for rep in range(4):
        u = I.uniforms(B * m, 11 + rep, V).reshape(B, m)
        n, path, nxt = P.tree_accept(_dev(p, torch.float32), _dev(tokens), _dev(parent), u.cuda(), mode=mode)
        on, opath, onxt = O.tree_accept(p, tokens, parent, u.numpy(), mode=mode)
        assert np.array_equal(n.cpu().numpy(), on) and np.array_equal(nxt.cpu().numpy(), onxt)
        for b in range(B):
            assert np.array_equal(path[b, :on[b]].cpu().numpy(), opath[b, :on[b]])
        total += int(on.sum())
    assert total > 0


SMALL = I.ModelShape("tree_small", 0, "fp32", 2, 32, 4, 8, 48, 12)
SMALL_BF = I.ModelShape("tree_small_bf", 0, "bf16", 2, 64, 4, 16, 128, 16)


@pytest.mark.parametrize("shape,std", [(SMALL, 0.4), (SMALL_BF, 0.3)], ids=["fp32", "bf16"])
def test_greedy_decoding_through_trees_with_commit_equals_plain_greedy_and_the_oracle(shape, std):
    """verify_tree -> tree_accept -> tree_commit, 30 tokens, trees of random shape and content over a small vocabulary
    (so candidates are kept): the tokens are the model's own greedy continuation (one row at a time on the GPU), and the
    fp32 run equals the oracle's tree decoding review for review."""
    import paper_2312_11462_amd as P
    from oracle import csd_oracle as O
    gm, om = make_pair(shape, 4, 1, 96, 16, std=std)
    prompt = [3, 7, 1, 0, 5]

    def plain_greedy(model_gpu):
        seq = list(prompt)
        model_gpu.verify_block(_dev([seq[:-1]]), _dev([0]))
        for _ in range(45):
            lg = model_gpu.verify_block(_dev([[seq[-1]]]), _dev([len(seq) - 1]))
            seq.append(int(lg[0, -1].argmax().item()))
        return seq[len(prompt):]

    want = plain_greedy(gm)
    got, ogot = list(prompt), list(prompt)
    gm.verify_block(_dev([got[:-1]]), _dev([0]))
    om.verify_block(np.array([got[:-1]], np.int32), [0])
    rng = np.random.default_rng(1)
    kept = 0
    while len(got) - len(prompt) < 30:
        m = int(rng.integers(2, 15))
        parent = _random_tree(m, rng, max_children=6)
        cand = rng.integers(0, shape.vocab, m - 1)
        tokens = np.concatenate([[got[-1]], cand]).astype(np.int32)[None]
        # along one root-to-node path most candidates are the true continuation, so that several rows are kept
        row, chain = int(rng.integers(1, m)), []
        while row > 0:
            chain.append(row)
            row = int(parent[row])
        done = len(got) - len(prompt)
        for dpt, row in enumerate(reversed(chain)):
            if rng.random() < 0.75 and done + dpt < len(want):
                tokens[0, row] = want[done + dpt]
        t = len(got) - 1
        cl = _dev([t])
        lg = gm.verify_tree(_dev(tokens), _dev(parent[None]), cl)
        n, path, nxt = P.tree_accept(lg, _dev(tokens), _dev(parent[None]), None, mode=1)
        gm.tree_commit(cl, path, n)
        nn = int(n.item())
        got += [int(tokens[0, j]) for j in path[0, :nn].cpu().numpy()] + [int(nxt.item())]
        kept += nn
        if shape.dtype == "fp32" and ogot == got[:len(ogot)]:
            olg = om.verify_tree(tokens, parent[None], [t])
            on, opath, onxt = O.tree_accept(olg.astype(np.float32), tokens, parent[None], np.zeros((1, m), np.float32), mode=1)
            om.tree_commit(0, t, opath[0, :int(on[0])])
            ogot += [int(tokens[0, j]) for j in opath[0, :int(on[0])]] + [int(onxt[0])]
            assert ogot == got, "GPU and oracle tree decoding diverged"
    assert got[len(prompt):len(prompt) + 30] == want[:30]
    assert kept > 8


def test_after_the_commit_the_next_plain_block_matches_the_oracle_bf16():
    gm, om = make_pair(BF, 12, 2, 128, 41, std=0.05)
    toks = I.token_ids(2 * 100, BF.vocab, 12, 1).reshape(2, 100)
    prefill_both(gm, om, toks[:, :64], 16)
    parent = np.stack([_caterpillar(5, 8), _caterpillar(5, 8)])
    rng = np.random.default_rng(8)
    tokens = np.stack([np.concatenate([[toks[b, 64]], rng.integers(0, BF.vocab, 40)]) for b in range(2)]).astype(np.int32)
    cl = [64, 64]
    gm.verify_tree(_dev(tokens), _dev(parent), _dev(cl))
    om.verify_tree(tokens, parent, cl)
    # keep a path of 4 rows in sequence 0 (lead, lead, lead, a non-lead child) and of 1 row in sequence 1
    paths = np.full((2, 41), -1, np.int32)
    paths[0, :4] = [1, 9, 17, 27]
    paths[1, :1] = [5]
    n = np.array([4, 1], np.int32)
    gm.tree_commit(_dev(cl), _dev(paths), _dev(n))
    for b in range(2):
        om.tree_commit(b, cl[b], paths[b, :n[b]])
    new_cl = [cl[b] + 1 + int(n[b]) for b in range(2)]
    nxt = toks[:, 70:76].numpy()
    lg = gm.verify_block(_dev(nxt), _dev(new_cl)).cpu().numpy().astype(np.float64)
    ref = om.verify_block(nxt, new_cl)
    ok, err = tol_ok(lg, ref, 2e-2, 1e-2)
    assert ok, err


def test_argument_errors():
    import paper_2312_11462_amd as P
    gm, _ = make_pair(FP, 1, 1, 128, 70)
    with pytest.raises(P.CsdError):       # more than 64 rows
        gm.verify_tree(_dev(np.zeros((1, 65))), _dev(np.zeros((1, 65))), _dev([0]))
    with pytest.raises(P.CsdError):
        P.tree_accept(torch.zeros((1, 3, 8), device="cuda"), _dev(np.zeros((1, 3))), _dev(np.zeros((1, 3))), None, mode=0)
