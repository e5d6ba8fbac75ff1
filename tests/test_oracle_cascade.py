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
