"""Minimal cascade driver on top of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Follows Algorithm 1 (CascadeSpeculativeDraftingStep) with the printed listing's slips
repaired as follows:
  * the base case is "the current reviewer is the statistical model": it returns the
    Max-Gram continuation (Section 3.3) with one-hot draft probabilities;
  * the horizontal loop records the length before its while loop and runs until k_i new
    tokens exist (the listing re-assigns the prefix inside the loop);
  * K is n x n over the n draft models including Max-Gram, as the decoder-only setting
    [[2, 10], [0, 10]] of Appendix B implies; row 0 belongs to the current reviewer;
  * what a level hands upward as draft probabilities are its own reviewer distributions
    of the tokens it emitted (that is what makes the upper review exact);
  * lenience is forced to 1 when the real target reviews (Section 3.1) and between
    Max-Gram and its reviewer (Appendix B).
It exists to pin the oracle: greedy cascaded decoding must emit exactly the target's own
greedy continuation (Sections 3.1, 5.1).
"""
from __future__ import annotations

import numpy as np

from . import csd_oracle as O


class Level:
    """A neural model with its KV cache bookkeeping."""

    def __init__(self, model: O.Model, max_block: int):
        self.model = model
        self.cached = 0
        self.max_block = max_block

    def rows_from(self, seq, first_row):
        """Logits for positions first_row .. len(seq)-1 (row j predicts token j+1); runs the
        model over every position not yet cached."""
        assert self.cached <= first_row
        outs = []
        pos = self.cached
        while pos < len(seq):
            m = min(self.max_block, len(seq) - pos)
            lg = self.model.verify_block(np.array([seq[pos:pos + m]], dtype=np.int32),
                                         np.array([pos], dtype=np.int32))[0]
            outs.append((pos, lg))
            pos += m
        lg = np.concatenate([x[1] for x in outs], axis=0)
        return lg[first_row - self.cached:]


def autoregressive(level: Level, prompt, n_new, mode=1, uniforms=None, temperature=1.0):
    """Plain one-token-at-a-time decoding from a single model."""
    seq = list(prompt)
    level.cached = 0
    for _ in range(n_new):
        lg = level.rows_from(seq, len(seq) - 1)
        level.cached = len(seq)
        if mode == 1:
            seq.append(int(np.argmax(lg[-1])))
        else:
            p = O.probs_f32(lg[-1:], temperature)
            _, nxt = O.accept(p[None], None, np.zeros((1, 0), np.int32), np.zeros((1, 0), np.float32),
                              np.array([next(uniforms)], np.float32))
            seq.append(int(nxt[0]))
    return seq[len(prompt):]


def _step(levels, next_table, seq, K, lenience, mode, uniforms, is_first, max_match, uniform_at=None, depth=0):
    """One CascadeSpeculativeDraftingStep with reviewer levels[0]; returns (tokens, q_rows).
    The random numbers are inputs: either an iterator `uniforms` drawn in review order, or a function
    uniform_at(depth, kind, position) with kind 0 = the acceptance test of the draft at that position and
    kind 1 = the draw of a review whose first draft sits at that position (depth = the reviewer's level)."""
    reviewer = levels[0]
    n_prefix = len(seq)
    cur = list(seq)
    q_rows = []          # per drafted token: fp32 row [V], or None when one-hot
    below = levels[1:]   # neural drafts below, then Max-Gram as the implicit last entry
    n_drafts = len(below) + 1
    for i in range(n_drafts):
        k_i = K[0][i]
        start = len(cur)
        while len(cur) - start < k_i:
            if i == n_drafts - 1:      # Max-Gram: the base case
                need = k_i - (len(cur) - start)
                toks, _ = O.bigram_draft(np.array(cur, np.int32), [len(cur)], next_table, need, max_match)
                cur += [int(t) for t in toks[0]]
                q_rows += [None] * need
            else:
                subK = [row[i + 1:] for row in K[i + 1:]]
                toks, qs = _step(below[i:], next_table, cur, subK, lenience, mode, uniforms, False, max_match,
                                 uniform_at, depth + 1 + i)
                cur += toks
                q_rows += qs
    drafts = cur[n_prefix:]
    k = len(drafts)
    lg = reviewer.rows_from(cur, n_prefix - 1)                      # k+1 rows
    all_onehot = all(q is None for q in q_rows)
    lvl_lenience = 1.0 if (is_first or len(levels) == 1) else lenience
    V = lg.shape[-1]
    if mode == 1:
        p = lg.astype(np.float32)[None]
        if lvl_lenience > 1.0:
            p = O.probs_f32(lg)[None]
        u_acc = np.zeros((1, k), np.float32)
        u_s = np.zeros(1, np.float32)
    else:
        p = O.probs_f32(lg)[None]
        if uniform_at is not None:
            u_acc = np.array([[uniform_at(depth, 0, n_prefix + j) for j in range(k)]], np.float32)
            u_s = np.array([uniform_at(depth, 1, n_prefix)], np.float32)
        else:
            u_acc = np.array([[next(uniforms) for _ in range(k)]], np.float32)
            u_s = np.array([next(uniforms)], np.float32)
    q = None
    onehot = None
    if not all_onehot:
        q = np.zeros((1, k, V), np.float32)
        onehot = np.zeros(k, np.uint8)
        for j, row in enumerate(q_rows):
            if row is None:
                onehot[j] = 1
            else:
                q[0, j] = row
    n_acc, nxt = O.accept(p, q, np.array([drafts], np.int32), u_acc, u_s, lvl_lenience, mode, onehot)
    n_acc = int(n_acc[0])
    out = drafts[:n_acc] + [int(nxt[0])]
    reviewer.cached = n_prefix + n_acc
    for lv in below:                      # lower levels keep only what is still on the path
        lv.cached = min(lv.cached, n_prefix + n_acc)
    if mode == 1:
        out_q = [None] * len(out)
    else:
        probs = O.probs_f32(lg)
        out_q = [probs[j] for j in range(len(out))]
    return out, out_q


def cascade_generate(levels, next_table, prompt, n_new, K, lenience=1.0, mode=1, uniforms=None,
                     max_match=0):
    """Generate >= n_new tokens with levels = [target, draft_1, ...] over Max-Gram."""
    seq = list(prompt)
    for lv in levels:
        lv.cached = 0
    steps = 0
    while len(seq) - len(prompt) < n_new:
        toks, _ = _step(levels, next_table, seq, K, lenience, mode, uniforms, True, max_match)
        seq += toks
        steps += 1
    return seq[len(prompt):len(prompt) + n_new], steps
