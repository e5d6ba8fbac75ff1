"""Cascade Speculative Drafting generation loop (Algorithm 1) on top of the C-ABI calls.

Control flow only: every draft (Max-Gram kernel), every review forward and every accept / resample
runs in the HIP library; distributions never leave the device (a level's reviewer probabilities are
handed upward as device rows and gathered on the device into the next review's q).  The host reads two
integers per review (accepted length, next token) to steer the loops, which is what makes this the
host-driven form of the driver.

Readings of Algorithm 1 (the printed listing has slips; Sections 3.1-3.3 and Appendix B decide):
  * levels = [target, draft_1, ..., draft_{n-1}]; the statistical Max-Gram model is the implicit last
    draft level and the base case of the recursion; its draft probabilities are one-hot;
  * K is n x n over the n draft levels including Max-Gram (the decoder-only setting of Appendix B is
    [[2, 10], [0, 10]]): row 0 belongs to the current reviewer, K[0][i] tokens come from draft level i
    (horizontal cascade), each produced by a recursive step whose reviewer is that level (vertical
    cascade) with the sub-matrix below and to the right;
  * a level hands upward, as draft probabilities, its own reviewer distributions of the tokens it
    emitted;
  * lenience applies only where a draft model reviews (Section 3.1): 1 when the real target reviews
    and between Max-Gram and its reviewer;
  * after a review, a level keeps cache rows only up to the last kept token (rejected rows are
    overwritten by the next block).
Batch 1 (sequences are independent; a batch is a loop over this).
"""
from __future__ import annotations

import torch

from . import binding as P


class Level:
    """A neural model of the cascade with its cache bookkeeping."""

    def __init__(self, model: "P.Model", max_block: int):
        self.model = model
        self.cached = 0            # rows of the cache that belong to the current sequence
        self.max_block = max_block
        self._cl = torch.zeros(1, dtype=torch.int32, device="cuda")

    def rows_from(self, ctx, n_tokens, first_row, want_probs=False, temperature=1.0):
        """Logits (device, [n][V]) of positions first_row .. n_tokens-1 (row j predicts token j+1), and
        their softmax when asked; runs the model over every position not yet cached, max_block rows per
        launch."""
        assert self.cached <= first_row < n_tokens
        outs, pouts = [], []
        pos = self.cached
        while pos < n_tokens:
            m = min(self.max_block, n_tokens - pos)
            self._cl.fill_(pos)
            blk = ctx[:, pos:pos + m].contiguous()
            if want_probs:
                lg, pr = self.model.verify_block(blk, self._cl, temperature=temperature, want_probs=True)
                pouts.append(pr[0])
            else:
                lg = self.model.verify_block(blk, self._cl)
            outs.append(lg[0])
            pos += m
        skip = first_row - self.cached
        lg = (outs[0] if len(outs) == 1 else torch.cat(outs, dim=0))[skip:]
        if not want_probs:
            return lg, None
        return lg, (pouts[0] if len(pouts) == 1 else torch.cat(pouts, dim=0))[skip:]


class Cascade:
    """levels = [target, draft_1, ...] over Max-Gram; one sequence; greedy (mode 1) or sampling (mode 0)."""

    def __init__(self, levels, next_table, K, max_ctx, lenience=1.0, mode=1, temperature=1.0, max_match=0):
        n_drafts = len(levels)                         # neural drafts below the target + Max-Gram
        if len(K) != n_drafts or any(len(r) != n_drafts for r in K):
            raise ValueError("K must be n x n over the draft levels including Max-Gram")
        self.levels, self.table, self.K = levels, next_table, K
        self.lenience, self.mode, self.temperature, self.max_match = float(lenience), mode, temperature, max_match
        self.V = levels[0].model.shape.vocab
        self.ctx = torch.zeros((1, max_ctx), dtype=torch.int32, device="cuda")
        self.n = 0                                     # tokens of the sequence so far (prompt + generation + drafts in flight)
        self._len = torch.zeros(1, dtype=torch.int32, device="cuda")
        self.reviews = 0

    # ------------------------------------------------------------------ sequence buffer
    def _append_host(self, toks):
        t = torch.tensor(toks, dtype=torch.int32)
        self.ctx[0, self.n:self.n + len(toks)] = t.cuda()
        self.n += len(toks)

    # ------------------------------------------------------------------ one step of Algorithm 1
    def _step(self, levels, K, uniforms, is_first):
        """Reviewer levels[0]; drafts come from levels[1:] and Max-Gram.  The sequence buffer holds the
        prefix (self.n tokens) on entry and prefix + kept tokens on exit.  Returns the device rows
        (or None for one-hot) of the reviewer's distributions of the tokens it emitted."""
        reviewer, below = levels[0], levels[1:]
        n_prefix = self.n
        q_rows = []
        n_drafts = len(below) + 1
        for i in range(n_drafts):
            k_i = K[0][i]
            start = self.n
            while self.n - start < k_i:
                if i == n_drafts - 1:                  # Max-Gram: the base case
                    need = k_i - (self.n - start)
                    self._len.fill_(self.n)
                    P.bigram_draft(self.ctx, self._len, self.table, need, self.max_match, want_match_len=False,
                                   out=self.ctx[:, self.n:self.n + need])
                    self.n += need
                    q_rows += [None] * need
                else:
                    sub = [row[i + 1:] for row in K[i + 1:]]
                    q_rows += self._step(below[i:], sub, uniforms, False)
        k = self.n - n_prefix
        lvl_lenience = 1.0 if (is_first or len(levels) == 1) else self.lenience
        greedy_plain = self.mode == 1 and lvl_lenience <= 1.0                # compares arg-maxes of the logits
        lg, probs = reviewer.rows_from(self.ctx, self.n, n_prefix - 1, want_probs=not greedy_plain,
                                       temperature=self.temperature)        # k + 1 rows
        self.reviews += 1
        p = (lg if greedy_plain else probs)[None]
        if self.mode == 1:
            u_acc = torch.zeros((1, k), dtype=torch.float32, device="cuda") if k else None
            u_s = torch.zeros(1, dtype=torch.float32, device="cuda")
        else:
            u_acc = torch.tensor([next(uniforms) for _ in range(k)], dtype=torch.float32).reshape(1, k).cuda() if k else None
            u_s = torch.tensor([next(uniforms)], dtype=torch.float32).cuda()
        q = onehot = None
        if any(r is not None for r in q_rows):
            q = torch.zeros((1, k, self.V), dtype=torch.float32, device="cuda")
            flags = []
            for j, row in enumerate(q_rows):
                flags.append(1 if row is None else 0)
                if row is not None:
                    q[0, j].copy_(row)
            onehot = torch.tensor(flags, dtype=torch.uint8).cuda()
        drafts = self.ctx[:, n_prefix:self.n].contiguous() if k else None
        n_acc_d, nxt_d = P.accept(p.contiguous(), q, drafts, u_acc, u_s, lvl_lenience, self.mode, onehot)
        n_acc, nxt = int(n_acc_d.item()), int(nxt_d.item())
        # keep the accepted drafts, replace what follows by the reviewer's own token
        self.n = n_prefix + n_acc
        self._append_host([nxt])
        reviewer.cached = n_prefix + n_acc
        for lv in below:
            lv.cached = min(lv.cached, n_prefix + n_acc)
        if self.mode == 1:
            return [None] * (n_acc + 1)
        return [probs[j] for j in range(n_acc + 1)]

    # ------------------------------------------------------------------ public
    def generate(self, prompt, n_new, uniforms=None):
        """Returns (tokens, target reviews): at least n_new tokens are generated, n_new returned."""
        for lv in self.levels:
            lv.cached = 0
        self.n = 0
        self.reviews = 0
        self._append_host(list(prompt))
        steps = 0
        while self.n - len(prompt) < n_new:
            self._step(self.levels, self.K, uniforms, True)
            steps += 1
        out = self.ctx[0, len(prompt):len(prompt) + n_new].cpu().tolist()
        return out, steps


def autoregressive(level: Level, prompt, n_new, max_ctx, mode=1, uniforms=None, temperature=1.0):
    """Plain one-token-at-a-time decoding from one model (the baseline the cascade must reproduce)."""
    c = Cascade([level], torch.zeros(level.model.shape.vocab, dtype=torch.int32, device="cuda"), [[0]], max_ctx,
                mode=mode, temperature=temperature)
    out, _ = c.generate(prompt, n_new, uniforms)
    return out


class ResidentCascade:
    """Algorithm 1 as a chain of enqueues with device-resident control: the sequence, every length, the loop
    conditions ("until k_i tokens exist") and the draft distributions handed upward live on the device, and a whole
    multi-level step runs with no host synchronisation (csd_review_ctx, csd_bigram_draft_append, csd_cascade_gate).
    A loop of Algorithm 1 whose trip count depends on accepted lengths is enqueued for its worst case (k_i rounds),
    each round gated per sequence on the device.  One sequence; levels = [target, draft_1, ...] over Max-Gram.
    Uniforms are taken by position from per-level tables (u_acc[level][pos], u_samp[level][pos]) that the caller
    fills (sampling mode)."""

    def __init__(self, levels, next_table, K, max_ctx, lenience=1.0, mode=1, temperature=1.0, max_match=0, q_stride=32):
        n = len(levels)
        if len(K) != n or any(len(r) != n for r in K):
            raise ValueError("K must be n x n over the draft levels including Max-Gram")
        self.levels, self.table, self.K = levels, next_table, K
        self.lenience, self.mode, self.temperature, self.max_match = float(lenience), mode, temperature, max_match
        self.V = levels[0].model.shape.vocab
        dev = "cuda"
        self.ctx = torch.zeros((1, max_ctx), dtype=torch.int32, device=dev)
        self.ctx_len = torch.zeros(1, dtype=torch.int32, device=dev)
        self.cache_len = [torch.zeros(1, dtype=torch.int32, device=dev) for _ in levels]
        self.status = [torch.zeros(1, dtype=torch.int32, device=dev) for _ in levels]
        self.n_acc = [torch.zeros(1, dtype=torch.int32, device=dev) for _ in levels]
        # what each level reviews against: rows and flags by position relative to the start of its step
        self.q_tab = [torch.zeros((1, q_stride, self.V), dtype=torch.float32, device=dev) if mode == 0 else None for _ in levels]
        self.onehot = [torch.ones((1, q_stride), dtype=torch.uint8, device=dev) for _ in levels]
        self.u_acc = [torch.zeros((1, max_ctx), dtype=torch.float32, device=dev) for _ in levels]
        self.u_samp = [torch.zeros((1, max_ctx), dtype=torch.float32, device=dev) for _ in levels]
        self._gates = []          # one tensor per call site, created on first use and reused every step
        self._site = 0
        self.enqueued_reviews = 0

    def _tensor(self):
        if self._site == len(self._gates):
            self._gates.append(torch.zeros(1, dtype=torch.int32, device="cuda"))
        t = self._gates[self._site]
        self._site += 1
        return t

    def start(self, prompt):
        """Host-driven setup: the prompt into the buffer, every level's cache filled with all but its last token."""
        n = len(prompt)
        self.ctx.zero_()
        self.ctx[0, :n] = torch.tensor(prompt, dtype=torch.int32).cuda()
        self.ctx_len.fill_(n)
        cl = torch.zeros(1, dtype=torch.int32, device="cuda")
        for lv, c in zip(self.levels, self.cache_len):
            pos = 0
            while pos < n - 1 and getattr(lv, "ext_rows", None) is None:
                m = min(lv.max_block, n - 1 - pos)
                cl.fill_(pos)
                lv.model.verify_block(self.ctx[:, pos:pos + m].contiguous(), cl)
                pos += m
            c.fill_(n - 1)

    def _step(self, li, K, gate, parent):
        """Enqueue one CascadeSpeculativeDraftingStep with reviewer levels[li] for the sequences whose gate is >= 0;
        gate holds the step's prefix length.  parent = (q_tab, onehot, base) of the level that will review what this
        step emits, or None at the top."""
        n_levels = len(self.levels)
        n_drafts = n_levels - li
        for i in range(n_drafts):
            k_i = K[0][i]
            if k_i == 0:
                continue
            if i == n_drafts - 1:                      # Max-Gram: the base case, k_i tokens at once
                P.bigram_draft_append(self.ctx, self.ctx_len, self.table, k_i, self.max_match, gate=gate,
                                      q_onehot_tab=self.onehot[li], q_base=gate)
            else:
                loop_start = self._tensor()
                P.cascade_gate(self.ctx_len, loop_start)                       # the length when the loop starts
                sub = [row[i + 1:] for row in K[i + 1:]]
                for _ in range(k_i):                                           # worst case: one token per round
                    g = self._tensor()
                    P.cascade_gate(self.ctx_len, g, loop_start=loop_start, need=k_i, parent_gate=gate)
                    self._step(li + 1 + i, sub, g, (self.q_tab[li], self.onehot[li], gate))
        lvl_lenience = 1.0 if (li == 0 or li == n_levels - 1) else self.lenience
        lv = self.levels[li]
        dense_below = self.mode == 0 and li < n_levels - 1
        lv.model.review_ctx(self.ctx, self.ctx_len, self.cache_len[li], gate, lv.max_block, self.status[li],
                            q_tab=self.q_tab[li] if dense_below else None,
                            q_onehot_tab=self.onehot[li] if dense_below else None, q_base=gate if dense_below else None,
                            u_acc_tab=self.u_acc[li], u_samp_tab=self.u_samp[li],
                            out_q_tab=parent[0] if parent else None, out_onehot_tab=parent[1] if parent else None,
                            out_base=parent[2] if parent else None, lower=self.cache_len[li + 1:],
                            n_accepted=self.n_acc[li], ext_rows=getattr(lv, "ext_rows", None), temperature=self.temperature,
                            lenience=lvl_lenience, mode=self.mode)
        self.enqueued_reviews += 1

    def step(self):
        """Enqueue one whole step of the target (no synchronisation)."""
        self._site = 0
        g0 = self._tensor()
        P.cascade_gate(self.ctx_len, g0)
        self._step(0, self.K, g0, None)

    def tokens(self):
        """The kept sequence (synchronises)."""
        n = int(self.ctx_len.item())
        return self.ctx[0, :n].cpu().tolist()
