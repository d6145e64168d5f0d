"""Shared checker of the GPU loops (helper module, not a test file).

A GPU generation call hands every sampling step and every ACCEPT stage to a trace callback together with the logits
rows it used.  Two things are checked there, step by step:
  * the decision: the oracle decides the same step again on the GPU's own logits; it must agree exactly, except at the
    documented near-ties (|div - tau| < 1e-6, coin within 1e-6 relative of p/q, two best race keys within 1e-5),
    which are counted;
  * the logits: the same rows are recomputed by the oracle's forward, teacher-forced on the GPU's own token
    sequence (TeacherForced), and must agree within the tolerance of the weight type.  This is what ties the rows
    inside the loop, after every cache rollback, to the oracle, not only the decisions taken on them.
"""
import numpy as np

import oracle

TIE_DIV, TIE_COIN, TIE_RACE = 1e-6, 1e-6, 1e-5
DIV_TOL = 1e-5
LOGIT_TOL = {0: 1e-4, 1: 3e-2}   # weight type (0 fp32, 1 bf16) -> largest |GPU logit - oracle logit|


class TeacherForced:
    """Oracle models that follow the GPU's own token sequence and recompute the logits rows it reports.

    models: oracle.Model per library model index (0 draft, 1 qualifier, 2 target; a missing entry switches the check off
    for that model).  The sequence is rebuilt from the trace events alone: a sampling event at position P appends its
    token after the first P tokens, a stage event at position P keeps the accepted proposals and the replacement."""

    def __init__(self, models, prompt, tol, max_rows=None):
        self.models, self.tol = dict(models), tol
        self.budget = dict(max_rows) if max_rows else {}   # model index -> rows still to be checked (absent: no limit)
        self.rows_of = {w: 0 for w in self.models}
        self.cur = [int(t) for t in prompt]
        self.cached = {w: [] for w in self.models}
        self.rows = 0
        self.max_err = 0.0

    def _rows(self, which, tokens, n_rows):
        """Oracle logits of the last n_rows positions of `tokens`, re-using the oracle's cache for the common prefix."""
        om, have = self.models[which], self.cached[which]
        common = 0
        while common < min(len(have), len(tokens)) and have[common] == tokens[common]:
            common += 1
        start = min(common, len(tokens) - n_rows)
        lg = om.forward(np.array(tokens[start:], dtype=np.int32), start)
        self.cached[which] = list(tokens)
        return lg[-n_rows:]

    def check(self, which, pos0, proposals, lp):
        """lp[i] must be the logits of the token at pos0 + i given cur[:pos0] + proposals[:i]."""
        if which not in self.models or self.budget.get(which, 1) <= 0:
            return
        if which in self.budget:
            self.budget[which] -= lp.shape[0]
        self.rows_of[which] += lp.shape[0]
        assert 1 <= pos0 <= len(self.cur), (pos0, len(self.cur))
        tokens = self.cur[:pos0] + [int(t) for t in proposals]
        want = self._rows(which, tokens, lp.shape[0])
        err = float(np.abs(lp.astype(np.float64) - want).max())
        self.max_err = max(self.max_err, err)
        self.rows += lp.shape[0]
        assert err <= self.tol, ("in-loop logits differ from the oracle's forward", which, pos0, err)

    def sampled(self, pos0, token):
        self.cur = self.cur[:pos0] + [int(token)]

    def decided(self, pos0, proposals, n_acc, nxt):
        self.cur = self.cur[:pos0] + [int(t) for t in proposals[:n_acc]] + ([int(nxt)] if nxt >= 0 else [])


class Replay:
    """Trace callback for psd_generate (fuzzy or assisted first stage) and psd_generate_sd.

    forced: optional TeacherForced; proposer: the model whose rows the sampling events carry (0 in the three-model loop)."""

    def __init__(self, seed, T_q, T_t, temperature=1.0, forced=None, proposer=0):
        self.seed, self.T, self.temp = seed, {1: T_q, 2: T_t}, temperature
        self.forced, self.proposer = forced, proposer
        self.events = self.ties = self.kinds = 0
        self.max_div_err = 0.0
        self.windows, self.counts = [], []

    def __call__(self, kind, pos0, k, bonus, lp, lq, tk, n_acc, nxt, div):
        self.events += 1
        self.kinds |= 1 << kind
        if kind == 7:   # adaptive controller: thresholds and windows in force from this outer iteration on
            self.T = {1: float(div[0]), 2: float(div[1])}
            self.windows.append((bonus, k, n_acc, nxt))      # (k1, k2, position of tau_Q, position of tau_T)
            self.counts.append([0, 0, 0])                    # this iteration's (stage-1 proposed, stage-1 accepted, stage-2 accepted)
            return
        if kind == 0:
            if self.forced:
                self.forced.check(self.proposer, pos0, [], lp)
                self.forced.sampled(pos0, nxt)
            want, gap = oracle.sample_row(lp[0], self.temp, self.seed, pos0)
            if want != nxt:
                assert gap < TIE_RACE, ("proposal", pos0, want, nxt, gap)
                self.ties += 1
            return
        if self.forced:
            self.forced.check(1 if kind in (1, 3) else 2, pos0, tk, lp)
            self.forced.decided(pos0, tk, n_acc, nxt)
        if kind == 3:   # assisted stage: token comparison is exact, only the replacement draw can tie
            res = oracle.accept_assisted(lp, tk, self.temp, self.seed, pos0, 1, bool(bonus))
            assert n_acc == res.n_accepted, ("assisted", pos0, n_acc, res.n_accepted)
            if nxt != res.next_token:
                assert res.margin_race < TIE_RACE
                self.ties += 1
            return
        assert kind in (1, 2)
        if self.counts:
            if kind == 1:
                self.counts[-1][0] += k
                self.counts[-1][1] += n_acc
            else:
                self.counts[-1][2] = n_acc
        res, odiv = oracle.accept(lp, lq, tk, self.T[kind], self.temp, self.seed, pos0, kind, bool(bonus))
        self.max_div_err = max(self.max_div_err, float(np.abs(div - odiv).max(initial=0.0)))
        assert self.max_div_err <= DIV_TOL
        if n_acc != res.n_accepted:
            assert res.margin_div < TIE_DIV or res.margin_coin < TIE_COIN, ("accept", kind, pos0, n_acc, res.n_accepted)
            self.ties += 1
        elif nxt != res.next_token:
            assert res.margin_race < TIE_RACE, ("token", kind, pos0, nxt, res.next_token, res.margin_race)
            self.ties += 1


class GreedyReplay:
    """Every proposal and every stage of a greedy run decided again by the oracle on the GPU's own logits: exact."""

    def __init__(self, forced=None, proposer=0):
        self.kinds = 0
        self.forced, self.proposer = forced, proposer

    def __call__(self, kind, pos0, k, bonus, lp, lq, tk, n_acc, nxt, div):
        self.kinds |= 1 << kind
        if kind == 6:
            if self.forced:
                self.forced.check(self.proposer, pos0, [], lp)
                self.forced.sampled(pos0, nxt)
            assert nxt == int(lp[0].argmax())
            return
        assert kind in (4, 5)
        if self.forced:
            self.forced.check(1 if kind == 4 else 2, pos0, tk, lp)
            self.forced.decided(pos0, tk, n_acc, nxt)
        res = oracle.accept_greedy(lp, tk, bool(bonus))
        assert (n_acc, nxt) == (res.n_accepted, res.next_token), (kind, pos0, n_acc, nxt, res.n_accepted, res.next_token)


def forced_for(shapes, blobs, dtype, theta, max_seq, prompt, which=(0, 1, 2), max_rows=None):
    """TeacherForced over fresh oracle models of the given library model indices; max_rows: {model index: rows to check}
    bounds the oracle's work on large models (the sequence is followed to the end either way)."""
    models = {w: oracle.Model(shapes[w], blobs[w], dtype, theta, max_seq) for w in which}
    return TeacherForced(models, prompt, LOGIT_TOL[dtype], max_rows)
