"""Pins of the oracle's two-model baseline (Section 3.3, first equation) and of the assisted variant (Section 3.4)."""
import numpy as np
import scipy.special
import scipy.stats

import oracle
from paper_2510_12966_amd import synth
from paper_2510_12966_amd.synth import ModelShape


def _m(shape, blob, cfg, ms):
    return oracle.Model(shape, blob, cfg.dtype, cfg.rope_theta, ms)


# ---- two-model speculative decoding -------------------------------------------------------------------

def test_sd_is_the_three_model_loop_with_a_transparent_first_stage(tiny_stack):
    # draft == qualifier and tau_Q above ln 2: the first stage accepts every round in full, the window holds the
    # proposer's own samples and rows, so the three-model loop (already pinned) must emit the same tokens
    cfg, d, q, t, prompt = tiny_stack
    for (k, tau, temp) in ((4, 0.0, 1.0), (7, 0.012, 1.0), (1, 0.0, 0.8), (5, 0.3, 1.0)):
        ms = len(prompt) + 40 + k + 2
        out, st = oracle.generate_sd(_m(cfg.qualifier, q, cfg, ms), _m(cfg.target, t, cfg, ms), prompt, 40, 9, k, tau, temp)
        ref, rst = oracle.generate(_m(cfg.qualifier, q, cfg, ms), _m(cfg.qualifier, q, cfg, ms), _m(cfg.target, t, cfg, ms),
                                   prompt, 40, 9, k, k, 1.0, tau, temp)
        assert np.array_equal(out, ref)
        for key in ("proposed_t", "accepted_t", "fuzzy_t", "passes_t"):
            assert st[key] == rst[key], key
        assert st["passes_d"] == rst["passes_d"] == k * st["passes_t"]
    assert 0 < st["accepted_t"]


def test_sd_identical_models_equal_plain_sampling(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ms = len(prompt) + 40 + 8
    for k, tau in ((3, 0.0), (6, 0.1)):
        out, st = oracle.generate_sd(_m(cfg.target, t, cfg, ms), _m(cfg.target, t, cfg, ms), prompt, 40, 2, k, tau)
        assert st["accepted_t"] == st["proposed_t"]
        assert np.array_equal(out, oracle.generate_plain(_m(cfg.target, t, cfg, ms), prompt, 40, 2))


def test_sd_tau0_reproduces_target_chain_on_vocab8():
    # standard speculative sampling is exact: the pair of emitted tokens follows the target's ancestral law
    V = 8
    sh = lambda L, dm: ModelShape(L, dm, 2, 1, 2 * dm, V)
    sP, sT = sh(1, 8), sh(2, 16)
    wP = synth.target_weights(sP, 21, synth.DTYPE_F32, sigma=0.6)
    wT = synth.target_weights(sT, 23, synth.DTYPE_F32, sigma=0.5)
    prompt = np.array([1, 6], dtype=np.int32)
    ms = 2 + 2 + 3 + 2
    T = oracle.Model(sT, wT, synth.DTYPE_F32, 10000.0, ms)
    P = oracle.Model(sP, wP, synth.DTYPE_F32, 10000.0, ms)
    p0 = oracle.softmax(T.forward(prompt, 0)[-1].astype(np.float32))
    joint = np.zeros((V, V))
    for a in range(V):
        joint[a] = p0[a] * oracle.softmax(T.forward(np.array([1, 6, a]), 0)[-1].astype(np.float32))
    N = 30000
    counts = np.zeros((V, V))
    acc = prop = 0
    for s in range(N):
        out, st = oracle.generate_sd(P, T, prompt, 2, s, 3, 0.0)
        counts[out[0], out[1]] += 1
        acc += st["accepted_t"]; prop += st["proposed_t"]
    assert 0.05 < acc / prop < 0.95
    exp = joint * N
    keep = exp > 5
    chi2 = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    assert chi2 < scipy.stats.chi2.ppf(0.9999, keep.sum() - 1)


# ---- assisted stage ------------------------------------------------------------------------------------

def test_assisted_accepts_exactly_the_argmax_prefix():
    rng = np.random.default_rng(0)
    k, V = 5, 40
    lp = rng.normal(0, 2, (k + 1, V)).astype(np.float32)
    top = lp.argmax(1)
    res = oracle.accept_assisted(lp, top[:k], 1.0, 3, 10, 1, True)
    assert res.n_accepted == k and res.n_fuzzy == 0
    assert res.next_token == oracle.sample_row(lp[k], 1.0, 3, 10 + k, oracle.DRAW_SAMPLE, 0)[0]   # bonus from row k
    assert oracle.accept_assisted(lp, top[:k], 1.0, 3, 10, 1, False).next_token == -1
    for n in range(k):
        x = top[:k].copy()
        x[n] = (x[n] + 1) % V
        x[n + 1:] = 0                                   # whatever follows a mismatch is ignored
        res = oracle.accept_assisted(lp, x, 0.7, 3, 10, 1, True)
        assert res.n_accepted == n
    # equal maxima: the lowest index is the top prediction
    lp[0, 7] = lp[0, 3] = lp[0].max() + 1
    assert oracle.accept_assisted(lp, [3, 0, 0, 0, 0], 1.0, 3, 10, 1, True).n_accepted >= 1
    assert oracle.accept_assisted(lp, [7, 0, 0, 0, 0], 1.0, 3, 10, 1, True).n_accepted == 0
    # k = 0: only the bonus draw
    assert oracle.accept_assisted(lp[:1], [], 1.0, 3, 10, 1, True).n_accepted == 0


def test_assisted_fallback_draws_from_the_verifier_distribution():
    # on a mismatch the emitted token follows softmax(logits_p[n] / temperature), whatever was proposed
    rng = np.random.default_rng(1)
    V, temp = 12, 0.8
    lp = rng.normal(0, 1.5, (2, V)).astype(np.float32)
    wrong = int((lp[0].argmax() + 5) % V)
    p = oracle.softmax(lp[0], temp)
    N = 40000
    counts = np.zeros(V)
    for s in range(N):
        res = oracle.accept_assisted(lp, [wrong], temp, s, 4, 1, True)
        assert res.n_accepted == 0
        counts[res.next_token] += 1
    assert ((counts - N * p) ** 2 / (N * p)).sum() < scipy.stats.chi2.ppf(0.9999, V - 1)
    # the draws are those of the replacement stream, not of the proposal stream
    t, _ = oracle.sample_row(lp[0], temp, 5, 4, oracle.DRAW_RESAMPLE, 1)
    assert oracle.accept_assisted(lp, [wrong], temp, 5, 4, 1, True).next_token == t


def test_assisted_loop_identical_models_and_counters(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ms = len(prompt) + 40 + 10
    # draft == qualifier == target at a low temperature: the draft's sample is usually, not always, the top
    # prediction, so the qualifier stage really rejects; the output still follows the qualifier / target law only in
    # distribution, so here we pin structure: counters, determinism, range
    mk = lambda: (_m(cfg.draft, d, cfg, ms), _m(cfg.qualifier, q, cfg, ms), _m(cfg.target, t, cfg, ms))
    out, st = oracle.generate_assisted(*mk(), prompt, 40, 3, 4, 8, 0.012, 0.3)
    out2, st2 = oracle.generate_assisted(*mk(), prompt, 40, 3, 4, 8, 0.012, 0.3)
    assert np.array_equal(out, out2) and st == st2
    assert (out >= 0).all() and (out < cfg.target.vocab).all()
    assert st["fuzzy_q"] == 0 and 0 < st["accepted_q"] < st["proposed_q"]
    assert st["proposed_t"] == 8 * st["passes_t"] and st["passes_d"] == st["proposed_q"]
    # greedy limit: at a very low temperature every model samples its top prediction; identical models then agree
    # at every position and the loop must emit the greedy continuation, all proposals accepted
    A = lambda: _m(cfg.qualifier, q, cfg, ms)
    out, st = oracle.generate_assisted(A(), A(), A(), prompt, 30, 1, 3, 6, 0.0, 1e-4)
    assert st["accepted_q"] == st["proposed_q"] and st["accepted_t"] == st["proposed_t"]
    M = A()
    seq = list(prompt)
    for _ in range(30):
        seq.append(int(M.forward(np.array(seq, dtype=np.int32), 0)[-1].argmax()))
    assert np.array_equal(out, np.array(seq[len(prompt):]))


def test_assisted_loop_first_token_law_on_vocab8():
    # k1 = k2 = 1, one emitted token.  Stage 1 hands over x = top(Q) with probability a = P_D(top(Q)), else a
    # sample of P_Q; stage 2 at tau_T = 0 keeps x with probability min(1, p(x)/q(x)), q = P_Q, else draws from
    # the residual of p over q.  (The result is NOT the target law: x is not distributed as q.)
    V = 8
    sh = lambda L, dm: ModelShape(L, dm, 2, 1, 2 * dm, V)
    sD, sQ, sT = sh(1, 8), sh(1, 16), sh(2, 16)
    wD = synth.target_weights(sD, 81, synth.DTYPE_F32, sigma=0.8)    # seeds chosen so that the law below is
    wQ = synth.target_weights(sQ, 181, synth.DTYPE_F32, sigma=0.8)   # far from the target's (0.076 in one cell)
    wT = synth.target_weights(sT, 281, synth.DTYPE_F32, sigma=0.5)   # and a is near 0.58
    prompt = np.array([2, 4], dtype=np.int32)
    ms = 2 + 1 + 1 + 2
    D, Q, T = (oracle.Model(s, w, synth.DTYPE_F32, 10000.0, ms) for s, w in ((sD, wD), (sQ, wQ), (sT, wT)))
    pd, pq, pt = (oracle.softmax(M.forward(prompt, 0)[-1].astype(np.float32)) for M in (D, Q, T))
    top = int(np.argmax(Q.forward(prompt, 0)[-1].astype(np.float32)))
    a = pd[top]
    r = (1 - a) * pq
    r[top] += a
    keep_p = np.minimum(1.0, pt / pq)
    res = np.maximum(0.0, pt - pq)
    res /= res.sum()
    law = r * keep_p + (r * (1 - keep_p)).sum() * res
    assert abs(law.sum() - 1) < 1e-12 and np.abs(law - pt).max() > 0.05     # visibly not the target law here
    N = 40000
    counts = np.zeros(V)
    acc_q = 0
    for s in range(N):
        out, st = oracle.generate_assisted(D, Q, T, prompt, 1, s, 1, 1, 0.0)
        counts[out[0]] += 1
        acc_q += st["accepted_q"]
    assert abs(acc_q / N - a) < 4 * np.sqrt(a * (1 - a) / N)
    assert ((counts - N * law) ** 2 / (N * law)).sum() < scipy.stats.chi2.ppf(0.9999, V - 1)


# ---- per-step statistics of the behaviour analysis (Section 4) ---------------------------------------------

def test_row_stats_closed_forms_and_library():
    import math
    V = 1000
    h, m = oracle.row_stats(np.full(V, 3.7, np.float32))
    assert abs(h - math.log(V)) < 1e-12 and abs(m - 1 / V) < 1e-15            # uniform
    z = np.full(V, -80.0, np.float32); z[17] = 30.0
    h, m = oracle.row_stats(z)
    assert h < 1e-40 and abs(m - 1) < 1e-15                                    # one-hot
    # two-point mass: logits (a, 0) -> p = sigmoid(a); entropy is the binary entropy
    for a in (0.3, 2.0, -1.5):
        p = 1 / (1 + math.exp(-a))
        h, m = oracle.row_stats(np.array([a, 0.0], np.float32))
        a32 = float(np.float32(a)); p = 1 / (1 + math.exp(-a32))
        assert abs(h - (-(p * math.log(p) + (1 - p) * math.log(1 - p)))) < 1e-12 and abs(m - max(p, 1 - p)) < 1e-12
    rng = np.random.default_rng(3)
    z = rng.normal(0, 2.5, 5000).astype(np.float32)
    for temp in (1.0, 0.6, 3.0):
        h, m = oracle.row_stats(z, temp)
        p = scipy.special.softmax(z.astype(np.float64) / temp)
        assert abs(h - scipy.stats.entropy(p)) < 1e-10 and abs(m - p.max()) < 1e-12
    # shift invariance, and the temperature limits
    assert np.allclose(oracle.row_stats(z), oracle.row_stats(z + np.float32(8.0)), rtol=0, atol=1e-6)
    assert abs(oracle.row_stats(z, 1e6)[0] - math.log(z.size)) < 1e-6
    assert oracle.row_stats(z, 1e-3)[1] > 0.999


# ---- greedy decoding through the loop (temperature -> 0 limit, Section 3.1) ------------------------------

def _greedy_continuation(M, prompt, n):
    seq = list(prompt)
    for _ in range(n):
        seq.append(int(M.forward(np.array(seq, dtype=np.int32), 0)[-1].astype(np.float32).argmax()))
    return np.array(seq[len(prompt):], dtype=np.int32)


def test_greedy_loop_is_lossless_for_any_draft_and_qualifier(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    n_new = 40
    ms = len(prompt) + n_new + 10
    want = _greedy_continuation(_m(cfg.target, t, cfg, ms), prompt, n_new)
    for k1, k2 in ((4, 8), (1, 1), (3, 7), (8, 3)):
        out, st = oracle.generate_greedy(_m(cfg.draft, d, cfg, ms), _m(cfg.qualifier, q, cfg, ms), _m(cfg.target, t, cfg, ms),
                                         prompt, n_new, k1, k2)
        assert np.array_equal(out, want)
        assert st["accepted_q"] <= st["proposed_q"] and st["accepted_t"] <= st["proposed_t"] and st["fuzzy_q"] == 0
        assert st["proposed_t"] == k2 * st["passes_t"]
    assert st["accepted_q"] < st["proposed_q"]            # different models do disagree on this stack
    # identical models: nothing is ever rejected
    A = lambda: _m(cfg.target, t, cfg, ms)
    out, st = oracle.generate_greedy(A(), A(), A(), prompt, n_new, 4, 8)
    assert np.array_equal(out, want) and st["accepted_q"] == st["proposed_q"] and st["accepted_t"] == st["proposed_t"]


def test_greedy_stage_is_the_low_temperature_limit_of_the_sampling_stage():
    rng = np.random.default_rng(5)
    k, V = 4, 30
    lp = rng.normal(0, 2, (k + 1, V)).astype(np.float32)
    lq = rng.normal(0, 2, (k, V)).astype(np.float32)
    for trial in range(6):
        x = lp.argmax(1)[:k].astype(np.int32)
        if trial:
            x[trial % k] = (x[trial % k] + 3) % V
        g = oracle.accept_greedy(lp, x, True)
        # at temperature 1e-3 both distributions are one-hot to 1e-300: divergence 0 or ln 2, coin 0 or 1
        s, _ = oracle.accept(lp, lq.copy() if trial else lp[:k], x, 0.0, 1e-3, trial, 0, 1, True)
        if trial == 0:
            assert g.n_accepted == k == s.n_accepted and g.next_token == s.next_token == lp[k].argmax()
        else:
            # proposer rows differ, so compare the greedy rule with the strict-match rule it must equal
            n = 0
            while n < k and x[n] == lp[n].argmax():
                n += 1
            assert g.n_accepted == n and g.next_token == lp[n].argmax()
    assert oracle.accept_greedy(lp, lp.argmax(1)[:k], False).next_token == -1
