"""Pins of the oracle's ACCEPT stage: the tau = 0 limit is standard speculative sampling
(Section 3.1), tau >= ln 2 accepts everything, in between the threshold of Section 3.2 decides."""
import math

import numpy as np
import scipy.stats

import oracle


def _logits(p):
    return np.log(np.asarray(p, dtype=np.float64)).astype(np.float32)


def test_scan_tau0_single_position_is_min_ratio_rule():
    # brute force over a fine grid of coin values: P(accept | x) = min(1, p(x)/q(x)),
    # hence P(accept) = sum_x min(p, q) = 1 - TV(p, q)
    rng = np.random.default_rng(0)
    p = rng.dirichlet(np.ones(8))
    q = rng.dirichlet(np.ones(8))
    N = 4000
    grid = (np.arange(N) + 0.5) / N
    total = 0.0
    for x in range(8):
        acc = sum(oracle.accept_scan(p[None], q[None], [x], 0.0, [u])[0] for u in grid) / N
        assert abs(acc - min(1.0, p[x] / q[x])) <= 1.0 / N
        total += q[x] * acc
    assert abs(total - (1 - 0.5 * np.abs(p - q).sum())) < 1e-3


def test_scan_threshold_is_non_strict_and_stops_at_first_reject():
    rng = np.random.default_rng(1)
    p = rng.dirichlet(np.ones(6), size=3)
    q = rng.dirichlet(np.ones(6), size=3)
    d = [oracle.jsd(p[i], q[i]) for i in range(3)]
    x = [int(np.argmin(p[i] / q[i])) for i in range(3)]   # tokens with ratio < 1
    u_fail = [0.999999] * 3                               # coin fails wherever it is consulted
    n, div, fuzzy = oracle.accept_scan(p, q, x, max(d), u_fail)
    assert n == 3 and fuzzy == 3                          # div == T is accepted (<=)
    np.testing.assert_allclose(div, d, rtol=0, atol=0)
    T = sorted(d)[1]                                      # exactly one position is over the threshold
    worst = int(np.argmax(d))
    n, div, fuzzy = oracle.accept_scan(p, q, x, T, u_fail)
    assert n == worst and fuzzy == worst
    assert np.isnan(div[worst + 1:]).all()                # nothing judged after the first rejection
    n, _, fuzzy = oracle.accept_scan(p, q, x, T, [0.0] * 3)  # coin succeeds -> accepted but not "fuzzy"
    assert n == 3 and fuzzy == 2
    n, _, _ = oracle.accept_scan(p, q, x, np.nextafter(max(d), 0), u_fail)
    assert n == worst


def _chain_tables(rng, V):
    q0 = rng.dirichlet(np.ones(V)); q1 = rng.dirichlet(np.ones(V), size=V)
    p0 = rng.dirichlet(np.ones(V)); p1 = rng.dirichlet(np.ones(V), size=V)
    p2 = rng.dirichlet(np.ones(V), size=(V, V))
    return q0, q1, p0, p1, p2


def _run_chain(tables, T, n_trials, V=8):
    q0, q1, p0, p1, p2 = tables
    first = np.zeros(V); second = np.zeros((V, V)); third = np.zeros(V); n_hist = np.zeros(3)
    third_exp = np.zeros(V)
    for s in range(n_trials):
        x0, _ = oracle.sample_row(_logits(q0), 1.0, s, 100)
        x1, _ = oracle.sample_row(_logits(q1[x0]), 1.0, s, 101)
        lp = np.stack([_logits(p0), _logits(p1[x0]), _logits(p2[x0, x1])])
        lq = np.stack([_logits(q0), _logits(q1[x0])])
        res, _ = oracle.accept(lp, lq, [x0, x1], T, 1.0, seed=s, position0=100, stage=2)
        out = [x0, x1][:res.n_accepted] + [res.next_token]
        n_hist[res.n_accepted] += 1
        first[out[0]] += 1
        if len(out) > 1:
            second[out[0], out[1]] += 1
        if len(out) > 2:  # bonus token: drawn from the verifier's last row, whatever the prefix was
            third[out[2]] += 1
            third_exp += p2[x0, x1]
    return first, second, (third, third_exp), n_hist


def test_tau0_vocab8_length2_reproduces_target_chain():
    # tau = 0 is standard SD: emitted tokens follow the target chain whatever the proposer is.
    V, N = 8, 60000
    rng = np.random.default_rng(7)
    tables = _chain_tables(rng, V)
    q0, q1, p0, p1, p2 = tables
    first, second, (third, third_exp), n_hist = _run_chain(tables, 0.0, N)
    crit = lambda k: scipy.stats.chi2.ppf(0.9999, k)
    assert ((first - N * p0) ** 2 / (N * p0)).sum() < crit(V - 1)
    # given the first token a was accepted, the second emitted token follows p1[a]
    for a in range(V):
        na = second[a].sum()
        if na > 500:
            assert ((second[a] - na * p1[a]) ** 2 / (na * p1[a])).sum() < crit(V - 1)
    # accept-length law: P(n >= 1) = sum_x min(p0, q0)
    p_acc0 = np.minimum(p0, q0).sum()
    assert abs((n_hist[1] + n_hist[2]) / N - p_acc0) < 4 * math.sqrt(p_acc0 * (1 - p_acc0) / N)
    # bonus token after two accepts follows p2[x0, x1]
    n3 = third.sum()
    assert n3 > 200
    assert ((third - third_exp) ** 2 / third_exp).sum() < crit(V - 1)


def test_tau_ln2_accepts_everything_and_bonus_follows_verifier():
    V, N = 8, 20000
    rng = np.random.default_rng(8)
    tables = _chain_tables(rng, V)
    q0, q1, p0, p1, p2 = tables
    first, second, (third, third_exp), n_hist = _run_chain(tables, math.log(2) + 1e-12, N)
    assert n_hist[2] == N
    # accepted tokens are the proposer's own draws
    assert ((first - N * q0) ** 2 / (N * q0)).sum() < scipy.stats.chi2.ppf(0.9999, V - 1)
    n3 = third.sum()
    assert n3 == N
    assert ((third - third_exp) ** 2 / third_exp).sum() < scipy.stats.chi2.ppf(0.9999, V - 1)


def test_threshold_between_switches_law_from_target_to_proposer():
    # one position: JSD <= tau -> the emitted token is the proposal (law q); JSD > tau -> law p
    V, N = 6, 20000
    rng = np.random.default_rng(9)
    p = rng.dirichlet(np.ones(V)); q = rng.dirichlet(np.ones(V))
    d = oracle.jsd(oracle.softmax(_logits(p)), oracle.softmax(_logits(q)))
    for T, law in ((d * 1.01, q), (d * 0.99, p)):
        counts = np.zeros(V); acc = 0
        for s in range(N):
            x, _ = oracle.sample_row(_logits(q), 1.0, s, 5)
            lp = np.stack([_logits(p), _logits(p)])
            res, div = oracle.accept(lp, _logits(q)[None], [x], T, 1.0, seed=s, position0=5, stage=1)
            assert abs(div[0] - d) < 1e-12
            acc += res.n_accepted
            counts[x if res.n_accepted == 1 else res.next_token] += 1
        assert ((counts - N * law) ** 2 / (N * law)).sum() < scipy.stats.chi2.ppf(0.9999, V - 1)
        p_acc = 1.0 if T > d else np.minimum(p, q).sum()
        assert abs(acc / N - p_acc) < 4 * math.sqrt(max(p_acc * (1 - p_acc), 1e-9) / N) + 1e-12


def test_accept_interface_details():
    rng = np.random.default_rng(3)
    V, k = 40, 5
    lp = rng.normal(0, 2, (k + 1, V)).astype(np.float32)
    lq = rng.normal(0, 2, (k, V)).astype(np.float32)
    x = rng.integers(0, V, k).astype(np.int32)
    for temp in (1.0, 0.7):
        res, div = oracle.accept(lp, lq, x, 0.0, temp, seed=11, position0=30, stage=1)
        # reported divergences: JSD of the tempered softmaxes, for every proposed position
        for i in range(k):
            assert abs(div[i] - oracle.jsd(oracle.softmax(lp[i], temp), oracle.softmax(lq[i], temp))) < 1e-15
        # the scan used the coin addressed by (position0 + i, COIN, stage)
        n = 0
        while n < k:
            pi, qi = oracle.softmax(lp[n], temp), oracle.softmax(lq[n], temp)
            if not (div[n] <= 0.0 or oracle.uniform(11, 0, 30 + n, oracle.DRAW_COIN, 1) < pi[x[n]] / qi[x[n]]):
                break
            n += 1
        assert res.n_accepted == n
        if n < k:  # residual resample: only tokens with p > q can come out
            pi, qi = oracle.softmax(lp[n], temp), oracle.softmax(lq[n], temp)
            assert pi[res.next_token] > qi[res.next_token]
            r = np.maximum(pi - qi, 0)
            assert res.next_token == oracle.race(r, 11, 30 + n, oracle.DRAW_RESAMPLE, 1)[0]
    res, _ = oracle.accept(lp, lq, x, 1.0, 1.0, seed=11, position0=30, stage=1, take_bonus=False)
    assert res.n_accepted == k and res.next_token == -1 and res.n_fuzzy == k
    res, _ = oracle.accept(lp, lq, x, 1.0, 1.0, seed=11, position0=30, stage=1, take_bonus=True)
    assert res.next_token == oracle.sample_row(lp[k], 1.0, 11, 30 + k)[0]


def test_identical_rows_always_accept_with_zero_divergence():
    rng = np.random.default_rng(4)
    lp = rng.normal(0, 3, (4, 100)).astype(np.float32)
    res, div = oracle.accept(lp, lp[:3], [1, 2, 3], 0.0, 1.0, seed=5, position0=0, stage=2)
    assert res.n_accepted == 3 and (div == 0.0).all()


def test_k_zero_draws_only_the_bonus():
    lp = np.log(np.array([[0.25, 0.75]])).astype(np.float32)
    res, div = oracle.accept(lp, np.zeros((0, 2), np.float32), [], 0.3, 1.0, seed=2, position0=9, stage=1)
    assert res.n_accepted == 0 and res.next_token in (0, 1) and div.size == 0


def _accept_threshold(p_rows, q_rows, x, pos):
    """Largest coin value at which position `pos` is still accepted at tau = 0, found on the oracle's own scan:
    the scan is monotone in every coin, so bisection on explicit coin values pins the switch to ~1e-16.  Earlier
    positions get coin 0 (always accepted); the result is P(accept at pos | reached, x)."""
    k = len(x)
    passes = lambda u: oracle.accept_scan(p_rows, q_rows, x, 0.0, [0.0] * pos + [u] + [0.0] * (k - pos - 1))[0] > pos
    if passes(np.nextafter(1.0, 0.0)):
        return 1.0
    lo, hi = 0.0, 1.0     # passes(lo) (coin 0 always passes when p(x) > 0), not passes(hi)
    if not passes(0.0):
        return 0.0
    for _ in range(70):
        mid = 0.5 * (lo + hi)
        if passes(mid):
            lo = mid
        else:
            hi = mid
    return 0.5 * (lo + hi)


def test_tau0_exact_enumeration_on_vocab8_length2_reproduces_the_target_chain():
    # tau = 0 is standard speculative decoding (Section 3.1), whose output law is the verifier's, exactly.
    # Enumerate every proposal pair (x0, x1); integrate the two coins exactly from the oracle's scan evaluated on
    # explicit coin values (bisection: no formula of the rule is retyped here); take the replacement law from the
    # oracle's residual weights, normalised.  The law of the emitted tokens must be the target chain to rounding.
    V = 8
    rng = np.random.default_rng(7)
    q0, q1, p0, p1, p2 = _chain_tables(rng, V)
    # make the case generic: a token the proposer over-weights, one it under-weights, one the verifier excludes
    p0 = p0.copy(); p0[2] = 0.0; p0 /= p0.sum()
    first = np.zeros(V)                 # law of the first emitted token
    pair = np.zeros((V, V))             # law of the first two emitted tokens, when the first proposal was accepted
    first_accepted = np.zeros(V)        # P(x0 = a and accepted)
    triple_ok = 0.0
    for x0 in range(V):
        P = np.stack([p0, p1[x0]]); Q = np.stack([q0, q1[x0]])
        a0 = _accept_threshold(P, Q, [x0, 0], 0)
        first[x0] += q0[x0] * a0
        first_accepted[x0] = q0[x0] * a0
        r0 = oracle.residual(p0, q0)
        if q0[x0] * (1 - a0) > 0:
            assert r0.sum() > 0
            first += q0[x0] * (1 - a0) * r0 / r0.sum()
        for x1 in range(V):
            a1 = _accept_threshold(P, Q, [x0, x1], 1)
            w = q0[x0] * a0 * q1[x0][x1]
            pair[x0, x1] += w * a1
            r1 = oracle.residual(p1[x0], q1[x0])
            if w * (1 - a1) > 0:
                pair[x0] += w * (1 - a1) * r1 / r1.sum()
            triple_ok += w * a1        # both accepted: the bonus token is a fresh sample of p2[x0, x1] (pinned elsewhere)
    np.testing.assert_allclose(first, p0, rtol=0, atol=1e-12)
    assert first[2] == 0.0                                  # a token outside the verifier's support never comes out
    # given that x0 = a was accepted, the next emitted token follows p1[a]; P(x0 = a accepted) = min(p0, q0)[a]
    np.testing.assert_allclose(first_accepted, np.minimum(p0, q0), rtol=0, atol=1e-12)
    np.testing.assert_allclose(pair, first_accepted[:, None] * p1, rtol=0, atol=1e-12)
    # chain law of two emitted tokens: a first token that came out of a rejection is followed by a fresh stage whose
    # first-token law is, by the statement just checked, its own verifier row p1[a]
    rejected_first = first - first_accepted
    joint = pair + rejected_first[:, None] * p1
    np.testing.assert_allclose(joint, p0[:, None] * p1, rtol=0, atol=1e-12)
    assert abs(triple_ok - sum(min(p0[a], q0[a]) * np.minimum(p1[a], q1[a]).sum() for a in range(V))) < 1e-12
    # the enumeration separates the rule from near misses: the proposer's law and the plain mixture are far away
    assert np.abs(first - q0).max() > 1e-2
