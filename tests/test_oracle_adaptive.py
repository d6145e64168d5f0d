"""Pins of the oracle's adaptive controller for (tau_Q, tau_T, l_D, l_Q).  The paper names such a controller as future
work (Conclusion) and gives no rule; the rule is this build's reading, so the pins are the properties the reading
states: nothing moves while the accept rates sit inside the band, every parameter stays in its range, tau_Q never
exceeds tau_T, the trajectory is a pure function of the counts, and a controller with nowhere to go is the plain loop."""
import itertools
import math

import numpy as np

import oracle
from paper_2510_12966_amd import synth


def _ad(k2_min=2, k2_max=12, k1_max=6, steps=8, period=4, bq=(0.0, 0.4), bt=(0.1, 0.5)):
    return oracle.Adapt(k2_min, k2_max, k1_max, steps, period, bq[0], bq[1], bt[0], bt[1])


def test_threshold_positions_are_the_bands_grid_rounded_to_float():
    for lo, hi, S in ((0.0, 0.4, 8), (0.1, 0.5, 5), (0.25, 0.25, 3)):
        for s in range(S + 1):
            want = float(np.float32(np.float64(np.float32(lo)) + (np.float64(np.float32(hi)) - np.float64(np.float32(lo))) * s / S))
            assert oracle.adapt_threshold(lo, hi, s, S) == want
    assert oracle.adapt_threshold(0.0, 0.4, 0, 8) == 0.0
    assert oracle.adapt_threshold(0.0, 0.4, 8, 8) == float(np.float32(0.4))


def test_init_brings_the_start_values_into_the_ranges():
    ad = _ad()
    st = oracle.adapt_init(ad, 0.21, 0.32, 20)
    assert st.params() == (6, 12, 4, 4)       # k2 clamped to 12, k1 = (12 + 1) // 2 = 6, 0.21 -> position 4 of 0..0.4, 0.32 -> 4 of 0.1..0.5 (4.4 rounds down)
    st = oracle.adapt_init(ad, 5.0, 0.0, 1)
    assert st.params() == (1, 2, 8, 0)        # thresholds clamped to the ends of their bands, k2 to its minimum
    st = oracle.adapt_init(_ad(bq=(0.3, 0.3)), 0.1, 0.3, 5)
    assert st.s_q == 0                        # a band of one point has one position


def test_nothing_moves_while_the_rates_sit_inside_the_band():
    # accepted fraction in [1/2, 7/8) in both stages and windows neither fully accepted nor mostly rejected: a no-op
    ad = _ad()
    st = oracle.adapt_init(ad, 0.2, 0.3, 8)
    start = st.params()
    for i in range(40):
        n_t = 4 + (i % 3)                      # 4, 5 or 6 of 8: 2 n >= k2 and n < k2
        oracle.adapt_step(ad, st, n_t, 10, 6 + (i % 3))   # 6..8 of 10 accepted: 8 a < 7 p and 2 a >= p
        assert st.params() == start


def test_window_grows_on_full_acceptance_and_shrinks_on_cascades_within_its_range():
    ad = _ad()
    st = oracle.adapt_init(ad, 0.2, 0.3, 8)
    seen = []
    for _ in range(10):
        oracle.adapt_step(ad, st, st.k2, 10, 7)           # everything accepted by the target
        seen.append(st.k2)
    assert seen == [9, 10, 11, 12, 12, 12, 12, 12, 12, 12]
    assert st.k1 == 6                                     # (12 + 1) // 2 = 6, also the cap
    seen = []
    for _ in range(14):
        oracle.adapt_step(ad, st, 0, 10, 7)               # nothing accepted
        seen.append((st.k1, st.k2))
    assert seen[:4] == [(6, 11), (5, 10), (5, 9), (4, 8)] and seen[-1] == (1, 2) and min(k for _, k in seen) == 2
    # exactly half accepted is not a cascade: 2 n < k2 is strict
    st = oracle.adapt_init(ad, 0.2, 0.3, 8)
    oracle.adapt_step(ad, st, 4, 10, 7)
    assert st.k2 == 8


def test_thresholds_tighten_on_easy_acceptance_loosen_on_cascades_every_period_and_keep_their_order():
    ad = _ad(period=3)
    st = oracle.adapt_init(ad, 0.2, 0.3, 8)
    assert (st.s_q, st.s_t) == (4, 4)
    for i in range(3):
        assert (st.s_q, st.s_t) == (4, 4)                 # only the third pass of a period adjusts
        oracle.adapt_step(ad, st, st.k2, 10, 9)           # 9/10 and k2/k2: both >= 7/8
    assert (st.s_q, st.s_t) == (3, 3) and st.since == 0 and (st.p_q, st.a_q, st.p_t, st.a_t) == (0, 0, 0, 0)
    for i in range(3 * 12):
        oracle.adapt_step(ad, st, st.k2, 10, 10)
    assert (st.s_q, st.s_t) == (0, 0)                     # clamped at the strict end
    for i in range(3 * 12):
        oracle.adapt_step(ad, st, 0, 10, 0)
    assert (st.s_t, st.s_q) == (8, 8)                     # clamped at the loose end: 0.4 <= 0.5 keeps the order
    # order: a loose first stage is pulled down to the second stage's threshold
    ad2 = _ad(period=1, bq=(0.0, 0.8), bt=(0.1, 0.3), steps=4)
    st = oracle.adapt_init(ad2, 0.8, 0.1, 8)
    assert (st.s_q, st.s_t) == (4, 0)
    oracle.adapt_step(ad2, st, 5, 10, 6)                  # rates inside the band: only the order rule acts
    assert oracle.adapt_threshold(0.0, 0.8, st.s_q, 4) <= oracle.adapt_threshold(0.1, 0.3, st.s_t, 4)
    assert (st.s_q, st.s_t) == (0, 0)                     # 0.2 > 0.1, so down to 0.0
    # exhaustive: from any state and any counts, one step keeps every parameter in range and moves each by at most one
    ad3 = _ad(k2_min=1, k2_max=5, k1_max=2, steps=3, period=1, bq=(0.0, 0.3), bt=(0.0, 0.3))
    for k2, sq, s_t in itertools.product(range(1, 6), range(4), range(4)):
        if sq > s_t:
            continue
        for n_t in range(k2 + 1):
            for p_q, a_q in ((0, 0), (4, 0), (4, 2), (4, 3), (8, 7), (4, 4)):
                st = oracle.AdaptState(min((k2 + 1) // 2, 2), k2, sq, s_t, 0, 0, 0, 0, 0)
                oracle.adapt_step(ad3, st, n_t, p_q, a_q)
                assert 1 <= st.k2 <= 5 and abs(st.k2 - k2) <= 1 and st.k1 == max(1, min((st.k2 + 1) // 2, 2))
                assert 0 <= st.s_t <= 3 and abs(st.s_t - s_t) <= 1 and 0 <= st.s_q <= st.s_t


def _tiny_models(tiny_stack, ms):
    cfg, d, q, t, prompt = tiny_stack
    return (oracle.Model(cfg.draft, d, cfg.dtype, cfg.rope_theta, ms), oracle.Model(cfg.qualifier, q, cfg.dtype, cfg.rope_theta, ms),
            oracle.Model(cfg.target, t, cfg.dtype, cfg.rope_theta, ms))


def test_a_controller_with_nowhere_to_go_is_the_plain_loop(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ms = 16 + 40 + 8 + 2
    for Tq, Tt in ((0.004, 0.012), (0.0, 0.0)):
        ad = oracle.Adapt(8, 8, 4, 1, 3, Tq, Tq, Tt, Tt)
        out, st, log = oracle.generate_adaptive(*_tiny_models(tiny_stack, ms), prompt, 40, 3, 8, Tq, Tt, ad)
        ref, rst = oracle.generate(*_tiny_models(tiny_stack, ms), prompt, 40, 3, 4, 8, Tq, Tt)
        assert np.array_equal(out, ref) and st == rst
        assert (log == [4, 8, 0, 0]).all() and len(log) == st["passes_t"]


def test_the_loop_follows_the_controller_and_the_controller_follows_the_counts(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ad = oracle.Adapt(2, 12, 5, 6, 2, 0.0, 0.012, 0.0, 0.024)
    ms = 16 + 64 + 12 + 2
    out, st, log = oracle.generate_adaptive(*_tiny_models(tiny_stack, ms), prompt, 64, 5, 6, 0.004, 0.012, ad)
    out2, st2, log2 = oracle.generate_adaptive(*_tiny_models(tiny_stack, ms), prompt, 64, 5, 6, 0.004, 0.012, ad)
    assert np.array_equal(out, out2) and st == st2 and np.array_equal(log, log2)          # deterministic
    assert len(log) == st["passes_t"] and (log[:, 1] >= 2).all() and (log[:, 1] <= 12).all() and (log[:, 0] <= 5).all()
    assert (log[:, 0] == np.clip((log[:, 1] + 1) // 2, 1, 5)).all()
    assert len({tuple(r) for r in log}) > 3                                                  # it really moved
    assert st["proposed_t"] == int(log[:, 1].sum())                                          # every window had the logged length
    for r in log:
        assert oracle.adapt_threshold(0.0, 0.012, r[2], 6) <= oracle.adapt_threshold(0.0, 0.024, r[3], 6)
    # identical models: everything is accepted, so the window climbs to its maximum and the thresholds to their strict end,
    # and the output is still plain ancestral sampling (the law does not depend on the window at 100 % acceptance)
    ms = 16 + 110 + 12 + 2
    same = [oracle.Model(cfg.qualifier, q, cfg.dtype, cfg.rope_theta, ms) for _ in range(3)]
    out, st, log = oracle.generate_adaptive(*same, prompt, 110, 9, 4, 0.006, 0.012, ad)
    assert st["accepted_t"] == st["proposed_t"] and tuple(log[-1][1:]) == (12, 0, 0) and (np.diff(log[:, 1]) >= 0).all()
    plain = oracle.generate_plain(oracle.Model(cfg.qualifier, q, cfg.dtype, cfg.rope_theta, ms), prompt, 110, 9)
    assert np.array_equal(out, plain)
