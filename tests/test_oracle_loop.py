"""Pins of the oracle's two-stage loop (Figure 1 caption, Sections 3.2-3.3)."""
import numpy as np
import scipy.stats

import oracle
from paper_2510_12966_amd import synth
from paper_2510_12966_amd.synth import ModelShape


def _models(cfg, d, q, t, max_seq):
    return (oracle.Model(cfg.draft, d, cfg.dtype, cfg.rope_theta, max_seq),
            oracle.Model(cfg.qualifier, q, cfg.dtype, cfg.rope_theta, max_seq),
            oracle.Model(cfg.target, t, cfg.dtype, cfg.rope_theta, max_seq))


def test_identical_models_accept_everything_and_equal_plain_sampling(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ms = 16 + 40 + 10
    for (k1, k2, tau) in ((4, 8, 0.0), (3, 7, 0.2), (1, 1, 0.0), (5, 3, 0.0)):
        A, B, C = (oracle.Model(cfg.qualifier, q, cfg.dtype, cfg.rope_theta, ms) for _ in range(3))
        out, st = oracle.generate(A, B, C, prompt, 40, 5, k1, k2, tau, tau)
        assert st["accepted_q"] == st["proposed_q"] and st["accepted_t"] == st["proposed_t"]
        assert st["fuzzy_q"] == st["proposed_q"]      # divergence is exactly 0 <= tau
        P = oracle.Model(cfg.qualifier, q, cfg.dtype, cfg.rope_theta, ms)
        plain = oracle.generate_plain(P, prompt, 40, 5)
        assert np.array_equal(out, plain)


def test_counters_and_determinism(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ms = cfg.n_prompt + cfg.n_new + cfg.k2 + 2
    for (Tq, Tt) in ((cfg.T_q, cfg.T_t), (0.004, 0.012), (0.0, 0.0)):
        D, Q, T = _models(cfg, d, q, t, ms)
        out, st = oracle.generate(D, Q, T, prompt, cfg.n_new, cfg.sample_seed, cfg.k1, cfg.k2, Tq, Tt)
        assert out.shape == (cfg.n_new,) and (out >= 0).all() and (out < cfg.target.vocab).all()
        assert st["accepted_q"] <= st["proposed_q"] and st["accepted_t"] <= st["proposed_t"]
        assert st["proposed_t"] == cfg.k2 * st["passes_t"]
        assert st["passes_d"] == st["proposed_q"]
        # every target pass commits between 1 and k2 + 1 tokens
        assert st["passes_t"] <= cfg.n_new and st["passes_t"] * (cfg.k2 + 1) >= cfg.n_new
        assert st["accepted_t"] + st["passes_t"] >= cfg.n_new
        D2, Q2, T2 = _models(cfg, d, q, t, ms)
        out2, st2 = oracle.generate(D2, Q2, T2, prompt, cfg.n_new, cfg.sample_seed, cfg.k1, cfg.k2, Tq, Tt)
        assert np.array_equal(out, out2) and st == st2
        if Tq == 0.004:
            assert 0 < st["accepted_q"] < st["proposed_q"]   # this setting exercises rejections
            assert 0 < st["accepted_t"] < st["proposed_t"]


def test_prefix_property_and_thresholds_matter(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ms = 16 + 48 + 10
    D, Q, T = _models(cfg, d, q, t, ms)
    a, _ = oracle.generate(D, Q, T, prompt, 48, 3, 4, 8, 0.004, 0.012)
    D, Q, T = _models(cfg, d, q, t, ms)
    b, _ = oracle.generate(D, Q, T, prompt, 20, 3, 4, 8, 0.004, 0.012)
    assert np.array_equal(a[:20], b)                       # n_new only truncates
    D, Q, T = _models(cfg, d, q, t, ms)
    c, stc = oracle.generate(D, Q, T, prompt, 48, 3, 4, 8, 1.0, 1.0)   # above ln 2: everything passes
    assert stc["accepted_q"] == stc["proposed_q"] and stc["accepted_t"] == stc["proposed_t"]
    assert not np.array_equal(a, c)


def test_tau0_loop_reproduces_target_chain_on_vocab8():
    # tau_Q = tau_T = 0: both stages are standard SD, so the emitted tokens follow the target's
    # ancestral law whatever draft and qualifier are.  Vocabulary 8, two generated tokens,
    # k1 = 1, k2 = 2, three unrelated tiny transformers with sharp-ish distributions.
    V = 8
    sh = lambda L, d: ModelShape(L, d, 2, 1, 2 * d, V)
    sD, sQ, sT = sh(1, 8), sh(1, 16), sh(2, 16)
    wD = synth.target_weights(sD, 11, synth.DTYPE_F32, sigma=0.6)
    wQ = synth.target_weights(sQ, 12, synth.DTYPE_F32, sigma=0.5)
    wT = synth.target_weights(sT, 13, synth.DTYPE_F32, sigma=0.5)
    prompt = np.array([3, 5], dtype=np.int32)
    ms = 2 + 2 + 2 + 2
    # exact target chain law from the target's own probabilities
    T = oracle.Model(sT, wT, synth.DTYPE_F32, 10000.0, ms)
    p0 = oracle.softmax(T.forward(prompt, 0)[-1].astype(np.float32))
    joint = np.zeros((V, V))
    for a in range(V):
        pa = oracle.softmax(T.forward(np.array([3, 5, a]), 0)[-1].astype(np.float32))
        joint[a] = p0[a] * pa
    D = oracle.Model(sD, wD, synth.DTYPE_F32, 10000.0, ms)
    Q = oracle.Model(sQ, wQ, synth.DTYPE_F32, 10000.0, ms)
    N = 30000
    counts = np.zeros((V, V))
    acc_q = prop_q = acc_t = prop_t = 0
    for s in range(N):
        out, st = oracle.generate(D, Q, T, prompt, 2, s, 1, 2, 0.0, 0.0)
        counts[out[0], out[1]] += 1
        acc_q += st["accepted_q"]; prop_q += st["proposed_q"]; acc_t += st["accepted_t"]; prop_t += st["proposed_t"]
    assert 0.05 < acc_q / prop_q < 0.95 and 0.05 < acc_t / prop_t < 0.95   # both stages really reject
    exp = joint * N
    keep = exp > 5
    chi2 = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    assert chi2 < scipy.stats.chi2.ppf(0.9999, keep.sum() - 1)
    first = counts.sum(1)
    assert ((first - N * p0) ** 2 / (N * p0)).sum() < scipy.stats.chi2.ppf(0.9999, V - 1)
