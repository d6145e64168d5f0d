"""Pins of the cache bookkeeping of the oracle's loops (Figure 1 caption: tokens rejected by the qualifier or the
target are discarded, so every model must go on from the tokens that survived).

Every law test of the loop is blind to the draft's and the qualifier's caches: at tau = 0 the output follows the
target whatever the other two models see, identical models never reject, greedy decoding is lossless for any
draft.  Two pins close that gap:
  * every logits row a loop consumes (observer hook) equals a fresh, cache-free recomputation of the same
    prefix: recomputation is the part of the forward pinned against library operators elsewhere;
  * with tau_Q = 0 and tau_T >= ln 2 the window is exact speculative sampling from the QUALIFIER and the target
    accepts all of it, so the emitted tokens follow the qualifier's ancestral chain: a law that depends on the
    qualifier seeing the right context after every rejection.
A planted mistake (in a patched copy of the oracle's source, on the CPU) shows that the first pin bites."""
import ctypes as C
import math
import os
import subprocess

import numpy as np
import pytest
import scipy.stats

import oracle
from paper_2510_12966_amd import synth
from paper_2510_12966_amd.synth import ModelShape

V = 8
THETA = 10000.0


def _shapes():
    sh = lambda L, d: ModelShape(L, d, 2, 1, 2 * d, V)
    return sh(1, 8), sh(1, 16), sh(2, 16)


def _weights():
    sD, sQ, sT = _shapes()
    return (synth.target_weights(sD, 21, synth.DTYPE_F32, sigma=0.6), synth.target_weights(sQ, 22, synth.DTYPE_F32, sigma=0.5),
            synth.target_weights(sT, 23, synth.DTYPE_F32, sigma=0.5))


class Recompute:
    """Cache-free logits of a prefix: a fresh forward over the whole prefix from position 0, memoised."""

    def __init__(self, shapes, blobs, max_seq):
        self.models = [oracle.Model(s, b, synth.DTYPE_F32, THETA, max_seq) for s, b in zip(shapes, blobs)]
        self.memo = [{}, {}, {}]

    def row(self, which, prefix):
        key = tuple(int(t) for t in prefix)
        if key not in self.memo[which]:
            self.memo[which][key] = self.models[which].forward(np.array(key, dtype=np.int32), 0)[-1]
        return self.memo[which][key]


def test_every_row_the_loops_consume_equals_a_cache_free_recomputation():
    shapes, blobs = _shapes(), _weights()
    prompt = np.array([3, 5, 1], dtype=np.int32)
    n_new = 9
    settings = [(2, 3, 0.0, 1.0), (2, 3, 0.0, 0.0), (3, 5, 0.02, 0.02), (1, 1, 0.0, 0.0), (4, 2, 0.0, 0.05), (2, 6, 0.0, 0.0)]
    seen = {0: 0, 1: 0, 2: 0}
    rejected_q = rejected_t = 0
    for k1, k2, Tq, Tt in settings:
        ms = len(prompt) + n_new + k2 + 2
        rec = Recompute(shapes, blobs, ms)
        worst = [0.0]

        def check(which, prefix, row):
            want = rec.row(which, prefix)
            worst[0] = max(worst[0], float(np.abs(row.astype(np.float64) - want.astype(np.float32)).max()))
            seen[which] += 1

        oracle.set_row_trace(check)
        try:
            for seed in range(40):
                D, Q, T = (oracle.Model(s, b, synth.DTYPE_F32, THETA, ms) for s, b in zip(shapes, blobs))
                out, st = oracle.generate(D, Q, T, prompt, n_new, seed, k1, k2, Tq, Tt)
                rejected_q += st["proposed_q"] - st["accepted_q"]
                rejected_t += st["proposed_t"] - st["accepted_t"]
        finally:
            oracle.set_row_trace(None)
        assert worst[0] == 0.0, (k1, k2, Tq, Tt, worst[0])   # same fp64 arithmetic per token, cached or not
    assert min(seen.values()) > 500 and rejected_q > 200 and rejected_t > 100   # rollbacks really happened
    # the two-model loop and the assisted loop roll back the same way
    ms = len(prompt) + n_new + 5 + 2
    rec = Recompute(shapes, blobs, ms)
    bad = []
    oracle.set_row_trace(lambda which, prefix, row: bad.append(1) if np.abs(row - rec.row(which, prefix).astype(np.float32)).max() != 0 else None)
    try:
        for seed in range(20):
            D, Q, T = (oracle.Model(s, b, synth.DTYPE_F32, THETA, ms) for s, b in zip(shapes, blobs))
            oracle.generate_assisted(D, Q, T, prompt, n_new, seed, 2, 4, 0.0)
        rec2 = Recompute((shapes[1], shapes[1], shapes[2]), (blobs[1], blobs[1], blobs[2]), ms)
        oracle.set_row_trace(lambda which, prefix, row: bad.append(1) if np.abs(row - rec2.row(which, prefix).astype(np.float32)).max() != 0 else None)
        for seed in range(20):
            P, T = oracle.Model(shapes[1], blobs[1], synth.DTYPE_F32, THETA, ms), oracle.Model(shapes[2], blobs[2], synth.DTYPE_F32, THETA, ms)
            oracle.generate_sd(P, T, prompt, n_new, seed, 3, 0.0)
    finally:
        oracle.set_row_trace(None)
    assert not bad


def test_strict_first_stage_and_open_second_stage_emit_the_qualifiers_chain():
    # tau_Q = 0: stage 1 is exact speculative sampling, the window follows the qualifier's law whatever the draft
    # proposes; tau_T >= ln 2: the target accepts the whole window and adds its bonus token.  k1 = 2, k2 = 3,
    # four new tokens = one outer iteration: tokens 1-3 ~ qualifier chain, token 4 ~ target given those three.
    shapes, blobs = _shapes(), _weights()
    prompt = np.array([3, 5], dtype=np.int32)
    ms = 2 + 4 + 3 + 2
    rec = Recompute(shapes, blobs, ms)
    pq = lambda prefix: oracle.softmax(rec.row(1, prefix).astype(np.float32))
    pt = lambda prefix: oracle.softmax(rec.row(2, prefix).astype(np.float32))
    law = np.zeros((V, V, V))
    for a in range(V):
        for b in range(V):
            law[a, b] = pq([3, 5])[a] * pq([3, 5, a])[b] * pq([3, 5, a, b])
    N = 40000
    counts = np.zeros((V, V, V))
    fourth = np.zeros(V); fourth_exp = np.zeros(V)
    rej = prop = 0
    D, Q, T = (oracle.Model(s, b, synth.DTYPE_F32, THETA, ms) for s, b in zip(shapes, blobs))
    for seed in range(N):
        out, st = oracle.generate(D, Q, T, prompt, 4, seed, 2, 3, 0.0, math.log(2) + 1e-9)
        assert st["accepted_t"] == st["proposed_t"] == 3 and st["passes_t"] == 1
        counts[out[0], out[1], out[2]] += 1
        rej += st["proposed_q"] - st["accepted_q"]; prop += st["proposed_q"]
        if seed < 6000:
            fourth[out[3]] += 1
            fourth_exp += pt([3, 5, out[0], out[1], out[2]])
    assert 0.15 < rej / prop < 0.9   # the qualifier really rejects, so its cache is rolled back all the time
    exp = law * N
    keep = exp > 5
    chi2 = ((counts[keep] - exp[keep]) ** 2 / exp[keep]).sum()
    assert chi2 < scipy.stats.chi2.ppf(0.9999, keep.sum() - 1), chi2
    assert ((fourth - fourth_exp) ** 2 / fourth_exp).sum() < scipy.stats.chi2.ppf(0.9999, V - 1)
    # and it is NOT the target's chain: the test separates the two laws
    lawT = np.zeros((V, V, V))
    for a in range(V):
        for b in range(V):
            lawT[a, b] = pt([3, 5])[a] * pt([3, 5, a])[b] * pt([3, 5, a, b])
    expT = lawT * N
    keepT = expT > 5
    assert ((counts[keepT] - expT[keepT]) ** 2 / expT[keepT]).sum() > 10 * scipy.stats.chi2.ppf(0.9999, keepT.sum() - 1)


MUTATIONS = [
    # the qualifier keeps the rejected proposal's cache row as if it were the replacement's
    ("lenQ = imin(lenQ, L + n);", "lenQ = imin(lenQ, L + n + 1);"),
    # the draft does
    ("lenD = imin(lenD, L + n);", "lenD = imin(lenD, L + n + 1);"),
    # after the target stage the qualifier is not cut back at all
    ("lenT = imin(lenT, C + n); lenQ = imin(lenQ, C + n); lenD = imin(lenD, C + n);",
     "lenT = imin(lenT, C + n); lenD = imin(lenD, C + n);"),
    # ... nor the draft
    ("lenT = imin(lenT, C + n); lenQ = imin(lenQ, C + n); lenD = imin(lenD, C + n);",
     "lenT = imin(lenT, C + n); lenQ = imin(lenQ, C + n);"),
]


@pytest.mark.parametrize("old,new", MUTATIONS)
def test_a_planted_rollback_mistake_is_caught_by_the_row_pin(tmp_path, old, new):
    src = open(os.path.join(os.path.dirname(oracle.__file__), "psd_oracle.c")).read()
    assert src.count(old) == 1
    c_file, so = tmp_path / "mutant.c", tmp_path / "mutant.so"
    c_file.write_text(src.replace(old, new))
    subprocess.check_call(["gcc", "-O1", "-fopenmp", "-shared", "-fPIC", "-o", str(so), str(c_file), "-lm"])
    L = C.CDLL(str(so))
    L.orc_model_create.restype = C.c_void_p
    L.orc_model_create.argtypes = [C.c_int] * 6 + [C.c_double, C.c_double, C.c_int, C.c_void_p, C.c_int]
    L.orc_model_destroy.argtypes = [C.c_void_p]
    L.orc_generate.restype = C.c_int
    L.orc_generate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(oracle.Params), C.c_void_p, C.c_int, C.c_int,
                               C.c_uint64, C.c_void_p, C.POINTER(oracle.Stats)]
    L.orc_set_row_trace.argtypes = [oracle.ROW_TRACE_FN, C.c_void_p]
    shapes, blobs = _shapes(), _weights()
    prompt = np.array([3, 5, 1], dtype=np.int32)
    n_new, k1, k2 = 9, 2, 3
    ms = len(prompt) + n_new + k2 + 2
    rec = Recompute(shapes, blobs, ms)   # the unpatched oracle's cache-free forward
    wrong = [0]

    def cb(user, which, prefix, n_prefix, row, Vv):
        got = np.ctypeslib.as_array(row, shape=(Vv,))
        want = rec.row(which, np.ctypeslib.as_array(prefix, shape=(n_prefix,))).astype(np.float32)
        wrong[0] += int(np.abs(got - want).max() > 1e-6)

    fn = oracle.ROW_TRACE_FN(cb)
    L.orc_set_row_trace(fn, None)
    for seed in range(30):
        hs = [L.orc_model_create(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.d_ffn, s.vocab, THETA, 1e-5, 0, b.ctypes.data, ms)
              for s, b in zip(shapes, blobs)]
        prm = oracle.Params(0.0, 0.0, 1.0, k1, k2)
        out = np.empty(n_new, dtype=np.int32)
        st = oracle.Stats()
        rc = L.orc_generate(hs[0], hs[1], hs[2], C.byref(prm), prompt.ctypes.data, prompt.size, n_new, seed, out.ctypes.data, C.byref(st))
        del rc   # (a loop whose cache lengths stop fitting the sequence also reports an error; the rows are the pin)
        for h in hs:
            L.orc_model_destroy(h)
    L.orc_set_row_trace(oracle.ROW_TRACE_FN(0), None)
    assert wrong[0] > 0
