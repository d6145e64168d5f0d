"""ctypes binding of the CPU oracle (``psd_oracle.c``).

TEST INFRASTRUCTURE ONLY: imported by tests/, by ``__graft_entry__.smoke()`` and by
the ``cpu_baseline`` leg of ``bench.py``.  The HIP library and its Python binding
never import this package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "psd_oracle.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-Wall", "-shared", "-fPIC", "-o", _SO, src, "-lm"])
    return _SO


class AcceptResult(C.Structure):
    _fields_ = [("n_accepted", C.c_int32), ("next_token", C.c_int32), ("n_fuzzy", C.c_int32), ("pad", C.c_int32),
                ("margin_div", C.c_double), ("margin_coin", C.c_double), ("margin_race", C.c_double)]


class Params(C.Structure):
    _fields_ = [("T_q", C.c_double), ("T_t", C.c_double), ("temperature", C.c_double),
                ("k1", C.c_int32), ("k2", C.c_int32)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("proposed_q", "accepted_q", "fuzzy_q", "proposed_t", "accepted_t",
                                         "fuzzy_t", "passes_d", "passes_q", "passes_t")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class Adapt(C.Structure):
    """Ranges of the adaptive controller (see psd_oracle.c)."""
    _fields_ = [("k2_min", C.c_int32), ("k2_max", C.c_int32), ("k1_max", C.c_int32), ("steps", C.c_int32),
                ("period", C.c_int32), ("T_q_min", C.c_float), ("T_q_max", C.c_float), ("T_t_min", C.c_float),
                ("T_t_max", C.c_float)]


class AdaptState(C.Structure):
    _fields_ = [("k1", C.c_int32), ("k2", C.c_int32), ("s_q", C.c_int32), ("s_t", C.c_int32), ("since", C.c_int32),
                ("p_q", C.c_int64), ("a_q", C.c_int64), ("p_t", C.c_int64), ("a_t", C.c_int64)]

    def params(self):
        return (self.k1, self.k2, self.s_q, self.s_t)


ROW_TRACE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_int, C.POINTER(C.c_int32), C.c_int, C.POINTER(C.c_float), C.c_int)

_LIB = None
_ROW_TRACE_CB = None


def lib():
    global _LIB
    if _LIB is None:
        L = C.CDLL(build())
        L.orc_philox4x32_10.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_uniform.restype = C.c_double
        L.orc_uniform.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32]
        L.orc_softmax.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_void_p]
        L.orc_jsd.restype = C.c_double
        L.orc_jsd.argtypes = [C.c_void_p, C.c_void_p, C.c_int]
        L.orc_race.restype = C.c_int
        L.orc_race.argtypes = [C.c_void_p, C.c_int, C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        L.orc_accept_scan.restype = C.c_int
        L.orc_accept_scan.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_void_p,
                                      C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
        L.orc_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_double,
                                 C.c_uint64, C.c_uint32, C.c_uint32, C.c_int, C.POINTER(AcceptResult), C.c_void_p]
        L.orc_sample_row.restype = C.c_int
        L.orc_sample_row.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_uint64, C.c_uint32, C.c_uint32,
                                     C.c_uint32, C.c_void_p]
        L.orc_model_create.restype = C.c_void_p
        L.orc_model_create.argtypes = [C.c_int] * 6 + [C.c_double, C.c_double, C.c_int, C.c_void_p, C.c_int]
        L.orc_model_destroy.argtypes = [C.c_void_p]
        L.orc_forward.restype = C.c_int
        L.orc_forward.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        L.orc_rope.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_double]
        L.orc_generate.restype = C.c_int
        L.orc_generate.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Params), C.c_void_p, C.c_int,
                                   C.c_int, C.c_uint64, C.c_void_p, C.POINTER(Stats)]
        L.orc_row_stats.argtypes = [C.c_void_p, C.c_int, C.c_double, C.c_void_p, C.c_void_p]
        L.orc_accept_assisted.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_double, C.c_uint64, C.c_uint32,
                                          C.c_uint32, C.c_int, C.c_void_p]
        L.orc_generate_assisted.restype = C.c_int
        L.orc_generate_assisted.argtypes = L.orc_generate.argtypes
        L.orc_accept_greedy.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        L.orc_generate_greedy.restype = C.c_int
        L.orc_generate_greedy.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Params), C.c_void_p, C.c_int,
                                          C.c_int, C.c_void_p, C.c_void_p]
        L.orc_generate_sd.restype = C.c_int
        L.orc_generate_sd.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_double, C.c_double, C.c_void_p, C.c_int,
                                      C.c_int, C.c_uint64, C.c_void_p, C.c_void_p]
        L.orc_generate_plain.restype = C.c_int
        L.orc_generate_plain.argtypes = [C.c_void_p, C.c_double, C.c_void_p, C.c_int, C.c_int, C.c_uint64,
                                         C.c_void_p]
        L.orc_adapt_threshold.restype = C.c_double
        L.orc_adapt_threshold.argtypes = [C.c_float, C.c_float, C.c_int, C.c_int]
        L.orc_adapt_init.argtypes = [C.POINTER(Adapt), C.c_double, C.c_double, C.c_int, C.POINTER(AdaptState)]
        L.orc_adapt_step.argtypes = [C.POINTER(Adapt), C.POINTER(AdaptState), C.c_int, C.c_int64, C.c_int64]
        L.orc_generate_adaptive.restype = C.c_int
        L.orc_generate_adaptive.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.POINTER(Params), C.POINTER(Adapt), C.c_void_p,
                                            C.c_int, C.c_int, C.c_uint64, C.c_void_p, C.POINTER(Stats), C.c_void_p, C.c_int]
        L.orc_philox_block.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_void_p]
        L.orc_residual.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_void_p]
        L.orc_set_row_trace.argtypes = [ROW_TRACE_FN, C.c_void_p]
        _LIB = L
    return _LIB


DRAW_SAMPLE, DRAW_COIN, DRAW_RESAMPLE = 0, 1, 2


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().orc_philox4x32_10(c.ctypes.data, k.ctypes.data, out.ctypes.data)
    return out


def philox_block(seed, c0, n, c1, c2, c3):
    """Generator output [n, 4] (uint32) for the counters (c0 .. c0 + n - 1, c1, c2, c3) under key `seed`."""
    out = np.empty((n, 4), dtype=np.uint32)
    lib().orc_philox_block(seed, c0, n, c1, c2, c3, out.ctypes.data)
    return out


def residual(p, q):
    """Un-normalised replacement weights max(0, p - q) of a rejected position."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    r = np.empty_like(p)
    lib().orc_residual(p.ctypes.data, q.ctypes.data, p.size, r.ctypes.data)
    return r


def set_row_trace(fn):
    """fn(which, prefix tokens (numpy copy), logits row (numpy copy)) for every row a generation loop consumes; None: off."""
    global _ROW_TRACE_CB
    if fn is None:
        _ROW_TRACE_CB = ROW_TRACE_FN(0)
    else:
        def cb(user, which, prefix, n_prefix, row, V):
            fn(which, np.ctypeslib.as_array(prefix, shape=(n_prefix,)).copy(), np.ctypeslib.as_array(row, shape=(V,)).copy())
        _ROW_TRACE_CB = ROW_TRACE_FN(cb)
    lib().orc_set_row_trace(_ROW_TRACE_CB, None)


def uniform(seed, v, position, purpose, stage):
    return lib().orc_uniform(seed, v, position, purpose, stage)


def softmax(logits, temperature=1.0):
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    p = np.empty(lg.shape[-1], dtype=np.float64)
    lib().orc_softmax(lg.ctypes.data, lg.shape[-1], temperature, p.ctypes.data)
    return p


def jsd(p, q):
    p = np.ascontiguousarray(p, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    return lib().orc_jsd(p.ctypes.data, q.ctypes.data, p.size)


def race(w, seed, position, purpose, stage):
    w = np.ascontiguousarray(w, dtype=np.float64)
    gap = C.c_double(0)
    t = lib().orc_race(w.ctypes.data, w.size, seed, position, purpose, stage, C.byref(gap))
    return t, gap.value


def accept_scan(p, q, x, T, u_coin):
    """Decision core on explicit distributions p [k, V], q [k, V] and explicit coin uniforms."""
    p = np.ascontiguousarray(p, dtype=np.float64)
    q = np.ascontiguousarray(q, dtype=np.float64)
    x = np.ascontiguousarray(x, dtype=np.int32)
    u = np.ascontiguousarray(u_coin, dtype=np.float64)
    k, V = q.shape
    div = np.full(k, np.nan)
    fuzzy = C.c_int32(0)
    n = lib().orc_accept_scan(p.ctypes.data, q.ctypes.data, x.ctypes.data, k, V, T, u.ctypes.data, div.ctypes.data,
                              C.byref(fuzzy), None, None)
    return n, div, fuzzy.value


def accept(logits_p, logits_q, x, T, temperature=1.0, seed=0, position0=0, stage=1, take_bonus=True):
    lp = np.ascontiguousarray(logits_p, dtype=np.float32)
    lq = np.ascontiguousarray(logits_q, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.int32)
    k, V = lq.shape if lq.ndim == 2 else (0, lp.shape[-1])
    assert lp.shape == (k + 1, V)
    div = np.zeros(max(k, 1), dtype=np.float64)
    res = AcceptResult()
    lib().orc_accept(lp.ctypes.data, lq.ctypes.data, x.ctypes.data, k, V, T, temperature, seed, position0, stage,
                     int(take_bonus), C.byref(res), div.ctypes.data)
    return res, div[:k]


def row_stats(logits, temperature=1.0):
    """(entropy in nats, largest probability) of softmax(logits / temperature), one row (Section 4)."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    h, m = C.c_double(0), C.c_double(0)
    lib().orc_row_stats(lg.ctypes.data, lg.size, temperature, C.byref(h), C.byref(m))
    return h.value, m.value


def accept_assisted(logits_p, x, temperature=1.0, seed=0, position0=0, stage=1, take_bonus=True):
    """Assisted stage (Section 3.4): strict token match against the verifier's argmax, fallback draw from the verifier."""
    lp = np.ascontiguousarray(logits_p, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.int32)
    k, V = lp.shape[0] - 1, lp.shape[1]
    assert x.size == k
    res = AcceptResult()
    lib().orc_accept_assisted(lp.ctypes.data, x.ctypes.data, k, V, temperature, seed, position0, stage,
                              int(take_bonus), C.byref(res))
    return res


def sample_row(logits, temperature, seed, position, purpose=DRAW_SAMPLE, stage=0):
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    gap = C.c_double(0)
    t = lib().orc_sample_row(lg.ctypes.data, lg.size, temperature, seed, position, purpose, stage, C.byref(gap))
    return t, gap.value


def rope(v, n_heads, hd, pos, theta):
    a = np.array(v, dtype=np.float64).reshape(n_heads * hd)
    lib().orc_rope(a.ctypes.data, n_heads, hd, pos, theta)
    return a


class Model:
    """One Llama-style decoder with its own fp64 KV cache.  ``blob`` must outlive the model."""

    def __init__(self, shape, blob, dtype, rope_theta, max_seq, rms_eps=1e-5):
        self.shape, self.blob, self.dtype = shape, blob, dtype
        self.h = lib().orc_model_create(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.d_ffn,
                                        shape.vocab, rope_theta, rms_eps, dtype, blob.ctypes.data, max_seq)

    def forward(self, tokens, pos0, want_logits=True):
        t = np.ascontiguousarray(tokens, dtype=np.int32)
        lg = np.empty((t.size, self.shape.vocab), dtype=np.float64) if want_logits else None
        rc = lib().orc_forward(self.h, t.ctypes.data, t.size, pos0, lg.ctypes.data if want_logits else None)
        if rc != 0:
            raise ValueError(f"orc_forward failed: {rc}")
        return lg

    def close(self):
        if self.h:
            lib().orc_model_destroy(self.h)
            self.h = None

    def __del__(self):
        self.close()


def generate(D, Q, T, prompt, n_new, seed, k1, k2, T_q, T_t, temperature=1.0):
    prm = Params(T_q, T_t, temperature, k1, k2)
    pr = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.empty(n_new, dtype=np.int32)
    st = Stats()
    rc = lib().orc_generate(D.h, Q.h, T.h, C.byref(prm), pr.ctypes.data, pr.size, n_new, seed, out.ctypes.data,
                            C.byref(st))
    if rc != 0:
        raise ValueError(f"orc_generate failed: {rc}")
    return out, st.as_dict()


def generate_assisted(D, Q, T, prompt, n_new, seed, k1, k2, T_t, temperature=1.0):
    prm = Params(0.0, T_t, temperature, k1, k2)
    pr = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.empty(n_new, dtype=np.int32)
    st = Stats()
    rc = lib().orc_generate_assisted(D.h, Q.h, T.h, C.byref(prm), pr.ctypes.data, pr.size, n_new, seed,
                                     out.ctypes.data, C.byref(st))
    if rc != 0:
        raise ValueError(f"orc_generate_assisted failed: {rc}")
    return out, st.as_dict()


def accept_greedy(logits_p, x, take_bonus=True):
    """Greedy stage (temperature -> 0 limit): exact match against the verifier's top prediction, no draws."""
    lp = np.ascontiguousarray(logits_p, dtype=np.float32)
    x = np.ascontiguousarray(x, dtype=np.int32)
    k, V = lp.shape[0] - 1, lp.shape[1]
    assert x.size == k
    res = AcceptResult()
    lib().orc_accept_greedy(lp.ctypes.data, x.ctypes.data, k, V, int(take_bonus), C.byref(res))
    return res


def generate_greedy(D, Q, T, prompt, n_new, k1, k2):
    prm = Params(0.0, 0.0, 1.0, k1, k2)
    pr = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.empty(n_new, dtype=np.int32)
    st = Stats()
    rc = lib().orc_generate_greedy(D.h, Q.h, T.h, C.byref(prm), pr.ctypes.data, pr.size, n_new, out.ctypes.data,
                                   C.byref(st))
    if rc != 0:
        raise ValueError(f"orc_generate_greedy failed: {rc}")
    return out, st.as_dict()


def generate_sd(P, T, prompt, n_new, seed, k, tau, temperature=1.0):
    """Two-model speculative decoding: P proposes k tokens, T verifies with threshold tau (0 = standard SD)."""
    pr = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.empty(n_new, dtype=np.int32)
    st = Stats()
    rc = lib().orc_generate_sd(P.h, T.h, k, tau, temperature, pr.ctypes.data, pr.size, n_new, seed, out.ctypes.data,
                               C.byref(st))
    if rc != 0:
        raise ValueError(f"orc_generate_sd failed: {rc}")
    return out, st.as_dict()


def generate_plain(M, prompt, n_new, seed, temperature=1.0):
    pr = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.empty(n_new, dtype=np.int32)
    rc = lib().orc_generate_plain(M.h, temperature, pr.ctypes.data, pr.size, n_new, seed, out.ctypes.data)
    if rc != 0:
        raise ValueError(f"orc_generate_plain failed: {rc}")
    return out


def adapt_threshold(lo, hi, s, steps):
    return lib().orc_adapt_threshold(lo, hi, s, steps)


def adapt_init(ad, T_q, T_t, k2):
    st = AdaptState()
    lib().orc_adapt_init(C.byref(ad), T_q, T_t, k2, C.byref(st))
    return st


def adapt_step(ad, st, n_t, p_q, a_q):
    lib().orc_adapt_step(C.byref(ad), C.byref(st), n_t, p_q, a_q)
    return st


def generate_adaptive(D, Q, T, prompt, n_new, seed, k2, T_q, T_t, ad, temperature=1.0):
    """The loop under the adaptive controller; returns (tokens, stats, log [iterations, 4] of (k1, k2, s_q, s_t))."""
    prm = Params(T_q, T_t, temperature, 1, k2)
    pr = np.ascontiguousarray(prompt, dtype=np.int32)
    out = np.empty(n_new, dtype=np.int32)
    st = Stats()
    log = np.full((max(n_new, 1), 4), -1, dtype=np.int32)
    rc = lib().orc_generate_adaptive(D.h, Q.h, T.h, C.byref(prm), C.byref(ad), pr.ctypes.data, pr.size, n_new, seed,
                                     out.ctypes.data, C.byref(st), log.ctypes.data, log.shape[0])
    if rc != 0:
        raise ValueError(f"orc_generate_adaptive failed: {rc}")
    return out, st.as_dict(), log[log[:, 0] >= 0]
