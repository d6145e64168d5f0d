"""ctypes binding of libpsd.so: same names as the C ABI in include/psd.h, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
F32, BF16 = 0, 1
FLAG_GRAPH = 1
FLAG_ASSISTED = 2
FLAG_ROW_STATS = 4
FLAG_GREEDY = 8
MAX_WIDTH = 32


class PsdError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"psd error {code}: {msg}")
        self.code = code


def lib_path() -> str:
    return os.path.join(_HERE, "libpsd.so")


class _ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rope_theta", C.c_float), ("rms_eps", C.c_float),
                ("dtype", C.c_int32), ("reserved", C.c_int32), ("weights", C.c_void_p), ("weights_bytes", C.c_size_t)]


class _Params(C.Structure):
    _fields_ = [("T_q", C.c_float), ("T_t", C.c_float), ("temperature", C.c_float), ("k1", C.c_int32),
                ("k2", C.c_int32), ("max_seq", C.c_int32), ("device", C.c_int32), ("flags", C.c_int32),
                ("pool_bytes", C.c_size_t)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in ("proposed_q", "accepted_q", "fuzzy_q", "proposed_t", "accepted_t", "fuzzy_t",
                                         "passes_d", "passes_q", "passes_t")] + \
               [(n, C.c_double) for n in ("ms_prefill", "ms_decode", "ms_d", "ms_q", "ms_t", "ms_accept")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class Adapt(C.Structure):
    """psd_adapt: ranges of the adaptive controller."""
    _fields_ = [("k2_min", C.c_int32), ("k2_max", C.c_int32), ("k1_max", C.c_int32), ("steps", C.c_int32),
                ("period", C.c_int32), ("T_q_min", C.c_float), ("T_q_max", C.c_float), ("T_t_min", C.c_float),
                ("T_t_max", C.c_float)]


class KernelStat(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("ms_total", C.c_double), ("bytes_total", C.c_double)]


TRACE_FN = C.CFUNCTYPE(None, C.c_void_p, C.c_int32, C.c_uint32, C.c_int32, C.c_int32, C.POINTER(C.c_float),
                       C.POINTER(C.c_float), C.POINTER(C.c_int32), C.c_int32, C.c_int32, C.POINTER(C.c_float))

_LIB = None


def lib():
    """Loads libpsd.so; there is no fallback: without the HIP library nothing on the decoding path runs."""
    global _LIB
    if _LIB is None:
        path = lib_path()
        if not os.path.exists(path):
            raise PsdError(-100, f"{path} is missing: build it with `python -m paper_2510_12966_amd.build`")
        L = C.CDLL(path)
        L.psd_strerror.restype = C.c_char_p
        L.psd_last_error.restype = C.c_char_p
        L.psd_last_error.argtypes = [C.c_void_p]
        L.psd_accept.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_float,
                                 C.c_uint64, C.c_uint32, C.c_uint32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p,
                                 C.c_void_p]
        L.psd_set_accept_path.argtypes = [C.c_int32]
        L.psd_accept_workspace_bytes.restype = C.c_size_t
        L.psd_accept_workspace_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
        L.psd_accept_batch.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_float,
                                       C.c_float, C.c_uint64, C.c_uint32, C.c_uint32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
        L.psd_accept_noalloc_capacity.restype = C.c_size_t
        L.psd_accept_batch_noalloc.argtypes = L.psd_accept_batch.argtypes[:15] + [C.c_void_p]
        L.psd_philox_block.argtypes = [C.c_uint64, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_uint32, C.c_int32,
                                       C.c_void_p, C.c_void_p]
        L.psd_sample.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_uint64, C.c_uint32, C.c_int32,
                                 C.c_void_p]
        L.psd_dev_alloc.argtypes = [C.c_size_t, C.POINTER(C.c_void_p)]
        L.psd_dev_free.argtypes = [C.c_void_p]
        L.psd_dev_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int32]
        L.psd_create.argtypes = [C.POINTER(_ModelDesc), C.POINTER(_ModelDesc), C.POINTER(_ModelDesc),
                                 C.POINTER(_Params), C.POINTER(C.c_void_p)]
        L.psd_destroy.argtypes = [C.c_void_p]
        L.psd_destroy.restype = None
        L.psd_pool_bytes_needed.restype = C.c_size_t
        L.psd_pool_bytes_needed.argtypes = [C.POINTER(_ModelDesc), C.POINTER(_ModelDesc), C.POINTER(_ModelDesc),
                                            C.POINTER(_Params)]
        L.psd_set_decoding.argtypes = [C.c_void_p, C.c_float, C.c_float, C.c_int32, C.c_int32, C.c_float]
        L.psd_generate.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64, C.c_void_p,
                                   C.POINTER(Stats)]
        L.psd_generate_plain.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_uint64,
                                         C.c_void_p, C.POINTER(Stats)]
        L.psd_generate_sd.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_void_p, C.c_int32, C.c_int32,
                                      C.c_uint64, C.c_void_p, C.POINTER(Stats)]
        L.psd_set_assisted.argtypes = [C.c_void_p, C.c_int32]
        L.psd_set_row_stats.argtypes = [C.c_void_p, C.c_int32]
        L.psd_set_greedy.argtypes = [C.c_void_p, C.c_int32]
        L.psd_get_row_stats.argtypes = [C.c_void_p, C.c_void_p]
        L.psd_row_stats.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_int32, C.c_void_p, C.c_void_p]
        L.psd_accept_assisted.argtypes = [C.c_void_p, C.c_void_p, C.c_int32, C.c_int32, C.c_float, C.c_uint64, C.c_uint32,
                                          C.c_uint32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        L.psd_set_adaptive.argtypes = [C.c_void_p, C.POINTER(Adapt)]
        L.psd_get_adaptive_log.argtypes = [C.c_void_p, C.c_void_p, C.c_int32]
        L.psd_forward.argtypes = [C.c_void_p, C.c_int32, C.c_void_p, C.c_int32, C.c_int32, C.c_void_p]
        L.psd_set_trace.argtypes = [C.c_void_p, TRACE_FN, C.c_void_p]
        L.psd_profile.argtypes = [C.c_void_p, C.c_int32]
        L.psd_kernel_stats.argtypes = [C.c_void_p, C.POINTER(KernelStat), C.c_int32]
        _LIB = L
    return _LIB


def _check(rc, ctx=None):
    if rc != 0:
        L = lib()
        msg = L.psd_last_error(ctx).decode(errors="replace")
        raise PsdError(rc, f"{L.psd_strerror(rc).decode()}: {msg}")


def _ptr(a):
    """Address of a numpy array (host) or of anything with data_ptr() (a device tensor)."""
    if a is None:
        return None
    if isinstance(a, np.ndarray):
        return a.ctypes.data
    return a.data_ptr()


class DeviceBuffer:
    """A hipMalloc'd buffer owned by Python (psd_dev_alloc / psd_dev_free); has data_ptr() like a tensor."""

    def __init__(self, nbytes: int):
        self.nbytes = int(nbytes)
        h = C.c_void_p(None)
        _check(lib().psd_dev_alloc(max(self.nbytes, 16), C.byref(h)))
        self._p = h.value

    @classmethod
    def from_numpy(cls, a: np.ndarray) -> "DeviceBuffer":
        a = np.ascontiguousarray(a)
        b = cls(a.nbytes)
        if a.nbytes:
            _check(lib().psd_dev_copy(b._p, a.ctypes.data, a.nbytes, 0))
        return b

    def data_ptr(self) -> int:
        return self._p

    def to_numpy(self, dtype, shape) -> np.ndarray:
        out = np.empty(shape, dtype=dtype)
        assert out.nbytes <= self.nbytes
        if out.nbytes:
            _check(lib().psd_dev_copy(out.ctypes.data, self._p, out.nbytes, 1))
        return out

    def free(self):
        if self._p:
            lib().psd_dev_free(self._p)
            self._p = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def dev_sync():
    _check(lib().psd_dev_sync())


def accept(logits_p, logits_q, tokens, T, temperature=1.0, seed=0, position0=0, stage=1, take_bonus=True):
    """psd_accept on host numpy arrays.  Returns (n_accepted, next_token, div[k])."""
    lp = np.ascontiguousarray(logits_p, dtype=np.float32)
    lq = np.ascontiguousarray(logits_q, dtype=np.float32)
    tk = np.ascontiguousarray(tokens, dtype=np.int32)
    k = tk.size
    V = lp.shape[-1]
    n = C.c_int32(0)
    t = C.c_int32(0)
    div = np.zeros(max(k, 1), dtype=np.float32)
    _check(lib().psd_accept(lp.ctypes.data, lq.ctypes.data if k else None, tk.ctypes.data if k else None, k, V, T,
                            temperature, seed, position0, stage, int(take_bonus), 0, C.byref(n), C.byref(t),
                            div.ctypes.data))
    return n.value, t.value, div[:k]


def accept_assisted(logits_p, tokens, temperature=1.0, seed=0, position0=0, stage=1, take_bonus=True):
    """psd_accept_assisted on host numpy arrays.  Returns (n_accepted, next_token)."""
    lp = np.ascontiguousarray(logits_p, dtype=np.float32)
    tk = np.ascontiguousarray(tokens, dtype=np.int32)
    k, V = tk.size, lp.shape[-1]
    n = C.c_int32(0)
    t = C.c_int32(0)
    _check(lib().psd_accept_assisted(lp.ctypes.data, tk.ctypes.data if k else None, k, V, temperature, seed, position0,
                                     stage, int(take_bonus), 0, C.byref(n), C.byref(t)))
    return n.value, t.value


def row_stats(logits, temperature=1.0):
    """psd_row_stats on a host array [n_rows, vocab].  Returns (entropy[n_rows], max_prob[n_rows])."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    lg = lg.reshape(1, -1) if lg.ndim == 1 else lg
    n, V = lg.shape
    h = np.empty(n, dtype=np.float32)
    m = np.empty(n, dtype=np.float32)
    _check(lib().psd_row_stats(lg.ctypes.data, n, V, temperature, 0, h.ctypes.data, m.ctypes.data))
    return h, m


def set_accept_path(path):
    _check(lib().psd_set_accept_path(path))


def get_accept_path():
    return lib().psd_get_accept_path()


def get_accept_expiries():
    f = lib().psd_get_accept_expiries
    f.restype = C.c_int64
    return int(f())


def accept_workspace_bytes(n_trials, k, vocab):
    return lib().psd_accept_workspace_bytes(n_trials, k, vocab)


def accept_batch(logits_p, logits_q, tokens, n_trials, k, vocab, T, temperature, seed, position0, stage, take_bonus,
                 n_accepted, next_token, div_out, workspace, workspace_bytes, stream=None):
    """psd_accept_batch on device buffers (objects with data_ptr(), e.g. torch tensors); only enqueues."""
    _check(lib().psd_accept_batch(_ptr(logits_p), _ptr(logits_q), _ptr(tokens), n_trials, k, vocab, T, temperature,
                                  seed, position0, stage, int(take_bonus), _ptr(n_accepted), _ptr(next_token),
                                  _ptr(div_out), _ptr(workspace), workspace_bytes, stream))


def accept_noalloc_capacity():
    return lib().psd_accept_noalloc_capacity()


def accept_noalloc_init():
    _check(lib().psd_accept_noalloc_init())


def accept_batch_noalloc(logits_p, logits_q, tokens, n_trials, k, vocab, T, temperature, seed, position0, stage,
                         take_bonus, n_accepted, next_token, div_out, stream=None):
    """psd_accept_batch_noalloc on device buffers: as accept_batch, scratch held by the library; only enqueues."""
    _check(lib().psd_accept_batch_noalloc(_ptr(logits_p), _ptr(logits_q), _ptr(tokens), n_trials, k, vocab, T,
                                          temperature, seed, position0, stage, int(take_bonus), _ptr(n_accepted),
                                          _ptr(next_token), _ptr(div_out), stream))


def sample_device(logits, n_rows, vocab, temperature, seed, position0, tokens_out):
    """psd_sample on device buffers: logits [n_rows, vocab] floats, tokens_out [n_rows] int32 (objects with data_ptr())."""
    _check(lib().psd_sample(_ptr(logits), n_rows, vocab, temperature, seed, position0, 1, _ptr(tokens_out)))


def philox_block(seed, c0, n, c1, c2, c3):
    """psd_philox_block into host arrays: (raw words [n, 4] uint32, uniforms [n, 4] float32)."""
    out = np.empty((n, 4), dtype=np.uint32)
    u = np.empty((n, 4), dtype=np.float32)
    _check(lib().psd_philox_block(seed, c0, n, c1, c2, c3, 0, out.ctypes.data, u.ctypes.data))
    return out, u


def sample(logits, temperature=1.0, seed=0, position0=0):
    """psd_sample on a host array [n_rows, vocab]; returns token ids."""
    lg = np.ascontiguousarray(logits, dtype=np.float32)
    lg = lg.reshape(-1, lg.shape[-1])
    out = np.empty(lg.shape[0], dtype=np.int32)
    _check(lib().psd_sample(lg.ctypes.data, lg.shape[0], lg.shape[1], temperature, seed, position0, 0,
                            out.ctypes.data))
    return out


@dataclass
class ModelDesc:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int
    rope_theta: float
    dtype: int
    weights: np.ndarray  # host blob, fp32 values or raw bf16 bits (uint16)
    rms_eps: float = 1e-5

    def c(self):
        w = self.weights
        assert w.flags["C_CONTIGUOUS"]
        return _ModelDesc(self.n_layers, self.d_model, self.n_heads, self.n_kv_heads, self.d_ffn, self.vocab,
                          self.rope_theta, self.rms_eps, self.dtype, 0, w.ctypes.data, w.nbytes)


class Context:
    """psd_create / psd_generate / psd_forward / psd_destroy."""

    def __init__(self, draft: ModelDesc, qualifier: ModelDesc, target: ModelDesc, T_q, T_t, k1, k2, max_seq,
                 temperature=1.0, device=0, flags=0, pool_bytes=0):
        self._h = C.c_void_p(None)
        self._keep = (draft.weights, qualifier.weights, target.weights)
        self._trace_cb = None
        self.vocab = target.vocab
        prm = _Params(T_q, T_t, temperature, k1, k2, max_seq, device, flags, pool_bytes)
        d, q, t = draft.c(), qualifier.c(), target.c()
        _check(lib().psd_create(C.byref(d), C.byref(q), C.byref(t), C.byref(prm), C.byref(self._h)))
        self._keep = None  # the library copied the weights

    def close(self):
        if self._h:
            lib().psd_destroy(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_decoding(self, T_q, T_t, k1, k2, temperature=1.0):
        _check(lib().psd_set_decoding(self._h, T_q, T_t, k1, k2, temperature), self._h)

    def generate(self, prompt, n_new, seed):
        pr = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(n_new, dtype=np.int32)
        st = Stats()
        _check(lib().psd_generate(self._h, pr.ctypes.data, pr.size, n_new, seed, out.ctypes.data, C.byref(st)), self._h)
        return out, st.as_dict()

    def generate_sd(self, proposer, k, tau, prompt, n_new, seed):
        """Two-model speculative decoding: model `proposer` (0 draft, 1 qualifier) -> target, threshold tau."""
        pr = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(n_new, dtype=np.int32)
        st = Stats()
        _check(lib().psd_generate_sd(self._h, proposer, k, tau, pr.ctypes.data, pr.size, n_new, seed, out.ctypes.data,
                                     C.byref(st)), self._h)
        return out, st.as_dict()

    def set_row_stats(self, on: bool):
        _check(lib().psd_set_row_stats(self._h, int(on)), self._h)

    def row_stats(self):
        """{model: (rows, mean entropy, mean largest probability)} of the last generation call."""
        out = np.zeros(9, dtype=np.float64)
        _check(lib().psd_get_row_stats(self._h, out.ctypes.data), self._h)
        return {name: (int(out[3 * i]), float(out[3 * i + 1]), float(out[3 * i + 2]))
                for i, name in enumerate(("draft", "qualifier", "target"))}

    def set_adaptive(self, cfg):
        """cfg: an Adapt (ranges of the controller) or None to switch it off."""
        _check(lib().psd_set_adaptive(self._h, C.byref(cfg) if cfg is not None else None), self._h)

    def adaptive_log(self):
        """(k1, k2, position of tau_Q, position of tau_T) per outer iteration of the last generate call, [n, 4]."""
        n = lib().psd_get_adaptive_log(self._h, None, 0)
        if n < 0:
            _check(n, self._h)
        out = np.zeros((max(n, 1), 4), dtype=np.int32)
        lib().psd_get_adaptive_log(self._h, out.ctypes.data, n)
        return out[:n]

    def set_greedy(self, on: bool):
        _check(lib().psd_set_greedy(self._h, int(on)), self._h)

    def set_assisted(self, on: bool):
        _check(lib().psd_set_assisted(self._h, int(on)), self._h)

    def generate_plain(self, which, prompt, n_new, seed):
        pr = np.ascontiguousarray(prompt, dtype=np.int32)
        out = np.empty(n_new, dtype=np.int32)
        st = Stats()
        _check(lib().psd_generate_plain(self._h, which, pr.ctypes.data, pr.size, n_new, seed, out.ctypes.data,
                                        C.byref(st)), self._h)
        return out, st.as_dict()

    def forward(self, which, tokens, pos0, want_logits=True):
        tk = np.ascontiguousarray(tokens, dtype=np.int32)
        lg = np.empty((tk.size, self.vocab), dtype=np.float32) if want_logits else None
        _check(lib().psd_forward(self._h, which, tk.ctypes.data, tk.size, pos0, lg.ctypes.data if want_logits else None),
               self._h)
        return lg

    def set_trace(self, fn):
        """fn(kind, position0, k, take_bonus, logits_p, logits_q, tokens, n_accepted, next_token, div) with numpy
        copies; None switches tracing off."""
        if fn is None:
            self._trace_cb = TRACE_FN(0)
            _check(lib().psd_set_trace(self._h, self._trace_cb, None), self._h)
            return
        V = self.vocab

        def cb(user, kind, position0, k, take_bonus, lp, lq, tk, n_acc, nxt, div):
            if kind == 7:   # controller state at the start of an outer iteration: div = (tau_Q, tau_T)
                fn(kind, position0, k, take_bonus, None, None, None, n_acc, nxt, np.ctypeslib.as_array(div, shape=(2,)).copy())
                return
            rows_p = 1 if kind in (0, 6) else k + 1
            a = np.ctypeslib.as_array(lp, shape=(rows_p, V)).copy()
            b = np.ctypeslib.as_array(lq, shape=(k, V)).copy() if k > 0 and lq else np.zeros((0, V), np.float32)
            t = np.ctypeslib.as_array(tk, shape=(k,)).copy() if k > 0 and tk else np.zeros(0, np.int32)
            d = np.ctypeslib.as_array(div, shape=(k,)).copy() if k > 0 and div else np.zeros(0, np.float32)
            fn(kind, position0, k, take_bonus, a, b, t, n_acc, nxt, d)

        self._trace_cb = TRACE_FN(cb)
        _check(lib().psd_set_trace(self._h, self._trace_cb, None), self._h)

    def profile(self, on: bool):
        _check(lib().psd_profile(self._h, int(on)), self._h)

    def kernel_stats(self):
        arr = (KernelStat * 128)()
        n = lib().psd_kernel_stats(self._h, arr, 128)
        if n < 0:
            _check(n, self._h)
        return [dict(name=arr[i].name.decode(), launches=arr[i].launches, ms_total=arr[i].ms_total,
                     bytes_total=arr[i].bytes_total) for i in range(n)]
