"""Seeded synthetic inputs (model weights, logits, prompts) for tests and benchmarks.

Thin ctypes wrapper over ``synth.c``.  It only manufactures inputs; none of the
decoding method's arithmetic lives here, so both the CPU oracle's tests and the
HIP library's callers may use it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SO = os.path.join(_HERE, "libsynth.so")


def build(force: bool = False) -> str:
    src = os.path.join(_HERE, "synth.c")
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _SO, src, "-lm"])
    return _SO


class _Shape(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_layers", "d_model", "n_heads", "n_kv_heads", "d_ffn", "vocab")]


@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_heads: int
    n_kv_heads: int
    d_ffn: int
    vocab: int

    @property
    def head_dim(self) -> int:
        return self.d_model // self.n_heads

    def c(self) -> _Shape:
        return _Shape(self.n_layers, self.d_model, self.n_heads, self.n_kv_heads, self.d_ffn, self.vocab)

    def n_elems(self) -> int:
        return int(_lib().synth_model_elems(ctypes.byref(self.c())))


_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        L = ctypes.CDLL(build())
        L.synth_model_elems.restype = ctypes.c_size_t
        L.synth_model_elems.argtypes = [ctypes.POINTER(_Shape)]
        L.synth_normal_f32.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_double,
                                       ctypes.c_double, ctypes.c_void_p]
        L.synth_correlated_f32.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_double,
                                           ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p]
        L.synth_tokens.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_size_t, ctypes.c_int32,
                                   ctypes.c_void_p]
        L.synth_target_weights.argtypes = [ctypes.POINTER(_Shape), ctypes.c_uint64, ctypes.c_double,
                                           ctypes.c_int, ctypes.c_void_p]
        L.synth_derived_weights.argtypes = [ctypes.POINTER(_Shape), ctypes.POINTER(_Shape), ctypes.c_uint64,
                                            ctypes.c_double, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_double,
                                            ctypes.c_uint64, ctypes.c_int, ctypes.c_void_p]
        _LIB = L
    return _LIB


def normal(seed: int, stream: int, n: int, mean: float = 0.0, sigma: float = 1.0) -> np.ndarray:
    out = np.empty(n, dtype=np.float32)
    _lib().synth_normal_f32(seed, stream, n, mean, sigma, out.ctypes.data)
    return out


def correlated(seed: int, stream: int, base: np.ndarray, rho: float, sigma: float) -> np.ndarray:
    base = np.ascontiguousarray(base, dtype=np.float32)
    out = np.empty_like(base)
    _lib().synth_correlated_f32(seed, stream, base.size, rho, sigma, base.ctypes.data, out.ctypes.data)
    return out


_DEV_LIB = None


def accept_logits_device(seed: int, trial0: int, n_trials: int, k: int, vocab: int, rho: float, t=None, q=None, d=None,
                         qk=None, dk=None, sigma: float = 3.0):
    """accept_logits for trials trial0 .. trial0 + n_trials - 1, written on the GPU into device buffers (objects with
    data_ptr()): t, q, d [n_trials, k + 1, vocab] floats, qk, dk [n_trials, k, vocab] = the first k rows of the qualifier and
    draft stacks, packed; None skips an output.  Same recipe as accept_logits; only enqueues work on the default
    stream.  Needs synth/libsynth_dev.so (built by paper_2510_12966_amd.build)."""
    global _DEV_LIB
    if _DEV_LIB is None:
        path = os.path.join(_HERE, "libsynth_dev.so")
        if not os.path.exists(path):
            raise RuntimeError(f"{path} is missing: build it with `python -m paper_2510_12966_amd.build`")
        L = ctypes.CDLL(path)
        L.synth_dev_accept_logits.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                              ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
                                              ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        _DEV_LIB = L
    ptr = lambda b: None if b is None else b.data_ptr()
    rc = _DEV_LIB.synth_dev_accept_logits(seed, trial0, n_trials, k, vocab, rho, sigma, ptr(t), ptr(q), ptr(d), ptr(qk), ptr(dk), None)
    if rc != 0:
        raise RuntimeError(f"synth_dev_accept_logits failed: {rc}")


def tokens(seed: int, stream: int, n: int, vocab: int) -> np.ndarray:
    out = np.empty(n, dtype=np.int32)
    _lib().synth_tokens(seed, stream, n, vocab, out.ctypes.data)
    return out


DTYPE_F32, DTYPE_BF16 = 0, 1


def _blob(shape: ModelShape, dtype: int) -> np.ndarray:
    return np.empty(shape.n_elems(), dtype=np.float32 if dtype == DTYPE_F32 else np.uint16)


def target_weights(shape: ModelShape, seed: int, dtype: int, sigma: float = 0.02) -> np.ndarray:
    out = _blob(shape, dtype)
    _lib().synth_target_weights(ctypes.byref(shape.c()), seed, sigma, dtype, out.ctypes.data)
    return out


def derived_weights(shape: ModelShape, target: ModelShape, seed: int, dtype: int, tag: int, sigma: float = 0.02,
                    noise_sigma: float = 0.01) -> np.ndarray:
    """Draft (tag 1) / qualifier (tag 2) weights derived from the target of the same ``seed``."""
    out = _blob(shape, dtype)
    _lib().synth_derived_weights(ctypes.byref(shape.c()), ctypes.byref(target.c()), seed, sigma,
                                 seed + 0x1000, seed + 0x2000, noise_sigma, tag, dtype, out.ctypes.data)
    return out


def bf16_to_f32(a: np.ndarray) -> np.ndarray:
    return (a.astype(np.uint32) << 16).view(np.float32)


@dataclass(frozen=True)
class StackConfig:
    name: str
    draft: ModelShape
    qualifier: ModelShape
    target: ModelShape
    dtype: int
    rope_theta: float
    n_prompt: int
    n_new: int
    k1: int
    k2: int
    T_q: float
    T_t: float
    temperature: float = 1.0
    weight_seed: int = 0
    prompt_seed: int = 1
    sample_seed: int = 1


def _stack(name, V, D, Q, T, dtype, theta, n_prompt, n_new, k1, k2, T_q, T_t):
    mk = lambda t: ModelShape(t[0], t[1], t[2], t[3], t[4], V)
    return StackConfig(name, mk(D), mk(Q), mk(T), dtype, theta, n_prompt, n_new, k1, k2, T_q, T_t)


CONFIGS = {
    # tiny fp32 stack: CPU-in-seconds plumbing
    "tiny": _stack("tiny", 512, (2, 64, 4, 2, 256), (4, 128, 4, 2, 512), (6, 256, 8, 4, 1024),
                   DTYPE_F32, 10000.0, 16, 64, 4, 8, 0.3, 0.2),
    # small bf16 stack
    "small": _stack("small", 32000, (4, 512, 8, 4, 1408), (8, 1024, 16, 4, 2816), (12, 2048, 16, 8, 5632),
                    DTYPE_BF16, 10000.0, 128, 256, 4, 8, 0.4, 0.3),
    # 1B / 3B / 8B shapes, bf16
    "paper": _stack("paper", 128256, (16, 2048, 32, 8, 8192), (28, 3072, 24, 8, 8192),
                    (32, 4096, 32, 8, 14336), DTYPE_BF16, 500000.0, 512, 512, 5, 10, 0.5, 0.3),
    # same models, long context
    "long": _stack("long", 128256, (16, 2048, 32, 8, 8192), (28, 3072, 24, 8, 8192),
                   (32, 4096, 32, 8, 14336), DTYPE_BF16, 500000.0, 4096, 1024, 5, 10, 0.5, 0.3),
}


def build_stack(cfg: StackConfig):
    """Returns (draft, qualifier, target) weight blobs and the prompt for a stack config."""
    t = target_weights(cfg.target, cfg.weight_seed, cfg.dtype)
    d = derived_weights(cfg.draft, cfg.target, cfg.weight_seed, cfg.dtype, tag=1)
    q = derived_weights(cfg.qualifier, cfg.target, cfg.weight_seed, cfg.dtype, tag=2)
    prompt = tokens(cfg.prompt_seed, 0, cfg.n_prompt, cfg.target.vocab)
    return d, q, t, prompt


def accept_logits(seed: int, trial: int, k: int, vocab: int, rho: float, sigma: float = 3.0):
    """Correlated (target, qualifier, draft) logit stacks of the acceptance microbenchmark, [k+1, vocab] each."""
    n = (k + 1) * vocab
    t = normal(seed, trial * 4 + 0, n, 0.0, sigma)
    q = correlated(seed, trial * 4 + 1, t, rho, sigma)
    d = correlated(seed, trial * 4 + 2, q, rho, sigma)
    return t.reshape(k + 1, vocab), q.reshape(k + 1, vocab), d.reshape(k + 1, vocab)
