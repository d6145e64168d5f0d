"""Pins of the oracle's decoder forward: a torch (CPU, fp64) restatement out of library
routines, and the invariants the architecture fixes."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
from paper_2510_12966_amd import synth
from paper_2510_12966_amd.synth import ModelShape


def _split(shape, blob):
    """Views of the blob's tensors, in the documented blob order."""
    d, H, KV, Fd, V = shape.d_model, shape.n_heads, shape.n_kv_heads, shape.d_ffn, shape.vocab
    hd = d // H
    w = torch.from_numpy(blob.astype(np.float64))
    off = 0

    def take(*dims):
        nonlocal off
        n = int(np.prod(dims))
        t = w[off:off + n].reshape(*dims)
        off += n
        return t

    out = {"embed": take(V, d), "layers": []}
    for _ in range(shape.n_layers):
        out["layers"].append(dict(an=take(d), wq=take(H * hd, d), wk=take(KV * hd, d), wv=take(KV * hd, d),
                                  wo=take(d, H * hd), fn=take(d), wg=take(Fd, d), wu=take(Fd, d), wd=take(d, Fd)))
    out["final"] = take(d)
    assert off == w.numel()
    return out


def _rope_complex(x, pos, theta):
    # x: [T, heads, hd]; pair (i, i + hd/2) read as one complex number, rotated by e^{i pos theta^(-2i/hd)}
    T, h, hd = x.shape
    half = hd // 2
    z = torch.complex(x[..., :half], x[..., half:])
    freq = theta ** (-torch.arange(half, dtype=torch.float64) * 2.0 / hd)
    ang = pos.to(torch.float64)[:, None] * freq[None, :]
    z = z * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def torch_forward(shape, blob, tokens, theta, eps=1e-5):
    """Full recompute over `tokens` with library ops (embedding, rms_norm, linear, SDPA with GQA, silu)."""
    W = _split(shape, blob)
    d, H, KV = shape.d_model, shape.n_heads, shape.n_kv_heads
    hd = d // H
    tok = torch.as_tensor(np.asarray(tokens), dtype=torch.long)
    T = tok.numel()
    pos = torch.arange(T)
    x = F.embedding(tok, W["embed"])
    for L in W["layers"]:
        h = F.rms_norm(x, (d,), L["an"], eps)
        q = _rope_complex(F.linear(h, L["wq"]).view(T, H, hd), pos, theta)
        k = _rope_complex(F.linear(h, L["wk"]).view(T, KV, hd), pos, theta)
        v = F.linear(h, L["wv"]).view(T, KV, hd)
        a = F.scaled_dot_product_attention(q.transpose(0, 1)[None], k.transpose(0, 1)[None], v.transpose(0, 1)[None],
                                           is_causal=True, enable_gqa=True)[0]
        x = x + F.linear(a.transpose(0, 1).reshape(T, H * hd), L["wo"])
        h = F.rms_norm(x, (d,), L["fn"], eps)
        x = x + F.linear(F.silu(F.linear(h, L["wg"])) * F.linear(h, L["wu"]), L["wd"])
    return F.linear(F.rms_norm(x, (d,), W["final"], eps), W["embed"]).numpy()


SHAPES = [
    ModelShape(2, 64, 4, 2, 256, 512),     # tiny draft
    ModelShape(3, 96, 6, 6, 160, 97),      # KV == H: plain multi-head attention, odd vocabulary
    ModelShape(2, 128, 8, 2, 192, 130),    # group of 4
]


def _weights(shape, seed, sigma=0.08):
    # larger sigma than the stack's so attention and the MLP are far from their linear regimes
    return synth.target_weights(shape, seed, synth.DTYPE_F32, sigma=sigma)


@pytest.mark.parametrize("shape", SHAPES)
def test_forward_matches_torch_library_restatement(shape):
    blob = _weights(shape, 3)
    toks = synth.tokens(9, 0, 23, shape.vocab)
    m = oracle.Model(shape, blob, synth.DTYPE_F32, 10000.0, 64)
    lg = m.forward(toks, 0)
    ref = torch_forward(shape, blob, toks, 10000.0)
    assert np.abs(ref).max() > 0.1
    np.testing.assert_allclose(lg, ref, rtol=0, atol=1e-10)


def test_bf16_weights_are_widened_exactly():
    shape = SHAPES[0]
    blob16 = synth.target_weights(shape, 3, synth.DTYPE_BF16, sigma=0.08)
    blob32 = synth.bf16_to_f32(blob16)
    toks = synth.tokens(9, 0, 11, shape.vocab)
    a = oracle.Model(shape, blob16, synth.DTYPE_BF16, 10000.0, 32).forward(toks, 0)
    b = oracle.Model(shape, blob32, synth.DTYPE_F32, 10000.0, 32).forward(toks, 0)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("shape", SHAPES[:2])
def test_kv_cached_equals_full_recompute_and_width_invariance(shape):
    blob = _weights(shape, 4)
    toks = synth.tokens(10, 0, 19, shape.vocab)
    full = oracle.Model(shape, blob, synth.DTYPE_F32, 10000.0, 32).forward(toks, 0)
    # one token at a time
    m = oracle.Model(shape, blob, synth.DTYPE_F32, 10000.0, 32)
    step = np.concatenate([m.forward(toks[i:i + 1], i) for i in range(19)])
    np.testing.assert_allclose(step, full, rtol=0, atol=1e-12)
    # ragged chunks, with a rollback in between: rows beyond the cut are recomputed with other tokens first
    m = oracle.Model(shape, blob, synth.DTYPE_F32, 32, 32) if False else oracle.Model(shape, blob, synth.DTYPE_F32, 10000.0, 32)
    a = m.forward(toks[0:7], 0)
    junk = (toks[7:12] + 1) % shape.vocab
    m.forward(junk, 7)                       # speculative rows that get rejected
    b = m.forward(toks[7:12], 7)             # overwrite after rollback to length 7
    c = m.forward(toks[12:19], 12)
    np.testing.assert_allclose(np.concatenate([a, b, c]), full, rtol=0, atol=1e-12)


def test_rope_group_and_relative_position_properties():
    rng = np.random.default_rng(0)
    hd, theta = 16, 10000.0
    a = rng.normal(size=hd); b = rng.normal(size=hd)
    # rotations compose: position p then q equals position p + q
    np.testing.assert_allclose(oracle.rope(oracle.rope(a, 1, hd, 3, theta), 1, hd, 9, theta),
                               oracle.rope(a, 1, hd, 12, theta), atol=1e-12)
    # position 0 is the identity, norms are preserved
    np.testing.assert_allclose(oracle.rope(a, 1, hd, 0, theta), a, atol=0)
    assert abs(np.linalg.norm(oracle.rope(a, 1, hd, 77, theta)) - np.linalg.norm(a)) < 1e-12
    # <R_i a, R_j b> depends on i - j only
    d1 = oracle.rope(a, 1, hd, 5, theta) @ oracle.rope(b, 1, hd, 2, theta)
    d2 = oracle.rope(a, 1, hd, 45, theta) @ oracle.rope(b, 1, hd, 42, theta)
    assert abs(d1 - d2) < 1e-12
    # first pair turns by exactly `pos` radians, the last pair by pos * theta^(-(hd-2)/hd)
    e = np.zeros(hd); e[0] = 1
    r = oracle.rope(e, 1, hd, 2, theta)
    assert abs(r[0] - math.cos(2)) < 1e-15 and abs(r[hd // 2] - math.sin(2)) < 1e-15
    e = np.zeros(hd); e[hd // 2 - 1] = 1
    r = oracle.rope(e, 1, hd, 2, theta)
    ang = 2 * theta ** (-(hd - 2) / hd)
    assert abs(r[hd // 2 - 1] - math.cos(ang)) < 1e-15 and abs(r[hd - 1] - math.sin(ang)) < 1e-15


def test_one_layer_toy_is_hand_computable():
    # d = 2, one head, one token: attention over a single key returns v, so
    # x1 = x0 + Wo Wv n(x0); with Wv = Wo = I, gains 1, zero MLP: x1 = x0 + n(x0); logits = E n(x1).
    shape = ModelShape(1, 2, 1, 1, 2, 3)
    E = np.array([[3.0, 4.0], [1.0, 0.0], [0.0, -2.0]])
    I = np.eye(2)
    blob = np.concatenate([E.ravel(), [1, 1], np.zeros(4), np.zeros(4), I.ravel(), I.ravel(), [1, 1],
                           np.zeros(4), np.zeros(4), np.zeros(4), [1, 1]]).astype(np.float32)
    m = oracle.Model(shape, blob, synth.DTYPE_F32, 10000.0, 4, rms_eps=0.0)
    lg = m.forward([0], 0)[0]
    x0 = np.array([3.0, 4.0])
    n0 = x0 / math.sqrt((x0 ** 2).mean())          # (3, 4) / sqrt(12.5)
    x1 = x0 + n0
    n1 = x1 / math.sqrt((x1 ** 2).mean())          # parallel to (3, 4): n1 = n0
    np.testing.assert_allclose(lg, E @ n1, atol=1e-12)
    np.testing.assert_allclose(lg, [25 / math.sqrt(12.5), 3 / math.sqrt(12.5), -8 / math.sqrt(12.5)], atol=1e-12)


def test_forward_rejects_bad_arguments():
    shape = SHAPES[0]
    m = oracle.Model(shape, _weights(shape, 1), synth.DTYPE_F32, 10000.0, 8)
    with pytest.raises(ValueError):
        m.forward([1, 2, 3], 6)          # would run past max_seq
    with pytest.raises(ValueError):
        m.forward([shape.vocab], 0)      # token out of range
