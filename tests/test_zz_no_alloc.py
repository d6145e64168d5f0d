"""psd_accept_batch_noalloc (the ACCEPT entry point that allocates nothing) against psd_accept_batch, through the C ABI:
same inputs, same kernels, so every output must agree bit for bit; two calls in a row on the library's scratch array,
the second one smaller, so that whatever the first call left behind is shown not to leak into the second."""
import numpy as np
import pytest

import paper_2510_12966_amd as psd

pytestmark = pytest.mark.gpu


def _inputs(seed, B, k, V):
    rng = np.random.default_rng(seed)
    P = rng.normal(0, 3, (B, k + 1, V)).astype(np.float32)
    Q = (0.9 * P[:, :k] + 0.44 * rng.normal(0, 3, (B, k, V))).astype(np.float32)
    X = rng.integers(0, V, (B, max(k, 1))).astype(np.int32)[:, :k]
    return P, Q, np.ascontiguousarray(X)


def _run(P, Q, X, T, temp, seed, pos0, stage, bonus, noalloc):
    B, k, V = P.shape[0], Q.shape[1], P.shape[2]
    dp, dq, dx = (psd.DeviceBuffer.from_numpy(a) for a in (P, Q, X))
    # outputs start from a pattern no result can have, so a slot that is never written shows
    na = psd.DeviceBuffer.from_numpy(np.full(B, -77, np.int32))
    nt = psd.DeviceBuffer.from_numpy(np.full(B, -77, np.int32))
    dv = psd.DeviceBuffer.from_numpy(np.full(B * max(k, 1), -77.0, np.float32))
    if noalloc:
        psd.accept_batch_noalloc(dp, dq, dx, B, k, V, T, temp, seed, pos0, stage, bonus, na, nt, dv, None)
    else:
        wsb = psd.accept_workspace_bytes(B, k, V)
        ws = psd.DeviceBuffer(wsb)
        psd.accept_batch(dp, dq, dx, B, k, V, T, temp, seed, pos0, stage, bonus, na, nt, dv, ws, wsb, None)
    psd.dev_sync()
    return na.to_numpy(np.int32, B), nt.to_numpy(np.int32, B), dv.to_numpy(np.float32, (B, max(k, 1)))[:, :k]


def test_noalloc_accept_equals_workspace_accept_on_two_calls_in_a_row():
    psd.accept_noalloc_init()
    cap = psd.accept_noalloc_capacity()
    assert cap == 8 << 20
    # first call: several trials at the full vocabulary; second call: fewer trials, a shorter window and a ragged
    # vocabulary, so its slots overlay different parts of what the first call wrote
    calls = [
        dict(seed=1, B=6, k=8, V=128256, T=0.2, temp=1.0, rs=11, pos0=40, stage=2, bonus=True),
        dict(seed=2, B=3, k=5, V=4099, T=0.05, temp=0.8, rs=5, pos0=7, stage=1, bonus=True),
        dict(seed=3, B=2, k=0, V=300, T=0.0, temp=1.0, rs=9, pos0=3, stage=1, bonus=True),   # bonus draw only
        dict(seed=4, B=4, k=31, V=2049, T=0.0, temp=1.0, rs=2, pos0=90, stage=2, bonus=False),
    ]
    inputs = [_inputs(c["seed"], c["B"], c["k"], c["V"]) for c in calls]
    want = [_run(*inp, c["T"], c["temp"], c["rs"], c["pos0"], c["stage"], c["bonus"], False) for c, inp in zip(calls, inputs)]
    got = [_run(*inp, c["T"], c["temp"], c["rs"], c["pos0"], c["stage"], c["bonus"], True) for c, inp in zip(calls, inputs)]
    for c, w, g in zip(calls, want, got):
        assert psd.accept_workspace_bytes(c["B"], c["k"], c["V"]) <= cap
        assert np.array_equal(w[0], g[0]), ("n_accepted", c, w[0], g[0])
        assert np.array_equal(w[1], g[1]), ("next_token", c, w[1], g[1])
        assert np.array_equal(w[2].view(np.uint32), g[2].view(np.uint32)), ("divergences", c)
        assert (g[0] >= 0).all() and (g[0] <= c["k"]).all()
        assert ((g[1] >= 0) == ((g[0] < c["k"]) | c["bonus"])).all()
    # the first two settings really decide something: some trials reject, not all at position 0
    assert len(set(got[0][0].tolist())) > 1 or 0 < got[0][0][0] < 8


def test_noalloc_accept_rejects_requests_beyond_its_scratch():
    cap = psd.accept_noalloc_capacity()
    B, k, V = 128, 31, 128256
    assert psd.accept_workspace_bytes(B, k, V) > cap
    one = psd.DeviceBuffer(64)
    with pytest.raises(psd.PsdError) as e:
        # sizes are checked before any pointer is touched, so small stand-in buffers are enough
        psd.accept_batch_noalloc(one, one, one, B, k, V, 0.1, 1.0, 0, 0, 1, True, one, one, None, None)
    assert e.value.code == -3 and "scratch" in str(e.value)
