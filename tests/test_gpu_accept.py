"""GPU parity of the ACCEPT stage and of fresh sampling against the CPU oracle, through the C ABI."""
import math

import numpy as np
import pytest

import oracle
import paper_2510_12966_amd as psd
from paper_2510_12966_amd import synth

pytestmark = pytest.mark.gpu

DIV_TOL = 1e-5       # fp32 kernel against the fp64 oracle on the same fp32 logits
TIE_DIV = 1e-6       # |div - T| below this: the threshold decision may differ
TIE_COIN = 1e-6      # relative distance of the coin from p/q
TIE_RACE = 1e-5      # relative gap of the two best race keys


def _stage_inputs(seed, trial, k, V, rho, stage):
    t, q, d = synth.accept_logits(seed, trial, k, V, rho)
    lp, lq = (q, d[:k]) if stage == 1 else (t, q[:k])
    # proposals: fresh samples from the proposer rows (the oracle draws them: they are inputs here)
    x = np.array([oracle.sample_row(lq[i], 1.0, seed + trial, 1000 + i)[0] for i in range(k)], dtype=np.int32)
    return lp, lq, x


def _compare(lp, lq, x, T, temp, seed, pos0, stage, bonus):
    n, tok, div = psd.accept(lp, lq, x, T, temp, seed, pos0, stage, bonus)
    res, odiv = oracle.accept(lp, lq, x, T, temp, seed, pos0, stage, bonus)
    assert np.abs(div - odiv).max(initial=0.0) <= DIV_TOL
    near = res.margin_div < TIE_DIV or res.margin_coin < TIE_COIN
    if n != res.n_accepted:
        assert near, (n, res.n_accepted, res.margin_div, res.margin_coin)
        return "tie"
    if tok != res.next_token:
        assert res.margin_race < TIE_RACE, (tok, res.next_token, res.margin_race)
        return "tie"
    return "exact"


@pytest.mark.parametrize("k", [4, 8])
@pytest.mark.parametrize("rho", [0.5, 0.8, 0.95])
def test_accept_full_vocab_microbench_inputs(k, rho):
    V = 128256
    ties = 0
    for trial, T in enumerate([0.0, 0.05, 0.2, 0.4, math.log(2)]):
        for stage in (1, 2):
            lp, lq, x = _stage_inputs(7, trial, k, V, rho, stage)
            ties += _compare(lp, lq, x, T, 1.0, 7 + trial, 300 + trial, stage, True) == "tie"
    assert ties <= 1


@pytest.mark.parametrize("V", [2, 3, 97, 512, 4096, 4099, 8193, 32000])
def test_accept_ragged_vocab_and_edge_k(V):
    rng = np.random.default_rng(V)
    for k in (0, 1, 5, 31):
        lp = rng.normal(0, 2.5, (k + 1, V)).astype(np.float32)
        lq = (0.8 * lp[:k] + 0.6 * rng.normal(0, 2.5, (k, V))).astype(np.float32)
        x = rng.integers(0, V, k).astype(np.int32)
        for T in (0.0, 0.1, 1.0):
            for temp in (1.0, 0.7):
                for bonus in (True, False):
                    _compare(lp, lq, x, T, temp, 11, 40, 1 + (k % 2), bonus)


def test_accept_identical_rows_and_extreme_logits():
    rng = np.random.default_rng(1)
    lp = rng.normal(0, 3, (4, 5000)).astype(np.float32)
    n, tok, div = psd.accept(lp, lp[:3], [1, 2, 3], 0.0, 1.0, 5, 0, 2, True)
    assert n == 3 and np.abs(div).max() <= 1e-6
    assert tok == oracle.accept(lp, lp[:3], [1, 2, 3], 0.0, 1.0, 5, 0, 2, True)[0].next_token
    # one-hot-like rows: same argmax -> divergence ~0, different argmax -> ~ln 2
    a = np.full((2, 300), -60.0, np.float32); a[:, 7] = 40.0
    b = np.full((1, 300), -60.0, np.float32); b[0, 9] = 40.0
    n, tok, div = psd.accept(a, b, [9], 0.5, 1.0, 1, 0, 1, True)
    assert abs(div[0] - math.log(2)) < 1e-5 and n == 0 and tok == 7
    n, tok, div = psd.accept(a, a[:1], [7], 0.0, 1.0, 1, 0, 1, True)
    assert div[0] <= 1e-6 and n == 1 and tok == 7


def test_accept_out_of_range_token_is_rejected_not_faulted():
    rng = np.random.default_rng(2)
    lp = rng.normal(0, 1, (3, 100)).astype(np.float32)
    lq = rng.normal(0, 1, (2, 100)).astype(np.float32)
    n, tok, _ = psd.accept(lp, lq, [100000, 3], 0.0, 1.0, 1, 0, 1, True)
    assert n == 0 and 0 <= tok < 100


def test_accept_argument_errors():
    lp = np.zeros((2, 10), np.float32)
    with pytest.raises(psd.PsdError):
        psd.accept(lp, lp[:1], [1], -0.1)
    with pytest.raises(psd.PsdError):
        psd.accept(lp, lp[:1], [1], 0.1, temperature=0.0)
    with pytest.raises(psd.PsdError):
        psd.accept(lp, lp[:1], [1], 0.1, stage=3)


@pytest.mark.parametrize("V", [5, 512, 4099, 128256])
def test_sample_matches_oracle(V):
    rows = 6
    lg = synth.normal(3, V, rows * V, 0.0, 3.0).reshape(rows, V)
    for temp in (1.0, 0.7):
        got = psd.sample(lg, temp, seed=21, position0=90)
        for r in range(rows):
            want, gap = oracle.sample_row(lg[r], temp, 21, 90 + r)
            assert got[r] == want or gap < TIE_RACE


def test_accept_histogram_matches_oracle_on_batched_trials():
    """Accept-length histogram of the batched entry point against the oracle, trial by trial."""
    k, V, B, rho, T = 4, 128256, 24, 0.8, 0.3
    P, Q, X = [], [], []
    for b in range(B):
        lp, lq, x = _stage_inputs(7, b, k, V, rho, 2)
        P.append(lp); Q.append(lq); X.append(x)
    dp = psd.DeviceBuffer.from_numpy(np.stack(P)); dq = psd.DeviceBuffer.from_numpy(np.stack(Q))
    dx = psd.DeviceBuffer.from_numpy(np.stack(X))
    na = psd.DeviceBuffer(4 * B); nt = psd.DeviceBuffer(4 * B); dv = psd.DeviceBuffer(4 * B * k)
    wsb = psd.accept_workspace_bytes(B, k, V)
    ws = psd.DeviceBuffer(wsb)
    psd.accept_batch(dp, dq, dx, B, k, V, T, 1.0, 100, 50, 2, True, na, nt, dv, ws, wsb, None)
    psd.dev_sync()
    na, nt, dv = na.to_numpy(np.int32, B), nt.to_numpy(np.int32, B), dv.to_numpy(np.float32, (B, k))
    hist_g = np.bincount(na, minlength=k + 1)
    hist_o = np.zeros(k + 1, dtype=np.int64)
    ties = 0
    for b in range(B):
        res, odiv = oracle.accept(P[b], Q[b], X[b], T, 1.0, 100 + b, 50, 2, True)
        hist_o[res.n_accepted] += 1
        assert np.abs(dv[b] - odiv).max() <= DIV_TOL
        if na[b] != res.n_accepted or nt[b] != res.next_token:
            assert res.margin_div < TIE_DIV or res.margin_coin < TIE_COIN or res.margin_race < TIE_RACE
            ties += 1
    assert ties <= 1
    if ties == 0:
        assert np.array_equal(hist_g, hist_o)


def _batched(P, Q, X, T, temp, seed, pos0, stage, bonus):
    B, k, V = len(P), Q[0].shape[0], P[0].shape[1]
    dp = psd.DeviceBuffer.from_numpy(np.stack(P)); dq = psd.DeviceBuffer.from_numpy(np.stack(Q))
    dx = psd.DeviceBuffer.from_numpy(np.stack(X))
    na = psd.DeviceBuffer(4 * B); nt = psd.DeviceBuffer(4 * B); dv = psd.DeviceBuffer(4 * B * k)
    wsb = psd.accept_workspace_bytes(B, k, V)
    ws = psd.DeviceBuffer(wsb)
    psd.accept_batch(dp, dq, dx, B, k, V, T, temp, seed, pos0, stage, bonus, na, nt, dv, ws, wsb, None)
    psd.dev_sync()
    return na.to_numpy(np.int32, B), nt.to_numpy(np.int32, B), dv.to_numpy(np.float32, (B, k))


@pytest.mark.parametrize("V,k,B", [(128256, 4, 6), (4099, 7, 40), (300, 32, 5), (2048, 1, 3), (2049, 2, 3)])
def test_one_launch_and_two_launch_sweeps_agree_bit_for_bit(V, k, B):
    rng = np.random.default_rng(V + k)
    P = [rng.normal(0, 3, (k + 1, V)).astype(np.float32) for _ in range(B)]
    Q = [(0.9 * p[:k] + 0.44 * rng.normal(0, 3, (k, V))).astype(np.float32) for p in P]
    X = [rng.integers(0, V, k).astype(np.int32) for _ in range(B)]
    try:
        psd.set_accept_path(1)
        two = _batched(P, Q, X, 0.15, 0.9, 3, 17, 1, True)
        psd.set_accept_path(0)
        one = _batched(P, Q, X, 0.15, 0.9, 3, 17, 1, True)
    finally:
        psd.set_accept_path(0)
    assert np.array_equal(one[0], two[0]) and np.array_equal(one[1], two[1])
    assert np.array_equal(one[2].view(np.uint32), two[2].view(np.uint32))
    assert (one[0] >= 0).all()
    # and both are the oracle's answer
    for b in range(min(B, 4)):
        res, odiv = oracle.accept(P[b], Q[b], X[b], 0.15, 0.9, 3 + b, 17, 1, True)
        assert np.abs(one[2][b] - odiv).max() <= DIV_TOL
        if one[0][b] != res.n_accepted or one[1][b] != res.next_token:
            assert res.margin_div < TIE_DIV or res.margin_coin < TIE_COIN or res.margin_race < TIE_RACE


def test_accept_masked_entries():
    """-inf logits carry probability zero, in one row or in both."""
    rng = np.random.default_rng(9)
    V, k = 5000, 3
    lp = rng.normal(0, 2, (k + 1, V)).astype(np.float32)
    lq = (0.8 * lp[:k] + 0.6 * rng.normal(0, 2, (k, V))).astype(np.float32)
    lp[:, 100:2300] = -np.inf
    lq[:, 1500:3000] = -np.inf
    lp[:, V - 3:] = -np.inf
    lq[:, V - 3:] = -np.inf
    for x in ([50, 3500, 4000], [200, 2500, 4999]):
        for T in (0.0, 0.3, 1.0):
            _compare(lp, lq, np.array(x, np.int32), T, 1.0, 4, 7, 2, True)


def test_expired_wait_falls_back_to_two_launches_and_still_matches_oracle():
    """A zero wait limit makes every unsatisfied wait between workgroups expire at once (all kernels still run to
    completion); the host notices, switches to the two-launch sweep and runs the stage again."""
    V, k = 128256, 6
    lp, lq, x = _stage_inputs(7, 3, k, V, 0.8, 2)
    try:
        psd.set_accept_path(3)
        for T in (0.0, 0.2):
            assert _compare(lp, lq, x, T, 1.0, 9, 40, 2, True) in ("exact", "tie")
        assert psd.get_accept_path() in (0, 1)          # 1 as soon as one wait has expired
        expired = psd.get_accept_path() == 1
        psd.set_accept_path(3)
        # the batched entry point only reports: -1 for every trial of a call in which a wait expired
        P = [lp] * 4; Q = [lq] * 4; X = [x] * 4
        na, nt, dv = _batched(P, Q, X, 0.2, 1.0, 9, 40, 2, True)
        assert (na == -1).all() or (na >= 0).all()
        expired = expired or (na == -1).all()
        assert expired                                    # 26 chunks per row: some workgroup always has to wait
    finally:
        psd.set_accept_path(0)
    assert psd.get_accept_path() == 0
    assert _compare(lp, lq, x, 0.2, 1.0, 9, 40, 2, True) in ("exact", "tie")


def test_accept_statistics_over_many_trials():
    """1024 trials per threshold in one launch sequence (vocabulary of three chunks with a ragged tail, k = 6):
    every trial against the oracle, the accept-length histograms, the mean accepted length per threshold, and
    its monotone growth with the threshold (Section 3.2: a larger threshold only ever accepts more)."""
    k, V, B, rho = 6, 12345, 1024, 0.8
    rng = np.random.default_rng(17)
    P = (3.0 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    Q = (rho * P[:, :k] + math.sqrt(1 - rho * rho) * 3.0 * rng.standard_normal((B, k, V))).astype(np.float32)
    X = np.array([[oracle.sample_row(Q[b, i], 1.0, 900 + b, 1000 + i)[0] for i in range(k)] for b in range(B)],
                 dtype=np.int32)
    means, ties = [], 0
    for T in (0.0, 0.3, 0.45):     # the divergences of these rows lie between 0.15 and 0.4
        na, nt, dv = _batched(list(P), list(Q), list(X), T, 1.0, 100, 50, 2, True)
        hist_g, hist_o = np.bincount(na, minlength=k + 1), np.zeros(k + 1, dtype=np.int64)
        for b in range(B):
            res, odiv = oracle.accept(P[b], Q[b], X[b], T, 1.0, 100 + b, 50, 2, True)
            hist_o[res.n_accepted] += 1
            assert np.abs(dv[b] - odiv).max() <= DIV_TOL
            if na[b] != res.n_accepted or nt[b] != res.next_token:
                assert res.margin_div < TIE_DIV or res.margin_coin < TIE_COIN or res.margin_race < TIE_RACE
                ties += 1
                hist_o[res.n_accepted] -= 1
                hist_o[na[b]] += 1          # a tie moves one trial between neighbouring bins, nothing else
        assert np.array_equal(hist_g, hist_o)
        assert 0 <= nt.min() and nt.max() < V
        means.append(float(na.mean()))
    assert ties <= 3
    assert means[0] < means[1] < means[2] and means[0] > 0.05 and means[2] < k


def test_accept_randomised_shapes_and_row_patterns():
    """40 seeded random (vocabulary, window, temperature, threshold) settings, 6 trials each, rows that are flat,
    peaked, masked with -inf, or equal in both stacks: every trial against the oracle."""
    rng = np.random.default_rng(23)
    ties = total = 0
    for case in range(40):
        V = int(rng.choice([1, 2, 3, 5, 64, 257, 1000, 4099, 5120, 5121, 10240, 20011]))
        k = int(rng.integers(0, 13))
        B = 6
        temp = float(rng.choice([1.0, 0.7, 1.5]))
        T = float(rng.choice([0.0, 0.05, 0.2, 0.5, math.log(2)]))
        scale = float(rng.choice([0.3, 3.0, 12.0]))            # flat ... sharply peaked
        P = (scale * rng.standard_normal((B, k + 1, V))).astype(np.float32)
        rho = float(rng.choice([0.0, 0.8, 1.0]))               # rho 1: both stacks equal, divergence exactly 0
        Q = (rho * P[:, :k] + math.sqrt(1 - rho * rho) * scale * rng.standard_normal((B, k, V))).astype(np.float32)
        if V > 4 and rng.random() < 0.4:                        # the same masked entries in both stacks
            mask = rng.random(V) < 0.3
            mask[int(rng.integers(V))] = False
            P[:, :, mask] = -np.inf
            Q[:, :, mask] = -np.inf
        X = np.zeros((B, k), dtype=np.int32)
        for b in range(B):
            for i in range(k):
                X[b, i] = oracle.sample_row(Q[b, i], temp, 50 + b, 1000 + i)[0]
        bonus = bool(rng.integers(2))
        stage = int(rng.integers(1, 3))
        if k == 0:
            for b in range(B):
                total += 1
                ties += _compare(P[b], Q[b], X[b], T, temp, 100 + b, 7, stage, True) == "tie"
            continue
        na, nt, dv = _batched(list(P), list(Q), list(X), T, temp, 100, 7, stage, bonus)
        for b in range(B):
            total += 1
            res, odiv = oracle.accept(P[b], Q[b], X[b], T, temp, 100 + b, 7, stage, bonus)
            assert np.abs(dv[b] - odiv).max(initial=0.0) <= DIV_TOL, (case, V, k)
            if rho == 1.0:
                assert (dv[b] == 0.0).all() and na[b] == k
            if na[b] != res.n_accepted or nt[b] != res.next_token:
                assert res.margin_div < TIE_DIV or res.margin_coin < TIE_COIN or res.margin_race < TIE_RACE, (case, V, k, b)
                ties += 1
    assert total == 240 and ties <= 4


def test_device_philox_equals_the_oracles_on_a_million_counters():
    """The two independent implementations of Philox4x32-10 (device, CPU oracle) agree word for word, and the device's
    uniforms are the oracle's, on 10^6 consecutive counters per setting: the addressing of every draw purpose."""
    n = 1_000_000
    for seed, c0, c1, c2, c3 in ((7, 0, 512, 0, 0), (0xDEADBEEFCAFEF00D, 0xFFFFFFF0, 4095, 1, 2), (2**63 + 5, 31000, 0, 2, 1)):
        words, u = psd.philox_block(seed, c0, n, c1, c2, c3)
        ref = oracle.philox_block(seed, c0, n, c1, c2, c3)     # c0 wraps modulo 2^32 on both sides
        assert np.array_equal(words, ref)
        assert np.array_equal(u, (((ref >> 9).astype(np.float64) + 0.5) / 8388608.0).astype(np.float32))
        assert u.min() > 0.0 and u.max() < 1.0
    # the oracle's own uniform, as its sampling code asks for it, on a sample of those counters
    words, u = psd.philox_block(7, 0, 1024, 512, 0, 0)
    for v in (0, 1, 2, 3, 5, 4094, 4095):
        assert oracle.uniform(7, v, 512, 0, 0) == float(u[v >> 2, v & 3])


def test_accept_batch_workspace_one_byte_short_is_enomem_and_writes_nothing():
    B, k, V = 3, 4, 4099
    rng = np.random.default_rng(1)
    dp = psd.DeviceBuffer.from_numpy(rng.normal(0, 2, (B, k + 1, V)).astype(np.float32))
    dq = psd.DeviceBuffer.from_numpy(rng.normal(0, 2, (B, k, V)).astype(np.float32))
    dx = psd.DeviceBuffer.from_numpy(rng.integers(0, V, (B, k)).astype(np.int32))
    na = psd.DeviceBuffer.from_numpy(np.full(B, -77, np.int32)); nt = psd.DeviceBuffer.from_numpy(np.full(B, -77, np.int32))
    dv = psd.DeviceBuffer.from_numpy(np.full(B * k, -77.0, np.float32))
    wsb = psd.accept_workspace_bytes(B, k, V)
    ws = psd.DeviceBuffer(wsb)
    with pytest.raises(psd.PsdError) as e:
        psd.accept_batch(dp, dq, dx, B, k, V, 0.1, 1.0, 1, 0, 1, True, na, nt, dv, ws, wsb - 1, None)
    assert e.value.code == -3 and "workspace" in str(e.value) and str(wsb) in str(e.value)   # PSD_ENOMEM, message set
    psd.dev_sync()
    assert (na.to_numpy(np.int32, B) == -77).all() and (nt.to_numpy(np.int32, B) == -77).all()
    assert (dv.to_numpy(np.float32, B * k) == -77.0).all()
    psd.accept_batch(dp, dq, dx, B, k, V, 0.1, 1.0, 1, 0, 1, True, na, nt, dv, ws, wsb, None)   # the exact size is enough
    psd.dev_sync()
    assert (na.to_numpy(np.int32, B) >= 0).all()


def test_device_input_generator_follows_the_host_recipe():
    """The microbenchmark's logits can be manufactured on the GPU (ten thousand trials per setting are terabytes of
    normals): same counter hash, same Box-Muller transform, so the stacks agree with the host generator's to the last
    bits of the double-precision library functions."""
    k, V, B, rho = 3, 1000, 4, 0.8
    bufs = {n: psd.DeviceBuffer(4 * B * rows * V) for n, rows in (("t", k + 1), ("q", k + 1), ("d", k + 1), ("qk", k), ("dk", k))}
    synth.accept_logits_device(7, 20, B, k, V, rho, **bufs)
    psd.dev_sync()
    got = {n: b.to_numpy(np.float32, (B, (k if n in ("qk", "dk") else k + 1), V)) for n, b in bufs.items()}
    same = total = 0
    for b in range(B):
        t, q, d = synth.accept_logits(7, 20 + b, k, V, rho)
        for name, want in (("t", t), ("q", q), ("d", d), ("qk", q[:k]), ("dk", d[:k])):
            assert np.abs(got[name][b] - want).max() <= 2e-6
            same += int((got[name][b] == want).sum()); total += want.size
    assert same >= 0.999 * total
    assert abs(float(got["t"].std()) - 3.0) < 0.1 and abs(float(np.corrcoef(got["t"].ravel(), got["q"].ravel())[0, 1]) - rho) < 0.03
