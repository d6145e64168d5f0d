#!/usr/bin/env python3
"""Benchmark of the three-model speculative loop on one MI355X.

A step is one psd_generate call: prefill of the synthetic prompt by the three models, then the
draft -> qualifier -> target loop until n_new tokens exist.  Prints ONE JSON line: throughput, per-pass times, the
dominant kernel's roofline, the CPU oracle's speed on a sample, comparison runs.  Weights, prompt and every random draw are seeded and synthetic.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0  # MI355X published HBM3E bandwidth

TRAFFIC_PROFILE = os.path.join("profiles", "gemm_gate_up_paper_hbm_counters.md")


def measured_traffic(workload: str, family: str):
    """HBM bytes per launch of a kernel family (FETCH_SIZE + WRITE_SIZE from two rocprofv3 --pmc runs, scaled by a copy
    kernel of known size), read from the machine-readable block of the committed profile summary; (None, None) when
    the summary has no row for it.  Nothing is measured here: rocprofv3 cannot run inside this process."""
    try:
        text = open(os.path.join(ROOT, TRAFFIC_PROFILE)).read()
        block = text.split("```json", 1)[1].split("```", 1)[0]
        rows = json.loads(block)["hbm_bytes_per_launch"]
    except (OSError, IndexError, KeyError, ValueError):
        return None, None
    val = rows.get(f"{workload}: {family}")
    return (float(val), TRAFFIC_PROFILE) if val is not None else (None, None)


def throughput_model(beta_qd, beta_tq, l_d, l_q, v_d, v_q, v_t):
    """Closed-form tokens/s of Section 3.3 from stage accept rates, speculative lengths and per-model speeds
    (tokens/s of one forward each).  Returns (V_FSD(Q,D), V_PSD, V_SD with the qualifier as proposer)."""
    v_fsd_qd = beta_qd * (l_d + 1) / (l_d / v_d + 1.0 / v_q)
    v_psd = beta_tq * (l_q + 1) / (l_q / v_fsd_qd + 1.0 / v_t)
    v_sd = beta_tq * (l_q + 1) / (l_q / v_q + 1.0 / v_t)
    return v_fsd_qd, v_psd, v_sd


LAUNCH_FLOOR_US = 4.3      # a dependent kernel launch, begin to begin of useful streaming (rocprofv3 timestamps of near-empty kernels)
STREAM_GBPS = 6600.0       # what a plain streaming read reaches on this part (non-temporal loads)


def cost_model(kernels, passes, measured_ms):
    """The two-constant model the forward kernels sit on, evaluated on this run's own launch counts and bytes:
    time of a pass = launches x LAUNCH_FLOOR_US + algorithmic bytes / STREAM_GBPS.  kernels: rows of the per-kernel table
    (name, launches, bytes_total); passes / measured_ms: per model name.  Ingestion launches (classes wider than 32
    tokens) are left out; the draft's sampling step counts as two launches per timed unit."""
    import re
    out = {"per_launch_us": LAUNCH_FLOOR_US, "stream_GBps": STREAM_GBPS, "pass": {}}
    for m in ("draft", "qualifier", "target"):
        rows = []
        for r in kernels:
            cls = re.search(r"w<=(\d+)", r["name"])
            if r["name"].split()[1:2] == [m] and (cls is None or int(cls.group(1)) <= 32):
                rows.append(r)
        n = passes.get(m, 0)
        if not rows or n <= 0:
            continue
        launches = sum(r["launches"] * (2 if r["name"].startswith("sample") else 1) for r in rows) / n
        gb = sum(r["bytes_total"] for r in rows) / n / 1e9
        pred = launches * LAUNCH_FLOOR_US * 1e-3 + gb * 1e9 / (STREAM_GBPS * 1e6)
        out["pass"][m] = {"launches": round(launches, 1), "GB": round(gb, 3), "predicted_ms": round(pred, 4),
                          "measured_ms": round(measured_ms[m], 4), "measured_over_predicted": round(measured_ms[m] / pred, 3),
                          "floor_share_of_predicted": round(launches * LAUNCH_FLOOR_US * 1e-3 / pred, 3)}
    return out


def log(*a):
    print(*a, file=sys.stderr, flush=True)


ACCEPT_V, ACCEPT_SEED = 128256, 7
ACCEPT_THRESHOLDS = (0.0, 0.05, 0.1, 0.2, 0.3, 0.4, 0.5, 0.6, 0.6931471805599453)
PAIRINGS = ("T<-Q", "Q<-D")   # (verifier <- proposer): target judging the qualifier's rows, qualifier judging the draft's


def _oracle_own_draws(args):
    """Worker (its own process, CPU only): the oracle's ACCEPT on trials it draws itself from the host generator, every
    threshold; returns {(pairing, T): accept-length histogram}.  Trials are numbered from 10^6 on, apart from the GPU's."""
    k, rho, trials = args
    os.environ["OMP_NUM_THREADS"] = "1"
    import oracle
    from paper_2510_12966_amd import synth

    hist = {(pr, T): np.zeros(k + 1, dtype=np.int64) for pr in PAIRINGS for T in ACCEPT_THRESHOLDS}
    for trial in trials:
        t, q, d = synth.accept_logits(ACCEPT_SEED, 1_000_000 + trial, k, ACCEPT_V, rho)
        for pr, (lp, lq) in zip(PAIRINGS, ((t, q[:k]), (q, d[:k]))):
            x = np.array([oracle.sample_row(lq[i], 1.0, ACCEPT_SEED + trial, 1000 + i)[0] for i in range(k)], dtype=np.int32)
            for T in ACCEPT_THRESHOLDS:
                res, _ = oracle.accept(lp, lq, x, T, 1.0, 100 + trial, 50, 2 if pr == "T<-Q" else 1, True)
                hist[(pr, T)][res.n_accepted] += 1
    return k, rho, hist


def accept_microbench(ks=(4, 8, 16, 32), rhos=(0.5, 0.8, 0.95), trials=10000, B=50, oracle_exact=2, oracle_own=32,
                      calibrate=False) -> int:
    """The stand-alone ACCEPT stage on the microbenchmark's inputs: vocabulary 128256, k + 1 rows, correlated synthetic
    logits generated on the device, `trials` trials per (k, rho, threshold) in launches of B trials, both stage pairings.
    Reports achieved GB/s (every logit counted once), the accept-length histograms, exact parity with the oracle on
    copied-back trials and a chi-square comparison with histograms of the oracle's own draws."""
    import multiprocessing as mp

    import scipy.stats

    # the oracle's own draws run in CPU worker processes, started before this process touches the GPU
    own = None
    if oracle_own > 0:
        pool = mp.get_context("spawn").Pool(min(16, int(os.environ.get("OMP_NUM_THREADS", "8"))))
        chunks = [list(range(i, min(i + 4, oracle_own))) for i in range(0, oracle_own, 4)]
        own = pool.map_async(_oracle_own_draws, [(k, rho, c) for k in ks for rho in rhos for c in chunks])

    import oracle
    import paper_2510_12966_amd as psd
    from paper_2510_12966_amd import synth

    V, seed = ACCEPT_V, ACCEPT_SEED
    if calibrate:   # a kernel of known traffic, for scaling hardware counters read under rocprofv3 --pmc
        a, b = psd.DeviceBuffer(256 << 20), psd.DeviceBuffer(256 << 20)
        psd.lib().psd_dev_copy(b.data_ptr(), a.data_ptr(), 256 << 20, 2)
        psd.dev_sync()
        a.free(); b.free()
    rows, exact_checked, exact_ties = [], 0, 0
    hists = {}
    for k in ks:
        n_full, n_lead = (k + 1) * V, k * V
        dT, dQ = psd.DeviceBuffer(4 * B * n_full), psd.DeviceBuffer(4 * B * n_full)
        dQk, dDk = psd.DeviceBuffer(4 * B * n_lead), psd.DeviceBuffer(4 * B * n_lead)
        dX = {pr: psd.DeviceBuffer(4 * B * k) for pr in PAIRINGS}
        nT = len(ACCEPT_THRESHOLDS)
        na, nt, dv = psd.DeviceBuffer(4 * B * nT), psd.DeviceBuffer(4 * B * nT), psd.DeviceBuffer(4 * B * k * nT)
        wsb = psd.accept_workspace_bytes(B, k, V)
        ws = psd.DeviceBuffer(wsb)
        stage = {"T<-Q": (dT, dQk, 2), "Q<-D": (dQ, dDk, 1)}

        class At:   # a position inside a device buffer
            def __init__(self, buf, byte_offset):
                self.p = buf.data_ptr() + byte_offset

            def data_ptr(self):
                return self.p
        for rho in rhos:
            hist = {(pr, T): np.zeros(k + 1, dtype=np.int64) for pr in PAIRINGS for T in ACCEPT_THRESHOLDS}
            secs = {pr: 0.0 for pr in PAIRINGS}
            calls = 0
            for b0 in range(0, trials, B):
                synth.accept_logits_device(seed, b0, B, k, V, rho, t=dT, q=dQ, qk=dQk, dk=dDk)
                for pr in PAIRINGS:   # proposals ~ the proposer's own rows, drawn on the device
                    psd.sample_device(stage[pr][1], B * k, V, 1.0, seed + b0, 1000, dX[pr])
                keep = None
                if b0 == 0 and oracle_exact > 0:   # a few trials of the first launch go back to the host for the oracle
                    n = oracle_exact
                    keep = {"T": dT.to_numpy(np.float32, (B, k + 1, V))[:n], "Q": dQ.to_numpy(np.float32, (B, k + 1, V))[:n],
                            "Qk": dQk.to_numpy(np.float32, (B, k, V))[:n], "Dk": dDk.to_numpy(np.float32, (B, k, V))[:n],
                            "X": {pr: dX[pr].to_numpy(np.int32, (B, k))[:n] for pr in PAIRINGS}}
                for pr in PAIRINGS:
                    lp, lq, stg = stage[pr]
                    psd.dev_sync()
                    t0 = time.perf_counter()
                    for i, T in enumerate(ACCEPT_THRESHOLDS):   # the launch sequences of all thresholds go out back to back
                        psd.accept_batch(lp, lq, dX[pr], B, k, V, T, 1.0, 100 + b0, 50, stg, True, At(na, 4 * B * i), At(nt, 4 * B * i),
                                         At(dv, 4 * B * k * i), ws, wsb, None)
                    psd.dev_sync()
                    if keep is None:   # the first launch of a setting (also the one that is checked) is not timed
                        secs[pr] += time.perf_counter() - t0
                        calls += pr == PAIRINGS[0]
                    h_na, h_nt = na.to_numpy(np.int32, (nT, B)), nt.to_numpy(np.int32, (nT, B))
                    h_dv = dv.to_numpy(np.float32, (nT, B, k)) if keep is not None else None
                    for i, T in enumerate(ACCEPT_THRESHOLDS):
                        hist[(pr, T)] += np.bincount(h_na[i], minlength=k + 1)
                        if keep is None:
                            continue
                        o = (h_na[i], h_nt[i], h_dv[i])
                        P = keep["T"] if pr == "T<-Q" else keep["Q"]
                        Qr = keep["Qk"] if pr == "T<-Q" else keep["Dk"]
                        for b in range(oracle_exact):
                            res, odiv = oracle.accept(P[b], Qr[b], keep["X"][pr][b], T, 1.0, 100 + b0 + b, 50, stg, True)
                            exact_checked += 1
                            assert np.abs(o[2][b] - odiv).max(initial=0.0) <= 1e-5, ("divergence", pr, k, rho, T, b)
                            if (o[0][b], o[1][b]) != (res.n_accepted, res.next_token):
                                assert res.margin_div < 1e-6 or res.margin_coin < 1e-6 or res.margin_race < 1e-5, (pr, k, rho, T, b)
                                exact_ties += 1
            per_call = {pr: secs[pr] / max(calls, 1) / len(ACCEPT_THRESHOLDS) for pr in PAIRINGS}
            for pr in PAIRINGS:
                gbs = B * (2 * k + 1) * V * 4 / per_call[pr] / 1e9 if per_call[pr] > 0 else 0.0
                for T in ACCEPT_THRESHOLDS:
                    hists[(pr, k, rho, T)] = hist[(pr, T)]
                rows.append({"pairing": pr, "k": k, "rho": rho, "GBps": round(gbs, 1), "us_per_trial": round(per_call[pr] / B * 1e6, 2),
                             "hist": {f"{T:.4f}": hist[(pr, T)].tolist() for T in ACCEPT_THRESHOLDS}})
                log(f"[accept] {pr} k={k:2d} rho={rho:.2f}: {gbs:7.1f} GB/s over {trials} trials x {len(ACCEPT_THRESHOLDS)} thresholds; "
                    f"mean accepted length at T=0 / 0.2 / ln2: " + " / ".join(
                        f"{(hist[(pr, T)] * np.arange(k + 1)).sum() / hist[(pr, T)].sum():.2f}" for T in (0.0, 0.2, ACCEPT_THRESHOLDS[-1])))
        for b_ in (dT, dQ, dQk, dDk, na, nt, dv, ws, *dX.values()):
            b_.free()
    # chi-square of the oracle's own histograms against the GPU's frequencies (cells with an expectation below 5 merged)
    stat = {"settings": 0, "rejected_at_0.001": 0, "min_p": 1.0}
    if own is not None:
        merged = {}
        for k, rho, h in own.get():
            for (pr, T), v in h.items():
                merged[(pr, k, rho, T)] = merged.get((pr, k, rho, T), 0) + v
        pool.close()
        for key, oh in merged.items():
            gh = hists[key].astype(np.float64)
            exp = gh / gh.sum() * oh.sum()
            order = np.argsort(-exp)
            cells_o, cells_e, acc_o, acc_e = [], [], 0.0, 0.0
            for i in order:
                acc_o += oh[i]; acc_e += exp[i]
                if acc_e >= 5:
                    cells_o.append(acc_o); cells_e.append(acc_e); acc_o = acc_e = 0.0
            if cells_e and acc_e > 0:
                cells_o[-1] += acc_o; cells_e[-1] += acc_e
            p = 1.0
            if len(cells_e) > 1:
                chi2 = sum((o - e) ** 2 / e for o, e in zip(cells_o, cells_e))
                p = float(scipy.stats.chi2.sf(chi2, len(cells_e) - 1))
            elif acc_e == 0 and not cells_e:
                p = 1.0
            stat["settings"] += 1
            stat["rejected_at_0.001"] += p < 1e-3
            stat["min_p"] = min(stat["min_p"], p)
        stat["oracle_trials_per_setting"] = oracle_own
        log(f"[accept] oracle's own draws ({oracle_own} trials per setting) against the GPU histograms: {stat}")
    best = max(r["GBps"] for r in rows)
    print(json.dumps({"metric": "stand-alone ACCEPT stage, achieved GB/s (logits read once)", "value": best, "unit": "GB/s",
                      "peak": HBM_PEAK_GBS, "frac": round(best / HBM_PEAK_GBS, 4), "trials_per_setting": trials, "trials_per_launch": B,
                      "single_trial_call_us": accept_single_trial_latency(psd, synth, ks),
                      "thresholds": list(ACCEPT_THRESHOLDS), "exact_parity": {"stages_checked": exact_checked, "near_ties": exact_ties},
                      "oracle_own_draws": stat, "rows": rows}), flush=True)
    return 0


def accept_single_trial_latency(psd, synth, ks=(4, 8, 16, 32), rho=0.8, T=0.2):
    """One trial per launch sequence (the in-loop shape): microseconds per call."""
    V, out = ACCEPT_V, {}
    for k in ks:
        t, q, _ = synth.accept_logits(ACCEPT_SEED, 0, k, V, rho)
        x = psd.sample(q[:k], 1.0, ACCEPT_SEED, 1000).astype(np.int32)
        dp, dq, dx = psd.DeviceBuffer.from_numpy(t), psd.DeviceBuffer.from_numpy(q[:k]), psd.DeviceBuffer.from_numpy(x)
        na, nt, dv = psd.DeviceBuffer(4), psd.DeviceBuffer(4), psd.DeviceBuffer(4 * k)
        wsb = psd.accept_workspace_bytes(1, k, V)
        ws = psd.DeviceBuffer(wsb)
        psd.accept_batch(dp, dq, dx, 1, k, V, T, 1.0, 100, 50, 2, True, na, nt, dv, ws, wsb, None)
        psd.dev_sync()
        t0 = time.perf_counter()
        for _ in range(20):
            psd.accept_batch(dp, dq, dx, 1, k, V, T, 1.0, 100, 50, 2, True, na, nt, dv, ws, wsb, None)
        psd.dev_sync()
        out[k] = round((time.perf_counter() - t0) / 20 * 1e6, 1)
        for b_ in (dp, dq, dx, na, nt, dv, ws):
            b_.free()
    return out


def accept_quick(psd, synth, ks=(4, 32), rho=0.8, T=0.2, B=48, reps=5):
    """Short stand-alone ACCEPT measurement for the benchmark line: B trials per launch sequence of the microbenchmark's
    inputs (vocabulary 128256, target <- qualifier pairing), GB/s counting every logit once, and the accept-length
    histogram against the oracle on the same trials."""
    import oracle

    V, seed, out = 128256, 7, []
    for k in ks:
        P, Q = [], []
        for b in range(B):
            t, q, _ = synth.accept_logits(seed, b, k, V, rho)
            P.append(t); Q.append(q[:k])
        X = np.stack([psd.sample(Q[b], 1.0, seed + b, 1000) for b in range(B)]).astype(np.int32)   # proposals ~ proposer rows
        dp, dq, dx = (psd.DeviceBuffer.from_numpy(np.stack(a)) for a in (P, Q, X))
        na, nt, dv = psd.DeviceBuffer(4 * B), psd.DeviceBuffer(4 * B), psd.DeviceBuffer(4 * B * k)
        wsb = psd.accept_workspace_bytes(B, k, V)
        ws = psd.DeviceBuffer(wsb)
        psd.accept_batch(dp, dq, dx, B, k, V, T, 1.0, 100, 50, 2, True, na, nt, dv, ws, wsb, None)
        psd.dev_sync()
        t0 = time.perf_counter()
        for _ in range(reps):
            psd.accept_batch(dp, dq, dx, B, k, V, T, 1.0, 100, 50, 2, True, na, nt, dv, ws, wsb, None)
        psd.dev_sync()
        dt = (time.perf_counter() - t0) / reps
        hist = np.bincount(na.to_numpy(np.int32, B), minlength=k + 1)
        oh = np.zeros(k + 1, dtype=np.int64)
        for b in range(B):
            res, _ = oracle.accept(P[b], Q[b], X[b], T, 1.0, 100 + b, 50, 2, True)
            oh[res.n_accepted] += 1
        gbs = B * (2 * k + 1) * V * 4 / dt / 1e9
        out.append({"k": k, "rho": rho, "T": T, "trials_per_launch": B, "GBps": round(gbs, 1),
                    "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4), "us_per_trial": round(dt / B * 1e6, 2),
                    "hist_equal": bool(np.array_equal(hist, oh))})
        log(f"[bench] ACCEPT alone, k={k}: {gbs:.0f} GB/s, histogram equal to the oracle's: {out[-1]['hist_equal']}")
        for b_ in (dp, dq, dx, na, nt, dv, ws):
            b_.free()
    return out


SWEEP_K1, SWEEP_K2 = (3, 5, 8), (6, 10, 16)


def sweep(ctx, cfg, prompt, n_new, only_k1=0) -> int:
    """k1 x k2 x T_q x T_t grid (81 points) on one context created with the largest windows of the grid; only_k1
    restricts the run to one draft length (27 points)."""
    print("k1 k2 T_q T_t decode_tok_s accept_q accept_t ms_d ms_q ms_t passes_d passes_q passes_t", flush=True)
    for (k1, k2) in [(a, b) for a in SWEEP_K1 for b in SWEEP_K2 if only_k1 in (0, a)]:
        for T_q in (0.2, 0.5, 0.8):
            for T_t in (0.0, 0.3, 0.6):
                ctx.set_decoding(T_q, T_t, k1, k2, cfg.temperature)
                out, st = ctx.generate(prompt, n_new, cfg.sample_seed)
                print(f"{k1} {k2} {T_q} {T_t} {n_new / st['ms_decode'] * 1e3:.1f} "
                      f"{st['accepted_q'] / max(st['proposed_q'], 1):.3f} {st['accepted_t'] / max(st['proposed_t'], 1):.3f} "
                      f"{st['ms_d'] / max(st['passes_d'], 1):.3f} {st['ms_q'] / max(st['passes_q'], 1):.3f} "
                      f"{st['ms_t'] / max(st['passes_t'], 1):.3f} {st['passes_d']} {st['passes_q']} {st['passes_t']}", flush=True)
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="paper", choices=["tiny", "small", "paper", "long"])
    ap.add_argument("--n-new", type=int, default=0, help="override the configuration's n_new")
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true")
    ap.add_argument("--no-accept", action="store_true", help="skip the short stand-alone ACCEPT measurement in the JSON line")
    ap.add_argument("--no-baselines", action="store_true",
                    help="skip the untimed comparison runs on the same context (plain target sampling, two-model SD and "
                         "fuzzy SD with the qualifier as proposer, assisted variant, strict thresholds)")
    ap.add_argument("--accept-microbench", action="store_true",
                    help="instead of the loop: time the stand-alone batched ACCEPT stage (vocab 128256, k in 4/8/16/32, "
                         "correlated synthetic logits) and check accept-length histograms against the oracle")
    ap.add_argument("--accept-k", default="4,8,16,32", help="window lengths of --accept-microbench")
    ap.add_argument("--accept-quick", action="store_true",
                    help="--accept-microbench on rho 0.8 only, 500 trials per setting, no oracle runs: short enough to run under a profiler")
    ap.add_argument("--accept-trials", type=int, default=10000, help="trials per (pairing, k, rho, threshold) of --accept-microbench")
    ap.add_argument("--sweep", action="store_true",
                    help="instead of the timed steps: sweep k1 x k2 x T_q x T_t on the chosen configuration and print a table")
    ap.add_argument("--sweep-k1", type=int, default=0, help="--sweep for this draft length only (0: all of 3, 5, 8)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 256 MiB device-to-device copy (a kernel of known traffic, for scaling "
                         "hardware counters read under rocprofv3 --pmc)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs the batch-1 loop on ONE GPU; --gpus N with N > 1 is not supported "
            "(the loop is a dependency chain: it would shard by model placement or tensor-parallel projections)")
        return 2

    if args.accept_microbench:   # starts its CPU workers before anything touches the GPU
        ks = tuple(int(x) for x in args.accept_k.split(","))
        if args.accept_quick:
            return accept_microbench(ks, (0.8,), min(args.accept_trials, 500), 50, 0, 0, args.calibrate_copy)
        return accept_microbench(ks, trials=args.accept_trials, calibrate=args.calibrate_copy)

    import paper_2510_12966_amd as psd
    from paper_2510_12966_amd import synth

    cfg = synth.CONFIGS[args.config]
    n_new = args.n_new or cfg.n_new
    t0 = time.time()
    d, q, t, prompt = synth.build_stack(cfg)
    log(f"[bench] synthetic weights for '{cfg.name}' built in {time.time() - t0:.1f} s "
        f"({(d.nbytes + q.nbytes + t.nbytes) / 1e9:.2f} GB)")
    shapes = (cfg.draft, cfg.qualifier, cfg.target)
    descs = [psd.ModelDesc(s.n_layers, s.d_model, s.n_heads, s.n_kv_heads, s.d_ffn, s.vocab, cfg.rope_theta,
                           cfg.dtype, b) for s, b in zip(shapes, (d, q, t))]
    k1_cap, k2_cap = (max(SWEEP_K1), max(SWEEP_K2)) if args.sweep else (cfg.k1, cfg.k2)
    max_seq = cfg.n_prompt + n_new + k2_cap + 2
    t0 = time.time()
    ctx = psd.Context(descs[0], descs[1], descs[2], cfg.T_q, cfg.T_t, k1_cap, k2_cap, max_seq,
                      temperature=cfg.temperature, flags=0 if args.no_graph else psd.FLAG_GRAPH)
    log(f"[bench] context created (weights uploaded and re-tiled) in {time.time() - t0:.1f} s")

    if args.calibrate_copy:
        a, b = psd.DeviceBuffer(256 << 20), psd.DeviceBuffer(256 << 20)
        psd.lib().psd_dev_copy(b.data_ptr(), a.data_ptr(), 256 << 20, 2)
        psd.dev_sync()
        a.free(); b.free()
    if args.sweep:
        return sweep(ctx, cfg, prompt, n_new, args.sweep_k1)
    for i in range(args.warmup):
        out, st = ctx.generate(prompt, n_new, cfg.sample_seed)
        log(f"[bench] warmup {i}: decode {st['ms_decode']:.1f} ms, prefill {st['ms_prefill']:.1f} ms")
    psd.dev_sync()
    decode_ms = prefill_ms = 0.0
    t0 = time.perf_counter()
    for i in range(args.steps):
        out, st = ctx.generate(prompt, n_new, cfg.sample_seed + i)
        decode_ms += st["ms_decode"]
        prefill_ms += st["ms_prefill"]
    psd.dev_sync()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    value = n_new * args.steps / wall
    log(f"[bench] {args.steps} steps: {ms_per_step:.1f} ms/step, decode-only {n_new * args.steps / decode_ms * 1e3:.1f} tok/s, "
        f"last stats {st}")

    # Whole loop against the HBM roofline: algorithmic bytes of the decoding passes of the last timed step (every weight
    # matrix once per pass, the KV cache of the context as bf16, the logits rows written, the ACCEPT rows read once)
    # over the device time between the end of prefill and the last token.
    def weight_bytes(sh):
        hd = sh.d_model // sh.n_heads
        per_layer = 2 * sh.d_model * sh.n_heads * hd + 2 * sh.d_model * sh.n_kv_heads * hd + 3 * sh.d_model * sh.d_ffn
        return 2.0 * (sh.n_layers * per_layer + sh.vocab * sh.d_model)
    ctx_mid = cfg.n_prompt + n_new / 2
    V = cfg.target.vocab
    loop_bytes = 0.0
    for sh, key, rows in ((cfg.draft, "passes_d", 1), (cfg.qualifier, "passes_q", cfg.k1 + 1), (cfg.target, "passes_t", cfg.k2 + 1)):
        kvb = 2 * sh.n_kv_heads * (sh.d_model // sh.n_heads) * 2 * sh.n_layers
        loop_bytes += st[key] * (weight_bytes(sh) + ctx_mid * kvb + rows * V * 4)
    loop_bytes += st["passes_q"] * (2 * cfg.k1 + 1) * V * 4 + st["passes_t"] * (2 * cfg.k2 + 1) * V * 4
    loop_gbps = loop_bytes / (st["ms_decode"] * 1e-3) / 1e9
    whole_loop = {"algorithmic_GB_per_step": round(loop_bytes / 1e9, 2), "achieved_GBps": round(loop_gbps, 1),
                  "frac_of_hbm_peak": round(loop_gbps / HBM_PEAK_GBS, 4)}
    log(f"[bench] whole decoding loop: {loop_bytes / 1e9:.1f} GB algorithmic in {st['ms_decode']:.1f} ms = {loop_gbps:.0f} GB/s "
        f"= {loop_gbps / HBM_PEAK_GBS:.3f} of the HBM peak")

    baselines = None
    if not args.no_baselines:
        # Untimed comparison runs on the same context, decode-only tokens/s each (Section 3.3: the speed-up is
        # quoted against two-model speculative decoding with the qualifier-sized model as proposer).
        def rate(fn, n):
            _, s_ = fn(n)
            return round(n / s_["ms_decode"] * 1e3, 1), s_
        seed = cfg.sample_seed
        baselines = {"psd_f": round(n_new * args.steps / decode_ms * 1e3, 1)}
        baselines["plain_target"], _ = rate(lambda n: ctx.generate_plain(2, prompt, n, seed), min(n_new, 128))
        for name, tau in (("sd", 0.0), ("fsd", cfg.T_t)):
            best = None
            for k in sorted({cfg.k1, cfg.k2}):
                r, s_ = rate(lambda n: ctx.generate_sd(1, k, tau, prompt, n, seed), n_new)
                row = {"k": k, "tokens_per_s": r, "accept_rate": round(s_["accepted_t"] / max(s_["proposed_t"], 1), 4)}
                if best is None or r > best["tokens_per_s"]:
                    best = row
            baselines[name + "_qualifier_to_target"] = best
        ctx.set_assisted(True)
        r, s_ = rate(lambda n: ctx.generate(prompt, n, seed), n_new)
        ctx.set_assisted(False)
        baselines["psd_a"] = {"tokens_per_s": r, "accept_rate_q": round(s_["accepted_q"] / max(s_["proposed_q"], 1), 4),
                              "accept_rate_t": round(s_["accepted_t"] / max(s_["proposed_t"], 1), 4)}
        ctx.set_decoding(0.0, 0.0, cfg.k1, cfg.k2, cfg.temperature)
        r, s_ = rate(lambda n: ctx.generate(prompt, n, seed), min(n_new, 128))
        ctx.set_decoding(cfg.T_q, cfg.T_t, cfg.k1, cfg.k2, cfg.temperature)
        baselines["psd_strict_thresholds"] = {"tokens_per_s": r,
                                              "accept_rate_q": round(s_["accepted_q"] / max(s_["proposed_q"], 1), 4),
                                              "accept_rate_t": round(s_["accepted_t"] / max(s_["proposed_t"], 1), 4)}
        # thresholds inside this synthetic stack's divergence range (paper shapes: stage 1 0.198-0.213, stage 2
        # 0.256-0.275), so that both stages accept by threshold, by coin, and reject: three points from strict to loose,
        # each with the closed forms of Section 3.3 evaluated at its own accept rates and per-pass speeds
        curve = {"paper": ((0.200, 0.260), (0.205, 0.266), (0.210, 0.272)), "long": ((0.200, 0.260), (0.205, 0.266), (0.210, 0.272)),
                 "small": ((0.03, 0.03), (0.05, 0.05), (0.08, 0.08)), "tiny": ((0.002, 0.006), (0.004, 0.012), (0.008, 0.02))}[cfg.name]
        points = []
        for tq, tt in curve:
            ctx.set_decoding(tq, tt, cfg.k1, cfg.k2, cfg.temperature)
            r, s_ = rate(lambda n: ctx.generate(prompt, n, seed), min(n_new, 256))
            bq, bt = s_["accepted_q"] / max(s_["proposed_q"], 1), s_["accepted_t"] / max(s_["proposed_t"], 1)
            vd, vq, vt = (1e3 * s_[p] / max(s_[m], 1e-9) for p, m in (("passes_d", "ms_d"), ("passes_q", "ms_q"), ("passes_t", "ms_t")))
            _, v_model, _ = throughput_model(bq, bt, cfg.k1, cfg.k2, vd, vq, vt)
            points.append({"T_q": tq, "T_t": tt, "tokens_per_s": r, "accept_rate_q": round(bq, 4), "accept_rate_t": round(bt, 4),
                           "threshold_accepts_q": round(s_["fuzzy_q"] / max(s_["proposed_q"], 1), 4),
                           "threshold_accepts_t": round(s_["fuzzy_t"] / max(s_["proposed_t"], 1), 4),
                           "section_3_3_V_PSD": round(v_model, 1)})
        ctx.set_decoding(cfg.T_q, cfg.T_t, cfg.k1, cfg.k2, cfg.temperature)
        baselines["psd_mid_thresholds"] = points[1]
        baselines["psd_threshold_curve"] = points
        ctx.set_greedy(True)      # temperature -> 0 limit: top predictions everywhere, exact token match in both stages
        r, s_ = rate(lambda n: ctx.generate(prompt, n, seed), min(n_new, 64))
        ctx.set_greedy(False)
        baselines["psd_greedy"] = {"tokens_per_s": r, "accept_rate_q": round(s_["accepted_q"] / max(s_["proposed_q"], 1), 4),
                                   "accept_rate_t": round(s_["accepted_t"] / max(s_["proposed_t"], 1), 4)}
        ctx.set_row_stats(True)   # entropy / confidence per model over one more run (Section 4's two statistics)
        ctx.generate(prompt, min(n_new, 128), seed)
        baselines["row_stats"] = {m: {"rows": v[0], "mean_entropy_nats": round(v[1], 4), "mean_max_prob": round(v[2], 6)}
                                  for m, v in ctx.row_stats().items()}
        ctx.set_row_stats(False)
        # Section 3.3's closed forms evaluated at this run's own accept rates and per-pass times; they ignore the
        # catch-up widths, the ACCEPT kernels and the host, so they bound the measured rate from above
        v_d, v_q, v_t = (1e3 * st[p] / max(st[m], 1e-9) for p, m in (("passes_d", "ms_d"), ("passes_q", "ms_q"), ("passes_t", "ms_t")))
        f_qd, f_psd, _ = throughput_model(st["accepted_q"] / max(st["proposed_q"], 1), st["accepted_t"] / max(st["proposed_t"], 1),
                                          cfg.k1, cfg.k2, v_d, v_q, v_t)
        baselines["section_3_3_model"] = {"V_FSD_QD": round(f_qd, 1), "V_PSD": round(f_psd, 1),
                                          "measured_over_model": round(baselines["psd_f"] / f_psd, 3)}
        baselines["psd_f_over_sd"] = round(baselines["psd_f"] / baselines["sd_qualifier_to_target"]["tokens_per_s"], 3)
        baselines["psd_f_over_fsd"] = round(baselines["psd_f"] / baselines["fsd_qualifier_to_target"]["tokens_per_s"], 3)
        log(f"[bench] comparison runs (decode tokens/s): {baselines}")

    bytes_per_pass = {"draft": None, "qualifier": None, "target": None}
    roofline = None
    kernels = []
    if not args.no_profile:
        # per-kernel device time: the same loop once more, launched kernel by kernel with a HIP event pair
        # around every launch on the library's stream
        ctx.profile(True)
        _, pst = ctx.generate(prompt, n_new, cfg.sample_seed)
        kernels = ctx.kernel_stats()
        ctx.profile(False)
        # one more row: an event pair around a kernel that does nothing, once per pass (what the intervals below
        # hold besides kernel time; rocprofv3's begin/end timestamps do not contain it)
        empty = [r for r in kernels if r["name"].startswith("empty kernel")]
        kernels = [r for r in kernels if not r["name"].startswith("empty kernel")]
        kernels.sort(key=lambda r: -r["ms_total"])
        tot = sum(r["ms_total"] for r in kernels)
        for r in kernels:
            gbs = r["bytes_total"] / r["ms_total"] / 1e6 if r["ms_total"] > 0 else 0.0
            log(f"[bench]   {r['name']:<34s} {r['launches']:>7d} launches {r['ms_total']:>9.2f} ms "
                f"({100 * r['ms_total'] / tot:4.1f}%)  {gbs:8.1f} GB/s")
        dom = kernels[0]
        ach = dom["bytes_total"] / dom["ms_total"] / 1e6
        roofline = {"bound": "hbm", "kernel": dom["name"], "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                    "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4),
                    "traffic": None, "traffic_source": None,
                    "avg_launch_us": round(dom["ms_total"] / dom["launches"] * 1e3, 2),
                    "bytes_per_launch": round(dom["bytes_total"] / dom["launches"]),
                    "all_gemm_GBps": None,
                    "empty_kernel_event_pair_us": round(empty[0]["ms_total"] / empty[0]["launches"] * 1e3, 2) if empty else None}
        roofline["traffic"], roofline["traffic_source"] = measured_traffic(cfg.name, dom["name"].rsplit(" w<=", 1)[0])
        g = [r for r in kernels if r["name"].startswith("gemm")]
        att = [r for r in kernels if r["name"].startswith("attn ") and "w<=512" not in r["name"] and r["ms_total"] > 0]
        if att:   # attention of the decoding passes: algorithmic KV bytes (bf16 K and V of every visible key) per second
            roofline["attention_GBps"] = round(sum(r["bytes_total"] for r in att) / sum(r["ms_total"] for r in att) / 1e6, 1)
        if g:
            roofline["all_gemm_GBps"] = round(sum(r["bytes_total"] for r in g) / sum(r["ms_total"] for r in g) / 1e6, 1)
        roofline["cost_model"] = cost_model(
            kernels, {"draft": pst["passes_d"], "qualifier": pst["passes_q"], "target": pst["passes_t"]},
            {m: st[k] / max(st[p_], 1) for m, k, p_ in (("draft", "ms_d", "passes_d"), ("qualifier", "ms_q", "passes_q"),
                                                         ("target", "ms_t", "passes_t"))})

    acc_mb = None
    if not args.no_accept:
        acc_mb = accept_quick(psd, synth)

    cpu = None
    if not args.no_cpu_baseline:
        import oracle

        cores = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        # bounded sample of the same workload: same models and decoding parameters, a short prompt and
        # roughly one target pass worth of tokens (the fp64 oracle needs ~0.2 TFLOP per target pass here)
        sp = {"tiny": (cfg.n_prompt, cfg.n_new), "small": (16, 24), "paper": (4, 8), "long": (4, 8)}[cfg.name]
        ms = sp[0] + sp[1] + cfg.k2 + 2
        oD = oracle.Model(cfg.draft, d, cfg.dtype, cfg.rope_theta, ms)
        oQ = oracle.Model(cfg.qualifier, q, cfg.dtype, cfg.rope_theta, ms)
        oT = oracle.Model(cfg.target, t, cfg.dtype, cfg.rope_theta, ms)
        t0 = time.perf_counter()
        oout, ost = oracle.generate(oD, oQ, oT, prompt[:sp[0]], sp[1], cfg.sample_seed, cfg.k1, cfg.k2, cfg.T_q, cfg.T_t,
                                    cfg.temperature)
        dt = time.perf_counter() - t0
        cpu = {"value": round(sp[1] / dt, 4), "unit": "tokens/s", "cores": cores, "kind": "oracle",
               "sample": f"same models and decoding parameters, prompt truncated to {sp[0]} tokens, {sp[1]} new tokens "
                         f"(prefill included), {dt:.1f} s"}
        log(f"[bench] oracle: {sp[1]} tokens in {dt:.1f} s on {cores} threads, stats {ost}")

    line = {
        "metric": "generated tokens/s (batch 1), three-model PyramidSD loop",
        "value": round(value, 2), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 2), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if cfg.dtype == synth.DTYPE_BF16 else "f32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: draft {cfg.draft.n_layers}L/{cfg.draft.d_model}, qualifier "
                               f"{cfg.qualifier.n_layers}L/{cfg.qualifier.d_model}, target {cfg.target.n_layers}L/"
                               f"{cfg.target.d_model}, vocab {cfg.target.vocab}; prompt {cfg.n_prompt}, n_new {n_new}, "
                               f"k1 {cfg.k1}, k2 {cfg.k2}, T_q {cfg.T_q}, T_t {cfg.T_t}, temperature {cfg.temperature}",
                   "graphs": not args.no_graph},
        "decode_tokens_per_s": round(n_new * args.steps / decode_ms * 1e3, 2),
        "prefill_ms_per_step": round(prefill_ms / args.steps, 2),
        "accept_rate_q": round(st["accepted_q"] / max(st["proposed_q"], 1), 4),
        "accept_rate_t": round(st["accepted_t"] / max(st["proposed_t"], 1), 4),
        "passes": {"draft": st["passes_d"], "qualifier": st["passes_q"], "target": st["passes_t"]},
        "ms_per_pass": {"draft": round(st["ms_d"] / max(st["passes_d"], 1), 4),
                        "qualifier": round(st["ms_q"] / max(st["passes_q"], 1), 4),
                        "target": round(st["ms_t"] / max(st["passes_t"], 1), 4),
                        "accept": round(st["ms_accept"] / max(st["passes_q"] + st["passes_t"], 1), 4)},
        "roofline": roofline, "whole_loop": whole_loop, "accept_microbench": acc_mb, "accept_wait_expiries": psd.get_accept_expiries(),
        "cpu_baseline": cpu, "comparison_runs": baselines,
        "paper_context": "124.13 tok/s PSD_F best, 1.91x over SD, RTX 4090, trained Llama 1B/3B/8B (Tables 2-3)",
    }
    print(json.dumps(line), flush=True)
    ctx.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
