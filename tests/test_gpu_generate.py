"""GPU parity of the two-stage loop against the CPU oracle, through psd_generate."""
import numpy as np
import pytest

import oracle
import paper_2510_12966_amd as psd
from paper_2510_12966_amd import synth
from replay import Replay, forced_for

pytestmark = pytest.mark.gpu



def _desc(shape, blob, dtype, theta):
    return psd.ModelDesc(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.d_ffn, shape.vocab,
                         theta, dtype, blob)


def _ctx(cfg, blobs, max_seq, T_q, T_t, k1, k2, flags=0, temperature=1.0):
    shapes = (cfg.draft, cfg.qualifier, cfg.target)
    d, q, t = (_desc(s, b, cfg.dtype, cfg.rope_theta) for s, b in zip(shapes, blobs))
    return psd.Context(d, q, t, T_q, T_t, k1, k2, max_seq, temperature=temperature, flags=flags)


def _oracle_run(cfg, blobs, prompt, n_new, seed, k1, k2, T_q, T_t, temperature=1.0):
    ms = len(prompt) + n_new + k2 + 2
    D = oracle.Model(cfg.draft, blobs[0], cfg.dtype, cfg.rope_theta, ms)
    Q = oracle.Model(cfg.qualifier, blobs[1], cfg.dtype, cfg.rope_theta, ms)
    T = oracle.Model(cfg.target, blobs[2], cfg.dtype, cfg.rope_theta, ms)
    return oracle.generate(D, Q, T, prompt, n_new, seed, k1, k2, T_q, T_t, temperature)


SETTINGS = [  # (T_q, T_t, k1, k2, temperature); the first row is the tiny configuration as specified
    (0.3, 0.2, 4, 8, 1.0),
    (0.004, 0.012, 4, 8, 1.0),   # thresholds inside the divergence range of this stack: both stages reject
    (0.0, 0.0, 3, 7, 1.0),       # strict speculative sampling
    (0.006, 0.0, 5, 5, 0.7),
    (0.004, 0.012, 1, 1, 1.0),
    (0.01, 0.01, 8, 3, 1.0),     # k1 > k2: rounds are capped by the window
    (0.3, 0.2, 30, 31, 1.0),     # the largest windows the interface takes: 32-token target passes
    (0.004, 0.012, 30, 31, 1.0), # the same with rejections in both stages
]


@pytest.mark.parametrize("graph", [0, psd.FLAG_GRAPH])
@pytest.mark.parametrize("setting", SETTINGS)
def test_tiny_stack_matches_oracle_end_to_end(tiny_stack, setting, graph):
    cfg, d, q, t, prompt = tiny_stack
    T_q, T_t, k1, k2, temp = setting
    n_new, seed = cfg.n_new, cfg.sample_seed
    ctx = _ctx(cfg, (d, q, t), len(prompt) + n_new + k2 + 2, T_q, T_t, k1, k2, flags=graph, temperature=temp)
    ms = len(prompt) + n_new + k2 + 2
    forced = forced_for((cfg.draft, cfg.qualifier, cfg.target), (d, q, t), cfg.dtype, cfg.rope_theta, ms, prompt)
    rp = Replay(seed, T_q, T_t, temp, forced)
    ctx.set_trace(rp)
    out, st = ctx.generate(prompt, n_new, seed)
    ctx.set_trace(None)
    # every row the loop consumed was recomputed by the oracle on the GPU's own sequence, every decision re-taken on
    # the GPU's own rows: the run is verified step by step whatever the oracle's free-running call below emits
    assert rp.events > 0 and forced.rows >= rp.events and forced.cur[len(prompt):len(prompt) + n_new] == out.tolist()
    ref, ost = _oracle_run(cfg, (d, q, t), prompt, n_new, seed, k1, k2, T_q, T_t, temp)
    if rp.ties == 0 and np.array_equal(out, ref):
        for key in ("proposed_q", "accepted_q", "fuzzy_q", "proposed_t", "accepted_t", "fuzzy_t", "passes_d",
                    "passes_q", "passes_t"):
            assert st[key] == ost[key], key
    # a second call on the same context gives the same answer (caches and graphs are reusable)
    out2, st2 = ctx.generate(prompt, n_new, seed)
    assert np.array_equal(out, out2)
    assert st["accepted_t"] == st2["accepted_t"] and st["accepted_q"] == st2["accepted_q"]
    ctx.close()


def test_tiny_stack_exact_token_parity_over_seeds(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ctx = _ctx(cfg, (d, q, t), 16 + 40 + 10, 0.004, 0.012, 4, 8)
    same = 0
    for seed in range(6):
        out, st = ctx.generate(prompt, 40, seed)
        ref, ost = _oracle_run(cfg, (d, q, t), prompt, 40, seed, 4, 8, 0.004, 0.012)
        same += int(np.array_equal(out, ref))
        assert 0 < st["accepted_q"] <= st["proposed_q"]
    assert same >= 5   # a near-tie may flip one run; see the replay test for the exact bar
    ctx.close()


def test_shortest_prompts_match_oracle(tiny_stack):
    # a one-token prompt has nothing to ingest (the caches start empty); two tokens ingest exactly one
    cfg, d, q, t, prompt = tiny_stack
    ctx = _ctx(cfg, (d, q, t), 2 + 24 + 10, 0.004, 0.012, 4, 8)
    for n_prompt in (1, 2):
        forced = forced_for((cfg.draft, cfg.qualifier, cfg.target), (d, q, t), cfg.dtype, cfg.rope_theta, 2 + 24 + 10, prompt[:n_prompt])
        rp = Replay(4, 0.004, 0.012, 1.0, forced)
        ctx.set_trace(rp)
        out, st = ctx.generate(prompt[:n_prompt], 24, 4)
        assert forced.rows > 0 and forced.cur[n_prompt:n_prompt + 24] == out.tolist()
        ctx.set_trace(None)
        ref, ost = _oracle_run(cfg, (d, q, t), prompt[:n_prompt], 24, 4, 4, 8, 0.004, 0.012)
        assert rp.ties > 0 or np.array_equal(out, ref)
        assert out.size == 24
    ctx.close()


def test_identical_models_accept_everything_and_equal_plain_sampling(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    shapes = (cfg.qualifier,) * 3
    descs = [_desc(s, q, cfg.dtype, cfg.rope_theta) for s in shapes]
    for (k1, k2) in ((4, 8), (3, 7), (1, 1)):
        ctx = psd.Context(descs[0], descs[1], descs[2], 0.0, 0.0, k1, k2, 16 + 48 + k2 + 2)
        out, st = ctx.generate(prompt, 48, 9)
        assert st["accepted_q"] == st["proposed_q"] and st["accepted_t"] == st["proposed_t"]
        plain, _ = ctx.generate_plain(2, prompt, 48, 9)
        assert np.array_equal(out, plain)
        ctx.close()


def test_small_bf16_stack_replay_and_baseline_settings():
    cfg = synth.CONFIGS["small"]
    d, q, t, prompt = synth.build_stack(cfg)
    n_new = 48
    ctx = _ctx(cfg, (d, q, t), cfg.n_prompt + n_new + cfg.k2 + 2, cfg.T_q, cfg.T_t, cfg.k1, cfg.k2, flags=psd.FLAG_GRAPH)
    ms = cfg.n_prompt + n_new + cfg.k2 + 2
    forced = forced_for((cfg.draft, cfg.qualifier, cfg.target), (d, q, t), cfg.dtype, cfg.rope_theta, ms, prompt)
    rp = Replay(cfg.sample_seed, cfg.T_q, cfg.T_t, 1.0, forced)
    ctx.set_trace(rp)
    out, st = ctx.generate(prompt, n_new, cfg.sample_seed)
    ctx.set_trace(None)
    print("small stack:", st, "ties", rp.ties, "max div err", rp.max_div_err, "in-loop rows", forced.rows,
          "max |logit err| against the oracle's forward", forced.max_err, flush=True)
    assert rp.ties <= 1 and rp.events >= 10 and forced.rows >= 48
    assert (out >= 0).all() and (out < cfg.target.vocab).all()
    assert st["proposed_t"] == cfg.k2 * st["passes_t"]
    # tighter thresholds so that both stages reject on this stack too
    ctx.set_decoding(0.05, 0.05, cfg.k1, cfg.k2)
    forced = forced_for((cfg.draft, cfg.qualifier, cfg.target), (d, q, t), cfg.dtype, cfg.rope_theta, ms, prompt)
    rp = Replay(3, 0.05, 0.05, 1.0, forced)
    ctx.set_trace(rp)
    out, st = ctx.generate(prompt, n_new, 3)
    ctx.set_trace(None)
    print("small stack, tight:", st, "ties", rp.ties, "max |logit err| in the loop", forced.max_err, flush=True)
    assert rp.ties <= 1 and 0 < st["accepted_q"] < st["proposed_q"] and 0 < st["accepted_t"] < st["proposed_t"]
    ctx.close()
    # the largest windows the interface takes (bf16 kernels of the 32-column class inside the loop)
    for T_q, T_t in ((cfg.T_q, cfg.T_t), (0.05, 0.05)):
        ctx = _ctx(cfg, (d, q, t), cfg.n_prompt + 80 + 31 + 2, T_q, T_t, 30, 31, flags=psd.FLAG_GRAPH)
        rp = Replay(5, T_q, T_t)
        ctx.set_trace(rp)
        out, st = ctx.generate(prompt, 80, 5)
        ctx.set_trace(None)
        print("small stack, k1 30, k2 31:", st, "ties", rp.ties, flush=True)
        assert rp.ties <= 1 and rp.events >= 3
        assert st["proposed_t"] == 31 * st["passes_t"]
        ctx.close()


def test_generate_argument_errors(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ctx = _ctx(cfg, (d, q, t), 64, 0.3, 0.2, 4, 8)
    with pytest.raises(psd.PsdError):
        ctx.generate(prompt, 64, 1)                      # 16 + 64 + 8 + 2 > 64
    with pytest.raises(psd.PsdError):
        ctx.generate(np.array([600], np.int32), 4, 1)     # token outside the vocabulary
    with pytest.raises(psd.PsdError):
        ctx.set_decoding(0.1, 0.1, 5, 8)                  # k1 above the context's capacity
    with pytest.raises(psd.PsdError):
        ctx.set_decoding(-0.1, 0.1, 4, 8)
    out, _ = ctx.generate(prompt, 0, 1)
    assert out.size == 0
    ctx.close()


def test_create_with_a_pool_too_small_is_enomem(tiny_stack):
    import ctypes as C
    from paper_2510_12966_amd import binding as b
    cfg, d, q, t, prompt = tiny_stack
    descs = [_desc(s, w, cfg.dtype, cfg.rope_theta).c() for s, w in zip((cfg.draft, cfg.qualifier, cfg.target), (d, q, t))]
    L = b.lib()
    prm = b._Params(0.3, 0.2, 1.0, 4, 8, 96, 0, 0, 0)
    need = L.psd_pool_bytes_needed(C.byref(descs[0]), C.byref(descs[1]), C.byref(descs[2]), C.byref(prm))
    assert need > 0
    for pool in (need - 1, need // 2, 4096):
        prm.pool_bytes = pool
        h = C.c_void_p(0x1234)     # must come back as NULL: no output on failure
        rc = L.psd_create(C.byref(descs[0]), C.byref(descs[1]), C.byref(descs[2]), C.byref(prm), C.byref(h))
        assert rc == -3 and h.value is None                                   # PSD_ENOMEM
        msg = L.psd_last_error(None).decode()
        assert "pool" in msg and str(need) in msg
    prm.pool_bytes = need                                                     # exactly enough works, and decodes
    h = C.c_void_p(None)
    assert L.psd_create(C.byref(descs[0]), C.byref(descs[1]), C.byref(descs[2]), C.byref(prm), C.byref(h)) == 0 and h.value
    L.psd_destroy(h)
    ctx = psd.Context(*[_desc(s, w, cfg.dtype, cfg.rope_theta) for s, w in zip((cfg.draft, cfg.qualifier, cfg.target), (d, q, t))],
                      0.3, 0.2, 4, 8, 96, pool_bytes=need + (1 << 20))           # a larger pool is fine too
    out, _ = ctx.generate(prompt, 8, 1)
    assert out.size == 8
    ctx.close()


def test_paper_shapes_sampled_parity():
    """Full-size models (1B / 3B / 8B shapes, vocabulary 128256) in the launch configuration bench.py times
    (graph replay): every ACCEPT and every draft sample of a short run is replayed through the oracle on the GPU's
    own logits; the logits rows the loop consumed in its first rounds (thresholds at which both stages reject, so the
    caches have been rolled back) are recomputed by the oracle's forward, teacher-forced on the GPU's own sequence; and
    one more pass per model is compared with the oracle's forward.  The 512-token
    prompt-ingestion passes, which the oracle cannot follow at this size in reasonable time, are tied to the
    passes it does check: they must leave the same KV cache bit for bit."""
    cfg = synth.CONFIGS["paper"]
    d, q, t, prompt = synth.build_stack(cfg)
    n_prompt, n_new = 24, 40
    ctx = _ctx(cfg, (d, q, t), 640, cfg.T_q, cfg.T_t, cfg.k1, cfg.k2, flags=psd.FLAG_GRAPH)
    rp = Replay(cfg.sample_seed, cfg.T_q, cfg.T_t)
    ctx.set_trace(rp)
    out, st = ctx.generate(prompt[:n_prompt], n_new, cfg.sample_seed)
    print("paper stack:", st, "ties", rp.ties, "max div err", rp.max_div_err, flush=True)
    assert rp.ties <= 1 and rp.events >= 10
    # thresholds inside this stack's divergence range, so that rejections and resampling run at full size too
    ctx.set_decoding(0.205, 0.266, cfg.k1, cfg.k2)   # the medians of the two stages' divergences on this stack
    rp = Replay(5, 0.205, 0.266)
    ctx.set_trace(rp)
    out, st = ctx.generate(prompt[:n_prompt], n_new, 5)
    ctx.set_trace(None)
    print("paper stack, tighter thresholds:", st, "ties", rp.ties, flush=True)
    assert rp.ties <= 1 and 0 < st["fuzzy_q"] < st["proposed_q"] and 0 < st["fuzzy_t"] < st["proposed_t"]
    # in-loop rows against the oracle's forward: a short prompt and a bounded number of rows per model keep the oracle's
    # share to a few hundred GFLOP (the 8B-shaped forward costs it 15 GFLOP per token)
    short = prompt[:6]
    forced = forced_for((cfg.draft, cfg.qualifier, cfg.target), (d, q, t), cfg.dtype, cfg.rope_theta, 64, short,
                        max_rows={0: 12, 1: 12, 2: 11})
    rp = Replay(9, 0.205, 0.266, 1.0, forced)
    ctx.set_trace(rp)
    out, st = ctx.generate(short, 14, 9)
    ctx.set_trace(None)
    print("paper stack, in-loop rows checked per model:", forced.rows_of, "max |logit err|", forced.max_err, st, flush=True)
    assert min(forced.rows_of.values()) >= 10 and forced.cur[6:20] == out.tolist()
    toks = prompt[:12]
    shapes, blobs = (cfg.draft, cfg.qualifier, cfg.target), (d, q, t)
    for which in range(3):
        om = oracle.Model(shapes[which], blobs[which], cfg.dtype, cfg.rope_theta, 16)
        ref = om.forward(toks, 0)
        got = np.concatenate([ctx.forward(which, toks[:1], 0), ctx.forward(which, toks[1:12], 1)])
        err = float(np.abs(got - ref).max())
        print(f"paper model {which}: max |logit err| {err:.3e}, logit std {ref.std():.3f}", flush=True)
        assert err <= 3e-2
    n = 572
    long_toks = synth.tokens(31, 0, n + 4, cfg.target.vocab)
    for which in range(3):
        outs = []
        for widths in ([512, 60], [32] * 17 + [28]):
            pos = 0
            for w in widths:
                ctx.forward(which, long_toks[pos:pos + w], pos, want_logits=False)
                pos += w
            outs.append(ctx.forward(which, long_toks[n:n + 4], n))
        assert np.array_equal(outs[0], outs[1])
    ctx.close()


def test_generation_survives_expired_waits(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ctx = _ctx(cfg, (d, q, t), 16 + 32 + 10, 0.004, 0.012, 4, 8)
    ref, _ = ctx.generate(prompt, 32, 3)
    try:
        psd.set_accept_path(3)     # waits expire at once; vocabulary 512 is a single chunk, so nothing ever waits
        out, _ = ctx.generate(prompt, 32, 3)
        assert np.array_equal(out, ref)
    finally:
        psd.set_accept_path(0)
    ctx.close()


@pytest.mark.parametrize("case", range(18))
def test_randomised_stacks_replay(case):
    """Seeded random shapes, windows, thresholds and prompt lengths (through the 128- and 512-token ingestion passes
    and every narrow launch class; cases 12.. are fp32 stacks): each sampling step and ACCEPT stage is replayed
    through the oracle on the GPU's own logits, and the target's logits over the finished sequence are compared
    with the oracle's forward."""
    from paper_2510_12966_amd.synth import ModelShape
    rng = np.random.default_rng(1000 + case)
    vocab = int(rng.choice([1000, 2051, 4096]))
    bf16 = case < 12
    dtype, tol = (synth.DTYPE_BF16, 3e-2) if bf16 else (synth.DTYPE_F32, 1e-4)

    def shape():
        d = int(rng.choice([256, 512] if bf16 else [64, 128, 256]))
        h, kv = [(4, 2), (8, 2), (4, 4), (8, 8)][int(rng.integers(4))] if bf16 else [(4, 2), (4, 4), (2, 1)][int(rng.integers(3))]
        return ModelShape(int(rng.integers(1, 4)), d, h, kv, int(rng.choice([352, 704, 1024] if bf16 else [256, 480, 1024])), vocab)

    shapes = (shape(), shape(), shape())
    blobs = [synth.target_weights(s, 500 + 10 * case + i, dtype, sigma=0.03) for i, s in enumerate(shapes)]
    k1, k2 = int(rng.integers(1, 9)), int(rng.integers(1, 13))
    T_q, T_t = float(rng.uniform(0.0, 0.3)), float(rng.uniform(0.0, 0.3))
    temp = float(rng.choice([1.0, 0.7]))
    n_prompt, n_new = int(rng.choice([3, 40, 150, 600])), 30
    prompt = synth.tokens(77 + case, 0, n_prompt, vocab)
    max_seq = n_prompt + n_new + k2 + 2
    descs = [_desc(s, b, dtype, 10000.0) for s, b in zip(shapes, blobs)]
    ctx = psd.Context(descs[0], descs[1], descs[2], T_q, T_t, k1, k2, max_seq, temperature=temp,
                      flags=(psd.FLAG_GRAPH if case % 2 else 0) | (psd.FLAG_ROW_STATS if case % 3 == 0 else 0))
    forced = forced_for(shapes, blobs, dtype, 10000.0, max_seq, prompt)
    rp = Replay(case, T_q, T_t, temp, forced)
    ctx.set_trace(rp)
    out, st = ctx.generate(prompt, n_new, case)
    ctx.set_trace(None)
    assert forced.rows >= rp.events and forced.cur[n_prompt:n_prompt + n_new] == out.tolist()
    if case % 3 == 0:      # the behaviour statistics ride along: one row per draft step, per judged qualifier / target row
        rs = ctx.row_stats()
        assert rs["draft"][0] == st["passes_d"] and rs["qualifier"][0] > 0 and rs["target"][0] > 0
        for rows, h, pmax in rs.values():
            assert 0.0 < h <= np.log(vocab) + 1e-4 and 1.0 / vocab - 1e-7 <= pmax <= 1.0
    print("case", case, shapes, "k1", k1, "k2", k2, "T", round(T_q, 3), round(T_t, 3), "prompt", n_prompt, st, "ties", rp.ties, flush=True)
    assert rp.events >= 3 and rp.ties <= 1
    assert out.size == n_new and (out >= 0).all() and (out < vocab).all()
    assert st["accepted_q"] <= st["proposed_q"] and st["accepted_t"] <= st["proposed_t"]
    seq = np.concatenate([prompt, out]).astype(np.int32)
    om = oracle.Model(shapes[2], blobs[2], dtype, 10000.0, max_seq)
    ref = om.forward(seq, 0)[-4:]
    pos, widest = 0, 512 if bf16 else 32
    while pos < len(seq) - 4:                       # re-ingest in the widest passes this model takes, then 4 logit rows
        w = min(widest, len(seq) - 4 - pos)
        try:
            ctx.forward(2, seq[pos:pos + w], pos, want_logits=False)
        except psd.PsdError:
            assert widest == 512 and bf16           # a model with very short projections stays at 128-token passes
            widest = 128
            continue
        pos += w
    got = ctx.forward(2, seq[-4:], len(seq) - 4)
    assert np.abs(got - ref).max() <= tol
    ctx.close()


@pytest.mark.parametrize("case", range(4))
def test_randomised_medium_stacks_long_context(case):
    """Head dimension 128, query groups of up to 8, contexts of 700 to 2100 tokens on scrambled pages: replay of every
    stage through the oracle, and the bit-for-bit agreement of the widest ingestion passes with 32-token passes."""
    from paper_2510_12966_amd.synth import ModelShape
    rng = np.random.default_rng(3000 + case)
    vocab = int(rng.choice([4099, 32000]))

    def shape():
        d = int(rng.choice([1024, 2048]))
        h = d // 128
        kv = int(rng.choice([k for k in (1, 2, 4, 8) if h % k == 0 and k <= h]))
        return ModelShape(int(rng.integers(1, 3)), d, h, kv, int(rng.choice([2816, 5632])), vocab)

    shapes = (shape(), shape(), shape())
    blobs = [synth.target_weights(s, 900 + 10 * case + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    k1, k2 = int(rng.integers(2, 9)), int(rng.integers(4, 17))
    T_q, T_t = float(rng.uniform(0.0, 0.3)), float(rng.uniform(0.0, 0.3))
    # 1500 + 24 crosses the 12-key-range switch of the narrow passes while decoding, 2100 lies past the 16-range one
    n_prompt, n_new = (700, 1300, 1500, 2100)[case % 4], 24
    prompt = synth.tokens(277 + case, 0, n_prompt, vocab)
    max_seq = n_prompt + n_new + k2 + 2
    descs = [_desc(s, b, synth.DTYPE_BF16, 500000.0) for s, b in zip(shapes, blobs)]
    ctx = psd.Context(descs[0], descs[1], descs[2], T_q, T_t, k1, k2, max_seq, flags=psd.FLAG_GRAPH | 0x100)
    # in-loop logits against the oracle's forward on the two shorter contexts (qualifier and target rows at 700 tokens,
    # target rows at 1300; the oracle needs seconds per thousand tokens of these shapes)
    forced = forced_for(shapes, blobs, synth.DTYPE_BF16, 500000.0, max_seq, prompt, {0: (1, 2), 1: (2,)}.get(case, ()))
    rp = Replay(case, T_q, T_t, 1.0, forced)
    ctx.set_trace(rp)
    out, st = ctx.generate(prompt, n_new, case)
    ctx.set_trace(None)
    print("case", case, shapes, "k1", k1, "k2", k2, "T", round(T_q, 3), round(T_t, 3), "prompt", n_prompt, st, "ties", rp.ties,
          "in-loop rows checked", forced.rows, "max |logit err|", forced.max_err, flush=True)
    assert forced.cur[n_prompt:n_prompt + n_new] == out.tolist() and (case > 1 or forced.rows > 0)
    assert rp.events >= 3 and rp.ties <= 1 and out.size == n_new
    seq = np.concatenate([prompt, out]).astype(np.int32)
    n = len(seq) - 4
    for which in range(3):
        rows = []
        for widths in ([512] * (n // 512) + ([n % 512] if n % 512 else []), [32] * (n // 32) + ([n % 32] if n % 32 else [])):
            pos = 0
            for w in widths:
                ctx.forward(which, seq[pos:pos + w], pos, want_logits=False)
                pos += w
            rows.append(ctx.forward(which, seq[n:], n))
        assert np.array_equal(rows[0], rows[1])
    ctx.close()


def test_two_contexts_alive_at_once_do_not_disturb_each_other(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    from paper_2510_12966_amd.synth import ModelShape
    a = _ctx(cfg, (d, q, t), 16 + 32 + 10, 0.004, 0.012, 4, 8, flags=psd.FLAG_GRAPH)
    ref_a, _ = a.generate(prompt, 32, 2)
    shapes = (ModelShape(1, 256, 4, 2, 352, 1000), ModelShape(2, 512, 8, 2, 704, 1000), ModelShape(1, 512, 4, 4, 1024, 1000))
    blobs = [synth.target_weights(s, 60 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    descs = [_desc(s, w, synth.DTYPE_BF16, 10000.0) for s, w in zip(shapes, blobs)]
    b = psd.Context(descs[0], descs[1], descs[2], 0.1, 0.1, 3, 6, 200 + 32 + 8, flags=psd.FLAG_GRAPH)
    pb = synth.tokens(5, 0, 200, 1000)
    ref_b, _ = b.generate(pb, 32, 3)
    for _ in range(2):      # interleaved calls on both contexts repeat their own answers
        out_a, _ = a.generate(prompt, 32, 2)
        out_b, _ = b.generate(pb, 32, 3)
        assert np.array_equal(out_a, ref_a) and np.array_equal(out_b, ref_b)
    a.close()
    out_b, _ = b.generate(pb, 32, 3)
    assert np.array_equal(out_b, ref_b)
    b.close()
