"""GPU parity of the decoder forward (logits) against the CPU oracle, through psd_forward."""
import numpy as np
import pytest

import oracle
import paper_2510_12966_amd as psd
from paper_2510_12966_amd import synth
from paper_2510_12966_amd.synth import ModelShape

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-4    # fp32 weights, fp32 accumulate
TOL_BF16 = 3e-2   # bf16 weights and KV cache, fp32 accumulate


def _desc(shape, blob, dtype, theta):
    return psd.ModelDesc(shape.n_layers, shape.d_model, shape.n_heads, shape.n_kv_heads, shape.d_ffn, shape.vocab,
                         theta, dtype, blob)


def _ctx(shapes, blobs, dtype, theta, max_seq, flags=0, k1=4, k2=8):
    d, q, t = (_desc(s, b, dtype, theta) for s, b in zip(shapes, blobs))
    return psd.Context(d, q, t, 0.3, 0.2, k1, k2, max_seq, flags=flags)


def test_tiny_fp32_stack_logits(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    shapes, blobs = (cfg.draft, cfg.qualifier, cfg.target), (d, q, t)
    ctx = _ctx(shapes, blobs, cfg.dtype, cfg.rope_theta, 96)
    toks = synth.tokens(5, 0, 60, cfg.target.vocab)
    for which in range(3):
        om = oracle.Model(shapes[which], blobs[which], cfg.dtype, cfg.rope_theta, 96)
        ref = om.forward(toks, 0)
        # ragged widths: 16 + 1 + 2 + 3 + 5 + 17 + 16
        pos, got = 0, []
        for w in (16, 1, 2, 3, 5, 17, 16):
            got.append(ctx.forward(which, toks[pos:pos + w], pos))
            pos += w
        got = np.concatenate(got)
        assert np.abs(got - ref).max() <= TOL_F32
        # rollback: overwrite rows 20.. with other tokens, then again with the right ones
        ctx.forward(which, (toks[20:31] + 7) % cfg.target.vocab, 20)
        again = ctx.forward(which, toks[20:31], 20)
        assert np.abs(again - ref[20:31]).max() <= TOL_F32
    ctx.close()


MINI = [  # bf16 shapes that cover head dims 64 / 128, group sizes 1..4, ragged vocabulary
    (ModelShape(2, 256, 4, 2, 352, 1000), ModelShape(3, 512, 8, 2, 704, 1000), ModelShape(2, 512, 4, 4, 1024, 1000)),
]


@pytest.mark.parametrize("scramble", [0, 0x100])
def test_bf16_logits_long_context_and_paging(scramble):
    shapes = MINI[0]
    blobs = [synth.target_weights(s, 20 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    n = 300   # spans three 128-key attention splits and five KV pages
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 384, flags=scramble)
    toks = synth.tokens(6, 0, n, 1000)
    for which in range(3):
        om = oracle.Model(shapes[which], blobs[which], synth.DTYPE_BF16, 10000.0, 384)
        ref = om.forward(toks, 0)
        pos, got = 0, []
        widths = [32] * 8 + [11, 1, 1, 6, 3, 17, 5]
        assert sum(widths) == n
        for w in widths:
            got.append(ctx.forward(which, toks[pos:pos + w], pos))
            pos += w
        got = np.concatenate(got)
        err = np.abs(got - ref).max()
        assert np.abs(ref).max() > 0.5 and err <= TOL_BF16, err
    ctx.close()


def test_bf16_width_invariance_is_bit_exact():
    # the same token at the same position gives the same logits bits whatever the width of the pass
    shapes = MINI[0]
    blobs = [synth.target_weights(s, 20 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 256)
    toks = synth.tokens(8, 0, 150, 1000)
    for which in (0, 2):
        ctx.forward(which, toks[:32], 0, want_logits=False)
        for p in range(32, 128, 32):
            ctx.forward(which, toks[p:p + 32], p, want_logits=False)
        wide = ctx.forward(which, toks[128:139], 128)            # width 11
        narrow = np.concatenate([ctx.forward(which, toks[128 + i:129 + i], 128 + i) for i in range(11)])
        assert np.array_equal(wide, narrow)
        two = np.concatenate([ctx.forward(which, toks[128:130], 128), ctx.forward(which, toks[130:139], 130)])
        assert np.array_equal(wide, two)
        wide32 = ctx.forward(which, toks[118:150], 118)           # 32-wide class
        assert np.array_equal(wide32[10:21], wide)
    ctx.close()


@pytest.mark.parametrize("scramble", [0, 0x100])
def test_bf16_prompt_ingestion_in_128_token_passes_is_bit_exact(scramble):
    # a prompt ingested in 128-token passes leaves the same KV cache, bit for bit, as 32-token and ragged passes:
    # the logits of what follows are identical; and they match the oracle
    shapes = MINI[0]
    blobs = [synth.target_weights(s, 20 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    n = 300
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 384, flags=scramble)
    toks = synth.tokens(9, 0, n + 7, 1000)
    for which in range(3):
        out = []
        for widths in ([128, 128, 44], [32] * 9 + [12], [128, 100, 7, 65], [1, 128, 43, 128]):
            assert sum(widths) == n
            pos = 0
            for w in widths:
                ctx.forward(which, toks[pos:pos + w], pos, want_logits=False)
                pos += w
            out.append(ctx.forward(which, toks[n:n + 7], n))
        for o in out[1:]:
            assert np.array_equal(out[0], o)
        om = oracle.Model(shapes[which], blobs[which], synth.DTYPE_BF16, 10000.0, 384)
        ref = om.forward(toks, 0)[n:]
        assert np.abs(out[0] - ref).max() <= TOL_BF16
    with pytest.raises(psd.PsdError):
        ctx.forward(0, toks[:64], 0)                      # logits only up to 32 tokens per pass
    with pytest.raises(psd.PsdError):
        ctx.forward(0, toks[:129], 0, want_logits=False)
    ctx.close()


WIDE = (ModelShape(2, 256, 4, 2, 352, 1000), ModelShape(2, 512, 8, 2, 2304, 1000), ModelShape(2, 1024, 8, 4, 2560, 1000))


def test_bf16_prompt_ingestion_in_512_token_passes_is_bit_exact():
    # passes of up to 512 tokens (several 128-column groups per launch, weights and operand shared through LDS) leave
    # the same KV cache, bit for bit, as 128-token, 32-token and ragged passes; row-tile counts that are not
    # multiples of 16, K ranges of one step, both K splits (8 and 16 ranges); and the logits match the oracle
    shapes = WIDE
    blobs = [synth.target_weights(s, 40 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    n = 700
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 768)
    toks = synth.tokens(11, 0, n + 5, 1000)
    for which in (1, 2):
        out = []
        for widths in ([512, 188], [128] * 5 + [60], [32] * 21 + [28], [300, 400], [1, 511, 129, 59]):
            assert sum(widths) == n
            pos = 0
            for w in widths:
                ctx.forward(which, toks[pos:pos + w], pos, want_logits=False)
                pos += w
            out.append(ctx.forward(which, toks[n:n + 5], n))
        for o in out[1:]:
            assert np.array_equal(out[0], o)
        om = oracle.Model(shapes[which], blobs[which], synth.DTYPE_BF16, 10000.0, 768)
        ref = om.forward(toks, 0)[n:]
        assert np.abs(out[0] - ref).max() <= TOL_BF16
    with pytest.raises(psd.PsdError):
        ctx.forward(0, toks[:129], 0, want_logits=False)   # a model too small for the widest kernel stays at 128
    with pytest.raises(psd.PsdError):
        ctx.forward(2, toks[:513], 0, want_logits=False)
    ctx.close()


def test_bf16_ingestion_at_page_split_and_pass_boundaries():
    # prompt lengths around the KV page (64), the attention key range (128) and the pass widths (128, 512):
    # the widest passes, 32-token passes and a ragged mix leave identical logits for the tokens that follow
    shapes = WIDE
    blobs = [synth.target_weights(s, 40 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 1100)
    toks = synth.tokens(12, 0, 1100, 1000)
    for n in (1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 191, 192, 193, 255, 256, 257, 511, 512, 513, 640, 1023, 1024, 1025):
        for which in (1, 2):
            rows = []
            for chunk in (512, 32, 100):
                pos = 0
                while pos < n:
                    w = min(chunk, n - pos)
                    ctx.forward(which, toks[pos:pos + w], pos, want_logits=False)
                    pos += w
                rows.append(ctx.forward(which, toks[n:n + 3], n))
            assert np.array_equal(rows[0], rows[1]) and np.array_equal(rows[0], rows[2]), (n, which)
    ctx.close()


def test_bf16_narrow_passes_across_the_merge_switch_are_bit_exact():
    # passes of up to 4 tokens let the o projection merge the attention partials itself while the context spans at
    # most a dozen key ranges, and hand the merge to a kernel of its own beyond that: on both sides of the switch
    # their logits have the bits of 11-token passes (which always use the separate kernel), and match the oracle
    shapes = MINI[0]
    blobs = [synth.target_weights(s, 20 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    n0, n1 = 1408, 1672
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 1700)
    toks = synth.tokens(13, 0, n1, 1000)
    for which in (0, 2):
        for pos in range(0, n0, 32):
            ctx.forward(which, toks[pos:pos + 32], pos, want_logits=False)
        pos, narrow, k = n0, [], 0
        while pos < n1:
            w = min((4, 1, 2, 3)[k % 4], n1 - pos)
            narrow.append(ctx.forward(which, toks[pos:pos + w], pos))
            pos += w
            k += 1
        narrow = np.concatenate(narrow)
        wide = np.concatenate([ctx.forward(which, toks[p:p + 11], p) for p in range(n0, n1, 11)])   # rolls the cache back to n0 first
        assert np.array_equal(narrow, wide)
        om = oracle.Model(shapes[which], blobs[which], synth.DTYPE_BF16, 10000.0, 1700)
        ref = om.forward(toks, 0)[n0:]
        assert np.abs(narrow - ref).max() <= TOL_BF16
    ctx.close()


def test_bf16_context_length_switches_are_bit_exact():
    # the launch shape depends on how far the context reaches (who merges the attention partials past 12 key ranges,
    # four query tiles per attention workgroup past 16): the same token at the same position has the same logits
    # bits when it is computed just before and just after each switch
    shapes = MINI[0]
    blobs = [synth.target_weights(s, 20 + i, synth.DTYPE_BF16, sigma=0.03) for i, s in enumerate(shapes)]
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 2100)
    toks = synth.tokens(14, 0, 2100, 1000)
    for which in (0, 2):
        pos = 0
        for edge, w in ((12 * 128, 4), (16 * 128, 11)):
            a = edge - 64 - w + 2            # a pass of w tokens from here is bounded by edge - 2 + ... : before the switch
            while pos < a:
                n = min(32, a - pos)
                ctx.forward(which, toks[pos:pos + n], pos, want_logits=False)
                pos += n
            before = ctx.forward(which, toks[a:a + w], a)                 # context bound a + 64 <= edge
            ctx.forward(which, toks[a:a + w - 1], a, want_logits=False)   # rolls back, keeps w - 1 of them
            after = ctx.forward(which, toks[a + w - 1:a + 2 * w - 1], a + w - 1)   # bound a + w - 1 + 64 > edge
            assert np.array_equal(before[w - 1], after[0]), (which, edge)
            pos = a + 2 * w - 1
    ctx.close()


def test_bf16_narrow_passes_with_long_k_ranges_are_bit_exact():
    # passes of up to 4 tokens read the operand of a down projection with long K ranges (here 12 and 13 K steps per
    # wave, odd and even, and a ragged split of K over the waves) and of every LM head from LDS instead of registers:
    # same bits as 5- and 11-token passes, which never do, and the logits match the oracle
    shapes = (ModelShape(2, 256, 4, 2, 6144, 1000), ModelShape(1, 512, 4, 4, 6560, 1000), ModelShape(1, 256, 4, 1, 6656, 1000))
    blobs = [synth.target_weights(s, 60 + i, synth.DTYPE_BF16, sigma=0.02) for i, s in enumerate(shapes)]
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 10000.0, 160)
    toks = synth.tokens(15, 0, 150, 1000)
    for which in range(3):
        pos, narrow, k = 0, [], 0
        while pos < 132:
            w = min((1, 4, 2, 3)[k % 4], 132 - pos)
            narrow.append(ctx.forward(which, toks[pos:pos + w], pos))
            pos += w
            k += 1
        narrow = np.concatenate(narrow)
        wide = np.concatenate([ctx.forward(which, toks[p:p + 11], p) for p in range(0, 132, 11)])
        five = np.concatenate([ctx.forward(which, toks[p:p + 5], p) for p in range(0, 130, 5)])
        assert np.array_equal(narrow, wide) and np.array_equal(narrow[:130], five)
        om = oracle.Model(shapes[which], blobs[which], synth.DTYPE_BF16, 10000.0, 160)
        assert np.abs(narrow - om.forward(toks[:132], 0)).max() <= TOL_BF16
    ctx.close()


def test_bf16_full_size_projection_variants_are_bit_exact():
    # one-layer stacks with the draft's, the qualifier's and the target's projection shapes (small vocabulary): these are the
    # shapes that select the per-shape GEMM variants (a wave's whole K range in one round of loads for the draft's q/k/v and
    # the qualifier's o projection, the windowed four-tile gate/up kernel, the seven-tile one): passes of 1, 5 and 11 tokens
    # take them, 20-token passes take the two-column-tile kernels, and all four give the same bits; the logits match the oracle
    shapes = (ModelShape(1, 2048, 32, 8, 8192, 512), ModelShape(1, 3072, 24, 8, 8192, 512), ModelShape(1, 4096, 32, 8, 14336, 512))
    blobs = [synth.target_weights(s, 70 + i, synth.DTYPE_BF16, sigma=0.02) for i, s in enumerate(shapes)]
    ctx = _ctx(shapes, blobs, synth.DTYPE_BF16, 500000.0, 128)
    toks = synth.tokens(16, 0, 60, 512)
    for which in range(3):
        runs = []
        for w in (1, 5, 11, 20):
            runs.append(np.concatenate([ctx.forward(which, toks[p:p + w], p) for p in range(0, 55 if w != 20 else 60, w)])[:55])
        for r in runs[1:]:
            assert np.array_equal(runs[0], r), which
        om = oracle.Model(shapes[which], blobs[which], synth.DTYPE_BF16, 500000.0, 128)
        assert np.abs(runs[0] - om.forward(toks[:55], 0)).max() <= TOL_BF16
    ctx.close()


def test_small_config_target_logits_sampled():
    """Config "small" shapes (bf16, vocab 32000): one teacher-forced 24-token pass per model against the oracle."""
    cfg = synth.CONFIGS["small"]
    d, q, t, prompt = synth.build_stack(cfg)
    shapes, blobs = (cfg.draft, cfg.qualifier, cfg.target), (d, q, t)
    ctx = _ctx(shapes, blobs, cfg.dtype, cfg.rope_theta, 64)
    toks = prompt[:24]
    for which in range(3):
        om = oracle.Model(shapes[which], blobs[which], cfg.dtype, cfg.rope_theta, 32)
        ref = om.forward(toks, 0)
        got = np.concatenate([ctx.forward(which, toks[:13], 0), ctx.forward(which, toks[13:24], 13)])
        err = np.abs(got - ref).max()
        print(f"model {which}: max |logit err| = {err:.3e}, logit std = {ref.std():.3f}", flush=True)
        assert err <= TOL_BF16
    ctx.close()


def test_full_width_layer_at_the_long_context_matches_the_oracle():
    """One layer of the 8B shape (d 4096, 32 query / 8 KV heads of 128) over a context of 4.2 K tokens, the context of the
    long-prompt configuration (33 key ranges, the 48-range launch bucket): logits of a 1-token, an 11-token and a
    17-token pass against the oracle's forward over the same 4229 tokens."""
    shape = ModelShape(1, 4096, 32, 8, 512, 512)
    blob = synth.target_weights(shape, 41, synth.DTYPE_BF16, sigma=0.02)
    n0, widths = 4200, (1, 11, 17)
    n = n0 + sum(widths)
    ms = n + 3
    toks = synth.tokens(43, 0, n, shape.vocab)
    ctx = _ctx((shape,) * 3, (blob,) * 3, synth.DTYPE_BF16, 500000.0, ms, k1=5, k2=16)
    pos = 0
    while pos < n0:
        w = min(512, n0 - pos)
        ctx.forward(2, toks[pos:pos + w], pos, want_logits=False)
        pos += w
    got = []
    for w in widths:
        got.append(ctx.forward(2, toks[pos:pos + w], pos))
        pos += w
    got = np.concatenate(got)
    ctx.close()
    om = oracle.Model(shape, blob, synth.DTYPE_BF16, 500000.0, ms)
    om.forward(toks[:n0], 0, want_logits=False)
    ref = om.forward(toks[n0:], n0)
    err = float(np.abs(got - ref).max())
    print(f"full-width layer at {n0} tokens of context: max |logit err| {err:.3e}, logit std {ref.std():.3f}", flush=True)
    assert ref.std() > 0.05          # the comparison is not between two flat rows
    assert err <= TOL_BF16


def test_forward_argument_errors(tiny_stack):
    cfg, d, q, t, prompt = tiny_stack
    ctx = _ctx((cfg.draft, cfg.qualifier, cfg.target), (d, q, t), cfg.dtype, cfg.rope_theta, 48)
    with pytest.raises(psd.PsdError):
        ctx.forward(0, [cfg.target.vocab], 0)            # token out of range
    with pytest.raises(psd.PsdError):
        ctx.forward(0, [1, 2], 5)                        # gap in the cache
    with pytest.raises(psd.PsdError):
        ctx.forward(0, np.zeros(33, np.int32), 0)        # too wide
    with pytest.raises(psd.PsdError):
        ctx.forward(3, [1], 0)
    ctx.forward(0, np.zeros(32, np.int32), 0, want_logits=False)
    with pytest.raises(psd.PsdError):
        ctx.forward(0, np.zeros(32, np.int32), 32)       # past max_seq
    ctx.close()
    bad = psd.ModelDesc(2, 64, 4, 2, 256, 100, 10000.0, psd.F32, d)   # vocab differs from the others
    with pytest.raises(psd.PsdError):
        psd.Context(bad, _desc(cfg.qualifier, q, cfg.dtype, 1e4), _desc(cfg.target, t, cfg.dtype, 1e4), 0.1, 0.1, 4, 8, 64)
