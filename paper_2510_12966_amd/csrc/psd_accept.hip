// ACCEPT stage of one verify pass on the GPU: vocabulary-wide softmax of the verifier and proposer
// rows, Jensen-Shannon divergence per position, threshold / coin / first-reject scan and the
// replacement draw (Sections 3.1-3.2 and the fallback rule named in Section 3.4).
//
// Three kernels, all bandwidth-shaped (each logit is read with coalesced 16-byte loads):
//   accept_lse      per (trial, position, chunk): running max and sum of exponentials of both rows
//   accept_div      per (trial, position, chunk): divergence partial, race partials, p(x), q(x)
//   accept_decide   per trial: fixed-order reduction of the partials, coins, scan, token choice
// The second sweep over the rows normally hits L2 / Infinity Cache because it follows the first
// one immediately.  No atomics: every partial has its own slot, reductions run in index order.
#include "psd_device.h"
#include "psd_host.h"

namespace psd {

constexpr int kAccThreads = 256;
constexpr int kQuadsPerThread = kAcceptChunk / 4 / kAccThreads;  // 4

struct LsePart { float mp, sp, mq, sq; };
struct DivPart { float jsd; float key; int idx; float key_fb; int idx_fb; int pad0, pad1, pad2; };
struct TokProb { float px, qx; };

// loads entries v .. v+3 of a row (entries >= V read as -inf: they carry no probability)
__device__ inline void load4(const float* row, int v, int V, bool vec, float out[4]) {
    if (vec && v + 3 < V) {
        float4 t = *reinterpret_cast<const float4*>(row + v);
        out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = (v + e < V) ? row[v + e] : -INFINITY;
    }
}

struct AcceptShape {
    const float* lp;  // [B][k+1][V]
    const float* lq;  // [B][k][V]
    const int32_t* tokens;  // [B][k]
    int k, V, nch;
    float inv_temp;
};

__global__ __launch_bounds__(kAccThreads) void accept_lse(AcceptShape s, LsePart* parts, TokProb* tokprob) {
    __shared__ float sm[4];
    const int ch = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const float* prow = s.lp + ((size_t)b * (s.k + 1) + i) * s.V;
    const bool has_q = i < s.k;
    const float* qrow = has_q ? s.lq + ((size_t)b * s.k + i) * s.V : prow;
    const bool vec = (s.V & 3) == 0;
    float a[kQuadsPerThread][4], c[kQuadsPerThread][4];
    float mp = -INFINITY, mq = -INFINITY;
#pragma unroll
    for (int j = 0; j < kQuadsPerThread; ++j) {
        int v = ch * kAcceptChunk + 4 * (threadIdx.x + kAccThreads * j);
        load4(prow, v, s.V, vec, a[j]);
        if (has_q) load4(qrow, v, s.V, vec, c[j]);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            a[j][e] *= s.inv_temp;
            mp = fmaxf(mp, a[j][e]);
            if (has_q) { c[j][e] *= s.inv_temp; mq = fmaxf(mq, c[j][e]); }
        }
    }
    mp = block_max<4>(mp, sm);
    if (has_q) mq = block_max<4>(mq, sm);
    float sp = 0.f, sq = 0.f;
#pragma unroll
    for (int j = 0; j < kQuadsPerThread; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sp += expf(a[j][e] - mp);  // exp(-inf) = 0 for padding
            if (has_q) sq += expf(c[j][e] - mq);
        }
    sp = block_sum<4>(sp, sm);
    if (has_q) sq = block_sum<4>(sq, sm);
    if (threadIdx.x == 0) {
        parts[((size_t)b * (s.k + 1) + i) * s.nch + ch] = LsePart{mp, sp, has_q ? mq : 0.f, has_q ? sq : 1.f};
        // default for a proposed id outside the vocabulary: probability 0 under the verifier -> rejected
        if (ch == 0) tokprob[(size_t)b * (s.k + 1) + i] = TokProb{0.f, 1.f};
    }
}

// log-sum-exp of a row from its chunk partials, summed in chunk order
__device__ inline void row_lse(const LsePart* parts, int nch, float& lse_p, float& lse_q) {
    float mp = -INFINITY, mq = -INFINITY;
    for (int c = 0; c < nch; ++c) { mp = fmaxf(mp, parts[c].mp); mq = fmaxf(mq, parts[c].mq); }
    float sp = 0.f, sq = 0.f;
    for (int c = 0; c < nch; ++c) { sp += parts[c].sp * expf(parts[c].mp - mp); sq += parts[c].sq * expf(parts[c].mq - mq); }
    lse_p = mp + logf(sp);
    lse_q = mq + logf(sq);
}

__global__ __launch_bounds__(kAccThreads) void accept_div(AcceptShape s, const LsePart* lse_parts, DivPart* parts,
                                                          TokProb* tokprob, uint64_t seed, uint32_t position0,
                                                          uint32_t stage) {
    __shared__ float sm[4];
    __shared__ KeyIdx smk[4];
    __shared__ float s_lse[2];
    const int ch = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const size_t row_id = (size_t)b * (s.k + 1) + i;
    const float* prow = s.lp + row_id * s.V;
    const bool has_q = i < s.k;
    const float* qrow = has_q ? s.lq + ((size_t)b * s.k + i) * s.V : prow;
    const bool vec = (s.V & 3) == 0;
    if (threadIdx.x == 0) {
        float lp_, lq_;
        row_lse(lse_parts + row_id * s.nch, s.nch, lp_, lq_);
        s_lse[0] = lp_; s_lse[1] = lq_;
    }
    __syncthreads();
    const float lse_p = s_lse[0], lse_q = s_lse[1];
    const uint64_t sd = seed + (uint64_t)b;
    const uint32_t pos = position0 + (uint32_t)i;
    const int x = has_q ? s.tokens[(size_t)b * s.k + i] : -1;
    float jsd = 0.f;
    // residual keys are positive; keys of the bonus race are logs and can have any sign
    KeyIdx best{has_q ? -1.f : -INFINITY, 0x7fffffff}, best_fb{-1.f, 0x7fffffff};
#pragma unroll
    for (int j = 0; j < kQuadsPerThread; ++j) {
        const int v = ch * kAcceptChunk + 4 * (threadIdx.x + kAccThreads * j);
        if (v >= s.V) continue;
        float a[4], c[4], u[4];
        load4(prow, v, s.V, vec, a);
        if (has_q) {
            load4(qrow, v, s.V, vec, c);
            draw4(sd, (uint32_t)(v >> 2), pos, DRAW_RESAMPLE, stage, u);
        } else {
            draw4(sd, (uint32_t)(v >> 2), pos, DRAW_SAMPLE, 0u, u);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (v + e >= s.V) continue;
            const float za = a[e] * s.inv_temp - lse_p;  // ln p
            const float p = expf(za);
            const float E = -logf(u[e]);
            if (has_q) {
                const float zb = c[e] * s.inv_temp - lse_q;  // ln q
                const float q = expf(zb);
                // ln(p/m) = ln 2 - softplus(zb - za), ln(q/m) = ln 2 - softplus(za - zb)
                const float t = zb - za, at = fabsf(t);
                const float l1 = log1pf(expf(-at));
                const float sp_pos = at + l1, sp_neg = l1;  // softplus(|t|), softplus(-|t|)
                const float sp_t = t >= 0.f ? sp_pos : sp_neg, sp_mt = t >= 0.f ? sp_neg : sp_pos;
                float term = 0.f;
                if (p > 0.f) term += p * (0.69314718055994531f - sp_t);
                if (q > 0.f) term += q * (0.69314718055994531f - sp_mt);
                jsd += 0.5f * term;
                const float r = p - q;
                if (r > 0.f) best = better(best, KeyIdx{r / E, v + e});
                if (p > 0.f) best_fb = better(best_fb, KeyIdx{p / E, v + e});
                if (v + e == x) tokprob[row_id] = TokProb{p, q};
            } else {
                // bonus row: race on ln p - ln E (same argmax as p / E)
                best = better(best, KeyIdx{za - logf(E), v + e});
            }
        }
    }
    jsd = block_sum<4>(jsd, sm);
    best = block_best<4>(best, smk);
    best_fb = block_best<4>(best_fb, smk);
    if (threadIdx.x == 0) parts[row_id * s.nch + ch] = DivPart{jsd, best.key, best.idx, best_fb.key, best_fb.idx, 0, 0, 0};
}

__global__ __launch_bounds__(64) void accept_decide(AcceptShape s, const DivPart* parts, const TokProb* tokprob,
                                                    float T, uint64_t seed, uint32_t position0, uint32_t stage,
                                                    int take_bonus, AcceptOut* out, float* div_out) {
    __shared__ float s_div[PSD_MAX_WIDTH];
    __shared__ int s_tok[PSD_MAX_WIDTH + 1];
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    if (i <= s.k) {
        const DivPart* pr = parts + ((size_t)b * (s.k + 1) + i) * s.nch;
        float d = 0.f;
        const bool bonus_row = i == s.k;
        KeyIdx best{bonus_row ? -INFINITY : -1.f, 0x7fffffff}, fb{-1.f, 0x7fffffff};
        for (int c = 0; c < s.nch; ++c) {
            d += pr[c].jsd;
            best = better(best, KeyIdx{pr[c].key, pr[c].idx});
            fb = better(fb, KeyIdx{pr[c].key_fb, pr[c].idx_fb});
        }
        // no residual mass at all (cannot happen in exact arithmetic): draw from p instead
        if (!bonus_row && !(best.key > 0.f)) best = fb;
        s_tok[i] = best.idx == 0x7fffffff ? -1 : best.idx;
        if (i < s.k) {
            s_div[i] = d;
            if (div_out) div_out[(size_t)b * s.k + i] = d;
        }
    }
    __syncthreads();
    if (i == 0) {
        const uint64_t sd = seed + (uint64_t)b;
        int n = 0, fuzzy = 0;
        for (; n < s.k; ++n) {
            if (s_div[n] <= T) { ++fuzzy; continue; }
            U4 r = philox4x32_10(U4{0u, position0 + (uint32_t)n, DRAW_COIN, stage}, (uint32_t)sd, (uint32_t)(sd >> 32));
            const float u = u01(r.x);
            const TokProb tp = tokprob[(size_t)b * (s.k + 1) + n];
            if (u * tp.qx < tp.px) continue;  // u < p(x)/q(x)
            break;
        }
        AcceptOut o;
        o.n_accepted = n;
        o.n_fuzzy = fuzzy;
        o.pad = 0;
        o.next_token = (n < s.k) ? s_tok[n] : (take_bonus ? s_tok[s.k] : -1);
        out[b] = o;
    }
}

static inline size_t align16(size_t n) { return (n + 15) & ~(size_t)15; }

size_t accept_workspace_bytes(int n_trials, int k, int vocab) {
    size_t rows = (size_t)n_trials * (k + 1), nch = accept_chunks(vocab);
    return align16(rows * nch * sizeof(LsePart)) + align16(rows * nch * sizeof(DivPart)) + align16(rows * sizeof(TokProb));
}

int accept_launch(const float* logits_p, const float* logits_q, const int32_t* tokens, int n_trials, int k,
                  int vocab, float T, float temperature, uint64_t seed, uint32_t position0, uint32_t stage,
                  int take_bonus, AcceptOut* out, float* div_out, void* workspace, size_t workspace_bytes,
                  hipStream_t stream, char* errbuf) {
    if (!logits_p || (k > 0 && (!logits_q || !tokens)) || !out || !workspace)
        PSD_FAIL(PSD_EINVAL, errbuf, "accept: null pointer");
    if (k < 0 || k > PSD_MAX_WIDTH || vocab < 1 || n_trials < 1 || n_trials > 65535)
        PSD_FAIL(PSD_EINVAL, errbuf, "accept: k=%d vocab=%d n_trials=%d out of range", k, vocab, n_trials);
    if (!(T >= 0.f) || !(temperature > 0.f)) PSD_FAIL(PSD_EINVAL, errbuf, "accept: T=%g temperature=%g", T, temperature);
    if (workspace_bytes < accept_workspace_bytes(n_trials, k, vocab))
        PSD_FAIL(PSD_ENOMEM, errbuf, "accept: workspace %zu < %zu bytes", workspace_bytes,
                 accept_workspace_bytes(n_trials, k, vocab));
    if (((uintptr_t)workspace & 15) || ((uintptr_t)logits_p & 15) || ((uintptr_t)logits_q & 15))
        PSD_FAIL(PSD_EINVAL, errbuf, "accept: logits and workspace must be 16-byte aligned");
    const int nch = accept_chunks(vocab);
    const size_t rows = (size_t)n_trials * (k + 1);
    LsePart* lse = (LsePart*)workspace;
    DivPart* dv = (DivPart*)((char*)lse + align16(rows * nch * sizeof(LsePart)));
    TokProb* tp = (TokProb*)((char*)dv + align16(rows * nch * sizeof(DivPart)));
    AcceptShape s{logits_p, logits_q, tokens, k, vocab, nch, 1.0f / temperature};
    dim3 grid(nch, k + 1, n_trials);
    accept_lse<<<grid, kAccThreads, 0, stream>>>(s, lse, tp);
    accept_div<<<grid, kAccThreads, 0, stream>>>(s, lse, dv, tp, seed, position0, stage);
    accept_decide<<<n_trials, 64, 0, stream>>>(s, dv, tp, T, seed, position0, stage, take_bonus, out, div_out);
    PSD_HIP(hipGetLastError(), errbuf);
    return PSD_OK;
}

// ---- fresh samples (draft proposals) ---------------------------------------------------------
// score_v = z_v / temperature - ln(-ln u_v); token = argmax (the exponential race in log form, so no
// normalisation pass is needed)
__global__ __launch_bounds__(kAccThreads) void sample_partial(const float* logits, int V, int nch, float inv_temp,
                                                              uint64_t seed, uint32_t position0,
                                                              const SampleCtl* ctl, KeyIdx* parts) {
    __shared__ KeyIdx smk[4];
    const int ch = blockIdx.x, r = blockIdx.y;
    int row0 = 0;
    if (ctl) { seed = ctl->seed; position0 = (uint32_t)ctl->position; row0 = ctl->row; }
    const float* row = logits + (size_t)(row0 + r) * V;
    const bool vec = (V & 3) == 0;
    const uint32_t pos = position0 + (uint32_t)r;
    KeyIdx best{-INFINITY, 0x7fffffff};
#pragma unroll
    for (int j = 0; j < kQuadsPerThread; ++j) {
        const int v = ch * kAcceptChunk + 4 * (threadIdx.x + kAccThreads * j);
        if (v >= V) continue;
        float a[4], u[4];
        load4(row, v, V, vec, a);
        draw4(seed, (uint32_t)(v >> 2), pos, DRAW_SAMPLE, 0u, u);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (v + e < V) best = better(best, KeyIdx{a[e] * inv_temp - logf(-logf(u[e])), v + e});
    }
    best = block_best<4>(best, smk);
    if (threadIdx.x == 0) parts[(size_t)r * nch + ch] = best;
}

__global__ void sample_final(const KeyIdx* parts, int nch, int32_t* tokens_out) {
    const int r = blockIdx.x;
    if (threadIdx.x == 0) {
        KeyIdx best{-INFINITY, 0x7fffffff};
        for (int c = 0; c < nch; ++c) best = better(best, parts[(size_t)r * nch + c]);
        tokens_out[r] = best.idx;
    }
}

int sample_launch(const float* logits, int n_rows, int vocab, float temperature, uint64_t seed, uint32_t position0,
                  const SampleCtl* ctl, int32_t* tokens_out, void* partial, hipStream_t stream, char* errbuf) {
    if (!logits || !tokens_out || !partial) PSD_FAIL(PSD_EINVAL, errbuf, "sample: null pointer");
    if (n_rows < 1 || n_rows > 65535 || vocab < 1 || !(temperature > 0.f))
        PSD_FAIL(PSD_EINVAL, errbuf, "sample: n_rows=%d vocab=%d temperature=%g", n_rows, vocab, temperature);
    if ((uintptr_t)logits & 15) PSD_FAIL(PSD_EINVAL, errbuf, "sample: logits must be 16-byte aligned");
    const int nch = accept_chunks(vocab);
    sample_partial<<<dim3(nch, n_rows), kAccThreads, 0, stream>>>(logits, vocab, nch, 1.0f / temperature, seed,
                                                                   position0, ctl, (KeyIdx*)partial);
    sample_final<<<n_rows, 64, 0, stream>>>((const KeyIdx*)partial, nch, tokens_out);
    PSD_HIP(hipGetLastError(), errbuf);
    return PSD_OK;
}

}  // namespace psd

// ---- C ABI --------------------------------------------------------------------------------------
using namespace psd;

extern "C" size_t psd_accept_workspace_bytes(int32_t n_trials, int32_t k, int32_t vocab) {
    if (n_trials < 1 || k < 0 || vocab < 1) return 0;
    return accept_workspace_bytes(n_trials, k, vocab) + align16((size_t)n_trials * sizeof(AcceptOut));
}

__global__ void unpack_accept(const AcceptOut* o, int n, int32_t* n_accepted, int32_t* next_token) {
    int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b < n) { n_accepted[b] = o[b].n_accepted; next_token[b] = o[b].next_token; }
}

extern "C" int psd_accept_batch(const float* logits_p, const float* logits_q, const int32_t* tokens,
                                int32_t n_trials, int32_t k, int32_t vocab, float T, float temperature,
                                uint64_t seed, uint32_t position0, uint32_t stage, int32_t take_bonus,
                                int32_t* n_accepted, int32_t* next_token, float* div_out, void* workspace,
                                size_t workspace_bytes, void* stream) {
    char* err = tls_error();
    if (!n_accepted || !next_token || !workspace) PSD_FAIL(PSD_EINVAL, err, "psd_accept_batch: null pointer");
    if (n_trials < 1 || k < 0 || vocab < 1) PSD_FAIL(PSD_EINVAL, err, "psd_accept_batch: bad sizes");
    if (stage != 1 && stage != 2) PSD_FAIL(PSD_EINVAL, err, "psd_accept_batch: stage must be 1 or 2");
    if (workspace_bytes < psd_accept_workspace_bytes(n_trials, k, vocab))
        PSD_FAIL(PSD_ENOMEM, err, "psd_accept_batch: workspace %zu < %zu bytes", workspace_bytes,
                 psd_accept_workspace_bytes(n_trials, k, vocab));
    const size_t inner = accept_workspace_bytes(n_trials, k, vocab);
    AcceptOut* out = (AcceptOut*)((char*)workspace + inner);
    hipStream_t st = (hipStream_t)stream;
    int rc = accept_launch(logits_p, logits_q, tokens, n_trials, k, vocab, T, temperature, seed, position0, stage,
                           take_bonus, out, div_out, workspace, inner, st, err);
    if (rc != PSD_OK) return rc;
    unpack_accept<<<(n_trials + 255) / 256, 256, 0, st>>>(out, n_trials, n_accepted, next_token);
    PSD_HIP(hipGetLastError(), err);
    return PSD_OK;
}
