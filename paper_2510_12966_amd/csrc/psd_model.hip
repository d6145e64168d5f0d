// Decoder forward pass for gfx950: kernels and their launcher.
//
// Every projection of a pass is a weight-streaming skinny GEMM Y[c][n] = sum_k W[n][k] X[c][k] with
// c < w <= 32 tokens.  bf16 weights are stored re-tiled in the order the MFMA consumes them, so a wave
// reads one contiguous 1 KiB block per (16 rows x 32 k) step; the activations are pre-split into
// bf16 hi + lo parts (x = hi + lo to 2^-17) in the matching B-operand order, so the product keeps
// fp32-like accuracy on the activation side and every output column depends on its own input column
// only: a token's result does not change with the width of the pass it is computed in.
// fp32 models (the tiny plumbing configuration) use plain VALU kernels.
#include "psd_device.h"
#include "psd_model.h"

#include <string.h>

#include <algorithm>

namespace psd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

enum { EPI_STORE = 0, EPI_RESID = 1, EPI_LOGITS = 2 };

// ---- operand packing ----------------------------------------------------------------------------
// GEMM input X[c][f] (c < 16 CT tokens, f < K features), bf16 path: [K/32][CT col tiles][hi, lo][64 lanes][8]
// (CT = 2 for passes of up to 32 tokens, 32 for the passes of up to 512 tokens that ingest a prompt),
// lane = ((f % 32) / 8) * 16 + c % 16: exactly the B operand of v_mfma_f32_16x16x32_bf16.
// fp32 path: plain rows [c][K].
template <bool BF16, int CT = 2>
__device__ inline void pack_store(void* xb, int K, int c, int f, float v) {
    if constexpr (BF16) {
        const int ks = f >> 5, g = (f & 31) >> 3, e = f & 7, t = c >> 4, cc = c & 15;
        uint16_t* p = (uint16_t*)xb;
        const size_t base = ((((size_t)ks * CT + t) * 2) * 64 + g * 16 + cc) * 8 + e;
        const uint16_t hi = f32_to_bf16(v);
        p[base] = hi;
        p[base + 64 * 8] = f32_to_bf16(v - bf16_to_f32(hi));
    } else {
        ((float*)xb)[(size_t)c * K + f] = v;
    }
}

// ---- small kernels ------------------------------------------------------------------------------
template <bool BF16>
__global__ __launch_bounds__(256) void embed_rows(const void* embed, const PassDesc* desc, float* x, int d, int V) {
    const int c = blockIdx.x;
    if (c >= desc->w) return;
    int tok = desc->tok[c];
    tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);  // ids are validated on the host; never index outside the table
    for (int f = threadIdx.x; f < d; f += 256) {
        float v;
        if constexpr (BF16) {
            const int KS = d >> 5;
            const size_t idx = ((((size_t)(tok >> 4) * KS + (f >> 5)) * 64) + ((f & 31) >> 3) * 16 + (tok & 15)) * 8 + (f & 7);
            v = bf16_to_f32(((const uint16_t*)embed)[idx]);
        } else {
            v = ((const float*)embed)[(size_t)tok * d + f];
        }
        x[(size_t)c * d + f] = v;
    }
}

template <bool BF16>
__global__ __launch_bounds__(256) void rmsnorm_pack(const float* x, const float* gain, const PassDesc* desc, void* xb,
                                                    int d, float eps) {
    __shared__ float sm[4];
    const int c = blockIdx.x;
    if (c >= desc->w) return;
    const float* row = x + (size_t)c * d;
    float ss = 0.f;
    for (int f = threadIdx.x; f < d; f += 256) ss += row[f] * row[f];
    ss = block_sum<4>(ss, sm);
    const float r = rsqrtf(ss / (float)d + eps);
    for (int f = threadIdx.x; f < d; f += 256) pack_store<BF16>(xb, d, c, f, row[f] * r * gain[f]);
}

template <bool BF16>
__global__ __launch_bounds__(256) void swiglu_pack(const float* gu, const PassDesc* desc, void* xb, int F) {
    const int c = blockIdx.x;
    if (c >= desc->w) return;
    const int f = blockIdx.y * 256 + threadIdx.x;
    if (f >= F) return;
    const float g = gu[(size_t)c * 2 * F + f], u = gu[(size_t)c * 2 * F + F + f];
    pack_store<BF16>(xb, F, c, f, g / (1.f + expf(-g)) * u);
}

__global__ void rope_table(float2* tab, int max_seq, int half, double theta) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= max_seq * half) return;
    const int pos = i / half, j = i % half;
    const double ang = (double)pos * pow(theta, -2.0 * j / (2.0 * half));
    tab[i] = make_float2((float)cos(ang), (float)sin(ang));
}

__global__ void bf16_to_f32_vec(const uint16_t* in, float* out, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) out[i] = bf16_to_f32(in[i]);
}

// row-major bf16 [N][K] -> MFMA A-operand tiles [Npad/16][K/32][64][8]; rows >= N become zeros.
// mode 1 (fused q/k/v projection): inside every head of `hd` rows, tile row 2e / 2e+1 of tile t holds the rotary
//   pair (j, j + hd/2), j = 8 t + e, so that one lane of the GEMM result owns both halves of a pair.
// mode 2 (fused gate/up projection, `hd` = F): tile row 2e / 2e+1 of tile t holds gate / up row 8 t + e.
__global__ __launch_bounds__(256) void tile_bf16(const uint4* src, uint4* dst, int N, int K, size_t n_chunks, int mode,
                                                 int hd) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_chunks) return;
    const int KS = K >> 5;
    const int lane = (int)(i & 63);
    const size_t t = i >> 6;
    const int ks = (int)(t % KS);
    const int tile = (int)(t / KS);
    int n = tile * 16 + (lane & 15);
    const int k = ks * 32 + (lane >> 4) * 8;
    if (mode == 1) {
        const int head = n / hd, within = n % hd, tt = within >> 4, tr = within & 15;
        n = head * hd + tt * 8 + (tr >> 1) + (tr & 1) * (hd >> 1);
    } else if (mode == 2) {
        const int tr = n & 15;
        n = (tr & 1) * hd + tile * 8 + (tr >> 1);
    }
    dst[i] = n < N ? src[((size_t)n * K + k) >> 3] : make_uint4(0, 0, 0, 0);
}

// ---- rotary embedding + KV append ------------------------------------------------------------------
template <typename KVT>
__device__ inline void kv_store(KVT* p, float v);
template <>
__device__ inline void kv_store<float>(float* p, float v) { *p = v; }
template <>
__device__ inline void kv_store<uint16_t>(uint16_t* p, float v) { *p = f32_to_bf16(v); }
template <typename KVT>
__device__ inline float kv_load(const KVT* p);
template <>
__device__ inline float kv_load<float>(const float* p) { return *p; }
template <>
__device__ inline float kv_load<uint16_t>(const uint16_t* p) { return bf16_to_f32(*p); }

// bf16 models keep every K and V element as a bf16 hi + lo pair (value = hi + lo to 2^-17) in four planes per
// (page, layer, kv head): K hi, K lo, V hi, V lo, each of kPage x hd elements.  One bf16 rounding of the
// cache alone would put ~0.1 % * sqrt(layers) of noise on the logits, which at 32 layers is past the tolerance.
__device__ inline size_t kv_plane(int page, int layer, int L, int g, int KV, int plane, int hd) {
    return ((((size_t)page * L + layer) * KV + g) * 4 + plane) * (size_t)kPage * hd;
}

// Inside a plane the elements sit in the order the attention MFMAs consume them, so that a wave's operand load is one
// contiguous block (1 KiB for K, 512 bytes for V) instead of sixteen strided pieces:
//   K planes: A-operand tiles of v_mfma_f32_16x16x32_bf16, [slot / 16][hd / 32][64 lanes][8], lane = (dim % 32) / 8 * 16 + slot % 16
//   V planes: B-operand tiles of v_mfma_f32_16x16x16_bf16, [hd / 16][slot / 16][64 lanes][4], lane = (slot % 16) / 4 * 16 + dim % 16
__device__ inline int kv_k_off(int slot, int dim, int hd) {
    return ((((slot >> 4) * (hd >> 5) + (dim >> 5)) * 64 + ((dim & 31) >> 3) * 16 + (slot & 15)) << 3) + (dim & 7);
}
__device__ inline int kv_v_off(int slot, int dim) {
    return ((((dim >> 4) * (kPage >> 4) + (slot >> 4)) * 64 + ((slot & 15) >> 2) * 16 + (dim & 15)) << 2) + (slot & 3);
}

__device__ inline size_t kv_base(int page, int layer, int L, int g, int KV, int which, int hd) {
    return ((((size_t)page * L + layer) * KV + g) * 2 + which) * (size_t)kPage * hd;
}

// grid (wmax, H + 2 KV), block hd/2: q heads are rotated in place, k heads rotated into the cache, v copied
template <typename KVT>
__global__ void rope_kv(float* qkv, const PassDesc* desc, const float2* rope, KVT* kv, const int32_t* page_table,
                        int layer, int L, int H, int KV, int hd, int nqkv) {
    const int c = blockIdx.x, h = blockIdx.y, i = threadIdx.x, half = hd >> 1;
    if (c >= desc->w) return;
    const int pos = desc->pos0 + c;
    float* v = qkv + (size_t)c * nqkv + (size_t)h * hd;
    const int page = page_table[pos / kPage], slot = pos % kPage;
    if (h < H + KV) {
        const float2 cs = rope[(size_t)pos * half + i];
        const float a = v[i], b = v[i + half];
        const float ra = a * cs.x - b * cs.y, rb = b * cs.x + a * cs.y;
        if (h < H) {
            v[i] = ra;
            v[i + half] = rb;
        } else {
            KVT* dst = kv + kv_base(page, layer, L, h - H, KV, 0, hd) + (size_t)slot * hd;
            kv_store<KVT>(dst + i, ra);
            kv_store<KVT>(dst + i + half, rb);
        }
    } else {
        KVT* dst = kv + kv_base(page, layer, L, h - H - KV, KV, 1, hd) + (size_t)slot * hd;
        kv_store<KVT>(dst + i, v[i]);
        kv_store<KVT>(dst + i + half, v[i + half]);
    }
}

// ---- attention -------------------------------------------------------------------------------------
// grid (H, nsplit_max), 256 threads.  A workgroup owns one query head and one absolute key range
// [split * 128, split * 128 + 128); wave j takes the queries c = j, j + 4, ...  Partial result per
// (split, query, head): running max m, sum l and the un-normalised output, merged by attn_combine in
// split order.  The arithmetic for a query at a given position is the same whatever the pass width.
template <typename KVT>
__global__ __launch_bounds__(256) void attn_partial(const float* qkv, const PassDesc* desc, const KVT* kv,
                                                    const int32_t* page_table, float* part, int layer, int L, int H,
                                                    int KV, int hd, int nqkv) {
    extern __shared__ float lds[];
    const int h = blockIdx.x, split = blockIdx.y;
    const int w = desc->w, pos0 = desc->pos0;
    const int key0 = split * kAttnSplit, kv_max = pos0 + w;
    if (key0 >= kv_max) return;
    const int nkeys = min(kAttnSplit, kv_max - key0);
    const int g = h / (H / KV), ld = hd + 1;
    float* Ks = lds;                       // [128][hd + 1]
    float* Vs = Ks + kAttnSplit * ld;      // [128][hd + 1]
    float* qs = Vs + kAttnSplit * ld;      // [4][hd]
    float* ps = qs + 4 * hd;               // [4][128]
    for (int idx = threadIdx.x; idx < nkeys * hd; idx += 256) {
        const int j = idx / hd, i = idx % hd, pos = key0 + j;
        const int page = page_table[pos / kPage], slot = pos % kPage;
        Ks[j * ld + i] = kv_load<KVT>(kv + kv_base(page, layer, L, g, KV, 0, hd) + (size_t)slot * hd + i);
        Vs[j * ld + i] = kv_load<KVT>(kv + kv_base(page, layer, L, g, KV, 1, hd) + (size_t)slot * hd + i);
    }
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const float scale = rsqrtf((float)hd);
    float* q = qs + wave * hd;
    float* p = ps + wave * kAttnSplit;
    for (int c = wave; c < w; c += 4) {
        const int visible = min(nkeys, pos0 + c + 1 - key0);
        float* out = part + (((size_t)split * kCols + c) * H + h) * (hd + 2);
        if (visible <= 0) {
            if (lane == 0) { out[0] = -INFINITY; out[1] = 0.f; }
            continue;
        }
        for (int i = lane; i < hd; i += 64) q[i] = qkv[(size_t)c * nqkv + (size_t)h * hd + i];
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        float s[2];
#pragma unroll
        for (int r = 0; r < 2; ++r) {
            const int j = lane + 64 * r;
            float acc = 0.f;
            if (j < visible)
                for (int i = 0; i < hd; ++i) acc += q[i] * Ks[j * ld + i];
            s[r] = j < visible ? acc * scale : -INFINITY;
        }
        const float m = wave_max(fmaxf(s[0], s[1]));
        const float p0 = expf(s[0] - m), p1 = expf(s[1] - m);  // exp(-inf) = 0 for masked keys
        const float l = wave_sum(p0 + p1);
        p[lane] = p0;
        p[lane + 64] = p1;
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        for (int i = lane; i < hd; i += 64) {
            float acc = 0.f;
            for (int j = 0; j < visible; ++j) acc += p[j] * Vs[j * ld + i];
            out[2 + i] = acc;
        }
        if (lane == 0) { out[0] = m; out[1] = l; }
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
    }
}

// grid (wmax, H), block hd: merges the split partials in order and writes the O-projection's input operand
template <bool BF16>
__global__ void attn_combine_pack(const float* part, const PassDesc* desc, void* xb, int H, int hd) {
    const int c = blockIdx.x, h = blockIdx.y, i = threadIdx.x;
    if (c >= desc->w) return;
    const int nsp = (desc->pos0 + c + kAttnSplit) / kAttnSplit;  // splits holding keys <= pos0 + c
    float M = -INFINITY;
    for (int s = 0; s < nsp; ++s) M = fmaxf(M, part[(((size_t)s * kCols + c) * H + h) * (hd + 2)]);
    float Lsum = 0.f, o = 0.f;
    for (int s = 0; s < nsp; ++s) {
        const float* pr = part + (((size_t)s * kCols + c) * H + h) * (hd + 2);
        const float f = expf(pr[0] - M);
        Lsum += pr[1] * f;
        o += pr[2 + i] * f;
    }
    pack_store<BF16>(xb, H * hd, c, h * hd + i, o / Lsum);
}

// Merge of the split partials of one (token, head): the same arithmetic wherever it is done, so that a token's
// attention output has the same bits whichever kernel merges it.  Returns the normalised output of head dims
// i .. i + N - 1.
template <int N>
__device__ inline void attn_merge(const float* part, int nsp, int c, int head, int H, int hd, int i, float out[N]) {
    const size_t stride = (size_t)kCols * H * (hd + 2);
    const float* p0 = part + ((size_t)c * H + head) * (hd + 2);
    float M = -INFINITY, Lsum = 0.f;
#pragma unroll
    for (int e = 0; e < N; ++e) out[e] = 0.f;
    if (nsp <= 8) {
        // all partials in flight at once (one memory round trip); the arithmetic below is the general loop's
        float m[8], l[8], o[8][N];
#pragma unroll
        for (int s = 0; s < 8; ++s)
            if (s < nsp) {
                const float* pr = p0 + s * stride;
                m[s] = pr[0];
                l[s] = pr[1];
#pragma unroll
                for (int e = 0; e < N; ++e) o[s][e] = pr[2 + i + e];
            }
#pragma unroll
        for (int s = 0; s < 8; ++s)
            if (s < nsp) M = fmaxf(M, m[s]);
#pragma unroll
        for (int s = 0; s < 8; ++s)
            if (s < nsp) {
                const float f = expf(m[s] - M);
                Lsum = fmaf(l[s], f, Lsum);
#pragma unroll
                for (int e = 0; e < N; ++e) out[e] = fmaf(o[s][e], f, out[e]);
            }
    } else {
        // long contexts: the same arithmetic in the same order, with the loads of 16 / 8 partials issued together
        for (int s0 = 0; s0 < nsp; s0 += 16) {
            float m[16];
#pragma unroll
            for (int s = 0; s < 16; ++s) m[s] = (s0 + s < nsp) ? p0[(size_t)(s0 + s) * stride] : -INFINITY;
#pragma unroll
            for (int s = 0; s < 16; ++s) M = fmaxf(M, m[s]);
        }
        for (int s0 = 0; s0 < nsp; s0 += 8) {
            float m[8], l[8], o[8][N];
#pragma unroll
            for (int s = 0; s < 8; ++s)
                if (s0 + s < nsp) {
                    const float* pr = p0 + (size_t)(s0 + s) * stride;
                    m[s] = pr[0];
                    l[s] = pr[1];
#pragma unroll
                    for (int e = 0; e < N; ++e) o[s][e] = pr[2 + i + e];
                }
#pragma unroll
            for (int s = 0; s < 8; ++s)
                if (s0 + s < nsp) {
                    const float f = expf(m[s] - M);
                    Lsum = fmaf(l[s], f, Lsum);
#pragma unroll
                    for (int e = 0; e < N; ++e) out[e] = fmaf(o[s][e], f, out[e]);
                }
        }
    }
#pragma unroll
    for (int e = 0; e < N; ++e) out[e] = out[e] / Lsum;
}

// ---- skinny GEMMs (bf16 weights, MFMA) ---------------------------------------------------------------
// Epilogues fused into the GEMM that produces the value:
//   EPI_QKV     rms scale, rotary embedding, q to the query buffer, k / v into the paged KV cache
//   EPI_RESID   x += y, then the next RMSNorm's operand (x * gain, bf16 hi/lo) and its sum-of-squares partials
//   EPI_SWIGLU  rms scale, silu(gate) * up, packed as the down projection's operand
//   EPI_LOGITS  rms scale, logits rows
// RMSNorm is split in two: the producer writes x * gain and per-tile partial sums of x^2, the consumer
// multiplies its result by rsqrt(mean x^2 + eps) (a per-token scalar commutes with the matrix product).
enum { EPI_QKV = 10, EPI_SWIGLU = 11 };

struct GemmArgs {
    const u32x4* Wt;       // tiled weights [Npad/16][KS][64] x 16 B
    const u32x4* XB;       // packed activations [KS][CT][2][64] x 16 B
    int N, KS;
    int wcap;              // widest pass this launch is meant for (its launch class): operand columns >= wcap are not loaded
    int lb_slots;          // LB kernels: 16-byte slots of a wave's staging area in LDS (64 per two K steps of its range)
    const PassDesc* desc;
    // rms scale of the input (EPI_QKV, EPI_SWIGLU, EPI_LOGITS): partial sums of squares [d/16][16 CT]
    const float* ss_in;
    int ss_tiles;
    float inv_d, eps;
    // outputs
    float* Y;              // RESID: residual stream [32][ldy]; LOGITS: logits [rows][ldy]; QKV: query buffer [32][ldy]
    int ldy;
    void* xb_out;          // RESID / SWIGLU: operand of the next GEMM
    const float* gain_out; // RESID: gain of the RMSNorm that follows
    float* ss_out;         // RESID: [N/16][16 CT]
    // QKV only
    const float2* rope;
    uint16_t* kv;
    const int32_t* page_table;
    int layer, L, H, KV, hd;
};

// stores 4 (or 2) consecutive features of column c into a packed operand
template <int CT>
__device__ inline void pack4(void* xb, int c, int f0, const float v[4]) {
    const int ks = f0 >> 5, gq = (f0 & 31) >> 3, e = f0 & 7, t = c >> 4, cc = c & 15;
    uint16_t* p = (uint16_t*)xb + ((((size_t)ks * CT + t) * 2) * 64 + gq * 16 + cc) * 8 + e;
    uint32_t hi[2], lo[2];
    f32x2_split(v[0], v[1], hi[0], lo[0]);
    f32x2_split(v[2], v[3], hi[1], lo[1]);
    *reinterpret_cast<uint2*>(p) = make_uint2(hi[0], hi[1]);
    *reinterpret_cast<uint2*>(p + 512) = make_uint2(lo[0], lo[1]);
}
template <int CT>
__device__ inline void pack2(void* xb, int c, int f0, float v0, float v1) {
    const int ks = f0 >> 5, gq = (f0 & 31) >> 3, e = f0 & 7, t = c >> 4, cc = c & 15;
    uint16_t* p = (uint16_t*)xb + ((((size_t)ks * CT + t) * 2) * 64 + gq * 16 + cc) * 8 + e;
    uint32_t hi, lo;
    f32x2_split(v0, v1, hi, lo);
    *reinterpret_cast<uint32_t*>(p) = hi;
    *reinterpret_cast<uint32_t*>(p + 512) = lo;
}

// the pass descriptor's scalars, asked for when a kernel starts so that nothing waits for them at its end
struct DescVals { int w, pos0, n_logit, row0; };
__device__ inline DescVals load_desc(const PassDesc* d) { return DescVals{d->w, d->pos0, d->n_logit, d->logit_row0}; }

// What an epilogue reads from memory besides its own result.  The narrow kernels ask for it while the weights
// stream, so that the answers are there when the K loop ends; the arithmetic is the same either way.
template <int EPI> struct EpiPre {};
template <> struct EpiPre<EPI_RESID> { float4 x, gn; };
template <> struct EpiPre<EPI_QKV> { int page; float2 cs[2]; };

template <int EPI>
__device__ inline void epi_prefetch(const GemmArgs& a, const DescVals& dv, int tile, int g, int c, EpiPre<EPI>& p) {
    const int n = tile * 16 + g * 4;
    if constexpr (EPI == EPI_RESID) {
        p.x = *reinterpret_cast<const float4*>(a.Y + (size_t)c * a.ldy + n);
        p.gn = *reinterpret_cast<const float4*>(a.gain_out + n);
    } else if constexpr (EPI == EPI_QKV) {
        const int hd = a.hd, half = hd >> 1;
        const int head = (tile * 16) / hd, t_in = ((tile * 16) % hd) >> 4;
        const int pos = dv.pos0 + c;
        p.page = a.page_table[pos / kPage];
#pragma unroll
        for (int pr = 0; pr < 2; ++pr)
            if (head < a.H + a.KV) p.cs[pr] = a.rope[(size_t)pos * half + t_in * 8 + g * 2 + pr];
    }
}

// value tile of one lane: rows n0 + 4 g + r (r = 0..3) of column c
// PRE: `pre` was filled by epi_prefetch; otherwise the reads happen here
template <int EPI, int CT, bool PRE>
__device__ inline void epilogue(const GemmArgs& a, const DescVals& dv, int tile, int g, int c, f32x4 v, float rs,
                                const EpiPre<EPI>& pre) {
    const int n = tile * 16 + g * 4;
    const int w = dv.w;
    if constexpr (EPI == EPI_LOGITS) {
        const int first = w - dv.n_logit;
        if (c < first || n >= a.N) return;
        float* dst = a.Y + (size_t)(dv.row0 + c - first) * a.ldy + n;
        if ((a.ldy & 3) == 0 && n + 3 < a.N) {
            *reinterpret_cast<float4*>(dst) = make_float4(v[0] * rs, v[1] * rs, v[2] * rs, v[3] * rs);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n + r < a.N) dst[r] = v[r] * rs;
        }
    } else if constexpr (EPI == EPI_RESID) {
        float* dst = a.Y + (size_t)c * a.ldy + n;
        float4 o, gn;
        if constexpr (PRE) { o = pre.x; gn = pre.gn; } else { o = *reinterpret_cast<const float4*>(dst); }
        o.x += v[0]; o.y += v[1]; o.z += v[2]; o.w += v[3];
        *reinterpret_cast<float4*>(dst) = o;
        if constexpr (!PRE) gn = *reinterpret_cast<const float4*>(a.gain_out + n);
        const float pk[4] = {o.x * gn.x, o.y * gn.y, o.z * gn.z, o.w * gn.w};
        pack4<CT>(a.xb_out, c, n, pk);
        float ss = o.x * o.x + o.y * o.y + o.z * o.z + o.w * o.w;
        ss += __shfl_xor(ss, 16, kWave);
        ss += __shfl_xor(ss, 32, kWave);
        if (g == 0) a.ss_out[tile * (16 * CT) + c] = ss;
    } else if constexpr (EPI == EPI_SWIGLU) {
        // weight rows are interleaved: tile row 2e = gate of feature 8 tile + e, tile row 2e + 1 = its up row
        const float g0 = v[0] * rs, u0 = v[1] * rs, g1 = v[2] * rs, u1 = v[3] * rs;
        pack2<CT>(a.xb_out, c, tile * 8 + g * 2, g0 / (1.f + expf(-g0)) * u0, g1 / (1.f + expf(-g1)) * u1);
    } else if constexpr (EPI == EPI_QKV) {
        // weight rows are permuted inside every head: tile row 2e, 2e + 1 = rotary pair (j, j + hd/2), j = 8 t + e;
        // a lane holds the pairs j0 and j0 + 1, so every store below covers two adjacent head dims
        const int hd = a.hd, half = hd >> 1;
        const int head = (tile * 16) / hd, t_in = ((tile * 16) % hd) >> 4;
        const int pos = dv.pos0 + c;
        int page;
        if constexpr (PRE) page = pre.page; else page = a.page_table[pos / kPage];
        const int slot = pos % kPage;
        const int j0 = t_in * 8 + g * 2;
        float x0[2], x1[2];
#pragma unroll
        for (int pr = 0; pr < 2; ++pr) {
            x0[pr] = v[2 * pr] * rs;
            x1[pr] = v[2 * pr + 1] * rs;
            if (head < a.H + a.KV) {
                float2 cs;
                if constexpr (PRE) cs = pre.cs[pr]; else cs = a.rope[(size_t)pos * half + j0 + pr];
                const float r0 = x0[pr] * cs.x - x1[pr] * cs.y, r1 = x1[pr] * cs.x + x0[pr] * cs.y;
                x0[pr] = r0; x1[pr] = r1;
            }
        }
        if (head < a.H) {
            float* q = a.Y + (size_t)c * a.ldy + (size_t)head * hd;
            *reinterpret_cast<float2*>(q + j0) = make_float2(x0[0], x0[1]);
            *reinterpret_cast<float2*>(q + j0 + half) = make_float2(x1[0], x1[1]);
        } else if (head < a.H + a.KV) {   // K planes
            uint16_t* kh = a.kv + kv_plane(page, a.layer, a.L, head - a.H, a.KV, 0, hd);
            uint16_t* kl = kh + (size_t)kPage * hd;
            uint32_t h0, l0, h1, l1;
            f32x2_split(x0[0], x0[1], h0, l0);
            f32x2_split(x1[0], x1[1], h1, l1);
            const int o0 = kv_k_off(slot, j0, hd), o1 = kv_k_off(slot, j0 + half, hd);   // j0 is even: the pair stays together
            *reinterpret_cast<uint32_t*>(kh + o0) = h0;
            *reinterpret_cast<uint32_t*>(kh + o1) = h1;
            *reinterpret_cast<uint32_t*>(kl + o0) = l0;
            *reinterpret_cast<uint32_t*>(kl + o1) = l1;
        } else {                          // V planes
            uint16_t* vh = a.kv + kv_plane(page, a.layer, a.L, head - a.H - a.KV, a.KV, 2, hd);
            uint16_t* vl = vh + (size_t)kPage * hd;
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                const int j = j0 + pr;
                uint32_t hi, lo;
                f32x2_split(x0[pr], x1[pr], hi, lo);
                const int o0 = kv_v_off(slot, j), o1 = kv_v_off(slot, j + half);
                vh[o0] = (uint16_t)hi;
                vh[o1] = (uint16_t)(hi >> 16);
                vl[o0] = (uint16_t)lo;
                vl[o1] = (uint16_t)(lo >> 16);
            }
        }
    }
}

// One workgroup of NW waves per RT tiles of 16 output rows; the waves split K and are summed in wave order.
// A wave multiplies RT row tiles by the same activation operand, which is loaded once per K step (the operand
// comes from L2 and would otherwise cost twice the weight bytes) and only by the lanes whose column is in use.
// Small projections get more waves and fewer tiles per workgroup so that enough loads are in flight.
// The rms scale of the input is gathered on the side: every thread loads a few sum-of-squares partials before
// the K loop and they are folded through LDS, in a fixed order, when the loop is done.
// LB (passes of at most 4 tokens, NT == 1): the few operand lanes that carry data are so little that a wave stages the
// operand of its whole K range in LDS before it asks for any weights: direct-to-LDS loads, 64 lanes x 16 bytes = the
// live blocks (4 columns x 4 k groups x hi, lo) of two K steps per instruction, no registers.  Loads return in order, so
// the staged blocks are there before the first weight block, and a K step then reads its operand from LDS (~100
// cycles) instead of L2 (~1400 cycles, of which a wave's two MFMAs per step hide nothing).
template <int NT, int NW, int RT, int EPI, int CT, bool LB = false, bool SK = false>
__global__ __launch_bounds__(64 * NW) void gemm_bf16(const GemmArgs a) {
    static_assert(!LB || NT == 1, "LDS staging of the operand is for one column tile");
    extern __shared__ u32x4 lb_buf[];
    constexpr int TG = NT > 2 ? 2 : NT;   // column tiles whose partials cross LDS together
    static_assert(RT <= NW, "one finishing wave per row tile");
    __shared__ f32x4 red[NW][RT][TG][64];
    constexpr bool kScaled = (EPI == EPI_QKV || EPI == EPI_SWIGLU || EPI == EPI_LOGITS);
    __shared__ float ssp[kScaled ? NW : 1][16 * NT];
    const int tile0 = blockIdx.x * RT, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int k0 = (int)(((long)a.KS * wave) / NW), k1 = (int)(((long)a.KS * (wave + 1)) / NW);
    const int g = lane >> 4, cc = lane & 15;
    const DescVals dv = load_desc(a.desc);
    // the epilogue's own reads: the narrow kernels' finishing wave asks for them once its first weights are on the way
    constexpr bool kEarly = NT <= 2;
    EpiPre<EPI> pre[kEarly ? NT : 1];   // wave r finishes row tile r
    float ss_mine[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) ss_mine[t] = 0.f;
    // Side reads (sum-of-squares partials for every wave, the epilogue's inputs for the finishing wave) are issued
    // right after a wave's first weight loads, never before them: the weight stream starts at once.
    bool want_pre = true;
    auto prefetch_all = [&]() {
        want_pre = false;
        if constexpr (kScaled) {
            const int gi = wave * 4 + g;
#pragma unroll
            for (int t = 0; t < NT; ++t) {
#pragma unroll 8
                for (int st = gi; st < a.ss_tiles; st += 4 * NW) ss_mine[t] += a.ss_in[st * (16 * CT) + t * 16 + cc];
            }
        }
        if constexpr (kEarly) {
            if (wave >= RT) return;
#pragma unroll
            for (int t = 0; t < NT; ++t)
                if (t * 16 + cc < dv.w) epi_prefetch<EPI>(a, dv, tile0 + wave, g, t * 16 + cc, pre[t]);
        }
    };
    const u32x4* a_ptr = a.Wt + ((size_t)tile0 * a.KS + k0) * 64 + lane;
    const size_t tile_stride = (size_t)a.KS * 64;
    constexpr int kBStep = CT * 128;   // 16-byte words of the operand per K step
    const u32x4* b_ptr = a.XB + (size_t)k0 * kBStep + lane;
    const u32x4* const b_base = b_ptr;
    bool col_live[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) col_live[t] = t * 16 + cc < a.wcap;   // known at launch: nothing waits for the descriptor
    f32x4 acc[RT][NT];
#pragma unroll
    for (int r = 0; r < RT; ++r)
#pragma unroll
        for (int t = 0; t < NT; ++t) acc[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};
    // K steps per batch: about 16 weight loads of 16 bytes in flight per lane; 28 with seven row tiles per wave (one
    // workgroup per CU, so registers do not limit residency there; measured: 71 -> 67 ms per 1504 launches); for the
    // four-tile variant 24 or 32 in flight were slower than 16
    constexpr int U = RT == 7 ? 4 : (NT > 2 ? (NW > 8 ? 4 : 8) : 16) / RT;
    static_assert(U >= 1, "too many row tiles per wave");
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    auto mfma_step = [&](const u32x4 (&wv)[RT], int t, const u32x4 bh, const u32x4 bl) {
#pragma unroll
        for (int r = 0; r < RT; ++r) {
            acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[r]),
                                                                __builtin_bit_cast(bf16x8, bh), acc[r][t], 0, 0, 0);
            acc[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[r]),
                                                                __builtin_bit_cast(bf16x8, bl), acc[r][t], 0, 0, 0);
        }
    };
    if constexpr (SK) {
        // Short K ranges (at most D steps per wave: the draft's q/k/v projection, the qualifier's o projection): a wave asks
        // for its whole range at once, weight blocks from memory and operand blocks from L2 side by side: one round of
        // loads instead of a weight batch followed by operand groups that each cost an exposed L2 round trip (draft q/k/v
        // 9.3 -> 8.6 us, qualifier o 9.8 -> 9.2 us between events).  A longer range would be walked D steps at a time; the
        // host does not pick this variant for one.  A window of D steps refilled step by step was measured for the long
        // ranges and loses to the batches below (target down 29.4 -> 31.1 us): loads return in order, so a window that
        // holds operand blocks next to the weight blocks has 7 instead of 16 weight blocks in flight.  Same K order, same bits.
        static_assert(NT == 1 && RT == 1 && !LB, "the short-range variant is for one tile per wave");
        constexpr int D = 7;
        for (int s0 = k0; s0 < k1; s0 += D) {
            const int n = min(D, k1 - s0);
            u32x4 wq[D], bq[D][2];
#pragma unroll
            for (int u = 0; u < D; ++u)
                if (u < n) {
                    wq[u] = __builtin_nontemporal_load(a_ptr + (size_t)u * 64);
                    bq[u][0] = zero; bq[u][1] = zero;
                    if (col_live[0]) {
                        const u32x4* bp = b_ptr + (size_t)u * kBStep;
                        bq[u][0] = bp[0]; bq[u][1] = bp[64];
                    }
                }
            if (want_pre) prefetch_all();
#pragma unroll
            for (int u = 0; u < D; ++u)
                if (u < n) {
                    const u32x4 w1[1] = {wq[u]};
                    mfma_step(w1, 0, bq[u][0], bq[u][1]);
                }
            a_ptr += (size_t)D * 64;
            b_ptr += (size_t)D * kBStep;
        }
    } else if constexpr (NT == 1 && RT == 4 && !LB) {
        // Four row tiles per wave (the qualifier's gate/up projection, one workgroup per CU, 12 K steps per wave): a step is
        // four weight blocks and one pair of operand blocks, and a window of D steps is on the way at all times: a step's
        // registers are asked for again, D steps ahead, as soon as its MFMAs are issued.  Loads return in the order they
        // were issued, which is the order the steps are used in.  Same K order, same bits as the batches that drain
        // (21.5 -> 20.4 us between events).  Measured and not kept: the same window for the seven-tile variant (4 steps are
        // all its registers hold: target gate/up 42.1 -> 42.6 us) and for the 8-wave q/k/v kernels (8 steps: qualifier 12.8
        // -> 13.9 us, target 16.3 -> 16.7 us).
        constexpr int D = 6;
        const int n = k1 - k0;
        u32x4 wq[D][RT], bq[D][2];
        auto fetch = [&](int slot, int st) {
#pragma unroll
            for (int r = 0; r < RT; ++r) wq[slot][r] = __builtin_nontemporal_load(a_ptr + r * tile_stride + (size_t)st * 64);
            bq[slot][0] = zero; bq[slot][1] = zero;
            if (col_live[0]) {
                const u32x4* bp = b_ptr + (size_t)st * kBStep;
                bq[slot][0] = bp[0]; bq[slot][1] = bp[64];
            }
        };
#pragma unroll
        for (int u = 0; u < D; ++u)
            if (u < n) fetch(u, u);
        if (want_pre) prefetch_all();
        int st = 0;
        for (; st + 2 * D <= n; st += D) {
#pragma unroll
            for (int u = 0; u < D; ++u) {
                mfma_step(wq[u], 0, bq[u][0], bq[u][1]);
                fetch(u, st + D + u);
            }
        }
        // fewer than 2 D steps left, the first D of them (or all) on the way
#pragma unroll
        for (int u = 0; u < D; ++u)
            if (st + u < n) {
                mfma_step(wq[u], 0, bq[u][0], bq[u][1]);
                if (st + D + u < n) fetch(u, st + D + u);
            }
#pragma unroll
        for (int u = 0; u < D; ++u)
            if (st + D + u < n) mfma_step(wq[u], 0, bq[u][0], bq[u][1]);
    } else if constexpr (NT == 1) {
        // Operand blocks come from L2.  BG steps' worth of them is asked for at a time; the first group goes out with the
        // batch's weights and is there long before them, every later group costs one exposed L2 round trip.  The whole
        // batch at once (BG = U) takes up to 64 registers: on in the variants that run at most one workgroup per CU
        // anyway (qualifier q/k/v 39.8 -> 34.7 ms per 2632 launches); where it would cost residency (the draft's gate/up,
        // the LM heads: 17.6 -> 18.5 us) groups of 2 are used (17.6 -> 16.7 us).
        constexpr int BG = (U <= 8 && (RT >= 4 || EPI == EPI_QKV)) ? U : (U < 2 ? U : 2);
        static_assert(U % BG == 0, "operand groups must tile a batch");
        u32x4 bpre[BG][2];
        const u32x4* my_b = nullptr;   // LB: this wave's staged operand, [pair of steps][step parity][hi, lo][k group][column < 4]
        if constexpr (LB) {
            const int n = k1 - k0;
            u32x4* stage = lb_buf + __builtin_amdgcn_readfirstlane(wave) * a.lb_slots;
            const int par = lane >> 5, half = (lane >> 4) & 1, sg = (lane >> 2) & 3, sc = lane & 3;
            for (int i = 0; 2 * i < n; ++i) {
                // a range with an odd number of steps: the last instruction's upper lanes fetch the last step again, into
                // slots no step reads
                const int st = min(2 * i + par, n - 1);
                const u32x4* src = a.XB + (size_t)(k0 + st) * kBStep + half * 64 + sg * 16 + sc;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)src,
                                                 (__attribute__((address_space(3))) void*)(stage + i * 64), 16, 0, 0);
            }
            my_b = stage + g * 4 + cc;
            asm volatile("" ::: "memory");   // the staging loads stay ahead of every other load of the wave
        }
        bool staged_ready = !LB;
        // LB: called once, right after the first batch's weight loads (`later` of them, and nothing else, were issued after
        // the staging loads): when at most `later` loads are outstanding the staged operand is in LDS
        auto staged_wait = [&](bool full_batch) {
            if constexpr (LB) {
                if (staged_ready) return;
                staged_ready = true;
                // Counts on the loads issued since the staging loads: exactly the U * RT weight loads of the first full batch,
                // all unconditional (a predicated or split weight load would make the count, and with it this wait, wrong:
                // then wait for vmcnt(0) instead).  The narrow-against-wide bit-exactness tests guard this.
                static_assert(!LB || U * RT <= 63, "the vmcnt field holds at most 63");
                if (full_batch) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(U * RT < 63 ? U * RT : 63) : "memory");
                else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            }
        };
        auto load_b = [&](int slot, const u32x4* bp) {
            bpre[slot][0] = zero; bpre[slot][1] = zero;
            if constexpr (LB) {
                // bp counts K steps in units of kBStep from the operand's start: recover the step within the wave's range
                const int s = (int)((bp - b_base) / kBStep);
                if (col_live[0]) {
                    const u32x4* q = my_b + (s >> 1) * 64 + (s & 1) * 32;
                    bpre[slot][0] = q[0]; bpre[slot][1] = q[16];
                }
            } else {
                if (col_live[0]) { bpre[slot][0] = bp[0]; bpre[slot][1] = bp[64]; }
            }
        };
        // batches of U K steps; the last batch of a range may be short (its loads still go out together)
        for (int ks = k0; ks < k1; ks += U) {
            u32x4 wv[U][RT];
            if (ks + U <= k1) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int r = 0; r < RT; ++r) wv[u][r] = __builtin_nontemporal_load(a_ptr + r * tile_stride + (size_t)u * 64);
                staged_wait(true);
#pragma unroll
                for (int u = 0; u < BG; ++u) load_b(u, b_ptr + (size_t)u * kBStep);
                if (want_pre) prefetch_all();
#pragma unroll
                for (int g0 = 0; g0 < U; g0 += BG) {
                    if (g0 > 0) {
#pragma unroll
                        for (int u = 0; u < BG; ++u) load_b(u, b_ptr + (size_t)(g0 + u) * kBStep);
                    }
#pragma unroll
                    for (int u = 0; u < BG; ++u) mfma_step(wv[g0 + u], 0, bpre[u][0], bpre[u][1]);
                }
            } else {
                const int cnt = k1 - ks;
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (u < cnt) {
#pragma unroll
                        for (int r = 0; r < RT; ++r) wv[u][r] = __builtin_nontemporal_load(a_ptr + r * tile_stride + (size_t)u * 64);
                    }
                staged_wait(false);
#pragma unroll
                for (int u = 0; u < BG; ++u)
                    if (u < cnt) load_b(u, b_ptr + (size_t)u * kBStep);
                if (want_pre) prefetch_all();
#pragma unroll
                for (int g0 = 0; g0 < U; g0 += BG) {
                    if (g0 > 0) {
#pragma unroll
                        for (int u = 0; u < BG; ++u)
                            if (g0 + u < cnt) load_b(u, b_ptr + (size_t)(g0 + u) * kBStep);
                    }
#pragma unroll
                    for (int u = 0; u < BG; ++u)
                        if (g0 + u < cnt) mfma_step(wv[g0 + u], 0, bpre[u][0], bpre[u][1]);
                }
            }
            a_ptr += (size_t)U * 64;
            b_ptr += (size_t)U * kBStep;
        }
    } else {
        // Several column tiles per wave: a step loads its operand blocks tile by tile right before it uses them (a group
        // of steps' blocks would not fit the registers: 302 spilled registers when tried)
        auto step = [&](const u32x4 (&wv)[RT], const u32x4* bp) {
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                u32x4 bh = zero, bl = zero;
                if (col_live[t]) { bh = bp[t * 128]; bl = bp[t * 128 + 64]; }
                mfma_step(wv, t, bh, bl);
            }
        };
        for (int ks = k0; ks < k1; ks += U) {
            u32x4 wv[U][RT];
            if (ks + U <= k1) {
#pragma unroll
                for (int u = 0; u < U; ++u)
#pragma unroll
                    for (int r = 0; r < RT; ++r) wv[u][r] = __builtin_nontemporal_load(a_ptr + r * tile_stride + (size_t)u * 64);
                if (want_pre) prefetch_all();
#pragma unroll
                for (int u = 0; u < U; ++u) step(wv[u], b_ptr + (size_t)u * kBStep);
            } else {
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (ks + u < k1) {
#pragma unroll
                        for (int r = 0; r < RT; ++r) wv[u][r] = __builtin_nontemporal_load(a_ptr + r * tile_stride + (size_t)u * 64);
                    }
                if (want_pre) prefetch_all();
#pragma unroll
                for (int u = 0; u < U; ++u)
                    if (ks + u < k1) step(wv[u], b_ptr + (size_t)u * kBStep);
            }
            a_ptr += (size_t)U * 64;
            b_ptr += (size_t)U * kBStep;
        }
    }
    if (want_pre) prefetch_all();   // a wave without K steps
    if constexpr (kScaled) {
        // a wave's four strided partial sums are folded pairwise, (0 + 1) + (2 + 3); the waves' results are added in
        // wave order by whoever needs the scale
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            float sw = ss_mine[t] + __shfl_xor(ss_mine[t], 16, kWave);
            sw = sw + __shfl_xor(sw, 32, kWave);
            if (g == 0) ssp[wave][t * 16 + cc] = sw;
        }
    }
    // the waves' partial sums meet in LDS TG column tiles at a time; wave r adds up row tile r in wave order and
    // finishes it, so the RT epilogues of a workgroup run side by side
    const int w = dv.w;
#pragma unroll
    for (int t0 = 0; t0 < NT; t0 += TG) {
        if (t0 > 0) __syncthreads();   // the finishing waves have read the previous group
#pragma unroll
        for (int r = 0; r < RT; ++r)
#pragma unroll
            for (int tt = 0; tt < TG; ++tt) red[wave][r][tt][lane] = acc[r][t0 + tt];
        __syncthreads();
        if (wave >= RT) continue;
#pragma unroll
        for (int tt = 0; tt < TG; ++tt) {
            const int t = t0 + tt;
            float rs = 1.f;
            if constexpr (kScaled) {
                float ssum = 0.f;
#pragma unroll
                for (int v = 0; v < NW; ++v) ssum += ssp[v][t * 16 + cc];
                rs = rsqrtf(ssum * a.inv_d + a.eps);
            }
            const int c = t * 16 + cc;
            f32x4 sum = red[0][wave][tt][lane];
#pragma unroll
            for (int v = 1; v < NW; ++v) sum += red[v][wave][tt][lane];
            // whole 16-lane groups agree on c < w, and the shuffles inside the epilogue cross g only
            if (c < w) epilogue<EPI, CT, kEarly>(a, dv, tile0 + wave, g, c, sum, rs, pre[kEarly ? t : 0]);
        }
    }
}

// Projections of a prompt-ingestion pass wider than 128 tokens.  A workgroup of eight waves owns 16 row tiles x
// 32 TC columns (ncg column groups per launch) and walks the whole of K: every K step's 16 weight blocks and
// the column group's operand (hi and lo halves) go through LDS once, double-buffered, and each wave multiplies a
// 4 x TC block of tiles out of it, so a weight block fetched from memory is used for 32 TC columns and an operand
// block for 256 rows.  TC = 4 moves the fewest bytes per MFMA; TC = 2 doubles the workgroups of a projection with
// few row tiles.  The arithmetic is that of gemm_bf16 with NW waves: K is cut at the same NW boundaries, each
// range is accumulated from zero by the same MFMA sequence, and the ranges are added in order, so the result has
// the same bits as the narrow kernels'.
template <int NW, int EPI, int TC>
__global__ __launch_bounds__(512) void gemm_panel(const GemmArgs a, const int tiles, const int ncg) {
    constexpr int CT = kWideCT;
    constexpr bool kScaled = (EPI == EPI_QKV || EPI == EPI_SWIGLU);
    constexpr int GC = 32 * TC, GW = 4 * TC * 64;             // columns, and operand words per K step, of a column group
    static_assert(TC == 2 || TC == 4, "column tiles per wave");
    __shared__ u32x4 smem[2 * 2 * 16 * 64];                   // 64 KB: weight blocks, then operand blocks, two buffers each
    u32x4 (*sA)[16][64] = reinterpret_cast<u32x4 (*)[16][64]>(smem);
    u32x4 (*sB)[16][64] = reinterpret_cast<u32x4 (*)[16][64]>(smem + 2 * 16 * 64);   // [column tile][hi, lo][lane] flattened
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 4, cc = lane & 15;
    const int wr = wave >> 1, wc = wave & 1;     // rows 4 wr .. + 4 of the 16 tiles, column tiles TC wc .. + TC of the group's
    // Workgroups go to the eight XCDs (one L2 each) round-robin in launch order.  The ncg column groups of a row
    // group take consecutive slots of one XCD, so they run side by side and its weights come from memory once.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int rgi = (slot / ncg) * 8 + xcd, cg = slot % ncg, KS = a.KS;
    if (rgi * 16 >= tiles) return;
    const int tile0 = rgi * 16;
    constexpr int kBStep = CT * 128;
    // what this thread stages per K step: two weight words and two operand words
    const int ta = tile0 + (tid >> 6);
    const u32x4* pa0 = a.Wt + (size_t)(ta < tiles ? ta : tiles - 1) * KS * 64 + lane;
    const u32x4* pa1 = a.Wt + (size_t)(ta + 8 < tiles ? ta + 8 : tiles - 1) * KS * 64 + lane;
    const u32x4* pb = a.XB + (size_t)cg * GW + tid;
    struct Stage { u32x4 a0, a1, b0, b1; };
    auto fetch = [&](Stage& s, int ks) {
        s.a0 = __builtin_nontemporal_load(pa0 + (size_t)ks * 64);
        s.a1 = __builtin_nontemporal_load(pa1 + (size_t)ks * 64);
        s.b0 = pb[(size_t)ks * kBStep];
        if constexpr (GW > 512) s.b1 = pb[(size_t)ks * kBStep + 512];
    };
    Stage s0, s1;
    fetch(s0, 0);
    if (KS > 1) fetch(s1, 1);
    float rs[TC];
#pragma unroll
    for (int t = 0; t < TC; ++t) rs[t] = 1.f;
    if constexpr (kScaled) {
        // the narrow kernels' 4 NW strided partial sums of the input's sums of squares, per column, folded as there:
        // (0 + 1) + (2 + 3) within each group of four, the groups added in order
        float (*ssp)[GC] = reinterpret_cast<float (*)[GC]>(smem);
        const int col = tid % GC;
        for (int slot = tid / GC; slot < 4 * NW; slot += 512 / GC) {
            float sum = 0.f;
            for (int st = slot; st < a.ss_tiles; st += 4 * NW) sum += a.ss_in[st * (16 * CT) + cg * GC + col];
            ssp[slot][col] = sum;
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < TC; ++t) {
            float ssum = 0.f;
#pragma unroll
            for (int u = 0; u < NW; ++u) {
                const int col = (wc * TC + t) * 16 + cc;
                ssum += (ssp[4 * u][col] + ssp[4 * u + 1][col]) + (ssp[4 * u + 2][col] + ssp[4 * u + 3][col]);
            }
            rs[t] = rsqrtf(ssum * a.inv_d + a.eps);
        }
        __syncthreads();
    }
    f32x4 cur[4][TC], tot[4][TC];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int t = 0; t < TC; ++t) { cur[r][t] = f32x4{0.f, 0.f, 0.f, 0.f}; tot[r][t] = f32x4{0.f, 0.f, 0.f, 0.f}; }
    // K ranges end at KS (v + 1) / NW; the launcher guarantees KS >= NW, so none is empty.  A range's sum starts from
    // +0 and can therefore never be -0: adding it to a zero total leaves its bits as they are.
    int v = 0, nb = KS / NW;
    auto fold = [&]() {
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int t = 0; t < TC; ++t) {
                tot[r][t] += cur[r][t];
                cur[r][t] = f32x4{0.f, 0.f, 0.f, 0.f};
            }
        ++v;
        nb = (int)(((long)KS * (v + 1)) / NW);
    };
    auto put = [&](const Stage& s, int buf) {
        sA[buf][tid >> 6][lane] = s.a0;
        sA[buf][8 + (tid >> 6)][lane] = s.a1;
        (&sB[buf][0][0])[tid] = s.b0;
        if constexpr (GW > 512) (&sB[buf][0][0])[tid + 512] = s.b1;
    };
    auto multiply = [&](int buf) {
        u32x4 wv[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) wv[r] = sA[buf][wr * 4 + r][lane];
#pragma unroll
        for (int t = 0; t < TC; ++t) {
            const u32x4 bh = sB[buf][(wc * TC + t) * 2][lane], bl = sB[buf][(wc * TC + t) * 2 + 1][lane];
#pragma unroll
            for (int r = 0; r < 4; ++r)
                cur[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[r]),
                                                                    __builtin_bit_cast(bf16x8, bh), cur[r][t], 0, 0, 0);
#pragma unroll
            for (int r = 0; r < 4; ++r)
                cur[r][t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wv[r]),
                                                                    __builtin_bit_cast(bf16x8, bl), cur[r][t], 0, 0, 0);
        }
    };
    // K step ks is multiplied out of LDS buffer ks & 1 while step ks + 1 is written to the other buffer and
    // steps ks + 2, ks + 3 are in flight in registers
    put(s0, 0);
    if (KS > 2) fetch(s0, 2);
    __syncthreads();
    for (int ks = 0; ks < KS; ks += 2) {
        if (ks == nb) fold();
        if (ks + 1 < KS) put(s1, 1);
        if (ks + 3 < KS) fetch(s1, ks + 3);
        multiply(0);
        __syncthreads();
        if (ks + 1 >= KS) break;
        if (ks + 1 == nb) fold();
        if (ks + 2 < KS) put(s0, 0);
        if (ks + 4 < KS) fetch(s0, ks + 4);
        multiply(1);
        __syncthreads();
    }
    fold();
    const DescVals dv = load_desc(a.desc);
    const int w = dv.w;
#pragma unroll
    for (int t = 0; t < TC; ++t) {
        const int c = cg * GC + (wc * TC + t) * 16 + cc;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            const int tile = tile0 + wr * 4 + r;
            // whole 16-lane groups agree on c < w, and the shuffles inside the epilogue cross g only
            if (tile < tiles && c < w) epilogue<EPI, CT, false>(a, dv, tile, g, c, tot[r][t], rs[t], EpiPre<EPI>{});
        }
    }
}

// o projection of a narrow pass (<= 4 tokens, K <= 2048, one row tile per workgroup): the merge of the attention
// split partials, otherwise a kernel of its own, is done here while the weight blocks are in flight; the merged
// rows go to LDS in B-operand order.  Same K split, MFMA order and reduction as gemm_bf16<1, 16, 1, EPI_RESID>, and
// the same merge arithmetic as attn_combine_bf16, so the result has the same bits as the two-kernel route.
__global__ __launch_bounds__(1024) void gemm_o_narrow(const GemmArgs a, const float* __restrict__ attn_part) {
    constexpr int NW = 16, KSMAX = 64;
    __shared__ f32x4 red[NW - 1][64];
    __shared__ u32x4 sB[KSMAX * 2 * 4 * 4];   // [k step][hi, lo][g][column < 4]
    const int tile = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int k0 = (int)(((long)a.KS * wave) / NW), k1 = (int)(((long)a.KS * (wave + 1)) / NW);
    const int g = lane >> 4, cc = lane & 15;
    const u32x4* a_ptr = a.Wt + ((size_t)tile * a.KS + k0) * 64 + lane;
    u32x4 wv[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (k0 + u < k1) wv[u] = __builtin_nontemporal_load(a_ptr + (size_t)u * 64);
    const DescVals dv = load_desc(a.desc);
    const int w = dv.w, pos0 = dv.pos0, K = a.KS * 32;
    EpiPre<EPI_RESID> pre;
    if (wave == 0 && cc < w) epi_prefetch<EPI_RESID>(a, dv, tile, g, cc, pre);   // answered while the partials are merged
    uint16_t* sB16 = reinterpret_cast<uint16_t*>(sB);
    // pairs of adjacent head dims: for one token that is exactly one pair per thread, i.e. one memory round trip
    for (int pidx = threadIdx.x; pidx < 2 * K; pidx += 1024) {
        const int c = pidx / (K >> 1), k = (pidx % (K >> 1)) * 2;
        float v[2] = {0.f, 0.f};
        if (c < w) attn_merge<2>(attn_part, (pos0 + c + kAttnSplit) / kAttnSplit, c, k / a.hd, a.H, a.hd, k % a.hd, v);
        uint32_t hi, lo;
        f32x2_split(v[0], v[1], hi, lo);
        const int ks = k >> 5, gq = (k & 31) >> 3, e = k & 7;
        *reinterpret_cast<uint32_t*>(sB16 + ((((ks * 2 + 0) * 4 + gq) * 4 + c) << 3) + e) = hi;
        *reinterpret_cast<uint32_t*>(sB16 + ((((ks * 2 + 1) * 4 + gq) * 4 + c) << 3) + e) = lo;
    }
    __syncthreads();
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
    const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
    auto step = [&](const u32x4 wblk, int ks) {
        u32x4 bh = zero, bl = zero;
        if (cc < 4) { bh = sB[((ks * 2 + 0) * 4 + g) * 4 + cc]; bl = sB[((ks * 2 + 1) * 4 + g) * 4 + cc]; }
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wblk), __builtin_bit_cast(bf16x8, bh), acc, 0, 0, 0);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wblk), __builtin_bit_cast(bf16x8, bl), acc, 0, 0, 0);
    };
#pragma unroll
    for (int u = 0; u < 4; ++u)
        if (k0 + u < k1) step(wv[u], k0 + u);
    for (int ks = k0 + 4; ks < k1; ++ks) step(__builtin_nontemporal_load(a_ptr + (size_t)(ks - k0) * 64), ks);
    if (wave > 0) red[wave - 1][lane] = acc;
    __syncthreads();
    if (wave != 0) return;
#pragma unroll
    for (int v = 0; v < NW - 1; ++v) acc += red[v][lane];
    if (cc < w) epilogue<EPI_RESID, 2, true>(a, dv, tile, g, cc, acc, 1.f, pre);
}

// token embedding: x = E[token]; also the first RMSNorm's operand and sum-of-squares partials.  grid d/16, 64 threads
template <int NT, int CT>
__global__ __launch_bounds__(64) void embed_pack(const uint16_t* embed, const PassDesc* desc, float* x, void* xb,
                                                 const float* gain, float* ss_out, int d, int V) {
    const int tile = blockIdx.x, lane = threadIdx.x, g = lane >> 4, cc = lane & 15;
    const int w = desc->w, KS = d >> 5;
#pragma unroll
    for (int t = 0; t < NT; ++t) {
        const int c = t * 16 + cc;
        if (c >= w) continue;
        int tok = desc->tok[c];
        tok = tok < 0 ? 0 : (tok >= V ? V - 1 : tok);
        const int n = tile * 16 + g * 4;
        const size_t idx = ((((size_t)(tok >> 4) * KS + (n >> 5)) * 64) + ((n & 31) >> 3) * 16 + (tok & 15)) * 8 + (n & 7);
        const uint2 raw = *reinterpret_cast<const uint2*>(embed + idx);
        const float v[4] = {bf16_to_f32(raw.x & 0xffff), bf16_to_f32(raw.x >> 16), bf16_to_f32(raw.y & 0xffff), bf16_to_f32(raw.y >> 16)};
        *reinterpret_cast<float4*>(x + (size_t)c * d + n) = make_float4(v[0], v[1], v[2], v[3]);
        const float4 gn = *reinterpret_cast<const float4*>(gain + n);
        const float pk[4] = {v[0] * gn.x, v[1] * gn.y, v[2] * gn.z, v[3] * gn.w};
        pack4<CT>(xb, c, n, pk);
        float ss = v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
        ss += __shfl_xor(ss, 16, kWave);
        ss += __shfl_xor(ss, 32, kWave);
        if (g == 0) ss_out[tile * (16 * CT) + c] = ss;
    }
}

// ---- attention, bf16 KV cache, MFMA ---------------------------------------------------------------------
// grid (KV heads, nsplit_max, query tiles), 256 threads.  A workgroup owns one KV head, the absolute key range
// [split * 128, +128) and 16 query rows rho = token * G + head_in_group; wave j owns the 32 keys
// [split * 128 + 32 j, +32):
//   S^T = K Q^T    v_mfma_f32_16x16x32_bf16, A = 16 keys x 32 head dims: one contiguous 1 KiB tile of the K planes
//                  (hi, lo), B = queries as bf16 hi + lo built in registers; result lane (g, c): keys 4g..4g+3 of query c
//   P   = exp(S - max) per query over the wave's 32 keys (masked causally), kept in registers: the result
//         layout of S^T is exactly the A operand layout of v_mfma_f32_16x16x16bf16_1k
//   O   = P V      B = 4 consecutive keys of one head dim: one contiguous 512-byte tile of the V planes
// The four waves' (max, sum, O) are merged through LDS in wave order and written as one partial per split.
// Memory round trips on the critical path: the pass descriptor and the page-table entry travel together, then the
// queries (from L2), keys and values go out back to back; the kernel is latency-bound, so that is what counts.
// Two waves per SIMD are asked for (at head dim 128 the kernel would otherwise take 284 registers and run one workgroup
// per CU): with dozens of key ranges a launch has several workgroups per CU, and their round trips then overlap.
typedef __attribute__((ext_vector_type(4))) short s16x4;

template <int HD>
__global__ __launch_bounds__(256, 2) void attn_mfma(const float* qkv, const PassDesc* desc, const uint16_t* kv,
                                                 const int32_t* page_table, int n_pages, float* part, int layer, int L, int H,
                                                 int KV, int nqkv, int qt_per_wg) {
    constexpr int KSQ = HD / 32, JT = HD / 16;
    __shared__ float mrg[4][16][HD + 2];
    const int gkv = blockIdx.x, split = blockIdx.y;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, g = lane >> 4, cq = lane & 15;
    const int key0 = split * kAttnSplit, wkey0 = key0 + wave * 32;
    // asked for together with the descriptor: the entry exists for every key range a launch covers
    const int page = page_table[min(wkey0 / kPage, n_pages - 1)];
    const int w = desc->w, pos0 = desc->pos0;
    const int kv_max = pos0 + w;
    const int G = H / KV, R = w * G;
    if (key0 >= kv_max || (int)blockIdx.z * qt_per_wg * 16 >= R) return;
    const bool wave_live = wkey0 < kv_max;
    const float scale = rsqrtf((float)HD);
    // query rows of the first tile, as they come from the q/k/v projection (fp32); converted when they are used
    auto load_q = [&](int qt, float (&v)[KSQ][8]) {
        const int rho = qt * 16 + cq;
        const float* qrow = qkv + (size_t)(rho / G) * nqkv + (size_t)(gkv * G + rho % G) * HD;
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
            if (rho < R) {
                const float4 a0 = *reinterpret_cast<const float4*>(qrow + ks * 32 + g * 8);
                const float4 a1 = *reinterpret_cast<const float4*>(qrow + ks * 32 + g * 8 + 4);
                v[ks][0] = a0.x; v[ks][1] = a0.y; v[ks][2] = a0.z; v[ks][3] = a0.w;
                v[ks][4] = a1.x; v[ks][5] = a1.y; v[ks][6] = a1.z; v[ks][7] = a1.w;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) v[ks][e] = 0.f;
            }
        }
    };
    float qraw[KSQ][8];
    if (wave_live) load_q(blockIdx.z * qt_per_wg, qraw);
    // the wave's keys and values stay in registers for all of the workgroup's query tiles
    u32x4 ka[2][KSQ], kb[2][KSQ];   // hi and lo halves
    uint2 vraw[JT][2], vlow[JT][2];
    if (wave_live) {
        // this wave's 32 keys are two 16-slot tiles of one page
        const int st0 = (wkey0 % kPage) >> 4;
        constexpr size_t kPlane = (size_t)kPage * HD;
        const uint16_t* Kp = kv + kv_plane(page, layer, L, gkv, KV, 0, HD);
        const uint16_t* Vp = Kp + 2 * kPlane;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int ks = 0; ks < KSQ; ++ks) {
                const uint16_t* p = Kp + ((size_t)((st0 + kt) * KSQ + ks) * 64 + lane) * 8;
                ka[kt][ks] = *reinterpret_cast<const u32x4*>(p);
                kb[kt][ks] = *reinterpret_cast<const u32x4*>(p + kPlane);
            }
#pragma unroll
        for (int j = 0; j < JT; ++j)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const uint16_t* p = Vp + ((size_t)(j * (kPage >> 4) + st0 + kt) * 64 + lane) * 4;
                vraw[j][kt] = *reinterpret_cast<const uint2*>(p);
                vlow[j][kt] = *reinterpret_cast<const uint2*>(p + kPlane);
            }
    }
    for (int qi = 0; qi < qt_per_wg; ++qi) {
    const int qt = blockIdx.z * qt_per_wg + qi;
    if (qt * 16 >= R) break;
    // every key of this split lies after the tile's last query: nothing to attend to, and the merge never reads it
    if (key0 > pos0 + ((qt * 16 + 15 < R ? qt * 16 + 15 : R - 1) / G)) {
        if (wave_live && qi + 1 < qt_per_wg) load_q(qt + 1, qraw);   // qraw always holds the queries of the tile about to be worked on
        continue;
    }
    const int rho = qt * 16 + cq;
    float m = -INFINITY, l = 0.f;
    f32x4 O[JT];
#pragma unroll
    for (int j = 0; j < JT; ++j) O[j] = f32x4{0.f, 0.f, 0.f, 0.f};
    if (wave_live) {
        // query row rho as B operand: lane (g, c) holds head dims 32 ks + 8 g .. + 8 of row c, scaled by 1/sqrt(hd)
        u32x4 qh[KSQ], ql[KSQ];
#pragma unroll
        for (int ks = 0; ks < KSQ; ++ks) {
            uint32_t hw[4], lw[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                f32x2_split(qraw[ks][2 * e] * scale, qraw[ks][2 * e + 1] * scale, hw[e], lw[e]);
            }
            qh[ks] = u32x4{hw[0], hw[1], hw[2], hw[3]};
            ql[ks] = u32x4{lw[0], lw[1], lw[2], lw[3]};
        }
        if (qi + 1 < qt_per_wg) load_q(qt + 1, qraw);   // the next tile's queries travel while this tile is worked on
        f32x4 Sx[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            Sx[kt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < KSQ; ++ks) {
                // (k_hi + k_lo)(q_hi + q_lo) without the lo * lo term (2^-18 relative)
                Sx[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kt][ks]), __builtin_bit_cast(bf16x8, qh[ks]), Sx[kt], 0, 0, 0);
                Sx[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, ka[kt][ks]), __builtin_bit_cast(bf16x8, ql[ks]), Sx[kt], 0, 0, 0);
                Sx[kt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kb[kt][ks]), __builtin_bit_cast(bf16x8, qh[ks]), Sx[kt], 0, 0, 0);
            }
        }
        // causal mask: key position <= query position; rows beyond R see nothing
        const int qpos = rho < R ? pos0 + rho / G : -1;
#pragma unroll
        for (int kt = 0; kt < 2; ++kt)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const int kp = wkey0 + kt * 16 + g * 4 + r;
                if (kp > qpos) Sx[kt][r] = -INFINITY;
                m = fmaxf(m, Sx[kt][r]);
            }
        m = fmaxf(m, __shfl_xor(m, 16, kWave));
        m = fmaxf(m, __shfl_xor(m, 32, kWave));
        const float msafe = m == -INFINITY ? 0.f : m;
        s16x4 Ph[2], Pl[2];
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            float p[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                p[r] = expf(Sx[kt][r] - msafe);   // exp(-inf) = 0 for masked keys
                l += p[r];
            }
            uint2 ph, pl;
            f32x2_split(p[0], p[1], ph.x, pl.x);
            f32x2_split(p[2], p[3], ph.y, pl.y);
            Ph[kt] = __builtin_bit_cast(s16x4, ph);
            Pl[kt] = __builtin_bit_cast(s16x4, pl);
        }
        l += __shfl_xor(l, 16, kWave);
        l += __shfl_xor(l, 32, kWave);
#pragma unroll
        for (int j = 0; j < JT; ++j)
#pragma unroll
            for (int kt = 0; kt < 2; ++kt) {
                const s16x4 vb = __builtin_bit_cast(s16x4, vraw[j][kt]), vl = __builtin_bit_cast(s16x4, vlow[j][kt]);
                O[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(Ph[kt], vb, O[j], 0, 0, 0);
                O[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(Pl[kt], vb, O[j], 0, 0, 0);
                O[j] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(Ph[kt], vl, O[j], 0, 0, 0);
            }
    }
    // merge the four waves: O lane (g, c) holds queries 4g + r, head dim 16 j + c
    if (g == 0) { mrg[wave][cq][0] = m; mrg[wave][cq][1] = l; }
#pragma unroll
    for (int j = 0; j < JT; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) mrg[wave][g * 4 + r][2 + j * 16 + cq] = O[j][r];
    __syncthreads();
    // sixteen threads per query row: each works out the row's merged maximum and the four waves' rescaling factors for
    // itself (the same arithmetic in every thread), one of them stores (max, sum), and together they merge the row's
    // head dims, sixteen at a time
    {
        const int qr = threadIdx.x >> 4, i0 = threadIdx.x & 15, rr = qt * 16 + qr;
        if (rr < R) {
            float M = -INFINITY;
#pragma unroll
            for (int v = 0; v < 4; ++v) M = fmaxf(M, mrg[v][qr][0]);
            float fac[4], Ls = 0.f;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                fac[v] = mrg[v][qr][0] == -INFINITY ? 0.f : expf(mrg[v][qr][0] - M);
                Ls = fmaf(mrg[v][qr][1], fac[v], Ls);
            }
            const int rh = (rr / G) * H + gkv * G + rr % G;
            float* out = part + ((size_t)split * kCols * H + rh) * (HD + 2);
            if (i0 == 0) { out[0] = M; out[1] = Ls; }
#pragma unroll
            for (int jj = 0; jj < JT; ++jj) {
                const int i = jj * 16 + i0;
                float o = 0.f;
#pragma unroll
                for (int v = 0; v < 4; ++v) o = fmaf(mrg[v][qr][2 + i], fac[v], o);
                out[2 + i] = o;
            }
        }
    }
    if (qi + 1 < qt_per_wg) __syncthreads();   // the merge buffer is reused by the next query tile
    }
}

// grid (wmax, H), block hd: merges the split partials and writes the O-projection's input operand (wide passes)
template <int CT>
__global__ void attn_combine_bf16(const float* part, const PassDesc* desc, void* xb, int H, int hd) {
    const int c = blockIdx.x, h = blockIdx.y, i = threadIdx.x;
    if (c >= desc->w) return;
    const int nsp = (desc->pos0 + c + kAttnSplit) / kAttnSplit;  // splits holding keys <= pos0 + c
    float o[1];
    attn_merge<1>(part, nsp, c, h, H, hd, i, o);
    pack_store<true, CT>(xb, H * hd, c, h * hd + i, o[0]);
}

// The same merge for long contexts (more than eight key ranges): one workgroup per (token, head) brings the partials of
// all its ranges into LDS with one round of loads (the thread-per-head-dim form above walks them in dependent rounds of
// sixteen: 9-11 us at 36 ranges), then takes the maximum (exact, so any order), the rescaling factors (one thread per
// range) and the sums in range order: the arithmetic, hence the bits, of attn_merge.
// grid (wmax, H), 256 threads, dynamic LDS: nsplit * (hd + 3) floats.
template <int CT>
__global__ __launch_bounds__(256) void attn_combine_long(const float* part, const PassDesc* desc, void* xb, int H, int hd, int nsp_cap) {
    extern __shared__ float cmb[];
    __shared__ float red[4];
    const int c = blockIdx.x, h = blockIdx.y;
    if (c >= desc->w) return;
    // splits holding keys <= pos0 + c; never more than the launch covers (the LDS area is sized for those)
    const int nsp = min((desc->pos0 + c + kAttnSplit) / kAttnSplit, nsp_cap);
    const int row = hd + 2;
    const size_t stride = (size_t)kCols * H * row;
    const float* p0 = part + ((size_t)c * H + h) * row;
    // batches of 24 loads per thread, all of a batch in flight together (one batch covers 47 ranges at head dim 128)
    constexpr int kBatch = 24;
    for (int base = 0; base < nsp * row; base += kBatch * 256) {
        float v[kBatch];
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int idx = base + u * 256 + (int)threadIdx.x;
            const int sp = idx / row, i = idx - sp * row;
            v[u] = idx < nsp * row ? p0[(size_t)sp * stride + i] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < kBatch; ++u) {
            const int idx = base + u * 256 + (int)threadIdx.x;
            if (idx < nsp * row) cmb[idx] = v[u];
        }
    }
    __syncthreads();
    float m = -INFINITY;
    for (int sp = threadIdx.x; sp < nsp; sp += 256) m = fmaxf(m, cmb[sp * row]);
    const float M = block_max<4>(m, red);
    float* fac = cmb + nsp * row;
    for (int sp = threadIdx.x; sp < nsp; sp += 256) fac[sp] = expf(cmb[sp * row] - M);
    __syncthreads();
    if ((int)threadIdx.x < hd) {
        const int i = threadIdx.x;
        float Lsum = 0.f, o = 0.f;
        for (int sp = 0; sp < nsp; ++sp) {
            const float f = fac[sp];
            Lsum = fmaf(cmb[sp * row + 1], f, Lsum);
            o = fmaf(cmb[sp * row + 2 + i], f, o);
        }
        pack_store<true, CT>(xb, H * hd, c, h * hd + i, o / Lsum);
    }
}

// fp32 weights, row-major [N][K]; X fp32 rows [c][K].  One wave per output row.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32(const float* __restrict__ W, const float* __restrict__ X,
                                                float* __restrict__ Y, int N, int K, int ldy,
                                                const PassDesc* __restrict__ desc) {
    const int n = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
    if (n >= N) return;
    const int w = desc->w;
    const float* wr = W + (size_t)n * K;
    for (int c = 0; c < w; ++c) {
        int row = c;
        if constexpr (EPI == EPI_LOGITS) {
            const int first = w - desc->n_logit;
            if (c < first) continue;
            row = desc->logit_row0 + c - first;
        }
        const float* xr = X + (size_t)c * K;
        float acc = 0.f;
        for (int k = lane; k < K; k += 64) acc += wr[k] * xr[k];
        acc = wave_sum(acc);
        if (lane == 0) {
            float* dst = Y + (size_t)row * ldy + n;
            if constexpr (EPI == EPI_RESID) *dst += acc;
            else *dst = acc;
        }
    }
}

// ---- profiler ---------------------------------------------------------------------------------------
int Profiler::row_of(const char* name) {
    for (size_t i = 0; i < rows.size(); ++i)
        if (!strncmp(rows[i].name, name, sizeof(rows[i].name))) return (int)i;
    KernelAcc r;
    memset(r.name, 0, sizeof(r.name));
    strncpy(r.name, name, sizeof(r.name) - 1);
    rows.push_back(r);
    return (int)rows.size() - 1;
}
hipEvent_t Profiler::get_event() {
    if (!free_events.empty()) { hipEvent_t e = free_events.back(); free_events.pop_back(); return e; }
    hipEvent_t e;
    (void)hipEventCreate(&e);
    return e;
}
void Profiler::begin(hipStream_t s, int row, double bytes) {
    Pending p{row, get_event(), get_event()};
    (void)hipEventRecord(p.a, s);
    pending.push_back(p);
    rows[row].launches++;
    rows[row].bytes += bytes;
}
void Profiler::end(hipStream_t s) { (void)hipEventRecord(pending.back().b, s); }
void Profiler::flush() {
    for (auto& p : pending) {
        (void)hipEventSynchronize(p.b);
        float ms = 0.f;
        (void)hipEventElapsedTime(&ms, p.a, p.b);
        rows[p.row].ms += ms;
        free_events.push_back(p.a);
        free_events.push_back(p.b);
    }
    pending.clear();
}
void Profiler::clear() { flush(); rows.clear(); }
Profiler::~Profiler() {
    flush();
    for (auto e : free_events) (void)hipEventDestroy(e);
}

// ---- sizing / init ----------------------------------------------------------------------------------
static size_t esize(int dtype) { return dtype == PSD_BF16 ? 2 : 4; }

static int round16(int n) { return (n + 15) & ~15; }

static int attn_lds_bytes(int hd) { return (2 * kAttnSplit * (hd + 1) + 4 * hd + 4 * kAttnSplit) * (int)sizeof(float); }

// most LDS a narrow GEMM may use for staging its operand (beside its 16 KB of partial sums)
constexpr size_t kLbMaxBytes = 128 * 1024;

template <int EPI>
static int lb_kernels_init(char* err) {
    PSD_HIP(hipFuncSetAttribute((const void*)gemm_bf16<1, 16, 1, EPI, 2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLbMaxBytes), err);
    PSD_HIP(hipFuncSetAttribute((const void*)gemm_bf16<1, 8, 2, EPI, 2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLbMaxBytes), err);
    PSD_HIP(hipFuncSetAttribute((const void*)gemm_bf16<1, 8, 1, EPI, 2, true>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)kLbMaxBytes), err);
    return PSD_OK;
}

int model_kernels_init(char* err) {
    // attention stages two pages of K and V as fp32 in LDS: up to ~135 KB of the 160 KB a gfx950 CU has
    PSD_HIP(hipFuncSetAttribute((const void*)attn_partial<float>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                attn_lds_bytes(128)), err);
    int rc;
    if ((rc = lb_kernels_init<EPI_RESID>(err)) != PSD_OK) return rc;
    if ((rc = lb_kernels_init<EPI_LOGITS>(err)) != PSD_OK) return rc;
    return PSD_OK;
}

// walks the allocation sequence; with a dry pool this only measures
static int model_carve(Model& M, Pool& pool) {
    const size_t es = esize(M.dtype);
    const size_t q = (size_t)M.H * M.hd;
    bool ok = true;
    auto take = [&](size_t bytes) { void* p = pool.take(bytes); if (!p && !pool.dry) ok = false; return p; };
    M.embed = take((size_t)M.Vpad * M.d * es);
    M.layers.resize(M.L);
    for (int l = 0; l < M.L; ++l) {
        LayerW& w = M.layers[l];
        w.attn_norm = (const float*)take(M.d * sizeof(float));
        w.wqkv = take((size_t)M.nqkv * M.d * es);
        w.wo = take((size_t)M.d * q * es);
        w.ffn_norm = (const float*)take(M.d * sizeof(float));
        w.wgu = take((size_t)2 * M.F * M.d * es);
        w.wd = take((size_t)M.d * M.F * es);
    }
    M.final_norm = (const float*)take(M.d * sizeof(float));
    M.rope = (const float2*)take((size_t)M.max_seq * (M.hd / 2) * sizeof(float2));
    M.kv = take((size_t)M.n_pages * M.L * M.KV * 2 * kPage * M.hd * 4);   // fp32, or bf16 hi + lo
    M.page_table = (int32_t*)take((size_t)M.n_pages * sizeof(int32_t));
    const size_t kmax = std::max((size_t)M.d, (size_t)M.F);
    M.x = (float*)take((size_t)kCols * M.d * sizeof(float));
    M.xb = take(kmax * 128);
    if (M.dtype == PSD_BF16) {
        M.xb2 = take(kmax * 128);
        M.ss = (float*)take((size_t)(M.d / 16) * 32 * sizeof(float));
        M.xbw = take(kmax * 4 * kCols);
        M.xbw2 = take(kmax * 4 * kCols);
        M.ssw = (float*)take((size_t)(M.d / 16) * kCols * sizeof(float));
    }
    M.qkv = (float*)take((size_t)kCols * M.nqkv * sizeof(float));
    M.gu = (float*)take((size_t)kMaxW * 2 * M.F * sizeof(float));
    M.attn_part = (float*)take((size_t)M.nsplit_max * kCols * M.H * (M.hd + 2) * sizeof(float));
    M.desc = (PassDesc*)take(sizeof(PassDesc));
    return ok ? PSD_OK : PSD_ENOMEM;
}

static void model_shape(Model& M, const psd_model_desc& m, int max_seq) {
    M.L = m.n_layers; M.d = m.d_model; M.H = m.n_heads; M.KV = m.n_kv_heads; M.hd = m.d_model / m.n_heads;
    M.F = m.d_ffn; M.V = m.vocab; M.Vpad = m.dtype == PSD_BF16 ? round16(m.vocab) : m.vocab;
    M.nqkv = (M.H + 2 * M.KV) * M.hd;
    M.dtype = m.dtype; M.theta = m.rope_theta; M.eps = m.rms_eps;
    M.max_seq = max_seq;
    M.n_pages = (max_seq + kPage - 1) / kPage;
    M.nsplit_max = (max_seq + kAttnSplit - 1) / kAttnSplit;
    // the panel kernel of the widest passes wants every K range of every projection non-empty
    auto panel_ok = [](int n, int k) { return k / 32 >= (round16(n) / 16 <= 256 ? 16 : 8); };
    M.ingest_max = m.dtype != PSD_BF16 ? kMaxW
                   : (panel_ok(M.nqkv, M.d) && panel_ok(M.d, M.H * M.hd) && panel_ok(2 * M.F, M.d) && panel_ok(M.d, M.F)) ? kCols : 128;
}

size_t model_pool_bytes(const psd_model_desc& m, int max_seq) {
    Model M;
    model_shape(M, m, max_seq);
    Pool p;
    p.dry = true;
    model_carve(M, p);
    return p.used + 256;
}

static size_t blob_elems(const psd_model_desc& m) {
    const size_t d = m.d_model, hd = d / m.n_heads, q = (size_t)m.n_heads * hd, kv = (size_t)m.n_kv_heads * hd, F = m.d_ffn;
    return (size_t)m.vocab * d + (size_t)m.n_layers * (d + q * d + 2 * kv * d + d * q + d + 2 * F * d + d * F) + d;
}

int model_init(Model& M, const psd_model_desc& m, const char* tag, int max_seq, bool scramble_pages, Pool& pool,
               hipStream_t stream, char* err) {
    if (!m.weights) PSD_FAIL(PSD_EINVAL, err, "%s: weights pointer is null", tag);
    if (m.dtype != PSD_F32 && m.dtype != PSD_BF16) PSD_FAIL(PSD_EINVAL, err, "%s: dtype %d", tag, m.dtype);
    if (m.n_layers < 1 || m.d_model < 32 || m.n_heads < 1 || m.n_kv_heads < 1 || m.d_ffn < 32 || m.vocab < 2)
        PSD_FAIL(PSD_EINVAL, err, "%s: bad shape", tag);
    if (m.d_model % m.n_heads || m.n_heads % m.n_kv_heads || m.d_model % 32 || m.d_ffn % 32)
        PSD_FAIL(PSD_EINVAL, err, "%s: d %% H, H %% KV, d %% 32 and F %% 32 must all be 0", tag);
    const int hd = m.d_model / m.n_heads;
    if (hd != 16 && hd != 32 && hd != 64 && hd != 128) PSD_FAIL(PSD_EINVAL, err, "%s: head dim %d not in {16,32,64,128}", tag, hd);
    if (m.dtype == PSD_BF16 && hd == 16) PSD_FAIL(PSD_EINVAL, err, "%s: bf16 models need a head dim of 32, 64 or 128", tag);
    if (!(m.rope_theta > 0.f) || !(m.rms_eps >= 0.f)) PSD_FAIL(PSD_EINVAL, err, "%s: rope_theta / rms_eps", tag);
    if (m.weights_bytes != blob_elems(m) * esize(m.dtype))
        PSD_FAIL(PSD_EINVAL, err, "%s: weights_bytes %zu, shape implies %zu", tag, m.weights_bytes, blob_elems(m) * esize(m.dtype));
    model_shape(M, m, max_seq);
    M.tag = tag;
    int rc = model_carve(M, pool);
    if (rc != PSD_OK) PSD_FAIL(PSD_ENOMEM, err, "%s: device pool too small (%zu bytes needed so far)", tag, pool.used);

    const bool bf = M.dtype == PSD_BF16;
    const size_t es = esize(M.dtype);
    const size_t q = (size_t)M.H * M.hd, d = M.d, F = M.F;
    const size_t biggest = std::max({(size_t)M.V * d, 2 * F * d, (size_t)M.nqkv * d});
    void* stage = nullptr;
    PSD_HIP(hipMalloc(&stage, biggest * es), err);
    struct Guard { void* p; ~Guard() { (void)hipFree(p); } } guard{stage};
    const char* src = (const char*)m.weights;
    // uploads `rows x cols` elements from the blob into dst, re-tiled when bf16
    auto put_matrix = [&](const void* dst, size_t rows, size_t cols, int mode = 0, int hd_arg = 0) -> int {
        const size_t bytes = rows * cols * es;
        if (bf) {
            PSD_HIP(hipMemcpyAsync(stage, src, bytes, hipMemcpyHostToDevice, stream), err);
            const size_t chunks = (size_t)round16((int)rows) / 16 * (cols / 32) * 64;
            tile_bf16<<<(unsigned)((chunks + 255) / 256), 256, 0, stream>>>((const uint4*)stage, (uint4*)dst, (int)rows, (int)cols, chunks, mode, hd_arg);
            PSD_HIP(hipStreamSynchronize(stream), err);  // the staging buffer is reused by the next tensor
        } else {
            PSD_HIP(hipMemcpyAsync((void*)dst, src, bytes, hipMemcpyHostToDevice, stream), err);
            PSD_HIP(hipStreamSynchronize(stream), err);
        }
        src += bytes;
        M.weight_bytes += bytes;
        return PSD_OK;
    };
    auto put_norm = [&](const float* dst) -> int {
        const size_t bytes = d * es;
        if (bf) {
            PSD_HIP(hipMemcpyAsync(stage, src, bytes, hipMemcpyHostToDevice, stream), err);
            bf16_to_f32_vec<<<(unsigned)((d + 255) / 256), 256, 0, stream>>>((const uint16_t*)stage, (float*)dst, (int)d);
            PSD_HIP(hipStreamSynchronize(stream), err);
        } else {
            PSD_HIP(hipMemcpyAsync((void*)dst, src, bytes, hipMemcpyHostToDevice, stream), err);
            PSD_HIP(hipStreamSynchronize(stream), err);
        }
        src += bytes;
        return PSD_OK;
    };
    M.weight_bytes = 0;
    if ((rc = put_matrix(M.embed, M.V, d)) != PSD_OK) return rc;
    for (int l = 0; l < M.L; ++l) {
        LayerW& w = M.layers[l];
        if ((rc = put_norm(w.attn_norm)) != PSD_OK) return rc;
        if ((rc = put_matrix(w.wqkv, M.nqkv, d, bf ? 1 : 0, M.hd)) != PSD_OK) return rc;  // wq, wk, wv are adjacent in the blob
        if ((rc = put_matrix(w.wo, d, q)) != PSD_OK) return rc;
        if ((rc = put_norm(w.ffn_norm)) != PSD_OK) return rc;
        if ((rc = put_matrix(w.wgu, 2 * F, d, bf ? 2 : 0, (int)F)) != PSD_OK) return rc;   // w_gate, w_up adjacent
        if ((rc = put_matrix(w.wd, d, F)) != PSD_OK) return rc;
    }
    if ((rc = put_norm(M.final_norm)) != PSD_OK) return rc;
    const int half = M.hd / 2, n_tab = M.max_seq * half;
    rope_table<<<(n_tab + 255) / 256, 256, 0, stream>>>((float2*)M.rope, M.max_seq, half, (double)M.theta);
    // scratch starts zeroed so that never-written operand columns hold finite values
    const size_t kmax = std::max(d, F);
    PSD_HIP(hipMemsetAsync(M.xb, 0, kmax * 128, stream), err);
    PSD_HIP(hipMemsetAsync(M.x, 0, (size_t)kCols * d * sizeof(float), stream), err);
    PSD_HIP(hipMemsetAsync(M.qkv, 0, (size_t)kCols * M.nqkv * sizeof(float), stream), err);
    PSD_HIP(hipMemsetAsync(M.gu, 0, (size_t)kMaxW * 2 * F * sizeof(float), stream), err);
    PSD_HIP(hipMemsetAsync(M.desc, 0, sizeof(PassDesc), stream), err);
    // KV pages start as zeros: attention may read (and mask) slots of a page that were never written
    PSD_HIP(hipMemsetAsync(M.kv, 0, (size_t)M.n_pages * M.L * M.KV * 2 * kPage * M.hd * 4, stream), err);
    if (bf) {
        PSD_HIP(hipMemsetAsync(M.xb2, 0, kmax * 128, stream), err);
        PSD_HIP(hipMemsetAsync(M.ss, 0, (size_t)(M.d / 16) * 32 * sizeof(float), stream), err);
        PSD_HIP(hipMemsetAsync(M.xbw, 0, kmax * 4 * kCols, stream), err);
        PSD_HIP(hipMemsetAsync(M.xbw2, 0, kmax * 4 * kCols, stream), err);
        PSD_HIP(hipMemsetAsync(M.ssw, 0, (size_t)(M.d / 16) * kCols * sizeof(float), stream), err);
    }
    // page bookkeeping: every logical block unmapped, free list in (optionally scrambled) order
    M.h_page_table.assign(M.n_pages, -1);
    M.free_pages.clear();
    for (int p = M.n_pages - 1; p >= 0; --p) M.free_pages.push_back(p);
    if (scramble_pages) {  // deterministic shuffle: physical pages no longer follow logical order
        uint64_t s = 0x9E3779B97F4A7C15ull;
        for (int i = M.n_pages - 1; i > 0; --i) {
            s = s * 6364136223846793005ull + 1442695040888963407ull;
            std::swap(M.free_pages[i], M.free_pages[(s >> 33) % (uint64_t)(i + 1)]);
        }
    }
    M.pages_mapped = 0;
    M.len = 0;
    PSD_HIP(hipStreamSynchronize(stream), err);
    PSD_HIP(hipGetLastError(), err);
    return PSD_OK;
}

int model_map_pages(Model& M, int keep, int upto, int* first_changed, int* n_changed, char* err) {
    *first_changed = 0;
    *n_changed = 0;
    if (upto > M.max_seq) PSD_FAIL(PSD_ESHAPE, err, "%s: position %d exceeds max_seq %d", M.tag, upto, M.max_seq);
    const int need = (upto + kPage - 1) / kPage, keep_pages = (keep + kPage - 1) / kPage;
    int lo = M.n_pages, hi = 0;
    // rollback: blocks wholly beyond the kept prefix go back to the free list (unless needed again right away)
    for (int b = M.pages_mapped - 1; b >= std::max(keep_pages, need); --b) {
        M.free_pages.push_back(M.h_page_table[b]);
        M.h_page_table[b] = -1;
        M.pages_mapped = b;
        lo = std::min(lo, b); hi = std::max(hi, b + 1);
    }
    for (int b = M.pages_mapped; b < need; ++b) {
        if (M.free_pages.empty()) PSD_FAIL(PSD_ENOMEM, err, "%s: out of KV pages", M.tag);
        M.h_page_table[b] = M.free_pages.back();
        M.free_pages.pop_back();
        M.pages_mapped = b + 1;
        lo = std::min(lo, b); hi = std::max(hi, b + 1);
    }
    if (hi > lo) { *first_changed = lo; *n_changed = hi - lo; }
    return PSD_OK;
}

// ---- forward ----------------------------------------------------------------------------------------
namespace {
struct Launch {
    Model& M;
    hipStream_t s;
    Profiler* prof;
    int wcls;  // launch class: one of kNarrowClasses, or a multiple of 128
    char name[48];
    void begin(const char* family, double bytes) {
        if (!prof || !prof->on) return;
        snprintf(name, sizeof(name), "%s %s w<=%d", family, M.tag, wcls);
        prof->begin(s, prof->row_of(name), bytes);
    }
    void end() {
        if (prof && prof->on) prof->end(s);
    }
};
}  // namespace

// fp32 models: unfused pipeline, plain VALU GEMM
template <int EPI>
static void launch_gemm_f32(Launch& L, const char* family, const void* W, float* Y, int N, int K, int ldy) {
    Model& M = L.M;
    L.begin(family, (double)N * K * 4);
    gemm_f32<EPI><<<(N + 3) / 4, 256, 0, L.s>>>((const float*)W, (const float*)M.xb, Y, N, K, ldy, M.desc);
    L.end();
}

static int forward_f32(Model& M, int wmax, float* logits, Launch& L) {
    hipStream_t stream = L.s;
    const int d = M.d, F = M.F, H = M.H, KV = M.KV, hd = M.hd;
    const double act = (double)wmax * d * 4;
    L.begin("embed", act);
    embed_rows<false><<<wmax, 256, 0, stream>>>(M.embed, M.desc, M.x, d, M.V);
    L.end();
    const int lds = attn_lds_bytes(hd);
    for (int l = 0; l < M.L; ++l) {
        const LayerW& w = M.layers[l];
        L.begin("rmsnorm", act);
        rmsnorm_pack<false><<<wmax, 256, 0, stream>>>(M.x, w.attn_norm, M.desc, M.xb, d, M.eps);
        L.end();
        launch_gemm_f32<EPI_STORE>(L, "gemm_qkv", w.wqkv, M.qkv, M.nqkv, d, M.nqkv);
        L.begin("rope_kv", (double)wmax * M.nqkv * 4);
        rope_kv<float><<<dim3(wmax, H + 2 * KV), hd / 2, 0, stream>>>(M.qkv, M.desc, M.rope, (float*)M.kv, M.page_table, l, M.L, H, KV, hd, M.nqkv);
        L.end();
        L.begin("attn", (double)std::min(M.max_seq, M.len + wmax) * KV * hd * 2 * 4 + (double)wmax * H * hd * 4 * 2);
        attn_partial<float><<<dim3(H, M.nsplit_max), 256, lds, stream>>>(M.qkv, M.desc, (const float*)M.kv, M.page_table, M.attn_part, l, M.L, H, KV, hd, M.nqkv);
        L.end();
        L.begin("attn_combine", act);
        attn_combine_pack<false><<<dim3(wmax, H), hd, 0, stream>>>(M.attn_part, M.desc, M.xb, H, hd);
        L.end();
        launch_gemm_f32<EPI_RESID>(L, "gemm_o", w.wo, M.x, d, H * hd, d);
        L.begin("rmsnorm", act);
        rmsnorm_pack<false><<<wmax, 256, 0, stream>>>(M.x, w.ffn_norm, M.desc, M.xb, d, M.eps);
        L.end();
        launch_gemm_f32<EPI_STORE>(L, "gemm_gate_up", w.wgu, M.gu, 2 * F, d, 2 * F);
        L.begin("swiglu", (double)wmax * 2 * F * 4);
        swiglu_pack<false><<<dim3(wmax, (F + 255) / 256), 256, 0, stream>>>(M.gu, M.desc, M.xb, F);
        L.end();
        launch_gemm_f32<EPI_RESID>(L, "gemm_down", w.wd, M.x, d, F, d);
    }
    if (logits) {
        L.begin("rmsnorm", act);
        rmsnorm_pack<false><<<wmax, 256, 0, stream>>>(M.x, M.final_norm, M.desc, M.xb, d, M.eps);
        L.end();
        launch_gemm_f32<EPI_LOGITS>(L, "gemm_lm_head", M.embed, logits, M.V, d, M.V);
    }
    return PSD_OK;
}

// bf16 models: five or six launches per layer (q/k/v projection, attention, merge, o, gate/up, down)
template <int EPI>
static void launch_gemm_bf16(Launch& L, const char* family, GemmArgs a) {
    Model& M = L.M;
    const int tiles = round16(a.N) / 16;
    a.desc = M.desc;
    a.wcap = L.wcls;
    L.begin(family, (double)a.N * a.KS * 32 * 2);
    // Waves per workgroup (the K split, hence the summation order) follow from the number of row tiles only, never
    // from the pass width: a token's result must not depend on the width of the pass that computes it.  Row tiles
    // per wave do not change the arithmetic and are picked per width class.
#define PSD_GEMM(NT_, NW_, RT_, CT_) gemm_bf16<NT_, NW_, RT_, EPI, CT_><<<tiles / RT_, 64 * NW_, 0, L.s>>>(a)
    if (L.wcls > 128) {   // several column groups of 128: weights and operand shared through LDS
        if constexpr (EPI != EPI_LOGITS) {
            // NW: the K split of the narrow kernels.  Column groups of 64 where groups of 128 would leave CUs idle.
            const int rg = (tiles + 15) / 16, rg8 = (rg + 7) / 8 * 8;
            if (rg * (L.wcls / 128) >= 192) {
                const int ncg = L.wcls / 128;
                if (tiles <= 256) gemm_panel<16, EPI, 4><<<rg8 * ncg, 512, 0, L.s>>>(a, tiles, ncg);
                else gemm_panel<8, EPI, 4><<<rg8 * ncg, 512, 0, L.s>>>(a, tiles, ncg);
            } else {
                const int ncg = L.wcls / 64;
                if (tiles <= 256) gemm_panel<16, EPI, 2><<<rg8 * ncg, 512, 0, L.s>>>(a, tiles, ncg);
                else gemm_panel<8, EPI, 2><<<rg8 * ncg, 512, 0, L.s>>>(a, tiles, ncg);
            }
        }
    } else if (L.wcls > 32) {   // 128 columns: every weight block is used 8 times as often, so more row tiles share an operand load
        if (tiles <= 256) {
            // two row tiles per wave only where the workgroup's LDS stays under 64 KB (no sum-of-squares table)
            if (EPI == EPI_RESID && tiles % 2 == 0) PSD_GEMM(8, 16, 2, kWideCT); else PSD_GEMM(8, 16, 1, kWideCT);
        } else if (tiles % 4 == 0) {
            PSD_GEMM(8, 8, 4, kWideCT);
        } else if (tiles % 2 == 0) {
            PSD_GEMM(8, 8, 2, kWideCT);
        } else {
            PSD_GEMM(8, 8, 1, kWideCT);
        }
    } else {
        const bool wide = L.wcls > 16;
        bool done = false;
        if constexpr (EPI == EPI_SWIGLU) {   // shapes measured one by one; only the gate/up kernels have such variants
            if (tiles % 7 == 0 && tiles / 7 >= 256) {
                // one workgroup per CU for the target's gate/up projection (1792 tiles): 44 us against 47
                if (wide) PSD_GEMM(2, 8, 7, 2); else PSD_GEMM(1, 8, 7, 2);
                done = true;
            } else if (!wide && tiles == 1024 && a.KS >= 96) {
                PSD_GEMM(1, 8, 4, 2);   // likewise the qualifier's (1024 tiles, K 3072): 20.2 us against 21.1; not for K 2048
                done = true;
            }
        }
        // passes of at most 4 tokens: the operand of a wave's whole K range is staged in LDS, 512 bytes per K step and wave
        const int nw = tiles <= 256 ? 16 : 8;
        const int lb_slots = 64 * (((a.KS + nw - 1) / nw + 1) / 2);
        const size_t lb_bytes = (size_t)nw * lb_slots * sizeof(u32x4);
        // Measured on the draft's shapes: long K ranges gain (down projection, 16 steps per wave: 14.3 -> 13.3 us) and
        // so does the LM head (89.6 -> 86.4 us); ranges of 4 or 8 steps lose 0.2 us to the wait for the staged blocks
        constexpr bool kHasLb = EPI == EPI_RESID || EPI == EPI_LOGITS;
        const bool lb = kHasLb && L.wcls <= 4 && lb_bytes <= kLbMaxBytes && (EPI == EPI_LOGITS || (a.KS + nw - 1) / nw >= 12);
        a.lb_slots = lb_slots;
#define PSD_GEMM_LB(NW_, RT_)                                                                                      \
    do {                                                                                                           \
        if constexpr (kHasLb) gemm_bf16<1, NW_, RT_, EPI, 2, true><<<tiles / RT_, 64 * NW_, lb_bytes, L.s>>>(a);   \
    } while (0)
        // one column tile, at most 7 K steps per wave: the variant that asks for a wave's whole range at once
        const bool short_k = !wide && !lb && (a.KS + 15) / 16 <= 7 && (EPI == EPI_RESID || EPI == EPI_QKV);
        if (done) {
        } else if (tiles <= 256) {
            if (lb) PSD_GEMM_LB(16, 1);
            else if (wide) PSD_GEMM(2, 16, 1, 2);
            else if (short_k) {
                if constexpr (EPI == EPI_RESID || EPI == EPI_QKV) gemm_bf16<1, 16, 1, EPI, 2, false, true><<<tiles, 64 * 16, 0, L.s>>>(a);
            }
            else PSD_GEMM(1, 16, 1, 2);
        } else if (tiles % 2 == 0) {
            if (lb) PSD_GEMM_LB(8, 2); else if (wide) PSD_GEMM(2, 8, 2, 2); else PSD_GEMM(1, 8, 2, 2);
        } else {
            if (lb) PSD_GEMM_LB(8, 1); else if (wide) PSD_GEMM(2, 8, 1, 2); else PSD_GEMM(1, 8, 1, 2);
        }
#undef PSD_GEMM_LB
    }
#undef PSD_GEMM
    L.end();
}

static int forward_bf16(Model& M, int wmax, float* logits, Launch& L) {
    hipStream_t stream = L.s;
    const int d = M.d, F = M.F, H = M.H, KV = M.KV, hd = M.hd, G = H / KV;
    const double act = (double)wmax * d * 4;
    const float inv_d = 1.0f / (float)d;
    const bool c128 = wmax > 32;   // prompt ingestion: operands with 32 column tiles in their own buffers
    void* xb = c128 ? M.xbw : M.xb;
    void* xb2 = c128 ? M.xbw2 : M.xb2;
    float* ss = c128 ? M.ssw : M.ss;
    L.begin("embed", act);
    if (c128) embed_pack<kWideCT, kWideCT><<<d / 16, 64, 0, stream>>>((const uint16_t*)M.embed, M.desc, M.x, xb, M.layers[0].attn_norm, ss, d, M.V);
    else if (wmax <= 16) embed_pack<1, 2><<<d / 16, 64, 0, stream>>>((const uint16_t*)M.embed, M.desc, M.x, xb, M.layers[0].attn_norm, ss, d, M.V);
    else embed_pack<2, 2><<<d / 16, 64, 0, stream>>>((const uint16_t*)M.embed, M.desc, M.x, xb, M.layers[0].attn_norm, ss, d, M.V);
    L.end();
    // key ranges this launch covers: the bucket of the pass's last position (the caller's bound), never beyond the cache
    const int nsplit = std::min(M.nsplit_max, kCtxBuckets[M.ctx_bucket]);
    // prompt-ingestion passes: four query tiles share one load of the keys and values.  Narrow passes take one tile per
    // workgroup at every context length: since the key and value planes are tiled their loads are cheap enough that more
    // workgroups beat fewer loads (target pass at 4.6 K tokens of context: 3.99 ms with one tile per workgroup, 4.06 ms with
    // the pass's three tiles sharing one load; with the untiled planes it was the other way round beyond 16 key ranges)
    const int qt_per_wg = wmax > kMaxW ? 4 : 1;
    const int qt_max = ((wmax * G + 15) / 16 + qt_per_wg - 1) / qt_per_wg;
    // narrow passes of small models: the o projection merges the attention split partials itself (one launch less).
    // Every workgroup of it repeats the merge, so past a dozen key ranges the separate merge kernel is cheaper
    // (draft o projection at 36 ranges: 19.8 us against 4.2 + 6.5 us); both routes give the same bits.
    // algorithmic bytes of one layer's attention: K and V of every key the pass can see, as bf16 (the cache holds a hi and a
    // lo plane per value, so the kernels move twice that), plus the queries in and the outputs back
    const double kv_bytes = (double)std::min(M.max_seq, M.len + wmax) * KV * hd * 2 * 2 + (double)wmax * H * hd * 4 * 2;
    const bool fold_merge = wmax <= 4 && d <= 2048 && d / 16 <= 256 && H * hd == d && nsplit <= kFoldSplits;
    GemmArgs base{};
    base.ss_in = ss; base.ss_tiles = d / 16; base.inv_d = inv_d; base.eps = M.eps;
    base.rope = M.rope; base.kv = (uint16_t*)M.kv; base.page_table = M.page_table;
    base.L = M.L; base.H = H; base.KV = KV; base.hd = hd;
    for (int l = 0; l < M.L; ++l) {
        const LayerW& w = M.layers[l];
        const float* next_gain = l + 1 < M.L ? M.layers[l + 1].attn_norm : M.final_norm;
        GemmArgs a = base;
        a.Wt = (const u32x4*)w.wqkv; a.XB = (const u32x4*)xb; a.N = M.nqkv; a.KS = d / 32;
        a.Y = M.qkv; a.ldy = M.nqkv; a.layer = l;
        launch_gemm_bf16<EPI_QKV>(L, "gemm_qkv", a);
        L.begin("attn", kv_bytes);
        const dim3 agrid(KV, nsplit, qt_max);
        if (hd == 128) attn_mfma<128><<<agrid, 256, 0, stream>>>(M.qkv, M.desc, (const uint16_t*)M.kv, M.page_table, M.n_pages, M.attn_part, l, M.L, H, KV, M.nqkv, qt_per_wg);
        else if (hd == 64) attn_mfma<64><<<agrid, 256, 0, stream>>>(M.qkv, M.desc, (const uint16_t*)M.kv, M.page_table, M.n_pages, M.attn_part, l, M.L, H, KV, M.nqkv, qt_per_wg);
        else attn_mfma<32><<<agrid, 256, 0, stream>>>(M.qkv, M.desc, (const uint16_t*)M.kv, M.page_table, M.n_pages, M.attn_part, l, M.L, H, KV, M.nqkv, qt_per_wg);
        L.end();
        a = base;
        a.Wt = (const u32x4*)w.wo; a.XB = (const u32x4*)xb2; a.N = d; a.KS = (H * hd) / 32;
        a.Y = M.x; a.ldy = d; a.xb_out = xb; a.gain_out = w.ffn_norm; a.ss_out = ss;
        if (fold_merge) {
            a.desc = M.desc; a.wcap = 4;
            L.begin("gemm_o", (double)d * d * 2);
            gemm_o_narrow<<<d / 16, 1024, 0, stream>>>(a, M.attn_part);
            L.end();
        } else {
            L.begin("attn_combine", act);
            // more than eight key ranges: the form that fetches a row's partials in one round (its LDS need grows with the
            // ranges; the dependent-rounds form takes over where that no longer fits)
            const size_t cmb_lds = (size_t)nsplit * (hd + 3) * sizeof(float);
            if (nsplit > 8 && cmb_lds <= 64 * 1024) {
                if (c128) attn_combine_long<kWideCT><<<dim3(wmax, H), 256, cmb_lds, stream>>>(M.attn_part, M.desc, xb2, H, hd, nsplit);
                else attn_combine_long<2><<<dim3(wmax, H), 256, cmb_lds, stream>>>(M.attn_part, M.desc, xb2, H, hd, nsplit);
            } else if (c128) {
                attn_combine_bf16<kWideCT><<<dim3(wmax, H), hd, 0, stream>>>(M.attn_part, M.desc, xb2, H, hd);
            } else {
                attn_combine_bf16<2><<<dim3(wmax, H), hd, 0, stream>>>(M.attn_part, M.desc, xb2, H, hd);
            }
            L.end();
            launch_gemm_bf16<EPI_RESID>(L, "gemm_o", a);
        }
        a = base;
        a.Wt = (const u32x4*)w.wgu; a.XB = (const u32x4*)xb; a.N = 2 * F; a.KS = d / 32; a.xb_out = xb2;
        launch_gemm_bf16<EPI_SWIGLU>(L, "gemm_gate_up", a);
        a = base;
        a.Wt = (const u32x4*)w.wd; a.XB = (const u32x4*)xb2; a.N = d; a.KS = F / 32;
        a.Y = M.x; a.ldy = d; a.xb_out = xb; a.gain_out = next_gain; a.ss_out = ss;
        launch_gemm_bf16<EPI_RESID>(L, "gemm_down", a);
    }
    if (logits) {
        GemmArgs a = base;
        a.Wt = (const u32x4*)M.embed; a.XB = (const u32x4*)xb; a.N = M.V; a.KS = d / 32; a.Y = logits; a.ldy = M.V;
        launch_gemm_bf16<EPI_LOGITS>(L, "gemm_lm_head", a);
    }
    return PSD_OK;
}

// what an event pair measures around a kernel that does nothing: the share of every profiled interval that is not kernel time
__global__ void empty_kernel() {}

int model_forward(Model& M, int wmax, float* logits, hipStream_t stream, Profiler* prof, char* err) {
    const bool ingest = wmax > kMaxW;
    if (ingest ? (wmax % 128 != 0 || wmax > M.ingest_max) : (narrow_class_index(wmax) < 0 || kNarrowClasses[narrow_class_index(wmax)] != wmax))
        PSD_FAIL(PSD_EINVAL, err, "forward: width class %d", wmax);
    if (ingest && (M.dtype != PSD_BF16 || logits)) PSD_FAIL(PSD_EINVAL, err, "forward: passes wider than %d tokens are for bf16 prompt ingestion only", kMaxW);
    Launch L{M, stream, prof, wmax, {0}};
    int rc = M.dtype == PSD_BF16 ? forward_bf16(M, wmax, logits, L) : forward_f32(M, wmax, logits, L);
    if (rc != PSD_OK) return rc;
    if (prof && prof->on) {
        prof->begin(stream, prof->row_of("empty kernel (event pair only)"), 0.0);
        empty_kernel<<<1, 64, 0, stream>>>();
        prof->end(stream);
    }
    PSD_HIP(hipGetLastError(), err);
    return PSD_OK;
}

}  // namespace psd
