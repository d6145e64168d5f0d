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
// GEMM input X[c][f] (c < 32 tokens, f < K features), bf16 path: [K/32][2 col tiles][hi, lo][64 lanes][8],
// lane = ((f % 32) / 8) * 16 + c % 16: exactly the B operand of v_mfma_f32_16x16x32_bf16.
// fp32 path: plain rows [c][K].
template <bool BF16>
__device__ inline void pack_store(void* xb, int K, int c, int f, float v) {
    if constexpr (BF16) {
        const int ks = f >> 5, g = (f & 31) >> 3, e = f & 7, t = c >> 4, cc = c & 15;
        uint16_t* p = (uint16_t*)xb;
        const size_t base = ((((size_t)ks * 2 + t) * 2) * 64 + g * 16 + cc) * 8 + e;
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

// row-major bf16 [N][K] -> MFMA A-operand tiles [Npad/16][K/32][64][8]; rows >= N become zeros
__global__ __launch_bounds__(256) void tile_bf16(const uint4* src, uint4* dst, int N, int K, size_t n_chunks) {
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_chunks) return;
    const int KS = K >> 5;
    const int lane = (int)(i & 63);
    const size_t t = i >> 6;
    const int ks = (int)(t % KS);
    const int tile = (int)(t / KS);
    const int n = tile * 16 + (lane & 15), k = ks * 32 + (lane >> 4) * 8;
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
        float* out = part + (((size_t)split * kMaxW + c) * H + h) * (hd + 2);
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
    for (int s = 0; s < nsp; ++s) M = fmaxf(M, part[(((size_t)s * kMaxW + c) * H + h) * (hd + 2)]);
    float Lsum = 0.f, o = 0.f;
    for (int s = 0; s < nsp; ++s) {
        const float* pr = part + (((size_t)s * kMaxW + c) * H + h) * (hd + 2);
        const float f = expf(pr[0] - M);
        Lsum += pr[1] * f;
        o += pr[2 + i] * f;
    }
    pack_store<BF16>(xb, H * hd, c, h * hd + i, o / Lsum);
}

// ---- skinny GEMMs -----------------------------------------------------------------------------------
template <int EPI>
__device__ inline void epi_store4(float* Y, int ldy, int N, int n, int c, const PassDesc* desc, f32x4 v) {
    int row = c;
    if constexpr (EPI == EPI_LOGITS) {
        const int first = desc->w - desc->n_logit;
        if (c < first) return;
        row = desc->logit_row0 + c - first;
    }
    float* dst = Y + (size_t)row * ldy + n;
    if constexpr (EPI == EPI_RESID) {
        // ldy and n are multiples of 4 here (model widths are multiples of 32)
        float4 o = *reinterpret_cast<float4*>(dst);
        o.x += v[0]; o.y += v[1]; o.z += v[2]; o.w += v[3];
        *reinterpret_cast<float4*>(dst) = o;
    } else {
        if ((ldy & 3) == 0 && n + 3 < N) {
            *reinterpret_cast<float4*>(dst) = make_float4(v[0], v[1], v[2], v[3]);
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (n + r < N) dst[r] = v[r];
        }
    }
}

// One workgroup (4 waves) per 16 output rows; the waves split K and are summed in wave order.
// Wt: tiled weights [Npad/16][KS][64] x 16 B, XB: packed activations [KS][2][2][64] x 16 B.
template <int NT, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16(const u32x4* __restrict__ Wt, const u32x4* __restrict__ XB,
                                                 float* __restrict__ Y, int N, int KS, int ldy,
                                                 const PassDesc* __restrict__ desc) {
    __shared__ f32x4 red[3][NT][64];
    const int tile = blockIdx.x, wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int k0 = (KS * wave) >> 2, k1 = (KS * (wave + 1)) >> 2;
    const u32x4* a_ptr = Wt + ((size_t)tile * KS + k0) * 64 + lane;
    const u32x4* b_ptr = XB + (size_t)k0 * 256 + lane;
    f32x4 acc[NT];
#pragma unroll
    for (int t = 0; t < NT; ++t) acc[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    constexpr int U = 4;
    int ks = k0;
    for (; ks + U <= k1; ks += U) {
        u32x4 a[U], b[U][NT][2];
#pragma unroll
        for (int u = 0; u < U; ++u) a[u] = __builtin_nontemporal_load(a_ptr + (size_t)u * 64);
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                b[u][t][0] = b_ptr[(size_t)u * 256 + t * 128];
                b[u][t][1] = b_ptr[(size_t)u * 256 + t * 128 + 64];
            }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < NT; ++t) {
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[u]),
                                                                 __builtin_bit_cast(bf16x8, b[u][t][0]), acc[t], 0, 0, 0);
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[u]),
                                                                 __builtin_bit_cast(bf16x8, b[u][t][1]), acc[t], 0, 0, 0);
            }
        a_ptr += (size_t)U * 64;
        b_ptr += (size_t)U * 256;
    }
    for (; ks < k1; ++ks) {
        const u32x4 a = __builtin_nontemporal_load(a_ptr);
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                             __builtin_bit_cast(bf16x8, b_ptr[t * 128]), acc[t], 0, 0, 0);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                             __builtin_bit_cast(bf16x8, b_ptr[t * 128 + 64]), acc[t], 0, 0, 0);
        }
        a_ptr += 64;
        b_ptr += 256;
    }
    if (wave > 0) {
#pragma unroll
        for (int t = 0; t < NT; ++t) red[wave - 1][t][lane] = acc[t];
    }
    __syncthreads();
    if (wave == 0) {
        const int w = desc->w;
        // D operand layout: lane holds rows 4 * (lane / 16) + r, r = 0..3, of column lane % 16
        const int n = tile * 16 + (lane >> 4) * 4;
#pragma unroll
        for (int t = 0; t < NT; ++t) {
            f32x4 v = acc[t];
            v += red[0][t][lane];
            v += red[1][t][lane];
            v += red[2][t][lane];
            const int c = t * 16 + (lane & 15);
            if (c < w && n < N) epi_store4<EPI>(Y, ldy, N, n, c, desc, v);
        }
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

int model_kernels_init(char* err) {
    // attention stages two pages of K and V as fp32 in LDS: up to ~135 KB of the 160 KB a gfx950 CU has
    PSD_HIP(hipFuncSetAttribute((const void*)attn_partial<uint16_t>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                attn_lds_bytes(128)), err);
    PSD_HIP(hipFuncSetAttribute((const void*)attn_partial<float>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                attn_lds_bytes(128)), err);
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
    M.kv = take((size_t)M.n_pages * M.L * M.KV * 2 * kPage * M.hd * es);
    M.page_table = (int32_t*)take((size_t)M.n_pages * sizeof(int32_t));
    const size_t kmax = std::max((size_t)M.d, (size_t)M.F);
    M.x = (float*)take((size_t)kMaxW * M.d * sizeof(float));
    M.xb = take(kmax * 128);
    M.qkv = (float*)take((size_t)kMaxW * M.nqkv * sizeof(float));
    M.gu = (float*)take((size_t)kMaxW * 2 * M.F * sizeof(float));
    M.attn_part = (float*)take((size_t)M.nsplit_max * kMaxW * M.H * (M.hd + 2) * sizeof(float));
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
    auto put_matrix = [&](const void* dst, size_t rows, size_t cols) -> int {
        const size_t bytes = rows * cols * es;
        if (bf) {
            PSD_HIP(hipMemcpyAsync(stage, src, bytes, hipMemcpyHostToDevice, stream), err);
            const size_t chunks = (size_t)round16((int)rows) / 16 * (cols / 32) * 64;
            tile_bf16<<<(unsigned)((chunks + 255) / 256), 256, 0, stream>>>((const uint4*)stage, (uint4*)dst, (int)rows, (int)cols, chunks);
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
        if ((rc = put_matrix(w.wqkv, M.nqkv, d)) != PSD_OK) return rc;  // wq, wk, wv are adjacent in the blob
        if ((rc = put_matrix(w.wo, d, q)) != PSD_OK) return rc;
        if ((rc = put_norm(w.ffn_norm)) != PSD_OK) return rc;
        if ((rc = put_matrix(w.wgu, 2 * F, d)) != PSD_OK) return rc;   // w_gate, w_up adjacent
        if ((rc = put_matrix(w.wd, d, F)) != PSD_OK) return rc;
    }
    if ((rc = put_norm(M.final_norm)) != PSD_OK) return rc;
    const int half = M.hd / 2, n_tab = M.max_seq * half;
    rope_table<<<(n_tab + 255) / 256, 256, 0, stream>>>((float2*)M.rope, M.max_seq, half, (double)M.theta);
    // scratch starts zeroed so that never-written operand columns hold finite values
    const size_t kmax = std::max(d, F);
    PSD_HIP(hipMemsetAsync(M.xb, 0, kmax * 128, stream), err);
    PSD_HIP(hipMemsetAsync(M.x, 0, (size_t)kMaxW * d * sizeof(float), stream), err);
    PSD_HIP(hipMemsetAsync(M.qkv, 0, (size_t)kMaxW * M.nqkv * sizeof(float), stream), err);
    PSD_HIP(hipMemsetAsync(M.gu, 0, (size_t)kMaxW * 2 * F * sizeof(float), stream), err);
    PSD_HIP(hipMemsetAsync(M.desc, 0, sizeof(PassDesc), stream), err);
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

int model_map_pages(Model& M, int keep, int upto, hipStream_t stream, char* err) {
    if (upto > M.max_seq) PSD_FAIL(PSD_ESHAPE, err, "%s: position %d exceeds max_seq %d", M.tag, upto, M.max_seq);
    const int need = (upto + kPage - 1) / kPage, keep_pages = (keep + kPage - 1) / kPage;
    bool changed = false;
    // rollback: blocks wholly beyond the kept prefix go back to the free list (unless needed again right away)
    for (int b = M.pages_mapped - 1; b >= std::max(keep_pages, need); --b) {
        M.free_pages.push_back(M.h_page_table[b]);
        M.h_page_table[b] = -1;
        M.pages_mapped = b;
        changed = true;
    }
    for (int b = M.pages_mapped; b < need; ++b) {
        if (M.free_pages.empty()) PSD_FAIL(PSD_ENOMEM, err, "%s: out of KV pages", M.tag);
        M.h_page_table[b] = M.free_pages.back();
        M.free_pages.pop_back();
        M.pages_mapped = b + 1;
        changed = true;
    }
    if (changed) {
        // unmapped blocks point at page 0 on the device: never read (attention stops at the pass's last position)
        std::vector<int32_t> tmp(M.h_page_table);
        for (auto& v : tmp) if (v < 0) v = 0;
        PSD_HIP(hipMemcpyAsync(M.page_table, tmp.data(), tmp.size() * sizeof(int32_t), hipMemcpyHostToDevice, stream), err);
        PSD_HIP(hipStreamSynchronize(stream), err);  // tmp is pageable host memory on this stack frame
    }
    return PSD_OK;
}

// ---- forward ----------------------------------------------------------------------------------------
namespace {
struct Launch {
    Model& M;
    hipStream_t s;
    Profiler* prof;
    int wcls;  // 16 or 32
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

template <int EPI>
static void launch_gemm(Launch& L, const char* family, const void* W, float* Y, int N, int K, int ldy) {
    Model& M = L.M;
    const double bytes = (double)N * K * esize(M.dtype);
    L.begin(family, bytes);
    if (M.dtype == PSD_BF16) {
        const int tiles = round16(N) / 16;
        if (L.wcls <= 16)
            gemm_bf16<1, EPI><<<tiles, 256, 0, L.s>>>((const u32x4*)W, (const u32x4*)M.xb, Y, N, K / 32, ldy, M.desc);
        else
            gemm_bf16<2, EPI><<<tiles, 256, 0, L.s>>>((const u32x4*)W, (const u32x4*)M.xb, Y, N, K / 32, ldy, M.desc);
    } else {
        gemm_f32<EPI><<<(N + 3) / 4, 256, 0, L.s>>>((const float*)W, (const float*)M.xb, Y, N, K, ldy, M.desc);
    }
    L.end();
}

int model_forward(Model& M, int wmax, float* logits, hipStream_t stream, Profiler* prof, char* err) {
    if (wmax != 16 && wmax != 32) PSD_FAIL(PSD_EINVAL, err, "forward: width class %d", wmax);
    Launch L{M, stream, prof, wmax, {0}};
    const bool bf = M.dtype == PSD_BF16;
    const int d = M.d, F = M.F, H = M.H, KV = M.KV, hd = M.hd;
    const double act = (double)wmax * d * 4;
    L.begin("embed", act);
    if (bf) embed_rows<true><<<wmax, 256, 0, stream>>>(M.embed, M.desc, M.x, d, M.V);
    else embed_rows<false><<<wmax, 256, 0, stream>>>(M.embed, M.desc, M.x, d, M.V);
    L.end();
    const int lds = attn_lds_bytes(hd);
    const double kv_bytes_layer = 0;  // KV traffic depends on the context; attributed by the caller
    (void)kv_bytes_layer;
    for (int l = 0; l < M.L; ++l) {
        const LayerW& w = M.layers[l];
        L.begin("rmsnorm", act);
        if (bf) rmsnorm_pack<true><<<wmax, 256, 0, stream>>>(M.x, w.attn_norm, M.desc, M.xb, d, M.eps);
        else rmsnorm_pack<false><<<wmax, 256, 0, stream>>>(M.x, w.attn_norm, M.desc, M.xb, d, M.eps);
        L.end();
        launch_gemm<EPI_STORE>(L, "gemm_qkv", w.wqkv, M.qkv, M.nqkv, d, M.nqkv);
        L.begin("rope_kv", (double)wmax * M.nqkv * 4);
        if (bf) rope_kv<uint16_t><<<dim3(wmax, H + 2 * KV), hd / 2, 0, stream>>>(M.qkv, M.desc, M.rope, (uint16_t*)M.kv, M.page_table, l, M.L, H, KV, hd, M.nqkv);
        else rope_kv<float><<<dim3(wmax, H + 2 * KV), hd / 2, 0, stream>>>(M.qkv, M.desc, M.rope, (float*)M.kv, M.page_table, l, M.L, H, KV, hd, M.nqkv);
        L.end();
        L.begin("attn", 0);
        if (bf) attn_partial<uint16_t><<<dim3(H, M.nsplit_max), 256, lds, stream>>>(M.qkv, M.desc, (const uint16_t*)M.kv, M.page_table, M.attn_part, l, M.L, H, KV, hd, M.nqkv);
        else attn_partial<float><<<dim3(H, M.nsplit_max), 256, lds, stream>>>(M.qkv, M.desc, (const float*)M.kv, M.page_table, M.attn_part, l, M.L, H, KV, hd, M.nqkv);
        L.end();
        L.begin("attn_combine", act);
        if (bf) attn_combine_pack<true><<<dim3(wmax, H), hd, 0, stream>>>(M.attn_part, M.desc, M.xb, H, hd);
        else attn_combine_pack<false><<<dim3(wmax, H), hd, 0, stream>>>(M.attn_part, M.desc, M.xb, H, hd);
        L.end();
        launch_gemm<EPI_RESID>(L, "gemm_o", w.wo, M.x, d, H * hd, d);
        L.begin("rmsnorm", act);
        if (bf) rmsnorm_pack<true><<<wmax, 256, 0, stream>>>(M.x, w.ffn_norm, M.desc, M.xb, d, M.eps);
        else rmsnorm_pack<false><<<wmax, 256, 0, stream>>>(M.x, w.ffn_norm, M.desc, M.xb, d, M.eps);
        L.end();
        launch_gemm<EPI_STORE>(L, "gemm_gate_up", w.wgu, M.gu, 2 * F, d, 2 * F);
        L.begin("swiglu", (double)wmax * 2 * F * 4);
        if (bf) swiglu_pack<true><<<dim3(wmax, (F + 255) / 256), 256, 0, stream>>>(M.gu, M.desc, M.xb, F);
        else swiglu_pack<false><<<dim3(wmax, (F + 255) / 256), 256, 0, stream>>>(M.gu, M.desc, M.xb, F);
        L.end();
        launch_gemm<EPI_RESID>(L, "gemm_down", w.wd, M.x, d, F, d);
    }
    if (logits) {
        L.begin("rmsnorm", act);
        if (bf) rmsnorm_pack<true><<<wmax, 256, 0, stream>>>(M.x, M.final_norm, M.desc, M.xb, d, M.eps);
        else rmsnorm_pack<false><<<wmax, 256, 0, stream>>>(M.x, M.final_norm, M.desc, M.xb, d, M.eps);
        L.end();
        launch_gemm<EPI_LOGITS>(L, "gemm_lm_head", M.embed, logits, M.V, d, M.V);
    }
    PSD_HIP(hipGetLastError(), err);
    return PSD_OK;
}

}  // namespace psd
