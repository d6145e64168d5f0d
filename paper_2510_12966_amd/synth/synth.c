/* Seeded synthetic-input generator (weights, logits, prompts).
 *
 * Shared by the CPU oracle's tests and by the HIP library's callers: it only
 * manufactures INPUTS.  It holds none of the decoding method's arithmetic
 * (no softmax, divergence, acceptance, attention, or the method's sampling
 * generator): just a stateless counter hash, Box-Muller normals, and the
 * index maps of the synthetic three-model stack.
 *
 * Every value is a pure function of (seed, stream, index), so tensors can be
 * produced in any order, in parallel, and element-by-element for the
 * target-derived small models.
 *
 * Model blob layout (all tensors row-major [out][in], dtype fp32 or bf16):
 *   embed[V][d]
 *   per layer: attn_norm[d], wq[H*hd][d], wk[KV*hd][d], wv[KV*hd][d],
 *              wo[d][H*hd], ffn_norm[d], w_gate[F][d], w_up[F][d], w_down[d][F]
 *   final_norm[d]
 * The LM head is tied to embed.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab;
} synth_shape;

static inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

static inline uint64_t hash3(uint64_t seed, uint64_t stream, uint64_t idx) {
    return mix64(mix64(mix64(seed) ^ (stream * 0xD6E8FEB86659FD93ull)) ^ idx);
}

static inline double u01(uint64_t h) { /* (0,1), 53 bits */
    return ((double)(h >> 11) + 0.5) * (1.0 / 9007199254740992.0);
}

/* standard normal number `idx` of stream `stream` (Box-Muller; idx pairs share a radius) */
static inline double normal_at(uint64_t seed, uint64_t stream, uint64_t idx) {
    uint64_t pair = idx >> 1;
    double u1 = u01(hash3(seed, stream, 2 * pair));
    double u2 = u01(hash3(seed, stream, 2 * pair + 1));
    double r = sqrt(-2.0 * log(u1));
    double a = 6.283185307179586476925286766559 * u2;
    return (idx & 1) ? r * sin(a) : r * cos(a);
}

static inline uint16_t f32_to_bf16(float f) {
    uint32_t x;
    memcpy(&x, &f, 4);
    uint32_t r = x + 0x7FFFu + ((x >> 16) & 1u); /* round to nearest even; inputs are finite */
    return (uint16_t)(r >> 16);
}

static inline void store(void* base, int dtype, size_t i, double v) {
    if (dtype == 0) ((float*)base)[i] = (float)v;
    else ((uint16_t*)base)[i] = f32_to_bf16((float)v);
}

/* ---- plain arrays ------------------------------------------------------- */

void synth_normal_f32(uint64_t seed, uint64_t stream, size_t n, double mean, double sigma, float* out) {
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i) out[i] = (float)(mean + sigma * normal_at(seed, stream, i));
}

/* out = rho * base + sqrt(1-rho^2) * N(0, sigma^2) */
void synth_correlated_f32(uint64_t seed, uint64_t stream, size_t n, double rho, double sigma,
                          const float* base, float* out) {
    double c = sqrt(1.0 - rho * rho);
#pragma omp parallel for schedule(static)
    for (size_t i = 0; i < n; ++i)
        out[i] = (float)(rho * (double)base[i] + c * sigma * normal_at(seed, stream, i));
}

void synth_tokens(uint64_t seed, uint64_t stream, size_t n, int32_t vocab, int32_t* out) {
    for (size_t i = 0; i < n; ++i) out[i] = (int32_t)(hash3(seed, stream, i) % (uint64_t)vocab);
}

/* ---- model blobs -------------------------------------------------------- */

enum { T_EMBED = 0, T_WQ = 1, T_WK = 2, T_WV = 3, T_WO = 4, T_GATE = 5, T_UP = 6, T_DOWN = 7 };

static uint64_t tensor_stream(int layer, int kind) { return (uint64_t)(layer + 1) * 16u + (uint64_t)kind; }

size_t synth_model_elems(const synth_shape* s) {
    size_t d = s->d_model, hd = d / s->n_heads, q = (size_t)s->n_heads * hd, kv = (size_t)s->n_kv_heads * hd,
           F = s->d_ffn;
    size_t per_layer = d + q * d + 2 * kv * d + d * q + d + 2 * F * d + d * F;
    return (size_t)s->vocab * d + (size_t)s->n_layers * per_layer + d;
}

static void fill_ones(void* base, int dtype, size_t off, size_t n) {
    for (size_t i = 0; i < n; ++i) store(base, dtype, off + i, 1.0);
}


/* n consecutive normals of one stream, scaled; one Box-Muller evaluation per pair */
static void fill_normal(void* out, int dtype, size_t off, size_t n, uint64_t seed, uint64_t st, double sigma) {
    size_t pairs = (n + 1) / 2;
#pragma omp parallel for schedule(static)
    for (size_t p = 0; p < pairs; ++p) {
        double u1 = u01(hash3(seed, st, 2 * p));
        double u2 = u01(hash3(seed, st, 2 * p + 1));
        double r = sqrt(-2.0 * log(u1));
        double a = 6.283185307179586476925286766559 * u2;
        store(out, dtype, off + 2 * p, sigma * r * cos(a));
        if (2 * p + 1 < n) store(out, dtype, off + 2 * p + 1, sigma * r * sin(a));
    }
}

/* target: every matrix ~ N(0, sigma^2), gains 1 */
void synth_target_weights(const synth_shape* s, uint64_t seed, double sigma, int dtype, void* out) {
    size_t d = s->d_model, hd = d / s->n_heads, q = (size_t)s->n_heads * hd, kv = (size_t)s->n_kv_heads * hd,
           F = s->d_ffn, V = s->vocab;
    size_t off = 0;
    {
        size_t n = V * d;
        fill_normal(out, dtype, 0, n, seed, tensor_stream(-1, T_EMBED), sigma);
        off += n;
    }
    for (int l = 0; l < s->n_layers; ++l) {
        fill_ones(out, dtype, off, d); off += d;
        size_t sizes[4] = {q * d, kv * d, kv * d, d * q};
        int kinds[4] = {T_WQ, T_WK, T_WV, T_WO};
        for (int t = 0; t < 4; ++t) {
            size_t n = sizes[t];
            fill_normal(out, dtype, off, n, seed, tensor_stream(l, kinds[t]), sigma);
            off += n;
        }
        fill_ones(out, dtype, off, d); off += d;
        int kinds2[3] = {T_GATE, T_UP, T_DOWN};
        for (int t = 0; t < 3; ++t) {
            size_t n = F * d;
            fill_normal(out, dtype, off, n, seed, tensor_stream(l, kinds2[t]), sigma);
            off += n;
        }
    }
    fill_ones(out, dtype, off, d);
}

/* seeded selection of n distinct indices out of N (partial Fisher-Yates), plus a sign each */
static void select_signed(uint64_t seed, uint64_t stream, size_t n, size_t N, int32_t* idx, int8_t* sign) {
    int32_t* perm = (int32_t*)malloc(N * sizeof(int32_t));
    for (size_t i = 0; i < N; ++i) perm[i] = (int32_t)i;
    for (size_t i = 0; i < n; ++i) {
        size_t j = i + (size_t)(hash3(seed, stream, i) % (uint64_t)(N - i));
        int32_t t = perm[i]; perm[i] = perm[j]; perm[j] = t;
        idx[i] = perm[i];
        sign[i] = (hash3(seed, stream ^ 0x5151u, i) & 1u) ? 1 : -1;
    }
    free(perm);
}

/* Small model derived from the target (draft / qualifier):
 *   layer l copies target layer floor(l * L_T / L_s);
 *   each matrix W_s = P_out^T (W_T) P_in + N(0, noise_sigma^2), with P signed column selections:
 *     model-width axis and ffn axis: seeded random distinct indices with random signs;
 *     head axes: q head h -> floor(h*H_T/H_s), kv head g -> floor(g*KV_T/KV_s),
 *                rotary pair j -> j*(hd_T/hd_s) (keeps the rotation frequency), sign +1;
 *   embedding E_s = E_T P_d (no noise), gains 1.
 * map_seed fixes the maps, noise_seed the additive noise; `tag` separates draft from qualifier. */
void synth_derived_weights(const synth_shape* s, const synth_shape* t, uint64_t target_seed, double sigma,
                           uint64_t map_seed, uint64_t noise_seed, double noise_sigma, uint64_t tag,
                           int dtype, void* out) {
    size_t d = s->d_model, hd = d / s->n_heads, H = s->n_heads, KV = s->n_kv_heads, F = s->d_ffn, V = s->vocab;
    size_t dT = t->d_model, hdT = dT / t->n_heads, HT = t->n_heads, KVT = t->n_kv_heads, FT = t->d_ffn;
    size_t q = H * hd, kv = KV * hd, qT = HT * hdT;
    int32_t* pd = (int32_t*)malloc(d * sizeof(int32_t)); int8_t* sd = (int8_t*)malloc(d);
    int32_t* pf = (int32_t*)malloc(F * sizeof(int32_t)); int8_t* sf = (int8_t*)malloc(F);
    select_signed(map_seed, tag * 4 + 0, d, dT, pd, sd);
    select_signed(map_seed, tag * 4 + 1, F, FT, pf, sf);
    /* head-axis maps: row index in the small q / kv projection -> row index in the target's */
    int32_t* pq = (int32_t*)malloc(q * sizeof(int32_t));
    int32_t* pk = (int32_t*)malloc(kv * sizeof(int32_t));
    size_t half = hd / 2, halfT = hdT / 2, stride = hdT / hd;
    for (size_t h = 0; h < H; ++h)
        for (size_t i = 0; i < hd; ++i) {
            size_t j = i % half, hi = i / half;
            pq[h * hd + i] = (int32_t)((h * HT / H) * hdT + hi * halfT + j * stride);
        }
    for (size_t g = 0; g < KV; ++g)
        for (size_t i = 0; i < hd; ++i) {
            size_t j = i % half, hi = i / half;
            pk[g * hd + i] = (int32_t)((g * KVT / KV) * hdT + hi * halfT + j * stride);
        }
    size_t off = 0;
    {
        uint64_t st = tensor_stream(-1, T_EMBED);
#pragma omp parallel for schedule(static)
        for (size_t v = 0; v < V; ++v)
            for (size_t b = 0; b < d; ++b)
                store(out, dtype, v * d + b, sd[b] * sigma * normal_at(target_seed, st, v * dT + (size_t)pd[b]));
        off += V * d;
    }
    for (int l = 0; l < s->n_layers; ++l) {
        int lt = (int)((long)l * t->n_layers / s->n_layers);
        uint64_t nz = (tag << 32) + (uint64_t)(l + 1) * 16u;
        fill_ones(out, dtype, off, d); off += d;
        /* wq, wk, wv: [rows][d] */
        const int32_t* rowmap[3] = {pq, pk, pk};
        size_t rows[3] = {q, kv, kv};
        int kinds[3] = {T_WQ, T_WK, T_WV};
        for (int m = 0; m < 3; ++m) {
            uint64_t st = tensor_stream(lt, kinds[m]);
            const int32_t* rm = rowmap[m];
            size_t R = rows[m];
#pragma omp parallel for schedule(static)
            for (size_t a = 0; a < R; ++a)
                for (size_t b = 0; b < d; ++b) {
                    double w = sd[b] * sigma * normal_at(target_seed, st, (size_t)rm[a] * dT + (size_t)pd[b]);
                    w += noise_sigma * normal_at(noise_seed, nz + (uint64_t)kinds[m], a * d + b);
                    store(out, dtype, off + a * d + b, w);
                }
            off += R * d;
        }
        { /* wo: [d][q] */
            uint64_t st = tensor_stream(lt, T_WO);
#pragma omp parallel for schedule(static)
            for (size_t a = 0; a < d; ++a)
                for (size_t b = 0; b < q; ++b) {
                    double w = sd[a] * sigma * normal_at(target_seed, st, (size_t)pd[a] * qT + (size_t)pq[b]);
                    w += noise_sigma * normal_at(noise_seed, nz + T_WO, a * q + b);
                    store(out, dtype, off + a * q + b, w);
                }
            off += d * q;
        }
        fill_ones(out, dtype, off, d); off += d;
        int kinds2[2] = {T_GATE, T_UP};
        for (int m = 0; m < 2; ++m) { /* [F][d] */
            uint64_t st = tensor_stream(lt, kinds2[m]);
#pragma omp parallel for schedule(static)
            for (size_t a = 0; a < F; ++a)
                for (size_t b = 0; b < d; ++b) {
                    double w = sf[a] * sd[b] * sigma * normal_at(target_seed, st, (size_t)pf[a] * dT + (size_t)pd[b]);
                    w += noise_sigma * normal_at(noise_seed, nz + (uint64_t)kinds2[m], a * d + b);
                    store(out, dtype, off + a * d + b, w);
                }
            off += F * d;
        }
        { /* w_down: [d][F] */
            uint64_t st = tensor_stream(lt, T_DOWN);
#pragma omp parallel for schedule(static)
            for (size_t a = 0; a < d; ++a)
                for (size_t b = 0; b < F; ++b) {
                    double w = sd[a] * sf[b] * sigma * normal_at(target_seed, st, (size_t)pd[a] * FT + (size_t)pf[b]);
                    w += noise_sigma * normal_at(noise_seed, nz + T_DOWN, a * F + b);
                    store(out, dtype, off + a * F + b, w);
                }
            off += d * F;
        }
    }
    fill_ones(out, dtype, off, d);
    free(pd); free(sd); free(pf); free(sf); free(pq); free(pk);
}
