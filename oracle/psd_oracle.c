/* CPU oracle for Pyramid Speculative Decoding (three-model speculative decoding
 * with fuzzy acceptance).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 statement of what the
 * hot path computes, written from the paper and independent of the HIP library:
 * it shares no code with it and is only ever called from tests/, the smoke
 * check and the benchmark's cpu_baseline leg.  Nothing in the product path may
 * call it.
 *
 * What follows the paper, and where:
 *   - two-stage loop: Figure 1 caption (draft l_D tokens, qualifier verifies,
 *     repeat until l_Q tokens exist, target verifies them, the qualifier's
 *     distribution stands in for the draft's in the target comparison);
 *   - acceptance criterion Div(P_verifier, P_proposer) <= tau per stage:
 *     Section 3.1 (definition of beta) and Section 3.2 (two-stage criterion);
 *   - fallback to the standard speculative-sampling probability rule when the
 *     divergence is over the threshold, tau = 0 being standard SD:
 *     Sections 3.1, 3.3 and 3.4;
 *   - "+1" bonus token of a fully accepted window: Section 3.3, factor (l + 1).
 * Readings the paper leaves open (divergence = Jensen-Shannon in nats, sampling
 * by an exponential race driven by Philox4x32-10, temperature applied to the
 * logits of all three models, full vocabulary) are this build's and are the same
 * ones the HIP library documents in its header.
 *
 * Precision: all arithmetic in double.  Weights are read as given (fp32, or
 * bf16 widened exactly); logits cross the acceptance interface as float rows,
 * because that is the interface's type.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------- */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as   */
/* easy as 1, 2, 3", SC'11): 10 rounds, multipliers and Weyl key increments  */
/* of the published generator.                                               */
/* ------------------------------------------------------------------------- */
void orc_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* The generator's output for n consecutive counters (c0 .. c0 + n - 1, c1, c2, c3) under one key:
 * out[i][0..3].  A plain loop over the function above, for comparisons against other implementations. */
void orc_philox_block(uint64_t seed, uint32_t c0, uint32_t n, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t* out) {
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    for (uint32_t i = 0; i < n; ++i) {
        uint32_t ctr[4] = {c0 + i, c1, c2, c3};
        orc_philox4x32_10(ctr, key, out + 4 * (size_t)i);
    }
}

/* Draw addressing.  One uniform per (seed, vocabulary index v, draw position,
 * purpose, stage): counter = (v / 4, position, purpose, stage), word v % 4,
 * key = the 64-bit seed.  u = (top 23 bits + 1/2) / 2^23 lies strictly inside
 * (0, 1) and is exact in both float and double. */
/* Purposes.  SAMPLE = a fresh token from a model's own distribution: the draft's
 * proposals and the bonus token of a fully accepted window both use it, always
 * with stage 0, so that a position decided by a fresh sample sees the same draw
 * whichever model provides the distribution.  COIN and RESAMPLE carry the stage
 * (1 = qualifier judging the draft, 2 = target judging the window). */
enum { ORC_DRAW_SAMPLE = 0, ORC_DRAW_COIN = 1, ORC_DRAW_RESAMPLE = 2 };

double orc_uniform(uint64_t seed, uint32_t v, uint32_t position, uint32_t purpose, uint32_t stage) {
    uint32_t ctr[4] = {v >> 2, position, purpose, stage};
    uint32_t key[2] = {(uint32_t)seed, (uint32_t)(seed >> 32)};
    uint32_t out[4];
    orc_philox4x32_10(ctr, key, out);
    return ((double)(out[v & 3u] >> 9) + 0.5) * (1.0 / 8388608.0);
}

/* ------------------------------------------------------------------------- */
/* Distributions                                                             */
/* ------------------------------------------------------------------------- */

/* p = softmax(logits / temperature): "P_M denotes the logit distribution over
 * the next token" (Section 3.1). */
void orc_softmax(const float* logits, int V, double temperature, double* p) {
    double mx = -INFINITY;
    for (int v = 0; v < V; ++v) {
        double z = (double)logits[v] / temperature;
        if (z > mx) mx = z;
    }
    double s = 0.0;
    for (int v = 0; v < V; ++v) {
        p[v] = exp((double)logits[v] / temperature - mx);
        s += p[v];
    }
    for (int v = 0; v < V; ++v) p[v] /= s;
}

/* Jensen-Shannon divergence in nats, the "Div" of Sections 3.1-3.2:
 * JSD(p, q) = 1/2 KL(p || m) + 1/2 KL(q || m), m = (p + q) / 2, 0 ln 0 := 0. */
double orc_jsd(const double* p, const double* q, int V) {
    double s = 0.0;
    for (int v = 0; v < V; ++v) {
        double m = 0.5 * (p[v] + q[v]);
        if (p[v] > 0.0) s += 0.5 * p[v] * log(p[v] / m);
        if (q[v] > 0.0) s += 0.5 * q[v] * log(q[v] / m);
    }
    return s;
}

/* Categorical sample by exponential race: token = argmax_v w_v / E_v with
 * E_v = -ln u_v iid Exp(1); P(token = v) = w_v / sum(w).  Works on
 * un-normalised weights; ties go to the lowest index; zero weights never win.
 * Returns -1 when no weight is positive.  *gap (optional) receives the relative
 * gap between the best and second-best key. */
int orc_race(const double* w, int V, uint64_t seed, uint32_t position, uint32_t purpose, uint32_t stage,
             double* gap) {
    int best = -1;
    double kb = 0.0, k2 = 0.0;
    for (int v = 0; v < V; ++v) {
        if (!(w[v] > 0.0)) continue;
        double e = -log(orc_uniform(seed, (uint32_t)v, position, purpose, stage));
        double key = w[v] / e;
        if (best < 0 || key > kb) { k2 = kb; kb = key; best = v; }
        else if (key > k2) k2 = key;
    }
    if (gap) *gap = (best >= 0 && kb > 0.0) ? (kb - k2) / kb : 0.0;
    return best;
}

/* Entropy (nats) and largest probability of softmax(logits / temperature): the two per-step
 * statistics of the model-behaviour analysis (Section 4, "Model Behavior Analysis":
 * entropy of the predictive distribution and the maximum predicted probability). */
void orc_row_stats(const float* logits, int V, double temperature, double* entropy, double* max_prob) {
    double* p = (double*)malloc((size_t)V * sizeof(double));
    orc_softmax(logits, V, temperature, p);
    double h = 0.0, mx = 0.0;
    for (int v = 0; v < V; ++v) {
        if (p[v] > 0.0) h -= p[v] * log(p[v]);
        if (p[v] > mx) mx = p[v];
    }
    *entropy = h;
    *max_prob = mx;
    free(p);
}

/* ------------------------------------------------------------------------- */
/* ACCEPT: one verify stage over k proposed tokens                           */
/* ------------------------------------------------------------------------- */

typedef struct {
    int32_t n_accepted;   /* tokens accepted before the first rejection (k if none) */
    int32_t next_token;   /* residual resample (n < k), bonus (n == k and take_bonus) or -1 */
    int32_t n_fuzzy;      /* accepted positions whose divergence was within the threshold */
    int32_t pad;
    double margin_div;    /* min |div_i - T| over the judged positions */
    double margin_coin;   /* min |u_i - p/q| / max(1, p/q) over the positions where the coin decided */
    double margin_race;   /* relative gap of the two best race keys of the sampled token (1 if none drawn) */
} orc_accept_result;

/* Decision core on explicit distributions and explicit coin uniforms.
 * Position i is accepted if Div(p_i, q_i) <= T (Section 3.2, the inequality is
 * non-strict as printed) or, failing that, if the standard speculative-sampling
 * coin succeeds: u_i < p_i(x_i) / q_i(x_i) (Sections 3.1 and 3.4).  The scan
 * stops at the first rejection.  Returns that index (k if none); div[k]
 * receives the divergences of the judged positions (later ones are left
 * untouched), fuzzy (optional) counts threshold accepts. */
int orc_accept_scan(const double* p, const double* q, const int32_t* x, int k, int V, double T,
                    const double* u_coin, double* div, int32_t* fuzzy, double* margin_div, double* margin_coin) {
    if (fuzzy) *fuzzy = 0;
    for (int i = 0; i < k; ++i) {
        const double* pi = p + (size_t)i * V;
        const double* qi = q + (size_t)i * V;
        double d = orc_jsd(pi, qi, V);
        if (div) div[i] = d;
        if (margin_div && fabs(d - T) < *margin_div) *margin_div = fabs(d - T);
        if (d <= T) { if (fuzzy) ++*fuzzy; continue; }
        double ratio = pi[x[i]] / qi[x[i]];
        if (margin_coin) {
            double mc = fabs(u_coin[i] - ratio) / (ratio > 1.0 ? ratio : 1.0);
            if (mc < *margin_coin) *margin_coin = mc;
        }
        if (u_coin[i] < ratio) continue;
        return i;
    }
    return k;
}

/* Un-normalised replacement distribution of a rejected position: the standard speculative-sampling
 * residual r_v = max(0, p_v - q_v) (the fallback rule Section 3.4 names; with it tau = 0 reproduces the
 * verifier's law, Section 3.1). */
void orc_residual(const double* p, const double* q, int V, double* r) {
    for (int v = 0; v < V; ++v) r[v] = p[v] > q[v] ? p[v] - q[v] : 0.0;
}

/* Full stage: softmax both logit stacks at `temperature`, scan, then draw the
 * replacement token: from norm(max(0, p_n - q_n)) at the first rejection n
 * (standard SD residual), or from p_k when every proposal was accepted and
 * take_bonus is set.  The token proposed at row i sits at absolute position
 * position0 + i; all draws of row i are addressed by that position.
 * logits_p: [k+1][V] verifier rows; logits_q: [k][V] proposer rows. */
void orc_accept(const float* logits_p, const float* logits_q, const int32_t* x, int k, int V, double T,
                double temperature, uint64_t seed, uint32_t position0, uint32_t stage, int take_bonus,
                orc_accept_result* res, double* div_out) {
    double* p = (double*)malloc((size_t)(k + 1) * V * sizeof(double));
    double* q = (double*)malloc((size_t)(k > 0 ? k : 1) * V * sizeof(double));
    double* u = (double*)malloc((size_t)(k > 0 ? k : 1) * sizeof(double));
    for (int i = 0; i <= k; ++i) orc_softmax(logits_p + (size_t)i * V, V, temperature, p + (size_t)i * V);
    for (int i = 0; i < k; ++i) {
        orc_softmax(logits_q + (size_t)i * V, V, temperature, q + (size_t)i * V);
        u[i] = orc_uniform(seed, 0u, position0 + (uint32_t)i, ORC_DRAW_COIN, stage); /* drawn even if unused */
    }
    res->margin_div = INFINITY; res->margin_coin = INFINITY; res->margin_race = 1.0;
    int n = orc_accept_scan(p, q, x, k, V, T, u, div_out, &res->n_fuzzy, &res->margin_div, &res->margin_coin);
    if (div_out) /* report the divergence of every proposed position, judged or not */
        for (int i = n + 1; i < k; ++i) div_out[i] = orc_jsd(p + (size_t)i * V, q + (size_t)i * V, V);
    res->n_accepted = n;
    res->next_token = -1;
    if (n < k) {
        double* r = (double*)malloc((size_t)V * sizeof(double));
        const double* pn = p + (size_t)n * V;
        const double* qn = q + (size_t)n * V;
        orc_residual(pn, qn, V, r);
        int t = orc_race(r, V, seed, position0 + (uint32_t)n, ORC_DRAW_RESAMPLE, stage, &res->margin_race);
        if (t < 0) /* no residual mass (cannot happen in exact arithmetic): fall back to p_n */
            t = orc_race(pn, V, seed, position0 + (uint32_t)n, ORC_DRAW_RESAMPLE, stage, &res->margin_race);
        res->next_token = t;
        free(r);
    } else if (take_bonus) {
        res->next_token = orc_race(p + (size_t)k * V, V, seed, position0 + (uint32_t)k, ORC_DRAW_SAMPLE, 0u,
                                   &res->margin_race);
    }
    free(p); free(q); free(u);
}

int orc_sample_row(const float* logits, int V, double temperature, uint64_t seed, uint32_t position,
                   uint32_t purpose, uint32_t stage, double* gap);

/* Assisted stage (Section 3.4; strict matching as described in Sections 3.1-3.2):
 * proposal i is accepted iff it equals the verifier's top prediction
 * argmax_v logits_p[i][v] (lowest index among equal maxima); no threshold, no
 * coin.  At the first mismatch n the replacement token is drawn from the
 * verifier's own distribution softmax(logits_p[n] / temperature), not from a
 * residual; a fully accepted run takes the bonus token from row k as in the
 * fuzzy stage.  The draws are addressed like those of orc_accept. */
void orc_accept_assisted(const float* logits_p, const int32_t* x, int k, int V, double temperature, uint64_t seed,
                         uint32_t position0, uint32_t stage, int take_bonus, orc_accept_result* res) {
    res->margin_div = INFINITY; res->margin_coin = INFINITY; res->margin_race = 1.0;
    res->n_fuzzy = 0; res->pad = 0; res->next_token = -1;
    int n = 0;
    for (; n < k; ++n) {
        const float* row = logits_p + (size_t)n * V;
        int top = 0;
        for (int v = 1; v < V; ++v) if (row[v] > row[top]) top = v;
        if (x[n] != top) break;
    }
    res->n_accepted = n;
    if (n < k)
        res->next_token = orc_sample_row(logits_p + (size_t)n * V, V, temperature, seed, position0 + (uint32_t)n,
                                         ORC_DRAW_RESAMPLE, stage, &res->margin_race);
    else if (take_bonus)
        res->next_token = orc_sample_row(logits_p + (size_t)k * V, V, temperature, seed, position0 + (uint32_t)k,
                                         ORC_DRAW_SAMPLE, 0u, &res->margin_race);
}

static int row_argmax(const float* row, int V) {
    int top = 0;
    for (int v = 1; v < V; ++v) if (row[v] > row[top]) top = v;   /* lowest index among equal maxima */
    return top;
}

/* Greedy stage: the temperature -> 0 limit of the rule (Section 3.1: with tau = 0 the proposer's top
 * prediction has to match the verifier's exactly).  All distributions are one-hot there, so proposal i
 * is accepted iff it equals argmax logits_p[i]; the replacement at the first mismatch n, and the bonus
 * token of a fully accepted run, are the verifier's top predictions of rows n and k.  No random draws. */
void orc_accept_greedy(const float* logits_p, const int32_t* x, int k, int V, int take_bonus, orc_accept_result* res) {
    res->margin_div = INFINITY; res->margin_coin = INFINITY; res->margin_race = 1.0;
    res->n_fuzzy = 0; res->pad = 0; res->next_token = -1;
    int n = 0;
    while (n < k && x[n] == row_argmax(logits_p + (size_t)n * V, V)) ++n;
    res->n_accepted = n;
    if (n < k || take_bonus) res->next_token = row_argmax(logits_p + (size_t)n * V, V);
}

/* Draft proposal: token ~ softmax(logits / temperature) by the race. */
int orc_sample_row(const float* logits, int V, double temperature, uint64_t seed, uint32_t position,
                   uint32_t purpose, uint32_t stage, double* gap) {
    double* p = (double*)malloc((size_t)V * sizeof(double));
    orc_softmax(logits, V, temperature, p);
    int t = orc_race(p, V, seed, position, purpose, stage, gap);
    free(p);
    return t;
}

/* ------------------------------------------------------------------------- */
/* Llama-style decoder forward with a KV cache.                              */
/* The paper only names the model family (Figure 1, Section 4.1); this is   */
/* the public architecture: token embedding, per layer                       */
/*   x += Wo Attn(RoPE(Wq n1(x)), RoPE(Wk n1(x)), Wv n1(x))                  */
/*   x += Wdown (silu(Wgate n2(x)) * Wup n2(x))                              */
/* final RMSNorm, logits = E h (tied head).  RMSNorm x * rsqrt(mean x^2 +    */
/* eps) * g; rotary embedding pairs (i, i + hd/2) with angle pos*theta^(-2i/hd); */
/* attention scale 1/sqrt(hd), causal, grouped-query (q head h uses kv head  */
/* h / (H / KV)); no biases.                                                 */
/* ------------------------------------------------------------------------- */

typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab;
    double rope_theta, rms_eps;
    int32_t dtype; /* 0 fp32, 1 bf16 */
    int32_t max_seq;
    const void* blob; /* caller-owned, layout: see weight_offsets() */
    double* kcache;   /* [L][max_seq][KV*hd] */
    double* vcache;
    int64_t passes;
} orc_model;

static inline double wload(const void* blob, int dtype, size_t i) {
    if (dtype == 0) return (double)((const float*)blob)[i];
    uint32_t b = (uint32_t)((const uint16_t*)blob)[i] << 16;
    float f;
    memcpy(&f, &b, 4);
    return (double)f;
}

orc_model* orc_model_create(int n_layers, int d_model, int n_heads, int n_kv_heads, int d_ffn, int vocab,
                            double rope_theta, double rms_eps, int dtype, const void* blob, int max_seq) {
    orc_model* m = (orc_model*)calloc(1, sizeof(orc_model));
    m->n_layers = n_layers; m->d_model = d_model; m->n_heads = n_heads; m->n_kv_heads = n_kv_heads;
    m->d_ffn = d_ffn; m->vocab = vocab; m->rope_theta = rope_theta; m->rms_eps = rms_eps;
    m->dtype = dtype; m->blob = blob; m->max_seq = max_seq;
    size_t kvw = (size_t)n_kv_heads * (d_model / n_heads);
    m->kcache = (double*)malloc((size_t)n_layers * max_seq * kvw * sizeof(double));
    m->vcache = (double*)malloc((size_t)n_layers * max_seq * kvw * sizeof(double));
    return m;
}

void orc_model_destroy(orc_model* m) {
    if (!m) return;
    free(m->kcache); free(m->vcache); free(m);
}

/* y[c][n] = sum_k W[n][k] x[c][k], W row-major [N][K] at element offset off */
static void matmul(const orc_model* m, size_t off, int N, int K, const double* x, int w, double* y) {
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int c = 0; c < w; ++c) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) s += wload(m->blob, m->dtype, off + (size_t)n * K + k) * x[(size_t)c * K + k];
            y[(size_t)c * N + n] = s;
        }
    }
}

static void rmsnorm(const orc_model* m, size_t goff, const double* x, int w, int d, double* y) {
    for (int c = 0; c < w; ++c) {
        double ss = 0.0;
        for (int i = 0; i < d; ++i) ss += x[(size_t)c * d + i] * x[(size_t)c * d + i];
        double r = 1.0 / sqrt(ss / d + m->rms_eps);
        for (int i = 0; i < d; ++i) y[(size_t)c * d + i] = x[(size_t)c * d + i] * r * wload(m->blob, m->dtype, goff + i);
    }
}

void orc_rope(double* v, int n_heads, int hd, int pos, double theta) {
    int half = hd / 2;
    for (int h = 0; h < n_heads; ++h)
        for (int i = 0; i < half; ++i) {
            double ang = (double)pos * pow(theta, -2.0 * i / hd);
            double c = cos(ang), s = sin(ang);
            double a = v[h * hd + i], b = v[h * hd + i + half];
            v[h * hd + i] = a * c - b * s;
            v[h * hd + i + half] = b * c + a * s;
        }
}

/* Runs `w` tokens occupying positions pos0 .. pos0+w-1; rows < pos0 of the KV
 * cache must hold the prefix.  logits (optional) receives [w][V] doubles. */
int orc_forward(orc_model* m, const int32_t* tokens, int w, int pos0, double* logits) {
    int d = m->d_model, H = m->n_heads, KV = m->n_kv_heads, hd = d / H, F = m->d_ffn, V = m->vocab;
    int qw = H * hd, kvw = KV * hd, G = H / KV;
    if (w <= 0 || pos0 < 0 || pos0 + w > m->max_seq) return -1;
    for (int c = 0; c < w; ++c) if (tokens[c] < 0 || tokens[c] >= V) return -2;
    double* x = (double*)malloc((size_t)w * d * sizeof(double));
    double* xn = (double*)malloc((size_t)w * d * sizeof(double));
    double* q = (double*)malloc((size_t)w * qw * sizeof(double));
    double* kk = (double*)malloc((size_t)w * kvw * sizeof(double));
    double* vv = (double*)malloc((size_t)w * kvw * sizeof(double));
    double* att = (double*)malloc((size_t)w * qw * sizeof(double));
    double* o = (double*)malloc((size_t)w * d * sizeof(double));
    double* g = (double*)malloc((size_t)w * F * sizeof(double));
    double* u = (double*)malloc((size_t)w * F * sizeof(double));
    for (int c = 0; c < w; ++c)
        for (int i = 0; i < d; ++i) x[(size_t)c * d + i] = wload(m->blob, m->dtype, (size_t)tokens[c] * d + i);
    size_t off = (size_t)V * d;
    for (int l = 0; l < m->n_layers; ++l) {
        size_t o_an = off; off += d;
        size_t o_wq = off; off += (size_t)qw * d;
        size_t o_wk = off; off += (size_t)kvw * d;
        size_t o_wv = off; off += (size_t)kvw * d;
        size_t o_wo = off; off += (size_t)d * qw;
        size_t o_fn = off; off += d;
        size_t o_wg = off; off += (size_t)F * d;
        size_t o_wu = off; off += (size_t)F * d;
        size_t o_wd = off; off += (size_t)d * F;
        double* kc = m->kcache + (size_t)l * m->max_seq * kvw;
        double* vc = m->vcache + (size_t)l * m->max_seq * kvw;
        /* attention block */
        rmsnorm(m, o_an, x, w, d, xn);
        matmul(m, o_wq, qw, d, xn, w, q);
        matmul(m, o_wk, kvw, d, xn, w, kk);
        matmul(m, o_wv, kvw, d, xn, w, vv);
        for (int c = 0; c < w; ++c) {
            orc_rope(q + (size_t)c * qw, H, hd, pos0 + c, m->rope_theta);
            orc_rope(kk + (size_t)c * kvw, KV, hd, pos0 + c, m->rope_theta);
            memcpy(kc + (size_t)(pos0 + c) * kvw, kk + (size_t)c * kvw, kvw * sizeof(double));
            memcpy(vc + (size_t)(pos0 + c) * kvw, vv + (size_t)c * kvw, kvw * sizeof(double));
        }
        /* every (token, head) pair is independent; the threads only share read-only data (speed, not arithmetic) */
#pragma omp parallel for collapse(2) schedule(dynamic)
        for (int c = 0; c < w; ++c) {
            for (int h = 0; h < H; ++h) {
                int nk = pos0 + c + 1; /* causal: keys 0 .. own position */
                double* sc = (double*)malloc((size_t)nk * sizeof(double));
                int kvh = h / G;
                const double* qh = q + (size_t)c * qw + (size_t)h * hd;
                double mx = -INFINITY;
                for (int t = 0; t < nk; ++t) {
                    double s = 0.0;
                    for (int i = 0; i < hd; ++i) s += qh[i] * kc[(size_t)t * kvw + (size_t)kvh * hd + i];
                    sc[t] = s / sqrt((double)hd);
                    if (sc[t] > mx) mx = sc[t];
                }
                double den = 0.0;
                for (int t = 0; t < nk; ++t) { sc[t] = exp(sc[t] - mx); den += sc[t]; }
                for (int i = 0; i < hd; ++i) {
                    double a = 0.0;
                    for (int t = 0; t < nk; ++t) a += sc[t] * vc[(size_t)t * kvw + (size_t)kvh * hd + i];
                    att[(size_t)c * qw + (size_t)h * hd + i] = a / den;
                }
                free(sc);
            }
        }
        matmul(m, o_wo, d, qw, att, w, o);
        for (size_t i = 0; i < (size_t)w * d; ++i) x[i] += o[i];
        /* feed-forward block */
        rmsnorm(m, o_fn, x, w, d, xn);
        matmul(m, o_wg, F, d, xn, w, g);
        matmul(m, o_wu, F, d, xn, w, u);
        for (size_t i = 0; i < (size_t)w * F; ++i) g[i] = g[i] / (1.0 + exp(-g[i])) * u[i];
        matmul(m, o_wd, d, F, g, w, o);
        for (size_t i = 0; i < (size_t)w * d; ++i) x[i] += o[i];
    }
    if (logits) {
        rmsnorm(m, off, x, w, d, xn);
        matmul(m, 0, V, d, xn, w, logits);
    }
    m->passes++;
    free(x); free(xn); free(q); free(kk); free(vv); free(att); free(o); free(g); free(u);
    return 0;
}

/* ------------------------------------------------------------------------- */
/* The two-stage loop (Figure 1 caption; Sections 3.2-3.3)                   */
/* ------------------------------------------------------------------------- */

typedef struct {
    double T_q, T_t, temperature;
    int32_t k1, k2; /* l_D and l_Q of the paper */
} orc_params;

typedef struct {
    int64_t proposed_q, accepted_q, fuzzy_q; /* stage draft -> qualifier */
    int64_t proposed_t, accepted_t, fuzzy_t; /* stage qualifier -> target */
    int64_t passes_d, passes_q, passes_t;
} orc_stats;

static int imin(int a, int b) { return a < b ? a : b; }

/* Observer for tests: called for every logits row a generation loop consumes, with the model that
 * produced it (0 draft / proposer, 1 qualifier, 2 target), the tokens the row is conditioned on
 * (prefix[0 .. n_prefix - 1], the loop's own sequence buffer) and the row itself.  Lets a test compare what
 * the loop saw, after all its cache rollbacks, with a fresh recomputation of the same prefix. */
typedef void (*orc_row_trace_fn)(void* user, int which, const int32_t* prefix, int n_prefix, const float* row, int V);
static orc_row_trace_fn g_row_trace = NULL;
static void* g_row_trace_user = NULL;
void orc_set_row_trace(orc_row_trace_fn fn, void* user) { g_row_trace = fn; g_row_trace_user = user; }

/* Runs model m over the tokens of seq it has not cached yet, up to index `upto`
 * (exclusive); writes the last n_rows logit rows as floats into rows_out. */
static int run_model(orc_model* m, int which, const int32_t* seq, int* len, int upto, int n_rows, float* rows_out) {
    int w = upto - *len, V = m->vocab;
    if (w < 1 || n_rows > w) return -4; /* the caller's cache bookkeeping is out of step with the sequence */
    double* lg = n_rows > 0 ? (double*)malloc((size_t)w * V * sizeof(double)) : NULL;
    int rc = orc_forward(m, seq + *len, w, *len, lg);
    if (rc == 0) {
        for (int j = 0; j < n_rows; ++j)
            for (int v = 0; v < V; ++v) rows_out[(size_t)j * V + v] = (float)lg[(size_t)(w - n_rows + j) * V + v];
        if (g_row_trace)
            for (int j = 0; j < n_rows; ++j)
                g_row_trace(g_row_trace_user, which, seq, upto - n_rows + j + 1, rows_out + (size_t)j * V, V);
        *len = upto;
    }
    free(lg);
    return rc;
}

/* ------------------------------------------------------------------------- */
/* Adaptive controller for (tau_Q, tau_T, l_D, l_Q)                          */
/* The paper only names it (Conclusion and Future Work: controllers that     */
/* adjust divergence thresholds and speculative lengths from the decoding    */
/* context); the rule below is this build's reading, assembled from what the */
/* paper observes: full acceptance invites a longer window and rejection     */
/* cascades a shorter one (Section 4.4), l_D about half of l_Q (Section 4.4), */
/* tau_Q <= tau_T (Section 4.2), thresholds only as loose as acceptance      */
/* needs (the stability / peak-speed trade-off of Section 4.2).  Integer     */
/* arithmetic throughout; thresholds sit on S + 1 positions of a band.       */
/*                                                                           */
/* After every target pass with window k2 and n accepted tokens:             */
/*   n == k2   -> k2 + 1 (at most k2_max);  2 n < k2 -> k2 - 1 (at least     */
/*   k2_min);  k1 = clamp((k2 + 1) / 2, 1, k1_max).                          */
/* Every `period` target passes, per stage, from the tokens proposed (p) and */
/* accepted (a) since the last adjustment:                                   */
/*   8 a >= 7 p -> one position tighter;  2 a < p -> one position looser;    */
/* then tau_Q is lowered position by position while it exceeds tau_T.        */
/* ------------------------------------------------------------------------- */
typedef struct {
    int32_t k2_min, k2_max, k1_max;
    int32_t steps, period; /* S >= 1 positions above the band's minimum; period >= 1 */
    float T_q_min, T_q_max, T_t_min, T_t_max;
} orc_adapt;

typedef struct {
    int32_t k1, k2, s_q, s_t;        /* lengths and threshold positions in force */
    int32_t since;                   /* target passes since the last threshold adjustment */
    int64_t p_q, a_q, p_t, a_t;      /* proposed / accepted per stage since then */
} orc_adapt_state;

/* threshold at position s of the band [lo, hi]: computed in double, rounded once to float (the type thresholds
 * have at the library's boundary) */
double orc_adapt_threshold(float lo, float hi, int s, int steps) {
    return (double)(float)((double)lo + ((double)hi - (double)lo) * (double)s / (double)steps);
}

static int iclamp(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

static int nearest_position(float lo, float hi, double T, int steps) {
    if (!(hi > lo)) return 0;
    double x = (T - (double)lo) / ((double)hi - (double)lo) * steps;
    return iclamp((int)floor(x + 0.5), 0, steps);
}

void orc_adapt_init(const orc_adapt* ad, double T_q, double T_t, int k2, orc_adapt_state* st) {
    memset(st, 0, sizeof(*st));
    st->k2 = iclamp(k2, ad->k2_min, ad->k2_max);
    st->k1 = iclamp((st->k2 + 1) / 2, 1, ad->k1_max);
    st->s_q = nearest_position(ad->T_q_min, ad->T_q_max, T_q, ad->steps);
    st->s_t = nearest_position(ad->T_t_min, ad->T_t_max, T_t, ad->steps);
}

/* one target pass is over: the window was st->k2 long, n_t of it were accepted; stage 1 proposed p_q and accepted
 * a_q draft tokens while the window was filled */
void orc_adapt_step(const orc_adapt* ad, orc_adapt_state* st, int n_t, int64_t p_q, int64_t a_q) {
    int k2 = st->k2;
    st->p_q += p_q; st->a_q += a_q; st->p_t += k2; st->a_t += n_t;
    if (n_t == k2) st->k2 = k2 + 1 > ad->k2_max ? ad->k2_max : k2 + 1;
    else if (2 * n_t < k2) st->k2 = k2 - 1 < ad->k2_min ? ad->k2_min : k2 - 1;
    st->k1 = iclamp((st->k2 + 1) / 2, 1, ad->k1_max);
    if (++st->since < ad->period) return;
    if (st->p_q > 0) {
        if (8 * st->a_q >= 7 * st->p_q) st->s_q = st->s_q > 0 ? st->s_q - 1 : 0;
        else if (2 * st->a_q < st->p_q) st->s_q = st->s_q < ad->steps ? st->s_q + 1 : ad->steps;
    }
    if (8 * st->a_t >= 7 * st->p_t) st->s_t = st->s_t > 0 ? st->s_t - 1 : 0;
    else if (2 * st->a_t < st->p_t) st->s_t = st->s_t < ad->steps ? st->s_t + 1 : ad->steps;
    while (st->s_q > 0 && orc_adapt_threshold(ad->T_q_min, ad->T_q_max, st->s_q, ad->steps) >
                              orc_adapt_threshold(ad->T_t_min, ad->T_t_max, st->s_t, ad->steps))
        st->s_q--;
    st->since = 0; st->p_q = st->a_q = st->p_t = st->a_t = 0;
}

/* Generates exactly n_new tokens after the prompt.  seq = committed tokens
 * followed by the window of qualified tokens; every model holds KV rows for a
 * prefix of seq and, before each pass, ingests whatever it has not cached.
 *
 *   outer iteration (one target pass):
 *     inner rounds until k2 tokens are qualified:
 *        m = min(k1, k2 - qualified); the draft proposes m tokens one at a time,
 *        the qualifier scores them in one pass, ACCEPT with tau_Q; accepted
 *        tokens and the replacement token (if any) join the window together
 *        with the qualifier row each was judged under; the bonus token is only
 *        taken while the window is not full;
 *     the target scores the window in one pass, ACCEPT with tau_T and the
 *     qualifier rows as proposer distributions; the accepted prefix plus the
 *     replacement / bonus token is committed.
 *   After each ACCEPT every cache is cut back to the tokens that survived.
 */
static int generate_loop(orc_model* D, orc_model* Q, orc_model* T, const orc_params* prm, int assisted,
                         const int32_t* prompt, int n_prompt, int n_new, uint64_t seed, int32_t* out_tokens,
                         orc_stats* st, const orc_adapt* ad, int32_t* adapt_log, int adapt_log_cap) {
    int V = T->vocab, k1 = prm->k1, k2 = prm->k2;
    double T_q = prm->T_q, T_t = prm->T_t;
    orc_adapt_state as;
    int k1_top = k1, k2_top = k2, n_logged = 0;   /* largest lengths the run can reach: buffer sizes */
    if (ad) {
        if (ad->k2_min < 1 || ad->k2_max < ad->k2_min || ad->k1_max < 1 || ad->steps < 1 || ad->period < 1 ||
            !(ad->T_q_max >= ad->T_q_min) || !(ad->T_t_max >= ad->T_t_min) || !(ad->T_q_min >= 0) || !(ad->T_t_min >= 0))
            return -1;
        orc_adapt_init(ad, T_q, T_t, k2, &as);
        k1 = as.k1; k2 = as.k2;
        T_q = orc_adapt_threshold(ad->T_q_min, ad->T_q_max, as.s_q, ad->steps);
        T_t = orc_adapt_threshold(ad->T_t_min, ad->T_t_max, as.s_t, ad->steps);
        k1_top = ad->k1_max; k2_top = ad->k2_max;
    }
    if (D->vocab != V || Q->vocab != V || k1 < 1 || k2 < 1 || n_prompt < 1 || n_new < 0) return -1;
    int cap = n_prompt + n_new + k2_top + 2;
    if (cap > D->max_seq || cap > Q->max_seq || cap > T->max_seq) return -3;
    int32_t* seq = (int32_t*)malloc((size_t)cap * sizeof(int32_t));
    float* dl = (float*)malloc((size_t)k1_top * V * sizeof(float));        /* draft rows of this round */
    float* ql = (float*)malloc((size_t)(k1_top + 1) * V * sizeof(float));  /* qualifier rows of this round */
    float* qrows = (float*)malloc((size_t)(k2_top + 1) * V * sizeof(float)); /* qualifier row per window token */
    float* tl = (float*)malloc((size_t)(k2_top + 1) * V * sizeof(float));
    memcpy(seq, prompt, (size_t)n_prompt * sizeof(int32_t));
    memset(st, 0, sizeof(*st));
    int C = n_prompt, lenD = 0, lenQ = 0, lenT = 0, rc = 0;
    /* prefill: everything but the last prompt token, which stays pending */
    if (C > 1) {
        rc |= run_model(D, 0, seq, &lenD, C - 1, 0, NULL);
        rc |= run_model(Q, 1, seq, &lenQ, C - 1, 0, NULL);
        rc |= run_model(T, 2, seq, &lenT, C - 1, 0, NULL);
    }
    orc_accept_result ar;
    while (rc == 0 && C - n_prompt < n_new) {
        int nbuf = 0;
        int64_t pq0 = st->proposed_q, aq0 = st->accepted_q;
        if (ad && adapt_log && n_logged < adapt_log_cap) {   /* parameters this outer iteration runs with */
            int32_t* e = adapt_log + 4 * (size_t)n_logged++;
            e[0] = k1; e[1] = k2; e[2] = as.s_q; e[3] = as.s_t;
        }
        while (nbuf < k2) {
            int m = imin(k1, k2 - nbuf), L = C + nbuf;
            for (int i = 0; i < m; ++i) {
                rc |= run_model(D, 0, seq, &lenD, L + i, 1, dl + (size_t)i * V);
                st->passes_d++;
                seq[L + i] = assisted == 2 ? row_argmax(dl + (size_t)i * V, V)
                                           : orc_sample_row(dl + (size_t)i * V, V, prm->temperature, seed, (uint32_t)(L + i),
                                                            ORC_DRAW_SAMPLE, 0u, NULL);
            }
            rc |= run_model(Q, 1, seq, &lenQ, L + m, m + 1, ql);
            st->passes_q++;
            int bonus = nbuf + m < k2;
            if (assisted == 2)
                orc_accept_greedy(ql, seq + L, m, V, bonus, &ar);
            else if (assisted)
                orc_accept_assisted(ql, seq + L, m, V, prm->temperature, seed, (uint32_t)L, 1u, bonus, &ar);
            else
                orc_accept(ql, dl, seq + L, m, V, T_q, prm->temperature, seed, (uint32_t)L, 1u, bonus, &ar, NULL);
            int n = ar.n_accepted, has_y = ar.next_token >= 0;
            memcpy(qrows + (size_t)nbuf * V, ql, (size_t)(n + has_y) * V * sizeof(float));
            if (has_y) seq[L + n] = ar.next_token;
            nbuf += n + has_y;
            lenQ = imin(lenQ, L + n);
            lenD = imin(lenD, L + n);
            st->proposed_q += m; st->accepted_q += n; st->fuzzy_q += ar.n_fuzzy;
        }
        rc |= run_model(T, 2, seq, &lenT, C + k2, k2 + 1, tl);
        st->passes_t++;
        if (assisted == 2)
            orc_accept_greedy(tl, seq + C, k2, V, 1, &ar);
        else
            orc_accept(tl, qrows, seq + C, k2, V, T_t, prm->temperature, seed, (uint32_t)C, 2u, 1, &ar, NULL);
        int n = ar.n_accepted;
        seq[C + n] = ar.next_token;
        lenT = imin(lenT, C + n); lenQ = imin(lenQ, C + n); lenD = imin(lenD, C + n);
        C += n + 1;
        st->proposed_t += k2; st->accepted_t += n; st->fuzzy_t += ar.n_fuzzy;
        if (ad) {   /* the controller sees this iteration's counts and sets the next iteration's parameters */
            orc_adapt_step(ad, &as, n, st->proposed_q - pq0, st->accepted_q - aq0);
            k1 = as.k1; k2 = as.k2;
            T_q = orc_adapt_threshold(ad->T_q_min, ad->T_q_max, as.s_q, ad->steps);
            T_t = orc_adapt_threshold(ad->T_t_min, ad->T_t_max, as.s_t, ad->steps);
        }
    }
    if (rc == 0) memcpy(out_tokens, seq + n_prompt, (size_t)n_new * sizeof(int32_t));
    free(seq); free(dl); free(ql); free(qrows); free(tl);
    return rc;
}

int orc_generate(orc_model* D, orc_model* Q, orc_model* T, const orc_params* prm, const int32_t* prompt,
                 int n_prompt, int n_new, uint64_t seed, int32_t* out_tokens, orc_stats* st) {
    return generate_loop(D, Q, T, prm, 0, prompt, n_prompt, n_new, seed, out_tokens, st, NULL, NULL, 0);
}

/* The loop under the adaptive controller: prm gives the starting thresholds and window (brought into the
 * controller's ranges), ad the ranges.  adapt_log (optional, [adapt_log_cap][4] ints) receives (k1, k2, position
 * of tau_Q, position of tau_T) of every outer iteration; *n_logged how many were written. */
int orc_generate_adaptive(orc_model* D, orc_model* Q, orc_model* T, const orc_params* prm, const orc_adapt* ad,
                          const int32_t* prompt, int n_prompt, int n_new, uint64_t seed, int32_t* out_tokens,
                          orc_stats* st, int32_t* adapt_log, int adapt_log_cap) {
    if (!ad) return -1;
    return generate_loop(D, Q, T, prm, 0, prompt, n_prompt, n_new, seed, out_tokens, st, ad, adapt_log, adapt_log_cap);
}

/* The assisted variant of the loop (Section 3.4): the qualifier stage matches tokens
 * strictly and falls back to the qualifier's own distribution; tau_Q is unused.  The
 * target stage is unchanged. */
int orc_generate_assisted(orc_model* D, orc_model* Q, orc_model* T, const orc_params* prm, const int32_t* prompt,
                          int n_prompt, int n_new, uint64_t seed, int32_t* out_tokens, orc_stats* st) {
    return generate_loop(D, Q, T, prm, 1, prompt, n_prompt, n_new, seed, out_tokens, st, NULL, NULL, 0);
}

/* Greedy decoding through the loop (temperature -> 0): proposals and replacements are top predictions,
 * both stages match tokens exactly; thresholds, temperature and seed play no part.  The output is the
 * target's own greedy continuation whatever draft and qualifier are. */
int orc_generate_greedy(orc_model* D, orc_model* Q, orc_model* T, const orc_params* prm, const int32_t* prompt,
                        int n_prompt, int n_new, int32_t* out_tokens, orc_stats* st) {
    return generate_loop(D, Q, T, prm, 2, prompt, n_prompt, n_new, 0, out_tokens, st, NULL, NULL, 0);
}

/* Two-model speculative decoding, the comparison the speed-up is quoted against
 * (Section 3.3, first equation, and its fuzzy extension): model P proposes k tokens one
 * at a time, the target scores them in one pass, ACCEPT with threshold tau (tau = 0:
 * standard speculative sampling; tau > 0: fuzzy speculative decoding), the accepted
 * prefix plus the replacement / bonus token is committed.  Draw addressing is that of
 * the three-model loop's target stage (stage 2), so a three-model run whose qualifier
 * stage accepts everything and whose draft equals its qualifier gives the same tokens.
 * passes_d counts the proposer's steps. */
int orc_generate_sd(orc_model* P, orc_model* T, int k, double tau, double temperature, const int32_t* prompt,
                    int n_prompt, int n_new, uint64_t seed, int32_t* out_tokens, orc_stats* st) {
    int V = T->vocab;
    if (P->vocab != V || k < 1 || n_prompt < 1 || n_new < 0) return -1;
    int cap = n_prompt + n_new + k + 2;
    if (cap > P->max_seq || cap > T->max_seq) return -3;
    int32_t* seq = (int32_t*)malloc((size_t)cap * sizeof(int32_t));
    float* pl = (float*)malloc((size_t)k * V * sizeof(float));
    float* tl = (float*)malloc((size_t)(k + 1) * V * sizeof(float));
    memcpy(seq, prompt, (size_t)n_prompt * sizeof(int32_t));
    memset(st, 0, sizeof(*st));
    int C = n_prompt, lenP = 0, lenT = 0, rc = 0;
    if (C > 1) {
        rc |= run_model(P, 0, seq, &lenP, C - 1, 0, NULL);
        rc |= run_model(T, 2, seq, &lenT, C - 1, 0, NULL);
    }
    orc_accept_result ar;
    while (rc == 0 && C - n_prompt < n_new) {
        for (int i = 0; i < k; ++i) {
            rc |= run_model(P, 0, seq, &lenP, C + i, 1, pl + (size_t)i * V);
            st->passes_d++;
            seq[C + i] = orc_sample_row(pl + (size_t)i * V, V, temperature, seed, (uint32_t)(C + i), ORC_DRAW_SAMPLE,
                                        0u, NULL);
        }
        rc |= run_model(T, 2, seq, &lenT, C + k, k + 1, tl);
        st->passes_t++;
        orc_accept(tl, pl, seq + C, k, V, tau, temperature, seed, (uint32_t)C, 2u, 1, &ar, NULL);
        int n = ar.n_accepted;
        seq[C + n] = ar.next_token;
        lenT = imin(lenT, C + n); lenP = imin(lenP, C + n);
        C += n + 1;
        st->proposed_t += k; st->accepted_t += n; st->fuzzy_t += ar.n_fuzzy;
    }
    if (rc == 0) memcpy(out_tokens, seq + n_prompt, (size_t)n_new * sizeof(int32_t));
    free(seq); free(pl); free(tl);
    return rc;
}

/* Plain ancestral sampling from one model with the draft-proposal draws: the
 * law the loop must reproduce when all three models are the same. */
int orc_generate_plain(orc_model* M, double temperature, const int32_t* prompt, int n_prompt, int n_new,
                       uint64_t seed, int32_t* out_tokens) {
    int V = M->vocab, cap = n_prompt + n_new;
    if (cap > M->max_seq) return -3;
    int32_t* seq = (int32_t*)malloc((size_t)cap * sizeof(int32_t));
    float* row = (float*)malloc((size_t)V * sizeof(float));
    memcpy(seq, prompt, (size_t)n_prompt * sizeof(int32_t));
    int len = 0, rc = 0;
    for (int i = 0; i < n_new && rc == 0; ++i) {
        int L = n_prompt + i;
        rc = run_model(M, 0, seq, &len, L, 1, row);
        seq[L] = orc_sample_row(row, V, temperature, seed, (uint32_t)L, ORC_DRAW_SAMPLE, 0u, NULL);
    }
    if (rc == 0) memcpy(out_tokens, seq + n_prompt, (size_t)n_new * sizeof(int32_t));
    free(seq); free(row);
    return rc;
}
