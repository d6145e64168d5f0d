/* psd.h - C ABI of the MI355X (gfx950) implementation of Pyramid Speculative
 * Decoding: a draft model proposes tokens, a qualifier model verifies them in
 * one multi-position pass, and the target model verifies the qualified window
 * in one pass; every verify pass is followed by a vocabulary-wide
 * softmax -> divergence -> fuzzy-threshold accept / first-reject scan /
 * resample step.
 *
 * Conventions
 *   - Every function returns PSD_OK (0) or a negative error code; nothing throws
 *     across this boundary.  On failure no output argument is written, except
 *     that psd_create sets *out = NULL.
 *   - "host" pointers are ordinary process memory, "device" pointers are HIP
 *     device memory of the context's (or the current) device.  Each argument
 *     says which it is.
 *   - The library owns every device allocation it makes; callers own every
 *     buffer they pass in, and may free it as soon as the call returns.
 *   - A context is not thread-safe: one call at a time per context.
 *   - Determinism: equal (weights, parameters, prompt, seed) give equal tokens
 *     on every run; no reduction in the library depends on scheduling order.
 *
 * Readings of the paper that this interface fixes (the paper leaves them open)
 *   - Div (Sections 3.1-3.2) is the Jensen-Shannon divergence in nats, so
 *     thresholds live in [0, ln 2]; the comparison is Div <= tau as printed.
 *   - A position over the threshold falls back to the standard
 *     speculative-sampling rule (accept with probability min(1, p(x)/q(x)),
 *     else resample from norm(max(0, p - q))); tau = 0 is therefore standard
 *     speculative decoding (Sections 3.1, 3.3, 3.4).
 *   - A fully accepted window earns one bonus token from the verifier's last
 *     row (the "+1" of Section 3.3).  The qualifier's bonus is only taken
 *     while the window of l_Q tokens is not yet full.
 *   - In the target stage the proposer distribution of a window token is the
 *     qualifier row it was judged under or drawn from (Figure 1 caption).
 *   - One temperature divides the logits of all three models before softmax;
 *     the full vocabulary is used (no top-k / top-p).
 *   - Random draws: Philox4x32-10, key = 64-bit seed, counter =
 *     (vocab index / 4, absolute position of the token being decided,
 *     purpose, stage), word = vocab index % 4, u = (top 23 bits + 1/2) / 2^23.
 *     Purposes: 0 fresh sample from a model's own distribution (draft proposals
 *     and bonus tokens; stage field 0), 1 acceptance coin (vocab index 0),
 *     2 residual resample; stage 1 = qualifier judging the draft, 2 = target
 *     judging the window.  Categorical draws are exponential races:
 *     token = argmax_v w_v / (-ln u_v), ties to the lowest index.
 */
#ifndef PSD_H
#define PSD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    PSD_OK = 0,
    PSD_EINVAL = -1, /* bad pointer, size, threshold, mismatched vocabularies, ... */
    PSD_ESHAPE = -2, /* sequence would exceed max_seq, or a width/shape the kernels do not support */
    PSD_ENOMEM = -3, /* device pool or workspace too small */
    PSD_EHIP = -4    /* a HIP runtime call failed; see psd_last_error */
};

enum { PSD_F32 = 0, PSD_BF16 = 1 };

#define PSD_MAX_WIDTH 32 /* most tokens one forward pass can take: k2 + 1 <= 32, k1 + 2 <= 32 */

typedef struct psd_ctx psd_ctx; /* opaque, library-owned */

/* One Llama-style decoder (RMSNorm, rotary embedding on pairs (i, i + hd/2),
 * grouped-query causal attention, SwiGLU MLP, LM head tied to the embedding).
 * `weights` is a HOST pointer to one blob of `dtype` elements in this order,
 * every matrix row-major [out][in]:
 *   embed[vocab][d]
 *   per layer: attn_norm[d], wq[H*hd][d], wk[KV*hd][d], wv[KV*hd][d], wo[d][H*hd],
 *              ffn_norm[d], w_gate[F][d], w_up[F][d], w_down[d][F]
 *   final_norm[d]
 * with hd = d / H.  Requirements: hd in {16, 32, 64, 128}, H % KV == 0,
 * d % 32 == 0, F % 32 == 0, H*hd == d.  The blob is copied (and re-tiled) into
 * the context's pool during psd_create. */
typedef struct {
    int32_t n_layers, d_model, n_heads, n_kv_heads, d_ffn, vocab;
    float rope_theta, rms_eps;
    int32_t dtype; /* PSD_F32 or PSD_BF16: storage type of the weights and of the KV cache */
    int32_t reserved;
    const void* weights; /* host */
    size_t weights_bytes; /* must equal the blob size implied by the shape */
} psd_model_desc;

enum {
    PSD_FLAG_GRAPH = 1,             /* replay captured hipGraphs for the decoding loop's passes instead of
                                       launching kernel by kernel */
    PSD_FLAG_ASSISTED = 2,          /* qualifier stage of psd_generate as in Section 3.4: a draft token passes iff it is
                                       the qualifier's top prediction, a rejected one is replaced by a sample of the
                                       qualifier's own distribution; T_q is unused */
    PSD_FLAG_GREEDY = 8,            /* greedy decoding, the temperature -> 0 limit (Section 3.1): proposals, replacements and
                                       bonus tokens are top predictions, both stages match tokens exactly; thresholds,
                                       temperature and seed play no part; the output is the target's greedy continuation */
    PSD_FLAG_ROW_STATS = 4,         /* collect entropy and largest probability of every logits row the loops produce
                                       (Section 4, model behaviour analysis); read with psd_get_row_stats */
    PSD_FLAG_SCRAMBLE_PAGES = 0x100 /* test aid: hand out physical KV pages in a shuffled order */
};

typedef struct {
    float T_q, T_t;      /* tau_Q, tau_T of Section 3.2, in nats, >= 0 */
    float temperature;   /* > 0 */
    int32_t k1, k2;      /* l_D, l_Q of the paper: 1 <= k1 <= 30, 1 <= k2 <= 31 */
    int32_t max_seq;     /* KV capacity in tokens; a generate call needs n_prompt + n_new + k2 + 2 <= max_seq */
    int32_t device;      /* HIP device ordinal */
    int32_t flags;       /* PSD_FLAG_* */
    size_t pool_bytes;   /* device pool size; 0 = exactly what the three models need */
} psd_params;

typedef struct {
    int64_t proposed_q, accepted_q, fuzzy_q; /* draft tokens judged by the qualifier / accepted / accepted by threshold */
    int64_t proposed_t, accepted_t, fuzzy_t; /* window tokens judged by the target / accepted / accepted by threshold */
    int64_t passes_d, passes_q, passes_t;    /* forward passes of each model during decoding */
    double ms_prefill;                       /* prompt ingestion, all three models */
    double ms_decode;                        /* from the end of prefill to the last token (device time, HIP events) */
    double ms_d, ms_q, ms_t, ms_accept;      /* device time inside ms_decode spent in draft steps (with sampling),
                                                qualifier passes, target passes and ACCEPT stages */
} psd_stats;

/* Builds a context: one device pool holding the three models' re-tiled weights,
 * their paged KV caches and all scratch.  The three models must share `vocab`
 * (the method compares their distributions entry by entry).
 * Errors: PSD_EINVAL (null pointer, unsupported shape, k1/k2/threshold/temperature out of range,
 * vocab mismatch, wrong weights_bytes), PSD_ENOMEM (pool_bytes too small), PSD_EHIP. */
int psd_create(const psd_model_desc* draft, const psd_model_desc* qualifier, const psd_model_desc* target,
               const psd_params* params, psd_ctx** out);

void psd_destroy(psd_ctx* ctx);

/* Device bytes a pool must have for these models and parameters. */
size_t psd_pool_bytes_needed(const psd_model_desc* draft, const psd_model_desc* qualifier,
                             const psd_model_desc* target, const psd_params* params);

/* Changes thresholds / window lengths / temperature of an existing context
 * (k2 must not exceed the k2 it was created with, nor k1 its k1). */
int psd_set_decoding(psd_ctx* ctx, float T_q, float T_t, int32_t k1, int32_t k2, float temperature);

/* The two-stage loop of Figure 1: prefill the prompt, then repeat
 * { draft k1 tokens, qualifier verifies (tau_Q) } until k2 tokens are qualified,
 * target verifies them (tau_T), commit the accepted prefix plus the replacement
 * or bonus token, roll every KV cache back to the committed length.
 *   prompt      host, n_prompt >= 1 token ids in [0, vocab)
 *   out_tokens  host, caller-owned, receives exactly n_new ids
 *   out_stats   host, caller-owned, may be NULL
 * Errors: PSD_EINVAL, PSD_ESHAPE (n_prompt + n_new + k2 + 2 > max_seq), PSD_EHIP. */
int psd_generate(psd_ctx* ctx, const int32_t* prompt, int32_t n_prompt, int32_t n_new, uint64_t seed,
                 int32_t* out_tokens, psd_stats* out_stats);

/* Two-model speculative decoding through the same scheduler, the comparison the paper's speed-up is quoted
 * against (Section 3.3, first equation): model `proposer` (0 draft, 1 qualifier) proposes k tokens one step at a
 * time, the target verifies them in one pass with threshold tau (0: standard speculative sampling; > 0: fuzzy
 * speculative decoding), the accepted prefix plus the replacement or bonus token is committed.  Random draws
 * are addressed as in the target stage of psd_generate.  1 <= k <= the k2 the context was created with.
 * Stats: proposed_t / accepted_t / fuzzy_t, passes_t, and the proposer's steps in passes_d or passes_q.
 * Errors: PSD_EINVAL, PSD_ESHAPE (n_prompt + n_new + k + 2 > max_seq), PSD_EHIP. */
int psd_generate_sd(psd_ctx* ctx, int32_t proposer, int32_t k, float tau, const int32_t* prompt, int32_t n_prompt,
                    int32_t n_new, uint64_t seed, int32_t* out_tokens, psd_stats* out_stats);

/* Per-step statistics of the behaviour analysis (Section 4): entropy in nats and largest probability of
 * softmax(row / temperature) for n_rows logits rows [n_rows][vocab].  where: 0 host pointers, 1 device pointers
 * (device logits must be 16-byte aligned; 4-byte when the vocabulary is not a multiple of 4).  entropy, max_prob: [n_rows] floats. */
int psd_row_stats(const float* logits, int32_t n_rows, int32_t vocab, float temperature, int32_t where,
                  float* entropy, float* max_prob);

/* In-loop collection of the same statistics, as PSD_FLAG_ROW_STATS does at creation: while on, psd_generate and
 * psd_generate_sd evaluate every logits row their passes produce (one extra sweep of those rows per pass).
 * psd_get_row_stats fills out[9] (host) = per model (draft, qualifier, target): number of rows, mean entropy,
 * mean largest probability, over the last generation call. */
int psd_set_row_stats(psd_ctx* ctx, int32_t on);
int psd_get_row_stats(psd_ctx* ctx, double* out);

/* Switches greedy decoding on or off, as PSD_FLAG_GREEDY does at creation (applies to psd_generate,
 * psd_generate_sd and psd_generate_plain; captured graphs of the sampling steps are dropped). */
int psd_set_greedy(psd_ctx* ctx, int32_t on);

/* Switches the qualifier stage of psd_generate between the fuzzy rule (0) and the assisted rule of
 * Section 3.4 (1), as PSD_FLAG_ASSISTED does at creation. */
int psd_set_assisted(psd_ctx* ctx, int32_t on);

/* Adaptive controller for (tau_Q, tau_T, l_D, l_Q) inside psd_generate.  The paper names such a controller as future
 * work (Conclusion and Future Work: adjust divergence thresholds and speculative lengths from the decoding context) and
 * gives no rule; this is the library's reading, built from the paper's observations (Sections 4.2 and 4.4): full
 * acceptance invites a longer window and a rejection cascade a shorter one, l_D about half of l_Q, tau_Q <= tau_T,
 * thresholds no looser than acceptance needs.  All decisions are integer comparisons of counts:
 *   after every target pass with window k2 and n accepted:  n == k2 -> k2 + 1 (<= k2_max);  2 n < k2 -> k2 - 1
 *   (>= k2_min);  k1 = clamp((k2 + 1) / 2, 1, k1_max);
 *   every `period` target passes, per stage, with p proposed and a accepted tokens since the last adjustment:
 *   8 a >= 7 p -> threshold one position lower;  2 a < p -> one position higher; then tau_Q is lowered while it
 *   exceeds tau_T.  Thresholds sit on the steps + 1 positions  min + (max - min) s / steps  of their band (evaluated in
 *   double, rounded once to float).
 * The run starts from the context's thresholds and k2, brought into the ranges (nearest position; clamped).
 * Requirements: 1 <= k2_min <= k2_max <= the context's k2, 1 <= k1_max <= the context's k1, steps >= 1, period >= 1,
 * 0 <= min <= max for both bands.  cfg == NULL switches the controller off.  psd_generate then needs
 * n_prompt + n_new + k2_max + 2 <= max_seq.  psd_get_adaptive_log copies (k1, k2, position of tau_Q, position of
 * tau_T) of up to `cap` outer iterations of the last psd_generate call into out[cap][4] (host) and returns how many
 * iterations there were (or a negative error). */
typedef struct {
    int32_t k2_min, k2_max, k1_max;
    int32_t steps, period;
    float T_q_min, T_q_max, T_t_min, T_t_max;
} psd_adapt;
int psd_set_adaptive(psd_ctx* ctx, const psd_adapt* cfg);
int psd_get_adaptive_log(psd_ctx* ctx, int32_t* out, int32_t cap);

/* Plain autoregressive sampling from one model (0 draft, 1 qualifier, 2 target)
 * with the same fresh-sample draws: the no-speculation baseline. */
int psd_generate_plain(psd_ctx* ctx, int32_t which, const int32_t* prompt, int32_t n_prompt, int32_t n_new,
                       uint64_t seed, int32_t* out_tokens, psd_stats* out_stats);

/* One forward pass of model `which` over `w` tokens (1 <= w <= PSD_MAX_WIDTH; up to 512 for a bf16 model
 * when logits_out is NULL: the wide passes that ingest a prompt) at positions pos0 .. pos0+w-1; KV rows below pos0 must have been written by
 * earlier calls (pos0 may also re-write older rows: that is a rollback).
 *   tokens      host, w ids
 *   logits_out  host, [w][vocab] floats, may be NULL (KV update only)
 * Test / measurement hook for logits parity; runs the same kernels psd_generate runs. */
int psd_forward(psd_ctx* ctx, int32_t which, const int32_t* tokens, int32_t w, int32_t pos0, float* logits_out);

/* ACCEPT of one verify stage (Sections 3.1-3.2, with the fallback rule of 3.4), stand-alone.
 *   logits_p  [k+1][vocab] verifier rows,  logits_q  [k][vocab] proposer rows,
 *   tokens    [k] proposed ids; token i sits at absolute position position0 + i
 *   where     0: all pointers are host memory, 1: all pointers are device memory
 *   stage     1 or 2 (selects the random streams, see top of file)
 *   take_bonus  when all k are accepted: draw one more token from verifier row k
 * Outputs (same memory space as the inputs): n_accepted (int32), next_token (int32, -1 if none),
 * div_out [k] floats (may be NULL): the divergence of every proposed position.
 * 0 <= k <= PSD_MAX_WIDTH.  Stateless: equal arguments give equal results.  The call allocates and frees its
 * device scratch (and, for host pointers, staging buffers) every time and synchronises the device: it is the
 * convenient form, for tests; time psd_accept_batch or psd_accept_batch_noalloc instead. */
int psd_accept(const float* logits_p, const float* logits_q, const int32_t* tokens, int32_t k, int32_t vocab,
               float T, float temperature, uint64_t seed, uint32_t position0, uint32_t stage, int32_t take_bonus,
               int32_t where, int32_t* n_accepted, int32_t* next_token, float* div_out);

/* ACCEPT of the assisted stage (Section 3.4) on its own: proposal i passes iff tokens[i] is the top
 * prediction of verifier row i (lowest index among equal maxima); at the first mismatch n the replacement is
 * drawn from softmax(logits_p[n] / temperature); a fully accepted run takes the bonus token from row k.
 * Arguments as for psd_accept (no proposer rows, no threshold, no divergences). */
int psd_accept_assisted(const float* logits_p, const int32_t* tokens, int32_t k, int32_t vocab, float temperature,
                        uint64_t seed, uint32_t position0, uint32_t stage, int32_t take_bonus, int32_t where,
                        int32_t* n_accepted, int32_t* next_token);

/* Batched ACCEPT for throughput measurement: n_trials independent stages of equal k in one launch
 * sequence.  All pointers are DEVICE memory; trial b uses seed + b.
 *   logits_p [n_trials][k+1][vocab], logits_q [n_trials][k][vocab], tokens [n_trials][k]
 *   n_accepted, next_token [n_trials]; div_out [n_trials][k] (may be NULL)
 *   workspace: device scratch of at least psd_accept_workspace_bytes(n_trials, k, vocab) bytes
 *   stream: a hipStream_t passed as void* (NULL = the default stream); the call only enqueues work.
 * Logits must be finite or -inf (-inf entries have probability 0).  The kernels of one row wait for each
 * other inside one launch; that wait is bounded by a clock, and if it ever expires (it cannot while the
 * device runs the launch alone) n_accepted[b] = -1 for every trial of the call: call psd_set_accept_path(1) and
 * run it again (psd_accept and the generation calls do that themselves). */
size_t psd_accept_workspace_bytes(int32_t n_trials, int32_t k, int32_t vocab);
int psd_accept_batch(const float* logits_p, const float* logits_q, const int32_t* tokens, int32_t n_trials,
                     int32_t k, int32_t vocab, float T, float temperature, uint64_t seed, uint32_t position0,
                     uint32_t stage, int32_t take_bonus, int32_t* n_accepted, int32_t* next_token, float* div_out,
                     void* workspace, size_t workspace_bytes, void* stream);

/* psd_accept_batch for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same arguments and results as psd_accept_batch (all pointers
 * DEVICE memory, the call only enqueues work on `stream`), but the scratch the kernels need comes from a fixed
 * array of PSD_ACCEPT_NOALLOC_SCRATCH_BYTES inside the library's code object instead of a caller workspace; each
 * GPU the library runs on holds that array until the process ends.  The call makes no hipMalloc / hipFree and no
 * allocating library call.
 *   - Limit: psd_accept_workspace_bytes(n_trials, k, vocab) <= psd_accept_noalloc_capacity() (e.g. one trial of
 *     k = 31 at vocabulary 128256 needs 82 KB, 48 trials of k = 32 about 4.1 MB); larger requests return PSD_ENOMEM and
 *     enqueue nothing.
 *   - All calls on one GPU share that GPU's array: two calls whose kernels may overlap (different streams, or
 *     different threads) race on it.  Serialise them, or use psd_accept_batch with separate workspaces.
 *   - The array keeps what the last call left; every slot a call reads is written earlier in that call's own
 *     launch sequence (a fill kernel, not a memset, so the sequence can be captured into a graph).
 *   - psd_accept_noalloc_init() looks up the array's device address for the current device (no allocation);
 *     psd_create calls it, and so does the first psd_accept_batch_noalloc on a device.  Call it once outside
 *     stream capture if the first use would otherwise fall inside one.
 * Errors: PSD_EINVAL, PSD_ENOMEM (request beyond the capacity), PSD_EHIP. */
#define PSD_ACCEPT_NOALLOC_SCRATCH_BYTES ((size_t)8 << 20)
size_t psd_accept_noalloc_capacity(void);
int psd_accept_noalloc_init(void);
int psd_accept_batch_noalloc(const float* logits_p, const float* logits_q, const int32_t* tokens, int32_t n_trials,
                             int32_t k, int32_t vocab, float T, float temperature, uint64_t seed, uint32_t position0,
                             uint32_t stage, int32_t take_bonus, int32_t* n_accepted, int32_t* next_token,
                             float* div_out, void* stream);

/* How the ACCEPT stage sweeps the logits (Section 3.2 divergence), process-wide; for measurement and tests.
 *   0  automatic: one launch that reads every logit once when a row has at most 64 chunks of 5120 entries,
 *      else two launches that read the logits twice
 *   1  always two launches     2  same as 0
 *   3  test aid: as 0, but a workgroup's wait for the rest of its row expires at once unless it is already
 *      satisfied, so the expiry handling below can be exercised without a stuck kernel
 * Both sweeps give bit-identical results.  When a wait expires, psd_accept, psd_generate and psd_generate_sd
 * switch the process to path 1 and run the stage again; psd_get_accept_path tells which path is in force.
 * The switch may be flipped while other threads run stages (they pick it up at their next stage).  Returns PSD_EINVAL
 * for other values. */
int psd_set_accept_path(int32_t path);
int psd_get_accept_path(void);
/* How many times, in this process, a bounded wait expired and the library ran a stage again on path 1: normally 0;
 * anything else explains an ACCEPT slowdown (the two-launch sweep reads the logits twice). */
int64_t psd_get_accept_expiries(void);

/* Fresh sample from softmax(logits / temperature) by the exponential race (how the
 * draft proposes, Figure 1): rows [n_rows][vocab], row r is decided for position position0 + r.
 * where: 0 host pointers, 1 device pointers.  tokens_out [n_rows]. */
int psd_sample(const float* logits, int32_t n_rows, int32_t vocab, float temperature, uint64_t seed,
               uint32_t position0, int32_t where, int32_t* tokens_out);

/* Test hook: the device's Philox4x32-10, the generator behind every draw above, for the n consecutive counters
 * (c0 .. c0 + n - 1, c1, c2, c3) under key = seed.  out [n][4] uint32 raw words and / or u_out [n][4] floats (the
 * uniforms the kernels derive from them: (top 23 bits + 1/2) / 2^23); either may be NULL.  where: 0 host pointers,
 * 1 device pointers (16-byte aligned).  1 <= n <= 2^26.  Lets a test compare the generator with an independent
 * implementation counter by counter. */
int psd_philox_block(uint64_t seed, uint32_t c0, uint32_t n, uint32_t c1, uint32_t c2, uint32_t c3, int32_t where,
                     uint32_t* out, float* u_out);

/* Trace hook for tests: when set, psd_generate copies the inputs of every draft
 * sample (kind 0, k = 0, logits_p = the draft row) and every ACCEPT (kind 1 / 2 =
 * stage; kind 3 = stage 1 under the assisted rule; greedy decoding: kind 6 = proposal, 4 / 5 = stage 1 / 2)
 * back to the host and calls fn after the step has been decided.  Under the adaptive controller every outer
 * iteration starts with a kind 7 call: position0 = committed length, k = k2, take_bonus = k1, n_accepted / next_token =
 * positions of tau_Q / tau_T, div = {tau_Q, tau_T}, the other pointers NULL.  All
 * pointers are host memory valid during the callback only.  Slow; tests only. */
typedef void (*psd_trace_fn)(void* user, int32_t kind, uint32_t position0, int32_t k, int32_t take_bonus,
                             const float* logits_p, const float* logits_q, const int32_t* tokens,
                             int32_t n_accepted, int32_t next_token, const float* div);
int psd_set_trace(psd_ctx* ctx, psd_trace_fn fn, void* user);

/* Per-kernel device time, measured with HIP events on the library's stream.
 * psd_profile(ctx, 1) switches to kernel-by-kernel launches with an event pair
 * around every launch (graphs are bypassed) and clears the table; psd_profile(ctx, 0)
 * switches back.  psd_kernel_stats copies up to `cap` rows to host memory and
 * returns the number of rows (or a negative error). */
typedef struct {
    char name[48];      /* kernel family and shape class, e.g. "gemm_bf16 draft w1" */
    int64_t launches;
    double ms_total;
    double bytes_total; /* algorithmic bytes those launches had to move (weights + activations + KV) */
} psd_kernel_stat;
int psd_profile(psd_ctx* ctx, int32_t on);
int psd_kernel_stats(psd_ctx* ctx, psd_kernel_stat* out, int32_t cap);

/* Device-memory plumbing for callers that have no other HIP binding (tests, benchmarks): plain
 * hipMalloc / hipFree / hipMemcpy / hipDeviceSynchronize on the current device.
 * kind: 0 host->device, 1 device->host, 2 device->device. */
int psd_dev_alloc(size_t bytes, void** out);
int psd_dev_free(void* ptr);
int psd_dev_copy(void* dst, const void* src, size_t bytes, int32_t kind);
int psd_dev_sync(void);

const char* psd_strerror(int code);
const char* psd_last_error(const psd_ctx* ctx); /* ctx may be NULL: last error of stand-alone calls on this thread */

#ifdef __cplusplus
}
#endif
#endif /* PSD_H */
