// Context, device pool and the two-stage scheduler (Figure 1 caption; Sections 3.2-3.3).
//
// The host keeps the token sequence (committed tokens followed by the window of qualified tokens) and,
// per model, how many KV rows are valid.  Before a pass a model ingests whatever part of the sequence it
// has not cached; a rollback is nothing more than lowering that count (and returning whole KV pages).
// The draft's chain of single-token steps stays on the device: the sampling kernels write the new token
// into the next draft pass descriptor and into the qualifier's, so the host synchronises once per
// qualifier round and once per target pass, when it reads the ACCEPT result.
#include <stddef.h>
#include <math.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "psd_device.h"
#include "psd_model.h"

namespace psd {

constexpr int kStageSlots = 64;
constexpr int kStageSlotBytes = 2304;  // a pass descriptor with 512 token ids fits

struct RoundResult {  // pinned host mirror of what a round leaves on the device
    AcceptOut acc;
    int32_t tok[kMaxW];
    float div[kMaxW];
};

// Adaptive controller (the header states the rule).  Pure host arithmetic on accept counts between outer iterations.
struct Controller {
    psd_adapt cfg{};
    bool on = false;
    int k1 = 0, k2 = 0, pos_q = 0, pos_t = 0;     // in force for the next outer iteration
    int passes = 0;                               // target passes since the thresholds were last looked at
    long long prop[2] = {0, 0}, acc[2] = {0, 0};  // per stage, since then
    std::vector<int32_t> log;                     // (k1, k2, pos_q, pos_t) per outer iteration of the last call

    static float at(float lo, float hi, int pos, int steps) {
        return (float)((double)lo + ((double)hi - (double)lo) * (double)pos / (double)steps);
    }
    static int nearest(float lo, float hi, float T, int steps) {
        if (!(hi > lo)) return 0;
        const double x = ((double)T - (double)lo) / ((double)hi - (double)lo) * (double)steps;
        return std::min(steps, std::max(0, (int)floor(x + 0.5)));
    }
    float tau_q() const { return at(cfg.T_q_min, cfg.T_q_max, pos_q, cfg.steps); }
    float tau_t() const { return at(cfg.T_t_min, cfg.T_t_max, pos_t, cfg.steps); }
    void set_window(int k) {
        k2 = std::min((int)cfg.k2_max, std::max((int)cfg.k2_min, k));
        k1 = std::min((int)cfg.k1_max, std::max(1, (k2 + 1) / 2));
    }
    void start(float T_q, float T_t, int k2_start) {
        set_window(k2_start);
        pos_q = nearest(cfg.T_q_min, cfg.T_q_max, T_q, cfg.steps);
        pos_t = nearest(cfg.T_t_min, cfg.T_t_max, T_t, cfg.steps);
        passes = 0;
        prop[0] = prop[1] = acc[0] = acc[1] = 0;
        log.clear();
    }
    // one outer iteration is over: the target accepted n of the k2 window tokens, the qualifier aq of pq draft tokens
    void observe(int n, long long pq, long long aq) {
        prop[0] += pq; acc[0] += aq; prop[1] += k2; acc[1] += n;
        if (n == k2) set_window(k2 + 1);
        else if (2 * n < k2) set_window(k2 - 1);
        else set_window(k2);
        if (++passes < cfg.period) return;
        int* pos[2] = {&pos_q, &pos_t};
        for (int s = 0; s < 2; ++s) {
            if (prop[s] == 0) continue;
            if (8 * acc[s] >= 7 * prop[s]) *pos[s] = std::max(0, *pos[s] - 1);
            else if (2 * acc[s] < prop[s]) *pos[s] = std::min((int)cfg.steps, *pos[s] + 1);
        }
        while (pos_q > 0 && tau_q() > tau_t()) --pos_q;
        passes = 0;
        prop[0] = prop[1] = acc[0] = acc[1] = 0;
    }
};

struct GraphSlot {
    hipGraphExec_t exec = nullptr;
};

// device time per stage of the loop: event pairs recorded in stream order, read once at the end of a call
struct StageTimer {
    struct Span { int kind; hipEvent_t a, b; };
    std::vector<Span> spans;
    std::vector<hipEvent_t> pool;
    hipEvent_t get() {
        if (!pool.empty()) { hipEvent_t e = pool.back(); pool.pop_back(); return e; }
        hipEvent_t e = nullptr;
        (void)hipEventCreate(&e);
        return e;
    }
    void begin(hipStream_t s, int kind) { spans.push_back({kind, get(), get()}); (void)hipEventRecord(spans.back().a, s); }
    void end(hipStream_t s) { (void)hipEventRecord(spans.back().b, s); }
    void collect(double ms[4]) {  // call after the stream has been synchronised
        for (auto& sp : spans) {
            float t = 0.f;
            if (hipEventElapsedTime(&t, sp.a, sp.b) == hipSuccess) ms[sp.kind] += t;
            pool.push_back(sp.a);
            pool.push_back(sp.b);
        }
        spans.clear();
    }
    ~StageTimer() {
        double dummy[4] = {0, 0, 0, 0};
        collect(dummy);
        for (auto e : pool) (void)hipEventDestroy(e);
    }
};

}  // namespace psd

using namespace psd;

struct psd_ctx {
    char err[512] = {0};
    int device = 0;
    hipStream_t stream = nullptr;
    void* pool_mem = nullptr;
    Pool pool;
    Model M[3];
    psd_params prm{};
    int k1cap = 0, k2cap = 0, V = 0;
    // logits rows
    float* DL = nullptr;  // [k1cap][V]   draft rows of the current round
    float* QL = nullptr;  // [k2cap+1][V] qualifier row per window slot
    float* TL = nullptr;  // [k2cap+1][V] target rows
    float* HL = nullptr;  // [32][V]      psd_forward / plain generation
    // ACCEPT
    void* acc_ws = nullptr;
    size_t acc_ws_bytes = 0;
    AcceptOut* acc_out = nullptr;
    float* acc_div = nullptr;
    void* samp_part = nullptr;
    int32_t* samp_tok = nullptr;   // [1] token just sampled
    SampleCtl* chain = nullptr;
    int32_t* round_tok = nullptr;  // [32] draft tokens of the round
    int32_t* win_tok = nullptr;    // [32] window tokens for the target stage
    void* rs_ws = nullptr;         // workspace of the per-row statistics kernels
    double* rs_acc = nullptr;      // [3 models][rows, sum of entropies, sum of largest probabilities]
    // pinned staging
    char* stage = nullptr;  // kStageSlots * kStageSlotBytes
    int stage_next = 0, stage_since_sync = 0;
    RoundResult* res = nullptr;
    // graphs: [model][width class 4 / 16 / 32]
    GraphSlot graphs[3][kNumNarrowClasses][kNumCtxBuckets];   // [model][launch class][context bucket]
    GraphSlot chain_graphs[3][3][kNumNarrowClasses][kNumCtxBuckets];  // sampling steps: [proposer][model whose pass descriptor receives the tokens][launch class][context bucket]
    Profiler prof;
    StageTimer timer;
    Controller ctl;
    psd_trace_fn trace = nullptr;
    void* trace_user = nullptr;
    hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
    // prompt ingestion: one stream per model, so that the three independent ingestions share the device
    hipStream_t aux[3] = {nullptr, nullptr, nullptr};
    hipEvent_t aux_ready[3] = {nullptr, nullptr, nullptr}, aux_done[3] = {nullptr, nullptr, nullptr};
};

namespace psd {

// one wave: picks the winner among the per-chunk winners of the sampling race (the comparisons of sample_final; equal
// keys resolve to the lowest index) and publishes the token to the next draft pass and to the qualifier pass
__global__ __launch_bounds__(64) void draft_pick_advance(const KeyIdx* parts, int nch, int32_t* samp_tok, SampleCtl* chain,
                                                         PassDesc* d_desc, PassDesc* q_desc, int32_t* round_tok) {
    KeyIdx best{-INFINITY, 0x7fffffff};
    for (int ch = threadIdx.x; ch < nch; ch += kWave) best = better(best, parts[ch]);
    best = wave_best(best);
    if (threadIdx.x != 0) return;
    const int t = best.idx, step = chain->row;
    samp_tok[0] = t;
    if (step < kMaxW) round_tok[step] = t;
    if (q_desc && chain->q_base >= 0 && chain->q_base + step < kMaxW) q_desc->tok[chain->q_base + step] = t;
    d_desc->pos0 += d_desc->w;
    d_desc->w = 1;
    d_desc->tok[0] = t;
    d_desc->logit_row0 = step + 1;
    chain->row = step + 1;
    chain->position += 1;
}

static int stage_sync(psd_ctx* c) {
    PSD_HIP(hipStreamSynchronize(c->stream), c->err);
    c->stage_since_sync = 0;
    return PSD_OK;
}

// copies `bytes` (<= kStageSlotBytes) of host data to device memory in stream order through a pinned ring slot
static int upload(psd_ctx* c, void* dst, const void* src, size_t bytes) {
    if (bytes > kStageSlotBytes) PSD_FAIL(PSD_EINVAL, c->err, "internal: staging slot overflow");
    if (c->stage_since_sync >= kStageSlots - 1) {
        int rc = stage_sync(c);
        if (rc != PSD_OK) return rc;
    }
    char* slot = c->stage + (size_t)c->stage_next * kStageSlotBytes;
    c->stage_next = (c->stage_next + 1) % kStageSlots;
    c->stage_since_sync++;
    memcpy(slot, src, bytes);
    PSD_HIP(hipMemcpyAsync(dst, slot, bytes, hipMemcpyHostToDevice, c->stream), c->err);
    return PSD_OK;
}

// KV pages for positions < upto of model M (pages wholly beyond `keep` are returned); the page-table entries that
// changed travel in stream order through the pinned ring, so the host does not wait for the device here
static int map_pages(psd_ctx* c, Model& M, int keep, int upto) {
    int first = 0, n = 0;
    int rc = model_map_pages(M, keep, upto, &first, &n, c->err);
    if (rc != PSD_OK) return rc;
    constexpr int kPerSlot = kStageSlotBytes / (int)sizeof(int32_t);
    int32_t tmp[kPerSlot];
    for (int done = 0; done < n; done += kPerSlot) {
        const int cnt = std::min(kPerSlot, n - done);
        for (int i = 0; i < cnt; ++i) tmp[i] = std::max(M.h_page_table[first + done + i], 0);   // unmapped: page 0, never read
        if ((rc = upload(c, M.page_table + first + done, tmp, (size_t)cnt * sizeof(int32_t))) != PSD_OK) return rc;
    }
    return PSD_OK;
}

// launch class of a pass of w tokens: the smallest narrow class that holds it, or (prompt ingestion only) the next
// multiple of 128
static int wclass(int w) { return w <= kMaxW ? kNarrowClasses[narrow_class_index(w)] : (w + 127) / 128 * 128; }

// bytes of a pass descriptor that have to travel: the header and the token slots the pass can read
static size_t desc_bytes(const PassDesc& d) {
    return offsetof(PassDesc, tok) + sizeof(int32_t) * (size_t)std::min(kCols, std::max((int)d.w, kMaxW));
}

// enqueues one pass of model `mi`; the descriptor is already on the device.  with_sample: the draft step
// also samples its token and advances the chain.
static int run_pass(psd_ctx* c, int mi, int wcls, float* logits, bool with_sample, bool allow_graph = false,
                    int verifier = 1, hipStream_t on_stream = nullptr) {
    Model& M = c->M[mi];
    hipStream_t stream = on_stream ? on_stream : c->stream;   // other than the context's: eager passes without sampling only
    // Upper bound of the pass's last position.  The host mirror of the length moves once per round: a catch-up pass of
    // up to kMaxW tokens and up to kMaxW - 1 single-token sampling steps may be launched from one value of it.
    M.ctx_bucket = ctx_bucket_index(std::min(M.max_seq, M.len + std::max(wcls, 2 * kMaxW)));
    // only the decoding loop's three pass shapes are captured; prefill, the test hook and plain generation stay eager
    const bool use_graph = allow_graph && (c->prm.flags & PSD_FLAG_GRAPH) && !c->prof.on;
    auto enqueue = [&](Profiler* prof) -> int {
        int rc = model_forward(M, wcls, logits, stream, prof, c->err);
        if (rc != PSD_OK) return rc;
        if (with_sample) {
            if (prof && prof->on) prof->begin(c->stream, prof->row_of("sample draft"), (double)c->V * 4);
            rc = sample_launch(logits, 1, c->V, c->prm.temperature, 0, 0, c->chain, nullptr, c->samp_part,
                               c->stream, c->err, (c->prm.flags & PSD_FLAG_GREEDY) ? 1 : 0);
            if (rc != PSD_OK) return rc;
            draft_pick_advance<<<1, 64, 0, c->stream>>>((const KeyIdx*)c->samp_part, accept_chunks(c->V), c->samp_tok, c->chain,
                                                         M.desc, c->M[verifier].desc, c->round_tok);
            if (prof && prof->on) prof->end(c->stream);
        }
        return PSD_OK;
    };
    if (!use_graph) return enqueue(&c->prof);
    GraphSlot& g = with_sample ? c->chain_graphs[mi][verifier][narrow_class_index(wcls)][M.ctx_bucket]
                               : c->graphs[mi][narrow_class_index(wcls)][M.ctx_bucket];
    if (!g.exec) {
        hipGraph_t graph = nullptr;
        PSD_HIP(hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal), c->err);
        int rc = enqueue(nullptr);
        hipError_t e = hipStreamEndCapture(c->stream, &graph);
        if (rc != PSD_OK) { if (graph) (void)hipGraphDestroy(graph); return rc; }
        PSD_HIP(e, c->err);
        PSD_HIP(hipGraphInstantiate(&g.exec, graph, nullptr, nullptr, 0), c->err);
        PSD_HIP(hipGraphDestroy(graph), c->err);
    }
    PSD_HIP(hipGraphLaunch(g.exec, c->stream), c->err);
    return PSD_OK;
}

static void drop_graphs(psd_ctx* c) {
    auto drop = [](GraphSlot& g) {
        if (g.exec) { (void)hipGraphExecDestroy(g.exec); g.exec = nullptr; }
    };
    for (auto& row : c->graphs)
        for (auto& cls : row)
            for (auto& g : cls) drop(g);
    for (auto& plane : c->chain_graphs)
        for (auto& row : plane)
            for (auto& cls : row)
                for (auto& g : cls) drop(g);
}

// host-known tokens seq[from, to) go into a pass descriptor that starts at KV row `from`
static void fill_desc(PassDesc& d, const int32_t* seq, int from, int to, int extra, int n_logit, int row0) {
    memset(&d, 0, sizeof(d));
    d.w = to - from + extra;
    d.pos0 = from;
    d.n_logit = n_logit;
    d.logit_row0 = row0;
    for (int i = from; i < to; ++i) d.tok[i - from] = seq[i];
}

// ingests seq[M.len, upto) with no logits, in chunks of up to 512 (bf16 models) or 32 tokens
static int prefill(psd_ctx* c, int mi, const int32_t* seq, int upto) {
    Model& M = c->M[mi];
    while (M.len < upto) {
        const int w = std::min(M.ingest_max, upto - M.len);
        int rc = map_pages(c, M, M.len, M.len + w);
        if (rc != PSD_OK) return rc;
        PassDesc d;
        fill_desc(d, seq, M.len, M.len + w, 0, 0, 0);
        if ((rc = upload(c, M.desc, &d, desc_bytes(d))) != PSD_OK) return rc;
        if ((rc = run_pass(c, mi, wclass(w), nullptr, false)) != PSD_OK) return rc;
        M.len += w;
    }
    return PSD_OK;
}

// Ingests seq[len, upto) into several models at once (`models`: bit i = model i).  The ingestions are independent
// and their launches are too small to fill the device one model at a time, so each model's passes run on a stream of
// their own; the context's stream carries the descriptors and page tables and is where everything meets again.
static int prefill_all(psd_ctx* c, const int32_t* seq, int upto, unsigned models = 7u) {
    if (c->prof.on) {   // per-kernel timing: one model after the other on the context's stream
        for (int mi = 0; mi < 3; ++mi) {
            if (!(models >> mi & 1u)) continue;
            int rc = prefill(c, mi, seq, upto);
            if (rc != PSD_OK) return rc;
        }
        return PSD_OK;
    }
    bool used[3] = {false, false, false};
    auto enqueue = [&]() -> int {
        for (bool more = true; more;) {
            more = false;
            for (int mi = 0; mi < 3; ++mi) {
                Model& M = c->M[mi];
                if (!(models >> mi & 1u) || M.len >= upto) continue;
                const int w = std::min(M.ingest_max, upto - M.len);
                // the model's descriptor and page table are free again once its previous pass is done
                if (used[mi]) PSD_HIP(hipStreamWaitEvent(c->stream, c->aux_done[mi], 0), c->err);
                int rc = map_pages(c, M, M.len, M.len + w);
                if (rc != PSD_OK) return rc;
                PassDesc d;
                fill_desc(d, seq, M.len, M.len + w, 0, 0, 0);
                if ((rc = upload(c, M.desc, &d, desc_bytes(d))) != PSD_OK) return rc;
                PSD_HIP(hipEventRecord(c->aux_ready[mi], c->stream), c->err);
                PSD_HIP(hipStreamWaitEvent(c->aux[mi], c->aux_ready[mi], 0), c->err);
                if ((rc = run_pass(c, mi, wclass(w), nullptr, false, false, 1, c->aux[mi])) != PSD_OK) return rc;
                PSD_HIP(hipEventRecord(c->aux_done[mi], c->aux[mi]), c->err);
                used[mi] = true;
                M.len += w;
                more = more || M.len < upto;
            }
        }
        for (int mi = 0; mi < 3; ++mi)
            if (used[mi]) PSD_HIP(hipStreamWaitEvent(c->stream, c->aux_done[mi], 0), c->err);
        return PSD_OK;
    };
    const int rc = enqueue();
    if (rc != PSD_OK)   // nothing of this context is left running on the side when an error is reported
        for (auto& st : c->aux) (void)hipStreamSynchronize(st);
    return rc;
}

// behaviour statistics (Section 4) of `rows` logits rows model `mi` has just produced; only when asked for
static int note_rows(psd_ctx* c, int mi, const float* rows, int n) {
    if (!(c->prm.flags & PSD_FLAG_ROW_STATS) || n < 1) return PSD_OK;
    return row_stats_launch(rows, n, c->V, c->prm.temperature, nullptr, nullptr, c->rs_acc + 3 * mi, c->rs_ws, c->stream, c->err);
}

// One ACCEPT stage on the stream, its result in c->res after one synchronisation.  n_tok: how many of the round's
// draft tokens to bring back as well.  The kernels of a row wait for each other under a clock; should that wait
// ever expire (n_accepted = -1: the launch was not resident as a whole), the library switches to the two-launch
// sweep for good and the stage is run again.
static int accept_sync(psd_ctx* c, const char* prof_row, const float* lp, const float* lq, const int32_t* toks, int k,
                       float T, uint64_t seed, uint32_t pos0, uint32_t stage, int bonus, int assisted, int n_tok) {
    for (int attempt = 0; attempt < 2; ++attempt) {
        if (c->prof.on) c->prof.begin(c->stream, c->prof.row_of(prof_row), (double)(2 * k + 1) * c->V * 4);
        c->timer.begin(c->stream, 3);
        int rc = accept_launch(lp, lq, toks, 1, k, c->V, T, c->prm.temperature, seed, pos0, stage, bonus, c->acc_out,
                               c->acc_div, c->acc_ws, c->acc_ws_bytes, c->stream, c->err, nullptr, nullptr, assisted);
        if (rc != PSD_OK) return rc;
        c->timer.end(c->stream);
        if (c->prof.on) c->prof.end(c->stream);
        PSD_HIP(hipMemcpyAsync(&c->res->acc, c->acc_out, sizeof(AcceptOut), hipMemcpyDeviceToHost, c->stream), c->err);
        if (n_tok > 0) PSD_HIP(hipMemcpyAsync(c->res->tok, c->round_tok, n_tok * sizeof(int32_t), hipMemcpyDeviceToHost, c->stream), c->err);
        if (c->trace && k > 0) PSD_HIP(hipMemcpyAsync(c->res->div, c->acc_div, k * sizeof(float), hipMemcpyDeviceToHost, c->stream), c->err);
        if ((rc = stage_sync(c)) != PSD_OK) return rc;
        if (c->res->acc.n_accepted >= 0) return PSD_OK;
        accept_wait_expired();
    }
    PSD_FAIL(PSD_EHIP, c->err, "ACCEPT: the kernels' bounded wait expired and the two-launch sweep failed as well");
}

static int check_tokens(psd_ctx* c, const int32_t* t, int n) {
    for (int i = 0; i < n; ++i)
        if (t[i] < 0 || t[i] >= c->V) PSD_FAIL(PSD_EINVAL, c->err, "token %d at index %d is outside [0, %d)", t[i], i, c->V);
    return PSD_OK;
}

static int copy_rows_to_host(psd_ctx* c, std::vector<float>& dst, const float* src, int rows) {
    dst.resize((size_t)std::max(rows, 1) * c->V);
    if (rows > 0) PSD_HIP(hipMemcpy(dst.data(), src, (size_t)rows * c->V * sizeof(float), hipMemcpyDeviceToHost), c->err);
    return PSD_OK;
}

}  // namespace psd

// ---- C ABI --------------------------------------------------------------------------------------------

static int validate_params(const psd_params* p, char* err) {
    if (!(p->T_q >= 0.f) || !(p->T_t >= 0.f)) PSD_FAIL(PSD_EINVAL, err, "thresholds must be >= 0 (T_q=%g T_t=%g)", p->T_q, p->T_t);
    if (!(p->temperature > 0.f)) PSD_FAIL(PSD_EINVAL, err, "temperature must be > 0");
    if (p->k1 < 1 || p->k1 > kMaxW - 2) PSD_FAIL(PSD_EINVAL, err, "k1=%d outside [1, %d]", p->k1, kMaxW - 2);
    if (p->k2 < 1 || p->k2 > kMaxW - 1) PSD_FAIL(PSD_EINVAL, err, "k2=%d outside [1, %d]", p->k2, kMaxW - 1);
    if (p->max_seq < 8) PSD_FAIL(PSD_EINVAL, err, "max_seq=%d too small", p->max_seq);
    return PSD_OK;
}

static size_t ctx_extra_bytes(int V, int k1, int k2) {
    size_t b = 0;
    auto add = [&](size_t n) { b = ((b + 255) & ~(size_t)255) + n; };
    add((size_t)k1 * V * 4);
    add((size_t)(k2 + 1) * V * 4);
    add((size_t)(k2 + 1) * V * 4);
    add((size_t)kMaxW * V * 4);
    add(accept_workspace_bytes(1, kMaxW - 1, V));
    add(sizeof(AcceptOut));
    add(kMaxW * 4);
    add((size_t)accept_chunks(V) * 8);
    add(4);
    add(sizeof(SampleCtl));
    add(kMaxW * 4);
    add(kMaxW * 4);
    add(row_stats_workspace_bytes(kMaxW, V));
    add(9 * sizeof(double));
    return b + 4096;
}

extern "C" size_t psd_pool_bytes_needed(const psd_model_desc* draft, const psd_model_desc* qualifier,
                                        const psd_model_desc* target, const psd_params* params) {
    if (!draft || !qualifier || !target || !params) return 0;
    if (draft->n_heads < 1 || qualifier->n_heads < 1 || target->n_heads < 1 || params->max_seq < 1) return 0;
    return model_pool_bytes(*draft, params->max_seq) + model_pool_bytes(*qualifier, params->max_seq) +
           model_pool_bytes(*target, params->max_seq) + ctx_extra_bytes(target->vocab, params->k1, params->k2);
}

extern "C" int psd_create(const psd_model_desc* draft, const psd_model_desc* qualifier, const psd_model_desc* target,
                          const psd_params* params, psd_ctx** out) {
    char* err = tls_error();
    if (out) *out = nullptr;
    if (!draft || !qualifier || !target || !params || !out) PSD_FAIL(PSD_EINVAL, err, "psd_create: null pointer");
    int rc = validate_params(params, err);
    if (rc != PSD_OK) return rc;
    if (draft->vocab != target->vocab || qualifier->vocab != target->vocab)
        PSD_FAIL(PSD_EINVAL, err, "psd_create: the three models must share one vocabulary (%d / %d / %d)", draft->vocab,
                 qualifier->vocab, target->vocab);
    const psd_model_desc* descs[3] = {draft, qualifier, target};
    for (auto* m : descs)
        if (m->n_heads < 1 || m->d_model < 1) PSD_FAIL(PSD_EINVAL, err, "psd_create: bad model shape");
    int ndev = 0;
    PSD_HIP(hipGetDeviceCount(&ndev), err);
    if (params->device < 0 || params->device >= ndev) PSD_FAIL(PSD_EINVAL, err, "psd_create: device %d of %d", params->device, ndev);
    PSD_HIP(hipSetDevice(params->device), err);
    psd_ctx* c = new psd_ctx();
    auto fail = [&](int code) { strncpy(err, c->err, 511); psd_destroy(c); return code; };
    c->device = params->device;
    c->prm = *params;
    c->k1cap = params->k1;
    c->k2cap = params->k2;
    c->V = target->vocab;
    const size_t need = psd_pool_bytes_needed(draft, qualifier, target, params);
    const size_t pool_bytes = params->pool_bytes ? params->pool_bytes : need;
    if (pool_bytes < need) {
        set_error(c->err, "psd_create: pool_bytes %zu < %zu needed", pool_bytes, need);
        return fail(PSD_ENOMEM);
    }
#define CK(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) { set_error(c->err, "%s: %s", #call, hipGetErrorString(e_)); return fail(PSD_EHIP); } } while (0)
    CK(hipStreamCreateWithFlags(&c->stream, hipStreamNonBlocking));
    CK(hipMalloc(&c->pool_mem, pool_bytes));
    c->pool.base = (char*)c->pool_mem;
    c->pool.size = pool_bytes;
    if ((rc = model_kernels_init(c->err)) != PSD_OK) return fail(rc);
    if ((rc = psd_accept_noalloc_init()) != PSD_OK) { strncpy(c->err, tls_error(), 511); return fail(rc); }
    const char* tags[3] = {"draft", "qualifier", "target"};
    const bool scramble = (params->flags & 0x100) != 0;  // test aid: physical KV pages out of logical order
    for (int i = 0; i < 3; ++i)
        if ((rc = model_init(c->M[i], *descs[i], tags[i], params->max_seq, scramble, c->pool, c->stream, c->err)) != PSD_OK)
            return fail(rc);
    const int V = c->V;
    bool ok = true;
    auto take = [&](size_t n) { void* p = c->pool.take(n); if (!p) ok = false; return p; };
    c->DL = (float*)take((size_t)c->k1cap * V * 4);
    c->QL = (float*)take((size_t)(c->k2cap + 1) * V * 4);
    c->TL = (float*)take((size_t)(c->k2cap + 1) * V * 4);
    c->HL = (float*)take((size_t)kMaxW * V * 4);
    c->acc_ws_bytes = accept_workspace_bytes(1, kMaxW - 1, V);
    c->acc_ws = take(c->acc_ws_bytes);
    c->acc_out = (AcceptOut*)take(sizeof(AcceptOut));
    c->acc_div = (float*)take(kMaxW * 4);
    c->samp_part = take((size_t)accept_chunks(V) * 8);
    c->samp_tok = (int32_t*)take(4);
    c->chain = (SampleCtl*)take(sizeof(SampleCtl));
    c->round_tok = (int32_t*)take(kMaxW * 4);
    c->win_tok = (int32_t*)take(kMaxW * 4);
    c->rs_ws = take(row_stats_workspace_bytes(kMaxW, V));
    c->rs_acc = (double*)take(9 * sizeof(double));
    if (!ok) { set_error(c->err, "psd_create: device pool too small"); return fail(PSD_ENOMEM); }
    CK(hipHostMalloc((void**)&c->stage, (size_t)kStageSlots * kStageSlotBytes, hipHostMallocDefault));
    CK(hipHostMalloc((void**)&c->res, sizeof(RoundResult), hipHostMallocDefault));
    for (auto& e : c->ev) CK(hipEventCreate(&e));
    for (auto& st : c->aux) CK(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    for (auto& e : c->aux_ready) CK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    for (auto& e : c->aux_done) CK(hipEventCreateWithFlags(&e, hipEventDisableTiming));
    CK(hipStreamSynchronize(c->stream));
#undef CK
    *out = c;
    return PSD_OK;
}

extern "C" void psd_destroy(psd_ctx* c) {
    if (!c) return;
    (void)hipSetDevice(c->device);
    if (c->stream) (void)hipStreamSynchronize(c->stream);
    for (auto& st : c->aux) if (st) { (void)hipStreamSynchronize(st); (void)hipStreamDestroy(st); }
    drop_graphs(c);
    c->prof.clear();
    for (auto& e : c->ev) if (e) (void)hipEventDestroy(e);
    for (auto& e : c->aux_ready) if (e) (void)hipEventDestroy(e);
    for (auto& e : c->aux_done) if (e) (void)hipEventDestroy(e);
    if (c->stage) (void)hipHostFree(c->stage);
    if (c->res) (void)hipHostFree(c->res);
    if (c->pool_mem) (void)hipFree(c->pool_mem);
    if (c->stream) (void)hipStreamDestroy(c->stream);
    delete c;
}

extern "C" const char* psd_last_error(const psd_ctx* c) { return c ? c->err : tls_error(); }

extern "C" int psd_set_decoding(psd_ctx* c, float T_q, float T_t, int32_t k1, int32_t k2, float temperature) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_set_decoding: null context");
    psd_params p = c->prm;
    p.T_q = T_q; p.T_t = T_t; p.k1 = k1; p.k2 = k2; p.temperature = temperature;
    int rc = validate_params(&p, c->err);
    if (rc != PSD_OK) return rc;
    if (k1 > c->k1cap || k2 > c->k2cap)
        PSD_FAIL(PSD_EINVAL, c->err, "psd_set_decoding: k1=%d k2=%d exceed the context's capacity (%d, %d)", k1, k2, c->k1cap, c->k2cap);
    if (temperature != c->prm.temperature) drop_graphs(c);  // the temperature is baked into captured sampling nodes
    c->prm = p;
    return PSD_OK;
}

extern "C" int psd_set_trace(psd_ctx* c, psd_trace_fn fn, void* user) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_set_trace: null context");
    c->trace = fn;
    c->trace_user = user;
    return PSD_OK;
}

extern "C" int psd_profile(psd_ctx* c, int32_t on) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_profile: null context");
    PSD_HIP(hipStreamSynchronize(c->stream), c->err);
    c->prof.flush();
    if (on) c->prof.clear();
    c->prof.on = on != 0;
    return PSD_OK;
}

extern "C" int psd_kernel_stats(psd_ctx* c, psd_kernel_stat* out, int32_t cap) {
    if (!c || !out || cap < 0) PSD_FAIL(PSD_EINVAL, c ? c->err : tls_error(), "psd_kernel_stats: bad argument");
    PSD_HIP(hipStreamSynchronize(c->stream), c->err);
    c->prof.flush();
    int n = std::min<int>(cap, (int)c->prof.rows.size());
    for (int i = 0; i < n; ++i) {
        memcpy(out[i].name, c->prof.rows[i].name, sizeof(out[i].name));
        out[i].launches = c->prof.rows[i].launches;
        out[i].ms_total = c->prof.rows[i].ms;
        out[i].bytes_total = c->prof.rows[i].bytes;
    }
    return n;
}

extern "C" int psd_forward(psd_ctx* c, int32_t which, const int32_t* tokens, int32_t w, int32_t pos0, float* logits_out) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_forward: null context");
    if (which < 0 || which > 2 || !tokens) PSD_FAIL(PSD_EINVAL, c->err, "psd_forward: bad argument");
    Model& M = c->M[which];
    const int wcap = logits_out ? kMaxW : M.ingest_max;   // wider passes only ingest
    if (w < 1 || w > wcap) PSD_FAIL(PSD_ESHAPE, c->err, "psd_forward: width %d outside [1, %d]", w, wcap);
    if (pos0 < 0 || pos0 + w > M.max_seq) PSD_FAIL(PSD_ESHAPE, c->err, "psd_forward: positions [%d, %d) exceed max_seq %d", pos0, pos0 + w, M.max_seq);
    if (pos0 > M.len) PSD_FAIL(PSD_EINVAL, c->err, "psd_forward: pos0 %d but only %d KV rows are valid", pos0, M.len);
    int rc = check_tokens(c, tokens, w);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipSetDevice(c->device), c->err);
    if ((rc = map_pages(c, M, pos0, pos0 + w)) != PSD_OK) return rc;
    PassDesc d;
    fill_desc(d, tokens, 0, w, 0, logits_out ? w : 0, 0);
    d.pos0 = pos0;
    if ((rc = upload(c, M.desc, &d, desc_bytes(d))) != PSD_OK) return rc;
    if ((rc = run_pass(c, which, wclass(w), logits_out ? c->HL : nullptr, false)) != PSD_OK) return rc;
    M.len = pos0 + w;
    if ((rc = stage_sync(c)) != PSD_OK) return rc;
    if (logits_out) PSD_HIP(hipMemcpy(logits_out, c->HL, (size_t)w * c->V * sizeof(float), hipMemcpyDeviceToHost), c->err);
    return PSD_OK;
}

extern "C" int psd_generate(psd_ctx* c, const int32_t* prompt, int32_t n_prompt, int32_t n_new, uint64_t seed,
                            int32_t* out_tokens, psd_stats* out_stats) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_generate: null context");
    if (!prompt || n_prompt < 1 || n_new < 0 || (n_new > 0 && !out_tokens)) PSD_FAIL(PSD_EINVAL, c->err, "psd_generate: bad argument");
    const int V = c->V;
    const int greedy = (c->prm.flags & PSD_FLAG_GREEDY) ? 1 : 0;
    const int assisted = greedy ? 2 : (c->prm.flags & PSD_FLAG_ASSISTED) ? 1 : 0;  // rule of the qualifier stage
    // thresholds and window lengths of the current outer iteration: fixed, or moved by the adaptive controller
    Controller& ctl = c->ctl;
    int k1 = c->prm.k1, k2 = c->prm.k2;
    float T_q = c->prm.T_q, T_t = c->prm.T_t;
    if (ctl.on) {
        ctl.start(T_q, T_t, k2);
        k1 = ctl.k1; k2 = ctl.k2; T_q = ctl.tau_q(); T_t = ctl.tau_t();
    }
    const int cap = n_prompt + n_new + (ctl.on ? (int)ctl.cfg.k2_max : k2) + 2;
    if (cap > c->prm.max_seq) PSD_FAIL(PSD_ESHAPE, c->err, "psd_generate: n_prompt + n_new + k2 + 2 = %d exceeds max_seq %d", cap, c->prm.max_seq);
    int rc = check_tokens(c, prompt, n_prompt);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipSetDevice(c->device), c->err);
    Model &D = c->M[0], &Q = c->M[1], &T = c->M[2];
    psd_stats st;
    memset(&st, 0, sizeof(st));
    std::vector<int32_t> seq(cap + kMaxW, 0);
    memcpy(seq.data(), prompt, (size_t)n_prompt * sizeof(int32_t));
    std::vector<float> tr_p, tr_q;  // trace copies
    int C = n_prompt;
    for (int i = 0; i < 3; ++i) c->M[i].len = 0;
    PSD_HIP(hipMemsetAsync(c->rs_acc, 0, 9 * sizeof(double), c->stream), c->err);

    PSD_HIP(hipEventRecord(c->ev[0], c->stream), c->err);
    if ((rc = prefill_all(c, seq.data(), C - 1)) != PSD_OK) return rc;
    PSD_HIP(hipEventRecord(c->ev[1], c->stream), c->err);

    while (C - n_prompt < n_new) {
        int nbuf = 0;
        const int64_t pq0 = st.proposed_q, aq0 = st.accepted_q;
        if (ctl.on) {
            const int32_t row[4] = {k1, k2, ctl.pos_q, ctl.pos_t};
            ctl.log.insert(ctl.log.end(), row, row + 4);
            if (c->trace) {
                const float thr[2] = {T_q, T_t};
                c->trace(c->trace_user, 7, (uint32_t)C, k2, k1, nullptr, nullptr, nullptr, ctl.pos_q, ctl.pos_t, thr);
            }
        }
        while (nbuf < k2) {
            const int m = std::min(k1, k2 - nbuf), L = C + nbuf;
            // draft: first step ingests the host-known uncached suffix, the rest chain on the device
            const int hq = L - Q.len;  // host-known tokens the qualifier still has to ingest
            if (L - D.len < 1 || L - D.len > 3 || hq < 1 || hq > 2)
                PSD_FAIL(PSD_EINVAL, c->err, "internal: cache lengths out of step (L=%d D=%d Q=%d)", L, D.len, Q.len);
            if ((rc = map_pages(c, D, D.len, L + m)) != PSD_OK) return rc;
            if ((rc = map_pages(c, Q, Q.len, L + m)) != PSD_OK) return rc;
            PassDesc dd, qd;
            fill_desc(dd, seq.data(), D.len, L, 0, 1, 0);
            fill_desc(qd, seq.data(), Q.len, L, m, m + 1, nbuf);
            SampleCtl sc{seed, L, 0, hq, 0};
            if ((rc = upload(c, D.desc, &dd, desc_bytes(dd))) != PSD_OK) return rc;
            if ((rc = upload(c, Q.desc, &qd, desc_bytes(qd))) != PSD_OK) return rc;
            if ((rc = upload(c, c->chain, &sc, sizeof(sc))) != PSD_OK) return rc;
            c->timer.begin(c->stream, 0);
            // the first step also ingests what the draft has not cached (1 to 3 tokens), the others one token each
            for (int i = 0; i < m; ++i)
                if ((rc = run_pass(c, 0, wclass(i == 0 ? L - D.len : 1), c->DL, true, true)) != PSD_OK) return rc;
            c->timer.end(c->stream);
            st.passes_d += m;
            c->timer.begin(c->stream, 1);
            if ((rc = run_pass(c, 1, wclass(hq + m), c->QL, false, true)) != PSD_OK) return rc;
            c->timer.end(c->stream);
            st.passes_q++;
            if ((rc = note_rows(c, 0, c->DL, m)) != PSD_OK) return rc;
            if ((rc = note_rows(c, 1, c->QL + (size_t)nbuf * V, m + 1)) != PSD_OK) return rc;
            const int bonus = nbuf + m < k2;
            if ((rc = accept_sync(c, "accept stage1", c->QL + (size_t)nbuf * V, c->DL, c->round_tok, m, T_q, seed,
                                  (uint32_t)L, 1u, bonus, assisted, m)) != PSD_OK) return rc;
            const int n = c->res->acc.n_accepted, y = c->res->acc.next_token, has_y = y >= 0;
            if (n < 0 || n > m || (!has_y && (n < m || bonus))) PSD_FAIL(PSD_EHIP, c->err, "internal: impossible ACCEPT result (n=%d y=%d)", n, y);
            if (c->trace) {
                if ((rc = copy_rows_to_host(c, tr_q, c->DL, m)) != PSD_OK) return rc;
                if ((rc = copy_rows_to_host(c, tr_p, c->QL + (size_t)nbuf * V, m + 1)) != PSD_OK) return rc;
                for (int i = 0; i < m; ++i)
                    c->trace(c->trace_user, greedy ? 6 : 0, (uint32_t)(L + i), 0, 0, tr_q.data() + (size_t)i * V, nullptr, nullptr, 0, c->res->tok[i], nullptr);
                c->trace(c->trace_user, greedy ? 4 : assisted ? 3 : 1, (uint32_t)L, m, bonus, tr_p.data(), tr_q.data(), c->res->tok, n, y,
                         c->res->div);
            }
            for (int i = 0; i < n; ++i) seq[L + i] = c->res->tok[i];
            if (has_y) seq[L + n] = y;
            nbuf += n + has_y;
            D.len = std::min(L + m - 1, L + n);  // the draft never ingested its last proposal
            Q.len = std::min(L + m, L + n);
            st.proposed_q += m;
            st.accepted_q += n;
            st.fuzzy_q += c->res->acc.n_fuzzy;
        }
        // target verifies the window
        const int wT = C + k2 - T.len;
        if (wT != k2 + 1) PSD_FAIL(PSD_EINVAL, c->err, "internal: target cache out of step (C=%d T=%d)", C, T.len);
        if ((rc = map_pages(c, T, T.len, C + k2)) != PSD_OK) return rc;
        PassDesc td;
        fill_desc(td, seq.data(), T.len, C + k2, 0, k2 + 1, 0);
        if ((rc = upload(c, T.desc, &td, desc_bytes(td))) != PSD_OK) return rc;
        if ((rc = upload(c, c->win_tok, seq.data() + C, k2 * sizeof(int32_t))) != PSD_OK) return rc;
        c->timer.begin(c->stream, 2);
        if ((rc = run_pass(c, 2, wclass(wT), c->TL, false, true)) != PSD_OK) return rc;
        c->timer.end(c->stream);
        st.passes_t++;
        if ((rc = note_rows(c, 2, c->TL, k2 + 1)) != PSD_OK) return rc;
        if ((rc = accept_sync(c, "accept stage2", c->TL, c->QL, c->win_tok, k2, T_t, seed, (uint32_t)C, 2u, 1,
                              greedy ? 2 : 0, 0)) != PSD_OK) return rc;
        const int n = c->res->acc.n_accepted, y = c->res->acc.next_token;
        if (n < 0 || n > k2 || y < 0) PSD_FAIL(PSD_EHIP, c->err, "internal: impossible ACCEPT result (n=%d y=%d)", n, y);
        if (c->trace) {
            if ((rc = copy_rows_to_host(c, tr_p, c->TL, k2 + 1)) != PSD_OK) return rc;
            if ((rc = copy_rows_to_host(c, tr_q, c->QL, k2)) != PSD_OK) return rc;
            c->trace(c->trace_user, greedy ? 5 : 2, (uint32_t)C, k2, 1, tr_p.data(), tr_q.data(), seq.data() + C, n, y, c->res->div);
        }
        seq[C + n] = y;
        T.len = std::min(T.len + wT, C + n);
        Q.len = std::min(Q.len, C + n);
        D.len = std::min(D.len, C + n);
        C += n + 1;
        st.proposed_t += k2;
        st.accepted_t += n;
        st.fuzzy_t += c->res->acc.n_fuzzy;
        if (ctl.on) {   // this iteration's counts set the next iteration's parameters
            ctl.observe(n, st.proposed_q - pq0, st.accepted_q - aq0);
            k1 = ctl.k1; k2 = ctl.k2; T_q = ctl.tau_q(); T_t = ctl.tau_t();
        }
    }
    PSD_HIP(hipEventRecord(c->ev[2], c->stream), c->err);
    PSD_HIP(hipEventSynchronize(c->ev[2]), c->err);
    float ms = 0.f;
    PSD_HIP(hipEventElapsedTime(&ms, c->ev[0], c->ev[1]), c->err);
    st.ms_prefill = ms;
    PSD_HIP(hipEventElapsedTime(&ms, c->ev[1], c->ev[2]), c->err);
    st.ms_decode = ms;
    double stage_ms[4] = {0, 0, 0, 0};
    c->timer.collect(stage_ms);
    st.ms_d = stage_ms[0]; st.ms_q = stage_ms[1]; st.ms_t = stage_ms[2]; st.ms_accept = stage_ms[3];
    if (n_new > 0) memcpy(out_tokens, seq.data() + n_prompt, (size_t)n_new * sizeof(int32_t));
    if (out_stats) *out_stats = st;
    return PSD_OK;
}

extern "C" int psd_set_adaptive(psd_ctx* c, const psd_adapt* cfg) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_set_adaptive: null context");
    if (!cfg) { c->ctl.on = false; return PSD_OK; }
    if (cfg->k2_min < 1 || cfg->k2_max < cfg->k2_min || cfg->k2_max > c->k2cap || cfg->k1_max < 1 || cfg->k1_max > c->k1cap)
        PSD_FAIL(PSD_EINVAL, c->err, "psd_set_adaptive: windows k2 [%d, %d], k1 <= %d outside the context's capacity (k1 %d, k2 %d)",
                 cfg->k2_min, cfg->k2_max, cfg->k1_max, c->k1cap, c->k2cap);
    if (cfg->steps < 1 || cfg->period < 1) PSD_FAIL(PSD_EINVAL, c->err, "psd_set_adaptive: steps=%d period=%d", cfg->steps, cfg->period);
    if (!(cfg->T_q_min >= 0.f) || !(cfg->T_q_max >= cfg->T_q_min) || !(cfg->T_t_min >= 0.f) || !(cfg->T_t_max >= cfg->T_t_min))
        PSD_FAIL(PSD_EINVAL, c->err, "psd_set_adaptive: threshold bands must satisfy 0 <= min <= max");
    c->ctl.cfg = *cfg;
    c->ctl.on = true;
    c->ctl.log.clear();
    return PSD_OK;
}

extern "C" int psd_get_adaptive_log(psd_ctx* c, int32_t* out, int32_t cap) {
    if (!c || (cap > 0 && !out) || cap < 0) PSD_FAIL(PSD_EINVAL, c ? c->err : tls_error(), "psd_get_adaptive_log: bad argument");
    const int n = (int)(c->ctl.log.size() / 4);
    if (cap > 0 && n > 0) memcpy(out, c->ctl.log.data(), (size_t)std::min(n, (int)cap) * 4 * sizeof(int32_t));
    return n;
}

extern "C" int psd_set_row_stats(psd_ctx* c, int32_t on) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_set_row_stats: null context");
    c->prm.flags = on ? (c->prm.flags | PSD_FLAG_ROW_STATS) : (c->prm.flags & ~PSD_FLAG_ROW_STATS);
    return PSD_OK;
}

extern "C" int psd_get_row_stats(psd_ctx* c, double* out) {
    if (!c || !out) PSD_FAIL(PSD_EINVAL, c ? c->err : tls_error(), "psd_get_row_stats: null pointer");
    PSD_HIP(hipSetDevice(c->device), c->err);
    PSD_HIP(hipStreamSynchronize(c->stream), c->err);
    double h[9];
    PSD_HIP(hipMemcpy(h, c->rs_acc, sizeof(h), hipMemcpyDeviceToHost), c->err);
    for (int m = 0; m < 3; ++m) {
        out[3 * m] = h[3 * m];
        out[3 * m + 1] = h[3 * m] > 0 ? h[3 * m + 1] / h[3 * m] : 0.0;
        out[3 * m + 2] = h[3 * m] > 0 ? h[3 * m + 2] / h[3 * m] : 0.0;
    }
    return PSD_OK;
}

extern "C" int psd_set_greedy(psd_ctx* c, int32_t on) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_set_greedy: null context");
    const int32_t before = c->prm.flags;
    c->prm.flags = on ? (c->prm.flags | PSD_FLAG_GREEDY) : (c->prm.flags & ~PSD_FLAG_GREEDY);
    if (before != c->prm.flags) {   // captured sampling steps hold the other rule
        PSD_HIP(hipSetDevice(c->device), c->err);
        PSD_HIP(hipStreamSynchronize(c->stream), c->err);
        drop_graphs(c);
    }
    return PSD_OK;
}

extern "C" int psd_set_assisted(psd_ctx* c, int32_t on) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_set_assisted: null context");
    c->prm.flags = on ? (c->prm.flags | PSD_FLAG_ASSISTED) : (c->prm.flags & ~PSD_FLAG_ASSISTED);
    return PSD_OK;
}

extern "C" int psd_generate_sd(psd_ctx* c, int32_t proposer, int32_t k, float tau, const int32_t* prompt,
                               int32_t n_prompt, int32_t n_new, uint64_t seed, int32_t* out_tokens,
                               psd_stats* out_stats) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_generate_sd: null context");
    if ((proposer != 0 && proposer != 1) || !prompt || n_prompt < 1 || n_new < 0 || (n_new > 0 && !out_tokens))
        PSD_FAIL(PSD_EINVAL, c->err, "psd_generate_sd: bad argument");
    if (k < 1 || k > c->k2cap) PSD_FAIL(PSD_EINVAL, c->err, "psd_generate_sd: k=%d outside [1, %d]", k, c->k2cap);
    if (!(tau >= 0.f)) PSD_FAIL(PSD_EINVAL, c->err, "psd_generate_sd: tau=%g", tau);
    const int V = c->V;
    const int greedy = (c->prm.flags & PSD_FLAG_GREEDY) ? 1 : 0;
    const int cap = n_prompt + n_new + k + 2;
    if (cap > c->prm.max_seq) PSD_FAIL(PSD_ESHAPE, c->err, "psd_generate_sd: n_prompt + n_new + k + 2 = %d exceeds max_seq %d", cap, c->prm.max_seq);
    int rc = check_tokens(c, prompt, n_prompt);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipSetDevice(c->device), c->err);
    Model &P = c->M[proposer], &T = c->M[2];
    psd_stats st;
    memset(&st, 0, sizeof(st));
    std::vector<int32_t> seq(cap + kMaxW, 0);
    memcpy(seq.data(), prompt, (size_t)n_prompt * sizeof(int32_t));
    std::vector<float> tr_p, tr_q;
    int C = n_prompt;
    P.len = 0; T.len = 0;
    PSD_HIP(hipMemsetAsync(c->rs_acc, 0, 9 * sizeof(double), c->stream), c->err);
    PSD_HIP(hipEventRecord(c->ev[0], c->stream), c->err);
    if ((rc = prefill_all(c, seq.data(), C - 1, (1u << proposer) | 4u)) != PSD_OK) return rc;
    PSD_HIP(hipEventRecord(c->ev[1], c->stream), c->err);
    while (C - n_prompt < n_new) {
        // the proposer's first step ingests the host-known uncached suffix (two tokens after a fully accepted
        // pass: its own last proposal and the bonus token), the rest chain on the device
        const int hp = C - P.len, ht = C - T.len;
        if (hp < 1 || hp > 2 || ht != 1)
            PSD_FAIL(PSD_EINVAL, c->err, "internal: cache lengths out of step (C=%d P=%d T=%d)", C, P.len, T.len);
        if ((rc = map_pages(c, P, P.len, C + k)) != PSD_OK) return rc;
        if ((rc = map_pages(c, T, T.len, C + k)) != PSD_OK) return rc;
        PassDesc pd, td;
        fill_desc(pd, seq.data(), P.len, C, 0, 1, 0);
        fill_desc(td, seq.data(), T.len, C, k, k + 1, 0);
        SampleCtl sc{seed, C, 0, ht, 0};
        if ((rc = upload(c, P.desc, &pd, desc_bytes(pd))) != PSD_OK) return rc;
        if ((rc = upload(c, T.desc, &td, desc_bytes(td))) != PSD_OK) return rc;
        if ((rc = upload(c, c->chain, &sc, sizeof(sc))) != PSD_OK) return rc;
        c->timer.begin(c->stream, proposer);
        for (int i = 0; i < k; ++i)
            if ((rc = run_pass(c, proposer, wclass(i == 0 ? C - P.len : 1), c->QL, true, true, 2)) != PSD_OK) return rc;
        c->timer.end(c->stream);
        (proposer == 0 ? st.passes_d : st.passes_q) += k;
        c->timer.begin(c->stream, 2);
        if ((rc = run_pass(c, 2, wclass(ht + k), c->TL, false, true)) != PSD_OK) return rc;
        c->timer.end(c->stream);
        st.passes_t++;
        if ((rc = note_rows(c, proposer, c->QL, k)) != PSD_OK) return rc;
        if ((rc = note_rows(c, 2, c->TL, k + 1)) != PSD_OK) return rc;
        if ((rc = accept_sync(c, "accept stage2", c->TL, c->QL, c->round_tok, k, tau, seed, (uint32_t)C, 2u, 1,
                              greedy ? 2 : 0, k)) != PSD_OK)
            return rc;
        const int n = c->res->acc.n_accepted, y = c->res->acc.next_token;
        if (n < 0 || n > k || y < 0) PSD_FAIL(PSD_EHIP, c->err, "internal: impossible ACCEPT result (n=%d y=%d)", n, y);
        if (c->trace) {
            if ((rc = copy_rows_to_host(c, tr_q, c->QL, k)) != PSD_OK) return rc;
            if ((rc = copy_rows_to_host(c, tr_p, c->TL, k + 1)) != PSD_OK) return rc;
            for (int i = 0; i < k; ++i)
                c->trace(c->trace_user, greedy ? 6 : 0, (uint32_t)(C + i), 0, 0, tr_q.data() + (size_t)i * V, nullptr, nullptr, 0, c->res->tok[i], nullptr);
            c->trace(c->trace_user, greedy ? 5 : 2, (uint32_t)C, k, 1, tr_p.data(), tr_q.data(), c->res->tok, n, y, c->res->div);
        }
        for (int i = 0; i < n; ++i) seq[C + i] = c->res->tok[i];
        seq[C + n] = y;
        P.len = std::min(C + k - 1, C + n);  // the proposer never ingested its last proposal
        T.len = std::min(T.len + ht + k, C + n);
        C += n + 1;
        st.proposed_t += k;
        st.accepted_t += n;
        st.fuzzy_t += c->res->acc.n_fuzzy;
    }
    PSD_HIP(hipEventRecord(c->ev[2], c->stream), c->err);
    PSD_HIP(hipEventSynchronize(c->ev[2]), c->err);
    float ms = 0.f;
    PSD_HIP(hipEventElapsedTime(&ms, c->ev[0], c->ev[1]), c->err);
    st.ms_prefill = ms;
    PSD_HIP(hipEventElapsedTime(&ms, c->ev[1], c->ev[2]), c->err);
    st.ms_decode = ms;
    double stage_ms[4] = {0, 0, 0, 0};
    c->timer.collect(stage_ms);
    st.ms_d = stage_ms[0]; st.ms_q = stage_ms[1]; st.ms_t = stage_ms[2]; st.ms_accept = stage_ms[3];
    if (n_new > 0) memcpy(out_tokens, seq.data() + n_prompt, (size_t)n_new * sizeof(int32_t));
    if (out_stats) *out_stats = st;
    return PSD_OK;
}

extern "C" int psd_generate_plain(psd_ctx* c, int32_t which, const int32_t* prompt, int32_t n_prompt, int32_t n_new,
                                  uint64_t seed, int32_t* out_tokens, psd_stats* out_stats) {
    if (!c) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_generate_plain: null context");
    if (which < 0 || which > 2 || !prompt || n_prompt < 1 || n_new < 0 || (n_new > 0 && !out_tokens))
        PSD_FAIL(PSD_EINVAL, c->err, "psd_generate_plain: bad argument");
    if (n_prompt + n_new > c->prm.max_seq) PSD_FAIL(PSD_ESHAPE, c->err, "psd_generate_plain: exceeds max_seq");
    int rc = check_tokens(c, prompt, n_prompt);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipSetDevice(c->device), c->err);
    Model& M = c->M[which];
    psd_stats st;
    memset(&st, 0, sizeof(st));
    std::vector<int32_t> seq(n_prompt + n_new + 1, 0);
    memcpy(seq.data(), prompt, (size_t)n_prompt * sizeof(int32_t));
    M.len = 0;
    PSD_HIP(hipEventRecord(c->ev[0], c->stream), c->err);
    if ((rc = prefill(c, which, seq.data(), n_prompt - 1)) != PSD_OK) return rc;
    PSD_HIP(hipEventRecord(c->ev[1], c->stream), c->err);
    for (int i = 0; i < n_new; ++i) {
        const int L = n_prompt + i;
        if ((rc = map_pages(c, M, M.len, L)) != PSD_OK) return rc;
        PassDesc d;
        fill_desc(d, seq.data(), M.len, L, 0, 1, 0);
        if ((rc = upload(c, M.desc, &d, desc_bytes(d))) != PSD_OK) return rc;
        if ((rc = run_pass(c, which, wclass(L - M.len), c->HL, false)) != PSD_OK) return rc;
        if ((rc = sample_launch(c->HL, 1, c->V, c->prm.temperature, seed, (uint32_t)L, nullptr, c->samp_tok, c->samp_part, c->stream, c->err,
                                (c->prm.flags & PSD_FLAG_GREEDY) ? 1 : 0)) != PSD_OK) return rc;
        PSD_HIP(hipMemcpyAsync(c->res->tok, c->samp_tok, sizeof(int32_t), hipMemcpyDeviceToHost, c->stream), c->err);
        if ((rc = stage_sync(c)) != PSD_OK) return rc;
        seq[L] = c->res->tok[0];
        M.len = L;
        (which == 0 ? st.passes_d : which == 1 ? st.passes_q : st.passes_t)++;
    }
    PSD_HIP(hipEventRecord(c->ev[2], c->stream), c->err);
    PSD_HIP(hipEventSynchronize(c->ev[2]), c->err);
    float ms = 0.f;
    PSD_HIP(hipEventElapsedTime(&ms, c->ev[0], c->ev[1]), c->err);
    st.ms_prefill = ms;
    PSD_HIP(hipEventElapsedTime(&ms, c->ev[1], c->ev[2]), c->err);
    st.ms_decode = ms;
    if (n_new > 0) memcpy(out_tokens, seq.data() + n_prompt, (size_t)n_new * sizeof(int32_t));
    if (out_stats) *out_stats = st;
    return PSD_OK;
}
