// One Llama-style decoder on the device: weight layout, KV pages, scratch and the forward pass.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "psd_host.h"

namespace psd {

constexpr int kPage = 64;        // tokens per KV page
constexpr int kAttnSplit = 128;  // keys per attention workgroup (two pages); boundaries are absolute positions
constexpr int kFoldSplits = 12;  // up to this many key ranges the narrow o projection merges the partials itself

// Context buckets: a pass is launched for the smallest bucket of key ranges that holds every key it can attend to
// (the host knows an upper bound of the pass's last position), so the attention grid does not grow with max_seq and
// the choices that depend on the context length are fixed per captured graph.  The last bucket stands for "all
// key ranges of the cache".
constexpr int kCtxBuckets[] = {8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 1 << 30};
constexpr int kNumCtxBuckets = sizeof(kCtxBuckets) / sizeof(kCtxBuckets[0]);
inline int ctx_bucket_index(int kv_upto) {   // kv_upto: upper bound of (first position + tokens) of the pass
    const int ranges = (kv_upto + kAttnSplit - 1) / kAttnSplit;
    int i = 0;
    while (kCtxBuckets[i] < ranges) ++i;
    return i;
}
constexpr int kMaxW = PSD_MAX_WIDTH;   // widest pass that can produce logits (and the widest the ABI takes)
constexpr int kCols = 512;             // widest pass at all: prompt ingestion of bf16 models, no logits
constexpr int kWideCT = kCols / 16;    // column tiles of the operand buffers those passes use

// Launch classes of the passes that can produce logits: a pass of w tokens is launched as the smallest class >= w.
// Kernels never load operand columns beyond their class, so a finer class moves fewer bytes; each class has its own
// captured graph.
constexpr int kNarrowClasses[] = {1, 2, 4, 6, 8, 12, 16, 24, 32};
constexpr int kNumNarrowClasses = sizeof(kNarrowClasses) / sizeof(kNarrowClasses[0]);
inline int narrow_class_index(int w) {   // -1 when w is wider than the widest class
    for (int i = 0; i < kNumNarrowClasses; ++i)
        if (w <= kNarrowClasses[i]) return i;
    return -1;
}

// What one forward pass has to do; lives in DEVICE memory so that a captured graph can be replayed
// with new contents.  Written by the host before a pass, or by the sampling kernel for the draft chain.
struct PassDesc {
    int32_t w;           // tokens in this pass (1..32; up to 512 while ingesting a prompt)
    int32_t pos0;        // position of the first token == number of valid KV rows before the pass
    int32_t n_logit;     // the last n_logit tokens get logit rows (0 = none)
    int32_t logit_row0;  // first destination row in the logits buffer
    int32_t tok[kCols];
};

struct LayerW {
    const float* attn_norm;
    const void* wqkv;  // [(H+2KV)*hd][d]
    const void* wo;    // [d][H*hd]
    const float* ffn_norm;
    const void* wgu;   // [2F][d]: gate rows, then up rows
    const void* wd;    // [d][F]
};

// Pool sub-allocator: bump pointer, 256-byte granules.  The pool itself is one hipMalloc owned by the context.
struct Pool {
    char* base = nullptr;
    size_t size = 0, used = 0;
    bool dry = false;  // sizing run: hands out nothing, only counts
    void* take(size_t bytes) {
        size_t off = (used + 255) & ~(size_t)255;
        used = off + bytes;
        if (dry) return nullptr;
        if (used > size) return nullptr;
        return base + off;
    }
};

struct KernelAcc {  // profiling row
    char name[48];
    int64_t launches = 0;
    double ms = 0, bytes = 0;
};

struct Profiler {
    bool on = false;
    std::vector<KernelAcc> rows;
    struct Pending { int row; hipEvent_t a, b; };
    std::vector<Pending> pending;
    std::vector<hipEvent_t> free_events;
    int row_of(const char* name);
    hipEvent_t get_event();
    void begin(hipStream_t s, int row, double bytes);
    void end(hipStream_t s);
    void flush();  // synchronises and folds pending event pairs into rows
    void clear();
    ~Profiler();
};

struct Model {
    // shape
    int L = 0, d = 0, H = 0, KV = 0, hd = 0, F = 0, V = 0, Vpad = 0, nqkv = 0;
    int dtype = 0;
    float theta = 0, eps = 0;
    int max_seq = 0, n_pages = 0, nsplit_max = 0;
    const char* tag = "";
    // weights (device)
    const void* embed = nullptr;  // bf16: tiled [Vpad/16][d/32][64][8]; f32: row-major [V][d]
    std::vector<LayerW> layers;
    const float* final_norm = nullptr;
    const float2* rope = nullptr;  // [max_seq][hd/2] (cos, sin)
    // KV cache, 4 bytes per element.  fp32 models: page p, layer l, kv head g, k/v -> [slot][hd] floats.
    // bf16 models: four bf16 planes per (p, l, g): K hi [slot][hd], K lo, V hi [hd][slot] (MFMA operand order), V lo
    void* kv = nullptr;
    int32_t* page_table = nullptr;  // device, [n_pages] logical block -> physical page
    std::vector<int32_t> h_page_table;
    std::vector<int32_t> free_pages;
    int pages_mapped = 0;
    // scratch (device)
    float* x = nullptr;       // residual stream [512][d]
    void* xb = nullptr;       // GEMM input operand (bf16 hi/lo tiles, or plain fp32 rows): normalised residual
    void* xb2 = nullptr;      // second operand buffer: attention output / SwiGLU output (bf16 path)
    float* ss = nullptr;      // [d/16][32] partial sums of squares of the residual stream (bf16 path)
    void* xbw = nullptr;      // the same three for prompt-ingestion passes: operands with 32 column tiles, [d/16][512] partials
    void* xbw2 = nullptr;
    float* ssw = nullptr;
    float* qkv = nullptr;     // [512][nqkv]
    float* gu = nullptr;      // [32][2F]
    float* attn_part = nullptr;  // [nsplit_max][512][H][hd + 2]
    PassDesc* desc = nullptr;
    // host mirror
    int len = 0;  // valid KV rows
    int ingest_max = 0;  // widest pass that may ingest a prompt (32 for fp32 models; 128 or 512 for bf16 ones)
    int ctx_bucket = kNumCtxBuckets - 1;  // set by the caller before model_forward: bucket of the pass's last position
    size_t weight_bytes = 0;  // bytes one pass streams (all matrices once)
};

size_t model_pool_bytes(const psd_model_desc& m, int max_seq);

// Carves a model out of the pool and uploads + re-tiles its weights (synchronous; uses a temporary staging buffer).
int model_init(Model& M, const psd_model_desc& desc, const char* tag, int max_seq, bool scramble_pages, Pool& pool,
               hipStream_t stream, char* err);

// Makes sure KV pages exist for positions < upto and frees pages wholly beyond `keep`, in the host mirror of the page
// table; reports which entries changed ([*first_changed, +*n_changed), none: 0 entries) so that the caller can upload
// just those (device entries of unmapped blocks are never read: attention stops at the pass's last position).
int model_map_pages(Model& M, int keep, int upto, int* first_changed, int* n_changed, char* err);

// Enqueues one pass described by *M.desc (already on the device).  wmax: one of kNarrowClasses = widest pass the launch must cover;
// 128, 256, 384 or 512 (bf16 models, logits == nullptr): prompt ingestion.
// logits: device [rows][V] destination (may be null when the pass produces none).
int model_forward(Model& M, int wmax, float* logits, hipStream_t stream, Profiler* prof, char* err);

int model_kernels_init(char* err);  // one-time function attributes

}  // namespace psd
