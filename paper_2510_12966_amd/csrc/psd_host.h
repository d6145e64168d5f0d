// Host-side plumbing shared by the library's translation units: error strings and HIP call checking.
#pragma once
#include <hip/hip_runtime.h>
#include <stdarg.h>
#include <stdio.h>

#include "../../include/psd.h"

namespace psd {

// last error of context-free calls on this thread (contexts keep their own copy as well)
char* tls_error();
void set_error(char* dst, const char* fmt, ...);

#define PSD_HIP(call, errbuf)                                                                         \
    do {                                                                                              \
        hipError_t e_ = (call);                                                                       \
        if (e_ != hipSuccess) {                                                                       \
            psd::set_error((errbuf), "%s failed at %s:%d: %s", #call, __FILE__, __LINE__,             \
                           hipGetErrorString(e_));                                                    \
            return PSD_EHIP;                                                                          \
        }                                                                                             \
    } while (0)

#define PSD_FAIL(code, errbuf, ...)                \
    do {                                           \
        psd::set_error((errbuf), __VA_ARGS__);     \
        return (code);                             \
    } while (0)

// ---- ACCEPT stage, device-level entry used by the scheduler and by the C ABI -------------------
struct AcceptOut {   // one per trial, device memory
    int32_t n_accepted;
    int32_t next_token;
    int32_t n_fuzzy;
    int32_t pad;
};

constexpr int kAcceptChunk = 2048;  // vocabulary entries per workgroup

inline int accept_chunks(int vocab) { return (vocab + kAcceptChunk - 1) / kAcceptChunk; }
size_t accept_workspace_bytes(int n_trials, int k, int vocab);

// Enqueues the ACCEPT kernels on `stream`.  All pointers are device memory.  div_out may be null.
// Every launch shape is checked against the workspace size before anything is enqueued.
// n_accepted_out / next_token_out (optional, both or neither): plain [n_trials] copies of the two results.
// out[b].n_accepted = -1 when the kernels' bounded wait for each other expired.
// assisted: strict match against the verifier's top prediction, replacement draw from the verifier's row
// (Section 3.4); logits_q and T are then unused and div_out receives -1.  assisted = 2: greedy stage, the
// temperature -> 0 limit (Section 3.1): the same match, replacement and bonus are the verifier's top predictions.
int accept_launch(const float* logits_p, const float* logits_q, const int32_t* tokens, int n_trials, int k,
                  int vocab, float T, float temperature, uint64_t seed, uint32_t position0, uint32_t stage,
                  int take_bonus, AcceptOut* out, float* div_out, void* workspace, size_t workspace_bytes,
                  hipStream_t stream, char* errbuf, int32_t* n_accepted_out = nullptr,
                  int32_t* next_token_out = nullptr, int assisted = 0);

// Called by whoever reads n_accepted = -1: from now on the sweep runs as two launches (no waiting between workgroups).
void accept_wait_expired();

// Where the draft chain is: device-resident so that a captured draft step can be replayed unchanged.
struct SampleCtl {
    uint64_t seed;
    int32_t position;  // absolute position of the token the next sample decides
    int32_t row;       // logits row the next sample reads (= index of the draft step in its round)
    int32_t q_base;    // slot of the qualifier pass descriptor that receives the first draft token (-1: none)
    int32_t pad;
};

// Fresh samples: row r -> token for position position0 + r.  partial: n_rows * accept_chunks(vocab) * 8 bytes.
// ctl (optional, device): when non-null, seed / position0 / first logits row come from *ctl instead.
// greedy: the top prediction of every row instead of a sample.
// tokens_out may be null: then the per-chunk winners stay in `partial` ([n_rows][accept_chunks(vocab)] KeyIdx) and the
// caller picks among them (in a kernel of its own that has more to do with the token).
int sample_launch(const float* logits, int n_rows, int vocab, float temperature, uint64_t seed, uint32_t position0,
                  const SampleCtl* ctl, int32_t* tokens_out, void* partial, hipStream_t stream, char* errbuf,
                  int greedy = 0);

// Entropy (nats) and largest probability of softmax(row / temperature) for n_rows logits rows (device memory).
// entropy / max_prob: optional [n_rows] outputs; acc: optional device double[3] {rows, sum H, sum p_max} that is
// added to.  workspace: row_stats_workspace_bytes(n_rows, vocab) bytes.
size_t row_stats_workspace_bytes(int n_rows, int vocab);
int row_stats_launch(const float* logits, int n_rows, int vocab, float temperature, float* entropy, float* max_prob,
                     double* acc, void* workspace, hipStream_t stream, char* errbuf);

}  // namespace psd
