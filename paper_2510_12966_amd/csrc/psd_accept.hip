// ACCEPT stage of one verify pass on the GPU: vocabulary-wide softmax of the verifier and proposer
// rows, Jensen-Shannon divergence per position, threshold / coin / first-reject scan and the
// replacement draw (Sections 3.1-3.2 and the fallback rule named in Section 3.4).
//
// Every logit of the k judged positions is read from HBM once.  Kernels, per call:
//   accept_clear   marks the per-chunk result slots "not written"
//   accept_sweep   one workgroup per (trial, position, chunk).  It keeps its chunk of both rows in
//                  registers, publishes the chunk's (max, sum of exponentials), waits until the other
//                  chunks of the same row have done so (they are launched next to it, so the wait is
//                  short; it is bounded by a clock and reports expiry instead of spinning on), then
//                  finishes the divergence partial from the registers.
//   accept_decide  per trial: divergence per position (fixed-order sums), coins, first-reject scan
//   accept_race    per (trial, chunk): exponential race over the ONE row that needs a replacement
//                  token: the residual max(0, p - q) of the first rejected position, or the verifier's
//                  last row for the bonus token.  Only this kernel draws vocabulary-wide random numbers.
//   accept_pick    per trial: winner of the race
// Bulk arithmetic runs in base 2 on the hardware exp2 / log2 units; the two probabilities the coin
// compares are evaluated with the accurate library functions.  No floating-point atomics: every
// partial has its own slot, reductions run in a fixed order, so results never depend on scheduling.
// When a row has more chunks than may safely wait on each other, the sweep runs as two launches
// (partials, then divergence) with the same arithmetic.
// The assisted stage (Section 3.4) needs no softmax at all: accept_top finds the verifier's top prediction
// per position, accept_decide_assisted compares tokens, and the replacement draw races over the verifier's
// own row in log form.
#include <atomic>
#include <mutex>

#include "psd_device.h"
#include "psd_host.h"

// Every fused multiply-add in this file is written out: the compiler may not fuse a product into a
// neighbouring sum on its own, so variants of one kernel round identically.
#pragma clang fp contract(off)

namespace psd {

constexpr int kAccThreads = 256;
constexpr int kQuadsPerThread = kAcceptChunk / 4 / kAccThreads;  // 2 (sampling and race kernels)
constexpr int kSweepQuads = 5, kSweepChunk = kSweepQuads * 4 * kAccThreads, kSweepWaves = kAccThreads / 64;
constexpr int kSweepMaxSlots = 256;    // per-wave results of a row that workgroups wait for in the one-launch sweep
constexpr float kLog2e = 1.4426950408889634f, kLn2 = 0.69314718055994531f;
constexpr float kBig = 1e30f;
constexpr unsigned long long kWaitTicks = 5000000ull;  // 50 ms of the 100 MHz wall clock
constexpr uint32_t kUnwritten = 0xffffffffu;           // a NaN pattern no maximum can have

// Process-wide switches, read once per launch sequence; atomics, so that contexts on different threads may read and
// flip them concurrently (a flip between two stages is harmless: both sweeps give the same bits).
static std::atomic<int> g_accept_path{0};   // 0 automatic, 1 two-launch sweep, 2 one-launch sweep where it is allowed
static std::atomic<unsigned long long> g_wait_ticks{kWaitTicks};  // bound of the wait between workgroups (0: test aid)
static std::atomic<long long> g_wait_expiries{0};   // how often a bounded wait ran out and a stage was run again

void accept_wait_expired() {
    g_accept_path.store(1);
    g_wait_expiries.fetch_add(1);
}

// base-2 maximum of a chunk and its sum of 2^(z - m), for the verifier row (p) and the proposer row (q);
// each half is published with one 64-bit store and is valid once its m is not the unwritten pattern
struct RowPart { float mp, sp, mq, sq; };
struct TokProb { float px, qx; };
struct RacePart { float key; int idx; float key_fb; int idx_fb; };

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
// the same, streaming: the sweep reads every entry exactly once
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ inline void load4_stream(const float* row, int v, int V, bool vec, float out[4]) {
    if (vec && v + 3 < V) {
        f32x4 t = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + v));
        out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
    } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = (v + e < V) ? row[v + e] : -INFINITY;
    }
}

__device__ inline float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ inline float fast_log2(float x) { return __builtin_amdgcn_logf(x); }

// ---- wave reductions on the data-parallel-primitive lanes (no LDS traffic) ----------------------
// xor 1, xor 2, mirror within 8, mirror within 16: every lane of a row of 16 then holds the row's
// result; two row broadcasts carry it to the last row, whose lane 63 is read out.  Fixed shape, so a
// sum has fixed rounding.  Results are wave-uniform.
template <int CTRL, int ROW_MASK, bool BOUND>
__device__ inline float dpp_move(float old, float v) {
    return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(old), __float_as_int(v), CTRL, ROW_MASK, 0xf, BOUND));
}
__device__ inline float wave_sum_dpp(float v) {
    v = v + dpp_move<0xB1, 0xf, true>(0.f, v);    // quad_perm [1,0,3,2]
    v = v + dpp_move<0x4E, 0xf, true>(0.f, v);    // quad_perm [2,3,0,1]
    v = v + dpp_move<0x141, 0xf, true>(0.f, v);   // row_half_mirror
    v = v + dpp_move<0x140, 0xf, true>(0.f, v);   // row_mirror
    v = v + dpp_move<0x142, 0xa, false>(0.f, v);  // row_bcast15 into rows 1 and 3
    v = v + dpp_move<0x143, 0xc, false>(0.f, v);  // row_bcast31 into rows 2 and 3
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// the same shape for the maximum; written as instructions because the generic maximum would re-quiet
// both operands at every step (s_nop 1: a lane-crossing read must not follow the write of its source directly)
__device__ inline float wave_max_dpp(float v) {
    asm volatile(
        "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_half_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_mirror row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
        "s_nop 1\n\tv_max_f32_dpp %0, %0, %0 row_bcast:31 row_mask:0xc bank_mask:0xf\n\t"
        "s_nop 1"
        : "+v"(v));
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

struct RowStats { float Mp, Sp, Mq, Sq; };  // base 2: p_v = 2^(z_v c2 - Mp) / Sp

struct AcceptShape {
    const float* lp;  // [B][k+1][V]
    const float* lq;  // [B][k][V]
    const int32_t* tokens;  // [B][k]
    int k, V, nch;          // nch: chunks of kAcceptChunk entries (sampling and race kernels)
    float inv_temp;
    int nsl;                // result slots per row of the sweep kernel: one per wave, 4 per workgroup
    unsigned long long wait_ticks;  // bound of the wait for the other chunks of a row, in wall-clock ticks
};

struct AcceptWs {  // carved out of the caller's workspace
    RowPart* part;       // [B*k][nsl]
    float* jsd;          // [B*k][nsl]
    RowStats* stats;     // [B*k] row maxima and sums, written by the row's first chunk
    RacePart* race;      // [B][nch]
    KeyIdx* top;         // [B*(k+1)][nch] per-chunk maximum logit of the verifier rows (assisted and greedy stages)
    uint32_t* expired;   // [1] set when a bounded wait ran out
};

__device__ inline void st_agent64(void* p, float lo, float hi) {
    __hip_atomic_store(reinterpret_cast<unsigned long long*>(p),
                       (unsigned long long)__float_as_uint(lo) | ((unsigned long long)__float_as_uint(hi) << 32),
                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline unsigned long long ld_agent64(const void* p) {
    return __hip_atomic_load(reinterpret_cast<const unsigned long long*>(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Row maxima and sums S = sum_c s_c 2^(m_c - M) of both rows from the per-wave partials.  Thread t folds
// slots t, t + 256, ... in increasing order, each wave reduces its share with the fixed tree, and the four
// wave results are combined in wave order: every workgroup that evaluates a row gets the same bits.
// WAIT: the partials come from workgroups of the running kernel; each thread polls its slot until both
// halves are written, or the clock runs out: then false is returned in every thread.  One barrier.
template <bool WAIT, int T>
__device__ inline bool row_stats(const RowPart* parts, int nsl, unsigned long long wait_ticks, float4* lds, RowStats& r) {
    constexpr int NW = T / 64;
    float mp = -INFINITY, mq = -INFINITY, sp = 0.f, sq = 0.f;
    const int wave = threadIdx.x >> 6;
    if (WAIT) {  // nsl <= 256: at most one slot per thread
        RowPart me{-INFINITY, 0.f, -INFINITY, 0.f};
        if ((int)threadIdx.x < nsl) {
            const RowPart* src = parts + threadIdx.x;
            const unsigned long long t0 = wall_clock64();
            for (;;) {
                const unsigned long long u0 = ld_agent64(&src->mp), u1 = ld_agent64(&src->mq);
                if ((uint32_t)u0 != kUnwritten && (uint32_t)u1 != kUnwritten) {
                    me = RowPart{__uint_as_float((uint32_t)u0), __uint_as_float((uint32_t)(u0 >> 32)),
                                 __uint_as_float((uint32_t)u1), __uint_as_float((uint32_t)(u1 >> 32))};
                    break;
                }
                if (wall_clock64() - t0 >= wait_ticks) { me.mp = INFINITY; break; }  // +inf marks the expiry
                __builtin_amdgcn_s_sleep(32);
            }
        }
        if (wave * 64 < nsl) {
            mp = wave_max_dpp(me.mp);
            mq = wave_max_dpp(me.mq);
            sp = wave_sum_dpp(me.sp * fast_exp2(me.mp - mp));
            sq = wave_sum_dpp(me.sq * fast_exp2(me.mq - mq));
        }
    } else {
        for (int c = threadIdx.x; c < nsl; c += T) { mp = fmaxf(mp, parts[c].mp); mq = fmaxf(mq, parts[c].mq); }
        mp = wave_max_dpp(mp);
        mq = wave_max_dpp(mq);
        for (int c = threadIdx.x; c < nsl; c += T) {
            const RowPart t = parts[c];
            sp = sp + t.sp * fast_exp2(t.mp - mp);
            sq = sq + t.sq * fast_exp2(t.mq - mq);
        }
        sp = wave_sum_dpp(sp);
        sq = wave_sum_dpp(sq);
    }
    if ((threadIdx.x & 63) == 0) lds[wave] = make_float4(mp, sp, mq, sq);
    __syncthreads();
    r.Mp = -INFINITY; r.Mq = -INFINITY;
#pragma unroll
    for (int i = 0; i < NW; ++i) { r.Mp = fmaxf(r.Mp, lds[i].x); r.Mq = fmaxf(r.Mq, lds[i].z); }
    if (WAIT && r.Mp == INFINITY) return false;
    r.Sp = 0.f; r.Sq = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) {
        const float4 wv = lds[i];
        r.Sp = r.Sp + wv.y * fast_exp2(wv.x - r.Mp);
        r.Sq = r.Sq + wv.w * fast_exp2(wv.z - r.Mq);
    }
    return true;
}

__global__ void accept_clear(AcceptWs w, size_t n_parts) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n_parts) w.part[i] = RowPart{__uint_as_float(kUnwritten), 0.f, __uint_as_float(kUnwritten), 0.f};
    if (i == 0) *w.expired = 0u;
}

enum { SWEEP_ONE_LAUNCH = 0, SWEEP_PARTIALS = 1, SWEEP_DIVERGENCE = 2 };

// ---- the sweep, in pieces -----------------------------------------------------------------------------------
// A work item is one chunk of kSweepChunk entries of one judged position: item = (trial * k + position) * chunks
// + chunk, so the chunks of a row are neighbours in item order.  kSweepQuads quads of 4 logits per thread and row
// stay in registers between the two halves (40 registers); the exponentials of the first half are evaluated
// again in the second.  Every wave keeps its own maximum, sum and divergence partial: the only barrier is the
// one inside row_stats.
struct SweepItem {
    const float *prow, *qrow;
    int pair, ch;
};
__device__ inline SweepItem sweep_item(const AcceptShape& s, int item) {
    const int nsw = s.nsl / kSweepWaves;
    SweepItem it;
    it.ch = item % nsw;
    it.pair = item / nsw;  // trial * k + position
    const int b = it.pair / s.k, i = it.pair - b * s.k;
    it.prow = s.lp + ((size_t)b * (s.k + 1) + i) * s.V;
    it.qrow = s.lq + (size_t)it.pair * s.V;
    return it;
}

// Issues the loads of an item and nothing else: no branch, so that the compiler can keep them in flight across
// the arithmetic of another item.  Needs V % 4 == 0 and V >= 4; quads beyond the row are read from the row's last
// quad instead and masked when they are first used.
__device__ inline void sweep_load(const AcceptShape& s, const SweepItem& it, float a[kSweepQuads][4], float c[kSweepQuads][4]) {
#pragma unroll
    for (int j = 0; j < kSweepQuads; ++j) {
        const int v = min(it.ch * kSweepChunk + 4 * ((int)threadIdx.x + kAccThreads * j), s.V - 4);
        const f32x4 ta = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(it.prow + v));
        const f32x4 tc = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(it.qrow + v));
        a[j][0] = ta.x; a[j][1] = ta.y; a[j][2] = ta.z; a[j][3] = ta.w;
        c[j][0] = tc.x; c[j][1] = tc.y; c[j][2] = tc.z; c[j][3] = tc.w;
    }
}

// the same for any vocabulary size and alignment (checked, element-wise where a quad is not whole)
__device__ inline void sweep_load_any(const AcceptShape& s, const SweepItem& it, float a[kSweepQuads][4], float c[kSweepQuads][4]) {
    const bool vec = (s.V & 3) == 0;
#pragma unroll
    for (int j = 0; j < kSweepQuads; ++j) {
        const int v = it.ch * kSweepChunk + 4 * (threadIdx.x + kAccThreads * j);
        load4_stream(it.prow, v, s.V, vec, a[j]);
        load4_stream(it.qrow, v, s.V, vec, c[j]);
    }
}

// first half: per-wave base-2 maximum and sum of both rows; PUBLISH: written where the row's other chunks poll
template <bool PUBLISH>
__device__ inline void sweep_first(const AcceptShape& s, const AcceptWs& w, const SweepItem& it,
                                   float a[kSweepQuads][4], float c[kSweepQuads][4]) {
    const float c2 = s.inv_temp * kLog2e;  // logit -> base-2 exponent
    if ((it.ch + 1) * kSweepChunk > s.V) {  // the row ends inside this chunk: entries beyond it carry no probability
#pragma unroll
        for (int j = 0; j < kSweepQuads; ++j)
            if (it.ch * kSweepChunk + 4 * ((int)threadIdx.x + kAccThreads * j) >= s.V) {
#pragma unroll
                for (int e = 0; e < 4; ++e) { a[j][e] = -INFINITY; c[j][e] = -INFINITY; }
            }
    }
    float ma = -INFINITY, mc = -INFINITY;
#pragma unroll
    for (int j = 0; j < kSweepQuads; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) { ma = fmaxf(ma, a[j][e]); mc = fmaxf(mc, c[j][e]); }
    // masked entries only: a finite floor, so that -inf logits give 2^(-inf) = 0 and not NaN
    const float mp = fmaxf(wave_max_dpp(ma) * c2, -kBig), mq = fmaxf(wave_max_dpp(mc) * c2, -kBig);
    float sp = 0.f, sq = 0.f;
#pragma unroll
    for (int j = 0; j < kSweepQuads; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            sp = sp + fast_exp2(fmaf(a[j][e], c2, -mp));
            sq = sq + fast_exp2(fmaf(c[j][e], c2, -mq));
        }
    sp = wave_sum_dpp(sp);
    sq = wave_sum_dpp(sq);
    if (PUBLISH && (threadIdx.x & 63) == 0) {
        RowPart* slot = w.part + (size_t)it.pair * s.nsl + it.ch * kSweepWaves + (threadIdx.x >> 6);
        st_agent64(&slot->mp, mp, sp);
        st_agent64(&slot->mq, mq, sq);
    }
}

// second half: row statistics from everybody's partials (WAIT: polled), then the divergence partial of the chunk.
// Returns false in every thread when the bounded wait expired.
template <bool WAIT>
__device__ inline bool sweep_second(const AcceptShape& s, const AcceptWs& w, const SweepItem& it,
                                    const float a[kSweepQuads][4], const float c[kSweepQuads][4], float4* lds) {
    const float c2 = s.inv_temp * kLog2e;
    RowStats R;
    if (!row_stats<WAIT, kAccThreads>(w.part + (size_t)it.pair * s.nsl, s.nsl, s.wait_ticks, lds, R)) {
        // the decision kernel reports the expiry; nothing below is waited for by anyone
        if (threadIdx.x == 0) __hip_atomic_store(w.expired, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return false;
    }
    // With xp = log2 p_v = a_v c2 - lp and xq = log2 q_v = c_v c2 - lq, call the larger probability B = 2^max(xp, xq) and
    // the smaller one S = B e with e = 2^-A, A = |xq - xp|.  Then m = (B + S) / 2 and
    //   log2(B / m) = 1 - log2(1 + e) =: u,    log2(S / m) = u - A,
    // so the entry contributes B u + S (u - A) whichever of p, q is the larger: three transcendentals (2^max, 2^-A,
    // log2(1 + e)), no selects.  Equal rows give A = 0, e = 1, u = 0 exactly, hence a divergence of exactly 0; there is no
    // cancellation anywhere.  Masked entries: A is clamped to a finite value, so they contribute B * 1 + 0 * finite (one
    // row has no mass there) or 0 * finite (neither has).
    const float lSp = log2f(R.Sp), lSq = log2f(R.Sq);
    const float lp = R.Mp + lSp, lq = R.Mq + lSq;   // base-2 log-sum-exp of the rows
    float acc = 0.f;
#pragma unroll
    for (int j = 0; j < kSweepQuads; ++j)
#pragma unroll
        for (int e4 = 0; e4 < 4; ++e4) {
            const float xp = fmaf(a[j][e4], c2, -lp), xq = fmaf(c[j][e4], c2, -lq);
            const float big = fast_exp2(fmaxf(fmaxf(xp, xq), -kBig));
            const float A = fabsf(__builtin_amdgcn_fmed3f(xq - xp, -kBig, kBig));   // inf - inf (both masked) clamps to a finite value too
            const float e = fast_exp2(-A);
            const float u = 1.f - fast_log2(1.f + e);
            acc = fmaf(big, u, acc);
            acc = fmaf(big * e, u - A, acc);
        }
    acc = wave_sum_dpp(acc);
    if ((threadIdx.x & 63) == 0)
        w.jsd[(size_t)it.pair * s.nsl + it.ch * kSweepWaves + (threadIdx.x >> 6)] = (0.5f * kLn2) * acc;
    if (it.ch == 0 && threadIdx.x == 0) w.stats[it.pair] = R;
    return true;
}

// One workgroup per item.  SWEEP_ONE_LAUNCH: publish, wait for the row, finish.  Two launches: SWEEP_PARTIALS stops
// after the first half, SWEEP_DIVERGENCE repeats the first half without publishing and reads the finished partials.
// The workgroups of a row are neighbours in launch order and consecutive ids go round the 8 accelerator dies, so
// the chunks a workgroup waits for are resident with it.
template <int MODE, bool VEC>
__global__ __launch_bounds__(kAccThreads, (MODE == SWEEP_ONE_LAUNCH && VEC) ? 8 : 6) void accept_sweep(AcceptShape s, AcceptWs w) {
    __shared__ float4 lds[kSweepWaves];
    const SweepItem it = sweep_item(s, blockIdx.x);
    float a[kSweepQuads][4], c[kSweepQuads][4];
    if (VEC) sweep_load(s, it, a, c);
    else sweep_load_any(s, it, a, c);
    sweep_first<MODE != SWEEP_DIVERGENCE>(s, w, it, a, c);
    if (MODE == SWEEP_PARTIALS) return;
    sweep_second<MODE == SWEEP_ONE_LAUNCH>(s, w, it, a, c, lds);
}

// One workgroup of 16 waves per trial: wave r sums the divergence partials of positions r, r + 16 (lane c
// takes chunks c, c + 64, ... in increasing order, then a fixed tree), thread i tosses the coin of position i.
__global__ __launch_bounds__(1024) void accept_decide(AcceptShape s, AcceptWs w, float T, uint64_t seed,
                                                      uint32_t position0, uint32_t stage, AcceptOut* out,
                                                      float* div_out, int32_t* n_out, int32_t* tok_out) {
    __shared__ float s_div[PSD_MAX_WIDTH];
    __shared__ int s_pass[PSD_MAX_WIDTH];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = wave; i < s.k; i += 16) {
        const float* pr = w.jsd + ((size_t)b * s.k + i) * s.nsl;
        float d = 0.f;
        for (int c = lane; c < s.nsl; c += 64) d = d + pr[c];
        d = wave_sum_dpp(d);
        if (lane == 0) s_div[i] = d;
    }
    __syncthreads();
    const int i = threadIdx.x;
    if (i < s.k) {
        const float d = s_div[i];
        if (div_out) div_out[(size_t)b * s.k + i] = d;
        int pass = 2;  // 2: within the threshold, 1: the coin accepted, 0: rejected
        if (!(d <= T)) {
            const uint64_t sd = seed + (uint64_t)b;
            U4 r = philox4x32_10(U4{0u, position0 + (uint32_t)i, DRAW_COIN, stage}, (uint32_t)sd, (uint32_t)(sd >> 32));
            // The coin compares p(x) and q(x): accurate exponentials of the natural-log probabilities.
            // An id outside the vocabulary has probability 0 under the verifier -> rejected.
            const size_t pair = (size_t)b * s.k + i;
            const int x = s.tokens[pair];
            TokProb tp{0.f, 1.f};
            if (x >= 0 && x < s.V) {
                const RowStats R = w.stats[pair];
                const float lse_p = (R.Mp + log2f(R.Sp)) * kLn2, lse_q = (R.Mq + log2f(R.Sq)) * kLn2;
                const float zp = s.lp[((size_t)b * (s.k + 1) + i) * s.V + x], zq = s.lq[pair * s.V + x];
                tp = TokProb{expf(fmaxf(zp, -kBig) * s.inv_temp - lse_p), expf(fmaxf(zq, -kBig) * s.inv_temp - lse_q)};
            }
            pass = (u01(r.x) * tp.qx < tp.px) ? 1 : 0;  // u < p(x)/q(x)
        }
        s_pass[i] = pass;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int n = 0, fuzzy = 0;
        for (; n < s.k && s_pass[n]; ++n) fuzzy += s_pass[n] == 2;
        AcceptOut o;
        o.n_accepted = *w.expired ? -1 : n;  // -1: the sweep's bounded wait expired
        o.n_fuzzy = fuzzy;
        o.pad = 0;
        o.next_token = -1;
        out[b] = o;
        if (n_out) { n_out[b] = o.n_accepted; tok_out[b] = -1; }
    }
}

// ---- assisted stage: strict match against the verifier's top prediction ---------------------------------
__global__ __launch_bounds__(kAccThreads) void accept_top(AcceptShape s, AcceptWs w) {
    __shared__ KeyIdx smk[4];
    const int ch = blockIdx.x, i = blockIdx.y, b = blockIdx.z;
    const float* prow = s.lp + ((size_t)b * (s.k + 1) + i) * s.V;
    const bool vec = (s.V & 3) == 0;
    KeyIdx best{-INFINITY, 0x7fffffff};
#pragma unroll
    for (int j = 0; j < kQuadsPerThread; ++j) {
        const int v = ch * kAcceptChunk + 4 * (threadIdx.x + kAccThreads * j);
        if (v >= s.V) continue;
        float a[4];
        load4(prow, v, s.V, vec, a);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (v + e < s.V) best = better(best, KeyIdx{a[e], v + e});  // equal maxima: lowest index
    }
    best = block_best<4>(best, smk);
    if (threadIdx.x == 0) w.top[((size_t)b * (s.k + 1) + i) * s.nch + ch] = best;
}

// one workgroup of 16 waves per trial: wave r reduces the chunk maxima of rows r, r + 16, ...
// greedy: rows 0 .. k are reduced and the replacement / bonus token is the top prediction of row n itself
// (temperature -> 0 limit, Section 3.1); otherwise rows 0 .. k - 1 and the token is drawn by the race kernels.
__global__ __launch_bounds__(1024) void accept_decide_assisted(AcceptShape s, AcceptWs w, int greedy, int take_bonus,
                                                               AcceptOut* out, float* div_out, int32_t* n_out,
                                                               int32_t* tok_out) {
    __shared__ int s_top[PSD_MAX_WIDTH + 1];
    const int b = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int rows = greedy ? s.k + 1 : s.k;
    for (int i = wave; i < rows; i += 16) {
        const KeyIdx* pr = w.top + ((size_t)b * (s.k + 1) + i) * s.nch;
        KeyIdx best{-INFINITY, 0x7fffffff};
        for (int c = lane; c < s.nch; c += 64) best = better(best, pr[c]);
        best = wave_best(best);
        if (lane == 0) {
            s_top[i] = best.idx;
            if (div_out && i < s.k) div_out[(size_t)b * s.k + i] = -1.f;  // no divergence is evaluated in this stage
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int n = 0;
        while (n < s.k && s.tokens[(size_t)b * s.k + n] == s_top[n]) ++n;
        const int tok = (greedy && (n < s.k || take_bonus)) ? s_top[n] : -1;
        out[b] = AcceptOut{n, tok, 0, 0};
        if (n_out) { n_out[b] = n; tok_out[b] = tok; }
    }
}

// Replacement draw, one row per trial.  First rejected position n < k: race r_v / E_v over the residual
// r = max(0, p - q) (and p_v / E_v beside it, used when the residual has no mass at all).  n == k and a
// bonus token is wanted: race over the verifier's last row in log form, z_v / temperature - ln E_v, which
// needs no normalisation.  E_v = -ln u_v.  Assisted stage: the draw at a rejection is from the verifier's
// row itself, in the same log form but with the replacement stream's random numbers.
__global__ __launch_bounds__(kAccThreads) void accept_race(AcceptShape s, AcceptWs w, const AcceptOut* out,
                                                           uint64_t seed, uint32_t position0, uint32_t stage,
                                                           int take_bonus, int assisted) {
    __shared__ KeyIdx smk[4];
    const int ch = blockIdx.x, b = blockIdx.y;
    const int n = out[b].n_accepted;
    if (n < 0 || (n == s.k && !take_bonus)) return;
    const uint64_t sd = seed + (uint64_t)b;
    const uint32_t pos = position0 + (uint32_t)n;
    const float* prow = s.lp + ((size_t)b * (s.k + 1) + n) * s.V;
    const bool vec = (s.V & 3) == 0;
    KeyIdx best{-INFINITY, 0x7fffffff}, best_fb{-1.f, 0x7fffffff};
    if (n == s.k || assisted) {
        const uint32_t purpose = n == s.k ? (uint32_t)DRAW_SAMPLE : (uint32_t)DRAW_RESAMPLE, stg = n == s.k ? 0u : stage;
#pragma unroll
        for (int j = 0; j < kQuadsPerThread; ++j) {
            const int v = ch * kAcceptChunk + 4 * (threadIdx.x + kAccThreads * j);
            if (v >= s.V) continue;
            float a[4], u[4];
            load4(prow, v, s.V, vec, a);
            draw4(sd, (uint32_t)(v >> 2), pos, purpose, stg, u);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (v + e >= s.V) continue;
                const float E = -kLn2 * fast_log2(u[e]);
                best = better(best, KeyIdx{fmaf(a[e], s.inv_temp, -kLn2 * fast_log2(E)), v + e});
            }
        }
    } else {
        const int pair = b * s.k + n;
        const float* qrow = s.lq + (size_t)pair * s.V;
        const RowStats R = w.stats[pair];
        const float c2 = s.inv_temp * kLog2e, ip = 1.f / R.Sp, iq = 1.f / R.Sq;
        best.key = -1.f;  // residual keys are positive
#pragma unroll
        for (int j = 0; j < kQuadsPerThread; ++j) {
            const int v = ch * kAcceptChunk + 4 * (threadIdx.x + kAccThreads * j);
            if (v >= s.V) continue;
            float a[4], c[4], u[4];
            load4(prow, v, s.V, vec, a);
            load4(qrow, v, s.V, vec, c);
            draw4(sd, (uint32_t)(v >> 2), pos, DRAW_RESAMPLE, stage, u);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                if (v + e >= s.V) continue;
                const float p = fast_exp2(fmaf(a[e], c2, -R.Mp)) * ip;  // -inf logits: 2^(-inf) = 0
                const float q = fast_exp2(fmaf(c[e], c2, -R.Mq)) * iq;
                const float iE = __builtin_amdgcn_rcpf(-kLn2 * fast_log2(u[e]));
                const float r = p - q;
                if (r > 0.f) best = better(best, KeyIdx{r * iE, v + e});
                if (p > 0.f) best_fb = better(best_fb, KeyIdx{p * iE, v + e});
            }
        }
    }
    best = block_best<4>(best, smk);
    best_fb = block_best<4>(best_fb, smk);
    if (threadIdx.x == 0) w.race[(size_t)b * s.nch + ch] = RacePart{best.key, best.idx, best_fb.key, best_fb.idx};
}

__global__ __launch_bounds__(kAccThreads) void accept_pick(AcceptShape s, AcceptWs w, int take_bonus, int assisted,
                                                           AcceptOut* out, int32_t* tok_out) {
    __shared__ KeyIdx smk[4];
    const int b = blockIdx.x;
    const int n = out[b].n_accepted;
    if (n < 0 || (n == s.k && !take_bonus)) return;  // next_token stays -1
    const bool bonus_row = n == s.k || assisted;  // keys in log form: any sign, and never without mass
    KeyIdx best{bonus_row ? -INFINITY : -1.f, 0x7fffffff}, fb{-1.f, 0x7fffffff};
    for (int c = threadIdx.x; c < s.nch; c += kAccThreads) {
        const RacePart r = w.race[(size_t)b * s.nch + c];
        best = better(best, KeyIdx{r.key, r.idx});
        fb = better(fb, KeyIdx{r.key_fb, r.idx_fb});
    }
    best = block_best<4>(best, smk);
    fb = block_best<4>(fb, smk);
    // no residual mass at all (cannot happen in exact arithmetic): draw from p instead
    if (!bonus_row && !(best.key > 0.f)) best = fb;
    if (threadIdx.x == 0) {
        const int tok = best.idx == 0x7fffffff ? -1 : best.idx;
        out[b].next_token = tok;
        if (tok_out) tok_out[b] = tok;
    }
}

static inline size_t align16(size_t n) { return (n + 15) & ~(size_t)15; }

static int sweep_chunks(int vocab) { return (vocab + kSweepChunk - 1) / kSweepChunk; }

static size_t carve(AcceptWs* w, void* base, int n_trials, int k, int vocab) {
    const size_t pairs = (size_t)n_trials * k;
    const int nsw_max = kSweepWaves * sweep_chunks(vocab), nch = accept_chunks(vocab);
    size_t off = 0;
    auto take = [&](size_t bytes) { char* p = (char*)base + off; off += align16(bytes); return (void*)p; };
    RowPart* part = (RowPart*)take(pairs * nsw_max * sizeof(RowPart));
    float* jsd = (float*)take(pairs * nsw_max * sizeof(float));
    RowStats* st = (RowStats*)take(pairs * sizeof(RowStats));
    RacePart* race = (RacePart*)take((size_t)n_trials * nch * sizeof(RacePart));
    KeyIdx* top = (KeyIdx*)take((pairs + n_trials) * nch * sizeof(KeyIdx));
    uint32_t* expired = (uint32_t*)take(sizeof(uint32_t));
    if (w) *w = AcceptWs{part, jsd, st, race, top, expired};
    return off;
}

size_t accept_workspace_bytes(int n_trials, int k, int vocab) { return carve(nullptr, nullptr, n_trials, k, vocab); }

int accept_launch(const float* logits_p, const float* logits_q, const int32_t* tokens, int n_trials, int k,
                  int vocab, float T, float temperature, uint64_t seed, uint32_t position0, uint32_t stage,
                  int take_bonus, AcceptOut* out, float* div_out, void* workspace, size_t workspace_bytes,
                  hipStream_t stream, char* errbuf, int32_t* n_accepted_out, int32_t* next_token_out, int assisted) {
    if (!logits_p || (k > 0 && ((!logits_q && !assisted) || !tokens)) || !out || !workspace)
        PSD_FAIL(PSD_EINVAL, errbuf, "accept: null pointer");
    if (k < 0 || k > PSD_MAX_WIDTH || vocab < 1 || n_trials < 1 || n_trials > 65535)
        PSD_FAIL(PSD_EINVAL, errbuf, "accept: k=%d vocab=%d n_trials=%d out of range", k, vocab, n_trials);
    if (!(T >= 0.f) || !(temperature > 0.f)) PSD_FAIL(PSD_EINVAL, errbuf, "accept: T=%g temperature=%g", T, temperature);
    if (workspace_bytes < accept_workspace_bytes(n_trials, k, vocab))
        PSD_FAIL(PSD_ENOMEM, errbuf, "accept: workspace %zu < %zu bytes", workspace_bytes,
                 accept_workspace_bytes(n_trials, k, vocab));
    // rows are read 16 bytes at a time only when every row starts on a 16-byte boundary (vocabulary a multiple of 4)
    const uintptr_t row_mask = (vocab & 3) == 0 ? 15 : 3;
    if (((uintptr_t)workspace & 15) || ((uintptr_t)logits_p & row_mask) || (logits_q && ((uintptr_t)logits_q & row_mask)))
        PSD_FAIL(PSD_EINVAL, errbuf, "accept: workspace must be 16-byte aligned, logits %d-byte aligned", (int)row_mask + 1);
    const int nch = accept_chunks(vocab), nsw = sweep_chunks(vocab);
    const int pairs = n_trials * k;
    if ((long long)pairs * nsw > 0x7fffffffLL) PSD_FAIL(PSD_EINVAL, errbuf, "accept: n_trials * k * chunks overflows the grid");
    AcceptWs w;
    carve(&w, workspace, n_trials, k, vocab);
    AcceptShape s{logits_p, logits_q, tokens, k, vocab, nch, 1.0f / temperature, kSweepWaves * nsw, g_wait_ticks.load()};
    const size_t n_parts = (size_t)pairs * nsw * kSweepWaves;
    if (assisted) {   // 1: assisted stage, 2: greedy stage
        const int greedy = assisted == 2, rows = greedy ? k + 1 : k;
        if (rows > 0) accept_top<<<dim3(nch, rows, n_trials), kAccThreads, 0, stream>>>(s, w);
        accept_decide_assisted<<<n_trials, 1024, 0, stream>>>(s, w, greedy, take_bonus, out, div_out, n_accepted_out,
                                                               next_token_out);
        if (!greedy) {
            accept_race<<<dim3(nch, n_trials), kAccThreads, 0, stream>>>(s, w, out, seed, position0, stage, take_bonus, 1);
            accept_pick<<<n_trials, kAccThreads, 0, stream>>>(s, w, take_bonus, 1, out, next_token_out);
        }
        PSD_HIP(hipGetLastError(), errbuf);
        return PSD_OK;
    }
    accept_clear<<<(unsigned)((n_parts + 256) / 256), 256, 0, stream>>>(w, n_parts);
    if (pairs > 0) {
        const int n_items = pairs * nsw;
        const bool vec = (vocab & 3) == 0;  // rows are then 16-byte aligned and hold whole quads
        const bool one_launch = g_accept_path.load() != 1 && kSweepWaves * nsw <= kSweepMaxSlots;
        if (one_launch) {
            if (vec) accept_sweep<SWEEP_ONE_LAUNCH, true><<<n_items, kAccThreads, 0, stream>>>(s, w);
            else accept_sweep<SWEEP_ONE_LAUNCH, false><<<n_items, kAccThreads, 0, stream>>>(s, w);
        } else if (vec) {
            accept_sweep<SWEEP_PARTIALS, true><<<n_items, kAccThreads, 0, stream>>>(s, w);
            accept_sweep<SWEEP_DIVERGENCE, true><<<n_items, kAccThreads, 0, stream>>>(s, w);
        } else {
            accept_sweep<SWEEP_PARTIALS, false><<<n_items, kAccThreads, 0, stream>>>(s, w);
            accept_sweep<SWEEP_DIVERGENCE, false><<<n_items, kAccThreads, 0, stream>>>(s, w);
        }
    }
    accept_decide<<<n_trials, 1024, 0, stream>>>(s, w, T, seed, position0, stage, out, div_out, n_accepted_out,
                                                 next_token_out);
    accept_race<<<dim3(nch, n_trials), kAccThreads, 0, stream>>>(s, w, out, seed, position0, stage, take_bonus, 0);
    accept_pick<<<n_trials, kAccThreads, 0, stream>>>(s, w, take_bonus, 0, out, next_token_out);
    PSD_HIP(hipGetLastError(), errbuf);
    return PSD_OK;
}

// ---- fresh samples (draft proposals) ---------------------------------------------------------
// score_v = z_v / temperature - ln(-ln u_v); token = argmax (the exponential race in log form, so no
// normalisation pass is needed)
// greedy: the key is the logit itself (the top prediction; no random numbers)
__global__ __launch_bounds__(kAccThreads) void sample_partial(const float* logits, int V, int nch, float inv_temp,
                                                              uint64_t seed, uint32_t position0,
                                                              const SampleCtl* ctl, KeyIdx* parts, int greedy) {
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
        if (greedy) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (v + e < V) best = better(best, KeyIdx{a[e], v + e});
            continue;
        }
        draw4(seed, (uint32_t)(v >> 2), pos, DRAW_SAMPLE, 0u, u);
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (v + e < V) best = better(best, KeyIdx{a[e] * inv_temp - logf(-logf(u[e])), v + e});
    }
    best = block_best<4>(best, smk);
    if (threadIdx.x == 0) parts[(size_t)r * nch + ch] = best;
}

// one wave per row; the order of the comparisons is free: equal keys always resolve to the lowest index
__global__ __launch_bounds__(64) void sample_final(const KeyIdx* parts, int nch, int32_t* tokens_out) {
    const int r = blockIdx.x;
    KeyIdx best{-INFINITY, 0x7fffffff};
    for (int c = threadIdx.x; c < nch; c += kWave) best = better(best, parts[(size_t)r * nch + c]);
    best = wave_best(best);
    if (threadIdx.x == 0) tokens_out[r] = best.idx;
}

int sample_launch(const float* logits, int n_rows, int vocab, float temperature, uint64_t seed, uint32_t position0,
                  const SampleCtl* ctl, int32_t* tokens_out, void* partial, hipStream_t stream, char* errbuf, int greedy) {
    if (!logits || !partial) PSD_FAIL(PSD_EINVAL, errbuf, "sample: null pointer");
    if (n_rows < 1 || n_rows > 65535 || vocab < 1 || !(temperature > 0.f))
        PSD_FAIL(PSD_EINVAL, errbuf, "sample: n_rows=%d vocab=%d temperature=%g", n_rows, vocab, temperature);
    if ((uintptr_t)logits & ((vocab & 3) == 0 ? 15 : 3)) PSD_FAIL(PSD_EINVAL, errbuf, "sample: logits rows must be 16-byte aligned (4-byte when the vocabulary is not a multiple of 4)");
    const int nch = accept_chunks(vocab);
    sample_partial<<<dim3(nch, n_rows), kAccThreads, 0, stream>>>(logits, vocab, nch, 1.0f / temperature, seed,
                                                                   position0, ctl, (KeyIdx*)partial, greedy);
    if (tokens_out) sample_final<<<n_rows, 64, 0, stream>>>((const KeyIdx*)partial, nch, tokens_out);
    PSD_HIP(hipGetLastError(), errbuf);
    return PSD_OK;
}

// ---- per-step statistics of the behaviour analysis (Section 4): entropy and largest probability ----------
// H = ln Z - sum_v p_v z_v with z = logit / temperature, Z = sum_v e^(z_v); per chunk: maximum, S = sum 2^(y - m)
// and U = sum 2^(y - m) (y - m) in base 2 (y = z log2 e); the second kernel folds the chunks in order.
struct StatPart { float m, s, u, pad; };

__global__ __launch_bounds__(kAccThreads) void row_stats_partial(const float* logits, int V, int nch, float inv_temp,
                                                                 StatPart* parts) {
    __shared__ float4 lds[4];
    const int ch = blockIdx.x, r = blockIdx.y;
    const float* row = logits + (size_t)r * V;
    const bool vec = (V & 3) == 0;
    const float c2 = inv_temp * kLog2e;
    float a[kQuadsPerThread][4];
    float mx = -INFINITY;
#pragma unroll
    for (int j = 0; j < kQuadsPerThread; ++j) {
        load4(row, ch * kAcceptChunk + 4 * (threadIdx.x + kAccThreads * j), V, vec, a[j]);
#pragma unroll
        for (int e = 0; e < 4; ++e) mx = fmaxf(mx, a[j][e]);
    }
    const float mw = fmaxf(wave_max_dpp(mx) * c2, -kBig);
    float sw = 0.f, uw = 0.f;
#pragma unroll
    for (int j = 0; j < kQuadsPerThread; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float d = fmaxf(fmaf(a[j][e], c2, -mw), -kBig);  // masked entries: 2^d = 0 and 0 * finite = 0
            const float x = fast_exp2(d);
            sw = sw + x;
            uw = fmaf(x, d, uw);
        }
    sw = wave_sum_dpp(sw);
    uw = wave_sum_dpp(uw);
    if ((threadIdx.x & 63) == 0) lds[threadIdx.x >> 6] = make_float4(mw, sw, uw, 0.f);
    __syncthreads();
    if (threadIdx.x == 0) {  // the four waves in order, relative to the chunk maximum
        float M = fmaxf(fmaxf(lds[0].x, lds[1].x), fmaxf(lds[2].x, lds[3].x)), S = 0.f, U = 0.f;
        for (int i = 0; i < 4; ++i) {
            const float f = fast_exp2(lds[i].x - M);
            S = fmaf(lds[i].y, f, S);
            U = fmaf(fmaf(lds[i].y, lds[i].x - M, lds[i].z), f, U);  // sum x (d + (m_w - M))
        }
        parts[(size_t)r * nch + ch] = StatPart{M, S, U, 0.f};
    }
}

// one wave per row; acc (optional, device): {rows, sum of entropies, sum of largest probabilities} as doubles,
// updated by a single lane in row order
__global__ __launch_bounds__(64) void row_stats_final(const StatPart* parts, int nch, int n_rows, float* entropy,
                                                      float* max_prob, double* acc) {
    const int lane = threadIdx.x;
    double h_sum = 0.0, p_sum = 0.0;
    for (int r = 0; r < n_rows; ++r) {
        const StatPart* pr = parts + (size_t)r * nch;
        float m = -INFINITY;
        for (int c = lane; c < nch; c += 64) m = fmaxf(m, pr[c].m);
        const float M = wave_max_dpp(m);
        float s = 0.f, u = 0.f;
        for (int c = lane; c < nch; c += 64) {
            const StatPart t = pr[c];
            const float f = fast_exp2(t.m - M);
            s = fmaf(t.s, f, s);
            u = fmaf(fmaf(t.s, t.m - M, t.u), f, u);
        }
        const float S = wave_sum_dpp(s), U = wave_sum_dpp(u);
        // base 2: log2 Z = M + log2 S, sum_v p_v (y_v - M) = U / S  ->  H = ln 2 (log2 S - U / S);  p_max = 1 / S
        const float H = kLn2 * (log2f(S) - U / S), P = 1.f / S;
        if (lane == 0) {
            if (entropy) entropy[r] = H;
            if (max_prob) max_prob[r] = P;
        }
        h_sum += H;
        p_sum += P;
    }
    if (acc && lane == 0) { acc[0] += n_rows; acc[1] += h_sum; acc[2] += p_sum; }
}

size_t row_stats_workspace_bytes(int n_rows, int vocab) { return (size_t)n_rows * accept_chunks(vocab) * sizeof(StatPart); }

int row_stats_launch(const float* logits, int n_rows, int vocab, float temperature, float* entropy, float* max_prob,
                     double* acc, void* workspace, hipStream_t stream, char* errbuf) {
    if (!logits || !workspace) PSD_FAIL(PSD_EINVAL, errbuf, "row_stats: null pointer");
    if (n_rows < 1 || n_rows > 65535 || vocab < 1 || !(temperature > 0.f))
        PSD_FAIL(PSD_EINVAL, errbuf, "row_stats: n_rows=%d vocab=%d temperature=%g", n_rows, vocab, temperature);
    if ((uintptr_t)logits & ((vocab & 3) == 0 ? 15 : 3)) PSD_FAIL(PSD_EINVAL, errbuf, "row_stats: logits rows must be 16-byte aligned (4-byte when the vocabulary is not a multiple of 4)");
    const int nch = accept_chunks(vocab);
    row_stats_partial<<<dim3(nch, n_rows), kAccThreads, 0, stream>>>(logits, vocab, nch, 1.0f / temperature,
                                                                    (StatPart*)workspace);
    row_stats_final<<<1, 64, 0, stream>>>((const StatPart*)workspace, nch, n_rows, entropy, max_prob, acc);
    PSD_HIP(hipGetLastError(), errbuf);
    return PSD_OK;
}

}  // namespace psd

// ---- C ABI --------------------------------------------------------------------------------------
using namespace psd;

extern "C" int psd_set_accept_path(int32_t path) {
    if (path < 0 || path > 3) PSD_FAIL(PSD_EINVAL, tls_error(), "psd_set_accept_path: path=%d", path);
    g_accept_path.store(path == 3 ? 0 : path);
    g_wait_ticks.store(path == 3 ? 0ull : kWaitTicks);
    return PSD_OK;
}

extern "C" int psd_get_accept_path(void) { return g_accept_path.load(); }

extern "C" int64_t psd_get_accept_expiries(void) { return g_wait_expiries.load(); }

extern "C" size_t psd_accept_workspace_bytes(int32_t n_trials, int32_t k, int32_t vocab) {
    if (n_trials < 1 || k < 0 || vocab < 1) return 0;
    return accept_workspace_bytes(n_trials, k, vocab) + align16((size_t)n_trials * sizeof(AcceptOut));
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
                           take_bonus, out, div_out, workspace, inner, st, err, n_accepted, next_token);
    return rc;
}

// ---- ACCEPT for callers that cannot allocate ------------------------------------------------------
// The workspace of psd_accept_batch (per-chunk partials, race winners, per-trial results) lives in a file-scope
// device array instead of caller memory.  The array's name is only a host-side handle: the address kernels and
// copies use is asked for once per device (with that device current) and kept; every GPU has its own copy.
constexpr size_t kNoallocScratchBytes = PSD_ACCEPT_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char g_noalloc_scratch[kNoallocScratchBytes];

namespace {
constexpr int kNoallocMaxDevices = 64;
std::atomic<void*> g_noalloc_ptr[kNoallocMaxDevices];
std::mutex g_noalloc_mutex;

// device address of the scratch array on the current device (no allocation: the array is part of the code object)
int noalloc_scratch(void** out, char* err) {
    int dev = -1;
    PSD_HIP(hipGetDevice(&dev), err);
    if (dev < 0 || dev >= kNoallocMaxDevices) PSD_FAIL(PSD_EINVAL, err, "psd_accept_batch_noalloc: device ordinal %d", dev);
    void* p = g_noalloc_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_noalloc_mutex);
        p = g_noalloc_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            PSD_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(g_noalloc_scratch)), err);
            if (!p || ((uintptr_t)p & 255)) PSD_FAIL(PSD_EHIP, err, "psd_accept_batch_noalloc: bad scratch address %p", p);
            g_noalloc_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return PSD_OK;
}
}  // namespace

extern "C" size_t psd_accept_noalloc_capacity(void) { return kNoallocScratchBytes; }

extern "C" int psd_accept_noalloc_init(void) {
    void* p = nullptr;
    return noalloc_scratch(&p, tls_error());
}

extern "C" int psd_accept_batch_noalloc(const float* logits_p, const float* logits_q, const int32_t* tokens,
                                        int32_t n_trials, int32_t k, int32_t vocab, float T, float temperature,
                                        uint64_t seed, uint32_t position0, uint32_t stage, int32_t take_bonus,
                                        int32_t* n_accepted, int32_t* next_token, float* div_out, void* stream) {
    char* err = tls_error();
    if (!n_accepted || !next_token) PSD_FAIL(PSD_EINVAL, err, "psd_accept_batch_noalloc: null pointer");
    if (n_trials < 1 || k < 0 || vocab < 1) PSD_FAIL(PSD_EINVAL, err, "psd_accept_batch_noalloc: bad sizes");
    if (stage != 1 && stage != 2) PSD_FAIL(PSD_EINVAL, err, "psd_accept_batch_noalloc: stage must be 1 or 2");
    const size_t need = psd_accept_workspace_bytes(n_trials, k, vocab);
    if (need > kNoallocScratchBytes)
        PSD_FAIL(PSD_ENOMEM, err, "psd_accept_batch_noalloc: n_trials=%d k=%d vocab=%d need %zu bytes of scratch, the library holds %zu",
                 n_trials, k, vocab, need, kNoallocScratchBytes);
    void* scratch = nullptr;
    int rc = noalloc_scratch(&scratch, err);
    if (rc != PSD_OK) return rc;
    const size_t inner = accept_workspace_bytes(n_trials, k, vocab);
    AcceptOut* out = (AcceptOut*)((char*)scratch + inner);
    // every slot the kernels read is written earlier in the same launch sequence (accept_clear marks the per-chunk
    // partials unwritten and clears the expiry flag), so whatever the previous call left behind is never seen
    return accept_launch(logits_p, logits_q, tokens, n_trials, k, vocab, T, temperature, seed, position0, stage,
                         take_bonus, out, div_out, scratch, inner, (hipStream_t)stream, err, n_accepted, next_token);
}
