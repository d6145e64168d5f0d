// Device-side twin of the acceptance-microbenchmark input recipe in synth.c: target logits ~ N(0, sigma^2), qualifier =
// rho * target + sqrt(1 - rho^2) * N(0, sigma^2), draft likewise from the qualifier, every value a pure function of
// (seed, stream, index) through the same counter hash and Box-Muller transform in double precision.  It only
// manufactures INPUTS (no softmax, divergence, acceptance or sampling lives here); it exists because ten thousand
// trials per setting at vocabulary 128256 are terabytes of normals, which the host cannot produce in reasonable time.
// Values agree with the host generator to the last bits of the double-precision library functions, i.e. almost always
// bit for bit after rounding to float; nothing relies on exact equality.
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

__device__ inline uint64_t mix64(uint64_t z) {
    z += 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
__device__ inline uint64_t hash3(uint64_t seed, uint64_t stream, uint64_t idx) {
    return mix64(mix64(mix64(seed) ^ (stream * 0xD6E8FEB86659FD93ull)) ^ idx);
}
__device__ inline double u01(uint64_t h) { return ((double)(h >> 11) + 0.5) * (1.0 / 9007199254740992.0); }

// the two standard normals of pair `pair` of one stream
__device__ inline void normal_pair(uint64_t seed, uint64_t stream, uint64_t pair, double& n0, double& n1) {
    const double u1 = u01(hash3(seed, stream, 2 * pair)), u2 = u01(hash3(seed, stream, 2 * pair + 1));
    const double r = sqrt(-2.0 * log(u1)), a = 6.283185307179586476925286766559 * u2;
    double s, c;
    sincos(a, &s, &c);
    n0 = r * c;
    n1 = r * s;
}

// one thread per pair of consecutive elements of one trial's [(k + 1) * vocab] stack; qk and dk receive only the first
// n_lead elements of a trial (its first k rows), packed [trial][n_lead]
__global__ __launch_bounds__(256) void accept_logits_kernel(uint64_t seed, uint64_t trial0, size_t n_per_trial, size_t n_lead,
                                                            double rho, double sigma, float* t, float* q, float* d,
                                                            float* qk, float* dk) {
    const size_t pairs = (n_per_trial + 1) / 2;
    const size_t pair = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (pair >= pairs) return;
    const uint64_t trial = trial0 + blockIdx.y;
    const double c = sqrt(1.0 - rho * rho);
    double a0, a1, b0, b1, e0, e1;
    normal_pair(seed, trial * 4 + 0, pair, a0, a1);
    normal_pair(seed, trial * 4 + 1, pair, b0, b1);
    normal_pair(seed, trial * 4 + 2, pair, e0, e1);
    // each stack is rounded to float before the next one is derived from it, as on the host
    const float t0 = (float)(sigma * a0), t1 = (float)(sigma * a1);
    const float q0 = (float)(rho * (double)t0 + c * sigma * b0), q1 = (float)(rho * (double)t1 + c * sigma * b1);
    const float d0 = (float)(rho * (double)q0 + c * sigma * e0), d1 = (float)(rho * (double)q1 + c * sigma * e1);
    const size_t i = (size_t)blockIdx.y * n_per_trial + 2 * pair;
    const bool two = 2 * pair + 1 < n_per_trial;
    if (t) { t[i] = t0; if (two) t[i + 1] = t1; }
    if (q) { q[i] = q0; if (two) q[i + 1] = q1; }
    if (d) { d[i] = d0; if (two) d[i + 1] = d1; }
    const size_t e = 2 * pair, il = (size_t)blockIdx.y * n_lead + e;
    if (qk && e < n_lead) { qk[il] = q0; if (e + 1 < n_lead) qk[il + 1] = q1; }
    if (dk && e < n_lead) { dk[il] = d0; if (e + 1 < n_lead) dk[il + 1] = d1; }
}

}  // namespace

// Fills the device arrays t, q, d ([n_trials][(k + 1) * vocab] floats each) with the stacks of trials
// trial0 .. trial0 + n_trials - 1, and qk, dk ([n_trials][k * vocab]) with the first k rows of the qualifier and draft
// stacks, packed (the layout a proposer's rows have at the ACCEPT boundary).  Any pointer may be NULL.
// stream: a hipStream_t as void* (NULL: the default stream); only enqueues.
// Returns 0, -1 for bad arguments, -4 for a HIP error.
extern "C" int synth_dev_accept_logits(uint64_t seed, uint64_t trial0, int32_t n_trials, int32_t k, int32_t vocab, double rho,
                                       double sigma, float* t, float* q, float* d, float* qk, float* dk, void* stream) {
    if (n_trials < 1 || n_trials > 65535 || k < 0 || vocab < 1 || !(rho >= -1.0 && rho <= 1.0)) return -1;
    const size_t n = (size_t)(k + 1) * vocab, pairs = (n + 1) / 2;
    const size_t blocks = (pairs + 255) / 256;
    if (blocks > 0x7fffffffull) return -1;
    accept_logits_kernel<<<dim3((unsigned)blocks, n_trials), 256, 0, (hipStream_t)stream>>>(seed, trial0, n, (size_t)k * vocab, rho, sigma, t, q, d,
                                                                                          qk, dk);
    return hipGetLastError() == hipSuccess ? 0 : -4;
}
