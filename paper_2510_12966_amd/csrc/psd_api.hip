// Context-free parts of the C ABI: error strings, and the host-pointer variants of ACCEPT and SAMPLE
// (they stage through temporary device buffers; the hot path never uses them).
#include <string.h>

#include "psd_device.h"
#include "psd_host.h"

namespace psd {

char* tls_error() {
    static thread_local char buf[512];
    return buf;
}

void set_error(char* dst, const char* fmt, ...) {
    if (!dst) return;
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(dst, 512, fmt, ap);
    va_end(ap);
}

// the generator exactly as the sampling and ACCEPT kernels call it, one counter per thread
__global__ void philox_block(uint64_t seed, uint32_t c0, uint32_t n, uint32_t c1, uint32_t c2, uint32_t c3, uint32_t* out,
                             float* u_out) {
    const uint32_t i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const U4 r = philox4x32_10(U4{c0 + i, c1, c2, c3}, (uint32_t)seed, (uint32_t)(seed >> 32));
    if (out) reinterpret_cast<uint4*>(out)[i] = make_uint4(r.x, r.y, r.z, r.w);
    if (u_out) reinterpret_cast<float4*>(u_out)[i] = make_float4(u01(r.x), u01(r.y), u01(r.z), u01(r.w));
}

struct DevBuf {  // frees on scope exit
    void* p = nullptr;
    ~DevBuf() { if (p) (void)hipFree(p); }
};

}  // namespace psd

using namespace psd;

extern "C" const char* psd_strerror(int code) {
    switch (code) {
        case PSD_OK: return "ok";
        case PSD_EINVAL: return "invalid argument";
        case PSD_ESHAPE: return "shape or sequence length out of range";
        case PSD_ENOMEM: return "device pool or workspace too small";
        case PSD_EHIP: return "HIP runtime error";
        default: return "unknown error";
    }
}

// shared body of psd_accept and psd_accept_assisted: stages host inputs on the device when asked to
static int accept_once(const char* who, const float* logits_p, const float* logits_q, const int32_t* tokens, int32_t k,
                       int32_t vocab, float T, float temperature, uint64_t seed, uint32_t position0, uint32_t stage,
                       int32_t take_bonus, int32_t where, int32_t* n_accepted, int32_t* next_token, float* div_out,
                       int assisted) {
    char* err = tls_error();
    if (!logits_p || !n_accepted || !next_token || (k > 0 && ((!logits_q && !assisted) || !tokens)))
        PSD_FAIL(PSD_EINVAL, err, "%s: null pointer", who);
    if (k < 0 || k > PSD_MAX_WIDTH || vocab < 1) PSD_FAIL(PSD_EINVAL, err, "%s: k=%d vocab=%d", who, k, vocab);
    if (stage != 1 && stage != 2) PSD_FAIL(PSD_EINVAL, err, "%s: stage must be 1 or 2", who);
    if (where != 0 && where != 1) PSD_FAIL(PSD_EINVAL, err, "%s: where must be 0 or 1", who);
    if (!(T >= 0.f) || !(temperature > 0.f)) PSD_FAIL(PSD_EINVAL, err, "%s: T=%g temperature=%g", who, T, temperature);
    const size_t ws_bytes = psd_accept_workspace_bytes(1, k, vocab);
    const size_t np = (size_t)(k + 1) * vocab, nq = (size_t)k * vocab;
    DevBuf ws, dp, dq, dt, dres, ddiv;
    PSD_HIP(hipMalloc(&ws.p, ws_bytes), err);
    PSD_HIP(hipMalloc(&dres.p, 2 * sizeof(int32_t)), err);
    const float *p = logits_p, *q = logits_q;
    const int32_t* t = tokens;
    float* dv = div_out;
    if (where == 0) {
        PSD_HIP(hipMalloc(&dp.p, np * sizeof(float)), err);
        PSD_HIP(hipMemcpy(dp.p, logits_p, np * sizeof(float), hipMemcpyHostToDevice), err);
        p = (const float*)dp.p;
        if (k > 0) {
            if (!assisted) {
                PSD_HIP(hipMalloc(&dq.p, nq * sizeof(float)), err);
                PSD_HIP(hipMemcpy(dq.p, logits_q, nq * sizeof(float), hipMemcpyHostToDevice), err);
                q = (const float*)dq.p;
            }
            PSD_HIP(hipMalloc(&dt.p, k * sizeof(int32_t)), err);
            PSD_HIP(hipMemcpy(dt.p, tokens, k * sizeof(int32_t), hipMemcpyHostToDevice), err);
            t = (const int32_t*)dt.p;
            if (div_out) {
                PSD_HIP(hipMalloc(&ddiv.p, k * sizeof(float)), err);
                dv = (float*)ddiv.p;
            }
        } else {
            dv = nullptr;
        }
    }
    int32_t* res = (int32_t*)dres.p;
    const size_t inner = accept_workspace_bytes(1, k, vocab);
    int32_t h[2] = {-1, -1};
    for (int attempt = 0; attempt < 2 && h[0] < 0; ++attempt) {
        int rc = accept_launch(p, q, t, 1, k, vocab, T, temperature, seed, position0, stage, take_bonus,
                               (AcceptOut*)((char*)ws.p + inner), dv, ws.p, inner, nullptr, err, res, res + 1, assisted);
        if (rc != PSD_OK) return rc;
        PSD_HIP(hipDeviceSynchronize(), err);
        PSD_HIP(hipMemcpy(h, res, sizeof(h), hipMemcpyDeviceToHost), err);
        if (h[0] < 0) accept_wait_expired();  // not resident as a whole: two launches from now on, and once more
    }
    if (h[0] < 0) PSD_FAIL(PSD_EHIP, err, "%s: the kernels' bounded wait for each other expired", who);
    if (where == 0) {
        *n_accepted = h[0];
        *next_token = h[1];
        if (div_out && k > 0) PSD_HIP(hipMemcpy(div_out, dv, k * sizeof(float), hipMemcpyDeviceToHost), err);
    } else {
        PSD_HIP(hipMemcpy(n_accepted, res, sizeof(int32_t), hipMemcpyDeviceToDevice), err);
        PSD_HIP(hipMemcpy(next_token, res + 1, sizeof(int32_t), hipMemcpyDeviceToDevice), err);
    }
    return PSD_OK;
}

extern "C" int psd_accept(const float* logits_p, const float* logits_q, const int32_t* tokens, int32_t k,
                          int32_t vocab, float T, float temperature, uint64_t seed, uint32_t position0,
                          uint32_t stage, int32_t take_bonus, int32_t where, int32_t* n_accepted,
                          int32_t* next_token, float* div_out) {
    return accept_once("psd_accept", logits_p, logits_q, tokens, k, vocab, T, temperature, seed, position0, stage,
                       take_bonus, where, n_accepted, next_token, div_out, 0);
}

extern "C" int psd_accept_assisted(const float* logits_p, const int32_t* tokens, int32_t k, int32_t vocab,
                                   float temperature, uint64_t seed, uint32_t position0, uint32_t stage,
                                   int32_t take_bonus, int32_t where, int32_t* n_accepted, int32_t* next_token) {
    return accept_once("psd_accept_assisted", logits_p, nullptr, tokens, k, vocab, 0.f, temperature, seed, position0,
                       stage, take_bonus, where, n_accepted, next_token, nullptr, 1);
}

extern "C" int psd_row_stats(const float* logits, int32_t n_rows, int32_t vocab, float temperature, int32_t where,
                             float* entropy, float* max_prob) {
    char* err = tls_error();
    if (!logits || !entropy || !max_prob) PSD_FAIL(PSD_EINVAL, err, "psd_row_stats: null pointer");
    if (n_rows < 1 || n_rows > 65535 || vocab < 1 || !(temperature > 0.f))
        PSD_FAIL(PSD_EINVAL, err, "psd_row_stats: n_rows=%d vocab=%d temperature=%g", n_rows, vocab, temperature);
    if (where != 0 && where != 1) PSD_FAIL(PSD_EINVAL, err, "psd_row_stats: where must be 0 or 1");
    DevBuf dl, ws, dout;
    const size_t nb = (size_t)n_rows * vocab * sizeof(float);
    const float* l = logits;
    float *e = entropy, *m = max_prob;
    PSD_HIP(hipMalloc(&ws.p, row_stats_workspace_bytes(n_rows, vocab)), err);
    if (where == 0) {
        PSD_HIP(hipMalloc(&dl.p, nb), err);
        PSD_HIP(hipMemcpy(dl.p, logits, nb, hipMemcpyHostToDevice), err);
        PSD_HIP(hipMalloc(&dout.p, 2 * (size_t)n_rows * sizeof(float)), err);
        l = (const float*)dl.p;
        e = (float*)dout.p;
        m = e + n_rows;
    }
    int rc = row_stats_launch(l, n_rows, vocab, temperature, e, m, nullptr, ws.p, nullptr, err);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipDeviceSynchronize(), err);
    if (where == 0) {
        PSD_HIP(hipMemcpy(entropy, e, (size_t)n_rows * sizeof(float), hipMemcpyDeviceToHost), err);
        PSD_HIP(hipMemcpy(max_prob, m, (size_t)n_rows * sizeof(float), hipMemcpyDeviceToHost), err);
    }
    return PSD_OK;
}

extern "C" int psd_sample(const float* logits, int32_t n_rows, int32_t vocab, float temperature, uint64_t seed,
                          uint32_t position0, int32_t where, int32_t* tokens_out) {
    char* err = tls_error();
    if (!logits || !tokens_out) PSD_FAIL(PSD_EINVAL, err, "psd_sample: null pointer");
    if (n_rows < 1 || n_rows > 65535 || vocab < 1 || !(temperature > 0.f))
        PSD_FAIL(PSD_EINVAL, err, "psd_sample: n_rows=%d vocab=%d temperature=%g", n_rows, vocab, temperature);
    if (where != 0 && where != 1) PSD_FAIL(PSD_EINVAL, err, "psd_sample: where must be 0 or 1");
    DevBuf part, dl, dt;
    PSD_HIP(hipMalloc(&part.p, (size_t)n_rows * accept_chunks(vocab) * 8), err);
    const float* l = logits;
    int32_t* t = tokens_out;
    if (where == 0) {
        PSD_HIP(hipMalloc(&dl.p, (size_t)n_rows * vocab * sizeof(float)), err);
        PSD_HIP(hipMemcpy(dl.p, logits, (size_t)n_rows * vocab * sizeof(float), hipMemcpyHostToDevice), err);
        PSD_HIP(hipMalloc(&dt.p, n_rows * sizeof(int32_t)), err);
        l = (const float*)dl.p;
        t = (int32_t*)dt.p;
    }
    int rc = sample_launch(l, n_rows, vocab, temperature, seed, position0, nullptr, t, part.p, nullptr, err);
    if (rc != PSD_OK) return rc;
    PSD_HIP(hipDeviceSynchronize(), err);
    if (where == 0) PSD_HIP(hipMemcpy(tokens_out, t, n_rows * sizeof(int32_t), hipMemcpyDeviceToHost), err);
    return PSD_OK;
}

extern "C" int psd_philox_block(uint64_t seed, uint32_t c0, uint32_t n, uint32_t c1, uint32_t c2, uint32_t c3,
                                int32_t where, uint32_t* out, float* u_out) {
    char* err = tls_error();
    if (!out && !u_out) PSD_FAIL(PSD_EINVAL, err, "psd_philox_block: no output");
    if (n < 1 || n > (1u << 26)) PSD_FAIL(PSD_EINVAL, err, "psd_philox_block: n=%u outside [1, 2^26]", n);
    if (where != 0 && where != 1) PSD_FAIL(PSD_EINVAL, err, "psd_philox_block: where must be 0 or 1");
    DevBuf d_out, d_u;
    uint32_t* o = out;
    float* u = u_out;
    const size_t bytes = (size_t)n * 16;
    if (where == 0) {
        if (out) { PSD_HIP(hipMalloc(&d_out.p, bytes), err); o = (uint32_t*)d_out.p; }
        if (u_out) { PSD_HIP(hipMalloc(&d_u.p, bytes), err); u = (float*)d_u.p; }
    } else if (((uintptr_t)out | (uintptr_t)u_out) & 15) {
        PSD_FAIL(PSD_EINVAL, err, "psd_philox_block: device outputs must be 16-byte aligned");
    }
    philox_block<<<(n + 255) / 256, 256>>>(seed, c0, n, c1, c2, c3, o, u);
    PSD_HIP(hipGetLastError(), err);
    PSD_HIP(hipDeviceSynchronize(), err);
    if (where == 0) {
        if (out) PSD_HIP(hipMemcpy(out, o, bytes, hipMemcpyDeviceToHost), err);
        if (u_out) PSD_HIP(hipMemcpy(u_out, u, bytes, hipMemcpyDeviceToHost), err);
    }
    return PSD_OK;
}

extern "C" int psd_dev_alloc(size_t bytes, void** out) {
    char* err = tls_error();
    if (!out || bytes == 0) PSD_FAIL(PSD_EINVAL, err, "psd_dev_alloc: bad argument");
    void* p = nullptr;
    PSD_HIP(hipMalloc(&p, bytes), err);
    *out = p;
    return PSD_OK;
}

extern "C" int psd_dev_free(void* ptr) {
    char* err = tls_error();
    if (ptr) PSD_HIP(hipFree(ptr), err);
    return PSD_OK;
}

extern "C" int psd_dev_copy(void* dst, const void* src, size_t bytes, int32_t kind) {
    char* err = tls_error();
    if (!dst || !src || kind < 0 || kind > 2) PSD_FAIL(PSD_EINVAL, err, "psd_dev_copy: bad argument");
    const hipMemcpyKind kinds[3] = {hipMemcpyHostToDevice, hipMemcpyDeviceToHost, hipMemcpyDeviceToDevice};
    PSD_HIP(hipMemcpy(dst, src, bytes, kinds[kind]), err);
    return PSD_OK;
}

extern "C" int psd_dev_sync(void) {
    char* err = tls_error();
    PSD_HIP(hipDeviceSynchronize(), err);
    return PSD_OK;
}
