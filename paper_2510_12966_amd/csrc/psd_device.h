// Device-side helpers shared by the library's HIP translation units (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace psd {

constexpr int kWave = 64;

// ---- Philox4x32-10 (Salmon et al., SC'11) ---------------------------------
struct U4 { uint32_t x, y, z, w; };

__host__ __device__ inline U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        uint64_t p0 = (uint64_t)0xD2511F53u * c.x;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c.z;
        U4 n;
        n.x = (uint32_t)(p1 >> 32) ^ c.y ^ k0;
        n.y = (uint32_t)p1;
        n.z = (uint32_t)(p0 >> 32) ^ c.w ^ k1;
        n.w = (uint32_t)p0;
        c = n;
        k0 += 0x9E3779B9u;
        k1 += 0xBB67AE85u;
    }
    return c;
}

// u in (0,1): top 23 bits plus one half, exact in fp32
__host__ __device__ inline float u01(uint32_t x) { return ((float)(x >> 9) + 0.5f) * (1.0f / 8388608.0f); }

enum : uint32_t { DRAW_SAMPLE = 0, DRAW_COIN = 1, DRAW_RESAMPLE = 2 };

// the four uniforms of vocabulary entries 4*block .. 4*block+3
__device__ inline void draw4(uint64_t seed, uint32_t block, uint32_t position, uint32_t purpose, uint32_t stage,
                             float u[4]) {
    U4 r = philox4x32_10(U4{block, position, purpose, stage}, (uint32_t)seed, (uint32_t)(seed >> 32));
    u[0] = u01(r.x); u[1] = u01(r.y); u[2] = u01(r.z); u[3] = u01(r.w);
}

// ---- reductions: fixed tree, so results never depend on scheduling --------
__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ inline float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}

// (key, index) maximum; equal keys -> lowest index
struct KeyIdx { float key; int idx; };
__device__ inline KeyIdx better(KeyIdx a, KeyIdx b) {
    if (b.key > a.key || (b.key == a.key && b.idx < a.idx)) return b;
    return a;
}
__device__ inline KeyIdx wave_best(KeyIdx v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        KeyIdx t{__shfl_xor(v.key, o, kWave), __shfl_xor(v.idx, o, kWave)};
        v = better(v, t);
    }
    return v;
}

// block-wide versions for blockDim.x = 64 * NW (NW <= 16); `sm` needs NW slots; result valid in all threads
template <int NW>
__device__ inline float block_sum(float v, float* sm) {
    v = wave_sum(v);
    if constexpr (NW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = 0.f;
#pragma unroll
    for (int i = 0; i < NW; ++i) r += sm[i];
    return r;
}
template <int NW>
__device__ inline float block_max(float v, float* sm) {
    v = wave_max(v);
    if constexpr (NW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    float r = sm[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = fmaxf(r, sm[i]);
    return r;
}
template <int NW>
__device__ inline KeyIdx block_best(KeyIdx v, KeyIdx* sm) {
    v = wave_best(v);
    if constexpr (NW == 1) return v;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) sm[threadIdx.x >> 6] = v;
    __syncthreads();
    KeyIdx r = sm[0];
#pragma unroll
    for (int i = 1; i < NW; ++i) r = better(r, sm[i]);
    return r;
}

// ---- bf16 ------------------------------------------------------------------
__device__ inline float bf16_to_f32(uint16_t h) { return __uint_as_float((uint32_t)h << 16); }
// float -> bf16, round to nearest even, on the hardware's packed conversion.  For every input that is not a NaN
// (denormals and infinities included) it returns what the integer form (x + 0x7FFF + bit 16 of x) >> 16 returns:
// compared on the device over all 2^32 bit patterns.
typedef float psd_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 psd_bf16x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t f32x2_to_bf16(float a, float b) {   // a in the low half
    const psd_f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, psd_bf16x2));
}
__device__ inline uint16_t f32_to_bf16(float f) { return (uint16_t)f32x2_to_bf16(f, f); }
// two values as bf16 hi + lo pairs (value = hi + lo to 2^-17 relative), each pair packed with a in the low half
__device__ inline void f32x2_split(float a, float b, uint32_t& hi, uint32_t& lo) {
    hi = f32x2_to_bf16(a, b);
    lo = f32x2_to_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

}  // namespace psd
