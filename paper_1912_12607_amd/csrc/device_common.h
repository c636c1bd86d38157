// Shared device helpers of the gfx950 INT8 training-convolution kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "kernels.h"

namespace int8t {

constexpr int kWave = 64;            // CDNA wavefront width

// ---------------------------------------------------------------------------
// Wavefront / block reductions (64-wide shuffles, then one LDS hop per wave).
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ unsigned long long wave_sum(unsigned long long v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// Block-wide max over 256 threads; result valid in every thread.
__device__ __forceinline__ float block_max_256(float v, float* lds4) {
    v = wave_max(v);
    const int w = threadIdx.x >> 6;
    __syncthreads();
    if ((threadIdx.x & 63) == 0) lds4[w] = v;
    __syncthreads();
    return fmaxf(fmaxf(lds4[0], lds4[1]), fmaxf(lds4[2], lds4[3]));
}

// max|x| from the per-block partials an absmax pass left behind (all threads get it).
__device__ __forceinline__ float reduce_absmax_partials(const float* __restrict__ part, int nparts,
                                                        float* lds4) {
    float m = 0.0f;
    for (int i = threadIdx.x; i < nparts; i += blockDim.x) m = fmaxf(m, part[i]);
    return block_max_256(m, lds4);
}

// ---------------------------------------------------------------------------
// Uniform draw for the stochastic rounding of Eq.3: 24 bits, a stateless function of
// (seed, logical element index).  The paper's in-kernel generator (Suppl. "Stochastic
// Rounding", Eq.8) is keyed by thread index; keying by element index instead makes the
// codes independent of launch geometry.  One avalanche finaliser (multiply / xor-shift)
// over the index xored with the low seed word plus the high seed word times an odd constant.
// ---------------------------------------------------------------------------
__device__ __forceinline__ uint32_t rng24(uint32_t seed_lo, uint32_t seed_hi_mul, uint32_t index) {
    uint32_t x = (index ^ seed_lo) + seed_hi_mul;
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x >> 8;
}
__host__ __device__ __forceinline__ uint32_t seed_hi_term(uint64_t seed) {
    return (uint32_t)(seed >> 32) * 0x9E3779B9u;
}

// 127 / c as one correctly rounded fp32 division; 0 for an all-zero tensor.
__device__ __forceinline__ float inv_scale_of(float c) { return (c > 0.0f) ? __fdiv_rn(127.0f, c) : 0.0f; }
__device__ __forceinline__ float scale_of(float c) { return (c > 0.0f) ? __fdiv_rn(c, 127.0f) : 0.0f; }

// floor(x) as int32 in one instruction (saturating).
__device__ __forceinline__ int floor_to_int(float x) {
    int r;
    asm("v_cvt_flr_i32_f32 %0, %1" : "=v"(r) : "v"(x));
    return r;
}

constexpr float kTwo24 = 16777216.0f;
constexpr float kCodeMax24 = 2130706432.0f;   // 127 * 2^24

// Eq.1 on the scaled value, nearest rounding: t = clip(x * inv, 127), |t| <= 127 exactly.
__device__ __forceinline__ int round_nearest_code(float x, float inv) {
    const float t = fminf(fmaxf(__fmul_rn(x, inv), -127.0f), 127.0f);
    return (int)rintf(t);
}
// Eq.3 with 24-bit probabilities on the scaled value carried with 24 fraction bits:
// T = clip(x * inv24, 127*2^24), inv24 = inv * 2^24;  q = floor((floor(T) + u) / 2^24).
// floor(T) + u <= 2^31 - 1, so the 32-bit sum cannot overflow and q stays in [-127, 127].
__device__ __forceinline__ int stochastic_sum(float x, float inv24, int u) {
    const float T = fminf(fmaxf(__fmul_rn(x, inv24), -kCodeMax24), kCodeMax24);
    return floor_to_int(T) + u;   // the code is this sum >> 24 (its signed top byte)
}

// One code, with NaN -> 0.
template <bool STOCH>
__device__ __forceinline__ int quantize_one(float x, float inv, uint32_t seed_lo, uint32_t seed_hi_mul,
                                            uint32_t index) {
    if (STOCH) {
        float T = __fmul_rn(x, __fmul_rn(inv, kTwo24));
        T = (T != T) ? 0.0f : T;
        T = fminf(fmaxf(T, -kCodeMax24), kCodeMax24);
        const int u = (int)rng24(seed_lo, seed_hi_mul, index);
        return (floor_to_int(T) + u) >> 24;
    } else {
        float t = __fmul_rn(x, inv);
        t = (t != t) ? 0.0f : t;
        t = fminf(fmaxf(t, -127.0f), 127.0f);
        return (int)rintf(t);
    }
}

__device__ __forceinline__ uint32_t pack4(int q0, int q1, int q2, int q3) {
    return (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) | ((uint32_t)(q2 & 0xff) << 16) |
           ((uint32_t)q3 << 24);
}

}  // namespace int8t
