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

// max|x| from the per-block partials an absmax pass left behind, in two halves so that a kernel can deal
// with the partials FIRST and ask for its own data after: loads return in order, and a block that fetches
// its tile and then the partials can start on nothing until both are there (a quantize pass of 3840 blocks:
// 21 us that way, 15.5 us with the clip value handed in).  The first wave fetches and reduces the partials
// and leaves the result in LDS -- all blocks of the consuming pass read the same few cache lines, one wave
// each is enough -- while the other waves go straight on to their loads; everybody picks the value up after
// a barrier.
__device__ __forceinline__ void absmax_partials_begin(const float* __restrict__ part, int nparts, float* lds4) {
    if (threadIdx.x < kWave) {
        // (straight-line loads: after a load inside a loop the compiler waits for ALL outstanding loads at
        // the next register it cannot account for, which serialised the tile loads that follow)
        float v[kAbsmaxPartials / kWave];
#pragma unroll
        for (int u = 0; u < kAbsmaxPartials / kWave; ++u) {
            const int i = (int)threadIdx.x + kWave * u;
            v[u] = part[i < nparts ? i : 0];      // (unconditional: a repeated partial does not change the max)
        }
        float m = 0.0f;
#pragma unroll
        for (int u = 0; u < kAbsmaxPartials / kWave; ++u) m = fmaxf(m, v[u]);
        m = wave_max(m);
        if (threadIdx.x == 0) lds4[0] = m;
    }
}
// (all threads get the result; a barrier inside)
__device__ __forceinline__ float absmax_partials_end(const float* lds4) {
    __syncthreads();
    return lds4[0];
}
__device__ __forceinline__ float reduce_absmax_partials(const float* __restrict__ part, int nparts,
                                                        float* lds4) {
    absmax_partials_begin(part, nparts, lds4);
    return absmax_partials_end(lds4);
}

// ---------------------------------------------------------------------------
// Uniform draw for the stochastic rounding of Eq.3: 24 bits, a stateless function of
// (seed, logical element index).  The paper's in-kernel generator (Suppl. "Stochastic
// Rounding", Eq.8) is keyed by thread index; keying by element index instead makes the
// codes independent of launch geometry.  The 64-bit seed is first hashed into two 32-bit
// keys (on the host, once per call); the draw is one avalanche finaliser (multiply /
// xor-shift) over (index ^ key_x) + key_a.  Hashing the seed first matters: with the raw
// seed words as keys, two seeds that differ by d in their low word gave the same table at
// indices xor-ed with d, so layers and iterations seeded 1, 2, 3, ... shared their noise.
// ---------------------------------------------------------------------------
__host__ __device__ __forceinline__ uint32_t rng_mix32(uint32_t x) {
    x ^= x >> 16;
    x *= 0x85EBCA6Bu;
    x ^= x >> 13;
    x *= 0xC2B2AE35u;
    x ^= x >> 16;
    return x;
}
__device__ __forceinline__ uint32_t rng24(uint32_t key_x, uint32_t key_a, uint32_t index) {
    return rng_mix32((index ^ key_x) + key_a) >> 8;
}
// the two keys of a seed: key_x = mix(low word ^ mix(high word + golden ratio)), key_a = mix(key_x + golden ratio)
__host__ __device__ __forceinline__ uint32_t seed_key_x(uint64_t seed) {
    return rng_mix32((uint32_t)seed ^ rng_mix32((uint32_t)(seed >> 32) + 0x9E3779B9u));
}
__host__ __device__ __forceinline__ uint32_t seed_key_a(uint64_t seed) { return rng_mix32(seed_key_x(seed) + 0x9E3779B9u); }

// 127 / c as one correctly rounded fp32 division; 0 for an all-zero tensor.
__device__ __forceinline__ float inv_scale_of(float c) { return (c > 0.0f) ? __fdiv_rn(127.0f, c) : 0.0f; }
__device__ __forceinline__ float scale_of(float c) { return (c > 0.0f) ? __fdiv_rn(c, 127.0f) : 0.0f; }

constexpr float kTwo24 = 16777216.0f;

// Eq.1 on the scaled value, nearest rounding: t = clip(x * inv, 127), |t| <= 127 exactly.
__device__ __forceinline__ int round_nearest_code(float x, float inv) {
    const float t = fminf(fmaxf(__fmul_rn(x, inv), -127.0f), 127.0f);
    return (int)rintf(t);
}

// ---------------------------------------------------------------------------
// Stochastic rounding (Eq.3) on the magnitude:  m = min(127, floor((|x| * inv24 + u) / 2^24)),
// inv24 = inv * 2^24, u a 24-bit draw; the code is sign(x) * m.  floor((P + u)/2^24) of the EXACT
// product P is obtained from one fp32 fused multiply-add evaluated with rounding toward minus
// infinity: every multiple of 2^24 below 2^31 is representable, so rounding the sum down never
// moves it across one, and the saturating float->int32 conversion caps the result at 2^31 - 1,
// whose top byte is 127.  Two instructions per code, no clamp.
// The wave's fp32 rounding mode is switched once; values that must have been computed in the
// default mode are passed through the switch so that the compiler cannot move their
// computation behind it.  fp64 arithmetic has its own mode bits and is not affected.
// ---------------------------------------------------------------------------
__device__ __forceinline__ void fp32_round_down_mode(float& keep0, float& keep1) {
    asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 2\n\ts_nop 3" : "+v"(keep0), "+v"(keep1));
}
// back to round-to-nearest-even (the default) for the fp32 operations that follow
__device__ __forceinline__ void fp32_round_nearest_mode(float& keep0) {
    asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 0, 2), 0\n\ts_nop 3" : "+v"(keep0));
}
// floor(|x| * inv24 + uf) as int32, saturated at 2^31 - 1 (needs the round-down mode).
__device__ __forceinline__ int stoch_fixed(float x, float inv24, float uf) {
    float t;
    int X;
    asm volatile("v_fma_f32 %0, |%1|, %2, %3" : "=v"(t) : "v"(x), "v"(inv24), "v"(uf));
    asm("v_cvt_i32_f32 %0, %1" : "=v"(X) : "v"(t));
    return X;
}
// same with the scale in a scalar register
__device__ __forceinline__ int stoch_fixed_s(float x, float inv24_uniform, float uf) {
    float t;
    int X;
    asm volatile("v_fma_f32 %0, |%1|, %2, %3" : "=v"(t) : "v"(x), "s"(inv24_uniform), "v"(uf));
    asm("v_cvt_i32_f32 %0, %1" : "=v"(X) : "v"(t));
    return X;
}

// Four elements against one (uniform) scale: the four magnitudes min(127, floor(|x_e| * inv + u_e)), u_e in [0, 1),
// packed as bytes [m0, m1, m2, m3].  The caller passes inv2 = 2 * inv and uf2 = 2 * u_e (both exact): in the
// round-down mode the fused multiply-add never crosses an integer, the float -> byte convert-and-pack follows the
// wave's rounding mode (so it floors) and saturates at 255, and floor(2t) >> 1 = floor(t) with 255 >> 1 = 127.
// Ten instructions for four codes; one instruction block, so they stay together and in this order.
__device__ __forceinline__ uint32_t stoch_codes4(const float x[4], float inv2_uniform, const float uf2[4]) {
    uint32_t a;
    float t0, t1, t2, t3;
    asm volatile(
        "v_fma_f32 %1, |%5|, %9, %10\n\t"
        "v_fma_f32 %2, |%6|, %9, %11\n\t"
        "v_fma_f32 %3, |%7|, %9, %12\n\t"
        "v_fma_f32 %4, |%8|, %9, %13\n\t"
        "v_cvt_pk_u8_f32 %0, %1, 0, 0\n\t"
        "v_cvt_pk_u8_f32 %0, %2, 1, %0\n\t"
        "v_cvt_pk_u8_f32 %0, %3, 2, %0\n\t"
        "v_cvt_pk_u8_f32 %0, %4, 3, %0\n\t"
        "v_lshrrev_b32 %0, 1, %0\n\t"
        "v_and_b32 %0, %14, %0"
        : "=&v"(a), "=&v"(t0), "=&v"(t1), "=&v"(t2), "=&v"(t3)
        : "v"(x[0]), "v"(x[1]), "v"(x[2]), "v"(x[3]), "s"(inv2_uniform), "v"(uf2[0]), "v"(uf2[1]), "v"(uf2[2]),
          "v"(uf2[3]), "s"(0x7f7f7f7fu));
    return a;
}

// One code, with NaN -> 0.  STOCH needs fp32_round_down_mode() and inv = inv24.
template <bool STOCH>
__device__ __forceinline__ int quantize_one(float x, float inv, uint32_t seed_lo, uint32_t seed_hi_mul,
                                            uint32_t index) {
    if (STOCH) {
        const float uf = (float)rng24(seed_lo, seed_hi_mul, index);   // exact: 24 bits
        const int m = stoch_fixed(x, inv, uf) >> 24;                  // NaN converts to 0
        return (x < 0.0f) ? -m : m;
    } else {
        float t = __fmul_rn(x, inv);
        t = (t != t) ? 0.0f : t;
        t = fminf(fmaxf(t, -127.0f), 127.0f);
        return (int)rintf(t);
    }
}

// 4x4 byte transpose with v_perm_b32 (the gfx950 byte permute; the paper's Suppl. "INT8 Convolution"
// does the same "4x4 8-bit integer block transpose" with prmt): in d[i] = bytes (i,0..3), out
// o[j] = bytes (0..3, j).  Two rounds of four permutes: pairs of rows interleaved, then the halves
// joined.  Used by the activation quantizer (channel-major dwords -> pixel-major) and by
// backward-weight's loader (image-major -> channel-major).
__device__ __forceinline__ void transpose4x4_bytes(const uint32_t d[4], uint32_t o[4]) {
    // v_perm_b32 picks 4 bytes out of the 8 bytes {hi, lo}; selector byte 0-3 = lo, 4-7 = hi
    const uint32_t t0 = __builtin_amdgcn_perm(d[1], d[0], 0x05010400u);  // d0.b0 d1.b0 d0.b1 d1.b1
    const uint32_t t1 = __builtin_amdgcn_perm(d[1], d[0], 0x07030602u);  // d0.b2 d1.b2 d0.b3 d1.b3
    const uint32_t t2 = __builtin_amdgcn_perm(d[3], d[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(d[3], d[2], 0x07030602u);
    o[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);  // t0.b0 t0.b1 t2.b0 t2.b1
    o[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);  // t0.b2 t0.b3 t2.b2 t2.b3
    o[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    o[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

__device__ __forceinline__ uint32_t pack4(int q0, int q1, int q2, int q3) {
    return (uint32_t)(q0 & 0xff) | ((uint32_t)(q1 & 0xff) << 8) | ((uint32_t)(q2 & 0xff) << 16) |
           ((uint32_t)q3 << 24);
}

}  // namespace int8t
