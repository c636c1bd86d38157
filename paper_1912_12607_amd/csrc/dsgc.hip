// Direction Sensitive Gradient Clipping (Sec.3.4 of the paper) as a candidate search.
//
// One sweep over the gradient evaluates the candidate clip values side by side.  Per candidate j
// it needs A_j = sum g*q_j and B_j = sum q_j^2 (and G = sum g^2 once); the deviation of Eq.6 is
// then d_j = 1 - A_j / sqrt(G * B_j): the scale s_j cancels between the numerator and |ghat|, so no
// dequantized tensor is ever formed.  The uniform draw of the stochastic rounding (Eq.3) is taken
// once per element and shared by all candidates -- the same draw the later quantize call uses,
// so the search scores exactly the codes that will be produced.
//
// The sweep is bound by the plain vector ALUs, not by HBM (4 bytes per element against several
// operations per element AND candidate), so the arithmetic is arranged to need few instructions:
//   * codes are sign(g) * m with m the rounded magnitude, so g*q = |g|*m and q^2 = m^2: the whole
//     search runs on magnitudes and never looks at a sign;
//   * m is the top byte of floor(|g| * inv24 + u), one round-down fused multiply-add and one
//     saturating convert (see device_common.h); four elements' bytes are gathered into one dword
//     by byte permutes;
//   * |g| is turned, once per element, into a 46-bit fixed-point integer relative to max|g|
//     (H * 2^23 + L, H <= 2^22, L <= 2^23), and both halves into three byte digits;
//   * A_j and B_j are then sums of uint8 x uint8 products, accumulated four at a time by the 4-way
//     dot-product instruction into 32-bit registers: 6 digit sums + 1 square sum per candidate.
// The integer sums are exact and order independent; the only error against an fp64 evaluation is
// the fixed-point rounding of |g|, |delta| <= max|g| * 2^-45 per element, i.e. at most
// 2^-45 * sqrt(n) in d_j (Cauchy-Schwarz), far below the resolution the search needs.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

constexpr int DSGC_JC = 16;       // candidates per block (7 32-bit accumulators each)
constexpr int DSGC_JPAD = 64;     // row pitch of the partial arrays (= INT8T_MAX_CANDIDATES)
constexpr int DSGC_MAX_BLOCKS = 512;

// bytes [a.b3, b.b3, c.b3, d.b3]: the top bytes of four 32-bit values
__device__ __forceinline__ uint32_t top_bytes(int a, int b, int c, int d) {
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0703u);   // a.b3 b.b3 0 0
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x07030c0cu);   // 0 0 c.b3 d.b3
    return lo | hi;
}
// bytes [a.b0, b.b0, c.b0, d.b0]
__device__ __forceinline__ uint32_t low_bytes(int a, int b, int c, int d) {
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x04000c0cu);
    return lo | hi;
}

// Byte digits of four integers 0 <= v < 2^24:  v = d0 + 256 d1 + 65536 d2.
// plane[b] packs digit b of the four values.
__device__ __forceinline__ void digit_planes(const uint32_t y[4], uint32_t plane[3]) {
    const uint32_t t0 = __builtin_amdgcn_perm(y[1], y[0], 0x05010400u);  // y0.b0 y1.b0 y0.b1 y1.b1
    const uint32_t t1 = __builtin_amdgcn_perm(y[1], y[0], 0x0c0c0602u);  // y0.b2 y1.b2 0 0
    const uint32_t t2 = __builtin_amdgcn_perm(y[3], y[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(y[3], y[2], 0x06020c0cu);  // 0 0 y2.b2 y3.b2
    plane[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    plane[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    plane[2] = t1 | t3;
}

template <bool STOCH>
__global__ __launch_bounds__(256) void dsgc_sweep_kernel(
    const float* __restrict__ g, size_t n, const float* __restrict__ ratios, int n_cand,
    const float* __restrict__ absmax_part, int nparts, uint32_t seed_lo, uint32_t seed_hi_mul,
    float* __restrict__ absmax_out, double* __restrict__ partA, unsigned long long* __restrict__ partB,
    double* __restrict__ partG) {
    constexpr int JC = DSGC_JC;
    __shared__ float lds4[4];
    __shared__ float s_inv[JC];
    __shared__ double s_red[4][JC + 1];
    __shared__ unsigned long long s_redB[4][JC];

    const int j0 = blockIdx.y * JC;
    const int jn = (n_cand - j0 < JC) ? (n_cand - j0) : JC;
    const bool want_g = blockIdx.y == 0;
    const float M = reduce_absmax_partials(absmax_part, nparts, lds4);
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) *absmax_out = M;
    if (threadIdx.x < JC) {
        const int j = threadIdx.x;
        const float c = (j < jn) ? __fmul_rn(M, ratios[j0 + j]) : 0.0f;
        // stochastic mode carries the scaled value with 24 fraction bits (exact power-of-two factor)
        s_inv[j] = STOCH ? __fmul_rn(inv_scale_of(c), kTwo24) : inv_scale_of(c);
    }
    __syncthreads();
    // fixed point: max|g| < 2^e, |g| * 2^(22-e) <= 2^22
    int e2 = 0;
    float mant = frexpf(M, &e2);
    float e2f = (float)e2;
    // From here on every fp32 operation of the stochastic sweep is either exact or the one
    // round-down multiply-add; the candidates' scales above were computed (by other lanes, before
    // the barrier) in the default mode.
    if (STOCH) fp32_round_down_mode(mant, e2f);
    const int shift = 22 - (int)e2f;
    float inv[JC];
#pragma unroll
    for (int j = 0; j < JC; ++j)
        inv[j] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_inv[j])));

    unsigned accA[JC][6];
    unsigned accB[JC];
#pragma unroll
    for (int j = 0; j < JC; ++j) {
        accB[j] = 0;
#pragma unroll
        for (int b = 0; b < 6; ++b) accA[j][b] = 0;
    }
    double G = 0.0;

    auto group = [&](const float x[4], uint32_t index0) {
        float uf[4] = {0.f, 0.f, 0.f, 0.f};
        uint32_t H[4], L[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (STOCH) uf[e] = (float)rng24(seed_lo, seed_hi_mul, index0 + e);   // exact: 24 bits
            const float xs = ldexpf(fabsf(x[e]), shift);     // exact, 0 .. 2^22
            const float h = floorf(xs);
            H[e] = (uint32_t)h;
            L[e] = (uint32_t)rintf((xs - h) * 8388608.0f);   // remainder * 2^23: exact before rint
            if (want_g) {
                const double xd = (double)x[e];
                G = fma(xd, xd, G);
            }
        }
        uint32_t pH[3], pL[3];
        digit_planes(H, pH);
        digit_planes(L, pL);
#pragma unroll
        for (int j = 0; j < JC; ++j) {
            uint32_t rp;
            if (STOCH) {
                rp = top_bytes(stoch_fixed_s(x[0], inv[j], uf[0]), stoch_fixed_s(x[1], inv[j], uf[1]),
                               stoch_fixed_s(x[2], inv[j], uf[2]), stoch_fixed_s(x[3], inv[j], uf[3]));
            } else {
                rp = low_bytes(round_nearest_code(fabsf(x[0]), inv[j]), round_nearest_code(fabsf(x[1]), inv[j]),
                               round_nearest_code(fabsf(x[2]), inv[j]), round_nearest_code(fabsf(x[3]), inv[j]));
            }
            accB[j] = __builtin_amdgcn_udot4(rp, rp, accB[j], false);
#pragma unroll
            for (int b = 0; b < 3; ++b) {
                accA[j][b] = __builtin_amdgcn_udot4(pH[b], rp, accA[j][b], false);
                accA[j][3 + b] = __builtin_amdgcn_udot4(pL[b], rp, accA[j][3 + b], false);
            }
        }
    };

    const size_t n4 = n >> 2;
    const float4* __restrict__ g4 = reinterpret_cast<const float4*>(g);
    const size_t stride = (size_t)gridDim.x * 256;
    {
        // the next iteration's 16 bytes are requested before this iteration's arithmetic starts
        size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
        float4 f = (i < n4) ? g4[i] : make_float4(0.f, 0.f, 0.f, 0.f);
        while (i < n4) {
            const size_t inext = i + stride;
            const float4 fn = (inext < n4) ? g4[inext] : make_float4(0.f, 0.f, 0.f, 0.f);
            const float vv[4] = {f.x, f.y, f.z, f.w};
            group(vv, (uint32_t)(4 * i));
            f = fn;
            i = inext;
        }
    }
    if (blockIdx.x == 0 && threadIdx.x == 0 && (n & 3)) {
        // ragged tail: missing elements are zeros (zero contributes nothing to A, B or G)
        float vv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int e = 0; e < (int)(n & 3); ++e) vv[e] = g[(n4 << 2) + e];
        group(vv, (uint32_t)(n4 << 2));
    }

    // per-thread totals: A = (2^23 * sum_b 256^b aH_b + sum_b 256^b aL_b) * 2^(e-45); the digit
    // sums are exact integers below 2^49 in double, the last additions round like any fp64 sum
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    G = wave_sum(G);
#pragma unroll
    for (int j = 0; j < JC; ++j) {
        const double dH = (double)accA[j][0] + 256.0 * (double)accA[j][1] + 65536.0 * (double)accA[j][2];
        const double dL = (double)accA[j][3] + 256.0 * (double)accA[j][4] + 65536.0 * (double)accA[j][5];
        const double at = ldexp(dH * 8388608.0 + dL, e2 - 45);
        const double asum = wave_sum(at);
        const unsigned long long b = wave_sum((unsigned long long)accB[j]);
        if (lane == 0) {
            s_red[w][j] = asum;
            s_redB[w][j] = b;
        }
    }
    if (lane == 0) s_red[w][JC] = G;
    __syncthreads();
    if (threadIdx.x < JC) {
        const int j = threadIdx.x;
        if (j < jn) {
            partA[(size_t)blockIdx.x * DSGC_JPAD + j0 + j] =
                (s_red[0][j] + s_red[1][j]) + (s_red[2][j] + s_red[3][j]);
            partB[(size_t)blockIdx.x * DSGC_JPAD + j0 + j] =
                s_redB[0][j] + s_redB[1][j] + s_redB[2][j] + s_redB[3][j];
        }
    }
    if (threadIdx.x == 0 && want_g)
        partG[blockIdx.x] = (s_red[0][JC] + s_red[1][JC]) + (s_red[2][JC] + s_red[3][JC]);
}

// Sums the per-block partials in a fixed order, evaluates Eq.6 for every candidate and picks the
// smallest deviation (ties: smallest j, i.e. the largest clip value for decreasing ratios).
// 1024 threads = 64 candidates x 16 block segments; the order of the additions depends on
// (nblocks, n_cand) only, so results are reproducible run to run.
constexpr int DSGC_SEGS = 16;

__global__ __launch_bounds__(1024) void dsgc_finish_kernel(
    const double* __restrict__ partA, const unsigned long long* __restrict__ partB,
    const double* __restrict__ partG, int nblocks, const float* __restrict__ ratios, int n_cand,
    const float* __restrict__ absmax, float* __restrict__ clip_out, double* __restrict__ dev_out,
    double* __restrict__ dev_all_out) {
    __shared__ double sA[DSGC_SEGS][DSGC_JPAD];
    __shared__ unsigned long long sB[DSGC_SEGS][DSGC_JPAD];
    __shared__ double sG[DSGC_SEGS];
    __shared__ double sD[DSGC_JPAD];
    const int j = threadIdx.x & 63, seg = threadIdx.x >> 6;
    const int b0 = (int)(((long long)nblocks * seg) / DSGC_SEGS);
    const int b1 = (int)(((long long)nblocks * (seg + 1)) / DSGC_SEGS);
    // every partial of this thread's segment is requested before the first one is used
    // (at most DSGC_MAX_BLOCKS / DSGC_SEGS = 32 per segment, in two batches of 16)
    const float M = *absmax;
    double a[4] = {0.0, 0.0, 0.0, 0.0};
    unsigned long long b[4] = {0, 0, 0, 0};
    if (j < n_cand) {
        for (int i = b0; i < b1; i += 16) {
            double av[16];
            unsigned long long bv[16];
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const size_t idx = (size_t)((i + k < b1) ? i + k : b0) * DSGC_JPAD + j;
                av[k] = partA[idx];
                bv[k] = partB[idx];
            }
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const bool in = i + k < b1;
                a[k & 3] += in ? av[k] : 0.0;
                b[k & 3] += in ? bv[k] : 0ull;
            }
        }
    }
    sA[seg][j] = (a[0] + a[1]) + (a[2] + a[3]);
    sB[seg][j] = b[0] + b[1] + b[2] + b[3];
    {
        // G: each segment's wave sums its blocks, lane-strided, then a shuffle tree
        double g = 0.0;
        for (int i = b0 + j; i < b1; i += 64) g += partG[i];
        g = wave_sum(g);
        if (j == 0) sG[seg] = g;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        double d = 0.0;
        if (j < n_cand) {
            double At = 0.0, Gt = 0.0;
            unsigned long long Bi = 0;
#pragma unroll
            for (int k = 0; k < DSGC_SEGS; ++k) {
                At += sA[k][j];
                Bi += sB[k][j];
                Gt += sG[k];
            }
            const double Bt = (double)Bi;
            if (Gt == 0.0) d = 0.0;
            else if (Bt == 0.0) d = 1.0;
            else d = 1.0 - At / (sqrt(Gt) * sqrt(Bt));
            if (dev_all_out) dev_all_out[j] = d;
        }
        sD[j] = d;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int best = 0;
        for (int k = 1; k < n_cand; ++k)
            if (sD[k] < sD[best]) best = k;
        if (M == 0.0f) best = 0;
        *clip_out = __fmul_rn(M, ratios[best]);
        *dev_out = sD[best];
    }
}

int dsgc_blocks(size_t n) {
    size_t want = (n / 4 + 255) / 256;
    return (int)(want < 1 ? 1 : (want > (size_t)DSGC_MAX_BLOCKS ? (size_t)DSGC_MAX_BLOCKS : want));
}

hipError_t launch_dsgc(const float* g, size_t n, const float* ratios, int n_cand, int stochastic,
                       uint64_t seed, const DsgcWs& ws, int nparts_absmax, float* clip_out,
                       double* dev_out, double* dev_all_out, hipStream_t st) {
    const int nchunks = (n_cand + DSGC_JC - 1) / DSGC_JC;
    // about two blocks per compute unit in total; every candidate chunk uses the same x-grid so
    // that the partial arrays have one row per x-block
    int blocks = dsgc_blocks(n);
    const int cap = (DSGC_MAX_BLOCKS + nchunks - 1) / nchunks;
    if (blocks > cap) blocks = cap;
    const uint32_t slo = (uint32_t)seed, shi = seed_hi_term(seed);
    dim3 grid(blocks, nchunks);
    {
    KernelTimer kt(KID_DSGC_SWEEP, st);
    if (stochastic)
        hipLaunchKernelGGL((dsgc_sweep_kernel<true>), grid, dim3(256), 0, st, g, n, ratios, n_cand,
                           ws.absmax_part, nparts_absmax, slo, shi, ws.absmax, ws.partA, ws.partB, ws.partG);
    else
        hipLaunchKernelGGL((dsgc_sweep_kernel<false>), grid, dim3(256), 0, st, g, n, ratios, n_cand,
                           ws.absmax_part, nparts_absmax, slo, shi, ws.absmax, ws.partA, ws.partB, ws.partG);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    KernelTimer kt(KID_DSGC_FINISH, st);
    hipLaunchKernelGGL(dsgc_finish_kernel, dim3(1), dim3(1024), 0, st, ws.partA, ws.partB, ws.partG,
                       blocks, ratios, n_cand, ws.absmax, clip_out, dev_out, dev_all_out);
    return hipGetLastError();
}

}  // namespace int8t
