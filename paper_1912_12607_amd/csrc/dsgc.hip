// Direction Sensitive Gradient Clipping (Sec.3.4 of the paper) as a candidate search.
//
// One sweep over the gradient evaluates every candidate clip value at once: each thread keeps,
// per candidate j, A_j = sum g*q_j (fp64) and B_j = sum q_j^2 (integer) in registers, and G =
// sum g^2 once.  The deviation of Eq.6 is then d_j = 1 - A_j / sqrt(G * B_j): the scale s_j
// cancels between the numerator and |ghat|, so no dequantized tensor is ever formed.  The
// uniform draw of the stochastic rounding (Eq.3) is taken once per element and shared by all
// candidates -- the same draw the later quantize call uses, so the search scores exactly the
// codes that will be produced.
//
// The sweep reads 4 bytes per element and spends ~10 vector-ALU operations per element and
// candidate: it is bound by the plain vector ALUs, not by HBM.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

constexpr int DSGC_JC = 32;       // candidates per sweep (register accumulators)
constexpr int DSGC_JPAD = 64;     // row pitch of the partial arrays (= INT8T_MAX_CANDIDATES)
constexpr int DSGC_MAX_BLOCKS = 512;

template <int JC, bool STOCH>
__global__ __launch_bounds__(256) void dsgc_sweep_kernel(
    const float* __restrict__ g, size_t n, const float* __restrict__ ratios, int j0, int jn,
    const float* __restrict__ absmax_part, int nparts, uint32_t seed_lo, uint32_t seed_hi_mul,
    float* __restrict__ absmax_out, double* __restrict__ partA, unsigned long long* __restrict__ partB,
    double* __restrict__ partG) {
    __shared__ float lds4[4];
    __shared__ float s_inv[JC];
    __shared__ double s_red[4][JC + 1];
    __shared__ unsigned long long s_redB[4][JC];

    const float M = reduce_absmax_partials(absmax_part, nparts, lds4);
    if (blockIdx.x == 0 && threadIdx.x == 0) *absmax_out = M;
    if (threadIdx.x < JC) {
        const int j = threadIdx.x;
        const float c = (j < jn) ? __fmul_rn(M, ratios[j0 + j]) : 0.0f;
        // stochastic mode carries the scaled value with 24 fraction bits (exact power-of-two factor)
        s_inv[j] = STOCH ? __fmul_rn(inv_scale_of(c), kTwo24) : inv_scale_of(c);
    }
    __syncthreads();
    float inv[JC];
#pragma unroll
    for (int j = 0; j < JC; ++j)
        inv[j] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_inv[j])));

    double A[JC];
    unsigned B[JC];
#pragma unroll
    for (int j = 0; j < JC; ++j) {
        A[j] = 0.0;
        B[j] = 0u;
    }
    double G = 0.0;

    const size_t n4 = n >> 2;
    const float4* __restrict__ g4 = reinterpret_cast<const float4*>(g);
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
        const float4 f = g4[i];
        const float vv[4] = {f.x, f.y, f.z, f.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const float x = vv[e];
            const double xd = (double)x;
            G = fma(xd, xd, G);
            int u = 0;
            if (STOCH) u = (int)rng24(seed_lo, seed_hi_mul, (uint32_t)(4 * i + e));
#pragma unroll
            for (int j = 0; j < JC; ++j) {
                const int r = STOCH ? (stochastic_sum(x, inv[j], u) >> 24) : round_nearest_code(x, inv[j]);
                A[j] = fma(xd, (double)r, A[j]);
                B[j] += (unsigned)(r * r);
            }
        }
    }
    if (blockIdx.x == 0 && threadIdx.x < (n & 3)) {
        const size_t i = (n4 << 2) + threadIdx.x;
        const float x = g[i];
        const double xd = (double)x;
        G = fma(xd, xd, G);
        int u = 0;
        if (STOCH) u = (int)rng24(seed_lo, seed_hi_mul, (uint32_t)i);
#pragma unroll
        for (int j = 0; j < JC; ++j) {
            const int r = STOCH ? (stochastic_sum(x, inv[j], u) >> 24) : round_nearest_code(x, inv[j]);
            A[j] = fma(xd, (double)r, A[j]);
            B[j] += (unsigned)(r * r);
        }
    }

    // block reduction: shuffles inside a wave, then the four waves through LDS in fixed order
    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    G = wave_sum(G);
#pragma unroll
    for (int j = 0; j < JC; ++j) {
        const double a = wave_sum(A[j]);
        const unsigned long long b = wave_sum((unsigned long long)B[j]);
        if (lane == 0) {
            s_red[w][j] = a;
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
    if (threadIdx.x == 0 && j0 == 0)
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
    // eight independent running sums per thread keep sixteen loads in flight
    double a[8];
    unsigned long long b[8];
#pragma unroll
    for (int k = 0; k < 8; ++k) {
        a[k] = 0.0;
        b[k] = 0;
    }
    if (j < n_cand) {
        for (int i = b0; i < b1; i += 8) {
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const bool in = i + k < b1;
                const size_t idx = (size_t)(in ? i + k : b0) * DSGC_JPAD + j;
                const double av = partA[idx];
                const unsigned long long bv = partB[idx];
                a[k] += in ? av : 0.0;
                b[k] += in ? bv : 0ull;
            }
        }
    }
    a[0] = (a[0] + a[4]); a[1] = (a[1] + a[5]); a[2] = (a[2] + a[6]); a[3] = (a[3] + a[7]);
    b[0] += b[4]; b[1] += b[5]; b[2] += b[6]; b[3] += b[7];
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
        const float M = *absmax;
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
    const int blocks = dsgc_blocks(n);
    const uint32_t slo = (uint32_t)seed, shi = seed_hi_term(seed);
    for (int j0 = 0; j0 < n_cand; j0 += DSGC_JC) {
        const int jn = (n_cand - j0 < DSGC_JC) ? (n_cand - j0) : DSGC_JC;
        if (stochastic)
            hipLaunchKernelGGL((dsgc_sweep_kernel<DSGC_JC, true>), dim3(blocks), dim3(256), 0, st, g, n,
                               ratios, j0, jn, ws.absmax_part, nparts_absmax, slo, shi, ws.absmax,
                               ws.partA, ws.partB, ws.partG);
        else
            hipLaunchKernelGGL((dsgc_sweep_kernel<DSGC_JC, false>), dim3(blocks), dim3(256), 0, st, g, n,
                               ratios, j0, jn, ws.absmax_part, nparts_absmax, slo, shi, ws.absmax,
                               ws.partA, ws.partB, ws.partG);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(dsgc_finish_kernel, dim3(1), dim3(1024), 0, st, ws.partA, ws.partB, ws.partG,
                       blocks, ratios, n_cand, ws.absmax, clip_out, dev_out, dev_all_out);
    return hipGetLastError();
}

}  // namespace int8t
