// Quantize passes (Eq.1 / Eq.3 of the paper), the absmax reduction that supplies the default
// clip value, and the scalar finish of the direction deviation (Eq.6).
//
// All of these are HBM-bandwidth bound: each fp32 element is read once and one code byte is
// written.  The layout change fp32 N,C,H,W -> int8 N,H,W,C (reduction dimension innermost, the
// analogue of the paper's NC4HW transposition) happens inside the quantize pass through an LDS
// tile, so it costs no extra HBM traffic.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

// ---------------------------------------------------------------------------------------------
// absmax: grid-stride float4 sweep, one partial per block.  SUMSQ also sums the squares in fp64
// (the |g|^2 of Eq.6; the pass is bound by HBM, the extra arithmetic is free), one partial per
// block, summed in a fixed order, and clears the clip search's accumulators (the sweep that
// follows adds into them).
// ---------------------------------------------------------------------------------------------
// Position of a block inside the (virtual) grid of one tensor's pass: the kernels below are
// written against it so that the batched launches can run several tensors' grids side by side.
struct VBlock {
    int x, y, z;       // block coordinates
    int gx, gy, gz;    // grid extents
};

constexpr int AM_THREADS = 1024;      // 16 waves per block
constexpr int AM_MAX_BLOCKS = kAbsmaxPartials;    // the partials of a pass

template <bool SUMSQ>
__device__ __forceinline__ void absmax_body(const float* __restrict__ x, size_t n, float* __restrict__ part,
                                            double* __restrict__ sumsq, unsigned long long* __restrict__ zero,
                                            int nzero, const int bx, const int gx) {
    // AM_THREADS threads per block: few, fat blocks leave few partials, and every block of the passes that
    // consume them reads all of them (a quantize pass of 3840 blocks spent 5 of its 21 us on 1024 partials)
    __shared__ float ldsm[AM_THREADS / 64];
    __shared__ double ldsd[AM_THREADS / 64];
    if (SUMSQ) {
        for (int z = bx * AM_THREADS + threadIdx.x; z < nzero; z += gx * AM_THREADS) zero[z] = 0ull;
    }
    const size_t n4 = n >> 2;
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(x);
    float m = 0.0f;
    double q[4] = {0.0, 0.0, 0.0, 0.0};
    auto take = [&](const float4& a) {
        m = fmaxf(m, fmaxf(fmaxf(fabsf(a.x), fabsf(a.y)), fmaxf(fabsf(a.z), fabsf(a.w))));
        if (SUMSQ) {
            q[0] = fma((double)a.x, (double)a.x, q[0]);
            q[1] = fma((double)a.y, (double)a.y, q[1]);
            q[2] = fma((double)a.z, (double)a.z, q[2]);
            q[3] = fma((double)a.w, (double)a.w, q[3]);
        }
    };
    const size_t stride = (size_t)gx * AM_THREADS;
    size_t i = (size_t)bx * AM_THREADS + threadIdx.x;
    // four independent 16-byte loads in flight per thread
    for (; i + 3 * stride < n4; i += 4 * stride) {
        float4 a = x4[i], b = x4[i + stride], c = x4[i + 2 * stride], d = x4[i + 3 * stride];
        take(a);
        take(b);
        take(c);
        take(d);
    }
    for (; i < n4; i += stride) take(x4[i]);
    if (bx == 0 && threadIdx.x < (n & 3)) {
        const float v = x[(n4 << 2) + threadIdx.x];
        m = fmaxf(m, fabsf(v));
        if (SUMSQ) q[0] = fma((double)v, (double)v, q[0]);
    }
    m = wave_max(m);
    double t = 0.0;
    if (SUMSQ) t = wave_sum((q[0] + q[1]) + (q[2] + q[3]));
    if ((threadIdx.x & 63) == 0) {
        ldsm[threadIdx.x >> 6] = m;
        if (SUMSQ) ldsd[threadIdx.x >> 6] = t;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        float mm = 0.0f;
        double ss = 0.0;
#pragma unroll
        for (int w = 0; w < AM_THREADS / 64; ++w) {      // fixed order: the sum does not depend on timing
            mm = fmaxf(mm, ldsm[w]);
            if (SUMSQ) ss += ldsd[w];
        }
        part[bx] = mm;
        if (SUMSQ) sumsq[bx] = ss;
    }
}

template <bool SUMSQ>
__global__ __launch_bounds__(AM_THREADS) void absmax_kernel(const float* __restrict__ x, size_t n,
                                                     float* __restrict__ part, double* __restrict__ sumsq,
                                                     unsigned long long* __restrict__ zero, int nzero) {
    absmax_body<SUMSQ>(x, n, part, sumsq, zero, nzero, (int)blockIdx.x, (int)gridDim.x);
}

// several tensors in one launch: block b serves the tensor whose block range holds it
__global__ __launch_bounds__(AM_THREADS) void absmax_batch_kernel(const AbsmaxBatch b) {
    int i = 0;
    while (i + 1 < b.count && (int)blockIdx.x >= b.it[i].block0 + b.it[i].nblocks) ++i;
    const AbsmaxBatchItem& t = b.it[i];
    if (t.sumsq) absmax_body<true>(t.x, t.n, t.part, t.sumsq, t.zero, t.nzero, (int)blockIdx.x - t.block0, t.nblocks);
    else absmax_body<false>(t.x, t.n, t.part, nullptr, nullptr, 0, (int)blockIdx.x - t.block0, t.nblocks);
}

int absmax_blocks(size_t n) {
    size_t want = (n / 4 + AM_THREADS * 8 - 1) / (AM_THREADS * 8);   // >= 8 float4 per thread before adding blocks
    return (int)(want < 1 ? 1 : (want > (size_t)AM_MAX_BLOCKS ? (size_t)AM_MAX_BLOCKS : want));
}

hipError_t launch_absmax_batch(const AbsmaxBatch& b, int total_blocks, hipStream_t st) {
    KernelTimer kt(KID_ABSMAX_BATCH, st);
    launch_timed(kt, absmax_batch_kernel, dim3(total_blocks), dim3(AM_THREADS), 0, st, b);
    return hipGetLastError();
}

hipError_t launch_absmax(const float* x, size_t n, float* part, int* nparts, hipStream_t st, double* sumsq,
                         unsigned long long* zero, int nzero) {
    const int blocks = absmax_blocks(n);
    *nparts = blocks;
    KernelTimer kt(KID_ABSMAX, st);
    if (sumsq) launch_timed(kt, absmax_kernel<true>, dim3(blocks), dim3(AM_THREADS), 0, st, x, n, part, sumsq, zero, nzero);
    else launch_timed(kt, absmax_kernel<false>, dim3(blocks), dim3(AM_THREADS), 0, st, x, n, part, sumsq, zero, 0);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Block-level reduction of the Eq.6 partial sums, one DevPartial per block.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void block_store_devpartial(double A, double G, unsigned long long B,
                                                       DevPartial* __restrict__ out) {
    __shared__ double ldsA[4], ldsG[4];
    __shared__ unsigned long long ldsB[4];
    A = wave_sum(A);
    G = wave_sum(G);
    B = wave_sum(B);
    const int w = threadIdx.x >> 6;
    if ((threadIdx.x & 63) == 0) {
        ldsA[w] = A;
        ldsG[w] = G;
        ldsB[w] = B;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        DevPartial p;
        p.A = (ldsA[0] + ldsA[1]) + (ldsA[2] + ldsA[3]);
        p.G = (ldsG[0] + ldsG[1]) + (ldsG[2] + ldsG[3]);
        p.B = ldsB[0] + ldsB[1] + ldsB[2] + ldsB[3];
        *out = p;
    }
}

__device__ __forceinline__ float resolve_clip(const float* __restrict__ clip,
                                              const float* __restrict__ part, int nparts, float* lds4) {
    if (clip) return *clip;
    return reduce_absmax_partials(part, nparts, lds4);
}

// ---------------------------------------------------------------------------------------------
// Activations / gradients: fp32 N,C,H,W -> int8 N,H,W,Cp.
// One block = 64 pixels x 64 channels of one image.  Loads walk pixels (contiguous in the
// source), each thread owns four consecutive channels of its pixel and packs them to one
// dword; the store phase walks channels (contiguous in the destination) in 16-byte pieces.
// ---------------------------------------------------------------------------------------------
constexpr int QA_PIX = 64;
constexpr int QA_CH = 64;
// Tensors of at most 16 channels (an image, the gradient of a narrow layer) have one 16-byte granule
// per pixel: a thread then makes one pixel's granule on its own -- up to 16 loads that walk the
// pixels of each channel plane, one 16-byte store -- and a block takes 256 pixels; the 64 x 64 tile
// would be a quarter full and the 3-channel image of a stem 50 000 blocks of 192 elements (112 us
// for 9.6 M elements).
constexpr int QA_NARROW_PIX = 256;
// A block takes quant_act_nsub() pixel tiles of 64 one after the other: a whole channel plane when that
// is at most 256 pixels and not a whole number of 128-byte lines (14 x 14 images).  The 256-byte run of
// a tile shares its first and last line with the neighbouring tiles there, and tiles quantized by
// different blocks at different times fetched those lines twice (measured at 14 x 14: 1.56 x the
// tensor fetched; 1024 channels, batch 128: 30.6 -> 25.5 us).  Larger planes gain nothing (17 x 17 and
// 28 x 28 lose a little to the ragged last block) and keep one tile per block.
__host__ __device__ inline int quant_act_nsub(int HW) {
    if ((HW * 4) % 128 == 0 || HW > 4 * QA_PIX) return 1;
    return (HW + QA_PIX - 1) / QA_PIX;
}
__host__ __device__ inline int quant_act_gx(int Cp, int HW) {
    return Cp == 16 ? (HW + QA_NARROW_PIX - 1) / QA_NARROW_PIX : (HW + QA_PIX * quant_act_nsub(HW) - 1) / (QA_PIX * quant_act_nsub(HW));
}

// VEC: H*W is a multiple of 4, so a thread can fetch four consecutive pixels of a channel with one
// 16-byte load; it then owns a 4-channel x 4-pixel block, transposes its codes in registers and
// writes one dword (4 channels) per pixel to the LDS tile.  Otherwise one pixel per lane, 4-byte loads.
template <bool STOCH, bool DEV, bool VEC>
__device__ __forceinline__ void quantize_act_body(
    const float* __restrict__ x, int C, int Cp, int HW, const float* __restrict__ clip,
    const float* __restrict__ absmax_part, int nparts, uint32_t seed_lo, uint32_t seed_hi_mul,
    int8_t* __restrict__ q, float* __restrict__ scale_out, DevPartial* __restrict__ devpart, const VBlock vb,
    float* lds4, uint32_t (*tile)[QA_CH / 4 + 1]) {
    // lds4: 4 floats, tile: [QA_PIX][QA_CH / 4 + 1] dwords of LDS supplied by the kernel
    const int n = vb.z;
    if (Cp == 16) {
        const int p = vb.x * QA_NARROW_PIX + (int)threadIdx.x;
        const bool pv = p < HW;
        const float clip_in = clip ? *clip : 0.0f;
        if (!clip) absmax_partials_begin(absmax_part, nparts, lds4);      // dealt with ahead of the pixels
        float v[16];
#pragma unroll
        for (int c = 0; c < 16; ++c) v[c] = (pv && c < C) ? x[((size_t)n * C + c) * HW + p] : 0.0f;
        float cval = clip_in;
        if (!clip) cval = absmax_partials_end(lds4);
        float inv = inv_scale_of(cval);
        float sc = scale_of(cval);
        if (STOCH) {
            inv = __fmul_rn(inv, kTwo24);        // the scaled value carries 24 fraction bits
            fp32_round_down_mode(inv, sc);
        }
        if (vb.x == 0 && vb.z == 0 && threadIdx.x == 0) *scale_out = sc;
        double A = 0.0, G = 0.0;
        unsigned long long B = 0;
        uint32_t d[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            int code[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int c = 4 * j + k;
                code[k] = 0;
                if (pv && c < C) {
                    code[k] = quantize_one<STOCH>(v[c], inv, seed_lo, seed_hi_mul, (uint32_t)(((size_t)n * C + c) * HW + p));
                    if (DEV) {
                        const double g = (double)v[c];
                        A = fma(g, (double)code[k], A);
                        G = fma(g, g, G);
                        B += (unsigned)(code[k] * code[k]);
                    }
                }
            }
            d[j] = pack4(code[0], code[1], code[2], code[3]);
        }
        if (pv) *reinterpret_cast<uint4*>(q + ((size_t)n * HW + p) * 16) = make_uint4(d[0], d[1], d[2], d[3]);
        if (DEV) block_store_devpartial(A, G, B, devpart + (vb.z * vb.gx + vb.x));
        return;
    }
    const int c0 = vb.y * QA_CH;
    // the clip value: handed in (read now, a scalar load), or the absmax partials, dealt with ahead of the tile
    const float clip_in = clip ? *clip : 0.0f;
    if (!clip) absmax_partials_begin(absmax_part, nparts, lds4);
    const int nsub = quant_act_nsub(HW);
    const int lane = threadIdx.x & 63;
    const int wv = threadIdx.x >> 6;
    const int pq = threadIdx.x & 15, cgp = threadIdx.x >> 4;      // VEC: pixel quad, 4-channel group
    float inv = 0.0f, sc = 0.0f;
    double A = 0.0, G = 0.0;
    unsigned long long B = 0;
    for (int sub = 0; sub < nsub; ++sub) {
        const int p0 = (vb.x * nsub + sub) * QA_PIX;
        if (p0 >= HW) break;                                      // (uniform over the block)
        const int p = p0 + lane;
        const bool pv = p < HW;

        // issue every global load of this thread before anything depends on them
        float v[4][4];
        if (VEC) {
            // unconditional loads (lanes outside the tensor re-read its first floats and are zeroed afterwards):
            // with a branch around each load the compiler has been seen to wait for one load before issuing the next
            float4 f[4];
            bool ok[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = c0 + 4 * cgp + j;
                ok[j] = p0 + 4 * pq < HW && c < C;
                f[j] = *reinterpret_cast<const float4*>(x + (ok[j] ? ((size_t)n * C + c) * HW + p0 + 4 * pq : (size_t)0));
            }
            const bool whole = p0 + QA_PIX <= HW && c0 + QA_CH <= C;      // (uniform) nothing to zero in this tile
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (!whole && !ok[j]) f[j] = make_float4(0.f, 0.f, 0.f, 0.f);
                v[j][0] = f[j].x; v[j][1] = f[j].y; v[j][2] = f[j].z; v[j][3] = f[j].w;     // v[channel][pixel]
            }
        } else {
            const bool whole = p0 + QA_PIX <= HW && c0 + QA_CH <= C;      // (uniform) nothing to zero in this tile
#pragma unroll
            for (int i = 0; i < 4; ++i) {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = c0 + 4 * (wv + 4 * i) + j;
                    v[i][j] = x[(pv && c < C) ? ((size_t)n * C + c) * HW + p : (size_t)0];      // unconditional, as above
                }
            }
            if (!whole) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        if (!(pv && c0 + 4 * (wv + 4 * i) + j < C)) v[i][j] = 0.0f;
            }
        }

        if (sub == 0) {
            float cval = clip_in;
            if (!clip) cval = absmax_partials_end(lds4);
            inv = inv_scale_of(cval);
            sc = scale_of(cval);
            if (STOCH) {
                inv = __fmul_rn(inv, kTwo24);        // the scaled value carries 24 fraction bits
                fp32_round_down_mode(inv, sc);
            }
            if (vb.x == 0 && vb.y == 0 && vb.z == 0 && threadIdx.x == 0) *scale_out = sc;
        } else {
            __syncthreads();                         // the previous tile's codes have left LDS
        }

        if (VEC) {
            uint32_t d[4], o[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int c = c0 + 4 * cgp + j;
                int code[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const uint32_t idx = (uint32_t)(((size_t)n * C + c) * HW + p0 + 4 * pq + k);
                    code[k] = quantize_one<STOCH>(v[j][k], inv, seed_lo, seed_hi_mul, idx);
                    if (DEV) {
                        const double g = (double)v[j][k];
                        A = fma(g, (double)code[k], A);
                        G = fma(g, g, G);
                        B += (unsigned)(code[k] * code[k]);
                    }
                }
                d[j] = pack4(code[0], code[1], code[2], code[3]);
            }
            transpose4x4_bytes(d, o);     // d[channel] = 4 pixels -> o[pixel] = 4 channels
#pragma unroll
            for (int k = 0; k < 4; ++k) tile[4 * pq + k][cgp] = o[k];
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                int code[4];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int c = c0 + 4 * (wv + 4 * i) + j;
                    const uint32_t idx = (uint32_t)(((size_t)n * C + c) * HW + p);
                    code[j] = quantize_one<STOCH>(v[i][j], inv, seed_lo, seed_hi_mul, idx);
                    if (DEV) {
                        const double g = (double)v[i][j];
                        A = fma(g, (double)code[j], A);
                        G = fma(g, g, G);
                        B += (unsigned)(code[j] * code[j]);
                    }
                }
                tile[lane][wv + 4 * i] = pack4(code[0], code[1], code[2], code[3]);
            }
        }
        __syncthreads();

        const int pl = threadIdx.x >> 2;
        const int chunk = threadIdx.x & 3;
        if (p0 + pl < HW && c0 + chunk * 16 < Cp) {
            uint4 o;
            o.x = tile[pl][chunk * 4 + 0];
            o.y = tile[pl][chunk * 4 + 1];
            o.z = tile[pl][chunk * 4 + 2];
            o.w = tile[pl][chunk * 4 + 3];
            *reinterpret_cast<uint4*>(q + ((size_t)n * HW + p0 + pl) * Cp + c0 + chunk * 16) = o;
        }
    }
    if (DEV) {
        const int b = (vb.z * vb.gy + vb.y) * vb.gx + vb.x;
        block_store_devpartial(A, G, B, devpart + b);
    }
}

template <bool STOCH, bool DEV, bool VEC>
__global__ __launch_bounds__(256) void quantize_act_kernel(
    const float* __restrict__ x, int C, int Cp, int HW, const float* __restrict__ clip,
    const float* __restrict__ absmax_part, int nparts, uint32_t seed_lo, uint32_t seed_hi_mul,
    int8_t* __restrict__ q, float* __restrict__ scale_out, DevPartial* __restrict__ devpart) {
    __shared__ float lds4[4];
    __shared__ uint32_t tile[QA_PIX][QA_CH / 4 + 1];
    const VBlock vb = {(int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, (int)gridDim.x, (int)gridDim.y, (int)gridDim.z};
    quantize_act_body<STOCH, DEV, VEC>(x, C, Cp, HW, clip, absmax_part, nparts, seed_lo, seed_hi_mul, q, scale_out,
                                       devpart, vb, lds4, tile);
}

int quant_blocks_act(int N, int Cp, int HW) {
    return quant_act_gx(Cp, HW) * ((Cp + QA_CH - 1) / QA_CH) * N;
}

hipError_t launch_quantize_act(const QuantArgs& a, hipStream_t st) {
    const int N = a.d0, C = a.d1, HW = a.d2 * a.d3, Cp = (C + 15) & ~15;
    dim3 grid(quant_act_gx(Cp, HW), (Cp + QA_CH - 1) / QA_CH, N);
    const uint32_t slo = seed_key_x(a.seed), shi = seed_key_a(a.seed);
    KernelTimer kt(KID_QUANTIZE_ACT, st);
#define LAUNCH(ST, DV)                                                                                      \
    do {                                                                                                    \
        if ((HW & 3) == 0)                                                                                  \
            launch_timed(kt, (quantize_act_kernel<ST, DV, true>), grid, dim3(256), 0, st, a.x, C, Cp, HW, \
                               a.clip, a.absmax_part, a.nparts, slo, shi, a.q, a.scale, a.devpart);         \
        else                                                                                                \
            launch_timed(kt, (quantize_act_kernel<ST, DV, false>), grid, dim3(256), 0, st, a.x, C, Cp, HW, \
                               a.clip, a.absmax_part, a.nparts, slo, shi, a.q, a.scale, a.devpart);         \
    } while (0)
    if (a.stochastic) {
        if (a.devpart) LAUNCH(true, true); else LAUNCH(true, false);
    } else {
        if (a.devpart) LAUNCH(false, true); else LAUNCH(false, false);
    }
#undef LAUNCH
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Planar codes (depthwise layers): element-wise, logical order kept.
// ---------------------------------------------------------------------------------------------
constexpr int QP_BLOCKS_MAX = 4096;

template <bool STOCH, bool DEV>
__device__ __forceinline__ void quantize_planar_body(
    const float* __restrict__ x, size_t n, const float* __restrict__ clip,
    const float* __restrict__ absmax_part, int nparts, uint32_t seed_lo, uint32_t seed_hi_mul,
    int8_t* __restrict__ q, float* __restrict__ scale_out, DevPartial* __restrict__ devpart, const int bx, const int gx,
    float* lds4) {
    const float cval = resolve_clip(clip, absmax_part, nparts, lds4);
    float inv = inv_scale_of(cval);
    float sc = scale_of(cval);
    if (STOCH) {
        inv = __fmul_rn(inv, kTwo24);        // the scaled value carries 24 fraction bits
        fp32_round_down_mode(inv, sc);
    }
    if (bx == 0 && threadIdx.x == 0) *scale_out = sc;

    double A = 0.0, G = 0.0;
    unsigned long long B = 0;
    const size_t n4 = n >> 2;
    const float4* __restrict__ x4 = reinterpret_cast<const float4*>(x);
    uint32_t* __restrict__ q4 = reinterpret_cast<uint32_t*>(q);
    const size_t stride = (size_t)gx * 256;
    for (size_t i = (size_t)bx * 256 + threadIdx.x; i < n4; i += stride) {
        const float4 f = x4[i];
        const float vv[4] = {f.x, f.y, f.z, f.w};
        int code[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            code[j] = quantize_one<STOCH>(vv[j], inv, seed_lo, seed_hi_mul, (uint32_t)(4 * i + j));
            if (DEV) {
                const double g = (double)vv[j];
                A = fma(g, (double)code[j], A);
                G = fma(g, g, G);
                B += (unsigned)(code[j] * code[j]);
            }
        }
        q4[i] = pack4(code[0], code[1], code[2], code[3]);
    }
    if (bx == 0 && threadIdx.x < (n & 3)) {
        const size_t i = (n4 << 2) + threadIdx.x;
        const float g32 = x[i];
        const int code = quantize_one<STOCH>(g32, inv, seed_lo, seed_hi_mul, (uint32_t)i);
        q[i] = (int8_t)code;
        if (DEV) {
            const double g = (double)g32;
            A = fma(g, (double)code, A);
            G = fma(g, g, G);
            B += (unsigned)(code * code);
        }
    }
    if (DEV) block_store_devpartial(A, G, B, devpart + bx);
}

template <bool STOCH, bool DEV>
__global__ __launch_bounds__(256) void quantize_planar_kernel(
    const float* __restrict__ x, size_t n, const float* __restrict__ clip,
    const float* __restrict__ absmax_part, int nparts, uint32_t seed_lo, uint32_t seed_hi_mul,
    int8_t* __restrict__ q, float* __restrict__ scale_out, DevPartial* __restrict__ devpart) {
    __shared__ float lds4[4];
    quantize_planar_body<STOCH, DEV>(x, n, clip, absmax_part, nparts, seed_lo, seed_hi_mul, q, scale_out, devpart,
                                     (int)blockIdx.x, (int)gridDim.x, lds4);
}

int quant_blocks_planar(size_t n) {
    size_t want = (n / 4 + 256 * 4 - 1) / (256 * 4);
    return (int)(want < 1 ? 1 : (want > (size_t)QP_BLOCKS_MAX ? (size_t)QP_BLOCKS_MAX : want));
}

hipError_t launch_quantize_planar(const QuantArgs& a, hipStream_t st) {
    const size_t n = (size_t)a.d0 * a.d1 * a.d2 * a.d3;
    const int blocks = quant_blocks_planar(n);
    const uint32_t slo = seed_key_x(a.seed), shi = seed_key_a(a.seed);
    KernelTimer kt(KID_QUANTIZE_PLANAR, st);
#define LAUNCH(ST, DV)                                                                              \
    launch_timed(kt, (quantize_planar_kernel<ST, DV>), dim3(blocks), dim3(256), 0, st, a.x, n,    \
                       a.clip, a.absmax_part, a.nparts, slo, shi, a.q, a.scale, a.devpart)
    if (a.stochastic) {
        if (a.devpart) LAUNCH(true, true); else LAUNCH(true, false);
    } else {
        if (a.devpart) LAUNCH(false, true); else LAUNCH(false, false);
    }
#undef LAUNCH
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Weights: fp32 K,Cg,R,S -> two int8 copies, [K][R][S][Cp] (forward / backward-weight view) and
// [Cg][R][S][Kp] (backward-data view).  A block owns 16 filters x 16 channels x (up to 64) taps:
// it reads, per filter, one contiguous run of 16 * taps floats, keeps the codes in LDS, and writes
// both views as 16-byte granules (16 channels of one filter and tap; 16 filters of one channel and
// tap).  Rows and channels beyond the tensor are zero codes, which fills the padded pitch.
// ---------------------------------------------------------------------------------------------
constexpr int QW_T = 16;
constexpr int QW_TAPS = 64;
static int quant_wgt_zsplit(int K, int Cg, int R, int S);
// Channel tiles per block.  A filter's share of a block is one contiguous run of 16 * taps floats;
// with one to three taps that is 64 to 192 bytes, a fraction of what a wave-wide load can fetch, and
// a fully connected layer's 2 M weights would be 8000 blocks of 256 elements (44 us).  Few-tap
// filters therefore take 64 or 32 channels per block.  So do filters of up to 16 taps when the tensor is
// large enough to leave 512 blocks: the forward view's granules of a (filter, tap) are then written 64 or 32
// bytes at a time instead of 16 (768 x 768 x 7 weights beside the activations of their layer: 33.0 -> 29.1 us).
__host__ __device__ inline int quant_wgt_cm(int K, int Cg, int R, int S) {
    const int RS = R * S;
    int cm = RS == 1 ? 4 : RS <= 3 ? 2 : 1;
    if (RS > 3 && RS <= 16) {
        const long long ktiles = (K + QW_T - 1) / QW_T;
        if (ktiles * ((Cg + 4 * QW_T - 1) / (4 * QW_T)) >= 512) cm = 4;
        else if (ktiles * ((Cg + 2 * QW_T - 1) / (2 * QW_T)) >= 512) cm = 2;
    }
    while (cm > 1 && Cg <= QW_T * (cm / 2)) cm /= 2;      // no wider than the tensor
    return cm;
}
static int quant_wgt_gx(int K, int Cg, int R, int S) {
    const int ct = QW_T * quant_wgt_cm(K, Cg, R, S);
    return (Cg + ct - 1) / ct;
}

template <bool STOCH, bool DEV>
__device__ __forceinline__ void quantize_wgt_body(
    const float* __restrict__ w, int K, int Cg, int R, int S, int Cp, int Kp, size_t off2,
    const float* __restrict__ clip, const float* __restrict__ absmax_part, int nparts,
    uint32_t seed_lo, uint32_t seed_hi_mul, int8_t* __restrict__ q, float* __restrict__ scale_out,
    DevPartial* __restrict__ devpart, const VBlock vb, float* lds4, int8_t* tile) {
    // lds4: 4 floats, tile: QW_T * CT * min(taps, QW_TAPS) bytes of LDS, [filter][channel][tap], supplied by the kernel
    const float cval = resolve_clip(clip, absmax_part, nparts, lds4);
    float inv = inv_scale_of(cval);
    float sc = scale_of(cval);
    if (STOCH) {
        inv = __fmul_rn(inv, kTwo24);        // the scaled value carries 24 fraction bits
        fp32_round_down_mode(inv, sc);
    }
    if (vb.x == 0 && vb.y == 0 && vb.z == 0 && threadIdx.x == 0) *scale_out = sc;

    const int RS = R * S;
    const int CM = quant_wgt_cm(K, Cg, R, S), CT = QW_T * CM;      // channels per block
    const int k0 = vb.y * QW_T, c0 = vb.x * CT;
    double A = 0.0, G = 0.0;
    unsigned long long B = 0;
    // small tensors spread their taps over blockIdx.z to have enough blocks
    const int tpb = (RS + vb.gz - 1) / vb.gz;
    const int rs_begin = vb.z * tpb, rs_end = (rs_begin + tpb < RS) ? rs_begin + tpb : RS;
    for (int rs0 = rs_begin; rs0 < rs_end; rs0 += QW_TAPS) {
        const int nrs = (rs_end - rs0 < QW_TAPS) ? (rs_end - rs0) : QW_TAPS;
        const int per_k = CT * nrs;
        if (rs0 != rs_begin) __syncthreads();
        const int cvalid = (Cg - c0 < CT) ? (Cg - c0) : CT;
        if (nrs == RS) {
            // all taps at once: a filter's 16 channels x taps are one contiguous run; a wave walks the
            // runs of four filters, 64 consecutive floats per load
            const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const int k_l = wave * 4 + kk, k = k0 + k_l;
                const size_t base = ((size_t)k * Cg + c0) * RS;
                // long runs: four loads in flight per lane; short ones (up to 256 floats): one trip each
                const int step4 = per_k > 256 ? 4 : 1;
                for (int rem0 = lane; rem0 < per_k; rem0 += 64 * step4) {
                    float g32[4];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int rem = rem0 + 64 * u;
                        g32[u] = (u < step4 && k < K && rem < cvalid * RS) ? w[base + rem] : 0.0f;
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const int rem = rem0 + 64 * u;
                        if (u >= step4 || rem >= per_k) break;
                        int code = 0;
                        if (k < K && rem < cvalid * RS) {
                            code = quantize_one<STOCH>(g32[u], inv, seed_lo, seed_hi_mul, (uint32_t)(base + rem));
                            if (DEV) {
                                const double g = (double)g32[u];
                                A = fma(g, (double)code, A);
                                G = fma(g, g, G);
                                B += (unsigned)(code * code);
                            }
                        }
                        tile[k_l * per_k + rem] = (int8_t)code;
                    }
                }
            }
        } else {
            for (int e = threadIdx.x; e < QW_T * per_k; e += 256) {
                const int k_l = e / per_k, rem = e - k_l * per_k;
                const int c_l = rem / nrs, rs_l = rem - c_l * nrs;
                const int k = k0 + k_l;
                int code = 0;
                if (k < K && c_l < cvalid) {
                    const size_t idx = ((size_t)k * Cg + c0 + c_l) * RS + rs0 + rs_l;
                    const float g32 = w[idx];
                    code = quantize_one<STOCH>(g32, inv, seed_lo, seed_hi_mul, (uint32_t)idx);
                    if (DEV) {
                        const double g = (double)g32;
                        A = fma(g, (double)code, A);
                        G = fma(g, g, G);
                        B += (unsigned)(code * code);
                    }
                }
                tile[e] = (int8_t)code;
            }
        }
        __syncthreads();
        // view 1: granule (filter, tap, channel tile) = 16 channels; the channel tile runs fastest
        for (int u = threadIdx.x; u < QW_T * nrs * CM; u += 256) {
            const int k_l = u / (nrs * CM), r2 = u - k_l * (nrs * CM);
            const int rs_l = r2 / CM, cb = (r2 - rs_l * CM) * QW_T;
            if (k0 + k_l < K && c0 + cb < Cp) {
                uint32_t d[4];
                const int8_t* __restrict__ tp = tile + (k_l * CT + cb) * nrs + rs_l;
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    d[j] = pack4(tp[(4 * j) * nrs], tp[(4 * j + 1) * nrs], tp[(4 * j + 2) * nrs], tp[(4 * j + 3) * nrs]);
                *reinterpret_cast<uint4*>(q + ((size_t)(k0 + k_l) * RS + rs0 + rs_l) * Cp + c0 + cb) = make_uint4(d[0], d[1], d[2], d[3]);
            }
        }
        // view 2: granule (channel, tap) = 16 filters
        for (int u = threadIdx.x; u < CT * nrs; u += 256) {
            const int c_l = u / nrs, rs_l = u - c_l * nrs;
            if (c0 + c_l < Cg) {
                uint32_t d[4];
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    d[j] = pack4(tile[((4 * j) * CT + c_l) * nrs + rs_l], tile[((4 * j + 1) * CT + c_l) * nrs + rs_l],
                                 tile[((4 * j + 2) * CT + c_l) * nrs + rs_l], tile[((4 * j + 3) * CT + c_l) * nrs + rs_l]);
                *reinterpret_cast<uint4*>(q + off2 + ((size_t)(c0 + c_l) * RS + rs0 + rs_l) * Kp + k0) = make_uint4(d[0], d[1], d[2], d[3]);
            }
        }
    }
    if (DEV) block_store_devpartial(A, G, B, devpart + (vb.z * vb.gy + vb.y) * vb.gx + vb.x);
}

template <bool STOCH, bool DEV>
__global__ __launch_bounds__(256) void quantize_wgt_kernel(
    const float* __restrict__ w, int K, int Cg, int R, int S, int Cp, int Kp, size_t off2,
    const float* __restrict__ clip, const float* __restrict__ absmax_part, int nparts,
    uint32_t seed_lo, uint32_t seed_hi_mul, int8_t* __restrict__ q, float* __restrict__ scale_out,
    DevPartial* __restrict__ devpart) {
    __shared__ float lds4[4];
    __shared__ __attribute__((aligned(16))) int8_t tile[QW_T * QW_T * QW_TAPS];
    const VBlock vb = {(int)blockIdx.x, (int)blockIdx.y, (int)blockIdx.z, (int)gridDim.x, (int)gridDim.y, (int)gridDim.z};
    quantize_wgt_body<STOCH, DEV>(w, K, Cg, R, S, Cp, Kp, off2, clip, absmax_part, nparts, seed_lo, seed_hi_mul, q,
                                  scale_out, devpart, vb, lds4, tile);
}

// ---------------------------------------------------------------------------------------------
// Batched quantization (Eq.1, or Eq.3 per item) of several tensors in one launch: the activations
// and the weights of a layer (and its output gradient when the clip value is kept), or the weights
// of many layers.  Small tensors otherwise pay a whole
// kernel launch each (a few microseconds of an idle GPU for a few thousand elements).  Block b
// serves the tensor whose block range holds it and runs that tensor's ordinary pass.
// ---------------------------------------------------------------------------------------------
// ANYSTOCH: some item rounds stochastically (Eq.3).  The round-to-nearest launch of a layer's a and
// W is a kernel of its own, so that it keeps its register count beside the clip search.
template <bool ANYSTOCH>
__global__ __launch_bounds__(256) void quantize_batch_kernel(const QuantBatch b) {
    // one LDS area for whichever pass this block runs, sized by the host for the tensors of this launch
    // (a 3x3 weight tensor needs 2.3 KB of tile, not the 16 KB of the largest case: the kernel then fits
    // beside other kernels' blocks on a compute unit)
    __shared__ float lds4[4];
    extern __shared__ __attribute__((aligned(16))) int8_t smem[];
    uint32_t (*const atile)[QA_CH / 4 + 1] = reinterpret_cast<uint32_t (*)[QA_CH / 4 + 1]>(smem);
    int i = 0;
    while (i + 1 < b.count && (int)blockIdx.x >= b.it[i].block0 + b.it[i].gx * b.it[i].gy * b.it[i].gz) ++i;
    const QuantBatchItem& t = b.it[i];
    const int local = (int)blockIdx.x - t.block0;
    const int gxy = t.gx * t.gy;
    const int z = local / gxy, rem = local - z * gxy;
    const int y = rem / t.gx;
    const VBlock vb = {rem - y * t.gx, y, z, t.gx, t.gy, t.gz};
    const bool st = ANYSTOCH && t.stoch;          // block-uniform
    if (t.kind == 0) {          // activations, N,C,H,W -> N,H,W,Cp
        const int HW = t.d2 * t.d3, Cp = (t.d1 + 15) & ~15;
#define ACT(STv, VECv) quantize_act_body<STv, false, VECv>(t.x, t.d1, Cp, HW, t.clip, t.absmax_part, t.nparts, t.seed_lo, t.seed_hi, t.q, t.scale, nullptr, vb, lds4, atile)
        if (ANYSTOCH && st) {
            if ((HW & 3) == 0) ACT(ANYSTOCH, true); else ACT(ANYSTOCH, false);
        } else {
            if ((HW & 3) == 0) ACT(false, true); else ACT(false, false);
        }
#undef ACT
    } else if (t.kind == 1) {   // weights, two views
        const int Cp = (t.d1 + 15) & ~15, Kp = (t.d0 + 15) & ~15;
        const size_t off2 = (((size_t)t.d0 * t.d2 * t.d3 * Cp) + 255) & ~(size_t)255;
        if (ANYSTOCH && st)
            quantize_wgt_body<ANYSTOCH, false>(t.x, t.d0, t.d1, t.d2, t.d3, Cp, Kp, off2, t.clip, t.absmax_part, t.nparts, t.seed_lo, t.seed_hi,
                                               t.q, t.scale, nullptr, vb, lds4, smem);
        else
            quantize_wgt_body<false, false>(t.x, t.d0, t.d1, t.d2, t.d3, Cp, Kp, off2, t.clip, t.absmax_part, t.nparts, 0u, 0u,
                                            t.q, t.scale, nullptr, vb, lds4, smem);
    } else {                    // planar
        const size_t n = (size_t)t.d0 * t.d1 * t.d2 * t.d3;
        if (ANYSTOCH && st)
            quantize_planar_body<ANYSTOCH, false>(t.x, n, t.clip, t.absmax_part, t.nparts, t.seed_lo, t.seed_hi, t.q, t.scale, nullptr, vb.x, vb.gx, lds4);
        else
            quantize_planar_body<false, false>(t.x, n, t.clip, t.absmax_part, t.nparts, 0u, 0u, t.q, t.scale, nullptr, vb.x, vb.gx, lds4);
    }
}

// grid of one tensor's quantize pass, by layout (0 activations, 1 weights, else planar)
void quant_grid(int kind, const int d[4], int* gx, int* gy, int* gz) {
    if (kind == 0) {
        const int HW = d[2] * d[3], Cp = (d[1] + 15) & ~15;
        *gx = quant_act_gx(Cp, HW); *gy = (Cp + QA_CH - 1) / QA_CH; *gz = d[0];
    } else if (kind == 1) {
        *gx = quant_wgt_gx(d[0], d[1], d[2], d[3]); *gy = (d[0] + QW_T - 1) / QW_T; *gz = quant_wgt_zsplit(d[0], d[1], d[2], d[3]);
    } else {
        *gx = quant_blocks_planar((size_t)d[0] * d[1] * d[2] * d[3]); *gy = 1; *gz = 1;
    }
}

hipError_t launch_quantize_batch(const QuantBatch& b, int total_blocks, hipStream_t st) {
    size_t lds = 16;
    for (int i = 0; i < b.count; ++i) {
        const QuantBatchItem& t = b.it[i];
        size_t need = 0;
        if (t.kind == 0) {
            need = sizeof(uint32_t) * QA_PIX * (QA_CH / 4 + 1);
        } else if (t.kind == 1) {
            const int tpb = (t.d2 * t.d3 + t.gz - 1) / t.gz;          // taps per block along z
            need = (size_t)QW_T * QW_T * quant_wgt_cm(t.d0, t.d1, t.d2, t.d3) * (tpb < QW_TAPS ? tpb : QW_TAPS);
        }
        if (need > lds) lds = need;
    }
    lds = (lds + 15) & ~(size_t)15;
    KernelTimer kt(KID_QUANTIZE_BATCH, st);
    bool any_stoch = false;
    for (int i = 0; i < b.count; ++i) any_stoch = any_stoch || b.it[i].stoch;
    if (any_stoch) launch_timed(kt, quantize_batch_kernel<true>, dim3(total_blocks), dim3(256), lds, st, b);
    else launch_timed(kt, quantize_batch_kernel<false>, dim3(total_blocks), dim3(256), lds, st, b);
    return hipGetLastError();
}

// blocks along the taps: 1 for tensors with many 16 x 16 tiles, up to R*S for small ones
static int quant_wgt_zsplit(int K, int Cg, int R, int S) {
    const int tiles = ((K + QW_T - 1) / QW_T) * quant_wgt_gx(K, Cg, R, S);
    int z = (256 + tiles - 1) / tiles;
    if (z > R * S) z = R * S;
    return z < 1 ? 1 : z;
}
int quant_blocks_wgt(int K, int Cg, int R, int S) {
    return ((K + QW_T - 1) / QW_T) * quant_wgt_gx(K, Cg, R, S) * quant_wgt_zsplit(K, Cg, R, S);
}

hipError_t launch_quantize_wgt(const QuantArgs& a, hipStream_t st) {
    const int K = a.d0, Cg = a.d1, R = a.d2, S = a.d3;
    const int Cp = (Cg + 15) & ~15, Kp = (K + 15) & ~15;
    const size_t off2 = (((size_t)K * R * S * Cp) + 255) & ~(size_t)255;
    const dim3 grid(quant_wgt_gx(K, Cg, R, S), (K + QW_T - 1) / QW_T, quant_wgt_zsplit(K, Cg, R, S));
    const uint32_t slo = seed_key_x(a.seed), shi = seed_key_a(a.seed);
    KernelTimer kt(KID_QUANTIZE_WGT, st);
#define LAUNCH(ST, DV)                                                                              \
    launch_timed(kt, (quantize_wgt_kernel<ST, DV>), grid, dim3(256), 0, st, a.x, K, Cg, R, \
                       S, Cp, Kp, off2, a.clip, a.absmax_part, a.nparts, slo, shi, a.q, a.scale,    \
                       a.devpart)
    if (a.stochastic) {
        if (a.devpart) LAUNCH(true, true); else LAUNCH(true, false);
    } else {
        if (a.devpart) LAUNCH(false, true); else LAUNCH(false, false);
    }
#undef LAUNCH
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Eq.6 finish: d = 1 - A / sqrt(G * B)  (the scale s cancels between numerator and |ghat|).
// Partials are summed in a fixed tree order, so the result is deterministic.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void deviation_finish_kernel(const DevPartial* __restrict__ part,
                                                               int nparts, double* __restrict__ out) {
    __shared__ double sA[256], sG[256];
    __shared__ unsigned long long sB[256];
    double A = 0.0, G = 0.0;
    unsigned long long B = 0;
    for (int i = threadIdx.x; i < nparts; i += 256) {
        A += part[i].A;
        G += part[i].G;
        B += part[i].B;
    }
    sA[threadIdx.x] = A;
    sG[threadIdx.x] = G;
    sB[threadIdx.x] = B;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) {
            sA[threadIdx.x] += sA[threadIdx.x + s];
            sG[threadIdx.x] += sG[threadIdx.x + s];
            sB[threadIdx.x] += sB[threadIdx.x + s];
        }
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double g = sG[0], b = (double)sB[0];
        double d;
        if (g == 0.0) d = 0.0;
        else if (b == 0.0) d = 1.0;
        else d = 1.0 - sA[0] / (sqrt(g) * sqrt(b));
        *out = d;
    }
}

hipError_t launch_deviation_finish(const DevPartial* part, int nparts, double* dev_out, hipStream_t st) {
    KernelTimer kt(KID_DEVIATION_FINISH, st);
    launch_timed(kt, deviation_finish_kernel, dim3(1), dim3(256), 0, st, part, nparts, dev_out);
    return hipGetLastError();
}

}  // namespace int8t
