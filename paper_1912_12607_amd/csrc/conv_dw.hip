// Depthwise convolution (groups == C == K) on planar int8 codes.  The paper singles the
// depthwise layer out as the structure with the hardest gradients (Sec.3.2, C4) but describes no
// kernel for it.  The reduction per output is only R*S taps (forward / backward-data), so this
// is not a dense contraction and the MFMA is of no use: every (n,c) plane is an independent 2-D
// filter, staged in LDS and evaluated on the plain integer ALUs; the kernels are HBM bound
// (1 byte in, 4 bytes out per element).
#include <type_traits>

#include "device_common.h"
#include "kernels.h"

namespace int8t {

constexpr int DW_MAX_TAPS = 64;   // R*S limit of the depthwise kernels

// One block per (n,c) plane.  Forward: in = codes of a, gather ih = oh*stride - pad + r.
// Backward-data: in = codes of g_z, gather ih = (oh + pad - r)/stride when divisible.
// ST: both strides when known at compile time (2: the divisions below become shifts), 0 = any.
// NT: threads per block (64, 128 or 256 by plane size, dw_threads()).
template <bool DGRAD, int ST, int NT>
__global__ __launch_bounds__(NT) void dw_conv_kernel(const DwArgs a) {
    const int stride_h = ST ? ST : a.stride_h, stride_w = ST ? ST : a.stride_w;
    extern __shared__ __attribute__((aligned(16))) int8_t plane[];
    __shared__ int wtap[DW_MAX_TAPS];
    const int nc = blockIdx.x;
    const int c = nc % a.C;
    const int IHW = a.IH * a.IW, OHW = a.OH * a.OW, RS = a.R * a.S;
    const int8_t* __restrict__ src = a.a + (size_t)nc * IHW;
    if ((IHW & 15) == 0) {
        for (int i = threadIdx.x; i < (IHW >> 4); i += NT)
            reinterpret_cast<uint4*>(plane)[i] = reinterpret_cast<const uint4*>(src)[i];
    } else {
        for (int i = threadIdx.x; i < IHW; i += NT) plane[i] = src[i];
    }
    if (threadIdx.x < RS) wtap[threadIdx.x] = (int)a.b[(size_t)c * RS + threadIdx.x];
    __syncthreads();

    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
    for (int o = threadIdx.x; o < OHW; o += NT) {
        const int oh = o / a.OW, ow = o - oh * a.OW;
        int sum = 0;
        if (DGRAD) {
            // Only the taps r = r0 + k * stride_h with r0 = (oh + pad_h) mod stride_h reach this pixel,
            // tap r0 from gradient row (oh + pad_h - r0) / stride_h and every further one from the row
            // above; the same along w.  Two divisions per pixel instead of one per tap, and the taps
            // that never divide are not visited at all.
            const int ph = oh + a.pad_h, pw = ow + a.pad_w;
            const int qh = ph / stride_h, qw = pw / stride_w;
            const int r0 = ph - qh * stride_h, s0 = pw - qw * stride_w;
            int ih = qh;
            for (int r = r0; r < a.R && ih >= 0; r += stride_h, --ih) {
                if (ih >= a.IH) continue;
                int iw = qw;
                for (int s = s0; s < a.S && iw >= 0; s += stride_w, --iw) {
                    if (iw >= a.IW) continue;
                    sum += (int)plane[ih * a.IW + iw] * wtap[r * a.S + s];
                }
            }
        } else {
            for (int r = 0; r < a.R; ++r) {
                const int ih = oh * stride_h - a.pad_h + r;
                if ((unsigned)ih >= (unsigned)a.IH) continue;
                for (int s = 0; s < a.S; ++s) {
                    const int iw = ow * stride_w - a.pad_w + s;
                    if ((unsigned)iw >= (unsigned)a.IW) continue;
                    sum += (int)plane[ih * a.IW + iw] * wtap[r * a.S + s];
                }
            }
        }
        const size_t idx = (size_t)nc * OHW + o;
        a.out[idx] = __fmul_rn((float)sum, scale);
        if (a.acc) a.acc[idx] = sum;
    }
}

// ---------------------------------------------------------------------------------------------
// Stride-1 fast path (filters up to 8 wide).  The plane is staged into LDS with its zero border
// (top = -drmin rows, left = -dsmin columns), so that the taps of output column ow start at LDS
// column ow: a thread owns four consecutive outputs of a row, fetches the S + 3 bytes they read
// from each filter row as aligned dwords, and forms each output's row sum with one byte-align and
// one 4-way int8 dot product against the row's packed weights.  No bounds tests, no divisions per
// tap; four results leave as one 16-byte store.
//   forward        LDS row oh + r', column ow + s'  holds a[oh - ph + r', ow - pw + s'],   weight w[r'][s']
//   backward-data  LDS row oh + r', column ow + s'  holds g[oh + ph - (R-1) + r', ...],    weight w[R-1-r'][S-1-s']
// ---------------------------------------------------------------------------------------------
constexpr int DW_FAST_MAXR = 8;

// Copy plane `src` (IH x IW, contiguous) into LDS `dst` (rows of `pitch` bytes) at (top, left).
template <int NT>
__device__ __forceinline__ void dw_fill_plane(const int8_t* __restrict__ src, int IH, int IW, int8_t* dst,
                                              int pitch, int top, int left) {
    const int IHW = IH * IW;
    if ((IHW & 15) == 0 && ((IW | left | pitch) & 3) == 0) {
        // rows of whole dwords at a dword-aligned place: four 4-byte stores per chunk (none straddles a row)
        for (int i = threadIdx.x; i < (IHW >> 4); i += NT) {
            const uint4 v = reinterpret_cast<const uint4*>(src)[i];
            const uint32_t d[4] = {v.x, v.y, v.z, v.w};
            int row = (16 * i) / IW, col = 16 * i - row * IW;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                *reinterpret_cast<uint32_t*>(dst + (row + top) * pitch + col + left) = d[w];
                col += 4;
                if (col == IW) {
                    col = 0;
                    ++row;
                }
            }
        }
    } else if ((IHW & 15) == 0) {
        // 16 source bytes per thread and pass; row / column advance without divisions
        for (int i = threadIdx.x; i < (IHW >> 4); i += NT) {
            const uint4 v = reinterpret_cast<const uint4*>(src)[i];
            const uint32_t d[4] = {v.x, v.y, v.z, v.w};
            int row = (16 * i) / IW, col = 16 * i - row * IW;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                dst[(row + top) * pitch + col + left] = (int8_t)(d[k >> 2] >> (8 * (k & 3)));
                if (++col == IW) {
                    col = 0;
                    ++row;
                }
            }
        }
    } else {
        for (int i = threadIdx.x; i < IHW; i += NT) {
            const int row = i / IW, col = i - row * IW;
            dst[(row + top) * pitch + col + left] = src[i];
        }
    }
}

// dw_fill_plane() in two halves for planes of a whole number of 16-byte chunks, at most CPT per thread:
// the chunks of a thread fetched into registers, and written to LDS later -- so that the next image's
// planes can be on their way while the current one is being worked on.
template <int NT, int CPT>
__device__ __forceinline__ void dw_plane_fetch(const int8_t* __restrict__ src, int IHW, uint4 (&regs)[CPT]) {
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
        const int i = (int)threadIdx.x + u * NT;
        regs[u] = reinterpret_cast<const uint4*>(src)[i < (IHW >> 4) ? i : 0];     // (unconditional; the surplus is not stored)
    }
}
template <int NT, int CPT>
__device__ __forceinline__ void dw_plane_store(const uint4 (&regs)[CPT], int IHW, int IW, int8_t* dst, int pitch, int top,
                                               int left) {
#pragma unroll
    for (int u = 0; u < CPT; ++u) {
        const int i = (int)threadIdx.x + u * NT;
        if (i < (IHW >> 4)) {
            const uint32_t d[4] = {regs[u].x, regs[u].y, regs[u].z, regs[u].w};
            int row = (16 * i) / IW, col = 16 * i - row * IW;
            if (((IW | left | pitch) & 3) == 0) {      // (uniform) whole dwords at a dword-aligned place
#pragma unroll
                for (int w = 0; w < 4; ++w) {
                    *reinterpret_cast<uint32_t*>(dst + (row + top) * pitch + col + left) = d[w];
                    col += 4;
                    if (col == IW) {
                        col = 0;
                        ++row;
                    }
                }
            } else {
#pragma unroll
                for (int k = 0; k < 16; ++k) {
                    dst[(row + top) * pitch + col + left] = (int8_t)(d[k >> 2] >> (8 * (k & 3)));
                    if (++col == IW) {
                        col = 0;
                        ++row;
                    }
                }
            }
        }
    }
}

// Stage a plane with its zero border: `rows` x `pitch` bytes of LDS, the plane at (top, left).
template <int NT>
__device__ __forceinline__ void dw_stage_plane(const int8_t* __restrict__ src, int IH, int IW, int8_t* dst,
                                               int rows, int pitch, int top, int left) {
    const int ndw = rows * pitch >> 2;          // pitch is a multiple of 4
    for (int i = threadIdx.x; i < ndw; i += NT) reinterpret_cast<uint32_t*>(dst)[i] = 0u;
    __syncthreads();
    dw_fill_plane<NT>(src, IH, IW, dst, pitch, top, left);
    __syncthreads();
}

// t / d for 0 <= t < 2^15 and quotients below 2^10, d >= 1, with inv = 1.0f / d: (t + 0.5) / d is at least 0.5 / d away
// from an integer and the fp32 product is off by less than 2^-13, so truncation gives the exact quotient -- four
// instructions where the integer division takes some thirty-five.
__device__ __forceinline__ int dw_div_small(int t, float inv) { return (int)(((float)t + 0.5f) * inv); }

// Small planes (7 x 7, 14 x 14, 28 x 28): a block takes `np` consecutive planes -- they are one contiguous run of
// np * IH * IW source bytes -- so that it has a few hundred results to form; one plane per block made a
// 7 x 7 layer 61 440 blocks of 49 results, each living two memory round trips (960 channels, batch 64: 23 us per
// pass for 15 MB of traffic).  Plane p is staged at dst + p * psize; 16-byte loads when the run is a whole number of
// aligned chunks (`vec`, uniform over the block).
// 16 bytes of the run starting at byte 16 * i, scattered to their planes' staged rows
__device__ __forceinline__ void dw_scatter_chunk(const uint4& v, int i, int IH, int IW, int IHW, int8_t* dst, int psize,
                                                 int pitch, int top, int left) {
    const uint32_t d[4] = {v.x, v.y, v.z, v.w};
    int pl = (16 * i) / IHW;
    const int rem = 16 * i - pl * IHW;
    int row = rem / IW, col = rem - row * IW;
    int8_t* rowp = dst + pl * psize + (row + top) * pitch + left;
    if (((IW | left | pitch | psize) & 3) == 0) {      // (uniform) rows of whole dwords at a dword-aligned place
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            *reinterpret_cast<uint32_t*>(rowp + col) = d[w];
            col += 4;
            if (col == IW) {
                col = 0;
                rowp += pitch;
                if (++row == IH) {
                    row = 0;
                    rowp += psize - IH * pitch;
                }
            }
        }
        return;
    }
    // (the byte loop is kept rolled: unrolled sixteen-fold in each of its callers it cost the kernels 100 registers)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        uint32_t dw = d[w];
#pragma unroll 1
        for (int b = 0; b < 4; ++b) {
            rowp[col] = (int8_t)dw;
            dw >>= 8;
            if (++col == IW) {
                col = 0;
                rowp += pitch;
                if (++row == IH) {
                    row = 0;
                    rowp += psize - IH * pitch;
                }
            }
        }
    }
}
// The first two chunks of every thread are requested by dw_planes_fetch() at the top of the kernel, ahead of the
// weights and of the zeroing of the staged area, and written by dw_planes_store(); blocks of at most
// 32 * NT source bytes (every case with more than one plane but 28 x 28 planes by the dozen) need no further loads.
template <int NT>
__device__ __forceinline__ void dw_planes_fetch(const int8_t* __restrict__ src, int nch, uint4 (&regs)[2]) {
    if (nch > 0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int i = (int)threadIdx.x + u * NT;
            regs[u] = reinterpret_cast<const uint4*>(src)[i < nch ? i : 0];     // (unconditional; the surplus is not stored)
        }
    }
}
template <int NT>
__device__ __forceinline__ void dw_planes_store(const int8_t* __restrict__ src, int np, int nch, const uint4 (&regs)[2], int IH,
                                                int IW, int8_t* dst, int rows, int pitch, int top, int left) {
    const int psize = rows * pitch;
    const int ndw = np * psize >> 2;          // pitch is a multiple of 4
    for (int i = threadIdx.x; i < ndw; i += NT) reinterpret_cast<uint32_t*>(dst)[i] = 0u;
    __syncthreads();
    const int IHW = IH * IW, total = np * IHW;
    if (nch > 0) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const int i = (int)threadIdx.x + u * NT;
            if (i < nch) dw_scatter_chunk(regs[u], i, IH, IW, IHW, dst, psize, pitch, top, left);
        }
        for (int i = (int)threadIdx.x + 2 * NT; i < nch; i += NT)
            dw_scatter_chunk(reinterpret_cast<const uint4*>(src)[i], i, IH, IW, IHW, dst, psize, pitch, top, left);
    } else {
        for (int i = threadIdx.x; i < total; i += NT) {
            const int pl = i / IHW, rem = i - pl * IHW;
            const int row = rem / IW, col = rem - row * IW;
            dst[pl * psize + (row + top) * pitch + col + left] = src[i];
        }
    }
    __syncthreads();
}

// ST = 2 (forward only): the four outputs of a thread read windows that start two bytes apart, from
// LDS row 2 * oh + r' and column 2 * ow; `rows` is the height of the staged area.
constexpr int DW_MAX_PPB = 32;        // planes per block of the fast path, at most

// OFF: the plane is staged OFF bytes further right than its border asks, so that its rows
// start on a dword of LDS and are written four bytes at a time (see dw_fill_plane); the windows then start OFF bytes
// further right as well.
template <bool DGRAD, int SD, int NT, int ST = 1, int OFF = 0>    // SD = dwords of packed weights per filter row (S <= 4*SD)
__global__ __launch_bounds__(NT) void dw_conv_fast_kernel(const DwArgs a, int pitch, int rows, int ppb) {
    static_assert(ST == 1 || (ST == 2 && !DGRAD), "the strided form is the forward pass at stride 2");
    extern __shared__ __attribute__((aligned(16))) int8_t plane[];
    __shared__ uint32_t wrow[DW_MAX_PPB][DW_FAST_MAXR][SD];
    const int nc0 = blockIdx.x * ppb;                            // the block's first plane (n * C + c)
    const int np = a.N * a.C - nc0 < ppb ? a.N * a.C - nc0 : ppb;
    const int OHW = a.OH * a.OW, RS = a.R * a.S, IHW = a.IH * a.IW;
    const int psize = rows * pitch;
    const int top = DGRAD ? (a.R - 1 - a.pad_h) : a.pad_h;     // = -drmin
    const int left = DGRAD ? (a.S - 1 - a.pad_w) : a.pad_w;    // = -dsmin
    const size_t src0 = (size_t)nc0 * IHW;
    // 16-byte chunks of the block's source run, 0 when it is not a whole number of aligned chunks (uniform)
    const int nch = (ppb > 1 && ((np * IHW) & 15) == 0 && (reinterpret_cast<uintptr_t>(a.a + src0) & 15) == 0) ? (np * IHW) >> 4 : 0;
    uint4 pregs[2];
    if (ppb > 1) dw_planes_fetch<NT>(a.a + src0, nch, pregs);
    for (int i = threadIdx.x; i < np * a.R * SD; i += NT) {
        const int pl = i / (a.R * SD), q = i - pl * (a.R * SD);
        const int rp = q / SD, d = q - rp * SD;
        const int c = (nc0 + pl) % a.C;
        uint32_t wv = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int sp = 4 * d + k;
            if (sp < a.S) {
                const int r = DGRAD ? (a.R - 1 - rp) : rp, sx = DGRAD ? (a.S - 1 - sp) : sp;
                wv |= (uint32_t)(uint8_t)a.b[(size_t)c * RS + r * a.S + sx] << (8 * k);
            }
        }
        wrow[pl][rp][d] = wv;
    }
    if (ppb == 1) dw_stage_plane<NT>(a.a + src0, a.IH, a.IW, plane, rows, pitch, top, left + OFF);
    else dw_planes_store<NT>(a.a + src0, np, nch, pregs, a.IH, a.IW, plane, rows, pitch, top, left + OFF);

    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
    const int QW = (a.OW + 3) >> 2;
    const int per = a.OH * QW;                                   // tasks of a plane: four results of a row each
    const bool vec = (a.OW & 3) == 0;
    const bool small = per < 1024;                               // (then t < 32 * 1024 as well: dw_div_small is exact)
    const float inv_per = 1.0f / (float)per, inv_qw = 1.0f / (float)QW;
    for (int t = threadIdx.x; t < np * per; t += NT) {
        const int pl = ppb == 1 ? 0 : small ? dw_div_small(t, inv_per) : t / per, tt = t - pl * per;
        const int oh = small ? dw_div_small(tt, inv_qw) : tt / QW, ow = (tt - oh * QW) << 2;
        const int8_t* __restrict__ pp = plane + pl * psize;
        float* __restrict__ outp = a.out + (size_t)(nc0 + pl) * OHW;
        int32_t* __restrict__ accp = a.acc ? a.acc + (size_t)(nc0 + pl) * OHW : nullptr;
        int sum[4] = {0, 0, 0, 0};
        for (int rp = 0; rp < a.R; ++rp) {
            const uint32_t* __restrict__ rowp = reinterpret_cast<const uint32_t*>(pp + (ST * oh + rp) * pitch + ST * ow);
            constexpr int ND = ((OFF + 3 * ST + 3) >> 2) + SD;       // dwords the four windows reach into
            uint32_t d[ND];
#pragma unroll
            for (int k = 0; k < ND; ++k) d[k] = rowp[k];
#pragma unroll
            for (int k = 0; k < SD; ++k) {
                const uint32_t wv = wrow[pl][rp][k];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    // output j's window starts OFF + ST * j bytes into the row segment
                    const int dwi = k + (OFF + ST * j) / 4, sh = (OFF + ST * j) % 4;
                    const uint32_t win = sh == 0 ? d[dwi] : __builtin_amdgcn_alignbyte(d[dwi + 1], d[dwi], sh);
                    sum[j] = __builtin_amdgcn_sdot4((int)win, (int)wv, sum[j], false);
                }
            }
        }
        const int o = oh * a.OW + ow;
        if (vec) {
            *reinterpret_cast<float4*>(outp + o) = make_float4(__fmul_rn((float)sum[0], scale), __fmul_rn((float)sum[1], scale),
                                                               __fmul_rn((float)sum[2], scale), __fmul_rn((float)sum[3], scale));
            if (accp) {   // the accumulator output is only required to be 4-byte aligned
#pragma unroll
                for (int j = 0; j < 4; ++j) accp[o + j] = sum[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (ow + j < a.OW) {
                    outp[o + j] = __fmul_rn((float)sum[j], scale);
                    if (accp) accp[o + j] = sum[j];
                }
            }
        }
    }
}


// ---------------------------------------------------------------------------------------------
// Backward-data at stride 2 for an R x S filter known at compile time.  Pixel (h, w) is reached by
// the taps r = r0 + 2a, r0 = (h + ph) & 1, from gradient row ((h + ph) >> 1) - a, and likewise
// along w: the gradient plane sits in LDS at (TB, LB) inside a zeroed area, so no tap needs a bounds
// test, a thread owns four consecutive pixels of a row (their column parities are known: w0 is a
// multiple of 4), reads the few gradient bytes they share once per tap row, and picks each tap
// row's weights by the row parity with selects -- no divisions, no loop over taps that never reach.
// ---------------------------------------------------------------------------------------------
template <int R, int S, int NT>
__global__ __launch_bounds__(NT) void dw_dgrad_s2_kernel(const DwArgs a, int pitch, int rows) {
    extern __shared__ __attribute__((aligned(16))) int8_t plane[];
    constexpr int TB = (R - 1) / 2, LB = (S - 1) / 2, NA = (R + 1) / 2;
    const int nc = blockIdx.x;
    const int c = nc % a.C;
    int wt[R][S];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int sx = 0; sx < S; ++sx) wt[r][sx] = (int)a.b[(size_t)c * (R * S) + r * S + sx];
    dw_stage_plane<NT>(a.a + (size_t)nc * a.IH * a.IW, a.IH, a.IW, plane, rows, pitch, TB, LB);

    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
    const int OHW = a.OH * a.OW;
    const int QW = (a.OW + 3) >> 2;
    const bool vec = (a.OW & 3) == 0;
    const int p0 = a.pad_w & 1;                        // column parity of a thread's first pixel
    float* __restrict__ outp = a.out + (size_t)nc * OHW;
    int32_t* __restrict__ accp = a.acc ? a.acc + (size_t)nc * OHW : nullptr;
    for (int t = threadIdx.x; t < a.OH * QW; t += NT) {
        const int h = t / QW, w0 = (t - h * QW) << 2;
        const int hh = h + a.pad_h;
        const bool rodd = hh & 1;
        const int8_t* __restrict__ base = plane + ((hh >> 1) + TB) * pitch + ((w0 + a.pad_w) >> 1) + LB;
        int sum[4] = {0, 0, 0, 0};
#pragma unroll
        for (int aa = 0; aa < NA; ++aa) {
            const int8_t* __restrict__ rowp = base - aa * pitch;
            int v[LB + 3];
#pragma unroll
            for (int i = 0; i < LB + 3; ++i) v[i] = (int)rowp[i - LB];
            int wr[S];                                 // weights of tap row r0 + 2 aa (zero beyond the filter)
#pragma unroll
            for (int sx = 0; sx < S; ++sx) {
                const int we = wt[2 * aa][sx];
                const int wo = (2 * aa + 1 < R) ? wt[2 * aa + 1 < R ? 2 * aa + 1 : 0][sx] : 0;     // (index kept inside the array)
                wr[sx] = rodd ? wo : we;
            }
            auto row_sum = [&](auto P0) {
                constexpr int p = decltype(P0)::value;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int q = (p + j) & 1, cr = (p + j) >> 1;
#pragma unroll
                    for (int b = 0; q + 2 * b < S; ++b) sum[j] += wr[q + 2 * b] * v[LB + cr - b];
                }
            };
            if (p0) row_sum(std::integral_constant<int, 1>{});
            else row_sum(std::integral_constant<int, 0>{});
        }
        const int o = h * a.OW + w0;
        if (vec) {
            *reinterpret_cast<float4*>(outp + o) = make_float4(__fmul_rn((float)sum[0], scale), __fmul_rn((float)sum[1], scale),
                                                               __fmul_rn((float)sum[2], scale), __fmul_rn((float)sum[3], scale));
            if (accp) {
#pragma unroll
                for (int j = 0; j < 4; ++j) accp[o + j] = sum[j];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (w0 + j < a.OW) {
                    outp[o + j] = __fmul_rn((float)sum[j], scale);
                    if (accp) accp[o + j] = sum[j];
                }
            }
        }
    }
}

// Backward-weight: g_W[c,r,s] = sum_{n,p,q} g_z[n,c,p,q] * a[n,c,p*sh+r-ph,q*sw+s-pw].
// grid (C, chunks); a block sums its share of the images for one channel and writes
// partial[chunk][c][rs]; the reduce kernel adds the chunks and applies Eq.2.
template <int NT>
__device__ __forceinline__ void dw_block_sum_store(int v, int* red, int32_t* dst) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = red[0];
        for (int w = 1; w < (int)(NT >> 6); ++w) t += red[w];
        *dst = t;
    }
}

// The same for NV sums at once, behind ONE barrier (red: NT / 64 x NV ints of LDS that nothing else uses).
template <int NT, int NV>
__device__ __forceinline__ void dw_block_sums_store(int (&v)[NV], int* red, int32_t* dst) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v[i] += __shfl_xor(v[i], o, kWave);
    }
    if ((threadIdx.x & 63) == 0) {
#pragma unroll
        for (int i = 0; i < NV; ++i) red[(threadIdx.x >> 6) * NV + i] = v[i];
    }
    __syncthreads();
    if ((int)threadIdx.x < NV) {
        int t = red[threadIdx.x];
        for (int w = 1; w < (int)(NT >> 6); ++w) t += red[w * NV + threadIdx.x];
        dst[threadIdx.x] = t;
    }
}

template <int NT>
__global__ __launch_bounds__(NT) void dw_wgrad_kernel(const DwArgs a) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    __shared__ int red[4];
    __shared__ int red9[(NT / 64) * 9];
    const int c = blockIdx.x, chunk = blockIdx.y;
    const int IHW = a.IH * a.IW, OHW = a.OH * a.OW, RS = a.R * a.S;
    const int n0 = (int)(((long long)a.N * chunk) / a.chunks);
    const int n1 = (int)(((long long)a.N * (chunk + 1)) / a.chunks);
    int32_t* __restrict__ part = a.partial + ((size_t)chunk * a.C + c) * RS;

    if (a.R == 3 && a.S == 3) {
        // common case: both planes staged in LDS, all nine taps in registers
        int8_t* xs = lds;                       // a plane   (IH x IW)
        int8_t* gs = lds + ((IHW + 15) & ~15);  // g_z plane (OH x OW)
        int acc9[9];
#pragma unroll
        for (int i = 0; i < 9; ++i) acc9[i] = 0;
        for (int n = n0; n < n1; ++n) {
            const int8_t* __restrict__ xsrc = a.a + ((size_t)n * a.C + c) * IHW;
            const int8_t* __restrict__ gsrc = a.b + ((size_t)n * a.C + c) * OHW;
            __syncthreads();
            // (planes of whole 16-byte chunks -- the planes are 16-byte aligned then -- move as such: a 112 x 112 plane
            // was 49 rounds of single-byte loads)
            if ((IHW & 15) == 0) {
                for (int i = threadIdx.x; i < (IHW >> 4); i += NT) reinterpret_cast<uint4*>(xs)[i] = reinterpret_cast<const uint4*>(xsrc)[i];
            } else {
                for (int i = threadIdx.x; i < IHW; i += NT) xs[i] = xsrc[i];
            }
            if ((OHW & 15) == 0) {
                for (int i = threadIdx.x; i < (OHW >> 4); i += NT) reinterpret_cast<uint4*>(gs)[i] = reinterpret_cast<const uint4*>(gsrc)[i];
            } else {
                for (int i = threadIdx.x; i < OHW; i += NT) gs[i] = gsrc[i];
            }
            __syncthreads();
            for (int o = threadIdx.x; o < OHW; o += NT) {
                const int p = o / a.OW, q = o - p * a.OW;
                const int g = (int)gs[o];
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const int ih = p * a.stride_h - a.pad_h + r;
#pragma unroll
                    for (int s = 0; s < 3; ++s) {
                        const int iw = q * a.stride_w - a.pad_w + s;
                        if ((unsigned)ih < (unsigned)a.IH && (unsigned)iw < (unsigned)a.IW)
                            acc9[r * 3 + s] += g * (int)xs[ih * a.IW + iw];
                    }
                }
            }
        }
        dw_block_sums_store<NT, 9>(acc9, red9, part);
    } else {
        // other filter sizes: one tap at a time, straight from global memory
        for (int rs = 0; rs < RS; ++rs) {
            const int r = rs / a.S, s = rs - r * a.S;
            int v = 0;
            for (int n = n0; n < n1; ++n) {
                const int8_t* __restrict__ xsrc = a.a + ((size_t)n * a.C + c) * IHW;
                const int8_t* __restrict__ gsrc = a.b + ((size_t)n * a.C + c) * OHW;
                for (int o = threadIdx.x; o < OHW; o += NT) {
                    const int p = o / a.OW, q = o - p * a.OW;
                    const int ih = p * a.stride_h - a.pad_h + r, iw = q * a.stride_w - a.pad_w + s;
                    if ((unsigned)ih < (unsigned)a.IH && (unsigned)iw < (unsigned)a.IW)
                        v += (int)gsrc[o] * (int)xsrc[ih * a.IW + iw];
                }
            }
            dw_block_sum_store<NT>(v, red, part + rs);
        }
    }
}

// Stride-1 fast path of the backward-weight pass for R x S known at compile time: both planes in
// LDS (the input with its zero border, so that tap (r,s) of output column q starts at LDS column
// q + s), a thread owns four consecutive outputs of a row and adds, per tap, one 4-way int8 dot
// product of the four gradient codes with the four input codes they meet.
// PF: the planes are whole 16-byte chunks, at most 256 of them (host: dw_wgrad_prefetch()): the next image's
// planes are fetched into registers while this image's dot products run.  A template flag, so that the
// other instantiations do not carry the registers (64-thread blocks on 7 x 7 planes fell from many to two
// waves per SIMD when it was a run-time choice).
// OFF: the input plane is staged OFF bytes further right than its padding asks (OFF = 4 - pad_w for rows of whole
// dwords, else 0), so that its rows start on a dword of LDS and are written four bytes at a time: the byte-by-byte
// scatter was most of this kernel's vector-ALU work.  Tap s of output column q then starts at LDS column q + OFF + s.
// ST = 2: the four gradient codes of a task meet input codes two bytes apart (LDS row 2 p + r, columns 2 q + OFF + s + 2 j):
// the seven bytes they span are cut out of the row's dwords by two byte-aligns and every other one picked by a byte
// permute -- three instructions and a dot product per tap and four results, where the generic kernel spends some
// seven per product on index arithmetic and bounds tests (96 channels at 112 x 112, batch 64: 62 us, compute-bound).
template <int R, int S, int NT, bool PF, int OFF, int ST = 1>
__global__ __launch_bounds__(NT) void dw_wgrad_fast_kernel(const DwArgs a, int pitch, int gpitch, int xrows) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    __shared__ int red[(NT / 64) * R * S];
    constexpr int SD = (S + 3) / 4;
    const int c = blockIdx.x, chunk = blockIdx.y;
    const int IHW = a.IH * a.IW, OHW = a.OH * a.OW;
    const int n0 = (int)(((long long)a.N * chunk) / a.chunks);
    const int n1 = (int)(((long long)a.N * (chunk + 1)) / a.chunks);
    int32_t* __restrict__ part = a.partial + ((size_t)chunk * a.C + c) * (R * S);
    int8_t* xs = lds;                                   // xrows x pitch (stride 1: OH + R - 1 rows), zero border
    int8_t* gs = lds + ((xrows * pitch + 15) & ~15);    // OH x gpitch, zero tail columns
    {
        const int ndw = (((xrows * pitch + 15) & ~15) + a.OH * gpitch) >> 2;
        for (int i = threadIdx.x; i < ndw; i += NT) reinterpret_cast<uint32_t*>(lds)[i] = 0u;
    }
    int acc[R][S];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int sx = 0; sx < S; ++sx) acc[r][sx] = 0;
    const int QW = (a.OW + 3) >> 2;
    // Planes of whole 16-byte chunks, at most 256 of them (DW_PF per thread): the next image's two planes are fetched
    // into registers while this image's dot products run (a block otherwise waits out a round trip to memory
    // per image: 56 x 56 planes, 144 channels, batch 64: 37.8 us of which little is arithmetic).
    constexpr int DW_PF = PF ? 256 / NT : 1;      // planes of up to 4 KB
    constexpr bool pf = PF;
    uint4 px[DW_PF], pg[DW_PF];
    if (pf && n0 < n1) {
        dw_plane_fetch<NT, DW_PF>(a.a + ((size_t)n0 * a.C + c) * IHW, IHW, px);
        dw_plane_fetch<NT, DW_PF>(a.b + ((size_t)n0 * a.C + c) * OHW, OHW, pg);
    }
    for (int n = n0; n < n1; ++n) {
        const int8_t* __restrict__ xsrc = a.a + ((size_t)n * a.C + c) * IHW;
        const int8_t* __restrict__ gsrc = a.b + ((size_t)n * a.C + c) * OHW;
        __syncthreads();   // the previous image's reads (and the zero fill) are done
        if (pf) {
            dw_plane_store<NT, DW_PF>(px, IHW, a.IW, xs, pitch, a.pad_h, a.pad_w + OFF);
            dw_plane_store<NT, DW_PF>(pg, OHW, a.OW, gs, gpitch, 0, 0);
        } else {
            dw_fill_plane<NT>(xsrc, a.IH, a.IW, xs, pitch, a.pad_h, a.pad_w + OFF);
            dw_fill_plane<NT>(gsrc, a.OH, a.OW, gs, gpitch, 0, 0);
        }
        __syncthreads();
        if (pf && n + 1 < n1) {
            dw_plane_fetch<NT, DW_PF>(xsrc + (size_t)a.C * IHW, IHW, px);
            dw_plane_fetch<NT, DW_PF>(gsrc + (size_t)a.C * OHW, OHW, pg);
        }
        for (int t = threadIdx.x; t < a.OH * QW; t += NT) {
            const int p = t / QW, q = (t - p * QW) << 2;
            const int g4 = *reinterpret_cast<const int*>(gs + p * gpitch + q);
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const uint32_t* __restrict__ rowp = reinterpret_cast<const uint32_t*>(xs + (ST * p + r) * pitch + ST * q);
                constexpr int ND = ST == 2 ? 4 : ((OFF + S - 1) >> 2) + 2;      // dwords that hold the windows of the four outputs
                static_assert(ST == 1 || ((OFF + S - 1) >> 2) + 2 <= 3, "stride 2: the windows end inside the fourth dword");
                uint32_t d[ND];
#pragma unroll
                for (int k = 0; k < ND; ++k) d[k] = rowp[k];
#pragma unroll
                for (int sx = 0; sx < S; ++sx) {
                    const int o = OFF + sx;
                    uint32_t win;
                    if (ST == 1) {
                        win = (o & 3) == 0 ? d[o >> 2] : __builtin_amdgcn_alignbyte(d[(o >> 2) + 1], d[o >> 2], o & 3);
                    } else {
                        const int k0 = o >> 2, sh = o & 3;
                        const uint32_t lo = sh == 0 ? d[k0] : __builtin_amdgcn_alignbyte(d[k0 + 1], d[k0], sh);          // bytes o .. o + 3
                        const uint32_t hi = sh == 0 ? d[k0 + 1] : __builtin_amdgcn_alignbyte(d[k0 + 2], d[k0 + 1], sh);  // bytes o + 4 .. o + 7
                        win = __builtin_amdgcn_perm(hi, lo, 0x06040200u);                                                // bytes o, o + 2, o + 4, o + 6
                    }
                    acc[r][sx] = __builtin_amdgcn_sdot4((int)win, g4, acc[r][sx], false);
                }
            }
        }
    }
    int flat[R * S];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int sx = 0; sx < S; ++sx) flat[r * S + sx] = acc[r][sx];
    dw_block_sums_store<NT, R * S>(flat, red, part);
}

// Stride-1 backward-weight for small planes (14 x 14, 7 x 7): a block takes `cg` consecutive channels -- their planes
// are one contiguous run of cg * IH * IW bytes per image -- and a share of the images; every thread owns one task (four
// gradient codes of a row) of one channel for all images, the run of the next image is fetched into registers while
// these images' dot products run (several images are staged per pass, see below); a channel's tasks sit in a group of `slot` lanes (a power of two, at most a wave), so
// that its tap sums are reduced by lane exchanges (LDS atomics of 56 lanes on one address took longer than the pass).  With a block per
// channel these planes are no whole 16-byte chunks (196, 49 bytes): each image cost eight memory round trips of
// single-byte loads (384 channels at 14 x 14, batch 64: 23.7 us for 9.6 MB).
// Host (dw_wgrad_shape): OH * ceil(OW / 4) <= slot <= 64, cg * slot <= 256 threads, cg * IH * IW and cg * OH * OW whole
// 16-byte chunks and at most 512 of them together, cg <= 32 and a divisor of C.
template <int R, int S>
__global__ __launch_bounds__(256) void dw_wgrad_group_kernel(const DwArgs a, int pitch, int gpitch, int slot, int ni) {
    constexpr int NT = 256, SD = (S + 3) / 4, RS = R * S;
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    __shared__ int red[32 * RS];
    const int cg = a.cg, c0 = blockIdx.x * cg, chunk = blockIdx.y;
    const int IHW = a.IH * a.IW, OHW = a.OH * a.OW;
    const int n0 = (int)(((long long)a.N * chunk) / a.chunks);
    const int n1 = (int)(((long long)a.N * (chunk + 1)) / a.chunks);
    const int xsize = ((a.OH + R - 1) * pitch + 15) & ~15, gsize = (a.OH * gpitch + 15) & ~15;
    const int isize = cg * (xsize + gsize);                 // one image: cg input planes with zero borders, then cg gradient planes
    for (int i = threadIdx.x; i < (ni * isize) >> 2; i += NT) reinterpret_cast<uint32_t*>(lds)[i] = 0u;
    // `ni` images are staged per pass: their 2 * ni runs are ni * (nchx + nchg) chunks, at most two per thread
    // (host), so that every thread takes part in the staging and a pass costs one memory round trip, not ni
    const int nchx = (cg * IHW) >> 4, nchg = (cg * OHW) >> 4, nch = nchx + nchg;
    const float inv_nch = 1.0f / (float)nch;
    const int QW = (a.OW + 3) >> 2, per = a.OH * QW;
    const int pl_raw = (int)threadIdx.x / slot, tt_raw = (int)threadIdx.x - pl_raw * slot;
    const bool active = pl_raw < cg && tt_raw < per;
    const int pl = active ? pl_raw : 0, tt = active ? tt_raw : 0;
    const int p = tt / QW, q = (tt - p * QW) << 2;
    int acc[R][S];
#pragma unroll
    for (int r = 0; r < R; ++r)
#pragma unroll
        for (int sx = 0; sx < S; ++sx) acc[r][sx] = 0;
    // chunk e of a pass that starts at image n: image n + e / nch, input chunk e % nch or gradient chunk e % nch - nchx
    int ej[2], ei[2];
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int e = (int)threadIdx.x + u * NT;
        ej[u] = dw_div_small(e, inv_nch);
        ei[u] = e - ej[u] * nch;
    }
    uint4 regs[2];
    auto fetch = [&](int n) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            const bool ok = ej[u] < ni && n + ej[u] < n1;
            const size_t img = (size_t)(n + (ok ? ej[u] : 0)) * a.C + c0;
            const uint4* src = ei[u] < nchx ? reinterpret_cast<const uint4*>(a.a + img * IHW) + ei[u]
                                            : reinterpret_cast<const uint4*>(a.b + img * OHW) + (ei[u] - nchx);
            regs[u] = *src;        // (unconditional: a chunk of the pass's first image when there is none; not stored)
        }
    };
    if (n0 < n1) fetch(n0);
    for (int n = n0; n < n1; n += ni) {
        const int cnt = n1 - n < ni ? n1 - n : ni;
        __syncthreads();   // the previous pass's reads (and the zero fill) are done
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            if (ej[u] < cnt) {
                int8_t* base = lds + ej[u] * isize;
                if (ei[u] < nchx) dw_scatter_chunk(regs[u], ei[u], a.IH, a.IW, IHW, base, xsize, pitch, a.pad_h, a.pad_w);
                else dw_scatter_chunk(regs[u], ei[u] - nchx, a.OH, a.OW, OHW, base + cg * xsize, gsize, gpitch, 0, 0);
            }
        }
        __syncthreads();
        if (n + ni < n1) fetch(n + ni);
        if (active) {
            for (int j = 0; j < cnt; ++j) {
                const int8_t* __restrict__ xs = lds + j * isize;
                const int8_t* __restrict__ gs = xs + cg * xsize;
                const int g4 = *reinterpret_cast<const int*>(gs + pl * gsize + p * gpitch + q);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    const uint32_t* __restrict__ rowp = reinterpret_cast<const uint32_t*>(xs + pl * xsize + (p + r) * pitch + q);
                    uint32_t d[SD + 1];
#pragma unroll
                    for (int k = 0; k <= SD; ++k) d[k] = rowp[k];
#pragma unroll
                    for (int sx = 0; sx < S; ++sx) {
                        const uint32_t win = (sx & 3) == 0 ? d[sx >> 2] : __builtin_amdgcn_alignbyte(d[(sx >> 2) + 1], d[sx >> 2], sx & 3);
                        acc[r][sx] = __builtin_amdgcn_sdot4((int)win, g4, acc[r][sx], false);
                    }
                }
            }
        }
    }
    // sums over the lanes of a channel's group (inactive lanes hold zeros); its first lane leaves them in LDS
    // (all R*S exchanges of a step are independent of each other: one LDS round trip per step, not per value)
    for (int o = slot >> 1; o > 0; o >>= 1) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int sx = 0; sx < S; ++sx) acc[r][sx] += __shfl_xor(acc[r][sx], o, kWave);
    }
    if (tt_raw == 0 && pl_raw < cg) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int sx = 0; sx < S; ++sx) red[pl_raw * RS + r * S + sx] = acc[r][sx];
    }
    __syncthreads();
    // [chunk][C][R*S]: the group's channels are consecutive
    for (int i = threadIdx.x; i < cg * RS; i += NT) a.partial[((size_t)chunk * a.C + c0) * RS + i] = red[i];
}

// 16 lanes per result: each adds every 16th share, then the lanes are summed (integer sums: any order is exact).
// With one thread per result a layer of 32 channels and 64 shares was one block walking 64 dependent loads: 15.5 us.
__global__ __launch_bounds__(256) void dw_wgrad_reduce_kernel(const DwArgs a) {
    const int RS = a.R * a.S;
    const int total = a.C * RS;
    const int t = (blockIdx.x * 256 + threadIdx.x) >> 4, sub = threadIdx.x & 15;
    int sum = 0;
    if (t < total)
        for (int z = sub; z < a.chunks; z += 16) sum += a.partial[(size_t)z * total + t];
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, kWave);
    if (t < total && sub == 0) {
        a.out[t] = __fmul_rn((float)sum, __fmul_rn(a.sa[0], a.sb[0]));
        if (a.acc) a.acc[t] = sum;
    }
}

// Threads per block of the depthwise kernels: a plane of OH x OW results is OH * ceil(OW / 4) tasks in
// the stride-1 kernels (one per result in the others).  A 7 x 7 or 14 x 14 plane keeps one wave
// busy, not four: small planes get small blocks, and a compute unit holds as many more of them.
int dw_threads(int OH, int OW, bool quads) {
    const long long tasks = (long long)OH * (quads ? (OW + 3) / 4 : OW);
    return tasks <= 64 ? 64 : tasks <= 128 ? 128 : 256;
}

// Blocks = C x chunks; 32 waves fit a compute unit: at most 2048 blocks of four waves run at once,
// and a grid just above that (144 channels x 15 chunks = 2160) would take two rounds for 5 % more blocks.
int dw_wgrad_chunks(int N, int C, int threads) {
    int chunks = 2048 * (256 / threads) / C;
    if (chunks > N) chunks = N;
    if (chunks < 1) chunks = 1;
    return chunks;
}

static int dw_fast_pitch(int OW, int S);

// lanes per channel in dw_wgrad_group_kernel: the tasks of a gradient plane, rounded up to a power of two
static int dw_wgrad_slot(int P, int Q) {
    const int per = P * ((Q + 3) / 4);
    int slot = 4;
    while (slot < per) slot *= 2;
    return slot;
}

// consecutive channels per block of dw_wgrad_group_kernel, 1 where it does not apply
static int dw_wgrad_group(int C, int IH, int IW, int P, int Q, int R, int S, int stride_h, int stride_w) {
    if (stride_h != 1 || stride_w != 1 || R != S || (R != 3 && R != 5)) return 1;
    const int per = P * ((Q + 3) / 4);
    if (per > 64) return 1;
    int cg = 256 / dw_wgrad_slot(P, Q);
    if (cg > 32) cg = 32;
    const int ihw = IH * IW, ohw = P * Q;
    int m = 16;                          // smallest count that makes both runs whole 16-byte chunks
    for (int g = ihw | ohw; m > 1 && g % 2 == 0; g /= 2) m /= 2;
    cg = cg / m * m;
    while (cg >= 2 && C % cg != 0) cg -= m;
    if (cg < 2) return 1;
    const size_t lds = (size_t)cg * ((((size_t)(P + R - 1) * dw_fast_pitch(Q, S) + 15) & ~(size_t)15) + (((size_t)P * ((Q + 3) & ~3) + 15) & ~(size_t)15));
    if (lds > 32 * 1024 || (size_t)cg * (ihw + ohw) > 8192) return 1;      // (at most 512 chunks per image: two per thread)
    return cg;
}

void dw_wgrad_shape(int N, int C, int IH, int IW, int P, int Q, int R, int S, int stride_h, int stride_w,
                    int* threads, int* chunks, int* cg) {
    *cg = dw_wgrad_group(C, IH, IW, P, Q, R, S, stride_h, stride_w);
    if (*cg > 1) {
        // about 1024 blocks of four waves: a block's fixed cost (staging set-up, the lane exchanges of its sums, its
        // partial results) is paid once per share, and more shares than resident blocks add whole rounds of it
        *threads = 256;
        int ch = 1024 / (C / *cg);
        *chunks = ch > N ? N : ch < 1 ? 1 : ch;
    } else {
        *threads = dw_wgrad_threads(P, Q, R, S, stride_h, stride_w);
        *chunks = dw_wgrad_chunks(N, C, *threads);
    }
}

// LDS row pitch of the fast path: the widest row read starts at column OW - 1 rounded down to 4 and
// takes 4 * (SD + 1) bytes
static int dw_fast_pitch(int OW, int S) {
    const int sd = (S + 3) / 4;
    return (((OW + 3) & ~3) + 4 * sd + 3) & ~3;
}

// Planes per block of the fast path: enough for about 256 tasks (four results of a row each) and, beyond that, for
// the whole grid to be resident at once (2048 blocks of four waves: every block's loads are then on their way from
// the start, instead of a second and third round of blocks each waiting out its own memory latency); a count that
// makes the block's source bytes a whole number of 16-byte chunks where one of at most DW_MAX_PPB exists; at most
// 48 KB of staged planes.
static int dw_fast_ppb(int NC, int OH, int OW, int IH, int IW, size_t plane_lds) {
    const int per = OH * ((OW + 3) / 4);
    int ppb = (256 + per - 1) / per;
    if (ppb > 1 || per < 512) {
        const int resident = (NC + 2047) / 2048;
        if (ppb < resident) ppb = resident;
    }
    if (ppb > DW_MAX_PPB) ppb = DW_MAX_PPB;
    int g = IH * IW;                     // 16 / gcd(IH * IW, 16): planes per whole chunk run
    int m = 16;
    while (m > 1 && g % 2 == 0) { g /= 2; m /= 2; }
    if (ppb > 1 && m <= DW_MAX_PPB) ppb = (ppb + m - 1) / m * m;
    if (ppb > DW_MAX_PPB) ppb = DW_MAX_PPB;
    while (ppb > 1 && (size_t)ppb * plane_lds > 48 * 1024) --ppb;
    return ppb;
}
static int dw_fast_threads(int OH, int OW, int ppb) {
    const long long tasks = (long long)ppb * OH * ((OW + 3) / 4);
    return tasks <= 64 ? 64 : tasks <= 128 ? 128 : 256;
}

hipError_t launch_dw_conv(const DwArgs& a, hipStream_t st) {
    KernelTimer kt(KID_DW_CONV, st);
    if (a.dgrad && a.stride_h == 2 && a.stride_w == 2 && a.R == a.S && (a.R == 3 || a.R == 5)) {
        // backward-data at stride 2: gradient plane (IH x IW) at (TB, LB) in an area that reaches as far
        // as the taps of the last pixels do
        const int TB = (a.R - 1) / 2, LB = (a.S - 1) / 2;
        int rows = ((a.OH - 1 + a.pad_h) >> 1) + TB + 1;
        if (rows < TB + a.IH) rows = TB + a.IH;
        int pitch = ((4 * ((a.OW + 3) / 4 - 1) + a.pad_w) >> 1) + LB + 3;
        if (pitch < LB + a.IW) pitch = LB + a.IW;
        pitch = (pitch + 3) & ~3;
        const size_t lds = (size_t)rows * pitch;
        if (lds <= 60 * 1024) {
            const int nt = dw_threads(a.OH, a.OW, true);
#define DG2(Rv)                                                                                                        \
    do {                                                                                                               \
        if (nt == 64) launch_timed(kt, (dw_dgrad_s2_kernel<Rv, Rv, 64>), dim3(a.N * a.C), dim3(64), lds, st, a, pitch, rows);        \
        else if (nt == 128) launch_timed(kt, (dw_dgrad_s2_kernel<Rv, Rv, 128>), dim3(a.N * a.C), dim3(128), lds, st, a, pitch, rows); \
        else launch_timed(kt, (dw_dgrad_s2_kernel<Rv, Rv, 256>), dim3(a.N * a.C), dim3(256), lds, st, a, pitch, rows);               \
    } while (0)
            if (a.R == 3) DG2(3); else DG2(5);
#undef DG2
            return hipGetLastError();
        }
    }
    if (!a.dgrad && a.stride_h == 2 && a.stride_w == 2 && a.S <= 8 && a.R <= DW_FAST_MAXR) {
        // forward at stride 2: the staged area holds the plane with its top / left border and reaches as
        // far as the last output's window does (four outputs per thread: 8 * ceil(OW / 4) columns + the
        // dwords of one row segment)
        const int sd = (a.S + 3) / 4;
        int pitch = 8 * ((a.OW + 3) / 4) + 4 * (sd + 2);
        if (pitch < a.pad_w + a.IW) pitch = a.pad_w + a.IW;
        pitch = (pitch + 3) & ~3;
        if (pitch < a.pad_w + 3 + a.IW) pitch = (a.pad_w + 3 + a.IW + 3) & ~3;      // (room for the dword-aligned staging)
        int rows = 2 * (a.OH - 1) + a.R;
        if (rows < a.pad_h + a.IH) rows = a.pad_h + a.IH;
        const size_t lds1 = (size_t)rows * pitch;
        if (lds1 <= 60 * 1024) {
            const int ppb = dw_fast_ppb(a.N * a.C, a.OH, a.OW, a.IH, a.IW, lds1), nt = dw_fast_threads(a.OH, a.OW, ppb);
            const size_t lds = lds1 * ppb;
            const dim3 grid((unsigned)((a.N * a.C + ppb - 1) / ppb));
            // rows of whole dwords, a border of 1 (3-wide) or 2 (5-wide) columns: staged from a dword boundary
            const bool al = (a.IW & 3) == 0 && a.pad_w == (sd == 1 ? 1 : 2);
#define FAST2(SDv, OFFv)                                                                                                       \
    do {                                                                                                                 \
        if (nt == 64) launch_timed(kt, (dw_conv_fast_kernel<false, SDv, 64, 2, OFFv>), grid, dim3(64), lds, st, a, pitch, rows, ppb);        \
        else if (nt == 128) launch_timed(kt, (dw_conv_fast_kernel<false, SDv, 128, 2, OFFv>), grid, dim3(128), lds, st, a, pitch, rows, ppb); \
        else launch_timed(kt, (dw_conv_fast_kernel<false, SDv, 256, 2, OFFv>), grid, dim3(256), lds, st, a, pitch, rows, ppb);               \
    } while (0)
            if (a.S > 4) { if (al) FAST2(2, 2); else FAST2(2, 0); }
            else { if (al) FAST2(1, 3); else FAST2(1, 0); }
#undef FAST2
            return hipGetLastError();
        }
    }
    if (a.stride_h == 1 && a.stride_w == 1 && a.S <= 8 && a.R <= DW_FAST_MAXR &&
        (a.dgrad ? (a.pad_h <= a.R - 1 && a.pad_w <= a.S - 1) : true)) {
        const int pitch = dw_fast_pitch(a.OW, a.S) + 4;      // (+ 4: room for the dword-aligned staging)
        const size_t lds1 = (size_t)(a.OH + a.R - 1) * pitch;
        if (lds1 <= 60 * 1024) {
            const bool two = a.S > 4;
            const int ppb = dw_fast_ppb(a.N * a.C, a.OH, a.OW, a.IH, a.IW, lds1), nt = dw_fast_threads(a.OH, a.OW, ppb);
            const size_t lds = lds1 * ppb;
            const dim3 grid((unsigned)((a.N * a.C + ppb - 1) / ppb));
            // rows of whole dwords, a border of 1 (up to 4 wide) or 2 (wider) columns: staged from a dword boundary
            const int left = a.dgrad ? (a.S - 1 - a.pad_w) : a.pad_w;
            const bool al = (a.IW & 3) == 0 && left == (two ? 2 : 1);
#define FAST(DG, SDv, OFFv)                                                                                              \
    do {                                                                                                           \
        if (nt == 64) launch_timed(kt, (dw_conv_fast_kernel<DG, SDv, 64, 1, OFFv>), grid, dim3(64), lds, st, a, pitch, a.OH + a.R - 1, ppb);        \
        else if (nt == 128) launch_timed(kt, (dw_conv_fast_kernel<DG, SDv, 128, 1, OFFv>), grid, dim3(128), lds, st, a, pitch, a.OH + a.R - 1, ppb); \
        else launch_timed(kt, (dw_conv_fast_kernel<DG, SDv, 256, 1, OFFv>), grid, dim3(256), lds, st, a, pitch, a.OH + a.R - 1, ppb);               \
    } while (0)
            if (a.dgrad) {
                if (two) { if (al) FAST(true, 2, 2); else FAST(true, 2, 0); }
                else { if (al) FAST(true, 1, 3); else FAST(true, 1, 0); }
            } else {
                if (two) { if (al) FAST(false, 2, 2); else FAST(false, 2, 0); }
                else { if (al) FAST(false, 1, 3); else FAST(false, 1, 0); }
            }
#undef FAST
            return hipGetLastError();
        }
    }
    const size_t lds = ((size_t)a.IH * a.IW + 15) & ~(size_t)15;
    const int nt = dw_threads(a.OH, a.OW, false);
    const bool s2 = a.stride_h == 2 && a.stride_w == 2;
#define GEN(DG, STv)                                                                                      \
    do {                                                                                                  \
        if (nt == 64) launch_timed(kt, (dw_conv_kernel<DG, STv, 64>), dim3(a.N * a.C), dim3(64), lds, st, a);        \
        else if (nt == 128) launch_timed(kt, (dw_conv_kernel<DG, STv, 128>), dim3(a.N * a.C), dim3(128), lds, st, a); \
        else launch_timed(kt, (dw_conv_kernel<DG, STv, 256>), dim3(a.N * a.C), dim3(256), lds, st, a);               \
    } while (0)
    if (a.dgrad) {
        if (s2) GEN(true, 2); else GEN(true, 0);
    } else {
        if (s2) GEN(false, 2); else GEN(false, 0);
    }
#undef GEN
    return hipGetLastError();
}

// block size of the backward-weight pass: its tasks are the gradient plane's results, in quads on the stride-1 path
int dw_wgrad_threads(int P, int Q, int R, int S, int stride_h, int stride_w) {
    const bool fast = stride_h == stride_w && (stride_h == 1 || stride_h == 2) && R == S && (R == 3 || R == 5);
    return dw_threads(P, Q, fast);
}

hipError_t launch_dw_wgrad(const DwArgs& a, hipStream_t st) {
    {
        KernelTimer kt(KID_DW_WGRAD, st);
        bool fast = false;
        if (a.cg > 1) {
            const int pitch = dw_fast_pitch(a.OW, a.S), gpitch = (a.OW + 3) & ~3;
            const size_t ldsg = (size_t)a.cg * ((((size_t)(a.OH + a.R - 1) * pitch + 15) & ~(size_t)15) + (((size_t)a.OH * gpitch + 15) & ~(size_t)15));
            const dim3 grid((unsigned)(a.C / a.cg), (unsigned)a.chunks);
            const int slot = dw_wgrad_slot(a.OH, a.OW);
            // images staged per pass: as many as two chunks per thread and 32 KB of LDS hold, at most 8
            const int nch = (a.cg * a.IH * a.IW + a.cg * a.OH * a.OW) >> 4;
            int ni = 512 / nch;
            if (ni > 8) ni = 8;
            while (ni > 1 && (size_t)ni * ldsg > 32 * 1024) --ni;
            if (ni < 1) ni = 1;
            if (a.R == 3) launch_timed(kt, (dw_wgrad_group_kernel<3, 3>), grid, dim3(256), ldsg * ni, st, a, pitch, gpitch, slot, ni);
            else launch_timed(kt, (dw_wgrad_group_kernel<5, 5>), grid, dim3(256), ldsg * ni, st, a, pitch, gpitch, slot, ni);
            fast = true;
        } else if (a.stride_h == a.stride_w && (a.stride_h == 1 || a.stride_h == 2) && a.R == a.S && (a.R == 3 || a.R == 5)) {
            // here IH x IW is the input plane and OH x OW the gradient plane
            // rows of whole dwords under "same" padding: staged from a dword boundary (OFF = 4 - pad_w, one more dword per row)
            const int stv = a.stride_h;
            const bool al = (a.IW & 3) == 0 && a.pad_w == a.S / 2 && a.pad_w > 0;
            const int off = al ? 4 - a.pad_w : 0;
            const int gpitch = (a.OW + 3) & ~3;
            int pitch, xrows;
            if (stv == 1) {
                pitch = dw_fast_pitch(a.OW, a.S) + (al ? 4 : 0);
                xrows = a.OH + a.R - 1;
            } else {
                // a task reads 16 bytes of row 2 p + r from column 2 q, q < OW rounded up to 4
                pitch = 2 * (gpitch - 4) + 16;
                if (pitch < a.pad_w + off + a.IW) pitch = a.pad_w + off + a.IW;
                pitch = (pitch + 3) & ~3;
                xrows = 2 * (a.OH - 1) + a.R;
                if (xrows < a.pad_h + a.IH) xrows = a.pad_h + a.IH;
            }
            const size_t ldsf = (((size_t)xrows * pitch + 15) & ~(size_t)15) + (size_t)a.OH * gpitch;
            // (stride 2 without the dword-aligned staging would need its own instantiations: the generic kernel serves it)
            if (ldsf <= 60 * 1024 && (stv == 1 || al)) {
                fast = true;
#define WFAST(Rv, PFv, OFFv, STv)                                                                                                \
    do {                                                                                                            \
        if (a.threads == 64) launch_timed(kt, (dw_wgrad_fast_kernel<Rv, Rv, 64, PFv, OFFv, STv>), dim3(a.C, a.chunks), dim3(64), ldsf, st, a, pitch, gpitch, xrows);        \
        else if (a.threads == 128) launch_timed(kt, (dw_wgrad_fast_kernel<Rv, Rv, 128, PFv, OFFv, STv>), dim3(a.C, a.chunks), dim3(128), ldsf, st, a, pitch, gpitch, xrows); \
        else launch_timed(kt, (dw_wgrad_fast_kernel<Rv, Rv, 256, PFv, OFFv, STv>), dim3(a.C, a.chunks), dim3(256), ldsf, st, a, pitch, gpitch, xrows);                      \
    } while (0)
                const int ihw = a.IH * a.IW, ohw = a.OH * a.OW;
                const bool pf = (ihw & 15) == 0 && (ohw & 15) == 0 && ihw <= 4096 && ohw <= 4096;
                if (stv == 2) {
                    if (a.R == 3) { if (pf) WFAST(3, true, 3, 2); else WFAST(3, false, 3, 2); }
                    else { if (pf) WFAST(5, true, 2, 2); else WFAST(5, false, 2, 2); }
                } else if (a.R == 3) {
                    if (pf) { if (al) WFAST(3, true, 3, 1); else WFAST(3, true, 0, 1); }
                    else { if (al) WFAST(3, false, 3, 1); else WFAST(3, false, 0, 1); }
                } else {
                    if (pf) { if (al) WFAST(5, true, 2, 1); else WFAST(5, true, 0, 1); }
                    else { if (al) WFAST(5, false, 2, 1); else WFAST(5, false, 0, 1); }
                }
#undef WFAST
            }
        }
        if (!fast) {
            const size_t lds = (((size_t)a.IH * a.IW + 15) & ~(size_t)15) + (((size_t)a.OH * a.OW + 15) & ~(size_t)15);
            if (a.threads == 64) launch_timed(kt, dw_wgrad_kernel<64>, dim3(a.C, a.chunks), dim3(64), lds, st, a);
            else if (a.threads == 128) launch_timed(kt, dw_wgrad_kernel<128>, dim3(a.C, a.chunks), dim3(128), lds, st, a);
            else launch_timed(kt, dw_wgrad_kernel<256>, dim3(a.C, a.chunks), dim3(256), lds, st, a);
        }
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int total = a.C * a.R * a.S;
    { KernelTimer kt(KID_DW_WGRAD_REDUCE, st); launch_timed(kt, dw_wgrad_reduce_kernel, dim3((total * 16 + 255) / 256), dim3(256), 0, st, a); }
    return hipGetLastError();
}

}  // namespace int8t
