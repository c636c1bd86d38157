// Dense backward-weight convolution on int8 codes (Sec.3.4: g_W = g_z^T a), int8 MFMA with int32
// accumulation, Eq.2 fused into the final reduction.
//
// GEMM view:  D[k][(tap,c)] = sum over (n,p,q) of  Gz[(n,p,q)][k] * A[(n, p*sh+r-ph, q*sw+s-pw)][c]
// The reduction runs over images and output pixels, but the channels-last code tensors keep the
// channel innermost, while the MFMA wants 16 consecutive reduction bytes per lane.  Any order of
// the reduction index is as good as any other, so the 16 bytes of a lane are made 16 different
// IMAGES at one pixel: the loader fetches, for one pixel and four channels, one dword from each of
// 16 images, swaps the 4x4 byte blocks with byte permutes -- the "4x4 8-bit integer block
// transpose" of the paper's Suppl. "INT8 Convolution" -- and stores [pixel][channel][16 images]
// granules to LDS.  A filter tap is then just a different PIXEL of the staged input window, i.e. a
// different, always 16-byte aligned LDS row: no im2col buffer, no unaligned operand reads, zero
// padding is written once by the loader.
//
// One block owns an output tile of 64 filters x CT channels x TB taps and a share of the
// reduction (split-K over image groups and output-pixel tiles); it writes an int32 partial tile.
// A second kernel sums the partials (integer addition: exact in any order, hence deterministic),
// applies Eq.2 and scatters [k][(tap,c)] to the K,C,R,S result.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int W2_BM = 64;              // filters per block
constexpr int W2_LDS_BUDGET = 64 * 1024;
constexpr int W2_TARGET_BLOCKS = 512;  // about two blocks per compute unit
constexpr int W2_TPT = 3;              // loader tasks per thread and reduction chunk (prefetched in registers)

// 4x4 byte transpose: in d[i] = 4 channels of image i; out o[c] = channel c of images 0..3.
__device__ __forceinline__ void transpose4x4(const uint32_t d[4], uint32_t o[4]) {
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

// Position of channel c inside a [channel][16 bytes] LDS row block.  MFMA operand reads walk 32
// consecutive channels, the loader's stores walk channels with a stride of four; the xor keeps
// both spread over all bank groups.
__device__ __forceinline__ int ch_slot(int c) { return c ^ ((c >> 3) & 3); }

// 16 images x 4 channels -> four [channel][16 images] granules.
__device__ __forceinline__ void transpose_store(const uint32_t d[16], uint4* __restrict__ row, int c4) {
    uint32_t o[4][4];
#pragma unroll
    for (int g = 0; g < 4; ++g) transpose4x4(d + 4 * g, o[g]);
#pragma unroll
    for (int j = 0; j < 4; ++j) row[ch_slot(c4 + j)] = make_uint4(o[0][j], o[1][j], o[2][j], o[3][j]);
}

// Extent of the taps [t0, t0+nt) of an R x S filter (taps numbered r*S + s).
__host__ __device__ inline void tap_extent(int t0, int nt, int S, int* rmin, int* rmax, int* smin, int* smax) {
    *rmin = t0 / S;
    *rmax = (t0 + nt - 1) / S;
    if (*rmin == *rmax) {
        *smin = t0 % S;
        *smax = (t0 + nt - 1) % S;
    } else {
        *smin = 0;
        *smax = S - 1;
    }
}

constexpr int W2_MAXSTEPS = 8;         // MFMA steps per chunk: at most 16 tile pixels

template <int TB, int CS>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradArgs a) {
    constexpr int CT = 64 * CS;   // channels per block
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    uint4* __restrict__ xT = lds;                   // [window pixel][CT channels] granules
    uint4* __restrict__ dyT = lds + a.xt_slots;     // [tile pixel][64 filters] granules, then one zero granule

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int mt = wave & 1, ch = wave >> 1, half = lane >> 5, l32 = lane & 31;

    int ot = blockIdx.x;
    const int tg = ot % a.tapgroups;
    ot /= a.tapgroups;
    const int ct = ot % a.ctiles;
    const int kt = ot / a.ctiles;
    const int RS = a.R * a.S;
    const int t0 = tg * TB;
    const int nt = (RS - t0 < TB) ? (RS - t0) : TB;
    int rmin, rmax, smin, smax;
    tap_extent(t0, nt, a.S, &rmin, &rmax, &smin, &smax);
    const int WH = (a.BP - 1) * a.stride_h + (rmax - rmin) + 1;
    const int WW = (a.BQ - 1) * a.stride_w + (smax - smin) + 1;
    int toff[TB];   // uniform: LDS offset of each tap inside the staged window
#pragma unroll
    for (int j = 0; j < TB; ++j) {
        const int t = t0 + ((j < nt) ? j : 0);
        toff[j] = __builtin_amdgcn_readfirstlane(((t / a.S - rmin) * WW + (t % a.S - smin)) * CT);
    }
    const int units = a.BP * a.BQ;
    const int nsteps = (units + 1) >> 1;
    const int zero_slot = units * W2_BM;            // in dyT
    if (tid == 0) dyT[zero_slot] = make_uint4(0, 0, 0, 0);

    // LDS operand positions of every MFMA step; they depend on the tile geometry only.  A step
    // feeds two tile pixels, one per half-wave, each with 16 images.
    int a_off[W2_MAXSTEPS], x_off[W2_MAXSTEPS];
#pragma unroll
    for (int s = 0; s < W2_MAXSTEPS; ++s) {
        const int u = 2 * s + half;
        const bool uv = u < units;
        const int uu = uv ? u : 0;
        const int pl = uu / a.BQ, ql = uu - pl * a.BQ;
        a_off[s] = uv ? (uu * W2_BM + ch_slot(mt * 32 + l32)) : zero_slot;
        x_off[s] = (pl * a.stride_h * WW + ql * a.stride_w) * CT + ch * CS * 32 + ch_slot(l32);
    }

    v16i acc[TB][CS];
#pragma unroll
    for (int j = 0; j < TB; ++j)
#pragma unroll
        for (int i = 0; i < CS; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0;

    const int c_begin = (int)(((long long)a.chunks * blockIdx.y) / gridDim.y);
    const int c_end = (int)(((long long)a.chunks * (blockIdx.y + 1)) / gridDim.y);
    const int tiles_per_group = a.ntp * a.ntq;
    const int ntask_x = WH * WW * (CT / 4);     // input window: (window pixel, channel quad)
    const int ntask = ntask_x + units * 16;     // + gradient tile: (tile pixel, filter quad)
    const uint32_t ximg = (uint32_t)a.H * a.W * a.Cp;     // image strides in bytes
    const uint32_t yimg = (uint32_t)a.P * a.Q * a.Kp;

    // Loader tasks of this thread (task = tid + 256*i): everything that does not depend on the
    // chunk is worked out once.  A task fetches one dword from each of 16 images.
    int t_kind[W2_TPT], t_c[W2_TPT], t_a[W2_TPT], t_b[W2_TPT], t_dst[W2_TPT];   // kind: 0 input, 1 gradient, 2 none
#pragma unroll
    for (int i = 0; i < W2_TPT; ++i) {
        const int task = tid + 256 * i;
        t_kind[i] = 2;
        t_a[i] = t_b[i] = t_c[i] = t_dst[i] = 0;
        if (task < ntask_x) {
            const int cq = task % (CT / 4), wp = task / (CT / 4);
            t_kind[i] = 0;
            t_a[i] = wp / WW;                 // window row
            t_b[i] = wp - t_a[i] * WW;        // window column
            t_c[i] = ct * CT + 4 * cq;        // >= Cp: nothing to fetch, zeros are staged
            t_dst[i] = wp * CT + 4 * cq;      // granule index in xT (before the channel swizzle)
        } else if (task < ntask) {
            const int kq = (task - ntask_x) & 15, u = (task - ntask_x) >> 4;
            t_kind[i] = 1;
            t_a[i] = u / a.BQ;                // tile row
            t_b[i] = u - t_a[i] * a.BQ;       // tile column
            t_c[i] = kt * W2_BM + 4 * kq;
            t_dst[i] = u * W2_BM + 4 * kq;
        }
    }

    // Prefetch registers.  Loads are unconditional: a task with nothing to fetch (padding, ragged
    // tile edge, channel beyond the tensor) reads offset 0 of its tensor and is zeroed when it is
    // staged; images beyond N re-read the group's last image and are zeroed the same way.
    uint32_t pre[W2_TPT][16];
    bool pre_ok[W2_TPT];
    int pre_nimg = 16;
    auto issue = [&](int chunk) {
        const int ng = chunk / tiles_per_group;
        const int trem = chunk - ng * tiles_per_group;
        const int tp = trem / a.ntq, tq = trem - tp * a.ntq;
        const int p0 = tp * a.BP, q0 = tq * a.BQ;
        const int ih0 = p0 * a.stride_h - a.pad_h + rmin, iw0 = q0 * a.stride_w - a.pad_w + smin;
        const int n0 = ng * 16;
        const int nimg = (a.N - n0 < 16) ? (a.N - n0) : 16;
        pre_nimg = nimg;
#pragma unroll
        for (int i = 0; i < W2_TPT; ++i) {
            if (t_kind[i] == 2) continue;
            const bool isx = t_kind[i] == 0;
            const int yy = (isx ? ih0 : p0) + t_a[i], xx = (isx ? iw0 : q0) + t_b[i];
            const int hh = isx ? a.H : a.P, ww = isx ? a.W : a.Q, cc = isx ? a.Cp : a.Kp;
            const bool ok = (unsigned)yy < (unsigned)hh && (unsigned)xx < (unsigned)ww && t_c[i] < cc;
            pre_ok[i] = ok;
            const uint32_t stride = isx ? ximg : yimg;
            const int8_t* base = isx ? a.x : a.dy;
            uint32_t off = ok ? (((uint32_t)n0 * hh + yy) * ww + xx) * cc + t_c[i] : (uint32_t)n0 * stride;
#pragma unroll
            for (int im = 0; im < 16; ++im) {
                pre[i][im] = *reinterpret_cast<const uint32_t*>(base + off);
                if (im + 1 < nimg) off += stride;
            }
        }
    };

    if (c_begin < c_end) issue(c_begin);
    for (int chunk = c_begin; chunk < c_end; ++chunk) {
        __syncthreads();   // the previous chunk's MFMA reads are done
#pragma unroll
        for (int i = 0; i < W2_TPT; ++i) {
            if (t_kind[i] == 2) continue;
            if (!pre_ok[i]) {
#pragma unroll
                for (int im = 0; im < 16; ++im) pre[i][im] = 0u;
            } else if (pre_nimg < 16) {
#pragma unroll
                for (int im = 0; im < 16; ++im)
                    if (im >= pre_nimg) pre[i][im] = 0u;
            }
            // t_dst = 64-granule row block + channel offset; the swizzle acts on the low bits only
            uint4* __restrict__ row = ((t_kind[i] == 1) ? dyT : xT) + (t_dst[i] & ~63);
            transpose_store(pre[i], row, t_dst[i] & 63);
        }
        __syncthreads();
        if (chunk + 1 < c_end) issue(chunk + 1);   // in flight while this chunk's MFMAs run

#pragma unroll
        for (int s = 0; s < W2_MAXSTEPS; ++s) {
            if (s < nsteps) {
                const uint4 ta = dyT[a_off[s]];
                const v4i fa = v4i{(int)ta.x, (int)ta.y, (int)ta.z, (int)ta.w};
#pragma unroll
                for (int j = 0; j < TB; ++j) {   // TB divides R*S: every tap of the group exists
#pragma unroll
                    for (int i = 0; i < CS; ++i) {
                        const uint4 tb = xT[x_off[s] + toff[j] + i * 32];
                        const v4i fb = v4i{(int)tb.x, (int)tb.y, (int)tb.z, (int)tb.w};
                        acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, acc[j][i], 0, 0, 0);
                    }
                }
            }
        }
    }

    // partial[z][k][(tap,c)], channel fastest: 32 consecutive columns per store instruction
    const int ncolsp = RS * a.Cp;
    int32_t* __restrict__ part = a.partial + (size_t)blockIdx.y * a.K * ncolsp;
#pragma unroll
    for (int j = 0; j < TB; ++j) {
        if (j >= nt) continue;
#pragma unroll
        for (int i = 0; i < CS; ++i) {
            const int c = ct * CT + (ch * CS + i) * 32 + l32;
            if (c >= a.Cp) continue;
            const int col = (t0 + j) * a.Cp + c;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kt * W2_BM + mt * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (k < a.K) part[(size_t)k * ncolsp + col] = acc[j][i][v];
            }
        }
    }
}

// Sum the split partials, apply Eq.2 and scatter [k][(r,s,c)] -> K,C,R,S.
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const WgradArgs a) {
    const int ncolsp = a.R * a.S * a.Cp;
    const size_t total = (size_t)a.K * ncolsp;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    const int k = (int)(t / ncolsp);
    const int col = (int)(t - (size_t)k * ncolsp);
    const int rs = col / a.Cp, c = col - rs * a.Cp;
    if (c >= a.C) return;
    int s4[4] = {0, 0, 0, 0};
    int z = 0;
    for (; z + 3 < a.splits; z += 4) {
#pragma unroll
        for (int u = 0; u < 4; ++u) s4[u] += a.partial[(size_t)(z + u) * total + t];
    }
    for (; z < a.splits; ++z) s4[0] += a.partial[(size_t)z * total + t];
    const int sum = (s4[0] + s4[1]) + (s4[2] + s4[3]);
    const size_t o = ((size_t)k * a.C + c) * (a.R * a.S) + rs;
    a.dw[o] = __fmul_rn((float)sum, __fmul_rn(a.sa[0], a.sb[0]));
    if (a.acc) a.acc[o] = sum;
}

// ---------------------------------------------------------------------------------------------
// Host-side plan: tile shapes, tap grouping, split count.  Shared by the workspace query and the
// launch so that both see the same numbers.
// ---------------------------------------------------------------------------------------------
void wgrad_plan(WgradArgs* a) {
    const int RS = a->R * a->S;
    // taps per block / channel slabs per wave: one filter row of a 3-wide filter, a whole 1x7 or
    // 7x1 filter, a wide channel tile for 1x1, one tap at a time otherwise
    if (RS == 1) { a->TB = 1; a->CS = (a->Cp >= 256) ? 4 : 1; }
    else if (RS % 3 == 0 && a->S == 3) { a->TB = 3; a->CS = 1; }
    else if (RS == 7) { a->TB = 7; a->CS = 1; }
    else { a->TB = 1; a->CS = 1; }
    // TB divides R*S in every case, so a tap group is never ragged
    const int CT = 64 * a->CS;
    a->tapgroups = (RS + a->TB - 1) / a->TB;
    a->ktiles = (a->K + W2_BM - 1) / W2_BM;
    a->ctiles = (a->Cp + CT - 1) / CT;
    // output-pixel tile: about 16 pixels, split evenly, shrunk until the staged window fits
    int nq = (a->Q + 7) / 8;
    int BQ = (a->Q + nq - 1) / nq;
    int BP = 16 / BQ;
    if (BP < 1) BP = 1;
    if (BP > a->P) BP = a->P;
    for (;;) {
        int maxwin = 0;
        for (int g = 0; g < a->tapgroups; ++g) {
            const int t0 = g * a->TB, nt = (RS - t0 < a->TB) ? (RS - t0) : a->TB;
            int rmin, rmax, smin, smax;
            tap_extent(t0, nt, a->S, &rmin, &rmax, &smin, &smax);
            const int WH = (BP - 1) * a->stride_h + (rmax - rmin) + 1;
            const int WW = (BQ - 1) * a->stride_w + (smax - smin) + 1;
            if (WH * WW > maxwin) maxwin = WH * WW;
        }
        a->xt_slots = maxwin * CT;
        a->lds_bytes = (size_t)(a->xt_slots + BP * BQ * W2_BM + 1) * 16;
        const int ntask = maxwin * (CT / 4) + BP * BQ * 16;
        if ((a->lds_bytes <= (size_t)W2_LDS_BUDGET && ntask <= 256 * W2_TPT && BP * BQ <= 2 * W2_MAXSTEPS) ||
            (BP == 1 && BQ == 1))
            break;
        if (BP > 1) BP = (BP + 1) / 2;
        else BQ = (BQ + 1) / 2;
    }
    const int np = (a->P + BP - 1) / BP;
    nq = (a->Q + BQ - 1) / BQ;
    a->BP = BP;
    a->BQ = BQ;
    a->ntp = np;
    a->ntq = nq;
    a->ngrp = (a->N + 15) / 16;
    a->chunks = a->ngrp * np * nq;
    const int out_tiles = a->ktiles * a->ctiles * a->tapgroups;
    int splits = (W2_TARGET_BLOCKS + out_tiles - 1) / out_tiles;
    if (splits > a->chunks) splits = a->chunks;
    if (splits < 1) splits = 1;
    a->splits = splits;
}

hipError_t launch_wgrad(const WgradArgs& a, hipStream_t st) {
    dim3 grid(a.ktiles * a.ctiles * a.tapgroups, a.splits);
#define LAUNCH(TBv, CSv) \
    hipLaunchKernelGGL((wgrad_kernel<TBv, CSv>), grid, dim3(256), a.lds_bytes, st, a)
    if (a.TB == 1 && a.CS == 1) LAUNCH(1, 1);
    else if (a.TB == 1 && a.CS == 4) LAUNCH(1, 4);
    else if (a.TB == 3) LAUNCH(3, 1);
    else if (a.TB == 7) LAUNCH(7, 1);
    else return hipErrorInvalidValue;
#undef LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t total = (size_t)a.K * a.R * a.S * a.Cp;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace int8t
