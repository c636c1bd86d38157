// Dense forward and backward-data convolution on int8 codes: implicit GEMM on the gfx950
// int8 MFMA (v_mfma_i32_32x32x32_i8: int8 x int8 products, int32 accumulators -- the matrix-core
// analogue of the 4-element dot product of the paper's Suppl. "INT8 Convolution"), with the
// dequantize step of Eq.2 fused into the epilogue.
//
// GEMM view:  D[row][col] = sum_red  Wt[row][red] * Act[red][col]
//   forward        rows = K,  cols = (n,p,q),  red = (r,s,c),  Act = codes of a   (N,H,W,Cp)
//   backward-data  rows = C,  cols = (n,h,w),  red = (r,s,k),  Act = codes of g_z (N,P,Q,Kp)
// The reduction index runs over 16-byte granules (16 consecutive channels of one filter tap),
// flattened across taps, so small channel counts waste no MFMA work on padding between taps.
// Weights are the MFMA "A" operand and pixels the "B" operand: a lane then holds 16 output
// channels of ONE pixel, and a store instruction writes 32 consecutive pixels of one channel
// (128 contiguous bytes) straight into the N,C,H,W result.
//
// Tile: BM (64 or 128) rows x 128 cols per 256-thread block, 64 reduction bytes per step, staged
// through LDS (im2col gather done by the loader, zero fill for padding / ragged edges), next
// step's global loads in flight while the current step's MFMAs run.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int IG_BN = 128;

// 16-byte slot of (row, granule) inside a [rows][4 granules] LDS tile.  The xor keeps both the
// loader's writes (4 lanes per row) and the MFMA operand reads (32 consecutive rows, one
// granule) spread over all banks.
__device__ __forceinline__ int lds_slot(int row, int g) { return row * 4 + (g ^ ((row >> 1) & 3)); }

template <int BM, bool DGRAD>
__global__ __launch_bounds__(256) void igemm_kernel(const IgemmArgs a) {
    constexpr int MI = BM / 64;   // 32-row MFMA tiles per wave
    __shared__ uint4 sA[BM * 4];
    __shared__ uint4 sB[IG_BN * 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    const int lrow = tid >> 2, lg = tid & 3;

    const int OHW = a.OH * a.OW;
    const int ncols = a.N * OHW;
    const int Cg16 = a.Ca >> 4;
    const int gtot = a.R * a.S * Cg16;
    const int nsteps = (gtot + 3) >> 2;
    const int rowbase = blockIdx.y * BM;
    const int colbase = blockIdx.x * IG_BN;

    // ---- loader state -----------------------------------------------------------------------
    // B (pixels): two columns per thread, fixed for the whole reduction
    int bh[2], bw[2];
    const int8_t* bimg[2];
    bool bvalid[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        const int col = colbase + i * 64 + lrow;
        bvalid[i] = col < ncols;
        const int cc = bvalid[i] ? col : 0;
        const int n = cc / OHW, rem = cc - n * OHW;
        const int oh = rem / a.OW, ow = rem - oh * a.OW;
        bh[i] = DGRAD ? (oh + a.pad_h) : (oh * a.stride_h - a.pad_h);
        bw[i] = DGRAD ? (ow + a.pad_w) : (ow * a.stride_w - a.pad_w);
        bimg[i] = a.act + (size_t)n * a.IH * a.IW * a.Ca;
    }
    // reduction position of this thread's granule: filter tap (r,s) and channel granule cg
    int r, s, cg;
    {
        const int tap = lg / Cg16;
        cg = lg - tap * Cg16;
        r = tap / a.S;
        s = tap - r * a.S;
    }
    // A (weights): MI rows per thread
    const int8_t* arow[MI];
    bool avalid[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int row = rowbase + i * 64 + lrow;
        avalid[i] = row < a.rows;
        arow[i] = a.wgt + (size_t)(avalid[i] ? row : 0) * gtot * 16;
    }

    uint4 ra[MI], rb[2];
    auto load_step = [&](int step) {
        const int q = step * 4 + lg;
        const bool qv = q < gtot;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            ra[i] = make_uint4(0, 0, 0, 0);
            if (qv && avalid[i]) ra[i] = *reinterpret_cast<const uint4*>(arow[i] + (size_t)q * 16);
        }
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            rb[i] = make_uint4(0, 0, 0, 0);
            int ih, iw;
            bool ok = qv && bvalid[i];
            if (DGRAD) {
                const int th = bh[i] - r, tw = bw[i] - s;
                if (a.stride_h == 1 && a.stride_w == 1) {
                    ih = th;
                    iw = tw;
                } else {
                    ih = th / a.stride_h;
                    iw = tw / a.stride_w;
                    ok = ok && th >= 0 && tw >= 0 && (ih * a.stride_h == th) && (iw * a.stride_w == tw);
                }
            } else {
                ih = bh[i] + r;
                iw = bw[i] + s;
            }
            ok = ok && (unsigned)ih < (unsigned)a.IH && (unsigned)iw < (unsigned)a.IW;
            if (ok)
                rb[i] = *reinterpret_cast<const uint4*>(bimg[i] + ((size_t)ih * a.IW + iw) * a.Ca + cg * 16);
        }
        // advance this thread's reduction position by one step (4 granules)
        cg += 4;
        while (cg >= Cg16) {
            cg -= Cg16;
            if (++s == a.S) {
                s = 0;
                ++r;
            }
        }
    };

    v16i acc[MI][2];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    load_step(0);
    for (int step = 0; step < nsteps; ++step) {
        __syncthreads();
#pragma unroll
        for (int i = 0; i < MI; ++i) sA[lds_slot(i * 64 + lrow, lg)] = ra[i];
#pragma unroll
        for (int i = 0; i < 2; ++i) sB[lds_slot(i * 64 + lrow, lg)] = rb[i];
        __syncthreads();
        if (step + 1 < nsteps) load_step(step + 1);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int g = kk * 2 + (lane >> 5);
            v4i fa[MI], fb[2];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const uint4 t = sA[lds_slot(wm * (BM / 2) + i * 32 + (lane & 31), g)];
                fa[i] = v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const uint4 t = sB[lds_slot(wn * 64 + j * 32 + (lane & 31), g)];
                fb[j] = v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // ---- epilogue: Eq.2, straight into N,C,H,W ----------------------------------------------
    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = colbase + wn * 64 + j * 32 + (lane & 31);
        if (col >= ncols) continue;
        const int n = col / OHW, opix = col - n * OHW;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rowbase + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < a.rows) {
                    const size_t idx = ((size_t)n * a.rows + row) * OHW + opix;
                    const int val = acc[i][j][v];
                    a.out[idx] = __fmul_rn((float)val, scale);
                    if (a.acc) a.acc[idx] = val;
                }
            }
        }
    }
}

hipError_t launch_igemm(const IgemmArgs& a, hipStream_t st) {
    hipError_t berr = hipSuccess;
    if (launch_band(a, st, &berr)) return berr;   // small filter bank: LDS-resident kernel
    const int ncols = a.N * a.OH * a.OW;
    const int ctiles = (ncols + IG_BN - 1) / IG_BN;
    KernelTimer kt(KID_IGEMM, st);
    if (a.rows <= 64) {
        dim3 grid(ctiles, 1);
        if (a.dgrad) hipLaunchKernelGGL((igemm_kernel<64, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((igemm_kernel<64, false>), grid, dim3(256), 0, st, a);
    } else {
        dim3 grid(ctiles, (a.rows + 127) / 128);
        if (a.dgrad) hipLaunchKernelGGL((igemm_kernel<128, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((igemm_kernel<128, false>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace int8t
