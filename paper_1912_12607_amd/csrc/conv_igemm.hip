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
// Tile: BM (64 or 128) rows x BN (128 or 256) cols per 256-thread block (2 x 2 waves, each
// BM/2 x BN/2), 64 reduction bytes per stage.  Two LDS buffers: while the MFMAs of a stage run, the
// next stage's global loads are in flight in registers and are written to the other buffer, so a
// stage costs one barrier.  The wide tile (128 x 256: 16 MFMAs per wave and barrier, 0.75 LDS
// operand reads per MFMA) serves the layers whose convolutions are bound by the matrix cores.
#include "device_common.h"
#include "kernels.h"
#include "lds_dma.h"

namespace int8t {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

// 16-byte slot of (row, granule) inside a [rows][4 granules] LDS tile.  LDS serves a 16-byte-per-lane
// access 16 lanes at a time, and those 16 lanes are conflict-free when their slots differ mod 16
// (64 banks of 4 bytes).  MFMA operand reads are 16 consecutive rows of one granule: slot mod 16 =
// 4 * (row & 3) + position, so the position must differ between rows r, r+4, r+8, r+12 -- the xor
// with bits 2..3 of the row.  The loader's writes (4 consecutive rows x 4 granules) stay 16
// consecutive slots.
__device__ __forceinline__ int lds_slot(int row, int g) { return row * 4 + (g ^ ((row >> 2) & 3)); }

// Strided backward-data by residue classes.  The input pixels (h, w) with h % stride_h == ch and
// w % stride_w == cw all receive the same filter taps: r = r0 + stride_h * tr, s = s0 + stride_w * ts,
// and for pixel h = ch + stride_h * i the tap tr reads gradient row i + bh - tr.  In the class's own
// coordinates (i, j, tr, ts) that is a stride-1 backward-data pass over nr x ns taps, so a tile whose
// columns are pixels of ONE class spends no matrix-core work on the taps that never reach it (a
// tile of neighbouring pixels multiplies stride_h * stride_w - 1 zeros for every useful product).
// A class without taps (1x1 filter, stride 2: three pixels in four) gets zeros.
struct DgradClass {
    int ch, cw;        // residues of the class
    int OHc, OWc;      // pixels of the class per image: rows, columns
    int r0, s0, nr, ns;
    int bh, bw;
};
__device__ __forceinline__ DgradClass dgrad_class(const IgemmArgs& a, int cls) {
    DgradClass c;
    const int csh = a.cls_h, csw = a.cls_w;     // the stride, or 1 where that direction is not split
    c.ch = cls / csw;
    c.cw = cls - c.ch * csw;
    c.OHc = (a.OH - c.ch + csh - 1) / csh;
    c.OWc = (a.OW - c.cw + csw - 1) / csw;
    c.r0 = (c.ch + a.pad_h) % csh;
    c.s0 = (c.cw + a.pad_w) % csw;
    c.nr = c.r0 < a.R ? (a.R - c.r0 + csh - 1) / csh : 0;
    c.ns = c.s0 < a.S ? (a.S - c.s0 + csw - 1) / csw : 0;
    c.bh = (c.ch + a.pad_h - c.r0) / csh;
    c.bw = (c.cw + a.pad_w - c.s0) / csw;
    return c;
}

// When only ONE class has taps (a 1x1 filter under a stride) the other pixels are zero, and the pass
// is bound by writing them.  "Cell" form (CELL, stride 2 x 2 and an even row length): the columns are
// the 2 x 2 cells of pixels, the tile runs the one class's taps, and the epilogue writes each cell
// whole -- the value at the class's pixel, zeros around it -- as two 8-byte stores, so that a lane
// stores neighbouring floats and a wave whole cache lines.  T = float (result) or int (partial sums,
// accumulators); `o` is the cell's top left element (even: 8-byte aligned).
template <typename T, typename T2>
__device__ __forceinline__ void store_cell(T* __restrict__ dst, size_t o, int OW, bool second_row, int ch, int cw, T v) {
    const T z = (T)0;
    T2 top, bot;
    top.x = (ch == 0 && cw == 0) ? v : z;
    top.y = (ch == 0 && cw == 1) ? v : z;
    bot.x = (ch == 1 && cw == 0) ? v : z;
    bot.y = (ch == 1 && cw == 1) ? v : z;
    *reinterpret_cast<T2*>(dst + o) = top;
    if (second_row) *reinterpret_cast<T2*>(dst + o + OW) = bot;
}

// CLS (backward-data with a stride only): blockIdx.x = column tile * classes + class.
// FUSEQ (forward, 1 x 1 filter, stride 1, no padding): the quantization of the activations (Eq.1) is fused
// into the load path -- the quantization-convolution fused kernel of the paper's Suppl. "INT8
// Convolution".  A thread then makes its 16-byte granule itself: 16 fp32 loads (16 consecutive
// channels of its pixel; a wave reads 64 consecutive pixels of a channel plane per instruction),
// Eq.1 on each, packed to codes.  The codes never make the round trip through HBM before the
// convolution reads them; the first row tile still writes them out when the caller wants them for
// the backward-weight pass.
template <int BM, int BN, bool DGRAD, bool CLS = false, bool CELL = false, bool FUSEQ = false>
__global__ __launch_bounds__(256, 2) void igemm_kernel(const IgemmArgs a) {
    static_assert(DGRAD || !CLS, "residue classes exist in the backward-data pass only");
    static_assert(CLS || !CELL, "the cell form is a residue-class form");
    static_assert(!FUSEQ || (!DGRAD && !CLS), "the fused quantizer serves the forward pass");
    constexpr int MI = BM / 64;   // 32-row MFMA tiles per wave
    constexpr int NJ = BN / 64;   // 32-column MFMA tiles per wave
    constexpr int NB = BN / 64;   // B-tile columns staged per thread
    __shared__ uint4 sA[2][BM * 4];
    __shared__ uint4 sB[2][BN * 4];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;
    // loader: (tile row or column, granule of the stage).  FUSEQ: a wave takes one granule of 64
    // consecutive pixels, so that its fp32 loads walk a channel plane
    const int lrow = FUSEQ ? (tid & 63) : (tid >> 2), lg = FUSEQ ? (tid >> 6) : (tid & 3);

    const int OHWfull = a.OH * a.OW;
    const int Cg16 = a.Ca >> 4;
    float qinv = 0.0f, qscale = 0.0f;
    if (FUSEQ) {
        __shared__ float lds4[4];
        const float cval = a.xclip ? a.xclip[0] : reduce_absmax_partials(a.xabs_part, a.xabs_nparts, lds4);
        qinv = inv_scale_of(cval);
        qscale = scale_of(cval);
        if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && tid == 0) a.sx_out[0] = qscale;
    }
    DgradClass dc;
    int colblock = blockIdx.x;
    if (CLS) {
        if (CELL) {
            dc = dgrad_class(a, a.cell - 1);
            dc.OHc = (a.OH + a.cls_h - 1) / a.cls_h;      // cells, not pixels of the class
            dc.OWc = (a.OW + a.cls_w - 1) / a.cls_w;
        } else {
            const int ncls = a.cls_h * a.cls_w;
            colblock = blockIdx.x / ncls;
            dc = dgrad_class(a, (int)blockIdx.x - colblock * ncls);
        }
    }
    const int OWc = CLS ? dc.OWc : a.OW;
    const int OHW = CLS ? dc.OHc * dc.OWc : OHWfull;     // columns per image
    const int ncols = a.N * OHW;
    const int nr = CLS ? dc.nr : a.R, ns = CLS ? dc.ns : a.S;
    const int gtot = nr * ns * Cg16;
    const int nsteps = (gtot + 3) >> 2;
    const int rowbase = blockIdx.y * BM;
    const int colbase = colblock * BN;
    // split reduction: block z works on the stages [step0, step1) and stores raw partial sums
    const int step0 = (int)(((long long)nsteps * blockIdx.z) / a.ksplit);
    const int step1 = (int)(((long long)nsteps * (blockIdx.z + 1)) / a.ksplit);

    // ---- loader state -----------------------------------------------------------------------
    // B (pixels): NB columns per thread, fixed for the whole reduction
    int bh[NB], bw[NB];
    const int8_t* bimg[NB];
    bool bvalid[NB];
#pragma unroll
    for (int i = 0; i < NB; ++i) {
        const int col = colbase + i * 64 + lrow;
        bvalid[i] = col < ncols;
        const int cc = bvalid[i] ? col : 0;
        const int n = cc / OHW, rem = cc - n * OHW;
        const int oh = rem / OWc, ow = rem - oh * OWc;
        bh[i] = CLS ? (oh + dc.bh) : DGRAD ? (oh + a.pad_h) : (oh * a.stride_h - a.pad_h);
        bw[i] = CLS ? (ow + dc.bw) : DGRAD ? (ow + a.pad_w) : (ow * a.stride_w - a.pad_w);
        bimg[i] = a.act + (size_t)n * a.IH * a.IW * a.Ca;
    }
    // reduction position of this thread's granule: filter tap (r,s) and channel granule cg
    int r, s, cg;
    {
        const int q0 = step0 * 4 + lg;
        const int tap = q0 / Cg16;
        cg = q0 - tap * Cg16;
        r = tap / (ns > 0 ? ns : 1);
        s = tap - r * ns;
    }
    // A (weights): MI rows per thread
    const int8_t* arow[MI];
    bool avalid[MI];
#pragma unroll
    for (int i = 0; i < MI; ++i) {
        const int row = rowbase + i * 64 + lrow;
        avalid[i] = row < a.rows;
        arow[i] = a.wgt + (size_t)(avalid[i] ? row : 0) * (a.R * a.S * Cg16) * 16;
    }

    uint4 ra[MI], rb[NB];
    auto load_step = [&](int step) {
        const int q = step * 4 + lg;
        const bool qv = q < gtot;
        // granule of the filter row: the taps of a class are a sub-grid of the R x S filter
        const int wq = CLS ? ((dc.r0 + a.cls_h * r) * a.S + dc.s0 + a.cls_w * s) * Cg16 + cg : q;
#pragma unroll
        for (int i = 0; i < MI; ++i) {
            ra[i] = make_uint4(0, 0, 0, 0);
            if (qv && avalid[i]) ra[i] = *reinterpret_cast<const uint4*>(arow[i] + (size_t)wq * 16);
        }
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            rb[i] = make_uint4(0, 0, 0, 0);
            if (FUSEQ) {
                // column = pixel (n, oh*OW + ow) of the input itself; granule cg = channels 16 cg .. 16 cg + 15
                if (qv && bvalid[i]) {
                    const int col = colbase + i * 64 + lrow;
                    const int n = col / OHW, pix = col - n * OHW;
                    const float* __restrict__ px = a.xf + ((size_t)n * a.C + 16 * cg) * OHW + pix;
                    float v[16];
#pragma unroll
                    for (int k = 0; k < 16; ++k) v[k] = (16 * cg + k < a.C) ? px[(size_t)k * OHW] : 0.0f;
                    uint32_t d[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
                        d[j] = pack4(quantize_one<false>(v[4 * j], qinv, 0, 0, 0), quantize_one<false>(v[4 * j + 1], qinv, 0, 0, 0),
                                     quantize_one<false>(v[4 * j + 2], qinv, 0, 0, 0), quantize_one<false>(v[4 * j + 3], qinv, 0, 0, 0));
                    rb[i] = make_uint4(d[0], d[1], d[2], d[3]);
                    if (a.xq_out && blockIdx.y == 0)
                        *reinterpret_cast<uint4*>(a.xq_out + ((size_t)n * OHW + pix) * a.Ca + 16 * cg) = rb[i];
                }
                continue;
            }
            int ih, iw;
            bool ok = qv && bvalid[i];
            if (DGRAD) {
                const int th = bh[i] - r, tw = bw[i] - s;
                // a direction split into classes is a stride-1 pass; otherwise only the taps that divide reach a pixel
                const int dsh = CLS ? a.stride_h / a.cls_h : a.stride_h, dsw = CLS ? a.stride_w / a.cls_w : a.stride_w;
                if (dsh == 1 && dsw == 1) {
                    ih = th;
                    iw = tw;
                } else {
                    ih = th / dsh;
                    iw = tw / dsw;
                    ok = ok && th >= 0 && tw >= 0 && (ih * dsh == th) && (iw * dsw == tw);
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
            if (++s == ns) {
                s = 0;
                ++r;
            }
        }
    };
    auto stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < MI; ++i) sA[buf][lds_slot(i * 64 + lrow, lg)] = ra[i];
#pragma unroll
        for (int i = 0; i < NB; ++i) sB[buf][lds_slot(i * 64 + lrow, lg)] = rb[i];
    };

    v16i acc[MI][NJ];
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NJ; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;

    load_step(step0);
    stage(step0 & 1);
    __syncthreads();
    for (int step = step0; step < step1; ++step) {
        const int buf = step & 1;
        if (step + 1 < step1) load_step(step + 1);      // in flight while this stage computes
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int g = kk * 2 + (lane >> 5);
            v4i fa[MI], fb[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const uint4 t = sA[buf][lds_slot(wm * (BM / 2) + i * 32 + (lane & 31), g)];
                fa[i] = v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint4 t = sB[buf][lds_slot(wn * (BN / 2) + j * 32 + (lane & 31), g)];
                fb[j] = v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
        // the other buffer was last read one stage ago, before the barrier that ended that stage
        if (step + 1 < step1) stage(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: Eq.2, straight into N,C,H,W; a split reduction leaves its share of the sums
    // in partial[z][N][rows][OH*OW] for igemm_reduce_kernel instead ---------------------------
    const bool split = a.ksplit > 1;
    int32_t* __restrict__ const part = split ? a.partial + (size_t)blockIdx.z * a.N * a.rows * OHWfull : nullptr;
    const float scale = __fmul_rn(FUSEQ ? qscale : a.sa[0], a.sb[0]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = colbase + wn * (BN / 2) + j * 32 + (lane & 31);
        if (col >= ncols) continue;
        const int n = col / OHW;
        int opix = col - n * OHW;
        int ci = 0, cj = 0;
        if (CLS) {
            ci = opix / OWc;
            cj = opix - ci * OWc;
            opix = (dc.ch + a.cls_h * ci) * a.OW + dc.cw + a.cls_w * cj;
        }
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rowbase + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < a.rows) {
                    const size_t idx = ((size_t)n * a.rows + row) * OHWfull + opix;
                    const int val = acc[i][j][v];
                    if (CELL) {
                        const size_t o = ((size_t)n * a.rows + row) * OHWfull + (size_t)(2 * ci) * a.OW + 2 * cj;
                        const bool two = 2 * ci + 1 < a.OH;
                        if (split) {
                            store_cell<int32_t, int2>(part, o, a.OW, two, dc.ch, dc.cw, val);
                        } else {
                            store_cell<float, float2>(a.out, o, a.OW, two, dc.ch, dc.cw, __fmul_rn((float)val, scale));
                            if (a.acc) store_cell<int32_t, int2>(a.acc, o, a.OW, two, dc.ch, dc.cw, val);
                        }
                    } else if (split) {
                        part[idx] = val;
                    } else {
                        a.out[idx] = __fmul_rn((float)val, scale);
                        if (a.acc) a.acc[idx] = val;
                    }
                }
            }
        }
    }
}

// Sum of the ksplit partial results (integer addition: exact in any order) and Eq.2.  A thread owns
// four consecutive results; VEC: the result count is a multiple of 4, so every slice is 16-byte aligned.
template <bool VEC>
__global__ __launch_bounds__(256) void igemm_reduce_kernel(const IgemmArgs a, size_t total) {
    const size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4;
    if (i >= total) return;
    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
    if (VEC) {
        int4 sum = make_int4(0, 0, 0, 0);
        int z = 0;
        for (; z + 4 <= a.ksplit; z += 4) {
            int4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) v[u] = *reinterpret_cast<const int4*>(a.partial + (size_t)(z + u) * total + i);
#pragma unroll
            for (int u = 0; u < 4; ++u) { sum.x += v[u].x; sum.y += v[u].y; sum.z += v[u].z; sum.w += v[u].w; }
        }
        for (; z < a.ksplit; ++z) {
            const int4 v = *reinterpret_cast<const int4*>(a.partial + (size_t)z * total + i);
            sum.x += v.x; sum.y += v.y; sum.z += v.z; sum.w += v.w;
        }
        *reinterpret_cast<float4*>(a.out + i) = make_float4(__fmul_rn((float)sum.x, scale), __fmul_rn((float)sum.y, scale),
                                                            __fmul_rn((float)sum.z, scale), __fmul_rn((float)sum.w, scale));
        if (a.acc) { a.acc[i] = sum.x; a.acc[i + 1] = sum.y; a.acc[i + 2] = sum.z; a.acc[i + 3] = sum.w; }
    } else {
        for (size_t e = i; e < total && e < i + 4; ++e) {
            int sum = 0;
            for (int z = 0; z < a.ksplit; ++z) sum += a.partial[(size_t)z * total + e];
            a.out[e] = __fmul_rn((float)sum, scale);
            if (a.acc) a.acc[e] = sum;
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Wide-tile variants for the layers bound by the matrix cores: (64*WM) rows x 256 columns per
// block of 2*WM waves (each 64 x 128), operands fetched by buffer loads that write straight into
// LDS (no staging registers), NSTAGE LDS buffers in a ring with the loads running NSTAGE-1 stages
// ahead of the MFMAs, one barrier per stage.  A stage is KG 16-byte granules of the reduction per
// row: KG = 8 makes every row's share of a stage one full 128-byte cache line.  A wave-wide load
// fills 64 consecutive 16-byte slots, lane l the slot base + l; which (row, granule) that slot
// holds follows from the slot index, so each lane simply fetches the granule that belongs there.
// Out-of-range rows, ragged columns, padding taps and the reduction tail carry an offset beyond the
// buffer descriptor: the hardware then writes zeros.
//   <WM=2, KG=4, NSTAGE=3>: 128 x 256, 72 KB of LDS, two blocks per compute unit
//   <WM=4, KG=8, NSTAGE=2>: 256 x 256, 128 KB of LDS, one block of eight waves per compute unit
//   <WM=2, KG=4, NSTAGE=3, BNT=128>: 128 x 128 (waves of 64 x 64), 48 KB of LDS, three blocks per compute unit: for
//   layers whose larger tiles would leave most compute units without one
//   <WM=2, KG=8, NSTAGE=2, BNT=128>: the same tile with 128-byte stages (64 KB, two blocks): half the barriers per MFMA,
//   better where the reduction is long
//   <WM=2, KG=8, NSTAGE=2, BNT=64>: 128 x 64 (waves of 64 x 32), 48 KB: twice the tiles for layers with few columns
//   (7 x 7 and 8 x 8 images), which otherwise leave more than half of the compute units idle
// ---------------------------------------------------------------------------------------------
//   ALLC (with CLS and CELL, stride 2 x 2, every class with taps): the columns are the 2 x 2 cells of pixels and the
//   block runs the four classes one after the other, each into accumulators of its own, then writes every cell
//   whole -- two neighbouring floats per lane and image row, whole cache lines per wave -- where the per-class
//   form writes every other float of a line from four different blocks and pays a block's fixed cost per class.
template <bool DGRAD, int WM, int KG, int NSTAGE, bool CLS = false, bool CELL = false, int BNT = IGD_BN, bool ALLC = false>
__global__ __launch_bounds__(128 * WM, WM == 2 ? (ALLC ? 2 : (BNT == 128 && KG == 4) || BNT == 64 ? 3 : 2) : 1) void igemm_dma_kernel(const IgemmArgs a) {
    static_assert(DGRAD || !CLS, "residue classes exist in the backward-data pass only");
    static_assert(CLS || !CELL, "the cell form is a residue-class form");
    static_assert(!ALLC || (CLS && CELL && BNT == 64), "all classes per block: cell columns, 64 of them");
    constexpr int BM = 64 * WM, BN = BNT, MI = 2, NJ = BN / 64, NW = 2 * WM;
    constexpr int NC = ALLC ? 4 : 1;                    // classes a block runs
    constexpr int STAGE_SLOTS = (BM + BN) * KG;         // 16-byte slots per stage: A tile, then B tile
    constexpr int RPL = 64 / KG;                        // tile rows covered by one wave-wide load
    constexpr int NLA = BM * KG / 64 / NW;              // A loads per wave and stage
    constexpr int NLB = BN * KG / 64 / NW;              // B loads per wave and stage
    constexpr int NL = NLA + NLB;
    static_assert(NSTAGE == 2 || NL == 6 || NL == 4, "vmcnt waits below are written for these");
    extern __shared__ __attribute__((aligned(16))) uint4 ring[];   // [NSTAGE][STAGE_SLOTS]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;

    const int OHWfull = a.OH * a.OW;
    const int Cg16 = a.Ca >> 4;
    const int gfull = a.R * a.S * Cg16;
    // Workgroups are dealt to the 8 XCDs round-robin (workgroup b runs on XCD b % 8).  Column tile
    // ct = 8 * (i / rtiles) + xcd, row tile i % rtiles, i = b / 8: all row tiles of a column tile --
    // they read the same pixels -- run on one XCD and share its L2, as do the column tiles of an XCD
    // that read the same filter rows.  The grid is padded to whole groups of 8 column tiles.
    // CLS: the residue classes of a column tile follow each other on the same XCD as well (they read
    // the same gradient pixels and write interleaved floats of the same cache lines).
    const int rtiles = (a.rows + BM - 1) / BM;
    const int wg_i = blockIdx.x >> 3;
    int cgroup = wg_i / rtiles;
    DgradClass dc;
    if (CLS) {
        if (CELL) {
            dc = dgrad_class(a, ALLC ? 0 : a.cell - 1);
            dc.OHc = (a.OH + a.cls_h - 1) / a.cls_h;      // cells, not pixels of the class
            dc.OWc = (a.OW + a.cls_w - 1) / a.cls_w;
        } else {
            const int ncls = a.cls_h * a.cls_w;
            const int g = cgroup / ncls;
            dc = dgrad_class(a, cgroup - g * ncls);
            cgroup = g;
        }
    }
    const int OWc = CLS ? dc.OWc : a.OW;
    const int OHW = CLS ? dc.OHc * dc.OWc : OHWfull;     // columns per image
    const int ncols = a.N * OHW;
    int nr = CLS ? dc.nr : a.R, ns = CLS ? dc.ns : a.S;  // (ALLC: of the class being run)
    int gtot = nr * ns * Cg16;
    int nsteps = (gtot + KG - 1) / KG;
    const int ctile = (cgroup << 3) + (int)(blockIdx.x & 7);
    if (ctile * BN >= ncols) return;
    const int rowbase = (wg_i % rtiles) * BM;
    const int colbase = ctile * BN;

    const v4i wr = igd_rsrc(a.wgt, (uint32_t)((size_t)a.rows * gfull * 16));
    const v4i xr = igd_rsrc(a.act, (uint32_t)((size_t)a.N * a.IH * a.IW * a.Ca));
    // LDS byte address of this wave's first A / B load slot in buffer 0 (wave-uniform)
    const uint32_t lds_a0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(size_t)(ring + 64 * wave));
    const uint32_t lds_b0 = lds_a0 + BM * KG * 16;

    // ---- loader state: this wave issues A loads {wave + NW*i} and B loads {wave + NW*i}.  Load
    // number wl covers tile rows RPL*wl .. RPL*wl + RPL-1; lane -> (row, granule) through the swizzle.
    const int lrow = lane / KG;                              // row inside the load's row group
    // granule held by this lane's slot: the inverse of igd_slot().  KG = 4: a load covers 16 rows from a
    // multiple of 16, bits 2..3 of the row are those of lrow.  KG = 8: a load covers 8 rows from
    // 8 * (wave + NW * i); with NW even, bit 3 of the row is the wave's parity for every i.
    static_assert(KG == 4 || (NW & 1) == 0, "the swizzle of the 8-granule tile needs an even wave count");
    const int gsw = KG == 4 ? ((lane & 3) ^ ((lrow >> 2) & 3)) : ((lane & 7) ^ (((lrow >> 1) & 3) | ((wave & 1) << 2)));
    uint32_t aoff[NLA];                                      // byte offset of (row, granule 0) or OOB
#pragma unroll
    for (int i = 0; i < NLA; ++i) {
        const int row = rowbase + RPL * (wave + NW * i) + lrow;
        aoff[i] = row < a.rows ? (uint32_t)row * (uint32_t)gfull * 16u : IGD_OOB;
    }
    int bh[NLB], bw[NLB];
    int boh[NLB], bow[NLB];                                  // (ALLC) the column's cell, to which each class adds its offset
    uint32_t bimg[NLB];                                      // byte offset of the column's image or OOB
#pragma unroll
    for (int i = 0; i < NLB; ++i) {
        const int col = colbase + RPL * (wave + NW * i) + lrow;
        const bool cv = col < ncols;
        const int cc = cv ? col : 0;
        const int n = cc / OHW, rem = cc - n * OHW;
        const int oh = rem / OWc, ow = rem - oh * OWc;
        boh[i] = oh;
        bow[i] = ow;
        bh[i] = CLS ? (oh + dc.bh) : DGRAD ? (oh + a.pad_h) : (oh * a.stride_h - a.pad_h);
        bw[i] = CLS ? (ow + dc.bw) : DGRAD ? (ow + a.pad_w) : (ow * a.stride_w - a.pad_w);
        bimg[i] = cv ? (uint32_t)n * (uint32_t)(a.IH * a.IW * a.Ca) : IGD_OOB;
    }
    // reduction position of this lane's granule: filter tap (r,s) and channel granule cg
    int r, s, cg;
    int qnext;                                               // granule index of the next stage to issue
    auto first_granule = [&]() {
        const int tap = gsw / Cg16;
        cg = gsw - tap * Cg16;
        r = tap / (ns > 0 ? ns : 1);
        s = tap - r * ns;
        qnext = gsw;
    };
    first_granule();

    auto issue_a = [&](int buf) {
        const uint32_t boff = (uint32_t)buf * (STAGE_SLOTS * 16u);
        const bool qv = qnext < gtot;
        // granule of the filter row: the taps of a class are a sub-grid of the R x S filter
        const int wq = CLS ? ((dc.r0 + a.cls_h * r) * a.S + dc.s0 + a.cls_w * s) * Cg16 + cg : qnext;
#pragma unroll
        for (int i = 0; i < NLA; ++i) {
            const uint32_t off = (qv && aoff[i] != IGD_OOB) ? aoff[i] + (uint32_t)wq * 16u : IGD_OOB;
            igd_load_lds(wr, lds_a0 + boff + (uint32_t)i * (NW * 64 * 16), off);
        }
    };
    auto issue_b = [&](int buf) {
        const uint32_t boff = (uint32_t)buf * (STAGE_SLOTS * 16u);
        const bool qv = qnext < gtot;
#pragma unroll
        for (int i = 0; i < NLB; ++i) {
            int ih, iw;
            bool ok = qv && bimg[i] != IGD_OOB;
            if (DGRAD) {
                const int th = bh[i] - r, tw = bw[i] - s;
                // a direction split into classes is a stride-1 pass; otherwise only the taps that divide reach a pixel
                const int dsh = CLS ? a.stride_h / a.cls_h : a.stride_h, dsw = CLS ? a.stride_w / a.cls_w : a.stride_w;
                if (dsh == 1 && dsw == 1) {
                    ih = th;
                    iw = tw;
                } else {
                    ih = th / dsh;
                    iw = tw / dsw;
                    ok = ok && th >= 0 && tw >= 0 && (ih * dsh == th) && (iw * dsw == tw);
                }
            } else {
                ih = bh[i] + r;
                iw = bw[i] + s;
            }
            ok = ok && (unsigned)ih < (unsigned)a.IH && (unsigned)iw < (unsigned)a.IW;
            const uint32_t off = ok ? bimg[i] + (uint32_t)((ih * a.IW + iw) * a.Ca + cg * 16) : IGD_OOB;
            igd_load_lds(xr, lds_b0 + boff + (uint32_t)i * (NW * 64 * 16), off);
        }
        // advance this lane's reduction position by one stage (KG granules)
        qnext += KG;
        cg += KG;
        while (cg >= Cg16) {
            cg -= Cg16;
            if (++s == ns) {
                s = 0;
                ++r;
            }
        }
    };

    v16i acc[NC][MI][NJ];
#pragma unroll
    for (int c = 0; c < NC; ++c)
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int j = 0; j < NJ; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[c][i][j][v] = 0;

#pragma unroll
    for (int c = 0; c < NC; ++c) {
    if (ALLC && c > 0) {
        // the next class: its taps and offsets; the ring is free once every wave has read the last stage
        dc = dgrad_class(a, c);
        nr = dc.nr;
        ns = dc.ns;
        gtot = nr * ns * Cg16;
        nsteps = (gtot + KG - 1) / KG;
#pragma unroll
        for (int i = 0; i < NLB; ++i) {
            bh[i] = boh[i] + dc.bh;
            bw[i] = bow[i] + dc.bw;
        }
        first_granule();
        __syncthreads();
    }
    // prologue: the first NSTAGE-1 stages on their way
    if (nsteps > 0) {     // (a class without taps has nothing to load: its pixels get zeros)
        issue_a(0);
        issue_b(0);
    }
#pragma unroll
    for (int p = 1; p < NSTAGE - 1; ++p) {
        if (nsteps > p) {
            issue_a(p);
            issue_b(p);
        }
    }
    for (int step = 0; step < nsteps; ++step) {
        const int buf = step % NSTAGE;
        // this stage's loads are the oldest outstanding ones; the loads of the up to NSTAGE - 2 stages
        // behind it may still be in flight
        if (NSTAGE == 4 && step + 2 < nsteps) igd_wait_vmcnt<NSTAGE == 4 ? 2 * NL : 0>();
        else if (NSTAGE >= 3 && step + 1 < nsteps) igd_wait_vmcnt<NSTAGE >= 3 ? NL : 0>();
        else igd_wait_vmcnt<0>();
        __syncthreads();   // every wave's part of this stage is in LDS; stage step-1 has been read by all
        // the next loads go into the buffer read in stage step-1; the weight half is requested now,
        // the pixel half in the middle of this stage's MFMAs, so the memory pipeline sees a steady
        // stream instead of one burst per stage
        const bool more = step + NSTAGE - 1 < nsteps;
        const int nbuf = (step + NSTAGE - 1) % NSTAGE;
        if (more) issue_a(nbuf);
        const uint4* __restrict__ sA = ring + buf * STAGE_SLOTS;
        const uint4* __restrict__ sB = sA + BM * KG;
#pragma unroll
        for (int kk = 0; kk < KG / 2; ++kk) {
            const int g = kk * 2 + (lane >> 5);
            v4i fa[MI], fb[NJ];
#pragma unroll
            for (int i = 0; i < MI; ++i) {
                const uint4 t = sA[igd_slot<KG>(wm * 64 + i * 32 + (lane & 31), g)];
                fa[i] = v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
#pragma unroll
            for (int j = 0; j < NJ; ++j) {
                const uint4 t = sB[igd_slot<KG>(wn * (BN / 2) + j * 32 + (lane & 31), g)];
                fb[j] = v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < NJ; ++j)
                    acc[c][i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[c][i][j], 0, 0, 0);
            if (kk == (KG >= 8 ? KG / 4 - 1 : 0) && more) issue_b(nbuf);
        }
    }
    }   // classes

    // ---- epilogue: Eq.2, straight into N,C,H,W ----------------------------------------------
    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
        const int col = colbase + wn * (BN / 2) + j * 32 + (lane & 31);
        if (col >= ncols) continue;
        const int n = col / OHW;
        int opix = col - n * OHW;
        int ci = 0, cj = 0;
        if (CLS) {
            ci = opix / OWc;
            cj = opix - ci * OWc;
            opix = (dc.ch + a.cls_h * ci) * a.OW + dc.cw + a.cls_w * cj;
        }
#pragma unroll
        for (int i = 0; i < MI; ++i) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = rowbase + wm * 64 + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (row < a.rows) {
                    const size_t idx = ((size_t)n * a.rows + row) * OHWfull + opix;
                    const int val = acc[0][i][j][v];
                    if (ALLC) {
                        // the cell's four pixels, classes (row parity, column parity) = 0 .. 3; the last cell row / column
                        // of an odd image holds one row / column only
                        const size_t o = ((size_t)n * a.rows + row) * OHWfull + (size_t)(2 * ci) * a.OW + 2 * cj;
                        const bool two = 2 * ci + 1 < a.OH, right = 2 * cj + 1 < a.OW;
                        const int v00 = val, v01 = acc[NC > 1 ? 1 : 0][i][j][v], v10 = acc[NC > 2 ? 2 : 0][i][j][v],
                                  v11 = acc[NC > 3 ? 3 : 0][i][j][v];
                        if (!(a.OW & 1)) {          // every cell starts on an 8-byte boundary
                            *reinterpret_cast<float2*>(a.out + o) = make_float2(__fmul_rn((float)v00, scale), __fmul_rn((float)v01, scale));
                            if (two) *reinterpret_cast<float2*>(a.out + o + a.OW) = make_float2(__fmul_rn((float)v10, scale), __fmul_rn((float)v11, scale));
                            if (a.acc) {
                                *reinterpret_cast<int2*>(a.acc + o) = make_int2(v00, v01);
                                if (two) *reinterpret_cast<int2*>(a.acc + o + a.OW) = make_int2(v10, v11);
                            }
                        } else {
                            a.out[o] = __fmul_rn((float)v00, scale);
                            if (right) a.out[o + 1] = __fmul_rn((float)v01, scale);
                            if (two) {
                                a.out[o + a.OW] = __fmul_rn((float)v10, scale);
                                if (right) a.out[o + a.OW + 1] = __fmul_rn((float)v11, scale);
                            }
                            if (a.acc) {
                                a.acc[o] = v00;
                                if (right) a.acc[o + 1] = v01;
                                if (two) {
                                    a.acc[o + a.OW] = v10;
                                    if (right) a.acc[o + a.OW + 1] = v11;
                                }
                            }
                        }
                    } else if (CELL) {
                        const size_t o = ((size_t)n * a.rows + row) * OHWfull + (size_t)(2 * ci) * a.OW + 2 * cj;
                        const bool two = 2 * ci + 1 < a.OH;
                        store_cell<float, float2>(a.out, o, a.OW, two, dc.ch, dc.cw, __fmul_rn((float)val, scale));
                        if (a.acc) store_cell<int32_t, int2>(a.acc, o, a.OW, two, dc.ch, dc.cw, val);
                    } else {
                        a.out[idx] = __fmul_rn((float)val, scale);
                        if (a.acc) a.acc[idx] = val;
                    }
                }
            }
        }
    }
}

namespace {
// Shape of the GEMM(s) a launch runs.  A strided backward-data pass is stride_h * stride_w stride-1
// problems, one per residue class of the pixels (dgrad_class): fewer columns and fewer taps each.
struct IgemmShape {
    int cell;          // 0, or 1 + the class of the cell form (store_cell)
    bool cls;
    int cls_h, cls_w;  // class strides (1, 1 when the pixels are not split)
    int ncls;
    long long ncols;   // columns of one GEMM (the largest class)
    long long gran;    // 16-byte reduction granules per column (the largest class)
};
IgemmShape igemm_shape(const IgemmArgs& a) {
    IgemmShape g;
    // Split when more than one class has taps; with a single one (a 1x1 filter) the cell form runs
    // (store_cell).  No split on small images with a short reduction: a store instruction covers 32 pixels of a class, which
    // are runs of OW / stride_w strided floats; with runs under 12 pixels the scattered stores cost
    // more than the zeros do unless a pixel's reduction is long (17 x 17 image, 192 channels: 56 us
    // split against 51 whole; 14 x 14, 512 channels: 40 against 85).
    const int tap_classes = (a.R < a.stride_h ? a.R : a.stride_h) * (a.S < a.stride_w ? a.S : a.stride_w);
    const bool short_runs = a.OW / a.stride_w < 12 && a.R * a.S * a.Ca < 2048;
    const bool strided = a.dgrad && (a.stride_h > 1 || a.stride_w > 1);
    g.cell = 0;
    if (strided && tap_classes == 1 && a.stride_h == 2 && a.stride_w == 2 && !(a.OW & 1)) {
        // the class whose residue makes the filter's first tap divide: r0 = (ch + pad_h) mod stride_h = 0
        const int ch = a.R < a.stride_h ? (a.stride_h - a.pad_h % a.stride_h) % a.stride_h : 0;
        const int cw = a.S < a.stride_w ? (a.stride_w - a.pad_w % a.stride_w) % a.stride_w : 0;
        g.cell = 1 + ch * a.stride_w + cw;
    }
    g.cls = strided && (g.cell || (tap_classes > 1 && !short_runs));
    g.cls_h = g.cls ? a.stride_h : 1;
    g.cls_w = g.cls ? a.stride_w : 1;
    if (g.cell) {
        g.ncls = 1;
        g.ncols = (long long)a.N * ((a.OH + g.cls_h - 1) / g.cls_h) * ((a.OW + g.cls_w - 1) / g.cls_w);
        g.gran = (long long)((a.R + g.cls_h - 1) / g.cls_h) * ((a.S + g.cls_w - 1) / g.cls_w) * (a.Ca >> 4);
    } else if (g.cls) {
        g.ncls = g.cls_h * g.cls_w;
        g.ncols = (long long)a.N * ((a.OH + g.cls_h - 1) / g.cls_h) * ((a.OW + g.cls_w - 1) / g.cls_w);
        g.gran = (long long)((a.R + g.cls_h - 1) / g.cls_h) * ((a.S + g.cls_w - 1) / g.cls_w) * (a.Ca >> 4);
    } else {
        g.ncls = 1;
        g.ncols = (long long)a.N * a.OH * a.OW;
        g.gran = (long long)a.R * a.S * (a.Ca >> 4);
    }
    return g;
}
}  // namespace

template <bool DGRAD, int WM, int KG, int NSTAGE, bool CLS, bool CELL, int BNT = IGD_BN, bool ALLC = false>
static hipError_t launch_igemm_dma(const IgemmArgs& a, const IgemmShape& g, hipStream_t st, const KernelTimer& kt) {
    const size_t lds = (size_t)NSTAGE * (64 * WM + BNT) * KG * 16;
    static std::atomic<unsigned long long> attr_done;
    {
        hipError_t e = raise_dynamic_lds(reinterpret_cast<const void*>(igemm_dma_kernel<DGRAD, WM, KG, NSTAGE, CLS, CELL, BNT, ALLC>), (int)lds, attr_done);
        if (e != hipSuccess) return e;
    }
    const unsigned ctiles = (unsigned)((g.ncols + BNT - 1) / BNT), rtiles = (unsigned)((a.rows + 64 * WM - 1) / (64 * WM));
    dim3 grid(((ctiles + 7) / 8) * 8 * rtiles * (unsigned)g.ncls);
    launch_timed(kt, (igemm_dma_kernel<DGRAD, WM, KG, NSTAGE, CLS, CELL, BNT, ALLC>), grid, dim3(128 * WM), lds, st, a);
    return hipGetLastError();
}
template <int WM, int KG, int NSTAGE, int BNT = IGD_BN>
static hipError_t launch_igemm_dma_any(const IgemmArgs& a, const IgemmShape& g, hipStream_t st, const KernelTimer& kt) {
    if (!a.dgrad) return launch_igemm_dma<false, WM, KG, NSTAGE, false, false, BNT>(a, g, st, kt);
    if (g.cell) return launch_igemm_dma<true, WM, KG, NSTAGE, true, true, BNT>(a, g, st, kt);
    if (g.cls) return launch_igemm_dma<true, WM, KG, NSTAGE, true, false, BNT>(a, g, st, kt);
    return launch_igemm_dma<true, WM, KG, NSTAGE, false, false, BNT>(a, g, st, kt);
}
template <int BM, int BN>
static void launch_igemm_generic(const IgemmArgs& a, const IgemmShape& g, int ksplit, hipStream_t st, const KernelTimer& kt) {
    dim3 grid((unsigned)((g.ncols + BN - 1) / BN) * (unsigned)g.ncls, (unsigned)((a.rows + BM - 1) / BM), (unsigned)ksplit);
    if (!a.dgrad) launch_timed(kt, (igemm_kernel<BM, BN, false, false, false>), grid, dim3(256), 0, st, a);
    else if (g.cell) launch_timed(kt, (igemm_kernel<BM, BN, true, true, true>), grid, dim3(256), 0, st, a);
    else if (g.cls) launch_timed(kt, (igemm_kernel<BM, BN, true, true, false>), grid, dim3(256), 0, st, a);
    else launch_timed(kt, (igemm_kernel<BM, BN, true, false, false>), grid, dim3(256), 0, st, a);
}

// Layers with few output tiles and a long reduction (a strided 3x3 on a small image, a fully
// connected layer) leave most compute units idle: their reduction is split over up to
// ceil(512 / tiles) blocks per tile, at least 4 stages each.  1 = no split.
int igemm_ksplit(const IgemmArgs& a) {
    if (a.rows <= 64) return 1;
    const IgemmShape g = igemm_shape(a);
    const long long tiles = g.ncls * ((g.ncols + 127) / 128) * ((a.rows + 127) / 128);
    const long long nsteps = (g.gran + 3) / 4;
    if (tiles >= 192 || nsteps < 8) return 1;
    long long ks = (512 + tiles - 1) / tiles;
    if (ks > nsteps / 4) ks = nsteps / 4;
    return ks < 2 ? 1 : (int)ks;
}

// the form that runs the four pixel classes of a stride-2 backward-data pass in one block: every class needs a tap
static bool igemm_cells_ok(const IgemmArgs& a) {
    return a.dgrad && a.stride_h == 2 && a.stride_w == 2 && a.R >= 2 && a.S >= 2;
}

// The variant the library picks on its own (rules from measurements over the layers of ResNet-50,
// MobileNetV2 and InceptionV3); a caller may overrule it per layer (include/int8t.h).
int igemm_auto_variant(const IgemmArgs& a, bool allow_split) {
    hipError_t e = hipSuccess;
    if (launch_band(a, nullptr, &e, true)) return VAR_BAND;
    // At most 64 rows and no band kernel (strides, filter banks too large for the chip): none of the three networks has
    // such a pass; on 25 random ones the 128 x 64 LDS-DMA tile, half empty, took 0.5 - 0.85 of the 64-row tile's time.
    if (a.rows <= 64) return VAR_WIDE_128X64;
    // Above 64 rows the 128 x 128 tiles of the LDS-DMA kernel win on nearly every layer of the three networks
    // (ResNet-50, batch 64: forward and backward-data 2.60 -> 2.11 ms in total; the best variant per layer would give 2.07):
    //  - 128 x 256 tiles of 4 waves per row pair where they are full, many, unsplit and the reduction is at least
    //    512 bytes (14 x 14, 256 channels, 3x3, batch 256: 41.6 against 46.3 us); the pixel classes of a strided
    //    backward-data pass leave them ragged (28 x 28, 512 -> 1024 shortcut: 33.5 against 28.7)
    //  - else 128 x 128: 128-byte stages (two blocks per compute unit) where a column's reduction is at least 1 KB, or 512 bytes
    //    with fewer than 512 tiles or the tap classes of a strided backward-data pass (56 x 56, 128 channels, 3x3, stride 2:
    //    44.7 against 53.9 us); 64-byte stages (three blocks) below (35 x 35, 96 channels, 3x3: 20.9 against 25.1 us)
    const IgemmShape g = igemm_shape(a);
    //  - few tiles and a very long reduction (5x5 and 7x7 filters on 1024 channels at 4 x 4 to 10 x 10, small batches): the
    //    split reduction of igemm_kernel, when the caller gave the scratch for it.  Over 40 such layers it won from about
    //    40 + 0.4 x (number of 128 x 64 tiles) stages of 128 bytes on, by up to 6.5x (16 tiles, 392 stages: 204 -> 31 us);
    //    no layer of the three networks is that shape (their closest: 7 x 7, 512 channels, 3x3 with 196 tiles and 36
    //    stages, 23 us on the LDS-DMA tiles against 35 split)
    {
        const long long t64s = g.ncls * ((g.ncols + 63) / 64) * ((a.rows + 127) / 128), stages = (g.gran + 7) / 8;
        if (allow_split && 5 * stages >= 200 + 2 * t64s && igemm_ksplit(a) > 1) return VAR_TILE_SPLIT;
    }
    //  - backward-data under stride 2 x 2 on images of at least 28 pixels a row, even row length: the four pixel classes in
    //    one block, whole 2 x 2 cells written (56 x 56, 128 channels, 3x3: 43.7 -> 37.0 us; 28 x 28, 256 channels: 36.4 ->
    //    28.1); on smaller images the four short reductions in a row cost more than the stores gain (14 x 14, 512 channels:
    //    28.8 against 32.9), and with odd rows the cells no longer start on 8-byte boundaries (35 x 35: 39.6 against 40.4)
    //    (and with long reductions the block count matters more: 5x5 on 1024 channels, 141 against 82 us)
    if (igemm_cells_ok(a) && g.cls && !g.cell && a.rows >= 128 && !(a.OW & 1) && a.OW >= 28 && g.gran <= 128) return VAR_WIDE_CELLS;
    const long long c256 = g.ncls * ((g.ncols + 255) / 256), c128 = g.ncls * ((g.ncols + 127) / 128);
    // (a column tile's row tiles all run on XCD (column tile) mod 8, one block per compute unit: 243 tiles that put 33 blocks
    // on an XCD of 32 compute units take two turns -- 1x1, 768 channels, 18 x 18, batch 64: 41.5 us against 29.8 on 128 x 128
    // tiles -- so the 256 x 256 tiles must fill at least 0.7 of the turns they take)
    const long long r256 = (a.rows + 255) / 256, t256 = c256 * r256, turns = (((c256 + 7) / 8) * r256 + 31) / 32;
    if (!g.cls && t256 >= 192 && a.rows > 128 && g.gran >= 32 && 10 * t256 >= 7 * turns * 256) return VAR_WIDE256;
    const long long rt = (a.rows + 127) / 128, tiles = c128 * rt;
    const bool deep = g.gran >= 64 || (g.gran >= 32 && (tiles < 512 || (g.cls && !g.cell)));
    //  - 128 x 64 tiles where they go round the chip's block slots (three per compute unit; two for the 128-byte
    //    stages) in fewer than twice the turns the 128 x 128 tiles need -- a tile of half the width takes a good half of
    //    the time -- which is the case for the 7 x 7, 8 x 8 and most 14 x 14 layers (7 x 7, 512 channels, 3x3, batch 64:
    //    100 tiles of 128 x 128 on 256 compute units, 31.9 -> 23.3 us; ResNet-50's forward and backward-data passes
    //    together 1.92 -> 1.70 ms)
    const long long t64 = g.ncls * ((g.ncols + 63) / 64) * rt, slots = deep ? 512 : 768;
    if (tiles <= 2000 && (t64 + 767) / 768 < 2 * ((tiles + slots - 1) / slots)) return VAR_WIDE_128X64;
    return deep ? VAR_WIDE_SQ128_DEEP : VAR_WIDE_SQ128;
}

bool igemm_variant_ok(const IgemmArgs& a, int variant) {
    hipError_t e = hipSuccess;
    switch (variant) {
        case VAR_AUTO: case VAR_TILE: case VAR_WIDE128: case VAR_WIDE256: case VAR_WIDE_SQ128: case VAR_WIDE_SQ128_DEEP: case VAR_WIDE_128X64: return true;
        case VAR_BAND: return launch_band(a, nullptr, &e, true);
        case VAR_TILE_SPLIT: return igemm_ksplit(a) > 1;
        case VAR_WIDE_CELLS: return igemm_cells_ok(a);
        default: return false;
    }
}

hipError_t launch_igemm_fused(const IgemmArgs& a_in, hipStream_t st) {
    IgemmArgs a = a_in;
    if (a.dgrad || a.R != 1 || a.S != 1 || a.stride_h != 1 || a.stride_w != 1 || a.pad_h || a.pad_w || !a.xf || !a.sx_out)
        return hipErrorInvalidValue;
    a.cls_h = a.cls_w = 1;
    a.cell = 0;
    a.ksplit = 1;
    const unsigned ncols = (unsigned)(a.N * a.OH * a.OW);
    KernelTimer kt(KID_IGEMM_FUSED, st);
    if (a.rows <= 64) {
        dim3 grid((ncols + 127) / 128, 1, 1);
        launch_timed(kt, (igemm_kernel<64, 128, false, false, false, true>), grid, dim3(256), 0, st, a);
    } else {
        dim3 grid((ncols + 127) / 128, (unsigned)((a.rows + 127) / 128), 1);
        launch_timed(kt, (igemm_kernel<128, 128, false, false, false, true>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

size_t igemm_s2d(IgemmArgs* a) {
    if (a->dgrad || a->C < 1 || a->Ca != 16 || !s2d_applies(a->C, a->stride_h, a->stride_w)) return 0;
    const S2dGeo g = s2d_geometry(a->R, a->S, a->pad_h, a->pad_w);
    a->C *= 4;
    a->IH = (a->IH + 1) / 2;
    a->IW = (a->IW + 1) / 2;
    a->R = g.R2;
    a->S = g.S2;
    a->pad_h = g.ph;
    a->pad_w = g.pw;
    a->stride_h = a->stride_w = 1;        // OH and OW stay: the rewritten layer has the same output pixels
    const size_t a256 = 255;
    return (((size_t)a->N * a->IH * a->IW * 16 + a256) & ~a256) + (((size_t)a->rows * g.R2 * g.S2 * 16 + a256) & ~a256);
}

hipError_t launch_igemm(const IgemmArgs& a_in, hipStream_t st) {
    IgemmArgs a = a_in;
    if (a.s2d) {
        // forward pass of a stride-2 layer with at most 4 channels: rewrite codes and geometry (s2d.hip)
        IgemmArgs t = a;
        if (igemm_s2d(&t)) {
            const S2dGeo g = s2d_geometry(a.R, a.S, a.pad_h, a.pad_w);
            int8_t* const xs = a.s2d;
            int8_t* const ws = a.s2d + (((size_t)t.N * t.IH * t.IW * 16 + 255) & ~(size_t)255);
            hipError_t e = launch_s2d_repack(a.act, xs, a.N, a.IH, a.IW, a.C, st);
            if (e != hipSuccess) return e;
            e = launch_s2d_weights(a.wgt, ws, a.rows, a.R, a.S, a.C, g, st);
            if (e != hipSuccess) return e;
            t.act = xs;
            t.wgt = ws;
            a = t;
        }
    }
    int variant = a.variant;
    if (variant == VAR_AUTO || !igemm_variant_ok(a, variant))
        variant = igemm_auto_variant(a, a.partial != nullptr && a.partial_bytes >= (size_t)igemm_ksplit(a) * a.rows * a.N * a.OH * a.OW * 4);
    if (variant == VAR_BAND) {
        hipError_t berr = hipSuccess;
        if (launch_band(a, st, &berr)) return berr;   // small filter bank: LDS-resident kernel
        return hipErrorInvalidValue;                  // (igemm_variant_ok said it fits)
    }
    const IgemmShape g = igemm_shape(a);
    a.cls_h = g.cls_h;
    a.cls_w = g.cls_w;
    a.cell = g.cell;
    const int ncols = a.N * a.OH * a.OW;
    // the split needs its scratch; without it the reduction simply stays whole
    a.ksplit = variant == VAR_TILE_SPLIT ? igemm_ksplit(a) : 1;
    if (a.ksplit > 1 && (a.partial == nullptr || a.partial_bytes < (size_t)a.ksplit * a.rows * ncols * 4)) a.ksplit = 1;
    if (a.ksplit > 1) {
        {
            KernelTimer kt(KID_IGEMM, st);
            launch_igemm_generic<128, 128>(a, g, a.ksplit, st, kt);
        }
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        const size_t total = (size_t)a.rows * ncols;
        KernelTimer kt(KID_IGEMM_REDUCE, st);
        const dim3 rgrid((unsigned)((total + 1023) / 1024));
        if ((total & 3) == 0) launch_timed(kt, igemm_reduce_kernel<true>, rgrid, dim3(256), 0, st, a, total);
        else launch_timed(kt, igemm_reduce_kernel<false>, rgrid, dim3(256), 0, st, a, total);
        return hipGetLastError();
    }
    if (variant == VAR_WIDE_CELLS) {
        IgemmShape gc = g;
        gc.cls = true;
        gc.cell = 0;
        gc.cls_h = gc.cls_w = 2;
        gc.ncls = 1;
        gc.ncols = (long long)a.N * ((a.OH + 1) / 2) * ((a.OW + 1) / 2);
        a.cls_h = a.cls_w = 2;
        a.cell = 0;
        KernelTimer kt(KID_IGEMM_DMA, st);
        return launch_igemm_dma<true, 2, 8, 2, true, true, 64, true>(a, gc, st, kt);
    }
    if (variant == VAR_WIDE128 || variant == VAR_WIDE256 || variant == VAR_WIDE_SQ128 || variant == VAR_WIDE_SQ128_DEEP ||
        variant == VAR_WIDE_128X64) {
        KernelTimer kt(KID_IGEMM_DMA, st);
        if (variant == VAR_WIDE256) return launch_igemm_dma_any<4, 8, 2>(a, g, st, kt);
        if (variant == VAR_WIDE_SQ128) return launch_igemm_dma_any<2, 4, 3, 128>(a, g, st, kt);
        if (variant == VAR_WIDE_SQ128_DEEP) return launch_igemm_dma_any<2, 8, 2, 128>(a, g, st, kt);
        if (variant == VAR_WIDE_128X64) return launch_igemm_dma_any<2, 8, 2, 64>(a, g, st, kt);
        return launch_igemm_dma_any<2, 4, 3>(a, g, st, kt);
    }
    KernelTimer kt(KID_IGEMM, st);
    if (a.rows <= 64) launch_igemm_generic<64, 128>(a, g, 1, st, kt);
    else launch_igemm_generic<128, 128>(a, g, 1, st, kt);
    return hipGetLastError();
}

}  // namespace int8t
