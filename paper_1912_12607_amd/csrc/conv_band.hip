// Dense forward / backward-data convolution for layers whose whole filter bank is small
// (at most 64 output rows and a few tens of KB of weight codes): the ResNet-18 3x3 layer, the
// MobileNetV2 1x1 layers.  Same arithmetic as conv_igemm.hip (int8 MFMA, int32 accumulators, Eq.2
// in the epilogue), different staging: such layers have a reduction of only a few hundred bytes
// per output, so a tile-by-tile pipeline spends its time waiting for memory.  Here a block keeps
// the complete weight matrix in LDS for its lifetime and, per band of output rows, stages the
// input rows it needs ONCE (with their zero padding); every filter tap is then a shifted view of
// that LDS window -- pixel-granular, so always 16-byte aligned -- and the whole reduction runs
// out of LDS without touching global memory again.
//
//   forward        rows = K, act = codes of a   (N,H,W,Cp), input pixel = (oh + r - ph, ow + s - pw)
//   backward-data  rows = C, act = codes of g_z (N,P,Q,Kp), input pixel = (oh + ph - r, ow + pw - s)
// (stride 1 only; other shapes go through the implicit-GEMM kernel.)
#include "device_common.h"
#include "kernels.h"

namespace int8t {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BAND_MAXPIX = 256;             // output pixels per band, at most (NTW = 2: 8 tiles of 32)
constexpr size_t BAND_LDS_MAX = 80 * 1024;   // two blocks per compute unit
constexpr int BAND_STAGE = 12;               // staged 16-byte granules per thread and band, at most
constexpr int BAND_MAXG = 64;                // reduction granules (16 bytes each) per output row, at most
constexpr int BAND_WJ = BAND_MAXG / 4;       // weight granules per thread
constexpr int BAND_REG_ROWS = 4;             // window rows of the register-weight variant, at most

// odd pitch (in 16-byte granules): rows of a tile read at one granule index land in distinct banks
__host__ __device__ inline int odd_pitch(int granules) { return (granules & 1) ? granules : granules + 1; }

// The kernel is written to keep the vector-ALU instruction count per MFMA small: everything that
// does not depend on the band (which granule a thread stages, the LDS offsets of every k-step,
// the output offsets of a lane) is worked out once per block.
// MT: 32-row tiles of output rows; NTW: 32-pixel tiles per wave; UNI: rows is a multiple of 8, so
// the "row exists" test of the epilogue is the same for every lane.
template <bool DGRAD, int MT, int NTW, bool UNI>
__global__ __launch_bounds__(256) void band_kernel(const IgemmArgs a, int BP, int nbands_h, int nbands) {
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int Cg16 = a.Ca >> 4;
    const int G = a.R * a.S * Cg16;          // reduction granules
    const int GP = odd_pitch(G);
    const int PG = odd_pitch(Cg16);
    const int WH = BP + a.R - 1, WW = a.OW + a.S - 1;
    const int nksteps = (G + 1) >> 1;
    uint4* __restrict__ wT = lds;                       // [64 rows][GP]
    uint4* __restrict__ xW = lds + 64 * GP;             // [WH*WW pixels][PG]
    uint4* __restrict__ zero = xW + WH * WW * PG;       // one zero granule
    int2* __restrict__ ktab = reinterpret_cast<int2*>(zero + 1);   // [nksteps + 1][2 halves]: {A offset, B offset}

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    // smallest input offset over the taps (rows / columns)
    const int drmin = DGRAD ? (a.pad_h - (a.R - 1)) : -a.pad_h;
    const int dsmin = DGRAD ? (a.pad_w - (a.S - 1)) : -a.pad_w;

    // ---- weights, once per block: thread = (row, granule mod 4); every load is issued before the
    // first store, so the whole matrix costs one memory round trip -------------------------------
    {
        const int row = tid >> 2, gq = tid & 3;
        const bool rv = row < a.rows;
        const int8_t* __restrict__ src = a.wgt + (size_t)(rv ? row : 0) * G * 16;
        uint4 v[BAND_WJ];
#pragma unroll
        for (int j = 0; j < BAND_WJ; ++j) {
            const int g = gq + 4 * j;
            v[j] = make_uint4(0, 0, 0, 0);
            if (rv && g < G) v[j] = *reinterpret_cast<const uint4*>(src + g * 16);
        }
#pragma unroll
        for (int j = 0; j < BAND_WJ; ++j) {
            const int g = gq + 4 * j;
            if (g < G) wT[row * GP + g] = v[j];
        }
    }
    if (tid == 0) *zero = make_uint4(0, 0, 0, 0);
    // ---- k-step table: granule g = 2*ks + half -> {weight granule index or -1, LDS offset of the
    // tap's pixel shift + channel granule}; one spare k-step so that the pipeline may read ahead ----
    if (tid < 2 * (nksteps + 1)) {
        const int g = tid;                       // = 2*ks + half
        int2 t;
        t.x = -1;
        t.y = 0;
        if (g < G) {
            const int tap = g / Cg16, cg = g - tap * Cg16;
            const int r = tap / a.S, s = tap - r * a.S;
            const int dr = DGRAD ? (a.pad_h - r) : (r - a.pad_h);
            const int ds = DGRAD ? (a.pad_w - s) : (s - a.pad_w);
            t.x = g;
            t.y = ((dr - drmin) * WW + (ds - dsmin)) * PG + cg;
        }
        ktab[tid] = t;
    }

    // ---- band-independent staging plan: slot k of this thread covers column granule
    // tid + 256*j of window row wy, k = wy * kw + j ----------------------------------------------------
    const int rowgran = WW * Cg16;
    const int kw = (rowgran + 255) >> 8;
    int s_goff[BAND_STAGE], s_ldst[BAND_STAGE], s_wy[BAND_STAGE];
    {
        int wy = 0, j = 0;
#pragma unroll
        for (int k = 0; k < BAND_STAGE; ++k) {
            const int col = tid + 256 * j;
            s_wy[k] = -1;
            s_goff[k] = 0;
            s_ldst[k] = 0;
            if (wy < WH && col < rowgran) {
                const int wx = col / Cg16, cg = col - wx * Cg16;
                const int iw = dsmin + wx;
                s_ldst[k] = (wy * WW + wx) * PG + cg;
                s_wy[k] = wy;
                s_goff[k] = ((unsigned)iw < (unsigned)a.IW) ? (iw * a.Ca + cg * 16) : -1;   // -1: padding column
            }
            if (++j == kw) {
                j = 0;
                ++wy;
            }
        }
    }

    // ---- per-lane output bookkeeping of the wave's n-tiles (pixel index inside the band) ---------
    const int npix = BP * a.OW;
    const int OHW = a.OH * a.OW;
    int pbase[NTW], pl[NTW];
    uint32_t obase[NTW];
    bool pvalid[NTW];
#pragma unroll
    for (int i = 0; i < NTW; ++i) {
        const int p = (wave + 4 * i) * 32 + l32;
        pvalid[i] = p < npix;
        const int pp = pvalid[i] ? p : 0;
        pl[i] = pp / a.OW;
        const int ql = pp - pl[i] * a.OW;
        pbase[i] = (pl[i] * WW + ql) * PG;
        obase[i] = (uint32_t)((4 * half) * OHW + pl[i] * a.OW + ql);   // + (n*rows)*OHW + oh0*OW + row term
    }
    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
    const int aoff0 = l32 * GP, aoff1 = (32 + l32) * GP;

    // Window loads of the NEXT band are in flight (in registers) while the current band computes.
    uint4 pre[BAND_STAGE];
    auto issue = [&](int band) {
        const int n = band / nbands_h;
        const int oh0 = (band - n * nbands_h) * BP;
        const int8_t* __restrict__ img = a.act + (size_t)n * a.IH * a.IW * a.Ca;
#pragma unroll
        for (int k = 0; k < BAND_STAGE; ++k) {
            pre[k] = make_uint4(0, 0, 0, 0);
            const int ih = oh0 + drmin + s_wy[k];
            if (s_wy[k] >= 0 && s_goff[k] >= 0 && (unsigned)ih < (unsigned)a.IH)
                pre[k] = *reinterpret_cast<const uint4*>(img + (size_t)ih * a.IW * a.Ca + s_goff[k]);
        }
    };
    if ((int)blockIdx.x < nbands) issue(blockIdx.x);

    // operand fetch of one k-step: weight fragments of the MT row tiles, pixel fragments of the NTW tiles
    auto fetch = [&](int ks, v4i (&fa)[MT], v4i (&fb)[NTW]) {
        const int2 t = ktab[2 * ks + half];
        const bool gv = t.x >= 0;
#pragma unroll
        for (int m = 0; m < MT; ++m) {
            const uint4 tw = gv ? wT[(m ? aoff1 : aoff0) + t.x] : *zero;
            fa[m] = v4i{(int)tw.x, (int)tw.y, (int)tw.z, (int)tw.w};
        }
#pragma unroll
        for (int i = 0; i < NTW; ++i) {
            const uint4 tb = xW[pbase[i] + t.y];
            fb[i] = v4i{(int)tb.x, (int)tb.y, (int)tb.z, (int)tb.w};
        }
    };

    for (int band = blockIdx.x; band < nbands; band += gridDim.x) {
        const int n = band / nbands_h;
        const int oh0 = (band - n * nbands_h) * BP;
        __syncthreads();   // previous band's reads are done (and weights / tables are in place)
#pragma unroll
        for (int k = 0; k < BAND_STAGE; ++k)
            if (s_wy[k] >= 0) xW[s_ldst[k]] = pre[k];
        __syncthreads();
        if (band + (int)gridDim.x < nbands) issue(band + gridDim.x);

        v16i acc[MT][NTW];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int i = 0; i < NTW; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[m][i][v] = 0;

        // k-loop, two steps per iteration with the operands of the following step requested before
        // the current step's MFMAs are issued (LDS latency hides behind the matrix pipeline)
        v4i fa0[MT], fb0[NTW], fa1[MT], fb1[NTW];
        fetch(0, fa0, fb0);
        for (int ks = 0; ks < nksteps; ks += 2) {
            fetch(ks + 1, fa1, fb1);             // ks + 1 <= nksteps: the spare table entry reads zeros
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int i = 0; i < NTW; ++i)
                    acc[m][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa0[m], fb0[i], acc[m][i], 0, 0, 0);
            if (ks + 2 < nksteps) fetch(ks + 2, fa0, fb0);
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int i = 0; i < NTW; ++i)
                    acc[m][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa1[m], fb1[i], acc[m][i], 0, 0, 0);
        }

        // ---- epilogue: Eq.2, 32 consecutive pixels of one output row per store -------------------
        const size_t bandoff = (size_t)n * a.rows * OHW + (size_t)oh0 * a.OW;
        float* __restrict__ outb = a.out + bandoff;
        int32_t* __restrict__ accb = a.acc ? a.acc + bandoff : nullptr;
#pragma unroll
        for (int i = 0; i < NTW; ++i) {
            if (!pvalid[i] || oh0 + pl[i] >= a.OH) continue;
#pragma unroll
            for (int m = 0; m < MT; ++m) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rowu = m * 32 + 8 * (v >> 2) + (v & 3);   // + 4*half, already in obase
                    const bool ok = UNI ? (m * 32 + 8 * (v >> 2) < a.rows) : (rowu + 4 * half < a.rows);
                    if (ok) {
                        const uint32_t o = obase[i] + (uint32_t)(rowu * OHW);
                        const int val = acc[m][i][v];
                        outb[o] = __fmul_rn((float)val, scale);
                        if (accb) accb[o] = val;
                    }
                }
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Variant with the weights in REGISTERS.  In the kernel above every k-step of a wave reads two
// weight fragments and one pixel fragment from LDS for two MFMAs, and with eight waves per compute
// unit the LDS port, not the matrix pipeline, sets the pace.  The weight fragments of a lane never
// change, though: lane (row, half) always multiplies rows {row, 32 + row} of the filter matrix.
// When the whole reduction is short (NKS k-steps, known at compile time) a lane keeps its 2*NKS
// fragments in registers for the block's lifetime and LDS serves the pixel fragment only -- one
// 16-byte read per two MFMAs.  The k-loop is fully unrolled; the tap offsets are scalars.
// The epilogue of a band is deferred: the scaled results wait in registers and are stored a few
// at a time between the MFMAs of the NEXT band, so the write stream and the matrix pipeline run
// side by side instead of taking turns.
// Needs an even number of channel granules (then the two halves of a k-step share a filter tap),
// at most 64 output rows, stride 1, a band of at most 128 pixels (one 32-pixel tile per wave) and a
// window of at most 4 rows of at most 256 granules (one granule per thread and row).
// ---------------------------------------------------------------------------------------------
struct BandRegTab {
    int koff[18];   // LDS offset (granules) of every k-step: tap shift + first channel granule of the pair
};

template <bool DGRAD, int NKS>
__global__ __launch_bounds__(256, 2) void band_reg_kernel(const IgemmArgs a, int BP, int nbands_h, int nbands,
                                                          const BandRegTab tab) {
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    const int Cg16 = a.Ca >> 4;
    constexpr int G = 2 * NKS;                // = R * S * Cg16 (host)
    const int PG = odd_pitch(Cg16);
    const int WH = BP + a.R - 1, WW = a.OW + a.S - 1;
    uint4* __restrict__ xW = lds;             // [WH*WW pixels][PG]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    const int drmin = DGRAD ? (a.pad_h - (a.R - 1)) : -a.pad_h;
    const int dsmin = DGRAD ? (a.pad_w - (a.S - 1)) : -a.pad_w;

    // (weights are fetched after the first window has been requested, see below)

    // ---- staging plan: thread = one 16-byte column granule of the window (a window row has at most
    // 256 granules), slot k = window row k ------------------------------------------------------------
    const int rowgran = WW * Cg16;
    int s_goff = -1, s_ldst = 0;               // s_goff -1: padding column or no column for this thread
    if (tid < rowgran) {
        const int wx = tid / Cg16, cg = tid - wx * Cg16;
        const int iw = dsmin + wx;
        s_ldst = wx * PG + cg;
        if ((unsigned)iw < (unsigned)a.IW) s_goff = iw * a.Ca + cg * 16;
    }
    const bool s_col = tid < rowgran;
    const int rowpitch = WW * PG;

    // ---- per-lane output bookkeeping: pixel p of the band, rows 4*half + ... ----------------------
    const int npix = BP * a.OW;
    const int OHW = a.OH * a.OW;
    const int p = wave * 32 + l32;
    const bool pvalid = p < npix;
    const int pp = pvalid ? p : 0;
    const int pl = pp / a.OW, ql = pp - pl * a.OW;
    const int pb = (pl * WW + ql) * PG + half;                     // + koff[ks]
    const uint32_t obase = (uint32_t)((4 * half) * OHW + pl * a.OW + ql);
    const float scale = __fmul_rn(a.sa[0], a.sb[0]);

    uint4 pre[BAND_REG_ROWS];
    auto issue = [&](int band) {
        const int n = band / nbands_h;
        const int oh0 = (band - n * nbands_h) * BP;
        const int8_t* __restrict__ img = a.act + (size_t)n * a.IH * a.IW * a.Ca;
#pragma unroll
        for (int k = 0; k < BAND_REG_ROWS; ++k) {
            pre[k] = make_uint4(0, 0, 0, 0);
            const int ih = oh0 + drmin + k;
            if (k < WH && s_goff >= 0 && (unsigned)ih < (unsigned)a.IH)
                pre[k] = *reinterpret_cast<const uint4*>(img + (size_t)ih * a.IW * a.Ca + s_goff);
        }
    };
    // Bands of a block: workgroups are dealt to the 8 XCDs round-robin, so workgroup b runs on XCD
    // b % 8.  Each XCD gets a contiguous range of bands and its workgroups walk it side by side:
    // neighbouring bands, which share input rows, then meet in the same L2.
    int band_first = blockIdx.x, band_step = gridDim.x, band_end = nbands;
    if ((gridDim.x & 7) == 0) {
        const int xcd = blockIdx.x & 7;
        band_first = (int)(((long long)nbands * xcd) >> 3) + (int)(blockIdx.x >> 3);
        band_end = (int)(((long long)nbands * (xcd + 1)) >> 3);
        band_step = gridDim.x >> 3;
    }
    if (band_first < band_end) issue(band_first);

    // ---- weight fragments, once per block.  Every wave needs the whole 64-row matrix; fetched by
    // each lane for itself that is four copies of it through the L1 per block, and the L1 fill rate
    // then sets the length of the prologue.  So the block fetches the matrix once, fully coalesced,
    // into LDS (the window buffer is not in use yet) and the lanes pick their fragments from there.
    // Buffer loads: a row beyond a.rows lies outside the descriptor and reads as zero.
    v4i fa[NKS][2];
    {
        constexpr int GPW = (G & 1) ? G : G + 1;       // odd pitch: a wave's 32 rows hit 32 different bank groups
        const __amdgpu_buffer_rsrc_t wr = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<int8_t*>(a.wgt), 0, (uint32_t)a.rows * G * 16u, 0x00020000);
        constexpr int PER = (64 * G + 255) / 256;
        uint4 tmp[PER];
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const uint32_t gi = (uint32_t)(tid + 256 * i);          // granule index in [row][G] order
            const auto t4 = __builtin_amdgcn_raw_buffer_load_b128(wr, gi < 64u * G ? gi * 16u : 0x80000000u, 0, 0);
            tmp[i] = make_uint4(t4[0], t4[1], t4[2], t4[3]);
        }
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int gi = tid + 256 * i;
            if (gi < 64 * G) lds[(gi / G) * GPW + (gi % G)] = tmp[i];
        }
        __syncthreads();
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                const uint4 t = lds[(m * 32 + l32) * GPW + 2 * ks + half];
                fa[ks][m] = v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w};
            }
        // (the band loop starts with a barrier, so the window may overwrite this area afterwards)
    }
    int koff[NKS];
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) koff[ks] = tab.koff[ks];

    // Results of the previous band, waiting to be stored.  Stores go through a buffer descriptor
    // that spans one image of the output: a lane without a valid pixel carries an offset beyond the
    // descriptor's range and rows beyond a.rows fall outside it too, and the hardware drops such
    // writes -- no branches between the MFMAs.
    float outv[2][16];
    __amdgpu_buffer_rsrc_t prev_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, 0, 0x00020000);
    uint32_t prev_voff = 0x80000000u;
    const uint32_t img_bytes = (uint32_t)a.rows * OHW * 4u;       // <= 2^31 (host)
    auto store_one = [&](int m, int v) {
        const int rowu = m * 32 + 8 * (v >> 2) + (v & 3);            // + 4*half, already in the lane's offset
        __builtin_amdgcn_raw_buffer_store_b32(__float_as_uint(outv[m][v]), prev_rsrc,
                                              prev_voff + (uint32_t)(rowu * OHW) * 4u, 0, 0);
    };

    for (int band = band_first; band < band_end; band += band_step) {
        const int n = band / nbands_h;
        const int oh0 = (band - n * nbands_h) * BP;
        __syncthreads();   // previous band's LDS reads are done
#pragma unroll
        for (int k = 0; k < BAND_REG_ROWS; ++k)
            if (k < WH && s_col) xW[k * rowpitch + s_ldst] = pre[k];
        __syncthreads();
        if (band + band_step < band_end) issue(band + band_step);

        v16i acc[2];
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[m][v] = 0;

        // pixel fragments are requested two k-steps ahead of their MFMAs
        // (the LDS address of a k-step is one add of a scalar; the empty asm keeps the compiler from
        // hoisting all NKS sums out of the band loop into registers the weights need)
        auto frag = [&](int ks) {
            int pbk = pb;
            asm volatile("" : "+v"(pbk));
            return xW[pbk + koff[ks]];
        };
        uint4 tb0 = frag(0);
        uint4 tb1 = frag(NKS > 1 ? 1 : 0);
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            const v4i fb = v4i{(int)tb0.x, (int)tb0.y, (int)tb0.z, (int)tb0.w};
            tb0 = tb1;
            if (ks + 2 < NKS) tb1 = frag(ks + 2 < NKS ? ks + 2 : 0);
            acc[0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks][0], fb, acc[0], 0, 0, 0);
            acc[1] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[ks][1], fb, acc[1], 0, 0, 0);
            // the previous band's 32 values, spread evenly over the k-steps
#pragma unroll
            for (int q = (32 * ks) / NKS; q < (32 * (ks + 1)) / NKS; ++q) store_one(q >> 4, q & 15);
        }

        // ---- Eq.2; the stores follow during the next band (or after the loop) -----------------------
        const size_t bandoff = (size_t)n * a.rows * OHW + (size_t)oh0 * a.OW;
        const bool ok = pvalid && oh0 + pl < a.OH;
        if (a.acc) {
            int32_t* __restrict__ accb = a.acc + bandoff;
#pragma unroll
            for (int m = 0; m < 2; ++m)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int rowu = m * 32 + 8 * (v >> 2) + (v & 3);
                    int32_t* __restrict__ rowp = accb + (size_t)rowu * OHW;
                    if (ok && rowu + 4 * half < a.rows) rowp[obase] = acc[m][v];
                }
        }
#pragma unroll
        for (int m = 0; m < 2; ++m)
#pragma unroll
            for (int v = 0; v < 16; ++v) outv[m][v] = __fmul_rn((float)acc[m][v], scale);
        prev_rsrc = __builtin_amdgcn_make_buffer_rsrc(a.out + (size_t)n * a.rows * OHW, 0, img_bytes, 0x00020000);
        prev_voff = ok ? (obase + (uint32_t)(oh0 * a.OW)) * 4u : 0x80000000u;
    }
#pragma unroll
    for (int q = 0; q < 32; ++q) store_one(q >> 4, q & 15);
}

// Returns true (and launches) when the layer fits this kernel; false: use the implicit GEMM.
bool launch_band(const IgemmArgs& a, hipStream_t st, hipError_t* err, bool dry_run) {
    if (a.stride_h != 1 || a.stride_w != 1 || a.rows > 64 || a.OW > BAND_MAXPIX) return false;
    const int Cg16 = a.Ca >> 4;
    const int G = a.R * a.S * Cg16;
    if (G > BAND_MAXG) return false;
    if ((size_t)a.N * a.rows * a.OH * a.OW > 0x7FFFFFFFull) return false;
    // band height: as many output rows as fit 128 pixels (one 32-pixel tile per wave; smaller bands
    // balance better over the persistent blocks than 256-pixel ones); one row of up to 256 pixels
    // (two tiles per wave) when a single row is wider than 128
    int ntw = 1;
    int BP = 128 / a.OW;
    if (BP < 1) { ntw = 2; BP = 1; }
    if (BP > a.OH) BP = a.OH;
    const int WW = a.OW + a.S - 1;
    const int kw = (WW * Cg16 + 255) / 256;
    while (BP > 1 && (BP + a.R - 1) * kw > BAND_STAGE) --BP;
    const int WH = BP + a.R - 1;
    if (WH * kw > BAND_STAGE) return false;
    const size_t lds = ((size_t)64 * odd_pitch(G) + (size_t)WH * WW * odd_pitch(Cg16) + 1) * 16 +
                       (size_t)(G + 4) * sizeof(int2);
    if (lds > BAND_LDS_MAX) return false;
    if (dry_run) return true;
    const int nbands_h = (a.OH + BP - 1) / BP;
    const int nbands = a.N * nbands_h;
    const int grid = nbands < 512 ? nbands : 512;
    // register-resident weights when the reduction length is one of the instantiated ones
    if (ntw == 1 && (Cg16 & 1) == 0 && WH <= BAND_REG_ROWS && WW * Cg16 <= 256 &&
        (size_t)a.rows * a.OH * a.OW <= ((size_t)1 << 29)) {
        typedef void (*kern_t)(const IgemmArgs, int, int, int, const BandRegTab);
        kern_t kr = nullptr;
        int slot = -1;
#define BR(NK, SL)                                                                          \
    if (G == 2 * NK) {                                                                       \
        kr = a.dgrad ? (kern_t)band_reg_kernel<true, NK> : (kern_t)band_reg_kernel<false, NK>; \
        slot = 2 * SL + (a.dgrad ? 1 : 0);                                                   \
    }
        BR(2, 0) BR(4, 1) BR(9, 2) BR(18, 3)
#undef BR
        if (kr) {
            size_t ldsr = (size_t)WH * WW * odd_pitch(Cg16) * 16;
            const size_t ldsw = (size_t)64 * odd_pitch(G) * 16;     // the weight matrix passes through LDS first
            if (ldsw > ldsr) ldsr = ldsw;
            static std::atomic<unsigned long long> attr_done_r[8];
            {
                hipError_t e = raise_dynamic_lds(reinterpret_cast<const void*>(kr), (int)BAND_LDS_MAX, attr_done_r[slot]);
                if (e != hipSuccess) { *err = e; return true; }
            }
            BandRegTab tab = {};
            {
                const int PG = odd_pitch(Cg16);
                const int drmin = a.dgrad ? (a.pad_h - (a.R - 1)) : -a.pad_h;
                const int dsmin = a.dgrad ? (a.pad_w - (a.S - 1)) : -a.pad_w;
                for (int ks = 0; 2 * ks < G; ++ks) {
                    const int g = 2 * ks, tap = g / Cg16, cg = g - tap * Cg16;
                    const int r = tap / a.S, sx = tap - r * a.S;
                    const int dr = a.dgrad ? (a.pad_h - r) : (r - a.pad_h);
                    const int ds = a.dgrad ? (a.pad_w - sx) : (sx - a.pad_w);
                    tab.koff[ks] = ((dr - drmin) * WW + (ds - dsmin)) * PG + cg;
                }
            }
            {
                KernelTimer kt(KID_BAND_REG, st);
                launch_timed(kt, kr, dim3(grid), dim3(256), ldsr, st, a, BP, nbands_h, nbands, tab);
            }
            *err = hipGetLastError();
            return true;
        }
    }
    const int mt = a.rows > 32 ? 2 : 1;
    const int uni = (a.rows % 8 == 0) ? 1 : 0;
    const int variant = (a.dgrad ? 8 : 0) + (mt - 1) * 4 + (ntw - 1) * 2 + uni;
    typedef void (*kern_t)(const IgemmArgs, int, int, int);
#define BK(D, M, N) band_kernel<D, M, N, false>, band_kernel<D, M, N, true>
    static const kern_t kerns[16] = {BK(false, 1, 1), BK(false, 1, 2), BK(false, 2, 1), BK(false, 2, 2),
                                     BK(true, 1, 1),  BK(true, 1, 2),  BK(true, 2, 1),  BK(true, 2, 2)};
#undef BK
    static std::atomic<unsigned long long> attr_done[16];
    {
        hipError_t e = raise_dynamic_lds(reinterpret_cast<const void*>(kerns[variant]), (int)BAND_LDS_MAX, attr_done[variant]);
        if (e != hipSuccess) { *err = e; return true; }
    }
    {
        KernelTimer kt(KID_BAND, st);
        launch_timed(kt, kerns[variant], dim3(grid), dim3(256), lds, st, a, BP, nbands_h, nbands);
    }
    *err = hipGetLastError();
    return true;
}

}  // namespace int8t
