// Dense backward-weight convolution (Sec.3.4: g_W = g_z^T a) for stride-1 filters with 1, 3 or 7 taps along
// one image axis, strided 1x1 filters and 3x3 filters under stride 2, on int8 MFMA with int32 accumulation.  Same result, partial-tile format and final
// reduction as conv_wgrad.hip; what differs is how the operands reach the matrix cores.
//
// GEMM view:  D[k][(tap,c)] = sum over (n,p,q) of  Gz[(n,p,q)][k] * A[(n, p+r-ph, q+s-pw)][c].
// The codes are channels-last, the reduction runs over pixels, and the MFMA wants 16 consecutive reduction
// bytes per lane.  Here nothing is transposed by hand:
//   * the loader copies [pixel][64 channels] rows of both tensors from HBM straight into LDS
//     (buffer loads with the LDS flag: no registers, no vector ALU work), two ring stages deep;
//   * the operand fetch is gfx950's transposing LDS read (ds_read_b64_tr_b8): in every group of 16
//     lanes, lane i receives byte i%8 of the 8-byte chunks that the lanes 2e + i/8 (e = 0..7) point
//     at.  Lane j of a group points at (reduction element j/2, channels 8*(j%2) .. +7 of the group's 16),
//     so lane i ends up with its own channel of 8 reduction elements -- the MFMA operand layout.
// The reduction elements of one MFMA are 32 LINES (image rows (n,p) when the taps run along W, image
// columns (n,q) when they run along H) at one position of the line.  With that choice the input operand of
// (gradient position q, tap s) depends on q + s alone: walking along the line, every position loads ONE
// input operand and ONE gradient operand and feeds up to 7 MFMAs -- the gradient operands of the last 7
// positions stay in registers (a sliding window), each tap has its own accumulator.  Positions in the zero
// padding are never multiplied at all.  (The kernel in conv_wgrad.hip reads 8 operands for 7 MFMAs.)
// A 3x3 filter under stride 2 x 2 walks the same way with two input positions per gradient position: with
// pl the padding along the line, gradient position u meets the inputs 2u - pl (tap 0) and 2u - pl + 1 (tap 1),
// and the first of them is also what tap 2 of gradient position u - 1 meets -- three MFMAs per step for one
// gradient operand and two input operands, the previous gradient operand kept in registers.
#include "device_common.h"
#include "kernels.h"
#include "lds_dma.h"

namespace int8t {

typedef int wl_v2i __attribute__((ext_vector_type(2)));
typedef int wl_v4i __attribute__((ext_vector_type(4)));
typedef int wl_v16i __attribute__((ext_vector_type(16)));

constexpr int WL_LINES = 32;                     // lines per chunk: the reduction depth of one MFMA
constexpr int WL_SUB = WL_LINES * 64;            // bytes of one position of 64 channels of one tensor
constexpr int WL_NSTAGE = 2;
// ring stage of a variant: GP positions, each the input's WN and the gradient's WM 64-channel slabs
// (XPS input positions per step: 2 under stride 2)
__host__ __device__ constexpr int wl_stage_bytes(int WM, int WN, int GP, int XPS = 1) { return GP * (WM + XPS * WN) * WL_SUB; }

typedef __attribute__((address_space(3))) wl_v2i* wl_lds_ptr;

// ST taps along the line; a wave owns WM x WN MFMA tiles (32 filters x 32 channels each) per tap, the block's
// four waves (2 x 2) a tile of 64 WM filters x 64 WN channels; GP positions per ring stage.
// S2: stride 2 x 2 (3 taps along the line, one MFMA tile per wave and tap).
template <int ST, int WM, int WN, int GP, bool S2 = false>
__global__ __launch_bounds__(256, 2) void wgrad_lines_kernel(const WgradArgs a) {
    // gradient operands kept: the window (ST positions; 2 under stride 2) plus the one being fetched
    constexpr int NSLOT = S2 ? 3 : ST + 1;
    static_assert(GP % NSLOT == 0, "the window slot of a position must not depend on the stage");
    static_assert((WM == 1 && WN == 1) || (WM == 2 && WN == 2), "loader roles below");
    static_assert(!S2 || (ST == 3 && WM == 1 && WN == 1), "stride 2: 3 taps, one tile per wave and tap");
    constexpr bool BOTH = WM + WN == 4;          // every wave loads both tensors (else waves 0,1 the input, 2,3 the gradient)
    constexpr int XPS = S2 ? 2 : 1;              // input positions per step
    constexpr int STAGE = wl_stage_bytes(WM, WN, GP, XPS);
    constexpr int XPOS = WN * WL_SUB, YPOS = WM * WL_SUB;   // bytes per position
    constexpr int YOFF = GP * XPS * XPOS;                  // gradient slabs follow the input slabs
    extern __shared__ __attribute__((aligned(1024))) unsigned char lsm[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = wave & 1, ch = wave >> 1, half = lane >> 5, l32 = lane & 31;

    // Output tile and reduction share of this block.  Workgroup b runs on XCD b % 8, and the blocks of an
    // XCD should read as few different slices of the two tensors as possible, since each XCD fills its own
    // L2.  With many output tiles (a.xgk > 0) an XCD owns a patch of the (filter tile, channel tile) grid
    // -- xgk x xgc patches, all tap groups and shares of a patch on its XCD: a block reads one filter slice
    // of the gradient and one channel slice of the input, so a patch of pk x pc tiles reads pk + pc slices
    // instead of one pair per tile.  With few tiles and many shares, as in wgrad_kernel: the tiles of one
    // share on one XCD.
    const int out_tiles = a.ktiles * a.ctiles * a.tapgroups;
    int zshare, tg, ct, kt;
    if (a.xgk > 0) {
        const int xcd = (int)(blockIdx.x & 7), i = (int)(blockIdx.x >> 3);
        const int pk = (a.ktiles + a.xgk - 1) / a.xgk, pc = (a.ctiles + a.xgc - 1) / a.xgc;
        const int per_share = pk * pc * a.tapgroups;
        zshare = i / per_share;
        int l = i - zshare * per_share;
        tg = l % a.tapgroups;
        l /= a.tapgroups;
        ct = (xcd % a.xgc) * pc + l % pc;
        kt = (xcd / a.xgc) * pk + l / pc;
        if (kt >= a.ktiles || ct >= a.ctiles) return;
    } else {
        int ot;
        if (wgrad_xcd_mapping(a.splits)) {
            const int wg_i = blockIdx.x >> 3;
            zshare = ((wg_i / out_tiles) << 3) + (int)(blockIdx.x & 7);
            if (zshare >= a.splits) return;
            ot = wg_i % out_tiles;
        } else {
            zshare = blockIdx.x / out_tiles;
            ot = blockIdx.x - zshare * out_tiles;
        }
        tg = ot % a.tapgroups;
        ot /= a.tapgroups;
        ct = ot % a.ctiles;
        kt = ot / a.ctiles;
    }

    // Lines and positions.  along_w: a line is an image row, positions run along W, the block owns tap
    // row tg; otherwise (R x 1 filters) a line is an image column and positions run along H.
    const bool along_w = wgrad_lines_along_w(a.R, a.S);
    const int NLI = along_w ? a.P : a.Q;          // gradient lines per image
    const int QL = along_w ? a.Q : a.P;           // gradient positions on a line
    // A strided 1x1 filter without padding (the shortcut of a residual stage) reads the sub-image of every stride_h-th
    // row and stride_w-th pixel: the same pass on an input of P x Q positions whose lines and positions lie further apart.
    const bool strided = !S2 && (a.stride_h != 1 || a.stride_w != 1);   // (1x1, no padding: wgrad_lines_applies)
    const int WLn = strided ? QL : along_w ? a.W : a.H;          // input positions on a line
    const int pl = along_w ? a.pad_w : a.pad_h;   // padding along the line
    const int XC = strided ? NLI : along_w ? a.H : a.W;           // input lines per image
    const int xshift = along_w ? tg - a.pad_h : -a.pad_w;   // gradient line l pairs with input line l + xshift
    const int t0 = along_w ? tg * a.S : 0;        // first tap of the block (taps numbered r*S + s)
    const uint32_t dy_ls = along_w ? (uint32_t)a.Q * a.Kp : (uint32_t)a.Kp;
    const uint32_t dy_ps = along_w ? (uint32_t)a.Kp : (uint32_t)a.Q * a.Kp;
    const uint32_t x_ls = S2 ? (uint32_t)a.W * a.Cp : along_w ? (uint32_t)a.W * a.Cp * a.stride_h : (uint32_t)a.Cp;
    const uint32_t x_ps = S2 ? (uint32_t)a.Cp : along_w ? (uint32_t)a.Cp * a.stride_w : (uint32_t)a.W * a.Cp;
    // Step u of a line: the gradient position u enters the window, the input position u - pl is
    // multiplied with the gradient positions u, u-1, .., u-ST+1 (taps 0 .. ST-1).  A ring stage holds GP
    // steps of one chunk.  (Letting the stages run on across chunk ends saves the idle steps of a chunk's last
    // stage, but the bookkeeping per step costs more than they do: measured 26 -> 28 us on 14 x 14 images.)
    // Stride 2: step u brings gradient position u and the input positions 2u - pl, 2u - pl + 1; steps 0 .. QL.
    const int U = S2 ? QL + 1 : WLn + pl;
    const int GC = (U + GP - 1) / GP;             // ring stages per chunk
    const int total_lines = a.N * NLI;
    const int c_begin = (int)(((uint32_t)a.chunks * (uint32_t)zshare) / (uint32_t)a.splits);
    const int c_end = (int)(((uint32_t)a.chunks * (uint32_t)(zshare + 1)) / (uint32_t)a.splits);
    const int NS = (c_end - c_begin) * GC;

    // ---- loader role.  A wave-wide load fills 16 lines x 64 channels of one position (1 KB of LDS in lane
    // order).  The 32-byte halves of a line are swapped in lines 4..7 (mod 8): the transposing reads below
    // then touch every LDS bank once.  NLD loads per wave and position: with one MFMA tile per wave and tap,
    // waves 0,1 fetch the input and waves 2,3 the gradient; with 2 x 2, wave w fetches lines 16 (w%2) .. +15 of
    // the 64-channel slab w/2 of both tensors.
    constexpr int NLD = BOTH ? 2 : 1;
    const int myline = 16 * (wave & 1) + (lane >> 2);
    const int gg = (lane & 3) ^ (((myline >> 2) & 1) << 1);           // granule of the line this lane fetches
    const uint32_t lds0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(size_t)lsm);
    wl_v4i rsrc[NLD];
    uint32_t ld_ps[NLD], ld_img[NLD], ld_ls[NLD], ld_dst[NLD], ld_pitch[NLD], ld_base[NLD];
    int ld_npos[NLD], ld_poff[NLD], ld_lshift[NLD], ld_nlines[NLD], ld_chan[NLD];
    bool ld_chan_ok[NLD];
    const bool ld_input = !BOTH && (wave >> 1) == 0;        // (stride 2) this wave fetches the input
    const int ld_lmul = (S2 && ld_input) ? 2 : 1;           // gradient line l of an image pairs with input line 2l + xshift
#pragma unroll
    for (int e = 0; e < NLD; ++e) {
        const int tensor = BOTH ? e : (wave >> 1);              // 0: input codes, 1: gradient codes
        const int sub = BOTH ? (wave >> 1) : 0;
        rsrc[e] = igd_rsrc(tensor ? (const void*)a.dy : (const void*)a.x,
                           tensor ? (uint32_t)a.N * a.P * a.Q * a.Kp : (uint32_t)a.N * a.H * a.W * a.Cp);
        ld_ls[e] = tensor ? dy_ls : x_ls;
        ld_ps[e] = tensor ? dy_ps : x_ps;
        ld_img[e] = tensor ? (uint32_t)a.P * a.Q * a.Kp : (uint32_t)a.H * a.W * a.Cp;
        ld_npos[e] = tensor ? QL : WLn;
        ld_poff[e] = tensor ? 0 : pl;
        ld_lshift[e] = tensor ? 0 : xshift;
        ld_nlines[e] = tensor ? NLI : XC;
        ld_chan[e] = (tensor ? kt * (64 * WM) : ct * (64 * WN)) + 64 * sub + 16 * gg;
        ld_chan_ok[e] = ld_chan[e] < (tensor ? a.Kp : a.Cp);
        ld_pitch[e] = tensor ? YPOS : XPOS;
        ld_dst[e] = lds0 + (uint32_t)((tensor ? YOFF : 0) + sub * WL_SUB + (wave & 1) * 1024);
        ld_base[e] = IGD_OOB;
    }
    // byte offset of this lane's line in chunk `chunk` (IGD_OOB: no such line -- zeros are loaded)
    auto line_base = [&](int e, int chunk) -> uint32_t {
        const int L = chunk * WL_LINES + myline;
        if (chunk >= c_end || L >= total_lines || !ld_chan_ok[e]) return IGD_OOB;
        const int n = L / NLI;
        const int l = (L - n * NLI) * ld_lmul + ld_lshift[e];
        if ((unsigned)l >= (unsigned)ld_nlines[e]) return IGD_OOB;
        return (uint32_t)n * ld_img[e] + (uint32_t)l * ld_ls[e] + (uint32_t)ld_chan[e];
    };
    int lc = c_begin, lg = 0;           // chunk and stage (of the chunk) that is fetched next
#pragma unroll
    for (int e = 0; e < NLD; ++e) ld_base[e] = line_base(e, lc);
    auto issue = [&](int slot) {
#pragma unroll
        for (int j = 0; j < GP; ++j) {
            if (S2) {
                if (ld_input) {
#pragma unroll
                    for (int h = 0; h < 2; ++h) {
                        const int pos = 2 * (lg * GP + j) - pl + h;
                        const bool ok = ld_base[0] != IGD_OOB && (unsigned)pos < (unsigned)ld_npos[0];
                        igd_load_lds(rsrc[0], ld_dst[0] + (uint32_t)slot * STAGE + (uint32_t)(2 * j + h) * XPOS,
                                     ok ? ld_base[0] + (uint32_t)pos * ld_ps[0] : IGD_OOB);
                    }
                } else {
                    const int pos = lg * GP + j;
                    const bool ok = ld_base[0] != IGD_OOB && (unsigned)pos < (unsigned)ld_npos[0];
                    igd_load_lds(rsrc[0], ld_dst[0] + (uint32_t)slot * STAGE + (uint32_t)j * YPOS,
                                 ok ? ld_base[0] + (uint32_t)pos * ld_ps[0] : IGD_OOB);
                }
                continue;
            }
#pragma unroll
            for (int e = 0; e < NLD; ++e) {
                const int pos = lg * GP + j - ld_poff[e];
                const bool ok = ld_base[e] != IGD_OOB && (unsigned)pos < (unsigned)ld_npos[e];
                igd_load_lds(rsrc[e], ld_dst[e] + (uint32_t)slot * STAGE + (uint32_t)j * ld_pitch[e],
                             ok ? ld_base[e] + (uint32_t)pos * ld_ps[e] : IGD_OOB);
            }
        }
        if (++lg == GC) {
            lg = 0;
            ++lc;
#pragma unroll
            for (int e = 0; e < NLD; ++e) ld_base[e] = line_base(e, lc);
        }
    };

    // ---- operand role: wave (mt, ch) owns WM x WN MFMA tiles.  Chunk address of this lane for the first of
    // an operand's two reads (the second: 8 lines on, +512 B).
    const int rl = ((lane & 15) >> 1) + 16 * half;
    const int b2 = (lane >> 3) & 1, hi = (lane >> 4) & 1;
    const uint32_t rd_common = (uint32_t)(rl * 64 + 16 * hi + 8 * (lane & 1));
    uint32_t offA[WM], offB[WN];
#pragma unroll
    for (int i = 0; i < WM; ++i) offA[i] = YOFF + rd_common + (WM == 2 ? (uint32_t)(mt * WL_SUB) + 32u * (uint32_t)(i ^ b2) : 32u * (uint32_t)(mt ^ b2));
#pragma unroll
    for (int i = 0; i < WN; ++i) offB[i] = rd_common + (WN == 2 ? (uint32_t)(ch * WL_SUB) + 32u * (uint32_t)(i ^ b2) : 32u * (uint32_t)(ch ^ b2));

    wl_v16i acc[ST][WM][WN];
#pragma unroll
    for (int s = 0; s < ST; ++s)
#pragma unroll
        for (int i = 0; i < WM; ++i)
#pragma unroll
            for (int k = 0; k < WN; ++k)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[s][i][k][v] = 0;
    wl_v4i A[NSLOT][WM];
#pragma unroll
    for (int s = 0; s < NSLOT; ++s)
#pragma unroll
        for (int i = 0; i < WM; ++i) A[s][i] = wl_v4i{0, 0, 0, 0};

    if (NS > 0) issue(0);
    int g = 0;                          // stage (of its chunk) that is multiplied next
    for (int i = 0; i < NS; ++i) {
        igd_wait_vmcnt<0>();            // this wave's loads of stage i have landed ...
        __syncthreads();                // ... and everyone's; all waves are done with stage i-1's slot
        if (i + 1 < NS) issue((i + 1) & 1);
        const uint32_t sbase = lds0 + (uint32_t)(i & 1) * STAGE;
        auto fetch = [&](uint32_t off, int bytes) -> wl_v4i {
            const wl_lds_ptr p = (wl_lds_ptr)(uintptr_t)(sbase + off);
            const wl_v2i r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(p + bytes / 8);
            const wl_v2i r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(p + (bytes + 512) / 8);
            return wl_v4i{r0.x, r0.y, r1.x, r1.y};
        };
        if constexpr (S2) {
            wl_v4i Ba_n = fetch(offB[0], 0), Bb_n = fetch(offB[0], XPOS);
            A[0][0] = fetch(offA[0], 0);
#pragma unroll
            for (int j = 0; j < GP; ++j) {
                const wl_v4i Ba = Ba_n, Bb = Bb_n;
                if (j + 1 < GP) {
                    A[(j + 1) % NSLOT][0] = fetch(offA[0], (j + 1) * YPOS);
                    Ba_n = fetch(offB[0], (2 * j + 2) * XPOS);
                    Bb_n = fetch(offB[0], (2 * j + 3) * XPOS);
                }
                const int u = g * GP + j;
                if (__builtin_expect(u < QL, 1)) {
                    acc[0][0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[j % NSLOT][0], Ba, acc[0][0][0], 0, 0, 0);
                    acc[1][0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[j % NSLOT][0], Bb, acc[1][0][0], 0, 0, 0);
                }
                // tap 2 of the previous gradient position (none at the start of a line; the last step has only this)
                if (__builtin_expect(u >= 1 && u <= QL, 1))
                    acc[2][0][0] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[(j + NSLOT - 1) % NSLOT][0], Ba, acc[2][0][0], 0, 0, 0);
            }
            if (++g == GC) g = 0;
            continue;
        }
        wl_v4i Bn[WN], Bc[WN];
#pragma unroll
        for (int k = 0; k < WN; ++k) Bn[k] = fetch(offB[k], 0);
#pragma unroll
        for (int k = 0; k < WM; ++k) A[0][k] = fetch(offA[k], 0);
#pragma unroll
        for (int j = 0; j < GP; ++j) {
#pragma unroll
            for (int k = 0; k < WN; ++k) Bc[k] = Bn[k];
            if (j + 1 < GP) {
#pragma unroll
                for (int k = 0; k < WM; ++k) A[(j + 1) % NSLOT][k] = fetch(offA[k], (j + 1) * YPOS);
#pragma unroll
                for (int k = 0; k < WN; ++k) Bn[k] = fetch(offB[k], (j + 1) * XPOS);
            }
            const int u = g * GP + j;
            if (__builtin_expect((unsigned)(u - pl) < (unsigned)WLn, 1)) {
#pragma unroll
                for (int s = 0; s < ST; ++s) {
                    if (__builtin_expect((unsigned)(u - s) < (unsigned)QL, 1)) {
#pragma unroll
                        for (int m = 0; m < WM; ++m)
#pragma unroll
                            for (int k = 0; k < WN; ++k)
                                acc[s][m][k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[(j - s + NSLOT) % NSLOT][m], Bc[k],
                                                                                     acc[s][m][k], 0, 0, 0);
                    }
                }
            }
        }
        if (++g == GC) g = 0;
    }

    // partial[z][k][(tap,c)], channel fastest: 32 consecutive columns per store instruction
    const int ncolsp = a.R * a.S * a.Cp;
    int32_t* __restrict__ part = a.partial + (size_t)zshare * a.K * ncolsp;
#pragma unroll
    for (int k2 = 0; k2 < WN; ++k2) {
        const int c = ct * (64 * WN) + (ch * WN + k2) * 32 + l32;
        if (c >= a.Cp) continue;
#pragma unroll
        for (int s = 0; s < ST; ++s) {
            const int col = (t0 + s) * a.Cp + c;
#pragma unroll
            for (int m = 0; m < WM; ++m)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int k = kt * (64 * WM) + (mt * WM + m) * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                    if (k < a.K) part[(size_t)k * ncolsp + col] = acc[s][m][k2][v];
                }
        }
    }
}

// the stride-2 form of the kernel: 3x3 filters, stride 2 x 2
bool wgrad_lines_s2(const WgradArgs& a) {
    return a.R == 3 && a.S == 3 && a.stride_h == 2 && a.stride_w == 2 && a.pad_h <= 2 && a.pad_w <= 2;
}

bool wgrad_lines_applies(const WgradArgs& a) {
    const bool one = a.R == 1 && a.S == 1;
    if (a.s2d) return false;
    // strides: 1x1 filters without padding (the pass then runs on every stride-th row and pixel), and 3x3 filters
    // under stride 2 x 2
    if ((a.stride_h != 1 || a.stride_w != 1) && !(one && a.pad_h == 0 && a.pad_w == 0) && !wgrad_lines_s2(a)) return false;
    const bool along_w = a.S == 3 || a.S == 7;
    const bool along_h = a.S == 1 && (a.R == 3 || a.R == 7);
    if (!one && !along_w && !along_h) return false;
    // byte offsets into either tensor stay below the value that stands for "nothing to load"
    if ((unsigned long long)a.N * a.H * a.W * a.Cp >= IGD_OOB || (unsigned long long)a.N * a.P * a.Q * a.Kp >= IGD_OOB) return false;
    return true;
}

void wgrad_plan_lines(WgradArgs* a) {
    const bool along_w = wgrad_lines_along_w(a->R, a->S);
    const int ST = along_w ? a->S : a->R;
    const int WT = ST == 1 ? 2 : 1;              // MFMA tiles per wave and tap in each direction
    const bool s2 = wgrad_lines_s2(*a);
    const int GP = ST == 1 ? 4 : s2 ? 3 : 8;
    a->lines = 1;
    a->TB = ST;
    a->CS = WT;
    a->BP = a->BQ = a->ntp = a->ntq = a->ngrp = 0;
    a->xt_slots = 0;
    a->tapgroups = along_w ? a->R : 1;
    a->ktiles = (a->K + 64 * WT - 1) / (64 * WT);
    a->ctiles = (a->Cp + 64 * WT - 1) / (64 * WT);
    const int NLI = along_w ? a->P : a->Q;
    const int QL = along_w ? a->Q : a->P;
    const int WLn = (a->stride_h != 1 || a->stride_w != 1) ? QL : along_w ? a->W : a->H;
    const int pl = s2 ? 1 : along_w ? a->pad_w : a->pad_h;      // (stride 2: QL + 1 steps per chunk)
    a->chunks = (a->N * NLI + WL_LINES - 1) / WL_LINES;
    a->lds_bytes = (size_t)WL_NSTAGE * wl_stage_bytes(WT, WT, GP, s2 ? 2 : 1);
    // Split count by the same estimate as wgrad_plan(): rounds of resident blocks (two per compute unit),
    // a block pays a prologue plus its stages, every split one write and one read of the partial tiles.
    const int out_tiles = a->ktiles * a->ctiles * a->tapgroups;
    const int slots = 512;
    const double stages_per_chunk = (double)(WLn + pl) / GP;
    const double mfma_per_chunk = (double)QL * ST * WT * WT;   // per wave, a little less at the image border
    const double t_chunk = stages_per_chunk * 0.45 + 0.014 * 2.0 * mfma_per_chunk;
    const double t_partial = (double)a->K * a->R * a->S * a->Cp * 8.0 / 4.0e6;
    int splits = 1;
    double best = 1e30;
    for (int sp = 1; sp <= a->chunks && sp <= 4096; ++sp) {
        const long long blocks = (long long)out_tiles * sp;
        const double rounds = (double)((blocks + slots - 1) / slots);
        const double t = rounds * (3.0 + ((a->chunks + sp - 1) / sp) * t_chunk) + sp * t_partial;
        if (t < best) { best = t; splits = sp; }
        if (blocks > 8LL * slots || (long long)a->chunks * (sp + 2) >= (1LL << 31)) break;
    }
    if (a->variant == VAR_WGRAD_FEWER) splits = splits > 1 ? splits / 2 : 1;
    if (a->variant == VAR_WGRAD_MORE) splits = (2 * splits <= a->chunks && 2 * splits <= 4096) ? 2 * splits : splits;
    a->splits = splits;
    // XCD patches (see the kernel): the split of 8 into xgk x xgc whose patches read the fewest slices
    a->xgk = a->xgc = 0;
    if (a->ktiles * a->ctiles >= 16) {
        int best = 1 << 30;
        for (int gk = 1; gk <= 8; gk *= 2) {
            const int gc = 8 / gk;
            if (gk > a->ktiles || gc > a->ctiles) continue;
            const int cost = (a->ktiles + gk - 1) / gk + (a->ctiles + gc - 1) / gc;
            if (cost < best) { best = cost; a->xgk = gk; a->xgc = gc; }
        }
    }
}

unsigned wgrad_lines_grid(const WgradArgs& a) {
    const unsigned out_tiles = (unsigned)(a.ktiles * a.ctiles * a.tapgroups);
    if (a.xgk > 0) {
        const unsigned pk = (unsigned)((a.ktiles + a.xgk - 1) / a.xgk), pc = (unsigned)((a.ctiles + a.xgc - 1) / a.xgc);
        return 8u * pk * pc * (unsigned)a.tapgroups * (unsigned)a.splits;
    }
    return wgrad_xcd_mapping(a.splits) ? out_tiles * 8u * (unsigned)((a.splits + 7) / 8) : out_tiles * (unsigned)a.splits;
}

hipError_t launch_wgrad_lines(const WgradArgs& a, hipStream_t st) {
    const dim3 grid(wgrad_lines_grid(a));
    KernelTimer kt(KID_WGRAD_LINES, st);
#define LAUNCH(STv, WTv, GPv, S2v)                                                                       \
    do {                                                                                                 \
        static std::atomic<unsigned long long> attr_done;                                                \
        hipError_t ea = raise_dynamic_lds(reinterpret_cast<const void*>(wgrad_lines_kernel<STv, WTv, WTv, GPv, S2v>), \
                                          WL_NSTAGE * wl_stage_bytes(WTv, WTv, GPv, S2v ? 2 : 1), attr_done); \
        if (ea != hipSuccess) return ea;                                                                 \
        launch_timed(kt, (wgrad_lines_kernel<STv, WTv, WTv, GPv, S2v>), grid, dim3(256), a.lds_bytes, st, a); \
    } while (0)
    if (a.TB == 3 && wgrad_lines_s2(a)) LAUNCH(3, 1, 3, true);
    else if (a.TB == 3) LAUNCH(3, 1, 8, false);
    else if (a.TB == 7) LAUNCH(7, 1, 8, false);
    else if (a.TB == 1) LAUNCH(1, 2, 4, false);
    else return hipErrorInvalidValue;
#undef LAUNCH
    return hipGetLastError();
}

}  // namespace int8t
