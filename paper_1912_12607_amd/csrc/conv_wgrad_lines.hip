// Dense backward-weight convolution (Sec.3.4: g_W = g_z^T a) for stride-1 filters with 3 or 7 taps along
// one image axis, on int8 MFMA with int32 accumulation.  Same result, partial-tile format and final
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
#include "device_common.h"
#include "kernels.h"
#include "lds_dma.h"

namespace int8t {

typedef int wl_v2i __attribute__((ext_vector_type(2)));
typedef int wl_v4i __attribute__((ext_vector_type(4)));
typedef int wl_v16i __attribute__((ext_vector_type(16)));

constexpr int WL_LINES = 32;                     // lines per chunk: the reduction depth of one MFMA
constexpr int WL_GP = 8;                         // positions per ring stage
constexpr int WL_SLAB = WL_LINES * 64;           // bytes of one position of one tensor: 32 lines x 64 channels
constexpr int WL_STAGE = 2 * WL_GP * WL_SLAB;    // input slabs, then gradient slabs
constexpr int WL_NSTAGE = 2;
constexpr int WL_BM = 64;                        // filters per block

typedef __attribute__((address_space(3))) wl_v2i* wl_lds_ptr;

template <int ST>
__global__ __launch_bounds__(256, 2) void wgrad_lines_kernel(const WgradArgs a) {
    constexpr int NSLOT = ST + 1;                // gradient operands kept: the window of ST plus the one being fetched
    static_assert(WL_GP % NSLOT == 0, "the window slot of a position must not depend on the stage");
    extern __shared__ __attribute__((aligned(1024))) unsigned char lsm[];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int mt = wave & 1, ch = wave >> 1, half = lane >> 5, l32 = lane & 31;

    // output tile and reduction share of this block: as in wgrad_kernel (shares of one XCD are neighbours)
    const int out_tiles = a.ktiles * a.ctiles * a.tapgroups;
    int zshare, ot;
    if (wgrad_xcd_mapping(a.splits)) {
        const int wg_i = blockIdx.x >> 3;
        zshare = ((wg_i / out_tiles) << 3) + (int)(blockIdx.x & 7);
        if (zshare >= a.splits) return;
        ot = wg_i % out_tiles;
    } else {
        zshare = blockIdx.x / out_tiles;
        ot = blockIdx.x - zshare * out_tiles;
    }
    const int tg = ot % a.tapgroups;
    ot /= a.tapgroups;
    const int ct = ot % a.ctiles;
    const int kt = ot / a.ctiles;

    // Lines and positions.  along_w: a line is an image row, positions run along W, the block owns tap
    // row tg; otherwise (R x 1 filters) a line is an image column and positions run along H.
    const bool along_w = a.S > 1;
    const int NLI = along_w ? a.P : a.Q;          // gradient lines per image
    const int QL = along_w ? a.Q : a.P;           // gradient positions on a line
    const int WLn = along_w ? a.W : a.H;          // input positions on a line
    const int pl = along_w ? a.pad_w : a.pad_h;   // padding along the line
    const int XC = along_w ? a.H : a.W;           // input lines per image
    const int xshift = along_w ? tg - a.pad_h : -a.pad_w;   // gradient line l pairs with input line l + xshift
    const int t0 = along_w ? tg * a.S : 0;        // first tap of the block (taps numbered r*S + s)
    const uint32_t dy_ls = along_w ? (uint32_t)a.Q * a.Kp : (uint32_t)a.Kp;
    const uint32_t dy_ps = along_w ? (uint32_t)a.Kp : (uint32_t)a.Q * a.Kp;
    const uint32_t x_ls = along_w ? (uint32_t)a.W * a.Cp : (uint32_t)a.Cp;
    const uint32_t x_ps = along_w ? (uint32_t)a.Cp : (uint32_t)a.W * a.Cp;
    // Step u of a line: the gradient position u enters the window, the input position u - pl is
    // multiplied with the gradient positions u, u-1, .., u-ST+1 (taps 0 .. ST-1).
    const int U = WLn + pl;
    const int GC = (U + WL_GP - 1) / WL_GP;       // ring stages per chunk
    const int total_lines = a.N * NLI;

    // ---- loader role: waves 0,1 fetch the input, waves 2,3 the gradient; a wave-wide load fills 16 lines
    // x 64 channels of one position (1 KB of LDS in lane order).  The 32-byte halves of a line are swapped
    // in lines 4..7 (mod 8): the transposing reads below then touch every LDS bank once.
    const int tensor = wave >> 1;
    const int myline = 16 * (wave & 1) + (lane >> 2);
    const int gg = (lane & 3) ^ (((myline >> 2) & 1) << 1);           // granule of the line this lane fetches
    const int chan = (tensor ? kt * WL_BM : ct * 64) + 16 * gg;
    const bool chan_ok = chan < (tensor ? a.Kp : a.Cp);
    const wl_v4i rsrc = igd_rsrc(tensor ? (const void*)a.dy : (const void*)a.x,
                                 tensor ? (uint32_t)a.N * a.P * a.Q * a.Kp : (uint32_t)a.N * a.H * a.W * a.Cp);
    const uint32_t my_ls = tensor ? dy_ls : x_ls, my_ps = tensor ? dy_ps : x_ps;
    const uint32_t my_img = tensor ? (uint32_t)a.P * a.Q * a.Kp : (uint32_t)a.H * a.W * a.Cp;
    const int my_npos = tensor ? QL : WLn, my_poff = tensor ? 0 : pl;
    const int my_lshift = tensor ? 0 : xshift, my_nlines = tensor ? NLI : XC;
    const uint32_t lds0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(size_t)lsm);
    const uint32_t lds_mine = lds0 + (uint32_t)(tensor * WL_GP * WL_SLAB + (wave & 1) * 1024);

    // byte offset of this lane's line in chunk `chunk` (IGD_OOB: no such line -- zeros are loaded)
    auto line_base = [&](int chunk) -> uint32_t {
        const int L = chunk * WL_LINES + myline;
        if (L >= total_lines || !chan_ok) return IGD_OOB;
        const int n = L / NLI;
        const int l = L - n * NLI + my_lshift;
        if ((unsigned)l >= (unsigned)my_nlines) return IGD_OOB;
        return (uint32_t)n * my_img + (uint32_t)l * my_ls + (uint32_t)chan;
    };
    auto issue = [&](uint32_t lb, int g, int slot) {
        const uint32_t dst = lds_mine + (uint32_t)slot * WL_STAGE;
        int pos = g * WL_GP - my_poff;
#pragma unroll
        for (int j = 0; j < WL_GP; ++j, ++pos) {
            const bool ok = lb != IGD_OOB && (unsigned)pos < (unsigned)my_npos;
            igd_load_lds(rsrc, dst + (uint32_t)j * WL_SLAB, ok ? lb + (uint32_t)pos * my_ps : IGD_OOB);
        }
    };

    // ---- operand role: wave (mt, ch) owns filters 32 mt .. +31 and channels 32 ch .. +31 of the block's tile.
    // Chunk address of this lane for the first of an operand's two reads (the second: 8 lines on, +512 B).
    const int rl = ((lane & 15) >> 1) + 16 * half;
    const int b2 = (lane >> 3) & 1, hi = (lane >> 4) & 1;
    const uint32_t rd_common = (uint32_t)(rl * 64 + 16 * hi + 8 * (lane & 1));
    const uint32_t offA = (uint32_t)(WL_GP * WL_SLAB) + rd_common + 32u * (uint32_t)(mt ^ b2);
    const uint32_t offB = rd_common + 32u * (uint32_t)(ch ^ b2);

    wl_v16i acc[ST];
#pragma unroll
    for (int s = 0; s < ST; ++s)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[s][v] = 0;
    wl_v4i A[NSLOT];
#pragma unroll
    for (int s = 0; s < NSLOT; ++s) A[s] = wl_v4i{0, 0, 0, 0};

    const int c_begin = (int)(((uint32_t)a.chunks * (uint32_t)zshare) / (uint32_t)a.splits);
    const int c_end = (int)(((uint32_t)a.chunks * (uint32_t)(zshare + 1)) / (uint32_t)a.splits);
    const int NS = (c_end - c_begin) * GC;

    int ci = c_begin, gi = 0;           // stage that is fetched next
    uint32_t lb = IGD_OOB;
    if (NS > 0) {
        lb = line_base(ci);
        issue(lb, 0, 0);
        if (++gi == GC) { gi = 0; ++ci; if (ci < c_end) lb = line_base(ci); }
    }
    int g = 0;                          // stage that is multiplied next (its chunk does not matter any more)
    for (int i = 0; i < NS; ++i) {
        igd_wait_vmcnt<0>();            // this wave's loads of stage i have landed ...
        __syncthreads();                // ... and everyone's; all waves are done with stage i-1's slot
        if (i + 1 < NS) {
            issue(lb, gi, (i + 1) & 1);
            if (++gi == GC) { gi = 0; ++ci; if (ci < c_end) lb = line_base(ci); }
        }
        const wl_lds_ptr pa = (wl_lds_ptr)(uintptr_t)(lds0 + (uint32_t)(i & 1) * WL_STAGE + offA);
        const wl_lds_ptr pb = (wl_lds_ptr)(uintptr_t)(lds0 + (uint32_t)(i & 1) * WL_STAGE + offB);
        auto fetch = [&](wl_lds_ptr p, int j) -> wl_v4i {
            const wl_v2i r0 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(p + (j * WL_SLAB) / 8);
            const wl_v2i r1 = __builtin_amdgcn_ds_read_tr8_b64_v2i32(p + (j * WL_SLAB + 512) / 8);
            return wl_v4i{r0.x, r0.y, r1.x, r1.y};
        };
        const int u0 = g * WL_GP;
        wl_v4i Bn = fetch(pb, 0), Bc;
        A[0] = fetch(pa, 0);
#pragma unroll
        for (int j = 0; j < WL_GP; ++j) {
            Bc = Bn;
            if (j + 1 < WL_GP) {
                A[(j + 1) % NSLOT] = fetch(pa, j + 1);
                Bn = fetch(pb, j + 1);
            }
            const int u = u0 + j;
            if ((unsigned)(u - pl) < (unsigned)WLn) {
#pragma unroll
                for (int s = 0; s < ST; ++s) {
                    if ((unsigned)(u - s) < (unsigned)QL)
                        acc[s] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[(j - s + NSLOT) % NSLOT], Bc, acc[s], 0, 0, 0);
                }
            }
        }
        if (++g == GC) g = 0;
    }

    // partial[z][k][(tap,c)], channel fastest: 32 consecutive columns per store instruction
    const int ncolsp = a.R * a.S * a.Cp;
    int32_t* __restrict__ part = a.partial + (size_t)zshare * a.K * ncolsp;
    const int c = ct * 64 + ch * 32 + l32;
    if (c < a.Cp) {
#pragma unroll
        for (int s = 0; s < ST; ++s) {
            const int col = (t0 + s) * a.Cp + c;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kt * WL_BM + mt * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (k < a.K) part[(size_t)k * ncolsp + col] = acc[s][v];
            }
        }
    }
}

bool wgrad_lines_applies(const WgradArgs& a) {
    if (a.s2d || a.stride_h != 1 || a.stride_w != 1) return false;
    const bool along_w = a.S == 3 || a.S == 7;
    const bool along_h = a.S == 1 && (a.R == 3 || a.R == 7);
    if (!along_w && !along_h) return false;
    // byte offsets into either tensor stay below the value that stands for "nothing to load"
    if ((unsigned long long)a.N * a.H * a.W * a.Cp >= IGD_OOB || (unsigned long long)a.N * a.P * a.Q * a.Kp >= IGD_OOB) return false;
    return true;
}

void wgrad_plan_lines(WgradArgs* a) {
    const bool along_w = a->S > 1;
    const int ST = along_w ? a->S : a->R;
    a->lines = 1;
    a->TB = ST;
    a->CS = 1;
    a->BP = a->BQ = a->ntp = a->ntq = a->ngrp = 0;
    a->xt_slots = 0;
    a->tapgroups = along_w ? a->R : 1;
    a->ktiles = (a->K + WL_BM - 1) / WL_BM;
    a->ctiles = (a->Cp + 63) / 64;
    const int NLI = along_w ? a->P : a->Q;
    const int QL = along_w ? a->Q : a->P;
    const int WLn = along_w ? a->W : a->H;
    const int pl = along_w ? a->pad_w : a->pad_h;
    a->chunks = (a->N * NLI + WL_LINES - 1) / WL_LINES;
    a->lds_bytes = (size_t)WL_NSTAGE * WL_STAGE;
    const int GC = (WLn + pl + WL_GP - 1) / WL_GP;
    // Split count by the same estimate as wgrad_plan(): rounds of resident blocks (two per compute unit),
    // a block pays a prologue plus its stages, every split one write and one read of the partial tiles.
    const int out_tiles = a->ktiles * a->ctiles * a->tapgroups;
    const int slots = 512;
    const double mfma_per_chunk = (double)QL * ST;   // per wave, a little less at the image border
    const double t_chunk = GC * 0.45 + 0.014 * 2.0 * mfma_per_chunk;
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
}

hipError_t launch_wgrad_lines(const WgradArgs& a, dim3 grid, hipStream_t st) {
    KernelTimer kt(KID_WGRAD_LINES, st);
#define LAUNCH(STv)                                                                                      \
    do {                                                                                                 \
        static std::atomic<unsigned long long> attr_done;                                                \
        hipError_t ea = raise_dynamic_lds(reinterpret_cast<const void*>(wgrad_lines_kernel<STv>),        \
                                          WL_NSTAGE * WL_STAGE, attr_done);                              \
        if (ea != hipSuccess) return ea;                                                                 \
        launch_timed(kt, (wgrad_lines_kernel<STv>), grid, dim3(256), a.lds_bytes, st, a);                \
    } while (0)
    if (a.TB == 3) LAUNCH(3);
    else if (a.TB == 7) LAUNCH(7);
    else return hipErrorInvalidValue;
#undef LAUNCH
    return hipGetLastError();
}

}  // namespace int8t
