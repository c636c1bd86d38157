// Dense backward-weight convolution on int8 codes (Sec.3.4: g_W = g_z^T a), int8 MFMA with int32
// accumulation, Eq.2 fused into the final reduction.
//
// GEMM view:  D[k][(tap,c)] = sum over (n,p,q) of  Gz[(n,p,q)][k] * A[(n, p*sh+r-ph, q*sw+s-pw)][c]
// The reduction runs over images and output pixels, but the channels-last code tensors keep the
// channel innermost, while the MFMA wants 16 consecutive reduction bytes per lane.  Any order of
// the reduction index is as good as any other, so the 16 bytes of a lane are made 16 different
// IMAGES at one pixel: a loader task fetches, for one pixel, the 16-channel granule of each of 16
// images (sixteen 16-byte loads), transposes the 16x16 byte block in registers with byte permutes
// -- built from the "4x4 8-bit integer block transpose" of the paper's Suppl. "INT8 Convolution"
// -- and stores [pixel][channel][16 images] granules to LDS.  A filter tap is then just a different
// PIXEL of the staged input window, i.e. a different, always 16-byte aligned LDS row: no im2col
// buffer, no unaligned operand reads, zero padding is written once by the loader.
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
constexpr int W2_LDS_BUDGET = 72 * 1024;   // two blocks per compute unit
// LDS tiles are [pixel][channels] in 16-byte granules with a pixel pitch of (channels + 4)
// granules, and inside each aligned group of 16 channels the position is xor-ed with the group's
// number.  The 16 consecutive loader lanes (4 or 16 channel granules per pixel, consecutive pixels)
// store the same channel-in-granule and land in 16 different bank groups (the xor separates the
// granules of a pixel, the pitch separates the pixels); the MFMA operand reads (32 consecutive
// channels of one pixel) are a permutation inside each group.  The pixel part stays linear, so a
// filter tap is a constant address offset.
constexpr int W2_PAD = 4;
__device__ __forceinline__ int swz_ch(int c) { return (c & ~15) | ((c & 15) ^ ((c >> 4) & 15)); }

// Component q of a 16-byte register granule.
__device__ __forceinline__ uint32_t comp(const uint4& v, int q) { return q == 0 ? v.x : q == 1 ? v.y : q == 2 ? v.z : v.w; }

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

constexpr int W2_MAXSTEPS = 16;        // MFMA steps per chunk: at most 32 tile pixels


// PK (tensors of 16 channels -- the space-to-depth image of a stem: TB = 4, CS = 1): the block's 64 columns are its
// four taps x 16 channels, not 64 channels of which 48 do not exist: a column's operand is the channel granule of the
// window pixel its tap points at, so one MFMA per step serves four taps, and a window pixel is one granule to stage,
// not four (7x7 stem of ResNet-50, batch 64: the 4 x 4 taps of the rewritten layer took 16 blocks of a quarter-full
// tile each).
template <int TB, int CS, bool PK = false>
__global__ __launch_bounds__(256, 2) void wgrad_kernel(const WgradArgs a) {
    static_assert(!PK || (TB == 4 && CS == 1), "packed taps: four taps of 16 channels");
    constexpr int CT = PK ? 16 : 64 * CS;         // channels staged per pixel
    constexpr int TBA = PK ? 1 : TB;              // accumulator tiles per wave along the taps
    constexpr int XP = CT + W2_PAD;               // pixel pitch of the input window tile
    constexpr int YP = W2_BM + W2_PAD;            // pixel pitch of the gradient tile
    static_assert(CS == 1 || CS == 4, "channel tile is 64 or 256");
    extern __shared__ __attribute__((aligned(16))) uint4 lds[];
    uint4* __restrict__ xT = lds;                   // [window pixel][CT channels] granules
    uint4* __restrict__ dyT = lds + a.xt_slots;     // [tile pixel][64 filters] granules, then one all-zero pixel

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int mt = wave & 1, ch = wave >> 1, half = lane >> 5, l32 = lane & 31;

    // Workgroups are dealt to the 8 XCDs round-robin (workgroup b runs on XCD b % 8).  The output
    // tiles of one reduction share -- the tap groups, channel and filter tiles that read the same
    // input and gradient pixels -- are given to consecutive workgroups of ONE XCD, so those pixels
    // are fetched into that XCD's L2 once.  Share z = 8 * (i / tiles) + xcd, tile = i % tiles, with
    // i = b / 8; the grid is padded to whole groups of 8 shares and the surplus workgroups leave.
    // With few shares (and not a multiple of 8) that would idle XCDs: then tiles simply follow each
    // other.
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
    const int RS = a.R * a.S;
    const int t0 = tg * TB;
    const int nt = (RS - t0 < TB) ? (RS - t0) : TB;
    int rmin, rmax, smin, smax;
    tap_extent(t0, nt, a.S, &rmin, &rmax, &smin, &smax);
    const int WH = (a.BP - 1) * a.stride_h + (rmax - rmin) + 1;
    const int WW = (a.BQ - 1) * a.stride_w + (smax - smin) + 1;
    int tpix[TB];   // uniform: LDS offset (granules) of each tap's pixel shift
#pragma unroll
    for (int j = 0; j < TB; ++j) {
        const int t = t0 + ((j < nt) ? j : 0);
        tpix[j] = __builtin_amdgcn_readfirstlane(((t / a.S - rmin) * WW + (t % a.S - smin)) * XP);
    }
    const int units = a.BP * a.BQ;
    const int nsteps = (units + 1) >> 1;
    // one all-zero tile pixel behind the real ones: the partner of the last pixel of an odd tile
    if (tid < W2_BM) dyT[units * YP + tid] = make_uint4(0, 0, 0, 0);
    // LDS operand positions of every MFMA step; they depend on the tile geometry only.  A step
    // feeds two tile pixels, one per half-wave, each with 16 images.  Entry u = 2*step + half:
    // {granule offset of the gradient tile pixel, granule offset of its window pixel}.
    int2* __restrict__ stab = reinterpret_cast<int2*>(dyT + (units + 1) * YP);
    if (tid < 2 * W2_MAXSTEPS) {
        const int u = tid;
        const bool uv = u < units;
        const int uu = uv ? u : 0;
        const int pl = uu / a.BQ, ql = uu - pl * a.BQ;
        stab[u] = make_int2((uv ? u : units) * YP, (pl * a.stride_h * WW + ql * a.stride_w) * XP);
    }
    // gradient operand of step s: tile pixel 2*s + half (the pixel `units` is the all-zero one)
    const int a_ch = swz_ch(mt * 32 + l32) + half * YP;
    int x_ch[CS];                                   // this lane's channel positions inside the block's tile
#pragma unroll
    for (int i = 0; i < CS; ++i) x_ch[i] = swz_ch((ch * CS + i) * 32 + l32);
    if (PK) {
        // column 32 * ch + l32 = tap 2 * ch + l32 / 16 of the block's four, channel l32 % 16 (a single group of 16: no xor)
        const int tlo = ch ? tpix[2 % TB] : tpix[0], thi = ch ? tpix[3 % TB] : tpix[1 % TB];
        x_ch[0] = ((l32 >> 4) ? thi : tlo) + (l32 & 15);
    }

    v16i acc[TBA][CS];
#pragma unroll
    for (int j = 0; j < TBA; ++j)
#pragma unroll
        for (int i = 0; i < CS; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[j][i][v] = 0;

    // window pixel of this half-wave in every step: the same for all chunks, kept in registers so
    // that the operand reads of a step depend on nothing that is read in that step
    // (only the variants with few accumulators have the registers for this and for the operand
    // prefetch below; the others look the position up in LDS step by step)
    constexpr bool PF = TBA * CS <= 3;
    __syncthreads();
    int wpix[PF ? W2_MAXSTEPS : 1];
    if (PF) {
#pragma unroll
        for (int s = 0; s < W2_MAXSTEPS; ++s) wpix[s] = stab[2 * s + half].y;
    }
    const int2* __restrict__ const stab_h = stab + half;

    const int c_begin = (int)(((uint32_t)a.chunks * (uint32_t)zshare) / (uint32_t)a.splits);   // chunks * splits < 2^31 (host)
    const int c_end = (int)(((uint32_t)a.chunks * (uint32_t)(zshare + 1)) / (uint32_t)a.splits);
    const int tiles_per_group = a.ntp * a.ntq;
    const int ntask_x = WH * WW * (CT / 16);    // input window: (window pixel, 16-channel granule)
    const int ntask = ntask_x + units * 4;      // + gradient tile: (tile pixel, 16-filter granule)
    const uint32_t ximg = (uint32_t)a.H * a.W * a.Cp;     // image strides in bytes
    const uint32_t yimg = (uint32_t)a.P * a.Q * a.Kp;

    // The loader task of this thread; tasks are dealt evenly to the four waves.  Everything that
    // does not depend on the chunk is worked out once.  A task fetches 16 bytes from each of 16
    // images.  kind: 0 input, 1 gradient, 2 none
    int t_kind = 2, t_a = 0, t_b = 0, t_c = 0, t_pix = 0, t_g = 0;
    {
        const int per_wave = (ntask + 3) >> 2;
        const int task = (lane < per_wave) ? wave * per_wave + lane : ntask;
        if (task < ntask_x) {
            t_g = task % (CT / 16);
            t_pix = task / (CT / 16);
            t_kind = 0;
            t_a = t_pix / WW;                 // window row
            t_b = t_pix - t_a * WW;           // window column
            t_c = ct * CT + 16 * t_g;         // >= Cp: nothing to fetch, zeros are staged
        } else if (task < ntask) {
            t_g = (task - ntask_x) & 3;
            t_pix = (task - ntask_x) >> 2;
            t_kind = 1;
            t_a = t_pix / a.BQ;               // tile row
            t_b = t_pix - t_a * a.BQ;         // tile column
            t_c = kt * W2_BM + 16 * t_g;
        }
    }
    // first granule of the task's 16 in LDS and the xor of swz_ch() for them
    uint4* __restrict__ const t_row = (t_kind == 1) ? (dyT + t_pix * YP + 16 * t_g) : (xT + t_pix * XP + 16 * t_g);
    const int t_xor = t_g & 15;

    // Prefetch registers.  Loads are unconditional: a task with nothing to fetch (padding, ragged
    // tile edge, channel beyond the tensor) reads offset 0 of its tensor and is zeroed when it is
    // staged; images beyond N re-read the group's last image and are zeroed the same way.
    uint4 pre[16];
    bool pre_ok = false;
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
        if (t_kind == 2) return;
        const bool isx = t_kind == 0;
        const int yy = (isx ? ih0 : p0) + t_a, xx = (isx ? iw0 : q0) + t_b;
        const int hh = isx ? a.H : a.P, ww = isx ? a.W : a.Q, cc = isx ? a.Cp : a.Kp;
        const bool ok = (unsigned)yy < (unsigned)hh && (unsigned)xx < (unsigned)ww && t_c < cc;
        pre_ok = ok;
        const uint32_t stride = isx ? ximg : yimg;
        const int8_t* base = isx ? a.x : a.dy;
        uint32_t off = ok ? (((uint32_t)n0 * hh + yy) * ww + xx) * cc + t_c : (uint32_t)n0 * stride;
#pragma unroll
        for (int im = 0; im < 16; ++im) {
            pre[im] = *reinterpret_cast<const uint4*>(base + off);
            if (im + 1 < nimg) off += stride;
        }
    };

    // 16 images x 16 channels -> sixteen [channel][16 images] granules, four channels at a time
    auto commit = [&](uint32_t m0, uint32_t m1, uint32_t m2, uint32_t m3) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            uint32_t o[4][4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const uint32_t d[4] = {comp(pre[4 * g], q), comp(pre[4 * g + 1], q), comp(pre[4 * g + 2], q),
                                       comp(pre[4 * g + 3], q)};
                transpose4x4_bytes(d, o[g]);
            }
#pragma unroll
            for (int j = 0; j < 4; ++j)
                t_row[(4 * q + j) ^ t_xor] = make_uint4(o[0][j] & m0, o[1][j] & m1, o[2][j] & m2, o[3][j] & m3);
        }
    };

    if (c_begin < c_end) issue(c_begin);
    for (int chunk = c_begin; chunk < c_end; ++chunk) {
        __syncthreads();   // the previous chunk's MFMA reads are done
        if (t_kind != 2) {
            if (!pre_ok) {
                // padding, ragged tile edge or channel beyond the tensor: zeros
#pragma unroll
                for (int k = 0; k < 16; ++k) t_row[k] = make_uint4(0, 0, 0, 0);
            } else if (pre_nimg == 16) {
                commit(0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu);
            } else {
                // last, partial image group: byte i of a granule is image i; images beyond N are zeroed
                uint32_t m[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int left = pre_nimg - 4 * k;
                    m[k] = left >= 4 ? 0xffffffffu : left <= 0 ? 0u : ((1u << (8 * left)) - 1u);
                }
                commit(m[0], m[1], m[2], m[3]);
            }
        }
        __syncthreads();
        if (chunk + 1 < c_end) issue(chunk + 1);   // in flight while this chunk's MFMAs run

        // The operands of step s+1 are requested before the MFMAs of step s are issued (two register
        // sets), so the LDS latency of a step hides behind the previous step's matrix work.
        constexpr int NSET = PF ? 2 : 1;
        uint4 ra[NSET], rb[NSET][TBA][CS];
        auto fetch = [&](int s, int set) {
            ra[set] = dyT[a_ch + 2 * s * YP];
            const int wp = PF ? wpix[PF ? s : 0] : stab_h[2 * s].y;
#pragma unroll
            for (int j = 0; j < TBA; ++j)   // TB divides R*S: every tap of the group exists
#pragma unroll
                for (int i = 0; i < CS; ++i) rb[set][j][i] = xT[wp + (PK ? 0 : tpix[j]) + x_ch[i]];
        };
        if (PF) fetch(0, 0);
#pragma unroll
        for (int s = 0; s < W2_MAXSTEPS; ++s) {
            if (s < nsteps) {
                if (PF) {
                    if (s + 1 < W2_MAXSTEPS && s + 1 < nsteps) fetch(s + 1, (s + 1) & 1);
                } else {
                    fetch(s, 0);
                }
                const uint4 ta = ra[s & (NSET - 1)];
                const v4i fa = v4i{(int)ta.x, (int)ta.y, (int)ta.z, (int)ta.w};
#pragma unroll
                for (int j = 0; j < TBA; ++j) {
#pragma unroll
                    for (int i = 0; i < CS; ++i) {
                        const uint4 tb = rb[s & (NSET - 1)][j][i];
                        const v4i fb = v4i{(int)tb.x, (int)tb.y, (int)tb.z, (int)tb.w};
                        acc[j][i] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa, fb, acc[j][i], 0, 0, 0);
                    }
                }
            }
        }
    }

    // partial[z][k][(tap,c)], channel fastest: 32 consecutive columns per store instruction
    const int ncolsp = RS * a.Cp;
    int32_t* __restrict__ part = a.partial + (size_t)zshare * a.K * ncolsp;
#pragma unroll
    for (int j = 0; j < TBA; ++j) {
        if (j >= nt) continue;
#pragma unroll
        for (int i = 0; i < CS; ++i) {
            // (PK: the 64 columns are taps t0 .. t0 + 3 x 16 channels, which is their order in the partial tile as well)
            const int c = PK ? ch * 32 + l32 : ct * CT + (ch * CS + i) * 32 + l32;
            if (!PK && c >= a.Cp) continue;
            const int col = (t0 + j) * a.Cp + c;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = kt * W2_BM + mt * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
                if (k < a.K) part[(size_t)k * ncolsp + col] = acc[j][i][v];
            }
        }
    }
}

// Sum the split partials, apply Eq.2 and scatter [k][(r,s,c)] -> K,C,R,S.  A block owns, for one filter k,
// 4*QN channels x RSC taps; its 256 threads are 256/QN split lanes x QN channel quads.  Every thread adds up the
// splits z = lane, lane + 256/QN, ... of its quad at each tap (independent 16-byte loads, RSC of them in flight
// per split), the lanes are combined through LDS, and the sums leave in the order of the result tensor -- with
// all taps of a filter in the block (RSC = R*S) that is one contiguous run of 4*QN*RSC floats.  LDS holds
// [split lane][channel quad][channel][tap] with an odd quad pitch of 4*RSC + 1 words: the stores of a wave
// (one word per quad at a time) then land in different banks for any RSC, and the final reads walk
// consecutive words with one word skipped per quad.
template <int QN, int RSC>
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const WgradArgs a) {
    constexpr int ZL = 256 / QN, CB = 4 * QN, QP = 4 * RSC + 1, PITCH = QN * QP;
    __shared__ int sred[ZL * PITCH];
    const int RS = a.R * a.S;
    const int ncolsp = RS * a.Cp;
    const size_t total = (size_t)a.K * ncolsp;
    const int nrg = RS / RSC, nct = a.Cp / CB;
    int b = blockIdx.x;
    const int rg = b % nrg;
    b /= nrg;
    const int ct = b % nct, k = b / nct;
    const int quad = threadIdx.x % QN, zl = threadIdx.x / QN;
    const int32_t* __restrict__ p = a.partial + (size_t)k * ncolsp + (size_t)(rg * RSC) * a.Cp + ct * CB + 4 * quad;
    int4 s4[RSC];
#pragma unroll
    for (int j = 0; j < RSC; ++j) s4[j] = make_int4(0, 0, 0, 0);
    // ZU splits at a time, so that a thread has ZU * RSC (at least 4) loads in flight
    constexpr int ZU = RSC >= 4 ? 1 : RSC == 3 ? 2 : 4;
    int z = zl;
    for (; z + (ZU - 1) * ZL < a.splits; z += ZU * ZL) {
        int4 v[ZU][RSC];
#pragma unroll
        for (int u = 0; u < ZU; ++u)
#pragma unroll
            for (int j = 0; j < RSC; ++j)
                v[u][j] = *reinterpret_cast<const int4*>(p + (size_t)(z + u * ZL) * total + (size_t)j * a.Cp);
#pragma unroll
        for (int u = 0; u < ZU; ++u)
#pragma unroll
            for (int j = 0; j < RSC; ++j) { s4[j].x += v[u][j].x; s4[j].y += v[u][j].y; s4[j].z += v[u][j].z; s4[j].w += v[u][j].w; }
    }
    for (; z < a.splits; z += ZL) {
#pragma unroll
        for (int j = 0; j < RSC; ++j) {
            const int4 v = *reinterpret_cast<const int4*>(p + (size_t)z * total + (size_t)j * a.Cp);
            s4[j].x += v.x; s4[j].y += v.y; s4[j].z += v.z; s4[j].w += v.w;
        }
    }
    int* __restrict__ mine = sred + zl * PITCH + quad * QP;
#pragma unroll
    for (int j = 0; j < RSC; ++j) {
        mine[j] = s4[j].x;
        mine[RSC + j] = s4[j].y;
        mine[2 * RSC + j] = s4[j].z;
        mine[3 * RSC + j] = s4[j].w;
    }
    __syncthreads();
    const int nz = a.splits < ZL ? a.splits : ZL;
    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
    for (int t = threadIdx.x; t < CB * RSC; t += 256) {
        const int cl = t / RSC;
        int sum = 0;
        for (int z = 0; z < nz; ++z) sum += sred[z * PITCH + t + (cl >> 2)];
        const int c = ct * CB + cl, rs = rg * RSC + (t - cl * RSC);
        if (c >= a.C) continue;
        size_t o = ((size_t)k * a.C + c) * RS + rs;
        if (a.s2d) {
            // back from the space-to-depth form: channel (2 dy + dx) * oC + c0 of tap (r', s') is channel c0
            // of tap (2 r' + dy - eh, 2 s' + dx - ew); taps outside the layer's own filter are dropped
            const int blk = c / a.oC, c0 = c - blk * a.oC;
            const int rr = rs / a.S;
            const int r = 2 * rr + (blk >> 1) - a.eh, s = 2 * (rs - rr * a.S) + (blk & 1) - a.ew;
            if (r < 0 || r >= a.oR || s < 0 || s >= a.oS) continue;
            o = (((size_t)k * a.oC + c0) * a.oR + r) * a.oS + s;
        }
        a.dw[o] = __fmul_rn((float)sum, scale);
        if (a.acc) a.acc[o] = sum;
    }
}

// The kernel VAR_AUTO runs: wgrad_lines_kernel wherever it applies (measured on the benchmark's 1x7, 7x1
// and 3x3 layers it needs 0.6 - 0.85 of wgrad_kernel's time), except for 1x1 filters on few channels: its
// 128 x 128 tile is mostly padding there (24 or 144 channels: 18 - 19 us against 17.5); with 256 or more input
// channels 64 filters are enough (56 x 56, 256 -> 64: 19.9 us against 27.5).
bool wgrad_auto_lines(const WgradArgs& a) {
    if (!wgrad_lines_applies(a)) return false;
    return !(a.R == 1 && a.S == 1) || (a.Cp >= 128 && a.Kp >= 128) || (a.Cp >= 256 && a.Kp >= 64);
}

size_t wgrad_s2d(WgradArgs* a) {
    a->s2d = 0;
    if (!s2d_applies(a->C, a->stride_h, a->stride_w)) return 0;
    const S2dGeo g = s2d_geometry(a->R, a->S, a->pad_h, a->pad_w);
    a->s2d = 1;
    a->oC = a->C; a->oR = a->R; a->oS = a->S; a->oH = a->H; a->oW = a->W;
    a->eh = g.eh;
    a->ew = g.ew;
    a->C = 4 * a->oC;
    a->Cp = 16;
    a->H = (a->H + 1) / 2;
    a->W = (a->W + 1) / 2;
    a->R = g.R2;
    a->S = g.S2;
    a->pad_h = g.ph;
    a->pad_w = g.pw;
    a->stride_h = a->stride_w = 1;        // P and Q stay: the rewritten layer has the same output pixels
    return (size_t)a->N * a->H * a->W * 16;
}

// ---------------------------------------------------------------------------------------------
// Host-side plan: tile shapes, tap grouping, split count.  Shared by the workspace query and the
// launch so that both see the same numbers.
// ---------------------------------------------------------------------------------------------
namespace {
// The plan of the most recent geometry, per host thread: a layer is planned once, not per call.
struct PlanCache {
    int key[16];
    WgradArgs plan;
    bool valid;
};
thread_local PlanCache g_plan_cache = {};

void plan_key(const WgradArgs* a, int key[16]) {
    const int k[16] = {a->N, a->C, a->Cp, a->H, a->W, a->K, a->Kp, a->P, a->Q, a->R, a->S,
                       a->stride_h, a->stride_w, a->pad_h, a->pad_w, a->variant};
    for (int i = 0; i < 16; ++i) key[i] = k[i];
}
void wgrad_plan_uncached(WgradArgs* a);
}  // namespace

void wgrad_plan(WgradArgs* a) {
    int key[16];
    plan_key(a, key);
    PlanCache& c = g_plan_cache;
    bool hit = c.valid;
    for (int i = 0; hit && i < 16; ++i) hit = c.key[i] == key[i];
    if (!hit) {
        wgrad_plan_uncached(a);
        for (int i = 0; i < 16; ++i) c.key[i] = key[i];
        c.plan = *a;
        c.valid = true;
        return;
    }
    const WgradArgs& p = c.plan;
    a->TB = p.TB; a->CS = p.CS; a->BP = p.BP; a->BQ = p.BQ; a->ntp = p.ntp; a->ntq = p.ntq;
    a->ngrp = p.ngrp; a->chunks = p.chunks; a->splits = p.splits;
    a->ktiles = p.ktiles; a->ctiles = p.ctiles; a->tapgroups = p.tapgroups;
    a->xt_slots = p.xt_slots; a->lds_bytes = p.lds_bytes; a->lines = p.lines; a->xgk = p.xgk; a->xgc = p.xgc; a->pk = p.pk;
}

namespace {
void wgrad_plan_uncached(WgradArgs* a) {
    a->lines = 0;
    a->xgk = a->xgc = 0;
    if (a->variant == VAR_WGRAD_LINES || (a->variant != VAR_WGRAD_IMAGES && wgrad_auto_lines(*a))) {
        wgrad_plan_lines(a);
        return;
    }
    const int RS = a->R * a->S;
    // taps per block / channel slabs per wave: one filter row of a 3-wide filter, a whole 1x7 or
    // 7x1 filter, a wide channel tile for 1x1, one tap at a time otherwise
    a->pk = 0;
    if (a->Cp == 16 && RS % 4 == 0) { a->TB = 4; a->CS = 1; a->pk = 1; }      // four taps side by side in the 64 columns
    else if (RS == 1) { a->TB = 1; a->CS = (a->Cp >= 256) ? 4 : 1; }
    else if (RS % 3 == 0 && a->S == 3) { a->TB = 3; a->CS = 1; }
    else if (RS == 7) { a->TB = 7; a->CS = 1; }
    else { a->TB = 1; a->CS = 1; }
    // TB divides R*S in every case, so a tap group is never ragged
    const int CT = a->pk ? 16 : 64 * a->CS;          // channels staged per window pixel
    a->tapgroups = (RS + a->TB - 1) / a->TB;
    a->ktiles = (a->K + W2_BM - 1) / W2_BM;
    a->ctiles = (a->Cp + CT - 1) / CT;
    // Output-pixel tile BP x BQ: the one that covers the most useful pixels per chunk among those
    // whose staged window fits LDS, whose loader tasks fit one per thread and whose pixel count fits
    // the unrolled MFMA steps.  (More pixels per chunk = more MFMAs per barrier pair and per
    // transposed byte; tiles that divide P and Q waste nothing at the edges.)
    int BP = 1, BQ = 1;
    double best_score = -1.0;
    for (int bp = 1; bp <= a->P && bp <= 2 * W2_MAXSTEPS; ++bp) {
        for (int bq = 1; bq <= a->Q && bp * bq <= 2 * W2_MAXSTEPS; ++bq) {
            int maxwin = 0;
            for (int g = 0; g < a->tapgroups; ++g) {
                const int t0 = g * a->TB, nt = (RS - t0 < a->TB) ? (RS - t0) : a->TB;
                int rmin, rmax, smin, smax;
                tap_extent(t0, nt, a->S, &rmin, &rmax, &smin, &smax);
                const int WH = (bp - 1) * a->stride_h + (rmax - rmin) + 1;
                const int WW = (bq - 1) * a->stride_w + (smax - smin) + 1;
                if (WH * WW > maxwin) maxwin = WH * WW;
            }
            const size_t lds = (size_t)(maxwin * (CT + W2_PAD) + (bp * bq + 1) * (W2_BM + W2_PAD)) * 16 +
                               2 * W2_MAXSTEPS * sizeof(int2);
            const int ntask = maxwin * (CT / 16) + bp * bq * 4;   // one loader task per thread
            const bool fits = lds <= (size_t)W2_LDS_BUDGET && ntask <= 256;
            if (!fits && !(bp == 1 && bq == 1)) continue;
            const int ntp = (a->P + bp - 1) / bp, ntq = (a->Q + bq - 1) / bq;
            const double cover = (double)a->P * a->Q / ((double)ntp * bp * ntq * bq);
            // useful pixels per chunk, discounted by the fixed cost of a chunk (about 6 pixels' worth)
            const double score = cover * (bp * bq) / (bp * bq + 6.0);
            if (score > best_score) {
                best_score = score;
                BP = bp;
                BQ = bq;
                a->xt_slots = maxwin * (CT + W2_PAD);
                a->lds_bytes = lds;
            }
        }
    }
    const int np = (a->P + BP - 1) / BP;
    const int nq = (a->Q + BQ - 1) / BQ;
    a->BP = BP;
    a->BQ = BQ;
    a->ntp = np;
    a->ntq = nq;
    a->ngrp = (a->N + 15) / 16;
    a->chunks = a->ngrp * np * nq;
    const int out_tiles = a->ktiles * a->ctiles * a->tapgroups;
    // Split count: the one with the smallest estimated time.  Blocks run in rounds of `slots`
    // (blocks resident on the chip: registers allow two per compute unit for the narrow tiles, one
    // for the wide ones); a block pays a prologue plus its chunks; every split adds one write and
    // one read of the int32 partial tile set.  The constants are rough measurements in microseconds.
    const int acc_tiles = a->pk ? 1 : a->TB * a->CS;
    const int per_cu_regs = acc_tiles == 1 ? 3 : 2;   // by register count of the variants
    int per_cu_lds = (int)((160 * 1024) / a->lds_bytes);
    if (per_cu_lds < 1) per_cu_lds = 1;
    const int slots = 256 * (per_cu_regs < per_cu_lds ? per_cu_regs : per_cu_lds);
    const double t_chunk = 1.2 * per_cu_regs + 0.014 * (BP * BQ + 1) / 2 * acc_tiles;
    const double t_partial = (double)a->K * RS * a->Cp * 8.0 / 4.0e6;
    int splits = 1;
    double best = 1e30;
    for (int sp = 1; sp <= a->chunks && sp <= 4096; ++sp) {
        const long long blocks = (long long)out_tiles * sp;
        const double rounds = (double)((blocks + slots - 1) / slots);
        const double t = rounds * (3.0 + ((a->chunks + sp - 1) / sp) * t_chunk) + sp * t_partial;
        if (t < best) { best = t; splits = sp; }
        if (blocks > 8LL * slots || (long long)a->chunks * (sp + 2) >= (1LL << 31)) break;
    }
    // a caller may ask for half or twice the shares of this choice (per-layer tuning by measurement)
    if (a->variant == VAR_WGRAD_FEWER) splits = splits > 1 ? splits / 2 : 1;
    if (a->variant == VAR_WGRAD_MORE) splits = (2 * splits <= a->chunks && 2 * splits <= 4096) ? 2 * splits : splits;
    a->splits = splits;
}
}  // namespace

hipError_t launch_wgrad(const WgradArgs& a_in, hipStream_t st) {
    WgradArgs a = a_in;
    if (a.s2d) {
        hipError_t e = launch_s2d_repack(a.x, a.xs, a.N, a.oH, a.oW, a.oC, st);
        if (e != hipSuccess) return e;
        a.x = a.xs;
    }
    const unsigned out_tiles = (unsigned)(a.ktiles * a.ctiles * a.tapgroups);
    dim3 grid(wgrad_xcd_mapping(a.splits) ? out_tiles * 8u * (unsigned)((a.splits + 7) / 8) : out_tiles * (unsigned)a.splits);
    // the staged tiles may exceed the default 64 KB of dynamic LDS: raise the limit once per variant
#define LAUNCH(TBv, CSv, PKv)                                                                                  \
    do {                                                                                                  \
        static std::atomic<unsigned long long> attr_done;                                                 \
        hipError_t ea = raise_dynamic_lds(reinterpret_cast<const void*>(wgrad_kernel<TBv, CSv, PKv>), W2_LDS_BUDGET, \
                                          attr_done);                                                     \
        if (ea != hipSuccess) return ea;                                                                  \
        launch_timed(kt, (wgrad_kernel<TBv, CSv, PKv>), grid, dim3(256), a.lds_bytes, st, a);                \
    } while (0)
    if (a.lines) {
        hipError_t el = launch_wgrad_lines(a, st);
        if (el != hipSuccess) return el;
    } else {
        KernelTimer kt(KID_WGRAD, st);
        if (a.pk) LAUNCH(4, 1, true);
        else if (a.TB == 1 && a.CS == 1) LAUNCH(1, 1, false);
        else if (a.TB == 1 && a.CS == 4) LAUNCH(1, 4, false);
        else if (a.TB == 3) LAUNCH(3, 1, false);
        else if (a.TB == 7) LAUNCH(7, 1, false);
        else return hipErrorInvalidValue;
    }
#undef LAUNCH
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    // Shape of the reducing blocks: the most taps (9, 7 or 3 where they divide R*S) and channels (256, 64 or
    // 16) per block that still give the chip 1024 blocks -- few fat blocks leave compute units idle and the
    // loads of a small layer are latency, not bandwidth; one tap x 16 channels if nothing does.  A block's
    // threads are (channels / 4) x (split lanes): 256 channels leave 4 split lanes, which is what few splits
    // can keep busy.
    const int RS = a.R * a.S;
    int rsc = 1, qn = 4;
    {
        const int cand[3] = {9, 7, 3};
        const int qns[3] = {64, 16, 4};
        bool found = false;
        for (int w = 0; w < 3 && !found; ++w) {
            if (a.Cp % (4 * qns[w]) != 0) continue;
            if (qns[w] == 64 && a.splits > 6) continue;
            for (int i = 0; i < 4 && !found; ++i) {
                const int r = i < 3 ? cand[i] : 1;
                if (RS % r != 0) continue;
                if ((long long)a.K * (a.Cp / (4 * qns[w])) * (RS / r) >= 1024) { rsc = r; qn = qns[w]; found = true; }
            }
        }
    }
    const unsigned rblocks = (unsigned)(a.K * (a.Cp / (4 * qn)) * (RS / rsc));
    {
        KernelTimer kt(KID_WGRAD_REDUCE, st);
#define REDUCE(RSCv)                                                                                         \
    do {                                                                                                     \
        if (qn == 64) launch_timed(kt, (wgrad_reduce_kernel<64, RSCv>), dim3(rblocks), dim3(256), 0, st, a); \
        else if (qn == 16) launch_timed(kt, (wgrad_reduce_kernel<16, RSCv>), dim3(rblocks), dim3(256), 0, st, a); \
        else launch_timed(kt, (wgrad_reduce_kernel<4, RSCv>), dim3(rblocks), dim3(256), 0, st, a);          \
    } while (0)
        if (rsc == 9) REDUCE(9);
        else if (rsc == 7) REDUCE(7);
        else if (rsc == 3) REDUCE(3);
        else REDUCE(1);
#undef REDUCE
    }
    return hipGetLastError();
}

}  // namespace int8t
