// Dense backward-weight convolution on int8 codes (Sec.3.4: g_W = g_z^T a), int8 MFMA with int32
// accumulation, Eq.2 fused into the final reduction.
//
// GEMM view:  D[k][col] = sum_pix  Gz^T[k][pix] * A^T[pix][col],   col = (r,s,c),  pix = (n,p,q)
// The reduction runs over output pixels, which are the OUTERMOST index of the channels-last code
// tensors, while the MFMA wants 16 consecutive reduction bytes per lane.  The loader therefore
// transposes on the fly: a thread fetches 4 pixels x 4 channels (four dwords), swaps them to
// 4 channels x 4 pixels with byte permutes -- the 4x4 int8 block transpose of the paper's Suppl.
// "INT8 Convolution" (its Fig. "4x4 8-bit integer block transpose"), here feeding LDS tiles laid
// out [channel][64 pixels] -- and the MFMA operand reads are then plain 16-byte LDS loads.
//
// The pixel reduction is long (N*P*Q) and the output small, so the reduction is split across
// blocks (grid.z); every split writes an int32 partial tile and a second kernel sums the
// partials (integer addition: exact in any order), applies Eq.2 and scatters to K,C,R,S.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WG_BN = 128;   // columns (r,s,c) per block
constexpr int WG_BK = 64;    // pixels per reduction step

// LDS tile [row][64 pixel bytes] with an 80-byte row pitch (20 dwords).  wg_slot() is the index of
// the 16-byte granule g of `row` in 16-byte units.  Eight consecutive rows at one granule land in
// eight different 16-byte bank groups (the MFMA operand reads are conflict free); the xor with
// row bits 3-4 spreads the loader's transposed stores, which walk rows with a stride of four.
constexpr int WG_PITCH16 = 5;
__device__ __forceinline__ int wg_slot(int row, int g) { return row * WG_PITCH16 + (g ^ ((row >> 3) & 3)); }

// 4x4 byte transpose: in d[i] = 4 channels of pixel i; out o[c] = channel c of pixels 0..3.
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

template <int BM>
__global__ __launch_bounds__(256) void wgrad_kernel(const WgradArgs a) {
    constexpr int MI = BM / 64;
    __shared__ __attribute__((aligned(16))) uint32_t sA[BM * WG_PITCH16 * 4];      // [k][64 pixel bytes]
    __shared__ __attribute__((aligned(16))) uint32_t sB[WG_BN * WG_PITCH16 * 4];   // [col][64 pixel bytes]

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wm = wave & 1, wn = wave >> 1;

    const int PQ = a.P * a.Q;
    const int ncolsp = a.R * a.S * a.Cp;
    const int rowbase = blockIdx.y * BM;
    const int colbase = blockIdx.x * WG_BN;
    const int cpi = (PQ + WG_BK - 1) / WG_BK;          // reduction chunks per image
    const int total = a.N * cpi;
    const int t_begin = (int)(((long long)total * blockIdx.z) / gridDim.z);
    const int t_end = (int)(((long long)total * (blockIdx.z + 1)) / gridDim.z);

    // ---- A loader (g_z): k-quad = tid % 16, pixel-quad = tid / 16, MI row halves --------------
    const int a_kq = tid & 15, a_pq = tid >> 4;
    // ---- B loader (a): column-quad = tid % 32, pixel octet = tid / 32 ---------------------------
    const int b_cq = tid & 31, b_po = tid >> 5;
    const int bcol = colbase + 4 * b_cq;
    const bool bcol_ok = bcol < ncolsp;
    int b_tr, b_ts, b_c;
    {
        const int tap = (bcol_ok ? bcol : 0) / a.Cp;
        b_c = (bcol_ok ? bcol : 0) - tap * a.Cp;
        b_tr = tap / a.S;
        b_ts = tap - b_tr * a.S;
    }
    const float invQ = 1.0f / (float)a.Q;

    uint32_t ra[MI][4], rb[2][4];
    auto load_step = [&](int t) {
        const int n = t / cpi;
        const int rem0 = (t - n * cpi) * WG_BK;
        // A: dy[(n*PQ + rem)*Kp + k .. k+3]
#pragma unroll
        for (int h = 0; h < MI; ++h) {
            const int k = rowbase + h * 64 + 4 * a_kq;
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int rem = rem0 + 4 * a_pq + i;
                ra[h][i] = 0;
                if (rem < PQ && k < a.Kp)
                    ra[h][i] = *reinterpret_cast<const uint32_t*>(a.dy + ((size_t)n * PQ + rem) * a.Kp + k);
            }
        }
        // B: x[((n*H + ih)*W + iw)*Cp + c .. c+3] at this thread's filter tap, 8 consecutive pixels
        {
            const int rem_first = rem0 + 8 * b_po;
            // (p,q) of the first pixel: float estimate, then exact correction
            int p = (int)((float)rem_first * invQ);
            int q = rem_first - p * a.Q;
            if (q < 0) { --p; q += a.Q; }
            if (q >= a.Q) { ++p; q -= a.Q; }
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                const int ih = p * a.stride_h - a.pad_h + b_tr;
                const int iw = q * a.stride_w - a.pad_w + b_ts;
                rb[i >> 2][i & 3] = 0;
                if (bcol_ok && (rem_first + i) < PQ && (unsigned)ih < (unsigned)a.H &&
                    (unsigned)iw < (unsigned)a.W)
                    rb[i >> 2][i & 3] = *reinterpret_cast<const uint32_t*>(
                        a.x + (((size_t)n * a.H + ih) * a.W + iw) * a.Cp + b_c);
                if (++q == a.Q) { q = 0; ++p; }
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

    if (t_begin < t_end) load_step(t_begin);
    for (int t = t_begin; t < t_end; ++t) {
        __syncthreads();
        // transpose in registers, then [channel][pixel] dwords into LDS
#pragma unroll
        for (int h = 0; h < MI; ++h) {
            uint32_t o[4];
            transpose4x4(ra[h], o);
#pragma unroll
            for (int c = 0; c < 4; ++c)
                sA[wg_slot(h * 64 + 4 * a_kq + c, a_pq >> 2) * 4 + (a_pq & 3)] = o[c];
        }
        {
            uint32_t o0[4], o1[4];
            transpose4x4(rb[0], o0);
            transpose4x4(rb[1], o1);
            // pixel octet b_po = dwords 2*b_po, 2*b_po+1 of the row: granule b_po/2, 8-byte half b_po%2
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                uint2 v;
                v.x = o0[c];
                v.y = o1[c];
                *reinterpret_cast<uint2*>(&sB[wg_slot(4 * b_cq + c, b_po >> 1) * 4 + (b_po & 1) * 2]) = v;
            }
        }
        __syncthreads();
        if (t + 1 < t_end) load_step(t + 1);
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            const int g = kk * 2 + (lane >> 5);
            v4i fa[MI], fb[2];
#pragma unroll
            for (int i = 0; i < MI; ++i)
                fa[i] = *reinterpret_cast<const v4i*>(&sA[wg_slot(wm * (BM / 2) + i * 32 + (lane & 31), g) * 4]);
#pragma unroll
            for (int j = 0; j < 2; ++j)
                fb[j] = *reinterpret_cast<const v4i*>(&sB[wg_slot(wn * 64 + j * 32 + (lane & 31), g) * 4]);
#pragma unroll
            for (int i = 0; i < MI; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }

    // partial[z][k][col], col fastest: 32 consecutive columns per store instruction
    int32_t* __restrict__ part = a.partial + (size_t)blockIdx.z * a.K * ncolsp;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
        const int col = colbase + wn * 64 + j * 32 + (lane & 31);
        if (col >= ncolsp) continue;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int k = rowbase + wm * (BM / 2) + i * 32 + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                if (k < a.K) part[(size_t)k * ncolsp + col] = acc[i][j][v];
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

int wgrad_splits(int N, int C, int K, int P, int Q, int R, int S) {
    const int Cp = (C + 15) & ~15;
    const int BM = (K <= 64) ? 64 : 128;
    const int tiles = ((K + BM - 1) / BM) * ((R * S * Cp + WG_BN - 1) / WG_BN);
    const int chunks = N * ((P * Q + WG_BK - 1) / WG_BK);
    int splits = (512 + tiles - 1) / tiles;          // about two blocks per compute unit
    if (splits > chunks / 4) splits = chunks / 4;     // at least four reduction steps per block
    if (splits < 1) splits = 1;
    return splits;
}

hipError_t launch_wgrad(const WgradArgs& a, hipStream_t st) {
    const int ncolsp = a.R * a.S * a.Cp;
    if (a.K <= 64) {
        dim3 grid((ncolsp + WG_BN - 1) / WG_BN, 1, a.splits);
        hipLaunchKernelGGL((wgrad_kernel<64>), grid, dim3(256), 0, st, a);
    } else {
        dim3 grid((ncolsp + WG_BN - 1) / WG_BN, (a.K + 127) / 128, a.splits);
        hipLaunchKernelGGL((wgrad_kernel<128>), grid, dim3(256), 0, st, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const size_t total = (size_t)a.K * ncolsp;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, a);
    return hipGetLastError();
}

}  // namespace int8t
