// Direction Sensitive Gradient Clipping (Sec.3.4 of the paper) as a candidate search.
//
// One sweep over the gradient evaluates the candidate clip values side by side.  Per candidate j
// it needs A_j = sum g*q_j and B_j = sum q_j^2 (and G = sum g^2 once); the deviation of Eq.6 is
// then d_j = 1 - A_j / sqrt(G * B_j): the scale s_j cancels between the numerator and |ghat|, so no
// dequantized tensor is ever formed.  The uniform draw of the stochastic rounding (Eq.3) is taken
// once per element and shared by all candidates -- the same draw the later quantize call uses,
// so the search scores exactly the codes that will be produced.
//
// The sweep is bound by the plain vector ALUs, not by HBM (4 bytes per element against several
// operations per element AND candidate), so the arithmetic is arranged to need few instructions:
//   * codes are sign(g) * m with m the rounded magnitude, so g*q = |g|*m and q^2 = m^2: the whole
//     search runs on magnitudes and never looks at a sign;
//   * m = floor(2 (|g| * inv + u)) >> 1: one round-down fused multiply-add and one convert that floors,
//     saturates and drops its byte into the dword of four elements, then one shift and one mask per dword
//     (see device_common.h).  These 2.5 instructions per element and candidate are all the vector ALU
//     does per evaluation;
//   * |g| is turned, once per element, into a 44-bit fixed-point integer relative to max|g|
//     (H * 2^22 + L, H, L <= 2^22), and both halves into three balanced (signed) byte digits;
//   * the sums A_j = sum |g| m_j (six digit sums) and B_j = sum m_j^2 are int8 x int8 products
//     with int32 accumulation, i.e. matrix products [digits x elements] * [elements x candidates]
//     and [candidates x elements] * [elements x candidates] (diagonal): they go to the matrix
//     cores.  A lane computes the codes of ITS four elements for all candidates, but an MFMA
//     operand wants one candidate's codes of 16 elements in a lane, so the code dwords take a trip
//     through a wave-private LDS tile (one byte per evaluation), which is cheap next to the ALU
//     work.  No barriers: a wave only reads what it wrote itself, and LDS serves a wave's
//     instructions in order.
// The integer sums are exact and order independent; the only error against an fp64 evaluation is
// the fixed-point rounding of |g|, |delta| <= max|g| * 2^-44 per element, i.e. at most
// 2^-44 * sqrt(n) in d_j (Cauchy-Schwarz), far below the resolution the search needs.
//
// Blocks add their 64-bit integer totals (sum H*m, sum L*m, sum m^2 per candidate) into one of
// DSGC_GROUPS accumulator sets with device-scope atomics -- integer addition, so the result does
// not depend on the order -- and take a ticket; the block that draws the last ticket sums the
// sets, evaluates Eq.6 for every candidate and picks the clip value.  The accumulators and the
// ticket are cleared by the absmax pass that always precedes the sweep.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int DSGC_JC = 32;        // candidates per block: the 32 columns of one MFMA tile
constexpr int DSGC_JPAD = 64;      // row pitch of the partial arrays (= INT8T_MAX_CANDIDATES)
// Three blocks per compute unit.  A fourth would fit (LDS 4 x 40 KB, 4 waves per SIMD) and is about
// 2 us faster when the sweep has the GPU to itself, but three leave 40 KB of LDS and half the wave
// slots to kernels of another stream: the sweep is bound by the vector ALUs, so HBM-bound kernels
// (quantizers, a forward convolution) can run beside it.
constexpr int DSGC_MAX_BLOCKS = 768;
constexpr int DSGC_GROUPS = 32;     // accumulator sets the blocks spread their atomics over
constexpr int DSGC_ROWS = DSGC_JC + 6;   // 32 code rows, then the 6 digit rows
// A wave's LDS tile holds 256 elements x DSGC_ROWS byte rows, stored by 16-element granule:
// [granule 0..15][row][16 bytes], with the granule pitch padded to 39 rows.  An MFMA operand read
// (32 lanes = 32 consecutive rows of one granule) is then 512 contiguous bytes, and the 16 granules
// a store instruction touches (4 lanes each) start 156 banks apart, i.e. in 16 different groups of
// 4 banks -- both free of bank conflicts, and 2.5 KB smaller per wave than padded rows, which is what
// lets a fourth block fit a compute unit.
constexpr int DSGC_GPITCH = (DSGC_ROWS + 1) * 16;   // 624 bytes
constexpr int DSGC_TILE = 16 * DSGC_GPITCH;         // 9984 bytes per wave
// int32 accumulators: |digit * code| <= 128 * 127 per element and lane sum; flushed well before 2^31
// (the bound is 256 iterations: 256 x 256 elements x 16256 < 2^31; 16 keeps the flush path in use at
// the benchmark sizes -- 12 to 28 iterations per block -- at a cost of under 1 % of the loop)
constexpr int DSGC_FLUSH_ITERS = 16;

// bytes [a.b3, b.b3, c.b3, d.b3]: the top bytes of four 32-bit values
__device__ __forceinline__ uint32_t top_bytes(int a, int b, int c, int d) {
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0703u);   // a.b3 b.b3 0 0
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x07030c0cu);   // 0 0 c.b3 d.b3
    return lo | hi;
}
// bytes [a.b0, b.b0, c.b0, d.b0]
__device__ __forceinline__ uint32_t low_bytes(int a, int b, int c, int d) {
    const uint32_t lo = __builtin_amdgcn_perm((uint32_t)b, (uint32_t)a, 0x0c0c0400u);
    const uint32_t hi = __builtin_amdgcn_perm((uint32_t)d, (uint32_t)c, 0x04000c0cu);
    return lo | hi;
}

// Balanced byte digits of four integers 0 <= v <= 2^22:  v = d0 + 256 d1 + 65536 d2 with
// -128 <= d < 128 (the bytes of v + 0x808080, each minus 128).  plane[b] packs digit b of the
// four values as signed bytes.
__device__ __forceinline__ void digit_planes(const uint32_t v[4], uint32_t plane[3]) {
    uint32_t y[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) y[e] = v[e] + 0x808080u;
    const uint32_t t0 = __builtin_amdgcn_perm(y[1], y[0], 0x05010400u);  // y0.b0 y1.b0 y0.b1 y1.b1
    const uint32_t t1 = __builtin_amdgcn_perm(y[1], y[0], 0x0c0c0602u);  // y0.b2 y1.b2 0 0
    const uint32_t t2 = __builtin_amdgcn_perm(y[3], y[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(y[3], y[2], 0x06020c0cu);  // 0 0 y2.b2 y3.b2
    plane[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u) ^ 0x80808080u;
    plane[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u) ^ 0x80808080u;
    plane[2] = (t1 | t3) ^ 0x80808080u;
}

template <bool STOCH>
__global__ __launch_bounds__(256) void dsgc_sweep_kernel(
    const float* __restrict__ g, size_t n, const float* __restrict__ ratios, int n_cand,
    const float* __restrict__ absmax_part, int nparts, uint32_t seed_lo, uint32_t seed_hi_mul,
    unsigned long long* __restrict__ acc, unsigned int* __restrict__ ticket, const double* __restrict__ partG,
    float* __restrict__ clip_out, double* __restrict__ dev_out, double* __restrict__ dev_all_out) {
    constexpr int JC = DSGC_JC;
    __shared__ float lds4[4];
    __shared__ float s_inv[JC];
    __shared__ unsigned int s_last;
    __shared__ __attribute__((aligned(16))) unsigned char s_tile[4][DSGC_TILE];
    // the block reductions after the sweep re-use the tiles' memory
    long long (*const s_red)[JC][3] = reinterpret_cast<long long (*)[JC][3]>(&s_tile[0][0]);
    static_assert(sizeof(long long) * 4 * JC * 3 <= sizeof(s_tile), "reduction scratch fits the tiles");

    const int j0 = blockIdx.y * JC;
    const int jn = (n_cand - j0 < JC) ? (n_cand - j0) : JC;
    // Everything the prologue fetches is requested before the first wait: the absmax partials, the ratios and
    // the block's first 16 bytes per lane of g (one memory round trip instead of three in a row, about 1 us
    // of a sweep that takes 10 us on a small tensor).
    absmax_partials_begin(absmax_part, nparts, lds4);
    const size_t n4 = n >> 2;
    const float4* __restrict__ g4 = reinterpret_cast<const float4*>(g);
    const size_t i_first = (size_t)blockIdx.x * 256 + threadIdx.x;
    const float4 f_first = (i_first < n4) ? g4[i_first] : make_float4(0.f, 0.f, 0.f, 0.f);
    const float ratio_j = ratios[j0 + ((int)threadIdx.x < jn ? (int)threadIdx.x : 0)];
    const float M = absmax_partials_end(lds4);
    if (threadIdx.x < JC) {
        const int j = threadIdx.x;
        const float c = (j < jn) ? __fmul_rn(M, ratio_j) : 0.0f;
        // the stochastic sweep works on twice the scaled value (exact power-of-two factor; stoch_codes4)
        s_inv[j] = STOCH ? __fmul_rn(inv_scale_of(c), 2.0f) : inv_scale_of(c);
    }
    __syncthreads();
    // fixed point: max|g| < 2^e, |g| * 2^(22-e) <= 2^22
    int e2 = 0;
    float mant = frexpf(M, &e2);
    float e2f = (float)e2;
    // From here on every fp32 operation of the stochastic sweep is either exact or the one
    // round-down multiply-add; the candidates' scales above were computed (by other lanes, before
    // the barrier) in the default mode.
    if (STOCH) fp32_round_down_mode(mant, e2f);
    const int shift = 22 - (int)e2f;
    float inv[JC];
#pragma unroll
    for (int j = 0; j < JC; ++j)
        inv[j] = __int_as_float(__builtin_amdgcn_readfirstlane(__float_as_int(s_inv[j])));

    const int w = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int l16 = lane & 15, kg = lane >> 4;
    unsigned char* __restrict__ const tile = s_tile[w];
    // this lane's four elements live in granule lane / 4, bytes 4 * (lane % 4) ..; + 16 * row
    uint32_t* __restrict__ const wr = reinterpret_cast<uint32_t*>(tile + (lane >> 2) * DSGC_GPITCH + 4 * (lane & 3));
    // MFMA operands of this lane (16 x 16 x 64 tiles: a lane supplies 16 reduction bytes of one row):
    // codes of candidate l16 (+ 16 for the second candidate group) / digit row min(l16, 5), granule
    // 4 * step + kg
    const unsigned char* __restrict__ const rd_code = tile + kg * DSGC_GPITCH + l16 * 16;
    const unsigned char* __restrict__ const rd_dig = tile + kg * DSGC_GPITCH + (JC + (l16 < 5 ? l16 : 5)) * 16;

    // per candidate group h: [digit row][candidate] (rows 0..5 used) and [candidate][candidate] (diagonal
    // used).  The 16-row tiles waste far fewer rows on the six digit rows than 32-row ones would.
    v4i accA[2], accB[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 4; ++v) accA[h][v] = accB[h][v] = 0;
    // lanes 0..15: totals so far (flushed part) of candidates l16 and 16 + l16: sum H*m, sum L*m, sum m^2
    long long runH[2] = {0, 0}, runL[2] = {0, 0}, runB[2] = {0, 0};

    // int32 tiles -> 64-bit per-candidate totals in lanes 0..15, accumulators cleared
    auto flush = [&]() {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            // accA[h]: lane (column l16, kg), register v holds digit row 4*kg + v: rows 0..3 (the H digits
            // and L digit 0) sit in the lanes kg = 0, rows 4..5 (L digits 1, 2) in registers 0..1 of kg = 1
            long long ph = 0, pl = 0;
            if (kg == 0) {
                ph = (long long)accA[h][0] + 256LL * accA[h][1] + 65536LL * accA[h][2];
                pl = (long long)accA[h][3];
            } else if (kg == 1) {
                pl = 256LL * accA[h][0] + 65536LL * accA[h][1];
            }
            pl += __shfl_xor(pl, 16, kWave);
            runH[h] += ph;       // meaningful in lanes 0..15 only
            runL[h] += pl;
            // accB[h]: the diagonal element of column l16 is row l16 = 4*kg + v
            int diag = 0;
#pragma unroll
            for (int v = 0; v < 4; ++v) diag = (v == (l16 & 3)) ? accB[h][v] : diag;
            long long bd = ((l16 >> 2) == kg) ? (long long)diag : 0LL;
            bd += __shfl_xor(bd, 16, kWave);
            bd += __shfl_xor(bd, 32, kWave);
            runB[h] += bd;
#pragma unroll
            for (int v = 0; v < 4; ++v) accA[h][v] = accB[h][v] = 0;
        }
    };

    // one wave iteration: 256 consecutive elements, four per lane
    auto group = [&](const float x[4], uint32_t index0) {
        float uf[4] = {0.f, 0.f, 0.f, 0.f};
        uint32_t H[4], L[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            if (STOCH) uf[e] = (float)rng24(seed_lo, seed_hi_mul, index0 + e) * 0x1p-23f;   // 2 u, u in [0, 1): exact
            const float xs = ldexpf(fabsf(x[e]), shift);     // exact, 0 .. 2^22
            const float h = floorf(xs);
            H[e] = (uint32_t)h;
            L[e] = (uint32_t)rintf((xs - h) * 4194304.0f);   // remainder * 2^22: exact before rint
        }
        uint32_t pH[3], pL[3];
        digit_planes(H, pH);
        digit_planes(L, pL);
#pragma unroll
        for (int b = 0; b < 3; ++b) {
            wr[(JC + b) * 4] = pH[b];
            wr[(JC + 3 + b) * 4] = pL[b];
        }
#pragma unroll
        for (int j = 0; j < JC; ++j) {
            uint32_t rp;
            if (STOCH) {
                rp = stoch_codes4(x, inv[j], uf);
            } else {
                rp = low_bytes(round_nearest_code(fabsf(x[0]), inv[j]), round_nearest_code(fabsf(x[1]), inv[j]),
                               round_nearest_code(fabsf(x[2]), inv[j]), round_nearest_code(fabsf(x[3]), inv[j]));
            }
            wr[j * 4] = rp;
        }
        __builtin_amdgcn_wave_barrier();   // keep the tile's stores ahead of its loads
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const uint4 td = *reinterpret_cast<const uint4*>(rd_dig + 4 * DSGC_GPITCH * s);
            const v4i fd = v4i{(int)td.x, (int)td.y, (int)td.z, (int)td.w};
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                const uint4 tc = *reinterpret_cast<const uint4*>(rd_code + 4 * DSGC_GPITCH * s + 256 * h);
                const v4i fc = v4i{(int)tc.x, (int)tc.y, (int)tc.z, (int)tc.w};
                accA[h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fd, fc, accA[h], 0, 0, 0);
                accB[h] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fc, fc, accB[h], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();   // and the next iteration's stores behind these loads
    };

    const size_t stride = (size_t)gridDim.x * 256;
    {
        // Wave-uniform trip count (the MFMAs need the whole wave): lanes beyond the end carry zeros,
        // which add nothing to A or B.  The next iteration's 16 bytes are requested before this
        // iteration's arithmetic starts.  The int32 tiles are turned into 64-bit totals after every
        // DSGC_FLUSH_ITERS iterations, outside the inner loop, so inside it only MFMAs touch them.
        size_t i = i_first;
        size_t ibase = (size_t)blockIdx.x * 256 + 64 * w;      // the wave's first float4
        float4 f = f_first;
        while (ibase < n4) {
            for (int it = 0; it < DSGC_FLUSH_ITERS && ibase < n4; ++it) {
                const size_t inext = i + stride;
                const float4 fn = (inext < n4) ? g4[inext] : make_float4(0.f, 0.f, 0.f, 0.f);
                const float vv[4] = {f.x, f.y, f.z, f.w};
                group(vv, (uint32_t)(4 * i));
                f = fn;
                i = inext;
                ibase += stride;
            }
            flush();
        }
    }
    if (blockIdx.x == 0 && w == 0 && (n & 3)) {
        // ragged tail (wave-uniform branch): lane 0 carries the last 1..3 elements, zeros elsewhere
        float vv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (lane == 0)
            for (int e = 0; e < (int)(n & 3); ++e) vv[e] = g[(n4 << 2) + e];
        group(vv, (uint32_t)(n4 << 2) + 4u * (uint32_t)lane);
        flush();
    }

    // block totals -> one of the accumulator sets
    __syncthreads();   // every wave is done with its tile: the memory now serves the reductions
    if (lane < 16) {
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            s_red[w][16 * h + lane][0] = runH[h];
            s_red[w][16 * h + lane][1] = runL[h];
            s_red[w][16 * h + lane][2] = runB[h];
        }
    }
    __syncthreads();
    if (threadIdx.x < 3 * JC) {
        const int j = threadIdx.x / 3, q = threadIdx.x - 3 * j;
        if (j < jn) {
            const long long t = (s_red[0][j][q] + s_red[1][j][q]) + (s_red[2][j][q] + s_red[3][j][q]);
            const int grp = (int)(blockIdx.x % DSGC_GROUPS);
            __hip_atomic_fetch_add(&acc[((size_t)grp * DSGC_JPAD + j0 + j) * 3 + q], (unsigned long long)t,
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    // All data moves through device-scope atomics (performed at the memory side) and is read back
    // with device-scope atomic loads, so no cache write-back is needed: it is enough that this
    // block's additions have been acknowledged before its ticket is drawn: every thread waits for
    // its outstanding memory operations, then the barrier.  (The memory model's own way to say this,
    // a device-scope release fence per thread in front of the barrier and an acquire fence in the
    // last block, was measured: each release fence writes the whole L2 of its XCD back, 768 blocks
    // of them stretch the sweep from 58 to 75 us with the GPU to itself and to 126 us beside another
    // stream's kernels, whose dirty lines they flush.  What the wait below relies on is only that an
    // atomic's vmcnt decrement means it has been performed, which the return path of a device-scope
    // atomic guarantees.)
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (threadIdx.x == 0)
        s_last = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == gridDim.x * gridDim.y - 1
                     ? 1u : 0u;
    __syncthreads();
    if (!s_last) return;
    float Mn = M;
    if (STOCH) fp32_round_nearest_mode(Mn);   // the clip value below is a default-mode product

    // ---- last block: sum the sets, Eq.6 per candidate, smallest deviation (ties: smallest j, i.e.
    // the largest clip value for decreasing ratios).  Every addition is in a fixed order. ----------
    long long (*const f_part)[DSGC_JPAD][3] = reinterpret_cast<long long (*)[DSGC_JPAD][3]>(&s_tile[0][0]);
    double* const f_g = reinterpret_cast<double*>(&s_tile[0][0] + sizeof(long long) * 4 * DSGC_JPAD * 3);
    static_assert(sizeof(long long) * 4 * DSGC_JPAD * 3 + sizeof(double) * 4 <= sizeof(s_tile), "fits the tiles");
    {
        const int j = threadIdx.x & 63, part = threadIdx.x >> 6;
        long long t[3] = {0, 0, 0};
        if (j < n_cand) {
            long long v[DSGC_GROUPS / 4][3];
#pragma unroll
            for (int k = 0; k < DSGC_GROUPS / 4; ++k)
#pragma unroll
                for (int q = 0; q < 3; ++q)
                    v[k][q] = (long long)__hip_atomic_load(&acc[((size_t)(4 * k + part) * DSGC_JPAD + j) * 3 + q],
                                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#pragma unroll
            for (int k = 0; k < DSGC_GROUPS / 4; ++k)
#pragma unroll
                for (int q = 0; q < 3; ++q) t[q] += v[k][q];
        }
#pragma unroll
        for (int q = 0; q < 3; ++q) f_part[part][j][q] = t[q];
        // G: the absmax pass's per-block sums of squares
        double gs = 0.0;
        for (int i = threadIdx.x; i < nparts; i += 256) gs += partG[i];
        gs = wave_sum(gs);
        if (j == 0) f_g[part] = gs;
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        const int j = threadIdx.x;
        double d = 0.0;
        if (j < n_cand) {
            long long t[3];
#pragma unroll
            for (int q = 0; q < 3; ++q) t[q] = (f_part[0][j][q] + f_part[1][j][q]) + (f_part[2][j][q] + f_part[3][j][q]);
            // A = (sumH * 2^22 + sumL) * 2^(e-44); the integer totals are exact, the conversions round once
            const double At = ldexp((double)t[0] * 4194304.0 + (double)t[1], e2 - 44);
            const double Bt = (double)t[2];
            const double Gt = (f_g[0] + f_g[1]) + (f_g[2] + f_g[3]);
            if (Gt == 0.0) d = 0.0;
            else if (Bt == 0.0) d = 1.0;
            else d = 1.0 - At / (sqrt(Gt) * sqrt(Bt));
            if (dev_all_out) dev_all_out[j] = d;
        }
        // The winner, over the lanes: a candidate replaces the best so far only with a strictly smaller deviation,
        // walking j upwards -- i.e. the smallest (d, j) in lexicographic order, where a deviation that is not
        // a number never wins, except candidate 0's, which then is never replaced.
        const double inf = __builtin_huge_val();
        double bd = (j < n_cand && d == d) ? d : (j == 0 ? -inf : inf);
        int bj = j;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const double od = __shfl_xor(bd, o, kWave);
            const int oj = __shfl_xor(bj, o, kWave);
            if (od < bd || (od == bd && oj < bj)) { bd = od; bj = oj; }
        }
        const int best = (Mn == 0.0f) ? 0 : bj;
        const double dbest = __shfl(d, best, kWave);
        if (j == 0) {
            *clip_out = __fmul_rn(Mn, ratios[best]);
            *dev_out = dbest;
        }
    }
}

// Blocks of the sweep: one per 1024 elements up to one per compute unit, then a quarter of that up to three per
// compute unit.  Every block ends with 96 device-scope atomic additions and a ticket, which the blocks of a
// mid-sized tensor all issue at the same moment: with 768 blocks of one or two iterations each that hand-over
// took 6 - 7 us of a 16 us sweep (0.8 M elements: 16.4 us with 768 blocks, 13.2 with 256; 1.6 M: 18.2 -> 16.7
// with 392; from 3 M elements on the full grid is fastest).
int dsgc_blocks(size_t n) {
    const size_t units = (n / 4 + 255) / 256;
    size_t want = units <= 256 ? units : (units / 4 < 256 ? 256 : units / 4);
    return (int)(want < 1 ? 1 : (want > (size_t)DSGC_MAX_BLOCKS ? (size_t)DSGC_MAX_BLOCKS : want));
}

hipError_t launch_dsgc(const float* g, size_t n, const float* ratios, int n_cand, int stochastic,
                       uint64_t seed, const DsgcWs& ws, int nparts_absmax, float* clip_out,
                       double* dev_out, double* dev_all_out, hipStream_t st) {
    const int nchunks = (n_cand + DSGC_JC - 1) / DSGC_JC;
    // about three blocks per compute unit in total; every candidate chunk walks the same x-grid
    int blocks = dsgc_blocks(n);
    const int cap = (DSGC_MAX_BLOCKS + nchunks - 1) / nchunks;
    if (blocks > cap) blocks = cap;
    const uint32_t slo = seed_key_x(seed), shi = seed_key_a(seed);
    dim3 grid(blocks, nchunks);
    KernelTimer kt(KID_DSGC_SWEEP, st);
    if (stochastic)
        launch_timed(kt, (dsgc_sweep_kernel<true>), grid, dim3(256), 0, st, g, n, ratios, n_cand,
                           ws.absmax_part, nparts_absmax, slo, shi, ws.acc, ws.ticket, ws.partG, clip_out,
                           dev_out, dev_all_out);
    else
        launch_timed(kt, (dsgc_sweep_kernel<false>), grid, dim3(256), 0, st, g, n, ratios, n_cand,
                           ws.absmax_part, nparts_absmax, slo, shi, ws.acc, ws.ticket, ws.partG, clip_out,
                           dev_out, dev_all_out);
    return hipGetLastError();
}

static_assert(kDsgcAccWords == (size_t)DSGC_GROUPS * DSGC_JPAD * 3, "accumulator layout known to the C-ABI layer");
size_t dsgc_acc_words() { return kDsgcAccWords; }

}  // namespace int8t
