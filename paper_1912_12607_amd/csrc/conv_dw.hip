// Depthwise convolution (groups == C == K) on planar int8 codes.  The paper singles the
// depthwise layer out as the structure with the hardest gradients (Sec.3.2, C4) but describes no
// kernel for it.  The reduction per output is only R*S taps (forward / backward-data), so this
// is not a dense contraction and the MFMA is of no use: every (n,c) plane is an independent 2-D
// filter, staged in LDS and evaluated on the plain integer ALUs; the kernels are HBM bound
// (1 byte in, 4 bytes out per element).
#include "device_common.h"
#include "kernels.h"

namespace int8t {

constexpr int DW_MAX_TAPS = 64;   // R*S limit of the depthwise kernels

// One block per (n,c) plane.  Forward: in = codes of a, gather ih = oh*stride - pad + r.
// Backward-data: in = codes of g_z, gather ih = (oh + pad - r)/stride when divisible.
template <bool DGRAD>
__global__ __launch_bounds__(256) void dw_conv_kernel(const DwArgs a) {
    extern __shared__ __attribute__((aligned(16))) int8_t plane[];
    __shared__ int wtap[DW_MAX_TAPS];
    const int nc = blockIdx.x;
    const int c = nc % a.C;
    const int IHW = a.IH * a.IW, OHW = a.OH * a.OW, RS = a.R * a.S;
    const int8_t* __restrict__ src = a.a + (size_t)nc * IHW;
    if ((IHW & 15) == 0) {
        for (int i = threadIdx.x; i < (IHW >> 4); i += 256)
            reinterpret_cast<uint4*>(plane)[i] = reinterpret_cast<const uint4*>(src)[i];
    } else {
        for (int i = threadIdx.x; i < IHW; i += 256) plane[i] = src[i];
    }
    if (threadIdx.x < RS) wtap[threadIdx.x] = (int)a.b[(size_t)c * RS + threadIdx.x];
    __syncthreads();

    const float scale = __fmul_rn(a.sa[0], a.sb[0]);
    for (int o = threadIdx.x; o < OHW; o += 256) {
        const int oh = o / a.OW, ow = o - oh * a.OW;
        int sum = 0;
        for (int r = 0; r < a.R; ++r) {
            int ih;
            if (DGRAD) {
                const int th = oh + a.pad_h - r;
                ih = th / a.stride_h;
                if (th < 0 || ih * a.stride_h != th) continue;
            } else {
                ih = oh * a.stride_h - a.pad_h + r;
            }
            if ((unsigned)ih >= (unsigned)a.IH) continue;
            for (int s = 0; s < a.S; ++s) {
                int iw;
                if (DGRAD) {
                    const int tw = ow + a.pad_w - s;
                    iw = tw / a.stride_w;
                    if (tw < 0 || iw * a.stride_w != tw) continue;
                } else {
                    iw = ow * a.stride_w - a.pad_w + s;
                }
                if ((unsigned)iw >= (unsigned)a.IW) continue;
                sum += (int)plane[ih * a.IW + iw] * wtap[r * a.S + s];
            }
        }
        const size_t idx = (size_t)nc * OHW + o;
        a.out[idx] = __fmul_rn((float)sum, scale);
        if (a.acc) a.acc[idx] = sum;
    }
}

// Backward-weight: g_W[c,r,s] = sum_{n,p,q} g_z[n,c,p,q] * a[n,c,p*sh+r-ph,q*sw+s-pw].
// grid (C, chunks); a block sums its share of the images for one channel and writes
// partial[chunk][c][rs]; the reduce kernel adds the chunks and applies Eq.2.
__device__ __forceinline__ void dw_block_sum_store(int v, int* red, int32_t* dst) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    if (threadIdx.x == 0) *dst = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void dw_wgrad_kernel(const DwArgs a) {
    extern __shared__ __attribute__((aligned(16))) int8_t lds[];
    __shared__ int red[4];
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
            for (int i = threadIdx.x; i < IHW; i += 256) xs[i] = xsrc[i];
            for (int i = threadIdx.x; i < OHW; i += 256) gs[i] = gsrc[i];
            __syncthreads();
            for (int o = threadIdx.x; o < OHW; o += 256) {
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
#pragma unroll
        for (int i = 0; i < 9; ++i) dw_block_sum_store(acc9[i], red, part + i);
    } else {
        // other filter sizes: one tap at a time, straight from global memory
        for (int rs = 0; rs < RS; ++rs) {
            const int r = rs / a.S, s = rs - r * a.S;
            int v = 0;
            for (int n = n0; n < n1; ++n) {
                const int8_t* __restrict__ xsrc = a.a + ((size_t)n * a.C + c) * IHW;
                const int8_t* __restrict__ gsrc = a.b + ((size_t)n * a.C + c) * OHW;
                for (int o = threadIdx.x; o < OHW; o += 256) {
                    const int p = o / a.OW, q = o - p * a.OW;
                    const int ih = p * a.stride_h - a.pad_h + r, iw = q * a.stride_w - a.pad_w + s;
                    if ((unsigned)ih < (unsigned)a.IH && (unsigned)iw < (unsigned)a.IW)
                        v += (int)gsrc[o] * (int)xsrc[ih * a.IW + iw];
                }
            }
            dw_block_sum_store(v, red, part + rs);
        }
    }
}

__global__ __launch_bounds__(256) void dw_wgrad_reduce_kernel(const DwArgs a) {
    const int RS = a.R * a.S;
    const int total = a.C * RS;
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= total) return;
    int sum = 0;
    for (int z = 0; z < a.chunks; ++z) sum += a.partial[(size_t)z * total + t];
    a.out[t] = __fmul_rn((float)sum, __fmul_rn(a.sa[0], a.sb[0]));
    if (a.acc) a.acc[t] = sum;
}

int dw_wgrad_chunks(int N, int C) {
    int chunks = (2048 + C - 1) / C;
    if (chunks > N) chunks = N;
    if (chunks < 1) chunks = 1;
    return chunks;
}

hipError_t launch_dw_conv(const DwArgs& a, hipStream_t st) {
    const size_t lds = ((size_t)a.IH * a.IW + 15) & ~(size_t)15;
    if (a.dgrad)
        { KernelTimer kt(KID_DW_CONV, st); hipLaunchKernelGGL((dw_conv_kernel<true>), dim3(a.N * a.C), dim3(256), lds, st, a); }
    else
        { KernelTimer kt(KID_DW_CONV, st); hipLaunchKernelGGL((dw_conv_kernel<false>), dim3(a.N * a.C), dim3(256), lds, st, a); }
    return hipGetLastError();
}

hipError_t launch_dw_wgrad(const DwArgs& a, hipStream_t st) {
    const size_t lds = (((size_t)a.IH * a.IW + 15) & ~(size_t)15) + (((size_t)a.OH * a.OW + 15) & ~(size_t)15);
    { KernelTimer kt(KID_DW_WGRAD, st); hipLaunchKernelGGL(dw_wgrad_kernel, dim3(a.C, a.chunks), dim3(256), lds, st, a); }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int total = a.C * a.R * a.S;
    { KernelTimer kt(KID_DW_WGRAD_REDUCE, st); hipLaunchKernelGGL(dw_wgrad_reduce_kernel, dim3((total + 255) / 256), dim3(256), 0, st, a); }
    return hipGetLastError();
}

}  // namespace int8t
