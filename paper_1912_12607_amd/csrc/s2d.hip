// Space-to-depth form of the codes of a stride-2 layer with at most 4 input channels (kernels.h has
// the index algebra).  Channels-last codes keep 16 bytes per pixel however few channels are in use:
// the 7x7 stride-2 stem of an image network on 3 channels would spend 13 of every 16 reduction bytes
// on padding.  The rewritten layer has 4 C channels in the granule and a quarter of the taps; the
// dense kernels then run on it unchanged.
#include "device_common.h"
#include "kernels.h"

namespace int8t {

// The first C bytes of four 32-bit words, packed back to back into 16 bytes (the rest zero).
__device__ __forceinline__ uint4 s2d_pack(const uint32_t px[4], int C) {
    const uint32_t keep = C >= 4 ? 0xffffffffu : ((1u << (8 * C)) - 1u);
    unsigned long long lo = 0, hi = 0;        // a 128-bit shift register
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const unsigned long long v = px[b] & keep;
        const int sh = 8 * C * b;             // 0 .. 96
        if (sh < 64) {
            lo |= v << sh;
            if (sh > 32) hi |= v >> (64 - sh);
        } else {
            hi |= v << (sh - 64);
        }
    }
    return make_uint4((uint32_t)lo, (uint32_t)(lo >> 32), (uint32_t)hi, (uint32_t)(hi >> 32));
}

// Input codes: byte (2 dy + dx) * C + c of pixel (h', w') is channel c of pixel (2 h' + dy, 2 w' + dx),
// zero where that pixel lies beyond an odd image.
// One thread per output pixel; it reads the first four bytes of four input pixels.
__global__ __launch_bounds__(256) void s2d_repack_kernel(const int8_t* __restrict__ x, int8_t* __restrict__ xs,
                                                         int N, int H, int W, int C) {
    const int H2 = (H + 1) >> 1, W2 = (W + 1) >> 1;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (t >= (size_t)N * H2 * W2) return;
    const int w2 = (int)(t % W2);
    const size_t nh = t / W2;
    const int h2 = (int)(nh % H2);
    const size_t n = nh / H2;
    const uint32_t* __restrict__ row0 = reinterpret_cast<const uint32_t*>(x) + ((n * H + 2 * h2) * (size_t)W + 2 * w2) * 4;
    const uint32_t* __restrict__ row1 = row0 + (size_t)W * 4;
    const bool w1 = 2 * w2 + 1 < W, h1 = 2 * h2 + 1 < H;     // the block's second column / row exists
    const uint32_t px[4] = {row0[0], w1 ? row0[4] : 0u, h1 ? row1[0] : 0u, (h1 && w1) ? row1[4] : 0u};
    reinterpret_cast<uint4*>(xs)[t] = s2d_pack(px, C);
}

// Filter codes: tap (r', s') of the rewritten filter gathers the taps (2 r' + dy - eh, 2 s' + dx - ew)
// of the layer's own filter in the same channel order; taps outside it are zero.
__global__ __launch_bounds__(256) void s2d_weights_kernel(const int8_t* __restrict__ w, int8_t* __restrict__ ws,
                                                          int K, int R, int S, int C, S2dGeo g) {
    const int t = blockIdx.x * 256 + threadIdx.x;
    if (t >= K * g.R2 * g.S2) return;
    const int s2 = t % g.S2, r2 = (t / g.S2) % g.R2, k = t / (g.S2 * g.R2);
    uint32_t px[4];
#pragma unroll
    for (int b = 0; b < 4; ++b) {
        const int r = 2 * r2 + (b >> 1) - g.eh, s = 2 * s2 + (b & 1) - g.ew;
        const bool ok = r >= 0 && r < R && s >= 0 && s < S;
        px[b] = ok ? reinterpret_cast<const uint32_t*>(w)[((size_t)(k * R + r) * S + s) * 4] : 0u;
    }
    reinterpret_cast<uint4*>(ws)[t] = s2d_pack(px, C);
}

hipError_t launch_s2d_repack(const int8_t* x, int8_t* xs, int N, int H, int W, int C, hipStream_t st) {
    const size_t npix = (size_t)N * ((H + 1) / 2) * ((W + 1) / 2);
    KernelTimer kt(KID_S2D_REPACK, st);
    launch_timed(kt, s2d_repack_kernel, dim3((unsigned)((npix + 255) / 256)), dim3(256), 0, st, x, xs, N, H, W, C);
    return hipGetLastError();
}

hipError_t launch_s2d_weights(const int8_t* w, int8_t* ws, int K, int R, int S, int C, const S2dGeo& g, hipStream_t st) {
    const int n = K * g.R2 * g.S2;
    KernelTimer kt(KID_S2D_WEIGHTS, st);
    launch_timed(kt, s2d_weights_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, w, ws, K, R, S, C, g);
    return hipGetLastError();
}

}  // namespace int8t
