// Per-kernel timing with HIP events on the launch stream (see profile.h).
#include "profile.h"

#include <stdint.h>

#include <cstring>
#include <vector>

#include "../../include/int8t.h"

namespace int8t {

int g_profile_select = -2;
int g_profile_every = 1;          // time every g_profile_every-th launch of a selected kernel
int g_profile_seen[KID_COUNT] = {0};

namespace {
struct Rec {
    int kid;
    hipEvent_t a, b;
    bool closed;     // a launch carried the events
};
std::vector<Rec> g_recs;

const char* const kNames[KID_COUNT] = {
    "absmax_kernel",       "absmax_batch_kernel", "quantize_act_kernel", "quantize_planar_kernel", "quantize_wgt_kernel",
    "quantize_batch_kernel",
    "deviation_finish_kernel", "dsgc_sweep_kernel",   "igemm_kernel", "igemm_dma_kernel", "igemm_fused_kernel", "igemm_reduce_kernel",
    "band_kernel",         "band_reg_kernel",     "wgrad_kernel",        "wgrad_lines_kernel", "wgrad_reduce_kernel",    "s2d_repack_kernel", "s2d_weights_kernel", "dw_conv_kernel",
    "dw_wgrad_kernel",     "dw_wgrad_reduce_kernel"};

void drop_all() {
    for (Rec& r : g_recs) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    g_recs.clear();
}
}  // namespace

void KernelTimer::begin(int kid) {
    if (g_profile_seen[kid]++ % g_profile_every != 0) return;
    Rec r;
    r.kid = kid;
    r.closed = false;
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) {
        (void)hipEventDestroy(r.a);
        return;
    }
    g_recs.push_back(r);
    slot_ = (int)g_recs.size() - 1;
}

void KernelTimer::end() {}

hipEvent_t KernelTimer::start_event() const { return g_recs[(size_t)slot_].a; }
hipEvent_t KernelTimer::stop_event() const { return g_recs[(size_t)slot_].b; }
void KernelTimer::mark_launched() const { g_recs[(size_t)slot_].closed = true; }

}  // namespace int8t

using namespace int8t;

extern "C" int8t_status int8t_profile_start_sampled(const char* kernel, int every) {
    drop_all();
    g_profile_select = -2;
    if (every < 1) return INT8T_ERR_ARG;
    g_profile_every = every;
    for (int k = 0; k < KID_COUNT; ++k) g_profile_seen[k] = 0;
    if (kernel == nullptr || kernel[0] == '\0') {
        g_profile_select = -1;
        return INT8T_OK;
    }
    for (int k = 0; k < KID_COUNT; ++k) {
        if (std::strcmp(kernel, kNames[k]) == 0) {
            g_profile_select = k;
            return INT8T_OK;
        }
    }
    return INT8T_ERR_ARG;
}

extern "C" int8t_status int8t_profile_start(const char* kernel) { return int8t_profile_start_sampled(kernel, 1); }

extern "C" int8t_status int8t_profile_stop(int8t_kernel_time* out, int capacity, int* count) {
    g_profile_select = -2;
    if (count == nullptr || capacity < 0 || (capacity > 0 && out == nullptr)) {
        drop_all();
        return INT8T_ERR_ARG;
    }
    int launches[KID_COUNT] = {0};
    double total[KID_COUNT] = {0.0};
    int8t_status status = INT8T_OK;
    for (Rec& r : g_recs) {
        if (!r.closed) continue;
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) {
            status = INT8T_ERR_RUNTIME;
            continue;
        }
        launches[r.kid] += 1;
        total[r.kid] += (double)ms;
    }
    drop_all();
    int n = 0;
    for (int k = 0; k < KID_COUNT; ++k) {
        if (launches[k] == 0) continue;
        if (n < capacity) {
            out[n].name = kNames[k];
            out[n].launches = launches[k];
            out[n].total_ms = total[k];
        }
        ++n;
    }
    *count = n;
    return status;
}

// ---------------------------------------------------------------------------------------------
// What the int8 matrix cores of this GPU sustain: a loop of independent v_mfma_i32_32x32x32_i8 on
// every SIMD (eight waves per compute unit, each a 64 x 128 tile of eight accumulators -- the wave
// tile of the wide convolution kernels), with the operands either held in registers or re-read from
// LDS before every eight MFMAs as an implicit GEMM does, and operand bytes either all zero or
// pseudo-random.  The kernel reads the shader clock counter and the constant 100 MHz counter around
// its loop, which gives the clock the chip actually ran at: under random operands the power limit
// pulls it far below the nominal 2.4 GHz, so the published peak is not reachable on real data.
// ---------------------------------------------------------------------------------------------
namespace int8t {
typedef int mc_v4i __attribute__((ext_vector_type(4)));
typedef int mc_v16i __attribute__((ext_vector_type(16)));

template <bool LDS_READS>
__global__ __launch_bounds__(512, 1) void mfma_ceiling_kernel(int iters, int random_operands, long long* __restrict__ out) {
    extern __shared__ __attribute__((aligned(16))) uint4 tile[];     // 512 rows x 4 granules
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, half = lane >> 5, l32 = lane & 31;
    for (int i = tid; i < 2048; i += 512) {
        uint32_t h = (uint32_t)i * 2654435761u;
        h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
        tile[i] = random_operands ? make_uint4(h, h * 3266489917u, h * 668265263u, h * 374761393u) : make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    auto slot = [](int row, int g) { return row * 4 + (g ^ ((row >> 2) & 3)); };
    auto rd = [&](int pos) { const uint4 t = tile[pos]; return mc_v4i{(int)t.x, (int)t.y, (int)t.z, (int)t.w}; };
    int apos[2][2], bpos[4][2];
    for (int i = 0; i < 2; ++i) for (int kk = 0; kk < 2; ++kk) apos[i][kk] = slot((wave * 64 + i * 32 + l32) & 255, 2 * kk + half);
    for (int j = 0; j < 4; ++j) for (int kk = 0; kk < 2; ++kk) bpos[j][kk] = slot(256 + ((wave * 128 + j * 32 + l32) & 255), 2 * kk + half);
    mc_v16i acc[2][4];
    for (int i = 0; i < 2; ++i) for (int j = 0; j < 4; ++j) for (int v = 0; v < 16; ++v) acc[i][j][v] = 0;
    mc_v4i fa[2], fb[4];
    for (int i = 0; i < 2; ++i) fa[i] = rd(apos[i][0]);
    for (int j = 0; j < 4; ++j) fb[j] = rd(bpos[j][0]);
    const long long c0 = clock64(), r0 = (long long)__builtin_amdgcn_s_memrealtime();
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            if (LDS_READS) {
#pragma unroll
                for (int i = 0; i < 2; ++i) fa[i] = rd(apos[i][kk]);
#pragma unroll
                for (int j = 0; j < 4; ++j) fb[j] = rd(bpos[j][kk]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
    const long long c1 = clock64(), r1 = (long long)__builtin_amdgcn_s_memrealtime();
    int s = 0;
    for (int i = 0; i < 2; ++i) for (int j = 0; j < 4; ++j) for (int v = 0; v < 16; ++v) s += acc[i][j][v];
    if (blockIdx.x == 0 && tid == 0) { out[0] = c1 - c0; out[1] = r1 - r0; }
    if (s == 0x7fffffff && iters < 0) out[2] = s;     // keeps the accumulators alive; never true in a run that matters
}
}  // namespace int8t

extern "C" int8t_status int8t_profile_mfma_ceiling(int random_operands, int lds_reads, int iters, double* tops_out,
                                                   double* ghz_out, void* ws_dev, void* stream) {
    if (!tops_out || !ghz_out || !ws_dev) return INT8T_ERR_NULL;
    if (iters < 1 || iters > (1 << 24) || (reinterpret_cast<uintptr_t>(ws_dev) & 7)) return INT8T_ERR_ARG;
    hipStream_t st = (hipStream_t)stream;
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
        return INT8T_ERR_RUNTIME;
    const size_t lds = 100 * 1024;      // more than half a compute unit's LDS: one block of eight waves per compute unit
    const void* fns[2] = {reinterpret_cast<const void*>(mfma_ceiling_kernel<false>), reinterpret_cast<const void*>(mfma_ceiling_kernel<true>)};
    if (hipFuncSetAttribute(fns[lds_reads ? 1 : 0], hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return INT8T_ERR_RUNTIME;
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return INT8T_ERR_RUNTIME;
    if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return INT8T_ERR_RUNTIME; }
    float ms = 0.f;
    long long host[2] = {0, 0};
    bool ok = true;
    for (int rep = 0; rep < 2 && ok; ++rep) {       // the second run is the one reported (clocks settled)
        ok = hipEventRecord(a, st) == hipSuccess;
        if (lds_reads) hipLaunchKernelGGL(mfma_ceiling_kernel<true>, dim3(cus), dim3(512), lds, st, iters, random_operands, (long long*)ws_dev);
        else hipLaunchKernelGGL(mfma_ceiling_kernel<false>, dim3(cus), dim3(512), lds, st, iters, random_operands, (long long*)ws_dev);
        ok = ok && hipGetLastError() == hipSuccess && hipEventRecord(b, st) == hipSuccess && hipEventSynchronize(b) == hipSuccess &&
             hipEventElapsedTime(&ms, a, b) == hipSuccess;
    }
    ok = ok && hipMemcpy(host, ws_dev, sizeof(host), hipMemcpyDeviceToHost) == hipSuccess;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (!ok || ms <= 0.f || host[1] <= 0) return INT8T_ERR_RUNTIME;
    const double mfmas = (double)cus * 8 * iters * 16;
    *tops_out = mfmas * 32768.0 * 2.0 / (ms * 1e-3) / 1e12;
    *ghz_out = (double)host[0] / (double)host[1] * 0.1;
    return INT8T_OK;
}
