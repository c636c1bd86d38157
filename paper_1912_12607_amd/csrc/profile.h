// Optional per-kernel timing inside the library.  A timed launch hands a pair of HIP events to the
// dispatch itself (hipExtLaunchKernelGGL): they take the kernel's own start and end time stamps,
// so nothing is put into the stream between kernels and the timing does not disturb the step it
// measures.  Off by default (then a KernelTimer costs one integer compare and launches are plain);
// switched on and read out through int8t_profile_start / int8t_profile_stop.  Not thread-safe: one
// thread drives the library while profiling is on.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>

#include <cstdint>

namespace int8t {

enum KernelId : int {
    KID_ABSMAX = 0,
    KID_ABSMAX_BATCH,
    KID_QUANTIZE_ACT,
    KID_QUANTIZE_PLANAR,
    KID_QUANTIZE_WGT,
    KID_QUANTIZE_BATCH,
    KID_DEVIATION_FINISH,
    KID_DSGC_SWEEP,
    KID_IGEMM,
    KID_IGEMM_DMA,
    KID_IGEMM_FUSED,
    KID_IGEMM_REDUCE,
    KID_BAND,
    KID_BAND_REG,
    KID_WGRAD,
    KID_WGRAD_LINES,
    KID_WGRAD_REDUCE,
    KID_S2D_REPACK,
    KID_S2D_WEIGHTS,
    KID_DW_CONV,
    KID_DW_WGRAD,
    KID_DW_WGRAD_REDUCE,
    KID_COUNT
};

extern int g_profile_select;   // -2 off, -1 every kernel, >= 0 that kernel only

class KernelTimer {
   public:
    KernelTimer(int kid, hipStream_t st) : slot_(-1), st_(st) {
        if (g_profile_select != -2 && (g_profile_select == -1 || g_profile_select == kid)) begin(kid);
    }
    ~KernelTimer() {
        if (slot_ >= 0) end();
    }
    KernelTimer(const KernelTimer&) = delete;
    KernelTimer& operator=(const KernelTimer&) = delete;
    bool active() const { return slot_ >= 0; }
    hipEvent_t start_event() const;   // valid while active()
    hipEvent_t stop_event() const;
    void mark_launched() const;

   private:
    void begin(int kid);
    void end();
    int slot_;
    hipStream_t st_;
};

// Launch `kernel` inside the scope of `kt`: timed when the timer is active, a plain launch otherwise.
// The arguments are converted to the kernel's parameter types first.
template <typename... KArgs, typename... Args>
inline void launch_timed(const KernelTimer& kt, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t lds,
                         hipStream_t st, Args&&... args) {
    static_assert(sizeof...(KArgs) == sizeof...(Args), "argument count must match the kernel's");
    if (kt.active()) {
        hipExtLaunchKernelGGL(kernel, grid, block, (std::uint32_t)lds, st, kt.start_event(), kt.stop_event(), 0,
                              static_cast<KArgs>(args)...);
        kt.mark_launched();
    } else {
        hipLaunchKernelGGL(kernel, grid, block, lds, st, static_cast<KArgs>(args)...);
    }
}

}  // namespace int8t
