// Optional per-kernel timing inside the library: HIP events recorded on the launch stream right
// before and after a kernel launch.  Off by default (then a KernelTimer costs one integer
// compare); switched on and read out through int8t_profile_start / int8t_profile_stop.  Not
// thread-safe: one thread drives the library while profiling is on.
#pragma once
#include <hip/hip_runtime.h>

namespace int8t {

enum KernelId : int {
    KID_ABSMAX = 0,
    KID_QUANTIZE_ACT,
    KID_QUANTIZE_PLANAR,
    KID_QUANTIZE_WGT,
    KID_DEVIATION_FINISH,
    KID_DSGC_SWEEP,
    KID_IGEMM,
    KID_IGEMM_REDUCE,
    KID_BAND,
    KID_WGRAD,
    KID_WGRAD_REDUCE,
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

   private:
    void begin(int kid);
    void end();
    int slot_;
    hipStream_t st_;
};

}  // namespace int8t
