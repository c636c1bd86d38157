// Per-kernel timing with HIP events on the launch stream (see profile.h).
#include "profile.h"

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
    "band_kernel",         "band_reg_kernel",     "wgrad_kernel",        "wgrad_reduce_kernel",    "s2d_repack_kernel", "s2d_weights_kernel", "dw_conv_kernel",
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
