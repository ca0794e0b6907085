// Stand-ins for the device side of libgorgo (kernels.hip), so that its host-side sources -- trace loading, the
// evolution-strategy arithmetic, argument and option checking, workspace planning -- can be built for the CPU with
// AddressSanitizer and UndefinedBehaviorSanitizer and driven by host_fuzz.cpp.  Every device operation fails.
#include "internal.h"

namespace gorgo {

static int no_device(const char* what) { return fail(GORGO_ERR_DEVICE, std::string(what) + ": no device in this build"); }

bool pack_replays(const Plan&, int64_t) { return false; }
int launch_replay(const gorgo_trace*, const Plan&, const double*, const double*, const double*, uint8_t*, uint16_t*, double*,
                  double*, void*, void*, const OnlineLaunch*, const PolicyLaunch*, const EngineLaunch*, const ProxyLaunch*,
                  unsigned long long*) {
    return no_device("launch_replay");
}
int launch_p95(const double*, int64_t, int32_t, double*, void*) { return no_device("launch_p95"); }
int last_eval_kernel_ms(double*, double*, double*) { return no_device("last_eval_kernel_ms"); }
int upload_trace(const gorgo_trace*) { return no_device("upload_trace"); }
bool trace_is_resident(const gorgo_trace*) { return false; }
int static_scratch(void**, size_t*) { return no_device("static_scratch"); }
void set_event_marks(bool) {}
void release_device_trace(gorgo_trace*) {}
int copy_small_to_device(void*, const void*, size_t, void*) { return no_device("copy_small_to_device"); }
int wait_for_copies(void*) { return no_device("wait_for_copies"); }
int copy_small_to_host_sync(void*, const void*, size_t, void*) { return no_device("copy_small_to_host_sync"); }

}  // namespace gorgo
