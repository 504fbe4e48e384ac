// Stand-ins for the device entry points of libstrassen_tc (tc_internal.h), for building the host planner alone:
// every call that would touch a GPU fails.  Host-only plans (tc_options_t.host_only) never reach them.
#include "tc_internal.h"

namespace tc {
int dev_static_workspace(void** ptr) { *ptr = nullptr; return 1; }
int bench_mfma_peak(int, int, void*, double*) { return 1; }
int dev_malloc(void**, size_t) { return 1; }
int dev_free(void*) { return 1; }
int dev_upload(void*, const void*, size_t, void*) { return 1; }
int dev_download(void*, const void*, size_t) { return 1; }
int dev_stream_sync(void*) { return 1; }
int dev_event_create(void**) { return 1; }
int dev_event_record(void*, void*) { return 1; }
int dev_event_sync(void*) { return 1; }
int dev_event_elapsed_ms(float*, void*, void*) { return 1; }
int dev_event_destroy(void*) { return 1; }
int launch_planner(const BundleDesc*, int, int64_t, int, int64_t*, void*) { return 1; }
int launch_fused(const FusedConfig&, const Product*, int, int, int64_t, int64_t, const double*, const double*, double*, double*, double, double,
                 int, int, int64_t, int64_t, void*) { return 1; }
int launch_lincomb(const Product*, int, int, int, int64_t, int64_t, int, const double*, const double*, double*, double*, int, double, void*) { return 1; }
}  // namespace tc
