// Stand-ins for the kernel launchers of libhzp in the host-only sanitizer build (test
// infrastructure).  The planner and the argument checks of the entry points are compiled from the
// library's own sources with -fsanitize=address,undefined; nothing may reach a GPU in that build,
// so every launcher refuses.
#include "hzp_internal.hpp"

namespace hzp {

static hzp_status_t no_gpu(const char *what) { return fail(HZP_ERR_HIP, "%s: host-only sanitizer build launches nothing", what); }

hzp_status_t launch_reduce(bool, const void *const *, uint32_t, uint64_t, float, int, float *, hipStream_t)
{
    return no_gpu("launch_reduce");
}
hzp_status_t launch_fused(const hzp_plan_t *, bool, bool, uint32_t, const FusedSegment *, size_t, const AdamScalars &,
                          hipStream_t)
{
    return no_gpu("launch_fused");
}
hzp_status_t launch_fused_dev(const hzp_plan_t *, bool, bool, uint32_t, const FusedSegment *, size_t, const AdamScalars *,
                              hipStream_t)
{
    return no_gpu("launch_fused_dev");
}
hzp_status_t launch_concat(const void *const *, uint32_t, uint64_t, void *, hipStream_t) { return no_gpu("launch_concat"); }
hzp_status_t launch_concat_layers(const void *const *, uint32_t, const uint64_t *, void *const *, uint32_t, hipStream_t)
{
    return no_gpu("launch_concat_layers");
}
hzp_status_t launch_concat_ranges(const void *const *, const uint64_t *, const uint64_t *, uint32_t, void *, hipStream_t)
{
    return no_gpu("launch_concat_ranges");
}
hzp_status_t launch_unpack(const hzp_plan_t *, const BucketRec &, const void *const *, uint32_t, void *const *, uint32_t,
                           uint32_t, hipStream_t)
{
    return no_gpu("launch_unpack");
}
hzp_status_t launch_unpack_static(const BucketRec &, const void *const *, uint32_t, void *const *, hipStream_t)
{
    return no_gpu("launch_unpack_static");
}
hzp_status_t device_tables(const hzp_plan_t *, const DeviceTables **) { return no_gpu("device_tables"); }
void free_device_tables(hzp_plan_t *) {}

}  // namespace hzp

extern "C" hzp_status_t hzp_plan_prepare(const hzp_plan_t *plan, hipStream_t)
{
    if (!plan) return hzp::fail(HZP_ERR_INVALID_ARG, "hzp_plan_prepare: NULL plan");
    return hzp::no_gpu("hzp_plan_prepare");
}
