// Device half of the library replaced by stubs, for a CPU-only build of the host logic (generator,
// planner, plan cache) under AddressSanitizer / UBSan: every call that would need a GPU reports
// FT_ERR_UNSUPPORTED; host-only plans (FT_PLAN_HOST_ONLY) work as in the real library.
#include "ft_internal.h"

ft_status ftd_upload(ft_plan *) { return FT_ERR_UNSUPPORTED; }
void ftd_release(ft_plan *) {}

extern "C" {
ft_status ft_hw_query(int32_t, ft_hw_model *) { return FT_ERR_UNSUPPORTED; }
// (the argument checks that need no device are those of the real entry points)
ft_status ft_launch_epilogue(const ft_plan *plan, const void *A, const void *B, void *C, const float *bias, void *) {
    if (!plan) return FT_ERR_INVALID_ARG;
    if ((plan->op.epilogue == FT_EPI_BIAS) != (bias != nullptr)) return FT_ERR_INVALID_ARG;
    if (plan->st.n_tiles == 0) return FT_OK;
    if (!A || !B || !C || !plan->d_descs) return FT_ERR_INVALID_ARG;
    return FT_ERR_UNSUPPORTED;
}
ft_status ft_launch(const ft_plan *plan, const void *A, const void *B, void *C, void *s) { return ft_launch_epilogue(plan, A, B, C, nullptr, s); }
ft_status ft_launch_noalloc(const ft_plan *, const void *, const void *, void *, const float *, void *) { return FT_ERR_UNSUPPORTED; }
ft_status ft_stream_rate(const void *, void *, uint64_t, uint32_t, void *, float *, float *, float *) { return FT_ERR_UNSUPPORTED; }
ft_status ft_launch_timed(const ft_plan *, const void *const *, const void *const *, void *const *, uint32_t, void *, uint32_t,
                          float *) { return FT_ERR_UNSUPPORTED; }
ft_status ft_launch_timed_graph(const ft_plan *, const void *const *, const void *const *, void *const *, uint32_t, void *,
                                uint32_t, float *) { return FT_ERR_UNSUPPORTED; }
}
