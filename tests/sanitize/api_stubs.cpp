// Host-only stand-ins for the kernel launchers of libthi (test infrastructure): they launch nothing,
// check the few preconditions the real launchers check, and report success -- so that csrc/api.hip's
// validation, workspace carving and dispatch arithmetic (with the library's own csrc/plan.hip) can run
// under AddressSanitizer / UndefinedBehaviorSanitizer on a machine without a GPU.
#include "../../paper_2605_25655_amd/csrc/thi_internal.h"

namespace thi {

static int g_launches = 0;
int stub_launch_count() { return g_launches; }

hipError_t launch_skinny(const SkinnyArgs& a, int, int, hipStream_t)
{
    ++g_launches;
    return (a.M >= 1 && a.M <= 16 * SK_MAX_MT && a.handover && a.counters) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_rowslab(const SkinnyArgs& a, int, int, hipStream_t)
{
    ++g_launches;
    return (a.K >= 1024 && a.K <= ROWSLAB_MAX_K && a.tiles >= 1 && a.M <= 32) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_rowblock(const SkinnyArgs& a, int epilogue, int num_cus, hipStream_t, int ksplit)
{
    ++g_launches;
    if (a.K < 1024 || a.K > ROWSLAB_MAX_K || a.N < 1 || a.M > 32) return hipErrorInvalidValue;
    if (ksplit > 1 && !rowblock_split_ok(a.N, a.K, epilogue, num_cus, ksplit)) return hipErrorInvalidValue;
    const RowBlockPlan p = plan_rowblock(a.N, epilogue, num_cus, ksplit);
    return (p.T >= 2 && p.T <= 6 && p.grid >= 1) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_mlp_fused(const SkinnyArgs& up, const SkinnyArgs& down, int epilogue_up, int num_cus, hipStream_t, int ksplit_down)
{
    ++g_launches;
    return (mlp_fused_ok(up.M, up.K, up.N, epilogue_up, num_cus, ksplit_down) && down.x == up.out) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_gemm(const GemmArgs& a, int epilogue, int, hipStream_t)
{
    ++g_launches;
    return (is_rms(epilogue) || !a.partials) ? hipErrorInvalidValue : hipSuccess;
}
hipError_t launch_rmsnorm_rows(const uint16_t*, const uint16_t*, float, uint16_t* xn, int, int, const RopeArgs&, hipStream_t)
{
    ++g_launches;
    return xn ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_attention(const AttnArgs& a, hipStream_t)
{
    ++g_launches;
    return (a.nsplit >= 1 && a.nsplit <= AT_MAX_SPLIT && a.chunk >= 1 && a.part) ? hipSuccess : hipErrorInvalidValue;
}
hipError_t launch_fill_words(void*, size_t, uint32_t, hipStream_t)
{
    ++g_launches;
    return hipSuccess;
}

}  // namespace thi
