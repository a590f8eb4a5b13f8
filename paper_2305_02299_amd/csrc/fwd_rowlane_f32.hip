// ROWLANE forward kernels, fp32 storage.
#include "fwd_rowlane.inl"
namespace srigl {
srigl_status launch_rowlane_f32(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) { return launch_rowlane_x<float, int32_t>(a, p, st); }
}  // namespace srigl

#ifdef SRIGL_TIMELINE   // development builds only
extern "C" int srigl_dbg_timeline(long long* host_out, int n) {
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(srigl::g_timeline), sizeof(long long) * (size_t)n);
}
#endif
