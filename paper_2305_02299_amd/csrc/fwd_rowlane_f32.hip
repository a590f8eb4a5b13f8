// ROWLANE forward kernels, fp32 storage.
#include "fwd_rowlane.inl"
namespace srigl {
srigl_status launch_rowlane_f32(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) { return launch_rowlane_x<float, int32_t>(a, p, st); }
}  // namespace srigl

