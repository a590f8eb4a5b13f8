// ROWLANE forward kernels, fp32 storage, 16-bit column indices.
#include "fwd_rowlane.inl"
namespace srigl {
srigl_status launch_rowlane_f32_i16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) { return launch_rowlane_x<float, uint16_t>(a, p, st); }
}  // namespace srigl
