// ROWLANE forward kernels, bf16 storage (fp32 accumulate).
#include "fwd_rowlane.inl"
namespace srigl {
srigl_status launch_rowlane_bf16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) { return launch_rowlane_x<uint16_t, int32_t>(a, p, st); }
}  // namespace srigl
