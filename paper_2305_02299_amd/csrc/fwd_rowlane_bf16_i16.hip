// ROWLANE forward kernels, bf16 storage, 16-bit column indices.
#include "fwd_rowlane.inl"
namespace srigl {
srigl_status launch_rowlane_bf16_i16(const FwdArgs& a, const RowlanePlan& p, hipStream_t st) { return launch_rowlane_x<uint16_t, uint16_t>(a, p, st); }
}  // namespace srigl
