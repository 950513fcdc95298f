// Stand-ins for the kernel launchers (defined in the .hip files) so that the four host files of
// the library link into a CPU-only program: the null device never launches anything.
#include "../../paper_2102_13267_amd/csrc/lt_launch.h"

namespace ltk {
hipError_t launch_ew(const EwArgs&, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_row_reduce(const RowArgs&, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_all_reduce(const AllArgs&, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_col_reduce(const ColArgs&, uint32_t, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_row_op(const RowOpArgs&, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_split_post(const SplitPostArgs&, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_slice_update(const SliceArgs&, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_gemm(const GemmArgs&, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_gemm_bf16(const GemmArgs&, hipStream_t) { return hipErrorInvalidValue; }
hipError_t static_scratch(int, void**, size_t*) { return hipErrorInvalidValue; }
hipError_t launch_fill_u32(uint32_t*, uint32_t, uint32_t, hipStream_t) { return hipErrorInvalidValue; }
}  // namespace ltk
