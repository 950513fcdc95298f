// Host-callable launchers of the kernel families (defined in the .hip files).
#ifndef LT_LAUNCH_H_
#define LT_LAUNCH_H_

#include <hip/hip_runtime_api.h>

#include "lt_kernels.h"

namespace ltk {
hipError_t launch_ew(const EwArgs& a, uint32_t grid, hipStream_t s);
hipError_t launch_row_reduce(const RowArgs& a, uint32_t grid, hipStream_t s);
hipError_t launch_all_reduce(const AllArgs& a, uint32_t grid, hipStream_t s);
hipError_t launch_col_reduce(const ColArgs& a, uint32_t grid_x, uint32_t grid_y, hipStream_t s);
hipError_t launch_row_op(const RowOpArgs& a, uint32_t grid, hipStream_t s);
hipError_t launch_split_post(const SplitPostArgs& a, uint32_t grid, hipStream_t s);
hipError_t launch_slice_update(const SliceArgs& a, uint32_t grid, hipStream_t s);
hipError_t launch_gemm(const GemmArgs& a, hipStream_t s);
hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s);   // 128 x 128 tiles, split-K (called by launch_gemm)

// The library's static device scratch (lt_static_scratch.hip): its size, its address on `device`
// (looked up once per device; `device` must be current), and a fill kernel.
constexpr size_t kStaticScratchBytes = (size_t)16 << 20;
hipError_t static_scratch(int device, void** ptr, size_t* bytes);
hipError_t launch_fill_u32(uint32_t* p, uint32_t n, uint32_t value, hipStream_t s);

// Name of the kernel instance that the calling thread launched last (per-launch records and
// profiles name the instance, not just its family).
void note_kernel(const char* name);
const char* last_kernel();
}  // namespace ltk

// Launch kernel instance K and note its name as written (template arguments included).
#define LT_LAUNCH(K, GRID, BLOCK, STREAM, ARGS)          \
  do {                                                   \
    ::ltk::note_kernel(#K);                              \
    hipLaunchKernelGGL(K, GRID, BLOCK, 0, STREAM, ARGS); \
  } while (0)
#endif
