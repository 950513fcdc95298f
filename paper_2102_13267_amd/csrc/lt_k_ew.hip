// Elementwise fused region: one coalesced HBM pass; the whole chain is interpreted in registers.
#include <hip/hip_runtime.h>

#include "lt_interp.h"
#include "lt_launch.h"

namespace ltk {

constexpr int kBlock = 256;
// ---- elementwise region: one coalesced pass, 16 bytes per lane and input ------------------
template <int NS>
__global__ __launch_bounds__(kBlock) void lt_ew_kernel(const EwArgs a) {
  const EwProg& p = a.prog;
  const uint64_t n = p.n;
  const uint64_t nvec = (n + kVec - 1) / kVec;
  for (uint64_t v = (uint64_t)blockIdx.x * kBlock + threadIdx.x; v < nvec; v += (uint64_t)gridDim.x * kBlock) {
    const uint64_t i = v * kVec;
    const uint32_t nvalid = (n - i >= (uint64_t)kVec) ? (uint32_t)kVec : (uint32_t)(n - i);
    RF<NS> f = load_inputs<NS>(rf_zero<NS>(), p, i, nvalid);
    f = interp<NS>(f, p);
    store_outputs<NS>(f, p, i, nvalid);
  }
}


hipError_t launch_ew(const EwArgs& a, uint32_t grid, hipStream_t s) {
  if (a.prog.n_slots <= 16u) hipLaunchKernelGGL(lt_ew_kernel<16>, dim3(grid), dim3(kBlock), 0, s, a);
  else hipLaunchKernelGGL(lt_ew_kernel<32>, dim3(grid), dim3(kBlock), 0, s, a);
  return hipGetLastError();
}

}  // namespace ltk
