// Elementwise fused region: one coalesced HBM pass; the whole chain is interpreted in registers.
#include <hip/hip_runtime.h>

#include "lt_interp.h"
#include "lt_launch.h"

namespace ltk {

constexpr int kBlock = 256;
// ---- elementwise region: one coalesced pass, 16 bytes per lane and input ------------------
// A workgroup walks tiles of kBlock * kVec = 1024 consecutive elements with a grid stride.  The
// tile base is wave-uniform (scalar registers); lanes differ only by a constant 32-bit offset.
template <int NS, int MAXIN, bool FAST, bool F32>
__global__ __launch_bounds__(kBlock) void lt_ew_kernel(const EwArgs a) {
  const EwProg& p = a.prog;
  const uint64_t n = p.n;
  constexpr uint64_t kTile = (uint64_t)kBlock * kVec;
  const uint64_t ntiles = (n + kTile - 1) / kTile;
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t lane = threadIdx.x * kVec;
  // (Prefetching the next tile's inputs during interpretation was measured and lost to the
  // occupancy it costs: 4 resident waves per SIMD hide HBM latency better than 3 pipelined ones.)
  for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint64_t base = tile * kTile;
    const uint64_t left = n - base;                       // >= 1
    if ((uint64_t)lane >= left) continue;
    const uint32_t nvalid = left - lane >= (uint64_t)kVec ? (uint32_t)kVec : (uint32_t)(left - lane);
    RF<NS> f = load_inputs<NS, MAXIN, FAST, F32>(rf_zero<NS>(), p, base, lane, nvalid);
    f = interp<NS>(f, pr, n_code);
    store_outputs<NS, FAST, F32>(f, p, base, lane, nvalid);
  }
}

hipError_t launch_ew(const EwArgs& a, uint32_t grid, hipStream_t s) {
  const EwProg& p = a.prog;
  const dim3 g(grid), b(kBlock);
  const bool f16 = p.fast && p.n_slots <= 16u;
  if (f16 && p.all_f32 && p.n_in <= 4u) hipLaunchKernelGGL((lt_ew_kernel<16, 4, true, true>), g, b, 0, s, a);
  else if (f16 && p.all_f32 && p.n_in <= 6u) hipLaunchKernelGGL((lt_ew_kernel<16, 6, true, true>), g, b, 0, s, a);
  else if (f16 && p.all_f32) hipLaunchKernelGGL((lt_ew_kernel<16, 8, true, true>), g, b, 0, s, a);
  else if (f16) hipLaunchKernelGGL((lt_ew_kernel<16, 8, true, false>), g, b, 0, s, a);
  else hipLaunchKernelGGL((lt_ew_kernel<32, 8, false, false>), g, b, 0, s, a);
  return hipGetLastError();
}

}  // namespace ltk
