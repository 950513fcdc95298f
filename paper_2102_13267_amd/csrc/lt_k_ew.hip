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

// Second half of a split-K contraction: add the splits' partial products (fixed order, so the
// sum does not depend on scheduling) and run the contraction's post program on the result.
template <int MAXIN, bool FAST>
__global__ __launch_bounds__(kBlock) void lt_split_post_kernel(const SplitPostArgs a) {
  const EwProg& p = a.prog;
  const uint64_t n = p.n;
  constexpr uint64_t kTile = (uint64_t)kBlock * kVec;
  const uint64_t ntiles = (n + kTile - 1) / kTile;
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t lane = threadIdx.x * kVec;
  const bool vec = (a.stride % 4u) == 0u;
  for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint64_t base = tile * kTile;
    const uint64_t left = n - base;
    if ((uint64_t)lane >= left) continue;
    const uint32_t nvalid = left - lane >= (uint64_t)kVec ? (uint32_t)kVec : (uint32_t)(left - lane);
    Quad anchor = splat(0.0f);
    for (uint32_t s = 0; s < a.splits; ++s) {
      const float* src = a.ws + (uint64_t)s * a.stride + base + lane;
      if (FAST || (vec && nvalid == (uint32_t)kVec)) {   // 16-byte aligned: every split starts at a multiple of 4 floats
        const float4 t = *(const float4*)src;
        anchor.v[0] += t.x; anchor.v[1] += t.y; anchor.v[2] += t.z; anchor.v[3] += t.w;
      } else {
        for (uint32_t e = 0; e < nvalid; ++e) anchor.v[e] += src[e];
      }
    }
    RF<16> f = load_inputs<16, MAXIN, FAST, false>(rf_zero<16>(), p, base, lane, nvalid);
    f = rf_set<16>(f, p.anchor_slot, anchor);
    f = interp<16>(f, pr, n_code);
    store_outputs<16, FAST, false>(f, p, base, lane, nvalid);
  }
}

hipError_t launch_split_post(const SplitPostArgs& a, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kBlock);
  // whole 4-vectors of partials need 16-byte aligned splits
  const bool fast = a.prog.fast && a.prog.n_in <= 4u && (a.stride % 4u) == 0u;
  if (fast) hipLaunchKernelGGL((lt_split_post_kernel<4, true>), g, b, 0, s, a);
  else hipLaunchKernelGGL((lt_split_post_kernel<8, false>), g, b, 0, s, a);
  return hipGetLastError();
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
