// Reduction regions: row, global (single launch) and column reductions, each with an interpreted
// elementwise prologue and an interpreted post program (epilogue / finaliser).
#include <hip/hip_runtime.h>

#include "lt_launch.h"
#include "lt_reduce.h"

namespace ltk {

// Run the post program of an anchored region for the flat elements i .. i+nvalid-1 of its
// space, with the anchor's value(s) already placed in slot post.anchor_slot.
__device__ __forceinline__ void run_post(const EwProg& post, const ProgRegs post_regs, Quad anchor, uint64_t i,
                                         uint32_t nvalid) {
  RF<16> f = load_inputs<16>(rf_zero<16>(), post, 0, (uint32_t)i, nvalid);
  f = rf_set(f, post.anchor_slot, anchor);
  f = interp<16>(f, post_regs, post.n_code);
  store_outputs<16>(f, post, 0, (uint32_t)i, nvalid);
}

// Row reduction.  threads_per_row is 64 (one wave per row, four rows per workgroup) or 256.
__global__ __launch_bounds__(kBlock) void lt_row_reduce_kernel(const RowArgs a) {
  __shared__ float lds[kBlock / 64];
  const EwProg& pro = a.pro;
  const ProgRegs pro_regs = load_prog_regs(a.pro), post_regs = load_prog_regs(a.post);
  const uint32_t pro_n = a.pro.n_code;
  const uint32_t tpr = a.threads_per_row;
  const uint32_t rows_per_block = kBlock / tpr;
  const uint32_t lane = threadIdx.x % tpr;
  const uint32_t sub = threadIdx.x / tpr;
  const uint32_t nblocks = (a.rows + rows_per_block - 1) / rows_per_block;
  for (uint32_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const uint32_t row = blk * rows_per_block + sub;
    float acc = red_identity(a.red);
    if (row < a.rows) {
      for (uint32_t c = lane * kVec; c < a.cols; c += tpr * kVec) {
        const uint32_t nvalid = (a.cols - c >= (uint32_t)kVec) ? (uint32_t)kVec : a.cols - c;
        const uint32_t i = row * a.cols + c;
        RF<16> f = load_inputs<16>(rf_zero<16>(), pro, 0, i, nvalid);
        f = interp<16>(f, pro_regs, pro_n);
        acc = fold_vec(a.red, acc, rf_get(f, pro.anchor_slot), nvalid);
      }
    }
    float r;
    if (tpr == 64u) r = wave_reduce(a.red, acc);
    else r = block_reduce(a.red, acc, lds);
    if (a.red == kRedMean) r = r / (float)a.cols;
    if (lane == 0 && row < a.rows) run_post(a.post, post_regs, splat(r), row, 1u);
  }
}

// Global reduction in one launch.  U independent 4-vectors per lane and loop trip: all their
// loads are issued before the first is interpreted (a reduction has few inputs, so memory-level
// parallelism has to come from unrolling).
template <int MAXIN, int U, bool FAST, bool F32>
__global__ __launch_bounds__(kBlock) void lt_all_reduce_kernel(const AllArgs a) {
  __shared__ float lds[kBlock / 64];
  __shared__ uint32_t is_last;
  const EwProg& pro = a.pro;
  const ProgRegs pro_regs = load_prog_regs(a.pro), post_regs = load_prog_regs(a.post);
  const uint32_t pro_n = a.pro.n_code;
  const uint64_t n = pro.n;
  const uint64_t nvec = (n + kVec - 1) / kVec;
  float acc = red_identity(a.red);
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  const uint64_t full_trips = FAST ? nvec / (stride * U) : 0;     // every lane has U whole vectors
  uint64_t v = (uint64_t)blockIdx.x * kBlock + threadIdx.x;
  for (uint64_t t = 0; t < full_trips; ++t) {
    Staged<MAXIN> st[U];
#pragma unroll
    for (int u = 0; u < U; ++u)
      st[u] = fetch_inputs<MAXIN, FAST, F32, false>(pro, 0, (uint32_t)((v + (uint64_t)u * stride) * kVec), kVec);
#pragma unroll
    for (int u = 0; u < U; ++u) pin_staged<MAXIN>(st[u]);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      RF<16> f = place_inputs<16, MAXIN, FAST, F32>(rf_zero<16>(), pro, st[u], kVec);
      f = interp<16>(f, pro_regs, pro_n);
      acc = fold_vec(a.red, acc, rf_get(f, pro.anchor_slot), kVec);
    }
    v += stride * U;
  }
  for (; v < nvec; v += stride) {
    const uint64_t i = v * kVec;
    const uint32_t nvalid = (n - i >= (uint64_t)kVec) ? (uint32_t)kVec : (uint32_t)(n - i);
    RF<16> f = load_inputs<16, MAXIN, false, false>(rf_zero<16>(), pro, 0, (uint32_t)i, nvalid);
    f = interp<16>(f, pro_regs, pro_n);
    acc = fold_vec(a.red, acc, rf_get(f, pro.anchor_slot), nvalid);
  }
  float r = block_reduce(a.red, acc, lds);
  if (threadIdx.x == 0) {
    __hip_atomic_store(&a.partials[blockIdx.x], r, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __threadfence();
    uint32_t t = atomicAdd(a.ticket, 1u);
    is_last = (t == gridDim.x - 1) ? 1u : 0u;
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  // the last workgroup combines the partials in a fixed order (deterministic for a given grid)
  acc = red_identity(a.red);
  for (uint32_t g = threadIdx.x; g < gridDim.x; g += kBlock)
    acc = red_combine(a.red, acc, __hip_atomic_load(&a.partials[g], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  r = block_reduce(a.red, acc, lds);
  if (a.red == kRedMean) r = r / (float)a.count;
  if (threadIdx.x == 0) *a.ticket = 0u;
  const EwProg& post = a.post;
  const uint64_t pn = post.n;
  const uint64_t pvec = (pn + kVec - 1) / kVec;
  for (uint64_t v = threadIdx.x; v < pvec; v += kBlock) {
    const uint64_t i = v * kVec;
    const uint32_t nvalid = (pn - i >= (uint64_t)kVec) ? (uint32_t)kVec : (uint32_t)(pn - i);
    run_post(post, post_regs, splat(r), i, nvalid);
  }
}

// Column reduction over axis 0 of [rows, cols].  blockIdx.x: strip of 256 columns (64 lanes x 4);
// the four waves of a workgroup take interleaved rows; blockIdx.y: slab of rows.
__global__ __launch_bounds__(kBlock) void lt_col_reduce_kernel(const ColArgs a) {
  __shared__ float4 lds[kBlock];
  __shared__ uint32_t is_last;
  const EwProg& pro = a.pro;
  const ProgRegs pro_regs = load_prog_regs(a.pro), post_regs = load_prog_regs(a.post);
  const uint32_t pro_n = a.pro.n_code;
  const uint32_t lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint32_t c = blockIdx.x * 256u + lane * kVec;
  const uint32_t nvalid = c >= a.cols ? 0u : ((a.cols - c >= (uint32_t)kVec) ? (uint32_t)kVec : a.cols - c);
  const uint32_t rows_per_slab = (a.rows + gridDim.y - 1) / gridDim.y;
  const uint32_t r0 = blockIdx.y * rows_per_slab;
  const uint32_t r1 = min(a.rows, r0 + rows_per_slab);
  const float id = red_identity(a.red);
  float4 acc = make_float4(id, id, id, id);
  if (nvalid) {
    for (uint32_t r = r0 + wave; r < r1; r += kBlock / 64) {
      const uint32_t i = r * a.cols + c;
      RF<16> f = load_inputs<16>(rf_zero<16>(), pro, 0, i, nvalid);
      f = interp<16>(f, pro_regs, pro_n);
      const Quad q = rf_get(f, pro.anchor_slot);
      acc.x = red_combine(a.red, acc.x, q.v[0]);
      acc.y = red_combine(a.red, acc.y, q.v[1]);
      acc.z = red_combine(a.red, acc.z, q.v[2]);
      acc.w = red_combine(a.red, acc.w, q.v[3]);
    }
  }
  lds[threadIdx.x] = acc;
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int w = 1; w < kBlock / 64; ++w) {
      float4 o = lds[w * 64 + lane];
      acc.x = red_combine(a.red, acc.x, o.x);
      acc.y = red_combine(a.red, acc.y, o.y);
      acc.z = red_combine(a.red, acc.z, o.z);
      acc.w = red_combine(a.red, acc.w, o.w);
    }
    if (nvalid) {
      float* dst = a.partials + (uint64_t)blockIdx.y * a.cols + c;
      if (nvalid > 0u) __hip_atomic_store(dst + 0, acc.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (nvalid > 1u) __hip_atomic_store(dst + 1, acc.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (nvalid > 2u) __hip_atomic_store(dst + 2, acc.z, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (nvalid > 3u) __hip_atomic_store(dst + 3, acc.w, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    uint32_t t = atomicAdd(&a.tickets[blockIdx.x], 1u);
    is_last = (t == gridDim.y - 1) ? 1u : 0u;
  }
  __syncthreads();
  if (!is_last) return;
  __threadfence();
  if (threadIdx.x == 0) a.tickets[blockIdx.x] = 0u;
  if (wave != 0 || !nvalid) return;
  acc = make_float4(id, id, id, id);
  for (uint32_t s = 0; s < gridDim.y; ++s) {
    const float* src = a.partials + (uint64_t)s * a.cols + c;
    if (nvalid > 0u) acc.x = red_combine(a.red, acc.x, __hip_atomic_load(src + 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (nvalid > 1u) acc.y = red_combine(a.red, acc.y, __hip_atomic_load(src + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (nvalid > 2u) acc.z = red_combine(a.red, acc.z, __hip_atomic_load(src + 2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
    if (nvalid > 3u) acc.w = red_combine(a.red, acc.w, __hip_atomic_load(src + 3, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
  }
  if (a.red == kRedMean) {
    const float inv = 1.0f / (float)a.rows;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  }
  Quad accq;
  accq.v[0] = acc.x; accq.v[1] = acc.y; accq.v[2] = acc.z; accq.v[3] = acc.w;
  run_post(a.post, post_regs, accq, c, nvalid);
}


hipError_t launch_row_reduce(const RowArgs& a, uint32_t grid, hipStream_t s) {
  hipLaunchKernelGGL(lt_row_reduce_kernel, dim3(grid), dim3(kBlock), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_all_reduce(const AllArgs& a, uint32_t grid, hipStream_t s) {
  if (a.pro.fast && a.pro.all_f32 && a.pro.n_in <= 2u)
    hipLaunchKernelGGL((lt_all_reduce_kernel<2, 4, true, true>), dim3(grid), dim3(kBlock), 0, s, a);
  else
    hipLaunchKernelGGL((lt_all_reduce_kernel<8, 1, false, false>), dim3(grid), dim3(kBlock), 0, s, a);
  return hipGetLastError();
}
hipError_t launch_col_reduce(const ColArgs& a, uint32_t grid_x, uint32_t grid_y, hipStream_t s) {
  hipLaunchKernelGGL(lt_col_reduce_kernel, dim3(grid_x, grid_y), dim3(kBlock), 0, s, a);
  return hipGetLastError();
}

}  // namespace ltk
