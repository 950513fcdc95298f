// Wavefront / workgroup reduction helpers shared by the reduction and row-operator kernels.
#ifndef LT_REDUCE_H_
#define LT_REDUCE_H_
#include "lt_interp.h"

namespace ltk {
constexpr int kBlock = 256;
__device__ __forceinline__ float red_identity(uint32_t red) { return red == kRedMax ? -INFINITY : 0.0f; }
__device__ __forceinline__ float red_combine(uint32_t red, float x, float y) {
  if (red == kRedMax) return (x != x || y != y) ? (x + y) : fmaxf(x, y);
  return x + y;
}

// Partial results travel between workgroups of one launch, which may sit on different dies with
// different L2 caches.  They are written and read with relaxed device-scope atomic accesses --
// stores and loads that go through to the memory side -- so that no cache has to be written back
// or invalidated as a whole, which is what a device-scope fence does (microseconds per fence, and
// every other workgroup of the die loses what it had cached).  Order: the writer waits for its
// stores (a workgroup-scope release: a wait, no cache operation) before it takes the ticket; the
// reader starts only after it has seen the last ticket.
__device__ __forceinline__ void publish(float* p, float v) { __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ float published(const float* p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); }
__device__ __forceinline__ void publish4(float* p, const float4& v) {   // p 16-byte aligned
  const uint64_t lo = (uint64_t)__float_as_uint(v.x) | ((uint64_t)__float_as_uint(v.y) << 32);
  const uint64_t hi = (uint64_t)__float_as_uint(v.z) | ((uint64_t)__float_as_uint(v.w) << 32);
  __hip_atomic_store((uint64_t*)p, lo, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  __hip_atomic_store((uint64_t*)p + 1, hi, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float4 published4(const float* p) {
  const uint64_t lo = __hip_atomic_load((const uint64_t*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  const uint64_t hi = __hip_atomic_load((const uint64_t*)p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float4(__uint_as_float((uint32_t)lo), __uint_as_float((uint32_t)(lo >> 32)), __uint_as_float((uint32_t)hi),
                     __uint_as_float((uint32_t)(hi >> 32)));
}

// One butterfly step inside a row of 16 lanes through the data-parallel-primitive lane crossbar
// (no LDS traffic).  CTRL: 0xB1 swaps neighbours, 0x4E swaps pairs, 0x141 mirrors each half row
// (reaches the other quad), 0x140 mirrors the row (reaches the other half).
template <int CTRL>
__device__ __forceinline__ float dpp_step(uint32_t red, float v) {
  const float o = __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), CTRL, 0xf, 0xf, true));
  return red_combine(red, v, o);
}

// Reduction over each aligned group of 16 lanes; every lane of the group gets the result.
__device__ __forceinline__ float row16_reduce(uint32_t red, float v) {
  v = dpp_step<0xB1>(red, v);
  v = dpp_step<0x4E>(red, v);
  v = dpp_step<0x141>(red, v);
  v = dpp_step<0x140>(red, v);
  return v;
}

// Reduction over the 64 lanes of a wavefront; every lane gets the result.  The four row results
// travel through scalar registers and are combined in a fixed order.
__device__ __forceinline__ float wave_reduce(uint32_t red, float v) {
  v = row16_reduce(red, v);
  const int b = __float_as_int(v);
  const float r0 = __int_as_float(__builtin_amdgcn_readlane(b, 0)), r1 = __int_as_float(__builtin_amdgcn_readlane(b, 16));
  const float r2 = __int_as_float(__builtin_amdgcn_readlane(b, 32)), r3 = __int_as_float(__builtin_amdgcn_readlane(b, 48));
  return red_combine(red, red_combine(red, r0, r1), red_combine(red, r2, r3));
}

// reduce over the kBlock threads of a workgroup; result valid in every thread
__device__ __forceinline__ float block_reduce(uint32_t red, float v, float* lds /* >= 4 floats */) {
  v = wave_reduce(red, v);
  const int wave = threadIdx.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) lds[wave] = v;
  __syncthreads();
  float r = lds[0];
#pragma unroll
  for (int w = 1; w < kBlock / 64; ++w) r = red_combine(red, r, lds[w]);
  return r;
}

// combine the (valid) element lanes of slot `slot`
__device__ __forceinline__ float fold_vec(uint32_t red, float acc, const Quad& q, uint32_t nvalid) {
  if (nvalid > 0u) acc = red_combine(red, acc, q.v[0]);
  if (nvalid > 1u) acc = red_combine(red, acc, q.v[1]);
  if (nvalid > 2u) acc = red_combine(red, acc, q.v[2]);
  if (nvalid > 3u) acc = red_combine(red, acc, q.v[3]);
  return acc;
}


}  // namespace ltk
#endif
