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

__device__ __forceinline__ float wave_reduce(uint32_t red, float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = red_combine(red, v, __shfl_xor(v, off, 64));
  return v;
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
