// Row operators with a fixed body (softmax, layer norm, cross-entropy and their gradients): one
// workgroup or wavefront per row, the row held in registers between passes, LDS only for the
// cross-wave step of the reductions.
#include <hip/hip_runtime.h>

#include <cstdio>

#include "lt_launch.h"
#include "lt_reduce.h"

namespace ltk {

// ---- fixed-body row operators: the row is held in registers between passes ----------------------
constexpr int kRowVecs = 4;   // 4-vectors per thread: rows up to threads_per_row * 16 columns

struct RowRegs {
  float4 v[kRowVecs];
};

// IO: 0 = element types read from the arguments at run time, 1 = every row-wide tensor is fp32,
// 2 = every row-wide tensor is bf16 (the type branches fold away).
template <int IO>
__device__ __forceinline__ uint32_t io_dtype(uint32_t dtype) {
  return IO == 1 ? (uint32_t)kF32 : IO == 2 ? (uint32_t)kBF16 : dtype;
}

template <int TPR, int IO>
__device__ __forceinline__ RowRegs row_load(const void* ptr, uint32_t dtype_rt, uint64_t base, uint32_t cols, uint32_t lane,
                                            bool vec_ok, float pad) {
  const uint32_t dtype = io_dtype<IO>(dtype_rt);
  RowRegs r;
  if (vec_ok) {
    RawVec raw[kRowVecs];
#pragma unroll
    for (int k = 0; k < kRowVecs; ++k) {   // all loads first, conversions afterwards
      const uint32_t c = (k * TPR + lane) * kVec;
      if (c < cols) raw[k] = fetch_vec4(ptr, dtype, base, c);
    }
#pragma unroll
    for (int k = 0; k < kRowVecs; ++k) {
      const uint32_t c = (k * TPR + lane) * kVec;
      float4 q = make_float4(pad, pad, pad, pad);
      if (c < cols) {
        const Quad t = finish_vec4(dtype, raw[k]);
        q = make_float4(t.v[0], t.v[1], t.v[2], t.v[3]);
      }
      r.v[k] = q;
    }
    return r;
  }
#pragma unroll
  for (int k = 0; k < kRowVecs; ++k) {
    const uint32_t c = (k * TPR + lane) * kVec;
    float4 q = make_float4(pad, pad, pad, pad);
    if (c < cols) {
      q.x = load_elem(ptr, dtype, base + c);
      if (c + 1 < cols) q.y = load_elem(ptr, dtype, base + c + 1);
      if (c + 2 < cols) q.z = load_elem(ptr, dtype, base + c + 2);
      if (c + 3 < cols) q.w = load_elem(ptr, dtype, base + c + 3);
    }
    r.v[k] = q;
  }
  return r;
}

template <int TPR, int IO>
__device__ __forceinline__ void row_store(void* ptr, uint32_t dtype_rt, uint64_t base, uint32_t cols, uint32_t lane, bool vec_ok,
                                          const RowRegs& r) {
  const uint32_t dtype = io_dtype<IO>(dtype_rt);
#pragma unroll
  for (int k = 0; k < kRowVecs; ++k) {
    const uint32_t c = (k * TPR + lane) * kVec;
    if (c >= cols) continue;
    const float4 q = r.v[k];
    if (vec_ok) {
      if (dtype == kBF16) {
        uint2 u;
        u.x = f32_to_bf16_pair(q.x, q.y);
        u.y = f32_to_bf16_pair(q.z, q.w);
        *(uint2*)((uint16_t*)ptr + base + c) = u;
      } else {
        *(float4*)((float*)ptr + base + c) = q;
      }
    } else {
      store_elem(ptr, dtype, base + c, q.x);
      if (c + 1 < cols) store_elem(ptr, dtype, base + c + 1, q.y);
      if (c + 2 < cols) store_elem(ptr, dtype, base + c + 2, q.z);
      if (c + 3 < cols) store_elem(ptr, dtype, base + c + 3, q.w);
    }
  }
}

// Reduce over the TPR lanes that share a row: 16 (a quarter wavefront), 64 or the workgroup.
template <int TPR>
__device__ __forceinline__ float row_reduce_regs(uint32_t red, const RowRegs& r, float* lds) {
  float acc = red_identity(red);
#pragma unroll
  for (int k = 0; k < kRowVecs; ++k) {
    acc = red_combine(red, acc, red_combine(red, red_combine(red, r.v[k].x, r.v[k].y),
                                            red_combine(red, r.v[k].z, r.v[k].w)));
  }
  return TPR == 16 ? row16_reduce(red, acc) : TPR == 64 ? wave_reduce(red, acc) : block_reduce(red, acc, lds);
}

#define LT_ROW_FOREACH(BODY)                                   \
  _Pragma("unroll") for (int k = 0; k < kRowVecs; ++k) {       \
    { float& e = x.v[k].x; const int j = 0; (void)j; BODY }    \
    { float& e = x.v[k].y; const int j = 1; (void)j; BODY }    \
    { float& e = x.v[k].z; const int j = 2; (void)j; BODY }    \
    { float& e = x.v[k].w; const int j = 3; (void)j; BODY }    \
  }

__device__ __forceinline__ float comp(const float4& q, int j) { return j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w; }

template <int OP, int TPR, int IO>
__global__ __launch_bounds__(kBlock) void lt_row_op_kernel(const RowOpArgs a) {
  __shared__ float lds[kBlock / 64];
  constexpr uint32_t tpr = TPR;
  constexpr uint32_t rows_per_block = kBlock / tpr;
  const uint32_t lane = threadIdx.x % tpr, sub = threadIdx.x / tpr;
  const uint32_t cols = a.cols;
  const bool vec_ok = (cols % kVec) == 0;
  const uint32_t nblocks = (a.rows + rows_per_block - 1) / rows_per_block;
  for (uint32_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const uint32_t row = blk * rows_per_block + sub;
    // with 256 threads per row every thread of the workgroup works on the same row, so the
    // workgroup barriers inside block_reduce are reached uniformly; with 64 there are none
    const bool live = row < a.rows;
    const uint64_t base = (uint64_t)(live ? row : 0) * cols;
    const uint32_t ecols = live ? cols : 0u;
    switch (OP) {
      case kSoftmax: {
        RowRegs x = row_load<TPR, IO>(a.in[0], a.in_dtype[0], base, ecols, lane, vec_ok, -INFINITY);
        const float m = row_reduce_regs<TPR>(kRedMax, x, lds);
        LT_ROW_FOREACH(e = __expf(e - m);)
        const float s = row_reduce_regs<TPR>(kRedSum, x, lds);
        const float inv = 1.0f / s;
        LT_ROW_FOREACH(e = e * inv;)
        row_store<TPR, IO>(a.out[0], a.out_dtype[0], base, ecols, lane, vec_ok, x);
      } break;
      case kSoftmaxGrad: {
        RowRegs x = row_load<TPR, IO>(a.in[0], a.in_dtype[0], base, ecols, lane, vec_ok, 0.0f);   // dy
        RowRegs y = row_load<TPR, IO>(a.in[1], a.in_dtype[1], base, ecols, lane, vec_ok, 0.0f);
        RowRegs t = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          t.v[k].x *= y.v[k].x; t.v[k].y *= y.v[k].y; t.v[k].z *= y.v[k].z; t.v[k].w *= y.v[k].w;
        }
        const float dot = row_reduce_regs<TPR>(kRedSum, t, lds);
        LT_ROW_FOREACH(e = comp(y.v[k], j) * (e - dot);)
        row_store<TPR, IO>(a.out[0], a.out_dtype[0], base, ecols, lane, vec_ok, x);
      } break;
      case kLayerNorm: {
        RowRegs x = row_load<TPR, IO>(a.in[0], a.in_dtype[0], base, ecols, lane, vec_ok, 0.0f);
        // scale and shift are asked for together with the row: their (cache) latency passes under
        // the two reductions instead of after them
        RowRegs g = row_load<TPR, IO>(a.in[1], a.in_dtype[1], 0, ecols, lane, vec_ok, 0.0f);
        RowRegs b = row_load<TPR, IO>(a.in[2], a.in_dtype[2], 0, ecols, lane, vec_ok, 0.0f);
        const float mean = row_reduce_regs<TPR>(kRedSum, x, lds) / (float)cols;
        RowRegs d = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          const uint32_t c = (k * tpr + lane) * kVec;
          d.v[k].x = (c + 0 < ecols) ? (x.v[k].x - mean) * (x.v[k].x - mean) : 0.0f;
          d.v[k].y = (c + 1 < ecols) ? (x.v[k].y - mean) * (x.v[k].y - mean) : 0.0f;
          d.v[k].z = (c + 2 < ecols) ? (x.v[k].z - mean) * (x.v[k].z - mean) : 0.0f;
          d.v[k].w = (c + 3 < ecols) ? (x.v[k].w - mean) * (x.v[k].w - mean) : 0.0f;
        }
        const float var = row_reduce_regs<TPR>(kRedSum, d, lds) / (float)cols;
        const float rstd = 1.0f / sqrtf(var + a.eps);
        LT_ROW_FOREACH(e = (e - mean) * rstd * comp(g.v[k], j) + comp(b.v[k], j);)
        row_store<TPR, IO>(a.out[0], a.out_dtype[0], base, ecols, lane, vec_ok, x);
        if (lane == 0 && live) {
          store_elem(a.out[1], a.out_dtype[1], row, mean);
          store_elem(a.out[2], a.out_dtype[2], row, rstd);
        }
      } break;
      case kLayerNormGrad: {
        // in: dy, x, gamma, mean, rstd
        RowRegs x = row_load<TPR, IO>(a.in[0], a.in_dtype[0], base, ecols, lane, vec_ok, 0.0f);   // dy -> g
        RowRegs xh = row_load<TPR, IO>(a.in[1], a.in_dtype[1], base, ecols, lane, vec_ok, 0.0f);
        RowRegs gm = row_load<TPR, IO>(a.in[2], a.in_dtype[2], 0, ecols, lane, vec_ok, 0.0f);
        const float mean = live ? load_elem(a.in[3], a.in_dtype[3], row) : 0.0f;
        const float rstd = live ? load_elem(a.in[4], a.in_dtype[4], row) : 0.0f;
        LT_ROW_FOREACH(e = e * comp(gm.v[k], j);)
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          const uint32_t c = (k * tpr + lane) * kVec;
          xh.v[k].x = (c + 0 < ecols) ? (xh.v[k].x - mean) * rstd : 0.0f;
          xh.v[k].y = (c + 1 < ecols) ? (xh.v[k].y - mean) * rstd : 0.0f;
          xh.v[k].z = (c + 2 < ecols) ? (xh.v[k].z - mean) * rstd : 0.0f;
          xh.v[k].w = (c + 3 < ecols) ? (xh.v[k].w - mean) * rstd : 0.0f;
        }
        const float mg = row_reduce_regs<TPR>(kRedSum, x, lds) / (float)cols;
        RowRegs t = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          t.v[k].x *= xh.v[k].x; t.v[k].y *= xh.v[k].y; t.v[k].z *= xh.v[k].z; t.v[k].w *= xh.v[k].w;
        }
        const float mgx = row_reduce_regs<TPR>(kRedSum, t, lds) / (float)cols;
        LT_ROW_FOREACH(e = rstd * (e - mg - comp(xh.v[k], j) * mgx);)
        row_store<TPR, IO>(a.out[0], a.out_dtype[0], base, ecols, lane, vec_ok, x);
      } break;
      case kXent:
      case kXentGrad: {
        RowRegs x = row_load<TPR, IO>(a.in[0], a.in_dtype[0], base, ecols, lane, vec_ok, -INFINITY);
        const int32_t label = live ? ((const int32_t*)a.in[1])[row] : 0;
        const float m = row_reduce_regs<TPR>(kRedMax, x, lds);
        RowRegs ex = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          ex.v[k].x = expf(x.v[k].x - m); ex.v[k].y = expf(x.v[k].y - m);
          ex.v[k].z = expf(x.v[k].z - m); ex.v[k].w = expf(x.v[k].w - m);
        }
        const float s = row_reduce_regs<TPR>(kRedSum, ex, lds);
        if (OP == kXent) {
          // the picked logit: only the lane holding column `label` contributes
          float picked = 0.0f;
#pragma unroll
          for (int k = 0; k < kRowVecs; ++k) {
            const int32_t c = (int32_t)((k * tpr + lane) * kVec);
            if (label == c) picked = x.v[k].x;
            if (label == c + 1) picked = x.v[k].y;
            if (label == c + 2) picked = x.v[k].z;
            if (label == c + 3) picked = x.v[k].w;
          }
          RowRegs pk;
#pragma unroll
          for (int k = 0; k < kRowVecs; ++k) pk.v[k] = make_float4(0.f, 0.f, 0.f, 0.f);
          pk.v[0].x = picked;
          const float pv = row_reduce_regs<TPR>(kRedSum, pk, lds);
          if (lane == 0 && live) store_elem(a.out[0], a.out_dtype[0], row, logf(s) + m - pv);
        } else {
          const float inv = 1.0f / s;
#pragma unroll
          for (int k = 0; k < kRowVecs; ++k) {
            const int32_t c = (int32_t)((k * tpr + lane) * kVec);
            ex.v[k].x = (ex.v[k].x * inv - (label == c ? 1.0f : 0.0f)) * a.scale;
            ex.v[k].y = (ex.v[k].y * inv - (label == c + 1 ? 1.0f : 0.0f)) * a.scale;
            ex.v[k].z = (ex.v[k].z * inv - (label == c + 2 ? 1.0f : 0.0f)) * a.scale;
            ex.v[k].w = (ex.v[k].w * inv - (label == c + 3 ? 1.0f : 0.0f)) * a.scale;
          }
          row_store<TPR, IO>(a.out[0], a.out_dtype[0], base, ecols, lane, vec_ok, ex);
        }
      } break;
      default: break;
    }
  }
}


template <int OP, int TPR>
static void launch_io(const RowOpArgs& a, int io, uint32_t grid, hipStream_t s) {
  if (io == 1) LT_LAUNCH((lt_row_op_kernel<OP, TPR, 1>), dim3(grid), dim3(kBlock), s, a);
  else if (io == 2) LT_LAUNCH((lt_row_op_kernel<OP, TPR, 2>), dim3(grid), dim3(kBlock), s, a);
  else LT_LAUNCH((lt_row_op_kernel<OP, TPR, 0>), dim3(grid), dim3(kBlock), s, a);
  char name[48];
  snprintf(name, sizeof(name), "lt_row_op_kernel<%d, %d, %d>", (int)OP, (int)TPR, io == 1 ? 1 : io == 2 ? 2 : 0);
  note_kernel(name);
}

template <int OP>
static hipError_t launch_tpr(const RowOpArgs& a, int io, uint32_t grid, hipStream_t s) {
  if (a.threads_per_row == 16u) launch_io<OP, 16>(a, io, grid, s);
  else if (a.threads_per_row == 64u) launch_io<OP, 64>(a, io, grid, s);
  else if (a.threads_per_row == 256u) launch_io<OP, 256>(a, io, grid, s);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

// Which tensors of an operator are read or written a whole row at a time (the others are one
// value per row and keep their run-time type).
hipError_t launch_row_op(const RowOpArgs& a, uint32_t grid, hipStream_t s) {
  uint32_t wide_in = 0, wide_out = 1;
  switch (a.op) {
    case kSoftmax: wide_in = 1; break;
    case kSoftmaxGrad: wide_in = 2; break;
    case kLayerNorm: wide_in = 3; break;
    case kLayerNormGrad: wide_in = 3; break;
    case kXent: wide_in = 1; wide_out = 0; break;
    case kXentGrad: wide_in = 1; break;
    default: return hipErrorInvalidValue;
  }
  bool f32 = true, bf16 = true;
  for (uint32_t i = 0; i < wide_in; ++i) { f32 &= a.in_dtype[i] == kF32; bf16 &= a.in_dtype[i] == kBF16; }
  for (uint32_t i = 0; i < wide_out; ++i) { f32 &= a.out_dtype[i] == kF32; bf16 &= a.out_dtype[i] == kBF16; }
  const int io = f32 ? 1 : bf16 ? 2 : 0;
  switch (a.op) {
    case kSoftmax: return launch_tpr<kSoftmax>(a, io, grid, s);
    case kSoftmaxGrad: return launch_tpr<kSoftmaxGrad>(a, io, grid, s);
    case kLayerNorm: return launch_tpr<kLayerNorm>(a, io, grid, s);
    case kLayerNormGrad: return launch_tpr<kLayerNormGrad>(a, io, grid, s);
    case kXent: return launch_tpr<kXent>(a, io, grid, s);
    default: return launch_tpr<kXentGrad>(a, io, grid, s);
  }
}

}  // namespace ltk
