// Row operators with a fixed body (softmax, layer norm, cross-entropy and their gradients): one
// workgroup or wavefront per row, the row held in registers between passes, LDS only for the
// cross-wave step of the reductions.
#include <hip/hip_runtime.h>

#include "lt_launch.h"
#include "lt_reduce.h"

namespace ltk {

// ---- fixed-body row operators: the row is held in registers between passes ----------------------
constexpr int kRowVecs = 4;   // 4-vectors per thread: rows up to threads_per_row * 16 columns

struct RowRegs {
  float4 v[kRowVecs];
};

__device__ __forceinline__ RowRegs row_load(const void* ptr, uint32_t dtype, uint64_t base, uint32_t cols,
                                            uint32_t lane, uint32_t tpr, bool vec_ok, float pad) {
  RowRegs r;
#pragma unroll
  for (int k = 0; k < kRowVecs; ++k) {
    const uint32_t c = (k * tpr + lane) * kVec;
    float4 q = make_float4(pad, pad, pad, pad);
    if (c < cols) {
      if (vec_ok) {
        const Quad t = finish_vec4(dtype, fetch_vec4(ptr, dtype, base, c));
        q = make_float4(t.v[0], t.v[1], t.v[2], t.v[3]);
      } else {
        q.x = load_elem(ptr, dtype, base + c);
        if (c + 1 < cols) q.y = load_elem(ptr, dtype, base + c + 1);
        if (c + 2 < cols) q.z = load_elem(ptr, dtype, base + c + 2);
        if (c + 3 < cols) q.w = load_elem(ptr, dtype, base + c + 3);
      }
    }
    r.v[k] = q;
  }
  return r;
}

__device__ __forceinline__ void row_store(void* ptr, uint32_t dtype, uint64_t base, uint32_t cols, uint32_t lane,
                                          uint32_t tpr, bool vec_ok, const RowRegs& r) {
#pragma unroll
  for (int k = 0; k < kRowVecs; ++k) {
    const uint32_t c = (k * tpr + lane) * kVec;
    if (c >= cols) continue;
    const float4 q = r.v[k];
    if (vec_ok) {
      if (dtype == kBF16) {
        uint2 u;
        u.x = (uint32_t)f32_to_bf16(q.x) | ((uint32_t)f32_to_bf16(q.y) << 16);
        u.y = (uint32_t)f32_to_bf16(q.z) | ((uint32_t)f32_to_bf16(q.w) << 16);
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

__device__ __forceinline__ float row_reduce_regs(uint32_t red, const RowRegs& r, uint32_t tpr, float* lds) {
  float acc = red_identity(red);
#pragma unroll
  for (int k = 0; k < kRowVecs; ++k) {
    acc = red_combine(red, acc, red_combine(red, red_combine(red, r.v[k].x, r.v[k].y),
                                            red_combine(red, r.v[k].z, r.v[k].w)));
  }
  return tpr == 64u ? wave_reduce(red, acc) : block_reduce(red, acc, lds);
}

#define LT_ROW_FOREACH(BODY)                                   \
  _Pragma("unroll") for (int k = 0; k < kRowVecs; ++k) {       \
    { float& e = x.v[k].x; const int j = 0; (void)j; BODY }    \
    { float& e = x.v[k].y; const int j = 1; (void)j; BODY }    \
    { float& e = x.v[k].z; const int j = 2; (void)j; BODY }    \
    { float& e = x.v[k].w; const int j = 3; (void)j; BODY }    \
  }

__device__ __forceinline__ float comp(const float4& q, int j) { return j == 0 ? q.x : j == 1 ? q.y : j == 2 ? q.z : q.w; }

__global__ __launch_bounds__(kBlock) void lt_row_op_kernel(const RowOpArgs a) {
  __shared__ float lds[kBlock / 64];
  const uint32_t tpr = a.threads_per_row;
  const uint32_t rows_per_block = kBlock / tpr;
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
    switch (a.op) {
      case kSoftmax: {
        RowRegs x = row_load(a.in[0], a.in_dtype[0], base, ecols, lane, tpr, vec_ok, -INFINITY);
        const float m = row_reduce_regs(kRedMax, x, tpr, lds);
        LT_ROW_FOREACH(e = __expf(e - m);)
        const float s = row_reduce_regs(kRedSum, x, tpr, lds);
        const float inv = 1.0f / s;
        LT_ROW_FOREACH(e = e * inv;)
        row_store(a.out[0], a.out_dtype[0], base, ecols, lane, tpr, vec_ok, x);
      } break;
      case kSoftmaxGrad: {
        RowRegs x = row_load(a.in[0], a.in_dtype[0], base, ecols, lane, tpr, vec_ok, 0.0f);   // dy
        RowRegs y = row_load(a.in[1], a.in_dtype[1], base, ecols, lane, tpr, vec_ok, 0.0f);
        RowRegs t = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          t.v[k].x *= y.v[k].x; t.v[k].y *= y.v[k].y; t.v[k].z *= y.v[k].z; t.v[k].w *= y.v[k].w;
        }
        const float dot = row_reduce_regs(kRedSum, t, tpr, lds);
        LT_ROW_FOREACH(e = comp(y.v[k], j) * (e - dot);)
        row_store(a.out[0], a.out_dtype[0], base, ecols, lane, tpr, vec_ok, x);
      } break;
      case kLayerNorm: {
        RowRegs x = row_load(a.in[0], a.in_dtype[0], base, ecols, lane, tpr, vec_ok, 0.0f);
        const float mean = row_reduce_regs(kRedSum, x, tpr, lds) / (float)cols;
        RowRegs d = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          const uint32_t c = (k * tpr + lane) * kVec;
          d.v[k].x = (c + 0 < ecols) ? (x.v[k].x - mean) * (x.v[k].x - mean) : 0.0f;
          d.v[k].y = (c + 1 < ecols) ? (x.v[k].y - mean) * (x.v[k].y - mean) : 0.0f;
          d.v[k].z = (c + 2 < ecols) ? (x.v[k].z - mean) * (x.v[k].z - mean) : 0.0f;
          d.v[k].w = (c + 3 < ecols) ? (x.v[k].w - mean) * (x.v[k].w - mean) : 0.0f;
        }
        const float var = row_reduce_regs(kRedSum, d, tpr, lds) / (float)cols;
        const float rstd = 1.0f / sqrtf(var + a.eps);
        RowRegs g = row_load(a.in[1], a.in_dtype[1], 0, ecols, lane, tpr, vec_ok, 0.0f);
        RowRegs b = row_load(a.in[2], a.in_dtype[2], 0, ecols, lane, tpr, vec_ok, 0.0f);
        LT_ROW_FOREACH(e = (e - mean) * rstd * comp(g.v[k], j) + comp(b.v[k], j);)
        row_store(a.out[0], a.out_dtype[0], base, ecols, lane, tpr, vec_ok, x);
        if (lane == 0 && live) {
          store_elem(a.out[1], a.out_dtype[1], row, mean);
          store_elem(a.out[2], a.out_dtype[2], row, rstd);
        }
      } break;
      case kLayerNormGrad: {
        // in: dy, x, gamma, mean, rstd
        RowRegs x = row_load(a.in[0], a.in_dtype[0], base, ecols, lane, tpr, vec_ok, 0.0f);   // dy -> g
        RowRegs xh = row_load(a.in[1], a.in_dtype[1], base, ecols, lane, tpr, vec_ok, 0.0f);
        RowRegs gm = row_load(a.in[2], a.in_dtype[2], 0, ecols, lane, tpr, vec_ok, 0.0f);
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
        const float mg = row_reduce_regs(kRedSum, x, tpr, lds) / (float)cols;
        RowRegs t = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          t.v[k].x *= xh.v[k].x; t.v[k].y *= xh.v[k].y; t.v[k].z *= xh.v[k].z; t.v[k].w *= xh.v[k].w;
        }
        const float mgx = row_reduce_regs(kRedSum, t, tpr, lds) / (float)cols;
        LT_ROW_FOREACH(e = rstd * (e - mg - comp(xh.v[k], j) * mgx);)
        row_store(a.out[0], a.out_dtype[0], base, ecols, lane, tpr, vec_ok, x);
      } break;
      case kXent:
      case kXentGrad: {
        RowRegs x = row_load(a.in[0], a.in_dtype[0], base, ecols, lane, tpr, vec_ok, -INFINITY);
        const int32_t label = live ? ((const int32_t*)a.in[1])[row] : 0;
        const float m = row_reduce_regs(kRedMax, x, tpr, lds);
        RowRegs ex = x;
#pragma unroll
        for (int k = 0; k < kRowVecs; ++k) {
          ex.v[k].x = expf(x.v[k].x - m); ex.v[k].y = expf(x.v[k].y - m);
          ex.v[k].z = expf(x.v[k].z - m); ex.v[k].w = expf(x.v[k].w - m);
        }
        const float s = row_reduce_regs(kRedSum, ex, tpr, lds);
        if (a.op == kXent) {
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
          const float pv = row_reduce_regs(kRedSum, pk, tpr, lds);
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
          row_store(a.out[0], a.out_dtype[0], base, ecols, lane, tpr, vec_ok, ex);
        }
      } break;
      default: break;
    }
  }
}


hipError_t launch_row_op(const RowOpArgs& a, uint32_t grid, hipStream_t s) {
  hipLaunchKernelGGL(lt_row_op_kernel, dim3(grid), dim3(kBlock), 0, s, a);
  return hipGetLastError();
}

}  // namespace ltk
