// Register-resident bytecode interpreter (device side).
//
// A program is a list of three-address instructions over up to 32 value slots.  Each lane
// processes kVec = 4 elements, so a slot is four vector registers; the four "columns" of
// the register file are kept in four 32-wide vector values that the compiler indexes with a
// wave-uniform index (the instruction word comes from the kernel-argument segment through
// scalar loads), which lowers to relative register addressing -- no scratch memory, no LDS.
// The register file is passed and returned BY VALUE on purpose: element-indexed access to a
// vector that lives behind a reference is turned into memory accesses and would spill it.
// For the same reason slot indices are NOT masked here: an index the optimiser can prove in
// range lets it rewrite "load vector, extract element" as a scalar load from a stack copy.
// The host validates every program (slots < n_slots <= NS) before it is ever launched.
#ifndef LT_INTERP_H_
#define LT_INTERP_H_

#include <hip/hip_runtime.h>

#include "lt_kernels.h"

namespace ltk {

template <int NS> struct SlotVec;
template <> struct SlotVec<16> { typedef float type __attribute__((ext_vector_type(16))); };
template <> struct SlotVec<32> { typedef float type __attribute__((ext_vector_type(32))); };

// Register file of NS value slots (16 or 32) x 4 element lanes.
template <int NS> struct RF {
  typedef typename SlotVec<NS>::type vec;
  vec e0, e1, e2, e3;   // element lane 0..3 of every slot
};

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round to nearest even; NaN stays NaN
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return (uint16_t)(u >> 16);
}

__device__ __forceinline__ float op_gelu(float x) { return 0.5f * x * (1.0f + erff(x * 0.70710678118654752f)); }
__device__ __forceinline__ float op_gelu_grad(float dy, float x) {
  float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
  float pdf = 0.39894228040143268f * __expf(-0.5f * x * x);
  return dy * (cdf + x * pdf);
}

#define LT_RD4(i) make_float4(r0[i], r1[i], r2[i], r3[i])
#define LT_WR4(i, q) \
  {                  \
    r0[i] = (q).x;   \
    r1[i] = (q).y;   \
    r2[i] = (q).z;   \
    r3[i] = (q).w;   \
  }
// apply EXPR (in terms of xa, xb, xc) to the four element lanes
#define LT_MAP(EXPR)                                   \
  {                                                    \
    float4 q;                                          \
    { float xa = A.x, xb = B.x, xc = C.x; (void)xb; (void)xc; q.x = (EXPR); } \
    { float xa = A.y, xb = B.y, xc = C.y; (void)xb; (void)xc; q.y = (EXPR); } \
    { float xa = A.z, xb = B.z, xc = C.z; (void)xb; (void)xc; q.z = (EXPR); } \
    { float xa = A.w, xb = B.w, xc = C.w; (void)xb; (void)xc; q.w = (EXPR); } \
    LT_WR4(d, q);                                      \
  }

template <int NS>
__device__ __forceinline__ RF<NS> interp(RF<NS> f, const EwProg& p) {
  typename RF<NS>::vec r0 = f.e0, r1 = f.e1, r2 = f.e2, r3 = f.e3;
  const uint32_t n = p.n_code;
  for (uint32_t pc = 0; pc < n; ++pc) {
    const uint32_t w = p.code[pc];
    const uint32_t op = w & 0xffu, d = (w >> 8) & 31u;
    const uint32_t ia = (w >> 13) & 63u, ib = (w >> 19) & 63u, ic = (w >> 25) & 63u;
    float4 A, B, C;
    if (ia < 32u) { A = LT_RD4(ia); } else { float s = p.scal[ia - 32u]; A = make_float4(s, s, s, s); }
    if (ib < 32u) { B = LT_RD4(ib); } else { float s = p.scal[ib - 32u]; B = make_float4(s, s, s, s); }
    C = A;
    if (op == kFma) {
      if (ic < 32u) { C = LT_RD4(ic); } else { float s = p.scal[ic - 32u]; C = make_float4(s, s, s, s); }
    }
    switch (op) {
      case kMov: LT_MAP(xa) break;
      case kNeg: LT_MAP(-xa) break;
      case kAbs: LT_MAP(fabsf(xa)) break;
      case kExp: LT_MAP(expf(xa)) break;
      case kLog: LT_MAP(logf(xa)) break;
      case kTanh: LT_MAP(tanhf(xa)) break;
      case kSqrt: LT_MAP(sqrtf(xa)) break;
      case kRsqrt: LT_MAP(rsqrtf(xa)) break;
      case kRecip: LT_MAP(1.0f / xa) break;
      case kRelu: LT_MAP(xa > 0.0f ? xa : 0.0f) break;
      case kGelu: LT_MAP(op_gelu(xa)) break;
      case kSquare: LT_MAP(xa * xa) break;
      case kSigmoid: LT_MAP(1.0f / (1.0f + expf(-xa))) break;
      case kRoundBf16: LT_MAP(bf16_to_f32(f32_to_bf16(xa))) break;
      case kAdd: LT_MAP(xa + xb) break;
      case kSub: LT_MAP(xa - xb) break;
      case kMul: LT_MAP(xa * xb) break;
      case kDiv: LT_MAP(xa / xb) break;
      case kMax: LT_MAP((xa != xa || xb != xb) ? (xa + xb) : fmaxf(xa, xb)) break;
      case kMin: LT_MAP((xa != xa || xb != xb) ? (xa + xb) : fminf(xa, xb)) break;
      case kReluGrad: LT_MAP(xb > 0.0f ? xa : 0.0f) break;
      case kGeluGrad: LT_MAP(op_gelu_grad(xa, xb)) break;
      case kFma: LT_MAP(fmaf(xa, xb, xc)) break;
      default: break;
    }
  }
  RF<NS> o;
  o.e0 = r0; o.e1 = r1; o.e2 = r2; o.e3 = r3;
  return o;
}

// ---- loads -------------------------------------------------------------------------------

__device__ __forceinline__ float load_elem(const void* ptr, uint32_t dtype, uint64_t idx) {
  if (dtype == kBF16) return bf16_to_f32(((const uint16_t*)ptr)[idx]);
  if (dtype == kI32) return (float)((const int32_t*)ptr)[idx];
  return ((const float*)ptr)[idx];
}

__device__ __forceinline__ float4 load_vec4(const void* ptr, uint32_t dtype, uint64_t idx) {
  if (dtype == kBF16) {
    uint2 u = *(const uint2*)((const uint16_t*)ptr + idx);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u),
                       __uint_as_float(u.y << 16), __uint_as_float(u.y & 0xffff0000u));
  }
  return *(const float4*)((const float*)ptr + idx);
}

__device__ __forceinline__ uint64_t strided_index(const EwProg& p, const EwIn& in, uint64_t i) {
  uint64_t c3 = i % p.dims[3]; i /= p.dims[3];
  uint64_t c2 = i % p.dims[2]; i /= p.dims[2];
  uint64_t c1 = i % p.dims[1]; i /= p.dims[1];
  return (uint64_t)((int64_t)i * in.stride[0] + (int64_t)c1 * in.stride[1] + (int64_t)c2 * in.stride[2] +
                    (int64_t)c3 * in.stride[3]);
}

// Load the (up to) four consecutive elements i .. i+3 of the iteration space for input k.
// nvalid < 4 at a ragged tail; missing elements read as `pad`.
__device__ __forceinline__ float4 load_input(const EwProg& p, int k, uint64_t i, uint32_t nvalid, float pad) {
  const EwIn& in = p.in[k];
  const uint32_t mode = in.mode, dt = in.dtype;
  if (mode == kScalar) {
    float s = load_elem(in.ptr, dt, 0);
    return make_float4(s, s, s, s);
  }
  const bool fast = p.vec_ok && nvalid == 4u;
  if (mode == kFull) {
    if (p.full_vec_ok && nvalid == 4u) return load_vec4(in.ptr, dt, i);
    float4 q = make_float4(pad, pad, pad, pad);
    if (nvalid > 0u) q.x = load_elem(in.ptr, dt, i);
    if (nvalid > 1u) q.y = load_elem(in.ptr, dt, i + 1);
    if (nvalid > 2u) q.z = load_elem(in.ptr, dt, i + 2);
    if (nvalid > 3u) q.w = load_elem(in.ptr, dt, i + 3);
    return q;
  }
  if (mode == kRowVec) {
    if (fast) return load_vec4(in.ptr, dt, i % p.cols);
    float4 q = make_float4(pad, pad, pad, pad);
    if (nvalid > 0u) q.x = load_elem(in.ptr, dt, i % p.cols);
    if (nvalid > 1u) q.y = load_elem(in.ptr, dt, (i + 1) % p.cols);
    if (nvalid > 2u) q.z = load_elem(in.ptr, dt, (i + 2) % p.cols);
    if (nvalid > 3u) q.w = load_elem(in.ptr, dt, (i + 3) % p.cols);
    return q;
  }
  if (mode == kColVec) {
    if (p.vec_ok) {
      float s = load_elem(in.ptr, dt, i / p.cols);
      return make_float4(s, s, s, s);
    }
    float4 q = make_float4(pad, pad, pad, pad);
    if (nvalid > 0u) q.x = load_elem(in.ptr, dt, i / p.cols);
    if (nvalid > 1u) q.y = load_elem(in.ptr, dt, (i + 1) / p.cols);
    if (nvalid > 2u) q.z = load_elem(in.ptr, dt, (i + 2) / p.cols);
    if (nvalid > 3u) q.w = load_elem(in.ptr, dt, (i + 3) / p.cols);
    return q;
  }
  // kStrided
  float4 q = make_float4(pad, pad, pad, pad);
  if (nvalid > 0u) q.x = load_elem(in.ptr, dt, strided_index(p, in, i));
  if (nvalid > 1u) q.y = load_elem(in.ptr, dt, strided_index(p, in, i + 1));
  if (nvalid > 2u) q.z = load_elem(in.ptr, dt, strided_index(p, in, i + 2));
  if (nvalid > 3u) q.w = load_elem(in.ptr, dt, strided_index(p, in, i + 3));
  return q;
}

// Put all inputs of the program into slots 0 .. n_in-1.  The loop is fully unrolled so the
// slot index is a compile-time constant and all loads are in flight before the first use.
template <int NS>
__device__ __forceinline__ RF<NS> load_inputs(RF<NS> f, const EwProg& p, uint64_t i, uint32_t nvalid) {
  typename RF<NS>::vec r0 = f.e0, r1 = f.e1, r2 = f.e2, r3 = f.e3;
  const uint32_t n_in = p.n_in;
#pragma unroll
  for (int k = 0; k < kMaxIn; ++k) {
    if ((uint32_t)k < n_in) {
      float4 q = load_input(p, k, i, nvalid, 0.0f);
      LT_WR4(k, q);
    }
  }
  RF<NS> o;
  o.e0 = r0; o.e1 = r1; o.e2 = r2; o.e3 = r3;
  return o;
}

template <int NS>
__device__ __forceinline__ float4 rf_get(RF<NS> f, uint32_t slot) {
  typename RF<NS>::vec r0 = f.e0, r1 = f.e1, r2 = f.e2, r3 = f.e3;
  return LT_RD4(slot);
}

template <int NS>
__device__ __forceinline__ RF<NS> rf_set(RF<NS> f, uint32_t slot, float4 q) {
  typename RF<NS>::vec r0 = f.e0, r1 = f.e1, r2 = f.e2, r3 = f.e3;
  LT_WR4(slot, q);
  RF<NS> o;
  o.e0 = r0; o.e1 = r1; o.e2 = r2; o.e3 = r3;
  return o;
}

__device__ __forceinline__ void store_elem(void* ptr, uint32_t dtype, uint64_t idx, float v) {
  if (dtype == kBF16) ((uint16_t*)ptr)[idx] = f32_to_bf16(v);
  else ((float*)ptr)[idx] = v;
}

// Store the outputs of the program for elements i .. i+nvalid-1 (flat, contiguous outputs).
template <int NS>
__device__ __forceinline__ void store_outputs(RF<NS> f, const EwProg& p, uint64_t i, uint32_t nvalid) {
  const uint32_t n_out = p.n_out;
#pragma unroll
  for (int o = 0; o < kMaxOut; ++o) {
    if ((uint32_t)o < n_out) {
      const EwOut& out = p.out[o];
      float4 q = rf_get(f, out.slot);
      if (out.scalar) {
        if (i == 0) store_elem(out.ptr, out.dtype, 0, q.x);
      } else if (p.full_vec_ok && nvalid == 4u) {
        if (out.dtype == kBF16) {
          uint2 u;
          u.x = (uint32_t)f32_to_bf16(q.x) | ((uint32_t)f32_to_bf16(q.y) << 16);
          u.y = (uint32_t)f32_to_bf16(q.z) | ((uint32_t)f32_to_bf16(q.w) << 16);
          *(uint2*)((uint16_t*)out.ptr + i) = u;
        } else {
          *(float4*)((float*)out.ptr + i) = q;
        }
      } else {
        if (nvalid > 0u) store_elem(out.ptr, out.dtype, i, q.x);
        if (nvalid > 1u) store_elem(out.ptr, out.dtype, i + 1, q.y);
        if (nvalid > 2u) store_elem(out.ptr, out.dtype, i + 2, q.z);
        if (nvalid > 3u) store_elem(out.ptr, out.dtype, i + 3, q.w);
      }
    }
  }
}

template <int NS>
__device__ __forceinline__ RF<NS> rf_zero() {
  RF<NS> f;
  f.e0 = 0.0f; f.e1 = 0.0f; f.e2 = 0.0f; f.e3 = 0.0f;
  return f;
}

}  // namespace ltk
#endif  // LT_INTERP_H_
