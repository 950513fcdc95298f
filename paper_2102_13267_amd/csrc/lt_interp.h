// Register-resident bytecode interpreter (device side).
//
// A program is a list of three-address instructions over up to 32 value slots.  Each lane
// processes kVec = 4 elements, so a slot is four vector registers; the register file is four
// NS-wide vector values (one per element lane) that the compiler indexes with a wave-uniform slot
// number, which lowers to relative register addressing (s_set_gpr_idx + v_mov) -- no scratch
// memory, no LDS.  Three rules keep it that way (each found by reading the generated ISA):
//  * the register file is passed and returned BY VALUE: element-indexed access to a vector that
//    lives behind a reference is turned into memory accesses;
//  * slot indices are NOT masked: an index the optimiser can prove in range lets it rewrite
//    "load vector, extract element" as a scalar load from a stack copy.  The host validates
//    every program (slots < n_slots <= NS) before it is launched;
//  * a slot is written exactly once per instruction, after the opcode switch, and input slots
//    are written outside their "is this input present" branch: a write inside a branch makes
//    the compiler copy the whole register file where the branches join.
// The program itself is held in two vector registers per wavefront (lane j keeps instruction word
// j and scalar-table entry j); fetching an instruction or a scalar operand is one v_readlane with
// a wave-uniform lane number, so the interpreter loop touches no memory at all.
// Multi-instruction math (division, square root, transcendentals) is evaluated one element lane
// at a time behind scheduling barriers: interleaving four copies only inflates register
// pressure, and occupancy is what hides HBM latency here.
#ifndef LT_INTERP_H_
#define LT_INTERP_H_

#include <hip/hip_runtime.h>

#include "lt_kernels.h"

namespace ltk {

template <int NS> struct SlotVec;
template <> struct SlotVec<16> { typedef float type __attribute__((ext_vector_type(16))); };
template <> struct SlotVec<32> { typedef float type __attribute__((ext_vector_type(32))); };

// Register file of NS value slots (16 or 32) x kVec element lanes.
template <int NS> struct RF {
  typedef typename SlotVec<NS>::type vec;
  vec e[kVec];
};

struct Quad {
  float v[kVec];
};

__device__ __forceinline__ Quad splat(float s) {
  Quad q;
#pragma unroll
  for (int v = 0; v < kVec; ++v) q.v[v] = s;
  return q;
}

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
  const float cdf = 0.5f * (1.0f + erff(x * 0.70710678118654752f));
  const float pdf = 0.39894228040143268f * __expf(-0.5f * x * x);
  return dy * (cdf + x * pdf);
}

struct ProgRegs {
  uint32_t code;   // lane j: code[j]  (j < kMaxCode <= 64)
  float scal;      // lane j: scal[j]  (j < kMaxScal)
};

__device__ __forceinline__ ProgRegs load_prog_regs(const EwProg& p) {
  const uint32_t lane = threadIdx.x & 63u;
  ProgRegs r;
  r.code = lane < (uint32_t)kMaxCode ? p.code[lane] : 0u;
  r.scal = lane < (uint32_t)kMaxScal ? p.scal[lane] : 0.0f;
  return r;
}

__device__ __forceinline__ float scal_at(const ProgRegs& pr, uint32_t idx) {
  return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(pr.scal), (int)idx));
}

// cheap ops: all element lanes at once
#define LT_MAP(EXPR)                                                \
  _Pragma("unroll") for (int v = 0; v < kVec; ++v) {                \
    const float xa = A.v[v], xb = B.v[v];                           \
    (void)xb;                                                       \
    q.v[v] = (EXPR);                                                \
  }
// multi-instruction ops: one element lane at a time
#define LT_MAP_SERIAL(EXPR)                                         \
  _Pragma("unroll") for (int v = 0; v < kVec; ++v) {                \
    const float xa = A.v[v], xb = B.v[v];                           \
    (void)xb;                                                       \
    q.v[v] = (EXPR);                                                \
    __builtin_amdgcn_sched_barrier(0);                              \
  }

template <int NS>
__device__ __forceinline__ RF<NS> interp(RF<NS> f, const ProgRegs pr, const uint32_t n) {
  typename RF<NS>::vec r[kVec];
#pragma unroll
  for (int v = 0; v < kVec; ++v) r[v] = f.e[v];
  for (uint32_t pc = 0; pc < n; ++pc) {
    const uint32_t w = (uint32_t)__builtin_amdgcn_readlane((int)pr.code, (int)pc);
    const uint32_t op = w & 0xffu, d = (w >> 8) & 31u;
    const uint32_t ia = (w >> 13) & 63u, ib = (w >> 19) & 63u, ic = (w >> 25) & 63u;
    Quad A, B = splat(0.0f), q;
    // operand a is always a slot: the lowering puts a scalar operand second (using the
    // reversed form of non-commutative ops) or materialises it with kSplat first
#pragma unroll
    for (int v = 0; v < kVec; ++v) A.v[v] = r[v][ia];
    if (op >= kAdd) {   // binary and ternary ops: operand b is a slot or a scalar-table entry
      if (ib < 32u) {
#pragma unroll
        for (int v = 0; v < kVec; ++v) B.v[v] = r[v][ib];
      } else {
        B = splat(scal_at(pr, ib - 32u));
      }
    }
    q = A;
    switch (op) {
      case kMul: LT_MAP(xa * xb) break;
      case kAdd: LT_MAP(xa + xb) break;
      case kFma: {
        Quad C;
        if (ic < 32u) {
#pragma unroll
          for (int v = 0; v < kVec; ++v) C.v[v] = r[v][ic];
        } else {
          C = splat(scal_at(pr, ic - 32u));
        }
#pragma unroll
        for (int v = 0; v < kVec; ++v) q.v[v] = fmaf(A.v[v], B.v[v], C.v[v]);
      } break;
      case kSub: LT_MAP(xa - xb) break;
      case kRsub: LT_MAP(xb - xa) break;
      case kDiv: LT_MAP_SERIAL(xa / xb) break;
      case kRdiv: LT_MAP_SERIAL(xb / xa) break;
      case kMax: LT_MAP((xa != xa || xb != xb) ? (xa + xb) : fmaxf(xa, xb)) break;
      case kMin: LT_MAP((xa != xa || xb != xb) ? (xa + xb) : fminf(xa, xb)) break;
      case kReluGrad: LT_MAP(xb > 0.0f ? xa : 0.0f) break;
      case kRreluGrad: LT_MAP(xa > 0.0f ? xb : 0.0f) break;
      case kGeluGrad: LT_MAP_SERIAL(op_gelu_grad(xa, xb)) break;
      case kRgeluGrad: LT_MAP_SERIAL(op_gelu_grad(xb, xa)) break;
      case kMov: break;
      case kNeg: LT_MAP(-xa) break;
      case kAbs: LT_MAP(fabsf(xa)) break;
      case kSquare: LT_MAP(xa * xa) break;
      case kRelu: LT_MAP(xa > 0.0f ? xa : 0.0f) break;
      case kSqrt: LT_MAP_SERIAL(sqrtf(xa)) break;
      case kRsqrt: LT_MAP_SERIAL(rsqrtf(xa)) break;
      case kRecip: LT_MAP_SERIAL(1.0f / xa) break;
      case kExp: LT_MAP_SERIAL(expf(xa)) break;
      case kLog: LT_MAP_SERIAL(logf(xa)) break;
      case kTanh: LT_MAP_SERIAL(tanhf(xa)) break;
      case kGelu: LT_MAP_SERIAL(op_gelu(xa)) break;
      case kSigmoid: LT_MAP_SERIAL(1.0f / (1.0f + expf(-xa))) break;
      case kRoundBf16: LT_MAP(bf16_to_f32(f32_to_bf16(xa))) break;
      case kSplat: q = splat(scal_at(pr, ib - 32u)); break;
      default: break;
    }
#pragma unroll
    for (int v = 0; v < kVec; ++v) r[v][d] = q.v[v];
  }
  RF<NS> o;
#pragma unroll
  for (int v = 0; v < kVec; ++v) o.e[v] = r[v];
  return o;
}

// ---- loads -------------------------------------------------------------------------------

// F32: the host promises that every input and output of the program is fp32, which removes the
// dtype branches (and their registers) from the streaming kernels.
template <bool F32 = false>
__device__ __forceinline__ float load_elem(const void* ptr, uint32_t dtype, uint64_t idx) {
  if (!F32) {
    if (dtype == kBF16) return bf16_to_f32(((const uint16_t*)ptr)[idx]);
    if (dtype == kI32) return (float)((const int32_t*)ptr)[idx];
  }
  return ((const float*)ptr)[idx];
}

// Four consecutive elements starting at element `base + lane` of `ptr`.  `base` is wave-uniform
// and is folded into the (scalar) base address; only the 32-bit lane offset lives in a vector
// register, so all inputs of a program share one address register per lane.
template <bool F32 = false>
__device__ __forceinline__ Quad load_vec4(const void* ptr, uint32_t dtype, uint64_t base, uint32_t lane) {
  Quad q;
  if (!F32 && dtype == kBF16) {
    const char* b = (const char*)ptr + base * 2u;
    const uint2 u = *(const uint2*)(b + lane * 2u);
    q.v[0] = __uint_as_float(u.x << 16);
    q.v[1] = __uint_as_float(u.x & 0xffff0000u);
    q.v[2] = __uint_as_float(u.y << 16);
    q.v[3] = __uint_as_float(u.y & 0xffff0000u);
  } else {
    const char* b = (const char*)ptr + base * 4u;
    const float4 t = *(const float4*)(b + lane * 4u);
    q.v[0] = t.x; q.v[1] = t.y; q.v[2] = t.z; q.v[3] = t.w;
  }
  return q;
}

__device__ __forceinline__ uint64_t strided_index(const EwProg& p, const EwIn& in, uint64_t i) {
  uint32_t j = (uint32_t)i;
  const uint32_t c3 = j % p.dims[3]; j /= p.dims[3];
  const uint32_t c2 = j % p.dims[2]; j /= p.dims[2];
  const uint32_t c1 = j % p.dims[1]; j /= p.dims[1];
  return (uint64_t)((int64_t)j * in.stride[0] + (int64_t)c1 * in.stride[1] + (int64_t)c2 * in.stride[2] +
                    (int64_t)c3 * in.stride[3]);
}

// Flat element index -> element offset inside input `in` (general, one element at a time).
__device__ __forceinline__ uint64_t elem_offset(const EwProg& p, const EwIn& in, uint64_t i) {
  const uint32_t mode = in.mode;
  if (mode == kFull) return i;
  if (mode == kScalar) return 0;
  if (mode == kRowVec) return (uint32_t)i % p.cols;
  if (mode == kColVec) return (uint32_t)i / p.cols;
  return strided_index(p, in, i);
}

// General path: ragged tails, rows that are not a multiple of four, strided views.  Kept as a
// rolled loop: it is rare, and code size matters more than its speed (the instruction cache is
// shared by neighbouring compute units).
__device__ __forceinline__ Quad load_input_slow(const EwProg& p, const EwIn& in, uint64_t i, uint32_t nvalid) {
  Quad q = splat(0.0f);
#pragma unroll 1
  for (uint32_t e = 0; e < nvalid; ++e) {
    const float x = load_elem<false>(in.ptr, in.dtype, elem_offset(p, in, i + e));
#pragma unroll
    for (int v = 0; v < kVec; ++v) q.v[v] = e == (uint32_t)v ? x : q.v[v];
  }
  return q;
}

// Fetch the four consecutive elements i .. i+3 (i = base + lane, base wave-uniform) of the
// iteration space for one input.  FAST: the host promises full, aligned 4-vectors and no strided
// input, so the element-by-element path is not even compiled in.
template <bool FAST, bool F32>
__device__ __forceinline__ Quad load_input(const EwProg& p, const EwIn& in, uint64_t base, uint32_t lane, uint32_t i_div,
                                           uint32_t i_mod, uint32_t nvalid) {
  const uint32_t fetch = (FAST || nvalid == (uint32_t)kVec) ? in.fetch : (uint32_t)kFetchSlow;
  if (!FAST && fetch == kFetchSlow) return load_input_slow(p, in, base + lane, nvalid);
  const uint32_t mode = in.mode;
  if (fetch == kFetchVec4) {
    if (mode == kFull) return load_vec4<F32>(in.ptr, in.dtype, base, lane);
    return load_vec4<F32>(in.ptr, in.dtype, 0, i_mod);   // kRowVec
  }
  return splat(load_elem<F32>(in.ptr, in.dtype, mode == kColVec ? i_div : 0u));
}

// Put the inputs of the program into slots 0 .. n_in-1.  The loop over inputs is fully unrolled
// so that the slot index is a compile-time constant and every load is in flight before the first
// use.  MAXIN bounds the unrolling (and with it the registers reserved for loads in flight).
template <int NS, int MAXIN = kMaxIn, bool FAST = false, bool F32 = false>
__device__ __forceinline__ RF<NS> load_inputs(RF<NS> f, const EwProg& p, uint64_t base, uint32_t lane, uint32_t nvalid) {
  const uint32_t n_in = p.n_in;
  uint32_t i_div = 0, i_mod = 0;
  if (p.needs_divmod) {
    const uint32_t i = (uint32_t)base + lane;
    i_div = i / p.cols;
    i_mod = i - i_div * p.cols;
  }
#pragma unroll
  for (int k = 0; k < MAXIN; ++k) {
    Quad q = splat(0.0f);
    if ((uint32_t)k < n_in) q = load_input<FAST, F32>(p, p.in[k], base, lane, i_div, i_mod, nvalid);
#pragma unroll
    for (int v = 0; v < kVec; ++v) f.e[v][k] = q.v[v];
  }
  return f;
}

template <int NS>
__device__ __forceinline__ Quad rf_get(RF<NS> f, uint32_t slot) {
  Quad q;
#pragma unroll
  for (int v = 0; v < kVec; ++v) {
    typename RF<NS>::vec t = f.e[v];
    q.v[v] = t[slot];
  }
  return q;
}

template <int NS>
__device__ __forceinline__ RF<NS> rf_set(RF<NS> f, uint32_t slot, Quad q) {
#pragma unroll
  for (int v = 0; v < kVec; ++v) {
    typename RF<NS>::vec t = f.e[v];
    t[slot] = q.v[v];
    f.e[v] = t;
  }
  return f;
}

template <bool F32 = false>
__device__ __forceinline__ void store_elem(void* ptr, uint32_t dtype, uint64_t idx, float v) {
  if (!F32 && dtype == kBF16) ((uint16_t*)ptr)[idx] = f32_to_bf16(v);
  else ((float*)ptr)[idx] = v;
}

template <bool F32 = false>
__device__ __forceinline__ void store_vec4(void* ptr, uint32_t dtype, uint64_t base, uint32_t lane, const Quad& q) {
  if (!F32 && dtype == kBF16) {
    uint2 u;
    u.x = (uint32_t)f32_to_bf16(q.v[0]) | ((uint32_t)f32_to_bf16(q.v[1]) << 16);
    u.y = (uint32_t)f32_to_bf16(q.v[2]) | ((uint32_t)f32_to_bf16(q.v[3]) << 16);
    char* b = (char*)ptr + base * 2u;
    *(uint2*)(b + lane * 2u) = u;
  } else {
    char* b = (char*)ptr + base * 4u;
    *(float4*)(b + lane * 4u) = make_float4(q.v[0], q.v[1], q.v[2], q.v[3]);
  }
}

// Store the outputs of the program for elements i .. i+nvalid-1, i = base + lane (flat,
// contiguous outputs).
template <int NS, bool FAST = false, bool F32 = false>
__device__ __forceinline__ void store_outputs(RF<NS> f, const EwProg& p, uint64_t base, uint32_t lane, uint32_t nvalid) {
  const uint32_t n_out = p.n_out;
#pragma unroll
  for (int o = 0; o < kMaxOut; ++o) {
    if ((uint32_t)o < n_out) {
      const EwOut& out = p.out[o];
      const Quad q = rf_get<NS>(f, out.slot);
      if (out.scalar) {
        if (base + lane == 0) store_elem<F32>(out.ptr, out.dtype, 0, q.v[0]);
      } else if (FAST || (p.full_vec_ok && nvalid == (uint32_t)kVec)) {
        store_vec4<F32>(out.ptr, out.dtype, base, lane, q);
      } else {
#pragma unroll 1
        for (uint32_t e = 0; e < nvalid; ++e)
          store_elem<F32>(out.ptr, out.dtype, base + lane + e, e == 0 ? q.v[0] : e == 1 ? q.v[1] : e == 2 ? q.v[2] : q.v[3]);
      }
    }
  }
}

template <int NS>
__device__ __forceinline__ RF<NS> rf_zero() {
  RF<NS> f;
#pragma unroll
  for (int v = 0; v < kVec; ++v) f.e[v] = 0.0f;
  return f;
}

}  // namespace ltk
#endif  // LT_INTERP_H_
