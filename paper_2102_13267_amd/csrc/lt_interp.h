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

typedef float RawVec __attribute__((ext_vector_type(4)));   // one 128-bit register tuple

__device__ __forceinline__ Quad splat(float s) {
  Quad q;
#pragma unroll
  for (int v = 0; v < kVec; ++v) q.v[v] = s;
  return q;
}

__device__ __forceinline__ float bf16_to_f32(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// fp32 -> bf16, round to nearest even, NaN stays NaN: the hardware conversion (two values per
// instruction; eight instructions per value when spelled out in integer arithmetic).
typedef __bf16 Bf16x2 __attribute__((ext_vector_type(2)));
typedef float F32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t f32_to_bf16_pair(float lo, float hi) {
  const F32x2 v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, Bf16x2));
}
__device__ __forceinline__ uint16_t f32_to_bf16(float f) { return __builtin_bit_cast(uint16_t, (__bf16)f); }

// a / b in six instructions instead of the IEEE sequence's twelve: reciprocal estimate (1 ulp), one
// residual correction.  Correctly rounded except in rare half-way cases (then 1 ulp off); x / x is
// exactly 1; zeros, infinities and NaNs give what IEEE division gives (the correction is skipped
// when the residual is not finite).  It does not rescale: a divisor beyond 2^126 or a subnormal
// one, whose reciprocal leaves the normal range, loses accuracy.
__device__ __forceinline__ float fast_div(float a, float b) {
  const float r = __builtin_amdgcn_rcpf(b);
  const float q = a * r;
  const float e = fmaf(-b, q, a);
  return __builtin_isfinite(e) ? fmaf(e, r, q) : q;
}

// Standard normal CDF Phi(x) = (1 + erf(x / sqrt 2)) / 2 without branches: the five-term rational
// approximation of erf (Abramowitz & Stegun 7.1.26, |error| <= 1.5e-7 in exact arithmetic) on |x|
// and the reflection Phi(-x) = 1 - Phi(x).  The library erff is exact to an ulp but takes two
// divergent polynomial paths, which is most of what a GELU epilogue costs.
__device__ __forceinline__ float normal_cdf(float x) {
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float tail = 0.5f * poly * t * __expf(-z * z);   // (1 - erf(z)) / 2
  return x >= 0.0f ? 1.0f - tail : tail;
}

__device__ __forceinline__ float op_gelu(float x) { return x * normal_cdf(x); }
// d/dx [x Phi(x)] = Phi(x) + x phi(x).  exp(-x^2 / 2) serves both the density and the tail of the
// distribution function (the exponential is a quarter-rate instruction, and half of what this
// costs).
__device__ __forceinline__ float op_gelu_grad(float dy, float x) {
  const float e = __expf(-0.5f * x * x);
  const float z = fabsf(x) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
  float poly = fmaf(1.061405429f, t, -1.453152027f);
  poly = fmaf(poly, t, 1.421413741f);
  poly = fmaf(poly, t, -0.284496736f);
  poly = fmaf(poly, t, 0.254829592f);
  const float tail = 0.5f * poly * t * e;
  const float cdf = x >= 0.0f ? 1.0f - tail : tail;
  return dy * fmaf(x, 0.39894228040143268f * e, cdf);
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
  _Pragma("unroll") for (int v = 0; v < kVec * Q; ++v) {            \
    const float xa = A[v], xb = B[v];                               \
    (void)xb;                                                       \
    q[v] = (EXPR);                                                  \
  }
// multi-instruction ops: one element lane at a time
#define LT_MAP_SERIAL(EXPR)                                         \
  _Pragma("unroll") for (int v = 0; v < kVec * Q; ++v) {            \
    const float xa = A[v], xb = B[v];                               \
    (void)xb;                                                       \
    q[v] = (EXPR);                                                  \
    __builtin_amdgcn_sched_barrier(0);                              \
  }

// Q = 1: the register file holds NS slots of one 4-vector.  Q = 2: it holds NS/2 slots of TWO
// 4-vectors (slot s of 4-vector j is element s + j * NS/2 of each register-file vector), and every
// instruction is fetched, decoded and dispatched once for both.  Fetch, decode and the opcode
// tree are scalar instructions and branches -- two thirds of what an interpreted instruction
// costs -- so this halves most of the interpreter's overhead per element with the same registers.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wuninitialized"
#pragma clang diagnostic ignored "-Wsometimes-uninitialized"
#pragma clang diagnostic ignored "-Wconditional-uninitialized"
template <int NS, int Q = 1>
__device__ __forceinline__ RF<NS> interp(RF<NS> f, const ProgRegs pr, const uint32_t n) {
  constexpr uint32_t SL = NS / Q;   // slots per 4-vector
  typename RF<NS>::vec r[kVec];
#pragma unroll
  for (int v = 0; v < kVec; ++v) r[v] = f.e[v];
  for (uint32_t pc = 0; pc < n; ++pc) {
    const uint32_t w = (uint32_t)__builtin_amdgcn_readlane((int)pr.code, (int)pc);
    const uint32_t op = w & 0xffu, d = (w >> 8) & 31u;
    const uint32_t ia = (w >> 13) & 63u, ib = (w >> 19) & 63u, ic = (w >> 25) & 63u;
    float A[kVec * Q], B[kVec * Q], q[kVec * Q];   // B stays undefined for unary ops, which never read it
    // operand a is always a slot: the lowering puts a scalar operand second (using the
    // reversed form of non-commutative ops) or materialises it with kSplat first
#pragma unroll
    for (int j = 0; j < Q; ++j)
#pragma unroll
      for (int v = 0; v < kVec; ++v) A[j * kVec + v] = r[v][ia + j * SL];
    if (op >= kAdd) {   // binary and ternary ops: operand b is a slot or a scalar-table entry
      if (ib < 32u) {
#pragma unroll
        for (int j = 0; j < Q; ++j)
#pragma unroll
          for (int v = 0; v < kVec; ++v) B[j * kVec + v] = r[v][ib + j * SL];
      } else {
        const float sb = scal_at(pr, ib - 32u);
#pragma unroll
        for (int v = 0; v < kVec * Q; ++v) B[v] = sb;
      }
    }
#pragma unroll
    for (int v = 0; v < kVec * Q; ++v) q[v] = A[v];
    switch (op) {
      case kMul: LT_MAP(xa * xb) break;
      case kAdd: LT_MAP(xa + xb) break;
      case kFma: {
        float C[kVec * Q];
        if (ic < 32u) {
#pragma unroll
          for (int j = 0; j < Q; ++j)
#pragma unroll
            for (int v = 0; v < kVec; ++v) C[j * kVec + v] = r[v][ic + j * SL];
        } else {
          const float sc = scal_at(pr, ic - 32u);
#pragma unroll
          for (int v = 0; v < kVec * Q; ++v) C[v] = sc;
        }
#pragma unroll
        for (int v = 0; v < kVec * Q; ++v) q[v] = fmaf(A[v], B[v], C[v]);
      } break;
      case kSub: LT_MAP(xa - xb) break;
      case kRsub: LT_MAP(xb - xa) break;
      case kDiv: LT_MAP(fast_div(xa, xb)) break;
      case kRdiv: LT_MAP(fast_div(xb, xa)) break;
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
      case kSqrt: LT_MAP(__builtin_amdgcn_sqrtf(xa)) break;   // hardware square root, 1 ulp
      case kRsqrt: LT_MAP(__builtin_amdgcn_rsqf(xa)) break;    // 1 ulp
      case kRecip: LT_MAP(__builtin_amdgcn_rcpf(xa)) break;    // 1 ulp
      case kExp: LT_MAP_SERIAL(expf(xa)) break;
      case kLog: LT_MAP_SERIAL(logf(xa)) break;
      case kTanh: LT_MAP_SERIAL(tanhf(xa)) break;
      case kGelu: LT_MAP_SERIAL(op_gelu(xa)) break;
      case kSigmoid: LT_MAP_SERIAL(fast_div(1.0f, 1.0f + expf(-xa))) break;
      case kRoundBf16: LT_MAP(bf16_to_f32(f32_to_bf16(xa))) break;
      case kSplat: {
        const float sb = scal_at(pr, ib - 32u);
#pragma unroll
        for (int v = 0; v < kVec * Q; ++v) q[v] = sb;
      } break;
      default: break;
    }
#pragma unroll
    for (int j = 0; j < Q; ++j)
#pragma unroll
      for (int v = 0; v < kVec; ++v) r[v][d + j * SL] = q[j * kVec + v];
  }
  RF<NS> o;
#pragma unroll
  for (int v = 0; v < kVec; ++v) o.e[v] = r[v];
  return o;
}
#pragma clang diagnostic pop

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

// Loads are split in two so that every load of a 4-vector's inputs is issued before any result
// is touched: fetch_* returns the RAW bits (a conversion right behind a load would make the
// compiler wait for it -- and for every other load in flight), finish_* converts them later.
//
// Raw fetch of four consecutive elements starting at element `base + lane` of `ptr`.  `base` is
// wave-uniform and folded into the scalar base address; only the lane offset is per lane.
template <bool F32 = false>
__device__ __forceinline__ RawVec fetch_vec4(const void* ptr, uint32_t dtype, uint64_t base, uint32_t lane) {
  RawVec q;
  if (!F32 && dtype == kBF16) {
    const char* b = (const char*)ptr + base * 2u;
    const uint2 u = *(const uint2*)(b + (size_t)lane * 2u);
    q.x = __uint_as_float(u.x);
    q.y = __uint_as_float(u.y);
    q.z = q.w = 0.0f;
  } else {
    const char* b = (const char*)ptr + base * 4u;
    q = *(const RawVec*)(b + (size_t)lane * 4u);
  }
  return q;
}

template <bool F32 = false>
__device__ __forceinline__ float fetch_elem(const void* ptr, uint32_t dtype, uint64_t idx) {
  if (!F32 && dtype == kBF16) return __uint_as_float((uint32_t)((const uint16_t*)ptr)[idx]);
  return ((const float*)ptr)[idx];   // fp32 and int32 are both one dword
}

template <bool F32 = false>
__device__ __forceinline__ Quad finish_vec4(uint32_t dtype, const RawVec raw) {
  Quad q;
  if (F32 || dtype != kBF16) {
    q.v[0] = raw.x; q.v[1] = raw.y; q.v[2] = raw.z; q.v[3] = raw.w;
    return q;
  }
  const uint32_t x = __float_as_uint(raw.x), y = __float_as_uint(raw.y);
  q.v[0] = __uint_as_float(x << 16);
  q.v[1] = __uint_as_float(x & 0xffff0000u);
  q.v[2] = __uint_as_float(y << 16);
  q.v[3] = __uint_as_float(y & 0xffff0000u);
  return q;
}

template <bool F32 = false>
__device__ __forceinline__ float finish_elem(uint32_t dtype, float raw) {
  if (F32 || dtype == kF32) return raw;
  if (dtype == kBF16) return __uint_as_float(__float_as_uint(raw) << 16);
  return (float)(int32_t)__float_as_uint(raw);   // kI32
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

// General path: ragged tails, rows that are not a multiple of four, strided views.
__device__ __forceinline__ Quad load_input_slow(const EwProg& p, const EwIn& in, uint64_t i, uint32_t nvalid) {
  // the (up to four) element loads are issued together: one after the other they would cost a
  // memory round trip each
  // (elements past nvalid re-read the last valid one, so that no load sits behind a branch)
  Quad q;
#pragma unroll
  for (int e = 0; e < kVec; ++e) {
    const uint32_t ee = (uint32_t)e < nvalid ? (uint32_t)e : nvalid - 1u;   // nvalid >= 1
    const float x = load_elem<false>(in.ptr, in.dtype, elem_offset(p, in, i + ee));
    q.v[e] = (uint32_t)e < nvalid ? x : 0.0f;
  }
  return q;
}

// The inputs of one 4-vector, as fetched (MAXIN bounds the unrolling and with it the registers
// reserved for loads in flight).  Vector loads and broadcast loads land in SEPARATE registers:
// merging the two kinds into one variable makes the compiler move loaded data right behind the
// load, and that move waits for the load (and every other load in flight).
template <int MAXIN> struct Staged {
  RawVec vec[MAXIN];   // kFetchVec4 (raw bits) or the slow path (converted values)
  float bc[MAXIN];     // kFetchBcast (raw bits)
};

// Issue the loads of every input for the 4-vector at base + lane (base wave-uniform).  Fully
// unrolled so that all loads are in flight together.  FAST: the host promises full, aligned
// 4-vectors and no strided input, so the element-by-element path is not even compiled in.
// Every use of fetched values is made to depend on this point.  Placed behind the last load it
// keeps the compiler from sinking each input's "move into the slot" into that input's own
// branch, right behind its load, which would wait for every load before issuing the next.
template <int MAXIN>
__device__ __forceinline__ void pin_staged(Staged<MAXIN>& st) {
#pragma unroll
  for (int k = 0; k < MAXIN; ++k) asm volatile("" : "+v"(st.vec[k]), "+v"(st.bc[k]));
}

template <int MAXIN, bool FAST, bool F32, bool PIN = true>
__device__ __forceinline__ Staged<MAXIN> fetch_inputs(const EwProg& p, uint64_t base, uint32_t lane, uint32_t nvalid) {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wuninitialized"
#pragma clang diagnostic ignored "-Wsometimes-uninitialized"
  Staged<MAXIN> st;
  const uint32_t n_in = p.n_in;
  uint32_t i_div = 0, i_mod = 0;
  if (p.needs_divmod) {
    const uint32_t i = (uint32_t)base + lane;
    i_div = i / p.cols;
    i_mod = i - i_div * p.cols;
  }
#pragma unroll
  for (int k = 0; k < MAXIN; ++k) {
    // (deliberately not zero-initialised: a "= 0" that the other branch overwrites with a load
    // becomes a register write that must wait for that load)
    if ((uint32_t)k < n_in) {
      const EwIn& in = p.in[k];
      const uint32_t fetch = (FAST || nvalid == (uint32_t)kVec) ? in.fetch : (uint32_t)kFetchSlow;
      const uint32_t mode = in.mode;
      if (!FAST && fetch == kFetchSlow) {
        const Quad t = load_input_slow(p, in, base + lane, nvalid);
        st.vec[k].x = t.v[0]; st.vec[k].y = t.v[1]; st.vec[k].z = t.v[2]; st.vec[k].w = t.v[3];
      } else if (fetch == kFetchVec4) {
        if (mode == kFull) st.vec[k] = fetch_vec4<F32>(in.ptr, in.dtype, base, lane);
        else st.vec[k] = fetch_vec4<F32>(in.ptr, in.dtype, 0, i_mod);   // kRowVec
      } else {
        st.bc[k] = fetch_elem<F32>(in.ptr, in.dtype, mode == kColVec ? i_div : 0u);
      }
    }
  }
  if (PIN) pin_staged<MAXIN>(st);
  return st;
#pragma clang diagnostic pop
}

// The same for a caller that already knows the row (i_div) and column (i_mod) of flat element i
// and promises whole, aligned 4-vectors and no strided input (no division, no slow path).
// PIN = false leaves the loads in flight (the caller pins the result where it wants to wait).
template <int MAXIN, bool F32, bool PIN = true>
__device__ __forceinline__ Staged<MAXIN> fetch_inputs_at(const EwProg& p, uint32_t i, uint32_t i_div, uint32_t i_mod) {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wuninitialized"
#pragma clang diagnostic ignored "-Wsometimes-uninitialized"
  Staged<MAXIN> st;
  const uint32_t n_in = p.n_in;
#pragma unroll
  for (int k = 0; k < MAXIN; ++k) {
    if ((uint32_t)k < n_in) {
      const EwIn& in = p.in[k];
      if (in.fetch == kFetchVec4) st.vec[k] = fetch_vec4<F32>(in.ptr, in.dtype, 0, in.mode == kFull ? i : i_mod);
      else st.bc[k] = fetch_elem<F32>(in.ptr, in.dtype, in.mode == kColVec ? i_div : 0u);
    }
  }
  if (PIN) pin_staged<MAXIN>(st);
  return st;
#pragma clang diagnostic pop
}

// Convert the fetched inputs and move them into slots 0 .. MAXIN-1 (compile-time slot numbers:
// plain register moves).
// OFF: first slot (NS/2 for the second 4-vector of a two-wide register file).
template <int NS, int MAXIN, bool FAST, bool F32, int OFF = 0>
__device__ __forceinline__ RF<NS> place_inputs(RF<NS> f, const EwProg& p, const Staged<MAXIN>& st, uint32_t nvalid) {
  const uint32_t n_in = p.n_in;
#pragma unroll
  for (int k = 0; k < MAXIN; ++k) {
    Quad q;
    q.v[0] = st.vec[k].x; q.v[1] = st.vec[k].y; q.v[2] = st.vec[k].z; q.v[3] = st.vec[k].w;
    if ((uint32_t)k < n_in) {
      const EwIn& in = p.in[k];
      const uint32_t fetch = (FAST || nvalid == (uint32_t)kVec) ? in.fetch : (uint32_t)kFetchSlow;
      if (fetch == kFetchVec4) q = finish_vec4<F32>(in.dtype, st.vec[k]);
      else if (fetch == kFetchBcast) q = splat(finish_elem<F32>(in.dtype, st.bc[k]));
    }
#pragma unroll
    for (int v = 0; v < kVec; ++v) f.e[v][k + OFF] = q.v[v];
  }
  return f;
}

template <int NS>
__device__ __forceinline__ RF<NS> rf_set(RF<NS> f, uint32_t slot, Quad q);

// The general path (ragged tails, rows that are not a multiple of four, strided views, small
// problems) as ONE rolled loop over the inputs: a kernel that runs it at all runs it a few times,
// so what it costs is the instructions it drags through the instruction cache, not its latency.
template <int NS>
__device__ __forceinline__ RF<NS> load_inputs_general(RF<NS> f, const EwProg& p, uint64_t base, uint32_t lane, uint32_t nvalid) {
  const uint32_t n_in = p.n_in;
  uint32_t i_div = 0, i_mod = 0;
  if (p.needs_divmod) {
    const uint32_t i = (uint32_t)base + lane;
    i_div = i / p.cols;
    i_mod = i - i_div * p.cols;
  }
#pragma unroll 1
  for (uint32_t k = 0; k < n_in; ++k) {
    const EwIn& in = p.in[k];
    const uint32_t fetch = nvalid == (uint32_t)kVec ? in.fetch : (uint32_t)kFetchSlow;
    const uint32_t mode = in.mode;
    Quad q;
    if (fetch == kFetchSlow) q = load_input_slow(p, in, base + lane, nvalid);
    else if (fetch == kFetchVec4)
      q = finish_vec4<false>(in.dtype, mode == kFull ? fetch_vec4<false>(in.ptr, in.dtype, base, lane)
                                                      : fetch_vec4<false>(in.ptr, in.dtype, 0, i_mod));
    else q = splat(finish_elem<false>(in.dtype, fetch_elem<false>(in.ptr, in.dtype, mode == kColVec ? i_div : 0u)));
    f = rf_set<NS>(f, k, q);
  }
  return f;
}

template <int NS, int MAXIN = kMaxIn, bool FAST = false, bool F32 = false>
__device__ __forceinline__ RF<NS> load_inputs(RF<NS> f, const EwProg& p, uint64_t base, uint32_t lane, uint32_t nvalid) {
  if (!FAST) return load_inputs_general<NS>(f, p, base, lane, nvalid);
  return place_inputs<NS, MAXIN, FAST, F32>(f, p, fetch_inputs<MAXIN, FAST, F32>(p, base, lane, nvalid), nvalid);
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

// NT: non-temporal store (the data is not read again by this kernel).
template <bool F32 = false, bool NT = false>
__device__ __forceinline__ void store_vec4(void* ptr, uint32_t dtype, uint64_t base, uint32_t lane, const Quad& q) {
  if (!F32 && dtype == kBF16) {
    uint2 u;
    u.x = f32_to_bf16_pair(q.v[0], q.v[1]);
    u.y = f32_to_bf16_pair(q.v[2], q.v[3]);
    char* b = (char*)ptr + base * 2u;
    *(uint2*)(b + (size_t)lane * 2u) = u;
  } else {
    char* b = (char*)ptr + base * 4u;
    if (NT) {
      const RawVec t = {q.v[0], q.v[1], q.v[2], q.v[3]};
      __builtin_nontemporal_store(t, (RawVec*)(b + (size_t)lane * 4u));
    } else {
      *(float4*)(b + (size_t)lane * 4u) = make_float4(q.v[0], q.v[1], q.v[2], q.v[3]);
    }
  }
}

// Store the outputs of the program for elements i .. i+nvalid-1, i = base + lane (flat,
// contiguous outputs).
template <int NS, bool FAST = false, bool F32 = false, int OFF = 0, bool NT = false>
__device__ __forceinline__ void store_outputs(RF<NS> f, const EwProg& p, uint64_t base, uint32_t lane, uint32_t nvalid) {
  const uint32_t n_out = p.n_out;
  if (!FAST) {   // general path: one rolled copy (see load_inputs_general)
#pragma unroll 1
    for (uint32_t o = 0; o < n_out; ++o) {
      const EwOut& out = p.out[o];
      const Quad q = rf_get<NS>(f, out.slot + (uint32_t)OFF);
      if (out.scalar) {
        if (base + lane == 0) store_elem<false>(out.ptr, out.dtype, 0, q.v[0]);
      } else if (p.full_vec_ok && nvalid == (uint32_t)kVec) {
        store_vec4<false>(out.ptr, out.dtype, base, lane, q);
      } else {
#pragma unroll 1
        for (uint32_t e = 0; e < nvalid; ++e)
          store_elem<false>(out.ptr, out.dtype, base + lane + e, e == 0 ? q.v[0] : e == 1 ? q.v[1] : e == 2 ? q.v[2] : q.v[3]);
      }
    }
    return;
  }
#pragma unroll
  for (int o = 0; o < kMaxOut; ++o) {
    if ((uint32_t)o < n_out) {
      const EwOut& out = p.out[o];
      const Quad q = rf_get<NS>(f, out.slot + (uint32_t)OFF);
      if (out.scalar) {
        if (base + lane == 0) store_elem<F32>(out.ptr, out.dtype, 0, q.v[0]);
      } else {
        store_vec4<F32, NT>(out.ptr, out.dtype, base, lane, q);
      }
    }
  }
}

// ---- streaming stage for reductions ---------------------------------------------------------
// A reduction has few inputs, so memory-level parallelism must come from fetching U 4-vectors per
// lane before any is used.  Unrolling the interpreter U times would multiply its code (and miss
// the instruction cache), so the U raw vectors of an input are kept in ONE wide register tuple
// and the interpreter runs in a rolled loop that picks vector u with a wave-uniform index
// (relative register addressing again).  Only for programs whose NIN inputs are all read in
// full, 4 elements at a time, and share one element type (BF: bf16, else fp32).
template <int N> struct WideVec { typedef float type __attribute__((ext_vector_type(N))); };

template <int NIN, int U, bool BF> struct Stream {
  typedef typename WideVec<(BF ? 2 : 4) * U>::type vec;
  vec s[NIN];
};

// fetch vector number u (a compile-time constant after unrolling) of every input
template <int NIN, int U, bool BF>
__device__ __forceinline__ void stream_fetch(Stream<NIN, U, BF>& st, const int u, const EwProg& p, uint64_t base, uint32_t lane) {
#pragma unroll
  for (int k = 0; k < NIN; ++k) {
    if (BF) {
      typedef uint32_t U32x2 __attribute__((ext_vector_type(2)));
      const U32x2 t = __builtin_nontemporal_load((const U32x2*)((const char*)p.in[k].ptr + base * 2u + (size_t)lane * 2u));
      st.s[k][2 * u] = __uint_as_float(t.x);
      st.s[k][2 * u + 1] = __uint_as_float(t.y);
    } else {
      const RawVec t = __builtin_nontemporal_load((const RawVec*)((const char*)p.in[k].ptr + base * 4u + (size_t)lane * 4u));
      st.s[k][4 * u] = t.x; st.s[k][4 * u + 1] = t.y; st.s[k][4 * u + 2] = t.z; st.s[k][4 * u + 3] = t.w;
    }
  }
}

// vector u (compile-time) of input k, converted
template <int NIN, int U, bool BF>
__device__ __forceinline__ Quad stream_quad(const Stream<NIN, U, BF>& st, const int k, const int u) {
  Quad q;
  if (BF) {
    const uint32_t x = __float_as_uint(st.s[k][2 * u]), y = __float_as_uint(st.s[k][2 * u + 1]);
    q.v[0] = __uint_as_float(x << 16);
    q.v[1] = __uint_as_float(x & 0xffff0000u);
    q.v[2] = __uint_as_float(y << 16);
    q.v[3] = __uint_as_float(y & 0xffff0000u);
  } else {
    q.v[0] = st.s[k][4 * u]; q.v[1] = st.s[k][4 * u + 1]; q.v[2] = st.s[k][4 * u + 2]; q.v[3] = st.s[k][4 * u + 3];
  }
  return q;
}

// move vector u (run-time, wave-uniform) of every input into slots 0 .. NIN-1
template <int NS, int NIN, int U, bool BF, int OFF = 0>
__device__ __forceinline__ RF<NS> stream_place(RF<NS> f, const Stream<NIN, U, BF> st, const uint32_t u) {
#pragma unroll
  for (int k = 0; k < NIN; ++k) {
    const typename Stream<NIN, U, BF>::vec t = st.s[k];
    Quad q;
    if (BF) {
      const uint32_t x = __float_as_uint(t[2 * u]), y = __float_as_uint(t[2 * u + 1]);
      q.v[0] = __uint_as_float(x << 16);
      q.v[1] = __uint_as_float(x & 0xffff0000u);
      q.v[2] = __uint_as_float(y << 16);
      q.v[3] = __uint_as_float(y & 0xffff0000u);
    } else {
      q.v[0] = t[4 * u]; q.v[1] = t[4 * u + 1]; q.v[2] = t[4 * u + 2]; q.v[3] = t[4 * u + 3];
    }
#pragma unroll
    for (int v = 0; v < kVec; ++v) f.e[v][k + OFF] = q.v[v];
  }
  return f;
}

// Host side: can this program be streamed, and with which element type?  0 = no, 1 = fp32, 2 = bf16.
inline int stream_kind(const EwProg& p) {
  if (!p.fast || p.n_in == 0u) return 0;
  for (uint32_t k = 0; k < p.n_in; ++k)
    if (p.in[k].mode != kFull || p.in[k].fetch != kFetchVec4 || p.in[k].dtype != p.in[0].dtype) return 0;
  return p.in[0].dtype == kF32 ? 1 : p.in[0].dtype == kBF16 ? 2 : 0;
}

// A fresh register file.  Its contents are deliberately left undefined: a valid program writes
// every slot before reading it (the host checks), and clearing NS x 4 registers per 4-vector is
// a measurable share of a short program's instructions.
template <int NS>
__device__ __forceinline__ RF<NS> rf_zero() {
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wuninitialized"
  RF<NS> f;
  return f;
#pragma clang diagnostic pop
}

}  // namespace ltk
#endif  // LT_INTERP_H_
