// Pieces shared by the contraction kernels: vector types and the interpreted epilogue.
#ifndef LT_GEMM_EPILOGUE_H_
#define LT_GEMM_EPILOGUE_H_
#include <hip/hip_runtime.h>

#include "lt_interp.h"

namespace ltk {

constexpr int kGemmThreads = 256;
constexpr int kCPad = 4;

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// ---- streamed post program -------------------------------------------------------------------
// Post programs whose inputs are all whole 4-vectors of one element type, addressed like the
// output (a residual) or by column (a bias).  What an interpreted epilogue costs is mostly fetch,
// decode and dispatch of the instruction -- scalar work, the same for one quad or many -- and it
// sits on the critical path: the workgroups of a launch reach their epilogues together, so nothing
// runs under it.  So a lane's quads go through the interpreter Q at a time (Q = 8: a register
// file of 4 slots x 8 quads, one or two trips per lane; Q = 4: 8 slots x 4 quads).  The inputs of
// the Q quads are fetched straight into the register file -- one memory round trip per trip, with
// nothing in the fetch that depends on the program.  A program with one input fetches it twice (no
// branch in the fetch); the copy lands in a slot that the program writes before it reads.
template <int BM, int BN, int Q>
__device__ __forceinline__ void post_wide(const GemmArgs& a, const ProgRegs pr, const float* Cs, uint32_t tile_m, uint32_t tile_n,
                                          int64_t base, const bool bf) {
  constexpr int NS = 32, SL = NS / Q;
  constexpr int kCStride = BN + kCPad;
  constexpr uint32_t kQuadsPerRow = BN / kVec, kRowStep = (uint32_t)kGemmThreads / kQuadsPerRow;
  constexpr uint32_t kTrips = (uint32_t)(BM * BN / kVec) / kGemmThreads;   // quads per lane
  static_assert(kTrips % (uint32_t)Q == 0u, "a lane's quads make whole trips");
  const EwProg& p = a.post;
  const uint32_t n_code = p.n_code;
  const uint32_t r0 = threadIdx.x / kQuadsPerRow, c = (threadIdx.x % kQuadsPerRow) * kVec;
  const uint32_t k1 = p.n_in > 1u ? 1u : 0u;
  const char* ptr0 = (const char*)p.in[0].ptr;
  const char* ptr1 = (const char*)p.in[k1].ptr;
  const bool full0 = p.in[0].mode == kFull, full1 = p.in[k1].mode == kFull;
  const uint32_t col = tile_n + c;
#pragma unroll 1
  for (uint32_t pass = 0; pass < kTrips / (uint32_t)Q; ++pass) {
    uint32_t idx[Q];   // flat output index of quad j of this trip
#pragma unroll
    for (int j = 0; j < Q; ++j) {
      const uint32_t r = r0 + (pass * (uint32_t)Q + (uint32_t)j) * kRowStep;
      idx[j] = (uint32_t)(base + (int64_t)(tile_m + r) * a.o_row + col);
    }
    RF<NS> f = rf_zero<NS>();
    if (bf) {
      typedef uint32_t U32x2 __attribute__((ext_vector_type(2)));
      U32x2 t0[Q], t1[Q];
#pragma unroll
      for (int j = 0; j < Q; ++j) {
        t0[j] = *(const U32x2*)(ptr0 + (size_t)(full0 ? idx[j] : col) * 2u);
        t1[j] = *(const U32x2*)(ptr1 + (size_t)(full1 ? idx[j] : col) * 2u);
      }
#pragma unroll
      for (int j = 0; j < Q; ++j) {
        f.e[0][j * SL] = __uint_as_float(t0[j].x << 16);
        f.e[1][j * SL] = __uint_as_float(t0[j].x & 0xffff0000u);
        f.e[2][j * SL] = __uint_as_float(t0[j].y << 16);
        f.e[3][j * SL] = __uint_as_float(t0[j].y & 0xffff0000u);
        f.e[0][j * SL + 1] = __uint_as_float(t1[j].x << 16);
        f.e[1][j * SL + 1] = __uint_as_float(t1[j].x & 0xffff0000u);
        f.e[2][j * SL + 1] = __uint_as_float(t1[j].y << 16);
        f.e[3][j * SL + 1] = __uint_as_float(t1[j].y & 0xffff0000u);
      }
    } else {
      RawVec t0[Q], t1[Q];
#pragma unroll
      for (int j = 0; j < Q; ++j) {
        t0[j] = *(const RawVec*)(ptr0 + (size_t)(full0 ? idx[j] : col) * 4u);
        t1[j] = *(const RawVec*)(ptr1 + (size_t)(full1 ? idx[j] : col) * 4u);
      }
#pragma unroll
      for (int j = 0; j < Q; ++j) {
        f.e[0][j * SL] = t0[j].x; f.e[1][j * SL] = t0[j].y; f.e[2][j * SL] = t0[j].z; f.e[3][j * SL] = t0[j].w;
        f.e[0][j * SL + 1] = t1[j].x; f.e[1][j * SL + 1] = t1[j].y; f.e[2][j * SL + 1] = t1[j].z; f.e[3][j * SL + 1] = t1[j].w;
      }
    }
#pragma unroll
    for (int j = 0; j < Q; ++j) {
      const uint32_t r = r0 + (pass * (uint32_t)Q + (uint32_t)j) * kRowStep;
      const float4 t = *(const float4*)&Cs[r * kCStride + c];
      Quad anchor;
      anchor.v[0] = t.x; anchor.v[1] = t.y; anchor.v[2] = t.z; anchor.v[3] = t.w;
      f = rf_set<NS>(f, p.anchor_slot + (uint32_t)(j * SL), anchor);
    }
    f = interp<NS, Q>(f, pr, n_code);
#pragma unroll
    for (int o = 0; o < kMaxOut; ++o) {
      if ((uint32_t)o < p.n_out) {
        const EwOut& out = p.out[o];
#pragma unroll
        for (int j = 0; j < Q; ++j) store_vec4<false>(out.ptr, out.dtype, 0, idx[j], rf_get<NS>(f, out.slot + (uint32_t)(j * SL)));
      }
    }
  }
}

// Host-independent test (wave-uniform): can the post program be streamed, and as which element
// type?  0 = no, 1 = fp32, 2 = bf16.
__device__ __forceinline__ int post_stream_kind(const EwProg& p) {
  if (p.n_in == 0u || p.n_in > 2u) return 0;
  const uint32_t dt = p.in[0].dtype;
  for (uint32_t k = 0; k < p.n_in; ++k) {
    const EwIn& in = p.in[k];
    if (in.fetch != kFetchVec4 || (in.mode != kFull && in.mode != kRowVec) || in.dtype != dt) return 0;
  }
  return dt == kF32 ? 1 : dt == kBF16 ? 2 : 0;
}

// ---- epilogue ------------------------------------------------------------------------------
// The accumulators leave the MFMA layout (a lane owns 4-row column segments) through LDS: the
// tile is written once, then every lane walks it in row-major 4-element quads, so the post
// program sees flat, contiguous indices exactly like the elementwise kernel does (16-byte loads
// of residuals, 16-byte stores) and is compiled in only once.
template <int BM, int BN, int MB, int NB>
__device__ __forceinline__ void epilogue(const GemmArgs& a, const v16f (&acc)[MB][NB], float* Cs, uint32_t tile_m,
                                         uint32_t tile_n, uint32_t wave_m, uint32_t wave_n, uint32_t lane, uint32_t batch,
                                         float* raw = nullptr) {
  constexpr int kCStride = BN + kCPad;
  __syncthreads();   // the operand tiles in the same LDS bytes are dead now
#pragma unroll
  for (int bm = 0; bm < MB; ++bm)
#pragma unroll
    for (int bn = 0; bn < NB; ++bn)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = wave_m * (MB * 32) + bm * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const uint32_t col = wave_n * (NB * 32) + bn * 32 + (lane & 31);
        Cs[row * kCStride + col] = acc[bm][bn][r];
      }
  __syncthreads();
  const EwProg& p = a.post;
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t b0 = batch / a.batch1, b1 = batch % a.batch1;
  const int64_t base = (int64_t)b0 * a.o_b0 + (int64_t)b1 * a.o_b1;
  if (raw) {
    // partial product of a k split: plain fp32, dense [batch * m, n]; the post program runs in a
    // second launch over the sum of the splits
    const uint32_t row_flat0 = (b0 * a.batch1 + b1) * a.m;
    const bool vec = (a.n % 4u) == 0u;
    for (uint32_t q = threadIdx.x; q < (uint32_t)(BM * BN / kVec); q += kGemmThreads) {
      const uint32_t r = q / (BN / kVec), c = (q % (BN / kVec)) * kVec;
      const uint32_t row = tile_m + r, col = tile_n + c;
      if (row >= a.m || col >= a.n) continue;
      float* dst = raw + (size_t)(row_flat0 + row) * a.n + col;
      const float4 t = *(const float4*)&Cs[r * kCStride + c];
      if (vec) {
        *(float4*)dst = t;
      } else {
        dst[0] = t.x;
        if (col + 1 < a.n) dst[1] = t.y;
        if (col + 2 < a.n) dst[2] = t.z;
        if (col + 3 < a.n) dst[3] = t.w;
      }
    }
    return;
  }
  // Whole tile, whole aligned 4-vectors, at most four inputs (none of them strided) and eight
  // slots: no bounds checks, no divisions (row and column are known).
  const bool fast = p.fast && p.full_vec_ok && p.n_in <= 4u && p.n_slots <= 8u && tile_m + BM <= a.m && tile_n + BN <= a.n;
  const uint32_t row_flat0 = (b0 * a.batch1 + b1) * a.m + tile_m;   // row number in the flattened [rows, n] output
  if (fast && n_code == 0u && p.n_in == 0u && p.n_out == 1u && !p.out[0].scalar && p.out[0].slot == p.anchor_slot) {
    // the product itself is the only output: convert and store, nothing to interpret
    const EwOut& o = p.out[0];
#pragma unroll 4
    for (uint32_t q = threadIdx.x; q < (uint32_t)(BM * BN / kVec); q += kGemmThreads) {
      const uint32_t r = q / (BN / kVec), c = (q % (BN / kVec)) * kVec;
      const uint32_t i = (uint32_t)(base + (int64_t)(tile_m + r) * a.o_row + tile_n + c);
      const float4 t = *(const float4*)&Cs[r * kCStride + c];
      Quad v;
      v.v[0] = t.x; v.v[1] = t.y; v.v[2] = t.z; v.v[3] = t.w;
      store_vec4<false>(o.ptr, o.dtype, 0, i, v);
    }
    return;
  }
  if (fast) {
    const int sk = post_stream_kind(p);
    constexpr uint32_t kTrips = (uint32_t)(BM * BN / kVec) / kGemmThreads;
    constexpr int Q8 = kTrips % 8u == 0u ? 8 : 4;
    if (sk != 0 && p.n_slots <= 32u / (uint32_t)Q8) {
      post_wide<BM, BN, Q8>(a, pr, Cs, tile_m, tile_n, base, sk == 2);
      return;
    }
    if (sk != 0 && Q8 != 4) {
      post_wide<BM, BN, 4>(a, pr, Cs, tile_m, tile_n, base, sk == 2);
      return;
    }
  }
  if (fast) {
    // two quads per trip (same columns, kGemmThreads quads apart): the interpreter is fetched,
    // decoded and dispatched once for both (register file = 8 slots x 2)
    constexpr uint32_t kRowStep = (uint32_t)kGemmThreads / (BN / kVec);
#pragma unroll 1
    for (uint32_t q = threadIdx.x; q < (uint32_t)(BM * BN / kVec); q += 2u * kGemmThreads) {
      const uint32_t ra = q / (BN / kVec), c = (q % (BN / kVec)) * kVec, rb = ra + kRowStep;
      const uint32_t ia = (uint32_t)(base + (int64_t)(tile_m + ra) * a.o_row + tile_n + c);
      const uint32_t ib = (uint32_t)(base + (int64_t)(tile_m + rb) * a.o_row + tile_n + c);
      const Staged<4> sa = fetch_inputs_at<4, false>(p, ia, row_flat0 + ra, tile_n + c);
      RF<16> f = place_inputs<16, 4, true, false, 0>(rf_zero<16>(), p, sa, kVec);
      const Staged<4> sb = fetch_inputs_at<4, false>(p, ib, row_flat0 + rb, tile_n + c);
      f = place_inputs<16, 4, true, false, 8>(f, p, sb, kVec);
      const float4 ta = *(const float4*)&Cs[ra * kCStride + c], tb = *(const float4*)&Cs[rb * kCStride + c];
      Quad anchor;
      anchor.v[0] = ta.x; anchor.v[1] = ta.y; anchor.v[2] = ta.z; anchor.v[3] = ta.w;
      f = rf_set<16>(f, p.anchor_slot, anchor);
      anchor.v[0] = tb.x; anchor.v[1] = tb.y; anchor.v[2] = tb.z; anchor.v[3] = tb.w;
      f = rf_set<16>(f, p.anchor_slot + 8u, anchor);
      f = interp<16, 2>(f, pr, n_code);
      store_outputs<16, true, false, 0>(f, p, 0, ia, kVec);
      store_outputs<16, true, false, 8>(f, p, 0, ib, kVec);
    }
    return;
  }
#pragma unroll 1
  for (uint32_t q = threadIdx.x; q < (uint32_t)(BM * BN / kVec); q += kGemmThreads) {
    const uint32_t r = q / (BN / kVec), c = (q % (BN / kVec)) * kVec;
    const uint32_t row = tile_m + r, col = tile_n + c;
    if (row >= a.m || col >= a.n) continue;
    const uint32_t nvalid = a.n - col >= (uint32_t)kVec ? (uint32_t)kVec : a.n - col;
    const uint32_t i = (uint32_t)(base + (int64_t)row * a.o_row + col);
    const float4 t = *(const float4*)&Cs[r * kCStride + c];
    Quad anchor;
    anchor.v[0] = t.x; anchor.v[1] = t.y; anchor.v[2] = t.z; anchor.v[3] = t.w;
    RF<16> f = load_inputs<16, kMaxIn, false, false>(rf_zero<16>(), p, 0, i, nvalid);
    f = rf_set<16>(f, p.anchor_slot, anchor);
    f = interp<16>(f, pr, n_code);
    store_outputs<16, false, false>(f, p, 0, i, nvalid);
  }
}

}  // namespace ltk
#endif  // LT_GEMM_EPILOGUE_H_
