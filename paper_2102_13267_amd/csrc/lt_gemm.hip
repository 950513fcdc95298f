// fp32 contraction region: C = post(A * B) on the MFMA matrix cores (gfx950), fp32 operands and
// accumulation (bf16 operands: lt_gemm_bf16.hip).  Operands are addressed through element strides,
// so transposed, batched and head-split layouts need no copies.  The elementwise chain that
// consumes the product (bias, activation, residual, optimiser update, cast ...) is interpreted on
// the accumulator tile before anything is written: the product itself never travels to HBM unless
// asked for.
//
// Structure: workgroup tile 128 x 128 (or 64 x 64 for small problems so that more compute units
// get a tile), four wavefronts in a 2 x 2 arrangement, each owning a quarter as MFMA 32x32x2
// blocks.  K is walked in slices of 32 with register prefetch: the global loads of slice k+1 are
// issued before the MFMAs of slice k and written to the other LDS buffer afterwards.  Global
// loads are 16 bytes per lane along whichever dimension of the operand is contiguous; an operand
// whose contiguous dimension is k is transposed on its way into LDS.  A long k over few tiles is
// split over workgroups (partial products to a workspace, summed by a second launch).
// Small products take another kernel further down (lt_gemm_small_kernel: no LDS staging, k split
// inside the workgroup and, for a long k, over a few workgroups that meet inside the launch).
#include <hip/hip_runtime.h>

#include <cstdio>

#include "lt_gemm_epilogue.h"
#include "lt_launch.h"
#include "lt_reduce.h"

namespace ltk {

// ---- operand staging --------------------------------------------------------------------------
// A "group" is what one lane fetches with one 16-byte load: G consecutive elements along the
// operand's contiguous dimension (4 fp32 or 8 bf16).  For element type T the raw group travels
// as uint4.
template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int G = 4; static constexpr int BK = 32; };

// Guarded fetch of G elements at (outer, inner .. inner+G-1); element (o, i) lives at
// base + o*s_outer + i (unit stride inside the group).  Out-of-range elements read as zero.
template <typename T>
__device__ __forceinline__ uint4 fetch_group(const T* base, int64_t s_outer, uint32_t outer, uint32_t inner, uint32_t n_outer,
                                             uint32_t n_inner, bool aligned) {
  constexpr int G = Elem<T>::G;
  uint4 v = make_uint4(0, 0, 0, 0);
  if (outer >= n_outer || inner >= n_inner) return v;
  const T* src = base + (int64_t)outer * s_outer + inner;
  if (aligned && inner + G <= n_inner) return *(const uint4*)src;
  T t[G];
#pragma unroll
  for (int j = 0; j < G; ++j) t[j] = (inner + j < n_inner) ? src[j] : (T)0;
  v = make_uint4(((const uint32_t*)t)[0], ((const uint32_t*)t)[1], ((const uint32_t*)t)[2], ((const uint32_t*)t)[3]);
  return v;
}

// LDS layout: tile[k][x] (x = m or n contiguous); an MFMA 32x32x2 lane reads one float.  Row stride:
// BX + 4 for an operand that arrives x-contiguous (16-byte row writes stay aligned).  An operand
// that arrives k-contiguous is transposed by scalar writes, eight lanes of a wave writing rows
// 4 apart: BX + 1 puts those rows 4 banks apart, so a wave's 32 writes per cycle hit 32 banks
// (with BX + 4 they hit 8: counters showed as many bank-conflict cycles as LDS cycles).  ELEMS is
// sized for the wider one, so buffers are interchangeable.
template <typename T, int BX> struct Tile;
template <int BX> struct Tile<float, BX> {
  static constexpr int BK = 32, ELEMS = BK * (BX + 4);
  static constexpr int stride(bool kc) { return kc ? BX + 1 : BX + 4; }
};
// Number of 16-byte groups per lane and k-slice for an operand tile of BX x BK elements.
template <typename T, int BX> struct Groups {
  static constexpr int N = BX * Elem<T>::BK / Elem<T>::G / kGemmThreads;   // 128: 2, 64: 1
};

// (a native vector type, not HIP's uint4 struct: sets of the struct kind that are only ever moved
// whole were left in scratch memory by the compiler)
typedef uint32_t U32x4 __attribute__((ext_vector_type(4)));
template <int N> struct GroupRegs {
  U32x4 g[N];
};

// Fetch this lane's groups of the slice starting at k0.  KC: the contraction dimension is the
// operand's contiguous one.  x0: first row (A) / column (B) of the tile.
template <typename T, int BX, bool KC>
__device__ __forceinline__ void fetch_tile(GroupRegs<Groups<T, BX>::N>& gr, const T* base, int64_t s_x, int64_t s_k, uint32_t x0,
                                           uint32_t k0, uint32_t nx, uint32_t nk, bool aligned) {
  constexpr int G = Elem<T>::G, BK = Elem<T>::BK, NG = Groups<T, BX>::N;
  const uint32_t t = threadIdx.x;
#pragma unroll
  for (int it = 0; it < NG; ++it) {
    const uint32_t e = it * kGemmThreads + t;
    if (KC) {
      const uint32_t x = e / (BK / G), kq = e % (BK / G);
      const uint4 v = fetch_group<T>(base, s_x, x0 + x, k0 + kq * G, nx, nk, aligned);
      gr.g[it] = U32x4{v.x, v.y, v.z, v.w};
    } else {
      const uint32_t k = e / (BX / G), xq = e % (BX / G);
      const uint4 v = fetch_group<T>(base, s_k, k0 + k, x0 + xq * G, nk, nx, aligned);
      gr.g[it] = U32x4{v.x, v.y, v.z, v.w};
    }
  }
}

template <int BX, bool KC>
__device__ __forceinline__ void stash_tile(const GroupRegs<Groups<float, BX>::N>& gr, float* tile) {
  constexpr int G = 4, BK = Elem<float>::BK, STRIDE = Tile<float, BX>::stride(KC), NG = Groups<float, BX>::N;
  const uint32_t t = threadIdx.x;
#pragma unroll
  for (int it = 0; it < NG; ++it) {
    const uint32_t e = it * kGemmThreads + t;
    if (KC) {   // transposing: four scalar writes
      const uint32_t x = e / (BK / G), kq = e % (BK / G);
      tile[(kq * G + 0) * STRIDE + x] = __uint_as_float(gr.g[it].x);
      tile[(kq * G + 1) * STRIDE + x] = __uint_as_float(gr.g[it].y);
      tile[(kq * G + 2) * STRIDE + x] = __uint_as_float(gr.g[it].z);
      tile[(kq * G + 3) * STRIDE + x] = __uint_as_float(gr.g[it].w);
    } else {
      const uint32_t k = e / (BX / G), xq = e % (BX / G);
      *(U32x4*)&tile[k * STRIDE + xq * G] = gr.g[it];
    }
  }
}

// Interior tiles of aligned operands: the slice at k0, 16 bytes per lane and load, no checks and
// no branches, so that all of a slice's loads are in flight together.
// x_last: the operand's last row (KC only): rows of a tile that hangs over the edge are read as
// copies of it -- in bounds, and their products are never stored -- so that a tile of a few rows
// (a small batch) still takes this path.
template <int BX, bool KC>
__device__ __forceinline__ void fetch_tile_whole(GroupRegs<Groups<float, BX>::N>& gr, const float* base, int64_t s_x, int64_t s_k,
                                                 uint32_t x0, uint32_t k0, uint32_t x_last) {
  constexpr int G = 4, BK = Elem<float>::BK, NG = Groups<float, BX>::N;
  const uint32_t t = threadIdx.x;
#pragma unroll
  for (int it = 0; it < NG; ++it) {
    const uint32_t e = it * kGemmThreads + t;
    const float* src = KC ? base + (int64_t)min(x0 + e / (BK / G), x_last) * s_x + (k0 + (e % (BK / G)) * G)
                          : base + (int64_t)(k0 + e / (BX / G)) * s_k + (x0 + (e % (BX / G)) * G);
    gr.g[it] = *(const U32x4*)src;
  }
}

// MFMAs of one k-slice, in groups of four k-steps: the fragments of the next group are read from
// LDS BEFORE the MFMAs of the current one are issued (two register sets; scheduling barriers keep
// the compiler from sinking the reads to their first use), so the matrix cores never wait for an
// LDS round trip inside a slice.
// acc has NCH accumulator sets ("chains"); k-step s adds into set s % NCH.  A wave that owns a
// single 32 x 32 block would otherwise issue nothing but MFMAs that each wait for the one before.
template <int BM, int BN, int MB, int NB, bool AKC, bool BKC, int NCH>
__device__ __forceinline__ void mma_slice(v16f (&acc)[NCH][MB][NB], const float* As, const float* Bs, uint32_t wave_m, uint32_t wave_n,
                                          uint32_t lane) {
  constexpr int SA = Tile<float, BM>::stride(AKC), SB = Tile<float, BN>::stride(BKC), BK = Elem<float>::BK;
  constexpr int KG = 4, NGRP = BK / 2 / KG;   // k-steps per group, groups per slice
  const float* ap = As + (lane >> 5) * SA + wave_m * (MB * 32) + (lane & 31);
  const float* bp = Bs + (lane >> 5) * SB + wave_n * (NB * 32) + (lane & 31);
  float af[2][KG][MB], bf[2][KG][NB];
  auto read_group = [&](int set, int g) {
#pragma unroll
    for (int s = 0; s < KG; ++s) {
      const int kk = (g * KG + s) * 2;
#pragma unroll
      for (int i = 0; i < MB; ++i) af[set][s][i] = ap[kk * SA + i * 32];
#pragma unroll
      for (int j = 0; j < NB; ++j) bf[set][s][j] = bp[kk * SB + j * 32];
    }
  };
  read_group(0, 0);
#pragma unroll
  for (int g = 0; g < NGRP; ++g) {
    if (g + 1 < NGRP) read_group((g + 1) & 1, g + 1);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int s = 0; s < KG; ++s)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
          acc[s % NCH][i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[g & 1][s][i], bf[g & 1][s][j], acc[s % NCH][i][j], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
}

template <typename T, int BM, int BN> struct Smem {
  static constexpr size_t kOperands = 2 * (Tile<T, BM>::ELEMS + Tile<T, BN>::ELEMS) * sizeof(T);   // double buffered
  static constexpr size_t kC = (size_t)BM * (BN + kCPad) * sizeof(float);
  static constexpr size_t kBytes = kOperands > kC ? kOperands : kC;
};

// T: float.  AKC / BKC: the operand's contiguous dimension is k.
template <typename T, int BM, int BN, bool AKC, bool BKC>
__global__ __launch_bounds__(kGemmThreads, BM == 64 ? 2 : 1) void lt_gemm_kernel(const GemmArgs a) {
  constexpr int MB = BM / 64, NB = BN / 64, BK = Elem<T>::BK;
  __shared__ __attribute__((aligned(16))) char smem[Smem<T, BM, BN>::kBytes];
  // LDS map: A buffer 0, A buffer 1, B buffer 0, B buffer 1 (the C tile of the epilogue reuses it)
  T* const lds = (T*)smem;
  auto As = [&](uint32_t buf) { return lds + buf * Tile<T, BM>::ELEMS; };
  auto Bs = [&](uint32_t buf) { return lds + 2 * Tile<T, BM>::ELEMS + buf * Tile<T, BN>::ELEMS; };
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t wave_m = wave >> 1, wave_n = wave & 1;
  const uint32_t tile_m = blockIdx.y * BM, tile_n = blockIdx.x * BN;
  const uint32_t batch = blockIdx.z / a.splits, split = blockIdx.z % a.splits;
  // this workgroup's share of k: whole slices, split evenly
  const uint32_t slices = (a.k + BK - 1) / BK, per = (slices + a.splits - 1) / a.splits;
  const uint32_t k_begin = min(a.k, split * per * BK), k_end = min(a.k, (split + 1) * per * BK);
  const uint32_t b0 = batch / a.batch1, b1 = batch % a.batch1;
  const T* A = (const T*)a.a.ptr + (int64_t)b0 * a.a.s_b0 + (int64_t)b1 * a.a.s_b1;
  const T* B = (const T*)a.b.ptr + (int64_t)b0 * a.b.s_b0 + (int64_t)b1 * a.b.s_b1;
  // 16-byte loads need 16-byte aligned groups: base, and the stride between groups' rows
  constexpr int G = Elem<T>::G;
  const int64_t a_outer = AKC ? a.a.s_row : a.a.s_col, b_outer = BKC ? a.b.s_col : a.b.s_row;
  const bool a_al = (((uintptr_t)A) & 15u) == 0 && (a_outer % G) == 0;
  const bool b_al = (((uintptr_t)B) & 15u) == 0 && (b_outer % G) == 0;
  constexpr int NCH = MB * NB == 1 ? 2 : 1;   // independent accumulator chains per block
  v16f accs[NCH][MB][NB];
#pragma unroll
  for (int c = 0; c < NCH; ++c)
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) accs[c][i][j][r] = 0.0f;

  GroupRegs<Groups<T, BM>::N> ga;
  GroupRegs<Groups<T, BN>::N> gb;
  const bool whole = a_al && b_al && (AKC || tile_m + BM <= a.m) && (BKC || tile_n + BN <= a.n) && ((k_end - k_begin) % BK) == 0u;
  if (k_begin < k_end && whole) {
    // Interior tile: unchecked 16-byte loads, D slices ahead in registers (a slice's MFMAs are over
    // in 1000 to 4000 cycles, a load under traffic takes longer: counters showed a wave of the
    // one-slice-ahead loop waiting two thirds of its life), two LDS buffers.  Slice i: start the
    // loads of slice i + D into the register set that slice i left when it was written to LDS;
    // multiply slice i from its LDS buffer; write slice i + 1 to the other buffer; barrier.  The
    // body is unrolled D times so that set and buffer numbers are compile-time; loads past the
    // end are clamped to the last slice (in bounds, unused).
    // (Four named register sets, not an array: an array of sets indexed by the unrolled loop
    // counter is left in scratch memory by the compiler, and every load then waits to be spilled.)
    const uint32_t n = (k_end - k_begin) / BK;
    typedef GroupRegs<Groups<T, BM>::N> RA;
    typedef GroupRegs<Groups<T, BN>::N> RB;
    RA ra0, ra1, ra2, ra3;
    RB rb0, rb1, rb2, rb3;
    constexpr uint32_t D = BM == 64 ? 4u : 2u;   // slices in flight (a 128 x 128 tile's sets are twice as large)
#define LT_FETCH(RA_, RB_, I)                                                                 \
  {                                                                                           \
    const uint32_t kf = k_begin + min((uint32_t)(I), n - 1u) * BK;                            \
    fetch_tile_whole<BM, AKC>(RA_, A, a.a.s_row, a.a.s_col, tile_m, kf, a.m - 1u);            \
    fetch_tile_whole<BN, BKC>(RB_, B, a.b.s_col, a.b.s_row, tile_n, kf, a.n - 1u);            \
  }
#define LT_STEP(J, RA_CUR, RB_CUR, RA_NEXT, RB_NEXT)                                          \
  {                                                                                           \
    const uint32_t i = i0 + (J);                                                              \
    LT_FETCH(RA_CUR, RB_CUR, i + D);                                                          \
    if (i < n) mma_slice<BM, BN, MB, NB, AKC, BKC, NCH>(accs, As((J) & 1), Bs((J) & 1), wave_m, wave_n, lane); \
    stash_tile<BM, AKC>(RA_NEXT, As(((J) + 1) & 1));                                          \
    stash_tile<BN, BKC>(RB_NEXT, Bs(((J) + 1) & 1));                                          \
    __syncthreads();                                                                          \
  }
    LT_FETCH(ra0, rb0, 0);
    LT_FETCH(ra1, rb1, 1);
    if (D == 4u) {
      LT_FETCH(ra2, rb2, 2);
      LT_FETCH(ra3, rb3, 3);
    }
    stash_tile<BM, AKC>(ra0, As(0));
    stash_tile<BN, BKC>(rb0, Bs(0));
    __syncthreads();
    if (D == 4u) {
      for (uint32_t i0 = 0; i0 < n; i0 += 4u) {
        LT_STEP(0u, ra0, rb0, ra1, rb1);
        LT_STEP(1u, ra1, rb1, ra2, rb2);
        LT_STEP(2u, ra2, rb2, ra3, rb3);
        LT_STEP(3u, ra3, rb3, ra0, rb0);
      }
    } else {
      for (uint32_t i0 = 0; i0 < n; i0 += 2u) {
        LT_STEP(0u, ra0, rb0, ra1, rb1);
        LT_STEP(1u, ra1, rb1, ra0, rb0);
      }
    }
#undef LT_STEP
#undef LT_FETCH
  } else if (k_begin < k_end) {
    fetch_tile<T, BM, AKC>(ga, A, a.a.s_row, a.a.s_col, tile_m, k_begin, a.m, k_end, a_al);
    fetch_tile<T, BN, BKC>(gb, B, a.b.s_col, a.b.s_row, tile_n, k_begin, a.n, k_end, b_al);
    stash_tile<BM, AKC>(ga, As(0));
    stash_tile<BN, BKC>(gb, Bs(0));
    __syncthreads();
    uint32_t cur = 0;
    for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
      const bool more = k0 + BK < k_end;
      if (more) {
        fetch_tile<T, BM, AKC>(ga, A, a.a.s_row, a.a.s_col, tile_m, k0 + BK, a.m, k_end, a_al);
        fetch_tile<T, BN, BKC>(gb, B, a.b.s_col, a.b.s_row, tile_n, k0 + BK, a.n, k_end, b_al);
      }
      mma_slice<BM, BN, MB, NB, AKC, BKC, NCH>(accs, As(cur), Bs(cur), wave_m, wave_n, lane);
      if (more) {
        stash_tile<BM, AKC>(ga, As(cur ^ 1));
        stash_tile<BN, BKC>(gb, Bs(cur ^ 1));
      }
      __syncthreads();
      cur ^= 1;
    }
  }
  v16f (&acc)[MB][NB] = accs[0];
  if (NCH > 1) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][j][r] += accs[NCH - 1][i][j][r];
  }
  // split-K: this workgroup's partial product goes to its own fp32 copy of the output, row major
  float* const raw = a.splits > 1u ? a.split_ws + (size_t)split * ((size_t)a.batch0 * a.batch1 * a.m * a.n) : nullptr;
  epilogue<BM, BN, MB, NB>(a, acc, (float*)smem, tile_m, tile_n, wave_m, wave_n, lane, batch, raw);
}

// ---- small contractions -------------------------------------------------------------------------
// A product of a few dozen 64 x 64 tiles leaves most compute units idle, and splitting its k over
// workgroups costs a second launch that adds the partial products up (for a 128 x 784 x 512 layer
// two launches of 5 to 7 microseconds each, most of it launch and memory latency).  Here a
// workgroup of eight wavefronts owns a 32 x 32 tile of the output and splits k INSIDE the
// workgroup: every wave contracts an eighth of k (whole groups of 8) for the whole tile, with its
// operands fetched from global memory straight into the MFMA 32x32x2 register layout -- lane
// (x, h) supplies A[x][k] and B[k][x] for the k of half h, and which k of a group goes into which
// of its four MFMAs is free as long as both operands agree, so a lane takes four CONSECUTIVE k
// (4 h .. 4 h + 3): one 16-byte load where k is the operand's contiguous dimension, four 4-byte
// loads that neighbouring lanes coalesce where it is not.  No LDS staging and no barrier in the
// loop; kSmallG groups (32 k) are in flight per wave while the previous ones are multiplied.  The
// partial tiles of the waves meet in LDS, are added in a fixed order, and the post program runs on
// the sum: one launch.  (A tile may also be two blocks of 32 x 32: then two times four waves.)
// A long k over very few tiles (a batch of 8 rows against a 2048 x 2048 weight: 64 tiles) would
// leave three quarters of the compute units idle and every wave with several dependent round trips
// to memory, so there `splits` workgroups share a tile, each with a slice of k.  Their partial
// tiles (4 KB each) go to a scratch with relaxed device-scope stores, each workgroup takes a ticket
// of its tile, and the one that draws the last ticket adds the partial tiles up in split order
// (deterministic) and runs the post program -- the same exchange as in the reductions, still one
// launch.
constexpr int kSmallThreads = 512, kSmallWaves = 8, kSmallG = 4, kSmallStride = 32 + kCPad;

template <bool V>
__device__ __forceinline__ void small_fetch(float (&v)[kSmallG][4], const float* base, int64_t s_k, uint32_t k0, uint32_t k_end) {
#pragma unroll
  for (int g = 0; g < kSmallG; ++g) {
    const uint32_t kg = k0 + (uint32_t)g * 8u;
    if (V) {   // k is contiguous and a multiple of 4: the four are valid together
      const bool ok = kg < k_end;
      const float4 t = *(const float4*)(base + (ok ? kg : 0u));
      v[g][0] = ok ? t.x : 0.0f; v[g][1] = ok ? t.y : 0.0f; v[g][2] = ok ? t.z : 0.0f; v[g][3] = ok ? t.w : 0.0f;
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const bool ok = kg + (uint32_t)j < k_end;
        const float t = base[(int64_t)(ok ? kg + (uint32_t)j : 0u) * s_k];   // (past the end: element 0 again, in bounds, zeroed)
        v[g][j] = ok ? t : 0.0f;
      }
    }
  }
}

__device__ __forceinline__ void small_mma(v16f& acc0, v16f& acc1, const float (&av)[kSmallG][4], const float (&bv)[kSmallG][4]) {
#pragma unroll
  for (int g = 0; g < kSmallG; ++g) {
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g][0], bv[g][0], acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g][1], bv[g][1], acc1, 0, 0, 0);
    acc0 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g][2], bv[g][2], acc0, 0, 0, 0);
    acc1 = __builtin_amdgcn_mfma_f32_32x32x2f32(av[g][3], bv[g][3], acc1, 0, 0, 0);
  }
}

__device__ __forceinline__ float small_colsum(const float (&bv)[kSmallG][4]) {
  float s = 0.0f;
#pragma unroll
  for (int g = 0; g < kSmallG; ++g) s += (bv[g][0] + bv[g][1]) + (bv[g][2] + bv[g][3]);
  return s;
}

// TM x TN: blocks of 32 x 32 per workgroup tile (1 x 1, 2 x 1 or 2 x 2); the eight waves are NB =
// TM * TN blocks times 8 / NB shares of k.  AV / BV: k is the operand's contiguous dimension and
// every group of four is a whole, 16-byte aligned vector (the launcher checks the pointer, the
// strides and k % 4).  CS: the column sums of B ride along (GemmArgs::col_sum); a variant of its own, because the
// second program costs 40 registers that the plain product does not have to carry.
template <int TM, int TN, bool AV, bool BV, bool CS>
__global__ __launch_bounds__(kSmallThreads) void lt_gemm_small_kernel(const GemmArgs a) {
  constexpr uint32_t NB = TM * TN, KW = kSmallWaves / NB;      // blocks, k shares inside the workgroup
  constexpr uint32_t kQuads = NB * 256u, QT = (kQuads + kSmallThreads - 1u) / kSmallThreads;   // quads of the tile, per thread
  __shared__ __attribute__((aligned(16))) float Cs[kSmallWaves * 32 * kSmallStride];
  __shared__ uint32_t is_last;
  __shared__ float colp[CS ? kSmallThreads : 1], coltot[CS ? 32 * TN : 1];
  const uint32_t lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t block = wave % NB, kway = wave / NB, bm = block / TN, bn = block % TN;
  const uint32_t per_batch = a.tiles_m * a.tiles_n;
  const uint32_t tile = blockIdx.x / a.splits, split = blockIdx.x % a.splits;   // (the workgroups of a tile are neighbours)
  const uint32_t batch = tile / per_batch, rem = tile % per_batch;
  const uint32_t tile_m = (rem / a.tiles_n) * (32u * TM), tile_n = (rem % a.tiles_n) * (32u * TN);
  const uint32_t b0 = batch / a.batch1, b1 = batch % a.batch1;
  const float* A = (const float*)a.a.ptr + (int64_t)b0 * a.a.s_b0 + (int64_t)b1 * a.a.s_b1;
  const float* B = (const float*)a.b.ptr + (int64_t)b0 * a.b.s_b0 + (int64_t)b1 * a.b.s_b1;
  // this workgroup's slice of k, and this wave's share of it: whole groups of 8
  const uint32_t per_wg = (((a.k + 7u) / 8u) + a.splits - 1u) / a.splits;
  const uint32_t wg_begin = min(a.k, split * per_wg * 8u), wg_end = min(a.k, (split + 1u) * per_wg * 8u);
  const uint32_t groups = (wg_end - wg_begin + 7u) / 8u, per = (groups + KW - 1u) / KW;
  const uint32_t k_begin = min(wg_end, wg_begin + kway * per * 8u), k_end = min(wg_end, wg_begin + (kway + 1u) * per * 8u);
  const uint32_t x = lane & 31u, h = lane >> 5;
  // rows and columns over the edge are read as copies of the last one (in bounds; never stored)
  const float* ap = A + (int64_t)min(tile_m + bm * 32u + x, a.m - 1u) * a.a.s_row;
  const float* bp = B + (int64_t)min(tile_n + bn * 32u + x, a.n - 1u) * a.b.s_col;
  // The post program and, where every quad of the tile is a whole aligned vector inside the
  // output, its inputs for this thread's quads are asked for now, so that they travel under the
  // contraction.  Quad q of the tile: block q / 256, row (q % 256) / 8 of it, columns 4 (q % 8) ..
  // (the program lives in the lanes of two registers: fetched while every lane is active)
  const EwProg& p = a.post;
  const ProgRegs pr = load_prog_regs(p);
  // column sums of B ride along in the first tile row (every column block exactly once)
  const bool cols_here = CS && tile_m == 0u;                    // (workgroup-uniform)
  const bool cols_mine = cols_here && bm == 0u;                 // (wave-uniform)
  const ProgRegs cpr = CS ? load_prog_regs(a.col_post) : ProgRegs{0u, 0.0f};
  float csum = 0.0f;
  const bool fast = p.fast && p.full_vec_ok && p.n_in <= 4u && p.n_slots <= 8u && tile_m + 32u * TM <= a.m && tile_n + 32u * TN <= a.n;
  uint32_t qrow[QT], qcol[QT], qi[QT];
#pragma unroll
  for (uint32_t j = 0; j < QT; ++j) {
    const uint32_t q = (threadIdx.x + j * kSmallThreads) % kQuads, qb = q >> 8;   // (threads past the last quad: a copy, never used)
    qrow[j] = tile_m + (qb / TN) * 32u + ((q & 255u) >> 3);
    qcol[j] = tile_n + (qb % TN) * 32u + (q & 7u) * (uint32_t)kVec;
    qi[j] = (uint32_t)((int64_t)b0 * a.o_b0 + (int64_t)b1 * a.o_b1 + (int64_t)qrow[j] * a.o_row + qcol[j]);
  }
  const bool has_quad = threadIdx.x < kQuads;   // (wave-uniform: kQuads is a multiple of 64)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Wuninitialized"
#pragma clang diagnostic ignored "-Wsometimes-uninitialized"
  Staged<4> staged[QT];
  if (fast && has_quad) {
#pragma unroll
    for (uint32_t j = 0; j < QT; ++j) staged[j] = fetch_inputs_at<4, false, false>(p, qi[j], (b0 * a.batch1 + b1) * a.m + qrow[j], qcol[j]);
  }
#pragma clang diagnostic pop
  v16f acc0, acc1;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc0[r] = acc1[r] = 0.0f;
  constexpr uint32_t kChunk = (uint32_t)kSmallG * 8u;
  const uint32_t nch = (k_end - k_begin + kChunk - 1u) / kChunk;   // (wave-uniform)
  float a0[kSmallG][4], b0v[kSmallG][4], a1[kSmallG][4], b1v[kSmallG][4];
  const uint32_t kl = k_begin + 4u * h;   // this lane's first k
  if (nch > 0u) {
    small_fetch<AV>(a0, ap, a.a.s_col, kl, k_end);
    small_fetch<BV>(b0v, bp, a.b.s_row, kl, k_end);
  }
  for (uint32_t c = 0; c < nch; c += 2u) {
    if (c + 1u < nch) {
      small_fetch<AV>(a1, ap, a.a.s_col, kl + (c + 1u) * kChunk, k_end);
      small_fetch<BV>(b1v, bp, a.b.s_row, kl + (c + 1u) * kChunk, k_end);
    }
    small_mma(acc0, acc1, a0, b0v);
    if (cols_mine) csum += small_colsum(b0v);
    if (c + 2u < nch) {
      small_fetch<AV>(a0, ap, a.a.s_col, kl + (c + 2u) * kChunk, k_end);
      small_fetch<BV>(b0v, bp, a.b.s_row, kl + (c + 2u) * kChunk, k_end);
    }
    if (c + 1u < nch) {
      small_mma(acc0, acc1, a1, b1v);
      if (cols_mine) csum += small_colsum(b1v);
    }
  }
  if (CS) colp[threadIdx.x] = csum;
  float* mine = Cs + wave * (32u * kSmallStride);   // (wave = kway * NB + block)
#pragma unroll
  for (int r = 0; r < 16; ++r) mine[((uint32_t)(r >> 2) * 8u + h * 4u + (uint32_t)(r & 3)) * kSmallStride + x] = acc0[r] + acc1[r];
  __syncthreads();
  float4 sum[QT];
#pragma unroll
  for (uint32_t j = 0; j < QT; ++j) {
    const uint32_t q = (threadIdx.x + j * kSmallThreads) % kQuads;
    const float* src = Cs + (q >> 8) * (32u * kSmallStride) + ((q & 255u) >> 3) * kSmallStride + (q & 7u) * (uint32_t)kVec;
    sum[j] = *(const float4*)src;
#pragma unroll
    for (uint32_t w = 1; w < KW; ++w) {   // share order: deterministic
      const float4 t = *(const float4*)(src + w * NB * (32u * kSmallStride));
      sum[j].x += t.x; sum[j].y += t.y; sum[j].z += t.z; sum[j].w += t.w;
    }
  }
  if (cols_here) {
    // column c of column block bn: the shares of k in order, lower half of the wave before the upper
    // (deterministic); then the column program on quads of four columns
    if (threadIdx.x < 32u * TN) {
      const uint32_t cb = threadIdx.x >> 5, cx = threadIdx.x & 31u;
      float t = 0.0f;
#pragma unroll
      for (uint32_t w = 0; w < KW; ++w) {
        const float* src = colp + (w * NB + cb) * 64u + cx;   // (wave = share * NB + block; block = bm * TN + bn with bm = 0)
        t += src[0];
        t += src[32];
      }
      if (a.col_red == kRedMean) t = t / (float)a.k;
      coltot[threadIdx.x] = t;
    }
    __syncthreads();
    const uint32_t cc = tile_n + threadIdx.x * (uint32_t)kVec;
    if (threadIdx.x < 8u * TN && cc < a.n) {
      const EwProg& cp = a.col_post;
      const uint32_t nv = a.n - cc >= (uint32_t)kVec ? (uint32_t)kVec : a.n - cc;
      Quad q;
#pragma unroll
      for (int e = 0; e < kVec; ++e) q.v[e] = coltot[threadIdx.x * (uint32_t)kVec + (uint32_t)e];
      RF<16> f = load_inputs<16, kMaxIn, false, false>(rf_zero<16>(), cp, 0, cc, nv);
      f = rf_set<16>(f, cp.anchor_slot, q);
      f = interp<16>(f, cpr, cp.n_code);
      store_outputs<16, false, false>(f, cp, 0, cc, nv);
    }
  }
  if (a.splits > 1u) {
    // leave this workgroup's partial tile, take a ticket; whoever draws the last one goes on
    float* const parts = a.split_ws + (size_t)tile * a.splits * (NB * 1024u);
    if (has_quad) {
#pragma unroll
      for (uint32_t j = 0; j < QT; ++j)
        publish4(parts + (size_t)split * (NB * 1024u) + (size_t)((threadIdx.x + j * kSmallThreads) % kQuads) * 4u, sum[j]);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // (this wave's stores have been performed before the ticket is taken)
    }
    __syncthreads();
    if (threadIdx.x == 0u) {
      const uint32_t t = atomicAdd(&a.tickets[tile], 1u);
      is_last = (t == a.splits - 1u) ? 1u : 0u;
      if (t == a.splits - 1u) a.tickets[tile] = 0u;   // (every workgroup of the tile has been here)
    }
    __syncthreads();
    if (!is_last) return;
    if (has_quad) {
#pragma unroll
      for (uint32_t j = 0; j < QT; ++j) {
        sum[j] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        for (uint32_t sp = 0; sp < a.splits; ++sp) {   // split order: deterministic
          const float4 t = published4(parts + (size_t)sp * (NB * 1024u) + (size_t)((threadIdx.x + j * kSmallThreads) % kQuads) * 4u);
          sum[j].x += t.x; sum[j].y += t.y; sum[j].z += t.z; sum[j].w += t.w;
        }
      }
    }
  }
  if (!has_quad) return;
  const uint32_t n_code = p.n_code;
#pragma unroll
  for (uint32_t j = 0; j < QT; ++j) {
    Quad anchor;
    anchor.v[0] = sum[j].x; anchor.v[1] = sum[j].y; anchor.v[2] = sum[j].z; anchor.v[3] = sum[j].w;
    if (fast) {
      RF<16> f = place_inputs<16, 4, true, false, 0>(rf_zero<16>(), p, staged[j], kVec);
      f = rf_set<16>(f, p.anchor_slot, anchor);
      f = interp<16>(f, pr, n_code);
      store_outputs<16, true, false, 0>(f, p, 0, qi[j], kVec);
    } else if (qrow[j] < a.m && qcol[j] < a.n) {
      const uint32_t nvalid = a.n - qcol[j] >= (uint32_t)kVec ? (uint32_t)kVec : a.n - qcol[j];
      RF<16> f = load_inputs<16, kMaxIn, false, false>(rf_zero<16>(), p, 0, qi[j], nvalid);
      f = rf_set<16>(f, p.anchor_slot, anchor);
      f = interp<16>(f, pr, n_code);
      store_outputs<16, false, false>(f, p, 0, qi[j], nvalid);
    }
  }
}

template <int TM, int TN, bool CS>
static void launch_small_tile(const GemmArgs& a, bool av, bool bv, dim3 grid, hipStream_t s) {
  const dim3 block(kSmallThreads);
  if (av && bv) LT_LAUNCH((lt_gemm_small_kernel<TM, TN, true, true, CS>), grid, block, s, a);
  else if (av) LT_LAUNCH((lt_gemm_small_kernel<TM, TN, true, false, CS>), grid, block, s, a);
  else if (bv) LT_LAUNCH((lt_gemm_small_kernel<TM, TN, false, true, CS>), grid, block, s, a);
  else LT_LAUNCH((lt_gemm_small_kernel<TM, TN, false, false, CS>), grid, block, s, a);
}

static hipError_t launch_small(const GemmArgs& args, hipStream_t s) {
  GemmArgs a = args;
  // (the kernel is written for 1 x 1, 2 x 1 and 2 x 2 blocks; 2 x 2 lost to the split pair on every
  // shape measured and is not built)
  const bool t11 = a.tile_m == 32u && a.tile_n == 32u, t21 = a.tile_m == 64u && a.tile_n == 32u;
  if (!t11 && !t21) return hipErrorInvalidValue;
  a.tiles_m = (a.m + a.tile_m - 1u) / a.tile_m;
  a.tiles_n = (a.n + a.tile_n - 1u) / a.tile_n;
  const uint64_t wgs = (uint64_t)a.tiles_m * a.tiles_n * a.batch0 * a.batch1;
  if (a.splits == 0u || wgs * a.splits > 0x7fffffffull) return hipErrorInvalidValue;
  if (a.splits > 1u && (!a.split_ws || !a.tickets)) return hipErrorInvalidValue;
  // column sums ride along only with an unshared, unbatched product whose B is [k, n] with rows contiguous
  if (a.col_sum && (!t11 || a.splits != 1u || a.batch0 * a.batch1 != 1u || a.b.s_col != 1 || a.col_post.n_slots > 16u)) return hipErrorInvalidValue;
  if (wgs == 0u) return hipSuccess;
  auto whole = [&](const GemmOperand& o, bool k_contiguous, int64_t s_outer) {
    return k_contiguous && (a.k % 4u) == 0u && (((uintptr_t)o.ptr) & 15u) == 0u && (s_outer % 4) == 0 && (o.s_b0 % 4) == 0 && (o.s_b1 % 4) == 0;
  };
  const bool av = whole(a.a, a.a.s_col == 1, a.a.s_row), bv = whole(a.b, a.b.s_row == 1, a.b.s_col);
  const dim3 grid((uint32_t)(wgs * a.splits));
  if (t11 && a.col_sum) launch_small_tile<1, 1, true>(a, av, bv, grid, s);
  else if (t11) launch_small_tile<1, 1, false>(a, av, bv, grid, s);
  else launch_small_tile<2, 1, false>(a, av, bv, grid, s);
  char name[64];
  snprintf(name, sizeof(name), "lt_gemm_small_kernel<%u, %u, %s, %s, %s>", a.tile_m / 32u, a.tile_n / 32u, av ? "true" : "false", bv ? "true" : "false",
           a.col_sum ? "true" : "false");
  note_kernel(name);
  return hipGetLastError();
}

template <typename T, int BM, int BN>
static void launch_variant(const GemmArgs& a, const dim3 grid, hipStream_t s) {
  const bool akc = a.a.s_col == 1, bkc = a.b.s_row == 1;
  if (akc && bkc) LT_LAUNCH((lt_gemm_kernel<T, BM, BN, true, true>), grid, dim3(kGemmThreads), s, a);
  else if (akc) LT_LAUNCH((lt_gemm_kernel<T, BM, BN, true, false>), grid, dim3(kGemmThreads), s, a);
  else if (bkc) LT_LAUNCH((lt_gemm_kernel<T, BM, BN, false, true>), grid, dim3(kGemmThreads), s, a);
  else LT_LAUNCH((lt_gemm_kernel<T, BM, BN, false, false>), grid, dim3(kGemmThreads), s, a);
  char name[48];
  snprintf(name, sizeof(name), "lt_gemm_kernel<float, %d, %d, %s, %s>", BM, BN, akc ? "true" : "false", bkc ? "true" : "false");
  note_kernel(name);
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  // an operand must have unit stride along one of its two dimensions
  if ((a.a.s_col != 1 && a.a.s_row != 1) || (a.b.s_col != 1 && a.b.s_row != 1)) return hipErrorInvalidValue;
  if (a.in_dtype == kBF16) return launch_gemm_bf16(a, s);
  const uint32_t batch = a.batch0 * a.batch1;
  if (a.direct) return launch_small(a, s);
  if (a.tile_m != a.tile_n || (a.tile_m != 64u && a.tile_m != 128u)) return hipErrorInvalidValue;
  const bool big = a.tile_m == 128u;   // the host picks big tiles only when they still give every compute unit work
  const uint32_t bm = a.tile_m;
  if (a.splits == 0u) return hipErrorInvalidValue;
  const dim3 grid((a.n + bm - 1) / bm, (a.m + bm - 1) / bm, batch * a.splits);
  if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
  if (big) launch_variant<float, 128, 128>(a, grid, s);
  else launch_variant<float, 64, 64>(a, grid, s);
  return hipGetLastError();
}

}  // namespace ltk
