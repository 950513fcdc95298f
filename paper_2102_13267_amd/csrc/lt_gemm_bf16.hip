// bf16 contraction on the gfx950 matrix cores: C = post(A * B), fp32 accumulation.
//
// Workgroup tile 128 x 128 (128 x 64 for narrow outputs), k walked in slices of 32, four
// wavefronts in a 2 x 2 arrangement, each owning 64 x 64 (64 x 32) as blocks of
// v_mfma_f32_32x32x16_bf16.  What bounds this kernel is the way into the matrix cores, not the
// matrix cores: per slice a workgroup brings 16 KiB through the L1 (64 bytes per cycle and compute
// unit: 256 cycles) and reads 32 KiB of fragments from LDS for 32 MFMAs (256 cycles per SIMD) --
// at the matrix cores' peak a 128 x 128 tile needs all of the L1's bandwidth.  Two workgroups
// share a compute unit, so one's matrix instructions run under the other's copies, LDS traffic,
// barriers and epilogue.
//
// Whole, 16-byte aligned tiles go from global memory into LDS without touching registers
// (global_load_lds_dwordx4), into dense tiles whose bank conflicts a swizzle takes care of; four
// stages, copies two to three slices ahead, in pairs of slices when an operand's rows are half
// cache lines (see "whole tiles" below).  An MFMA lane wants 8 consecutive k of one row (A) or
// column (B):
//  * k is the operand's contiguous dimension: the tile is [x][k] and a fragment is one
//    ds_read_b128;
//  * x (m or n) is the contiguous dimension: the tile stays as it arrives, [k][x], and the
//    transpose happens in the LDS read: ds_read_b64_tr_b16 hands each lane of a 16-lane group one
//    column of a 4 x 16 sub-tile (lane i gets element i of each of the four rows that lanes
//    4j .. 4j+3 point at), so two such reads give the 8 k values of one x.
// Nothing is transposed by scalar code.  Ragged or unaligned tiles take a second path: every
// access checked, global -> registers -> padded LDS tiles, one slice at a time.
//
// Epilogue (lt_gemm_epilogue.h): the accumulators leave the MFMA layout through LDS, the whole tile
// at once, and are then walked in row-major 4-element quads by the interpreter (bias, activation,
// residual, optimiser update, cast ...), so the product itself never travels to HBM unless
// asked for.
//
// Split-K: when a problem has few output tiles but a long k, `splits` workgroups share a tile and
// each leaves its fp32 partial product in a workspace; a second, elementwise launch adds them in
// split order and runs the post program at full occupancy (an interpreted epilogue run by one
// workgroup per tile would leave most of the chip idle).
//
// Tile order: workgroups are handed to the eight XCDs round robin, so consecutive workgroup
// numbers are remapped to make each XCD's share a contiguous block of tiles (one set of A and B
// panels per L2).
#include <hip/hip_runtime.h>

#include <cstdio>

#include "lt_gemm_epilogue.h"
#include "lt_launch.h"

namespace ltk {

namespace bf {
constexpr int BK = 32;
constexpr int kStrideKC = 80;    // bytes per row of an [x][k] tile: 64 + 16 of padding

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;

// Geometry of one padded operand tile of BX rows/columns by 32 k (ragged-tile path).
template <int BX> struct Geo {
  static constexpr int kChunks = BX / 64;              // 16-byte chunks per lane and slice
  static constexpr int kStrideXC = BX * 2 + 32;        // bytes per row of a [k][x] tile
  static constexpr int kBytes = BX * kStrideKC;        // >= 32 * kStrideXC
};

template <int N> struct Chunks {
  uint4 g[N];
};

// (outer, inner) coordinates inside the tile of this lane's chunk number `it`.  KC: rows are x,
// 4 chunks of 8 k each; otherwise rows are k, BX/8 chunks of 8 x each.
template <int BX, bool KC>
__device__ __forceinline__ void chunk_pos(uint32_t it, uint32_t* outer, uint32_t* inner) {
  const uint32_t e = it * kGemmThreads + threadIdx.x;
  if (KC) {
    *outer = e >> 2;
    *inner = (e & 3u) * 8u;
  } else {
    *outer = e / (BX / 8);
    *inner = (e % (BX / 8)) * 8u;
  }
}

// Guarded fetch of 8 elements at (outer, inner .. inner+7); out-of-range elements read as zero.
__device__ __noinline__ uint4 fetch_guarded(const uint16_t* base, int64_t s_outer, uint32_t outer, uint32_t inner,
                                            uint32_t n_outer, uint32_t n_inner, bool aligned) {
  uint4 v = make_uint4(0, 0, 0, 0);
  if (outer >= n_outer || inner >= n_inner) return v;
  const uint16_t* src = base + (int64_t)outer * s_outer + inner;
  if (aligned && inner + 8u <= n_inner) return *(const uint4*)src;
  uint32_t w0 = 0, w1 = 0, w2 = 0, w3 = 0;
  if (inner + 0 < n_inner) w0 |= (uint32_t)src[0];
  if (inner + 1 < n_inner) w0 |= (uint32_t)src[1] << 16;
  if (inner + 2 < n_inner) w1 |= (uint32_t)src[2];
  if (inner + 3 < n_inner) w1 |= (uint32_t)src[3] << 16;
  if (inner + 4 < n_inner) w2 |= (uint32_t)src[4];
  if (inner + 5 < n_inner) w2 |= (uint32_t)src[5] << 16;
  if (inner + 6 < n_inner) w3 |= (uint32_t)src[6];
  if (inner + 7 < n_inner) w3 |= (uint32_t)src[7] << 16;
  return make_uint4(w0, w1, w2, w3);
}

// Global -> registers for the slice starting at k0, every access checked.
template <int BX, bool KC>
__device__ __forceinline__ Chunks<Geo<BX>::kChunks> fetch_checked(const uint16_t* base, int64_t s_x, int64_t s_k, uint32_t x0,
                                                                  uint32_t k0, uint32_t nx, uint32_t nk, bool aligned) {
  Chunks<Geo<BX>::kChunks> c;
#pragma unroll
  for (int it = 0; it < Geo<BX>::kChunks; ++it) {
    uint32_t o, i;
    chunk_pos<BX, KC>(it, &o, &i);
    c.g[it] = KC ? fetch_guarded(base, s_x, x0 + o, k0 + i, nx, nk, aligned)
                 : fetch_guarded(base, s_k, k0 + o, x0 + i, nk, nx, aligned);
  }
  return c;
}

template <int BX, bool KC>
__device__ __forceinline__ void stash(const Chunks<Geo<BX>::kChunks>& c, char* tile) {
#pragma unroll
  for (int it = 0; it < Geo<BX>::kChunks; ++it) {
    uint32_t o, i;
    chunk_pos<BX, KC>(it, &o, &i);
    *(uint4*)(tile + o * (KC ? kStrideKC : Geo<BX>::kStrideXC) + i * 2u) = c.g[it];
  }
}

// The MFMA fragment of a 32-row (or 32-column) block starting at x_blk for k16 step kk.
template <int BX, bool KC>
__device__ __forceinline__ v8bf fragment(const char* tile, uint32_t x_blk, uint32_t kk, uint32_t lane) {
  const uint32_t kb = kk * 16u + (lane >> 5) * 8u;   // first of this lane's 8 k
  if (KC) {
    return *(const v8bf*)(tile + (x_blk + (lane & 31u)) * kStrideKC + kb * 2u);
  } else {
    constexpr int S = Geo<BX>::kStrideXC;
    const uint32_t i16 = lane & 15u;
    const uint32_t xb = x_blk + ((lane & 31u) >> 4) * 16u;
    const char* p = tile + (kb + (i16 >> 2)) * S + (xb + 4u * (i16 & 3u)) * 2u;
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)p);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(p + 4 * S));
    v8s r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return __builtin_bit_cast(v8bf, r);
  }
}

// ---- whole tiles: global memory -> LDS without passing through registers -----------------------
// `global_load_lds_dwordx4`: every lane names its own 16 global bytes, the hardware writes them to
// LDS at a wave-uniform base + lane * 16 (checked with an in-bounds probe), so a wave instruction
// fills 1 KiB of consecutive LDS.  Tiles are therefore dense (no row padding), and bank conflicts
// of the fragment reads are avoided by a swizzle instead: the 16-byte chunk at (row, c) lives at
// position c ^ f(row) of its row.  The swizzle costs nothing in the loop: it is folded into each
// lane's global offset (which chunk it fetches for its LDS slot) and into the fragment addresses.
//   [x][k] tile (k contiguous in memory): rows of 64 bytes, f(x) = (x >> 2) & 3 -- the sixteen rows
//     that one cycle of a ds_read_b128 touches then cover all sixteen 16-byte bank groups;
//   [k][x] tile (x contiguous): rows of BX * 2 bytes, f(k) = (k & 3) << 2 for 256-byte rows
//     (((k >> 1) & 1) << 2 for 128-byte rows): the four k rows of a transposing read land in four
//     different 64-byte bank ranges.
template <int BX, bool KC> struct Dense {
  static constexpr uint32_t kBytes = BX * 64;            // BX x 32 bf16
  static constexpr uint32_t kInstr = BX / 64;            // wave instructions per slice (4 waves x 1 KiB each)
  static constexpr uint32_t kPerRow = BX / 8;            // chunks per k row of a [k][x] tile
  static constexpr uint32_t kRowsPer256 = 256 / (BX * 2) ? 256 / (BX * 2) : 1;   // [k][x] rows per 256 bytes
  __device__ static __forceinline__ uint32_t swz_k(uint32_t k) { return ((k / kRowsPer256) & (4u / kRowsPer256 - 1u)) << 2; }
  __device__ static __forceinline__ uint32_t swz_x(uint32_t x) { return (x >> 2) & 3u; }
};

// This lane's byte offset from the (wave-uniform) origin of an instruction's 64 rows (KC) or
// 256 / kPerRow k rows (otherwise): the same for every instruction and every slice.
template <int BX, bool KC>
__device__ __forceinline__ uint32_t dma_lane_offset(int64_t s_x, int64_t s_k) {
  typedef Dense<BX, KC> D;
  const uint32_t t = threadIdx.x;
  if (KC) {
    const uint32_t row = t >> 2, c = (t & 3u) ^ D::swz_x(row);
    return (uint32_t)((row * s_x + c * 8u) * 2);
  }
  const uint32_t k = t / D::kPerRow, xc = (t % D::kPerRow) ^ D::swz_k(k);
  return (uint32_t)((k * s_k + xc * 8u) * 2);
}

// One wave instruction of such a copy.  Written in assembly on purpose: the compiler orders every
// later LDS read behind every copy it knows to be in flight (and loses track of them around a
// loop's back edge), so a pipeline deeper than one slice needs copies it does not know about and
// waits that the code spells out (landed(), below).  M0 holds the LDS base of the instruction;
// nothing else in the loop uses it, and the interpreter's register indexing sets it afresh.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void copy_1k(const void* gptr, uint32_t lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" : : "s"(lds_base), "v"(gptr) : "memory", "m0");
}
#pragma clang diagnostic pop

// Wait until at most `outstanding` of this wave's copies are still in flight (they complete in
// order).  s_waitcnt immediate: vmcnt in bits 3:0 and 15:14, the other counters left alone.
template <uint32_t outstanding>
__device__ __forceinline__ void landed() {
  static_assert(outstanding < 64u, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((int)((outstanding & 15u) | ((outstanding >> 4) << 14) | 0x0f70u));
}

// Start the copy of the slice at k0 of the BX-wide panel at x0 into the tile at LDS address `tile`.
template <int BX, bool KC>
__device__ __forceinline__ void dma_tile(const uint16_t* base, int64_t s_x, int64_t s_k, uint32_t x0, uint32_t k0, uint32_t lane_off,
                                         uint32_t tile, uint32_t wave) {
  typedef Dense<BX, KC> D;
  constexpr uint32_t rows_per_instr = KC ? 64u : (uint32_t)kGemmThreads / D::kPerRow;
#pragma unroll
  for (uint32_t it = 0; it < D::kInstr; ++it) {
    const uint16_t* u = KC ? base + (int64_t)(x0 + it * rows_per_instr) * s_x + k0
                           : base + (int64_t)(k0 + it * rows_per_instr) * s_k + x0;
    copy_1k((const char*)u + lane_off, tile + (it * (uint32_t)kGemmThreads + wave * 64u) * 16u);
  }
}

// Two consecutive slices (ka, kb = ka + 32 unless clamped) at once, instruction by instruction.
// A row of an [x][k] slice is 64 bytes, half a cache line; fetched one slice per iteration, the
// second half comes a whole iteration's traffic later, misses the L1 again and costs a second
// request to L2 (measured: 1.8 times the L2 requests, the address unit stalled by the cache for
// 40 % of the kernel).  Back to back, the second access finds the line already on its way.
template <int BX, bool KC>
__device__ __forceinline__ void dma_tile2(const uint16_t* base, int64_t s_x, int64_t s_k, uint32_t x0, uint32_t ka, uint32_t kb,
                                          uint32_t lane_off, uint32_t tile_a, uint32_t tile_b, uint32_t wave) {
  typedef Dense<BX, KC> D;
  constexpr uint32_t rows_per_instr = KC ? 64u : (uint32_t)kGemmThreads / D::kPerRow;
#pragma unroll
  for (uint32_t it = 0; it < D::kInstr; ++it) {
    const uint16_t* ua = KC ? base + (int64_t)(x0 + it * rows_per_instr) * s_x + ka
                            : base + (int64_t)(ka + it * rows_per_instr) * s_k + x0;
    const uint16_t* ub = KC ? base + (int64_t)(x0 + it * rows_per_instr) * s_x + kb
                            : base + (int64_t)(kb + it * rows_per_instr) * s_k + x0;
    const uint32_t dst = (it * (uint32_t)kGemmThreads + wave * 64u) * 16u;
    copy_1k((const char*)ua + lane_off, tile_a + dst);
    copy_1k((const char*)ub + lane_off, tile_b + dst);
  }
}

// The MFMA fragment of a 32-row (or 32-column) block of a dense, swizzled tile.
template <int BX, bool KC>
__device__ __forceinline__ v8bf fragment_dense(const char* tile, uint32_t x_blk, uint32_t kk, uint32_t lane) {
  typedef Dense<BX, KC> D;
  if (KC) {
    const uint32_t row = x_blk + (lane & 31u), c = kk * 2u + (lane >> 5);
    return *(const v8bf*)(tile + row * 64u + ((c ^ D::swz_x(row)) << 4));
  } else {
    constexpr uint32_t S = BX * 2;
    const uint32_t i16 = lane & 15u;
    const uint32_t k = kk * 16u + (lane >> 5) * 8u + (i16 >> 2);
    const uint32_t col = (x_blk + ((lane & 31u) >> 4) * 16u + 4u * (i16 & 3u)) * 2u;   // byte column
    const char* p = tile + k * S + (((col >> 4) ^ D::swz_k(k)) << 4) + (col & 15u);
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)p);
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s_ptr)(p + 4 * S));   // k + 4: same swizzle
    v8s r;
    r[0] = lo[0]; r[1] = lo[1]; r[2] = lo[2]; r[3] = lo[3];
    r[4] = hi[0]; r[5] = hi[1]; r[6] = hi[2]; r[7] = hi[3];
    return __builtin_bit_cast(v8bf, r);
  }
}

// The same, and every LDS read of this wave has returned as well (lgkmcnt = 0).
template <uint32_t outstanding>
__device__ __forceinline__ void landed_and_read() {
  static_assert(outstanding < 64u, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt((int)((outstanding & 15u) | ((outstanding >> 4) << 14) | 0x0070u));
}

template <int BM, int BN> struct Smem {
  static constexpr size_t kStage = Geo<BM>::kBytes + Geo<BN>::kBytes;
  static constexpr size_t kStripBytes = (size_t)BM * (BN + kCPad) * sizeof(float);   // the whole tile
  static constexpr size_t kDense = 4 * (size_t)(BM + BN) * 64;                        // four dense stages
  static constexpr size_t kMax2 = kStage > kStripBytes ? kStage : kStripBytes;   // (ragged tiles: one padded stage)
  static constexpr size_t kBytes = kMax2 > kDense ? kMax2 : kDense;
};

template <int BM, int BN, bool AKC, bool BKC>
__global__ __launch_bounds__(kGemmThreads, 2) void lt_gemm_bf16_kernel(const GemmArgs a) {
  constexpr int MB = BM / 64, NB = BN / 64;   // 32 x 32 blocks per wave: rows, columns
  __shared__ __attribute__((aligned(16))) char smem[Smem<BM, BN>::kBytes];
  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t wave_m = wave >> 1, wave_n = wave & 1u;
  // tile number: remap so that each XCD (workgroup number mod 8) owns a contiguous range
  const uint32_t nt = gridDim.x;
  uint32_t t = blockIdx.x;
  if ((nt & 7u) == 0u) t = (blockIdx.x & 7u) * (nt >> 3) + (blockIdx.x >> 3);
  const uint32_t tile_m = (t / a.tiles_n) * BM, tile_n = (t % a.tiles_n) * BN;
  const uint32_t batch = blockIdx.y / a.splits, split = blockIdx.y % a.splits;
  const uint32_t b0 = batch / a.batch1, b1 = batch % a.batch1;
  const uint16_t* A = (const uint16_t*)a.a.ptr + (int64_t)b0 * a.a.s_b0 + (int64_t)b1 * a.a.s_b1;
  const uint16_t* B = (const uint16_t*)a.b.ptr + (int64_t)b0 * a.b.s_b0 + (int64_t)b1 * a.b.s_b1;
  // this workgroup's share of k: whole slices, split evenly
  const uint32_t slices = (a.k + BK - 1) / BK;
  const uint32_t per = (slices + a.splits - 1) / a.splits;
  const uint32_t k_begin = min(a.k, split * per * BK), k_end = min(a.k, (split + 1) * per * BK);
  const int64_t a_outer = AKC ? a.a.s_row : a.a.s_col, b_outer = BKC ? a.b.s_col : a.b.s_row;
  const bool a_al = (((uintptr_t)A) & 15u) == 0 && (a_outer % 8) == 0;
  const bool b_al = (((uintptr_t)B) & 15u) == 0 && (b_outer % 8) == 0;
  const bool a_in = a_al && tile_m + BM <= a.m, b_in = b_al && tile_n + BN <= a.n;

    constexpr uint32_t kStage = (uint32_t)Smem<BM, BN>::kStage;   // padded layout (ragged tiles): A tile then B tile
  v16f acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // fragments of one slice: every MFMA operand of this wave, both k16 steps
  struct Frags {
    v8bf a[BK / 16][MB], b[BK / 16][NB];
  };
  auto load_frags = [&](uint32_t stage) {
    const char* As = smem + stage * kStage;
    const char* Bs = As + Geo<BM>::kBytes;
    Frags f;
#pragma unroll
    for (uint32_t kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
      for (int i = 0; i < MB; ++i) f.a[kk][i] = fragment<BM, AKC>(As, wave_m * (BM / 2) + i * 32u, kk, lane);
#pragma unroll
      for (int j = 0; j < NB; ++j) f.b[kk][j] = fragment<BN, BKC>(Bs, wave_n * (BN / 2) + j * 32u, kk, lane);
    }
    return f;
  };
  auto mma = [&](const Frags& f) {
#pragma unroll
    for (uint32_t kk = 0; kk < BK / 16; ++kk)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[kk][i], f.b[kk][j], acc[i][j], 0, 0, 0);
  };
  const bool whole = a_in && b_in && ((k_end - k_begin) % BK) == 0u;
  if (k_begin < k_end && whole) {
    // Software pipeline over slices j = 0 .. n-1, four LDS stages: the MFMAs of slice j run from
    // fragment registers, the fragments of slice j+1 are read from the stage that holds it, and
    // later slices are on their way from global memory straight into their stages -- no
    // registers, no LDS write instructions, two iterations for a copy to land.  (Copies past the
    // end are clamped to the last slice: in bounds, unused.)
    constexpr uint32_t kDenseStage = Dense<BM, AKC>::kBytes + Dense<BN, BKC>::kBytes;
    constexpr uint32_t kPer = Dense<BM, AKC>::kInstr + Dense<BN, BKC>::kInstr;   // copy instructions per wave and slice
    static_assert(4 * kDenseStage <= Smem<BM, BN>::kBytes, "four dense stages fit the tile's LDS");
    const uint32_t n = (k_end - k_begin) / BK;
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    const uint32_t lds0 = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)smem;
    const uint32_t a_off = dma_lane_offset<BM, AKC>(a.a.s_row, a.a.s_col), b_off = dma_lane_offset<BN, BKC>(a.b.s_col, a.b.s_row);
#define LT_COPY(I, STAGE)                                                                                          \
  {                                                                                                               \
    const uint32_t kf = k_begin + min((uint32_t)(I), n - 1u) * BK;                                                \
    dma_tile<BM, AKC>(A, a.a.s_row, a.a.s_col, tile_m, kf, a_off, lds0 + (STAGE) * kDenseStage, wave_u);          \
    dma_tile<BN, BKC>(B, a.b.s_col, a.b.s_row, tile_n, kf, b_off, lds0 + (STAGE) * kDenseStage + Dense<BM, AKC>::kBytes, wave_u); \
  }
#define LT_COPY2(I0, S0, I1, S1)                                                                                   \
  {                                                                                                               \
    const uint32_t ka = k_begin + min((uint32_t)(I0), n - 1u) * BK, kb = k_begin + min((uint32_t)(I1), n - 1u) * BK; \
    dma_tile2<BM, AKC>(A, a.a.s_row, a.a.s_col, tile_m, ka, kb, a_off, lds0 + (S0) * kDenseStage,                  \
                       lds0 + (S1) * kDenseStage, wave_u);                                                        \
    dma_tile2<BN, BKC>(B, a.b.s_col, a.b.s_row, tile_n, ka, kb, b_off, lds0 + (S0) * kDenseStage + Dense<BM, AKC>::kBytes, \
                       lds0 + (S1) * kDenseStage + Dense<BM, AKC>::kBytes, wave_u);                               \
  }
    auto dense_frags = [&](uint32_t stage) {
      const char* As = smem + stage * kDenseStage;
      const char* Bs = As + Dense<BM, AKC>::kBytes;
      Frags f;
#pragma unroll
      for (uint32_t kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
        for (int i = 0; i < MB; ++i) f.a[kk][i] = fragment_dense<BM, AKC>(As, wave_m * (BM / 2) + i * 32u, kk, lane);
#pragma unroll
        for (int j = 0; j < NB; ++j) f.b[kk][j] = fragment_dense<BN, BKC>(Bs, wave_n * (BN / 2) + j * 32u, kk, lane);
      }
      return f;
    };
    if (n <= 3u) {
      // a short k (attention scores and contexts: k = 64) fits the stages at once: every slice is
      // copied, one wait, one barrier, and the slices are multiplied straight from LDS
      LT_COPY(0, 0);
      if (n > 1u) LT_COPY(1, 1);
      if (n > 2u) LT_COPY(2, 2);
      landed<0>();
      __syncthreads();
      for (uint32_t j = 0; j < n; ++j) {
        const Frags f = j == 0u ? dense_frags(0) : j == 1u ? dense_frags(1) : dense_frags(2);
        mma(f);
      }
    } else {
    // Four slices per trip: stage numbers and the two fragment sets are compile-time.
    //  * Some operand has k contiguous (64-byte rows per slice): copies go out in pairs, at odd
    //    slices: slices i+J+3 and i+J+4 into the stages of slices i+J-1 (long read) and i+J (read
    //    one iteration ago).  Waits and barriers are then needed at odd slices only: behind the
    //    barrier of slice j (odd) the pair copied two slices earlier -- slices j+1 and j+2, whose
    //    fragments are read in this iteration and the next -- has landed for every wave, and every
    //    wave's reads of the two stages about to be overwritten have returned (each wave waits for
    //    its own LDS reads before the barrier).
    //  * Otherwise (rows of a slice are whole cache lines) pairs gain nothing and their bursts cost
    //    a few percent: one copy per slice, slice i+J+4 into the stage of slice i+J behind the
    //    barrier of slice i+J, which also tells that slice i+J+1 has landed for every wave.
    // Past the end the body copies into stages nobody reads and reads fragments nobody uses; only
    // the MFMAs are guarded.
    constexpr bool kPairs = AKC || BKC;
    if (kPairs) {
      LT_COPY2(0, 0, 1, 1);
      LT_COPY2(2, 2, 3, 3);
      landed<2 * kPer>();   // slices 0 and 1
    } else {
      LT_COPY(0, 0);
      LT_COPY(1, 1);
      LT_COPY(2, 2);
      LT_COPY(3, 3);
      landed<3 * kPer>();   // slice 0
    }
    __syncthreads();
    Frags f0 = dense_frags(0), f1;
#define LT_SLICE(J, CUR, NEXT, GUARD)                                            \
  {                                                                            \
    if (kPairs) {                                                              \
      if ((J) & 1) {                                                           \
        landed_and_read<0>();                                                  \
        __syncthreads();                                                       \
        LT_COPY2(i + (J) + 3u, ((J) + 3) & 3, i + (J) + 4u, (J) & 3);          \
      }                                                                        \
    } else {                                                                   \
      landed_and_read<2 * kPer>();                                             \
      __syncthreads();                                                         \
      LT_COPY(i + (J) + 4u, (J) & 3);                                          \
    }                                                                          \
    NEXT = dense_frags(((J) + 1) & 3);                                         \
    if (!(GUARD) || i + (J) < n) mma(CUR);                                     \
  }
    uint32_t i = 0;
    for (; i + 4u <= n; i += 4u) {   // straight-line code: copies, LDS reads and MFMAs interleave
      LT_SLICE(0, f0, f1, false);
      LT_SLICE(1, f1, f0, false);
      LT_SLICE(2, f0, f1, false);
      LT_SLICE(3, f1, f0, false);
    }
    if (i < n) {                     // one to three slices left
      LT_SLICE(0, f0, f1, true);
      LT_SLICE(1, f1, f0, true);
      LT_SLICE(2, f0, f1, true);
    }
    landed<0>();   // nothing may still be on its way into LDS when the epilogue reuses it
    }
#undef LT_SLICE
#undef LT_COPY2
#undef LT_COPY
  } else if (k_begin < k_end) {
    // ragged or unaligned tile: every access checked, one slice at a time
#pragma unroll 1
    for (uint32_t k0 = k_begin; k0 < k_end; k0 += BK) {
      const Chunks<Geo<BM>::kChunks> ca = fetch_checked<BM, AKC>(A, a.a.s_row, a.a.s_col, tile_m, k0, a.m, k_end, a_al);
      const Chunks<Geo<BN>::kChunks> cb = fetch_checked<BN, BKC>(B, a.b.s_col, a.b.s_row, tile_n, k0, a.n, k_end, b_al);
      __syncthreads();
      stash<BM, AKC>(ca, smem);
      stash<BN, BKC>(cb, smem + Geo<BM>::kBytes);
      __syncthreads();
      const Frags f = load_frags(0);
      mma(f);
    }
  }

  // split-K: this workgroup's partial product goes to its own fp32 copy of the output, row major
  float* const raw = a.splits > 1u ? a.split_ws + (size_t)split * ((size_t)a.batch0 * a.batch1 * a.m * a.n) : nullptr;
  epilogue<BM, BN, MB, NB>(a, acc, (float*)smem, tile_m, tile_n, wave_m, wave_n, lane, batch, raw);
}

template <int BM, int BN>
static void launch_tile(const GemmArgs& a, dim3 grid, hipStream_t s) {
  const dim3 block(kGemmThreads);
  const bool akc = a.a.s_col == 1, bkc = a.b.s_row == 1;
  if (akc && bkc) LT_LAUNCH((lt_gemm_bf16_kernel<BM, BN, true, true>), grid, block, s, a);
  else if (akc) LT_LAUNCH((lt_gemm_bf16_kernel<BM, BN, true, false>), grid, block, s, a);
  else if (bkc) LT_LAUNCH((lt_gemm_bf16_kernel<BM, BN, false, true>), grid, block, s, a);
  else LT_LAUNCH((lt_gemm_bf16_kernel<BM, BN, false, false>), grid, block, s, a);
  char name[48];
  snprintf(name, sizeof(name), "lt_gemm_bf16_kernel<%d, %d, %s, %s>", BM, BN, akc ? "true" : "false", bkc ? "true" : "false");
  note_kernel(name);
}

}  // namespace bf

// a.tile_m, a.tile_n: rows and columns per workgroup tile (128 x 128, or 128 x 64 for narrow outputs).  The kernel is written for 128 or 256; only 128 is built: the
// 256 x 128 variant needs more than the 256 registers that two wavefronts per SIMD leave each, and
// measured slower both ways (two workgroups per compute unit with spills, or one with 385 registers).
// A 256 x 256 tile (128 x 128 per wave, one workgroup per compute unit, 512 registers) runs its main
// loop at twice the matrix-core utilisation of this one (54 % against 28 %), but the layer's shapes
// give it 128 to 512 tiles for 256 compute units and its epilogue has nothing to overlap with:
// 8192 x 4096 x 1024 gains 8 %, 8192 x 1024 x k loses.  Worth it only inside a persistent kernel
// that overlaps one tile's epilogue with the next tile's main loop.
hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  const uint32_t batch = a.batch0 * a.batch1;
  const uint32_t tiles = a.tiles_m * a.tiles_n;
  if (a.splits == 0u || (uint64_t)batch * a.splits > 65535u) return hipErrorInvalidValue;
  if (a.tile_m != 128u || (a.tile_n != 128u && a.tile_n != 64u)) return hipErrorInvalidValue;
  if (a.tiles_m != (a.m + a.tile_m - 1) / a.tile_m || a.tiles_n != (a.n + a.tile_n - 1) / a.tile_n) return hipErrorInvalidValue;
  const dim3 grid(tiles, batch * a.splits);
  if (a.tile_n == 64u) bf::launch_tile<128, 64>(a, grid, s);
  else bf::launch_tile<128, 128>(a, grid, s);
  return hipGetLastError();
}

}  // namespace ltk
