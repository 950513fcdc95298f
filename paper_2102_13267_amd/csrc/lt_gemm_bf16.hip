// bf16 contraction on the gfx950 matrix cores: C = post(A * B), fp32 accumulation.
//
// Workgroup tile BM x 128 (BM = 128 as built), k walked in slices of 32,
// four wavefronts in a 2 x 2 arrangement, each owning (BM/2) x 64 as blocks of
// v_mfma_f32_32x32x16_bf16.  What bounds this kernel is LDS bandwidth, not the matrix cores: every
// MFMA of a 64 x 64 wavefront tile needs a kilobyte of fragments from LDS, which at four SIMDs per
// compute unit is the whole LDS read rate; the 128 x 64 wavefront tile of BM = 256 needs a
// quarter less, and its A tile is shared by twice the work.  Two LDS stages of 30 KiB let two
// workgroups share a compute unit, so one's matrix instructions run under the other's loads,
// stores and barriers; the registers stay under the 256 that two wavefronts per SIMD allow.
//
// Operand staging.  An MFMA lane wants 8 consecutive k of one row (A) or column (B).
//  * k is the operand's contiguous dimension: global 16-byte loads land in LDS as [x][k] rows of
//    80 bytes (64 + 16 of padding: eight consecutive rows hit eight different 16-byte bank
//    groups) and a lane's fragment is one ds_read_b128;
//  * x (m or n) is the contiguous dimension: the tile is stored as it arrives, [k][x] rows padded
//    by 32 bytes, and the transpose happens in the LDS read: ds_read_b64_tr_b16 hands each lane of
//    a 16-lane group one column of a 4 x 16 sub-tile (lane i gets element i of each of the four
//    rows that lanes 4j .. 4j+3 point at), so two such reads give the 8 k values of one x.
// Either way global loads and LDS writes are 16 bytes per lane and nothing is transposed by
// scalar code.  The loop is software pipelined three deep (MFMAs of slice i from registers, LDS
// fragment reads of slice i+1, global loads and LDS writes of slice i+2), one barrier per slice.
//
// Epilogue: the accumulators leave the MFMA layout through LDS in strips of 64 rows; each strip is
// then walked in row-major 4-element quads by the interpreter (bias, activation, residual,
// optimiser update, cast ...), so the product itself never travels to HBM unless asked for.
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

#include "lt_gemm_epilogue.h"
#include "lt_launch.h"

namespace ltk {

namespace bf {
constexpr int BK = 32;
constexpr int kStrideKC = 80;    // bytes per row of an [x][k] tile: 64 + 16 of padding

typedef short v4s __attribute__((ext_vector_type(4)));
typedef short v8s __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) v4s* lds_v4s_ptr;

// Geometry of one operand tile of BX rows/columns by 32 k.
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

// The same for a tile and slice that are whole and 16-byte aligned.  A chunk's address is split
// into a wave-uniform part (tile origin, slice, chunk number: scalar registers) and this lane's
// byte offset inside a chunk row group, which is the same for every chunk and every slice: one
// vector register per operand instead of a 64-bit address per chunk.
template <int BX, bool KC>
__device__ __forceinline__ uint32_t lane_offset(int64_t s_x, int64_t s_k) {
  const uint32_t t = threadIdx.x;
  if (KC) return (uint32_t)(((t >> 2) * s_x + (t & 3u) * 8u) * 2);
  constexpr uint32_t per_row = BX / 8;
  return (uint32_t)(((t / per_row) * s_k + (t % per_row) * 8u) * 2);
}

template <int BX, bool KC>
__device__ __forceinline__ Chunks<Geo<BX>::kChunks> fetch_whole(const uint16_t* base, int64_t s_x, int64_t s_k, uint32_t x0,
                                                                uint32_t k0, uint32_t lane_off) {
  Chunks<Geo<BX>::kChunks> c;
  // rows advance by 64 (KC) or by 256 / (BX / 8) (otherwise) from one chunk to the next
  constexpr uint32_t rows_per_chunk = KC ? 64u : (uint32_t)kGemmThreads / (BX / 8);
#pragma unroll
  for (int it = 0; it < Geo<BX>::kChunks; ++it) {
    const uint16_t* u = KC ? base + (int64_t)(x0 + it * rows_per_chunk) * s_x + k0
                           : base + (int64_t)(k0 + it * rows_per_chunk) * s_k + x0;
    c.g[it] = *(const uint4*)((const char*)u + lane_off);
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

constexpr int kStripRows = 64;                       // epilogue strip: 32 rows of each wave row

template <int BM, int BN> struct Smem {
  static constexpr size_t kStage = Geo<BM>::kBytes + Geo<BN>::kBytes;
  static constexpr size_t kOperands = 2 * kStage;
  static constexpr size_t kStripBytes = (size_t)BM * (BN + kCPad) * sizeof(float);   // the whole tile
  static constexpr size_t kBytes = kOperands > kStripBytes ? kOperands : kStripBytes;
};

// Epilogue over the workgroup's BM x BN tile.  Strip p holds block row p of both wave rows:
// LDS row r is tile row (r / 32) * (BM / 2) + p * 32 + r % 32.
template <int BM, int BN, int MB, int NB>
__device__ __forceinline__ void epilogue_strips(const GemmArgs& a, const v16f (&acc)[MB][NB], float* Cs, uint32_t tile_m,
                                                uint32_t tile_n, uint32_t wave_m, uint32_t wave_n, uint32_t lane,
                                                uint32_t batch, float* raw) {
  constexpr int kCStride = BN + kCPad;
  const EwProg& p = a.post;
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t b0 = batch / a.batch1, b1 = batch % a.batch1;
  const int64_t base = (int64_t)b0 * a.o_b0 + (int64_t)b1 * a.o_b1;
  const uint32_t row_flat0 = (b0 * a.batch1 + b1) * a.m;   // first row of this batch in the flattened [rows, n] output
  // whole tile, whole aligned 4-vectors, at most four inputs and none of them strided: no bounds
  // checks, no divisions (row and column are known), loads of a quad issued together
  const bool fast = p.fast && p.full_vec_ok && p.n_in <= 4u && tile_m + BM <= a.m && tile_n + BN <= a.n;
  const bool plain = n_code == 0u && p.n_in == 0u && p.n_out == 1u && !p.out[0].scalar && p.out[0].slot == p.anchor_slot;
  // The strip loop stays rolled (one copy of the interpreter); the strip's accumulators are picked
  // with compile-time indices so that the accumulator array never has to live in memory.
#pragma unroll 1
  for (int s = 0; s < MB; ++s) {
    v16f strip[NB];
#pragma unroll
    for (int ss = 0; ss < MB; ++ss)
      if (ss == s) {
#pragma unroll
        for (int bn = 0; bn < NB; ++bn) strip[bn] = acc[ss][bn];
      }
    __syncthreads();   // the LDS bytes (operand tiles, or the previous strip) are dead now
#pragma unroll
    for (int bn = 0; bn < NB; ++bn)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const uint32_t row = wave_m * 32u + (r >> 2) * 8u + (lane >> 5) * 4u + (r & 3);
        const uint32_t col = wave_n * (BN / 2) + bn * 32u + (lane & 31u);
        Cs[row * kCStride + col] = strip[bn][r];
      }
    __syncthreads();
    if (raw) {
      // partial product of a split: plain fp32, dense [batch * m, n]
      const bool vec = (a.n % 4u) == 0u;
#pragma unroll 4
      for (uint32_t q = threadIdx.x; q < (uint32_t)(kStripRows * BN / kVec); q += kGemmThreads) {
        const uint32_t r = q / (BN / kVec), c = (q % (BN / kVec)) * kVec;
        const uint32_t row = tile_m + (r >> 5) * (BM / 2) + s * 32u + (r & 31u), col = tile_n + c;
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
    } else if (fast && plain) {
      // the product itself is the only output: convert and store, nothing to interpret
      const EwOut& o = p.out[0];
#pragma unroll 4
      for (uint32_t q = threadIdx.x; q < (uint32_t)(kStripRows * BN / kVec); q += kGemmThreads) {
        const uint32_t r = q / (BN / kVec), c = (q % (BN / kVec)) * kVec;
        const uint32_t row = tile_m + (r >> 5) * (BM / 2) + s * 32u + (r & 31u);
        const uint32_t i = (uint32_t)(base + (int64_t)row * a.o_row + tile_n + c);
        const float4 t = *(const float4*)&Cs[r * kCStride + c];
        Quad v;
        v.v[0] = t.x; v.v[1] = t.y; v.v[2] = t.z; v.v[3] = t.w;
        store_vec4<false>(o.ptr, o.dtype, 0, i, v);
      }
    } else if (fast) {
#pragma unroll 1
      for (uint32_t q = threadIdx.x; q < (uint32_t)(kStripRows * BN / kVec); q += kGemmThreads) {
        const uint32_t r = q / (BN / kVec), c = (q % (BN / kVec)) * kVec;
        const uint32_t row = tile_m + (r >> 5) * (BM / 2) + s * 32u + (r & 31u);
        const uint32_t i = (uint32_t)(base + (int64_t)row * a.o_row + tile_n + c);
        const Staged<4> st = fetch_inputs_at<4, false>(p, i, row_flat0 + row, tile_n + c);
        const float4 t = *(const float4*)&Cs[r * kCStride + c];
        Quad anchor;
        anchor.v[0] = t.x; anchor.v[1] = t.y; anchor.v[2] = t.z; anchor.v[3] = t.w;
        RF<16> f = place_inputs<16, 4, true, false>(rf_zero<16>(), p, st, kVec);
        f = rf_set<16>(f, p.anchor_slot, anchor);
        f = interp<16>(f, pr, n_code);
        store_outputs<16, true, false>(f, p, 0, i, kVec);
      }
    } else {
#pragma unroll 1
      for (uint32_t q = threadIdx.x; q < (uint32_t)(kStripRows * BN / kVec); q += kGemmThreads) {
        const uint32_t r = q / (BN / kVec), c = (q % (BN / kVec)) * kVec;
        const uint32_t row = tile_m + (r >> 5) * (BM / 2) + s * 32u + (r & 31u), col = tile_n + c;
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
  }
}

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

  // LDS: two stages, each the A tile then the B tile
  constexpr uint32_t kStage = (uint32_t)Smem<BM, BN>::kStage;
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
    // Software pipeline over slices i = 0 .. n-1, three things in flight at once: the MFMAs of
    // slice i run from fragment registers; the fragments of slice i+1 are read from the LDS stage
    // that holds it; slice i+2 travels global -> registers -> the stage slice i has just left.
    // So no MFMA ever waits for an LDS read of its own iteration, and one barrier per slice
    // orders the stage hand-over.  (Fetches past the end are clamped to the last slice: in
    // bounds, unused.)
    const uint32_t n = (k_end - k_begin) / BK;
    const uint32_t a_off = lane_offset<BM, AKC>(a.a.s_row, a.a.s_col), b_off = lane_offset<BN, BKC>(a.b.s_col, a.b.s_row);
#define LT_FETCH(I)                                                                                       \
  {                                                                                                      \
    const uint32_t kf = k_begin + min((uint32_t)(I), n - 1u) * BK;                                       \
    ca = fetch_whole<BM, AKC>(A, a.a.s_row, a.a.s_col, tile_m, kf, a_off);                               \
    cb = fetch_whole<BN, BKC>(B, a.b.s_col, a.b.s_row, tile_n, kf, b_off);                               \
  }
#define LT_STASH(STAGE)                                                    \
  {                                                                       \
    stash<BM, AKC>(ca, smem + (STAGE) * kStage);                          \
    stash<BN, BKC>(cb, smem + (STAGE) * kStage + Geo<BM>::kBytes);        \
  }
    Chunks<Geo<BM>::kChunks> ca;
    Chunks<Geo<BN>::kChunks> cb;
    LT_FETCH(0);
    LT_STASH(0);
    LT_FETCH(1);
    LT_STASH(1);
    LT_FETCH(2);
    __syncthreads();
    Frags f0 = load_frags(0), f1;
    __syncthreads();   // nobody overwrites stage 0 before everybody has read slice 0 from it
    // Two slices per trip so that the two fragment sets swap roles without register copies.  The
    // body is branch free: past the end it reads fragments nobody uses and writes a stage nobody
    // reads (all inside the workgroup's own LDS).
    uint32_t i = 0;
    for (; i + 1u < n; i += 2u) {
      f1 = load_frags(1);
      mma(f0);
      LT_STASH(0);
      LT_FETCH(i + 3u);
      __syncthreads();
      f0 = load_frags(0);
      mma(f1);
      LT_STASH(1);
      LT_FETCH(i + 4u);
      __syncthreads();
    }
    if (i < n) mma(f0);   // odd number of slices: the last one is already in registers
#undef LT_FETCH
#undef LT_STASH
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
  if (akc && bkc) hipLaunchKernelGGL((lt_gemm_bf16_kernel<BM, BN, true, true>), grid, block, 0, s, a);
  else if (akc) hipLaunchKernelGGL((lt_gemm_bf16_kernel<BM, BN, true, false>), grid, block, 0, s, a);
  else if (bkc) hipLaunchKernelGGL((lt_gemm_bf16_kernel<BM, BN, false, true>), grid, block, 0, s, a);
  else hipLaunchKernelGGL((lt_gemm_bf16_kernel<BM, BN, false, false>), grid, block, 0, s, a);
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
