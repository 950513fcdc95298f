// fp32 contraction region: C = post(A * B) on the MFMA matrix cores (gfx950), fp32 operands and
// accumulation (bf16 operands: lt_gemm_bf16.hip).  Operands are addressed through element strides,
// so transposed, batched and head-split layouts need no copies.  The elementwise chain that
// consumes the product (bias, activation, residual, optimiser update, cast ...) is interpreted on
// the accumulator tile before anything is written: the product itself never travels to HBM unless
// asked for.
//
// Structure: workgroup tile 128 x 128 (or 64 x 64 for small problems so that more compute units
// get a tile), four wavefronts in a 2 x 2 arrangement, each owning a quarter as MFMA 32x32x2
// blocks.  K is walked in slices of 16 with register prefetch: the global loads of slice k+1 are
// issued before the MFMAs of slice k and written to the other LDS buffer afterwards.  Global
// loads are 16 bytes per lane along whichever dimension of the operand is contiguous; an operand
// whose contiguous dimension is k is transposed on its way into LDS.  A long k over few tiles is
// split over workgroups (partial products to a workspace, summed by a second launch).
#include <hip/hip_runtime.h>

#include "lt_gemm_epilogue.h"
#include "lt_launch.h"

namespace ltk {

// ---- operand staging --------------------------------------------------------------------------
// A "group" is what one lane fetches with one 16-byte load: G consecutive elements along the
// operand's contiguous dimension (4 fp32 or 8 bf16).  For element type T the raw group travels
// as uint4.
template <typename T> struct Elem;
template <> struct Elem<float> { static constexpr int G = 4; static constexpr int BK = 16; };

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

// LDS layout: tile[k][x] (x = m or n contiguous), row stride BX + 4 -> MFMA 32x32x2 reads one float
template <typename T, int BX> struct Tile;
template <int BX> struct Tile<float, BX> {
  static constexpr int BK = 16, STRIDE = BX + 4, ELEMS = BK * STRIDE;
};
// Number of 16-byte groups per lane and k-slice for an operand tile of BX x BK elements.
template <typename T, int BX> struct Groups {
  static constexpr int N = BX * Elem<T>::BK / Elem<T>::G / kGemmThreads;   // 128: 2, 64: 1
};

template <int N> struct GroupRegs {
  uint4 g[N];
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
      gr.g[it] = fetch_group<T>(base, s_x, x0 + x, k0 + kq * G, nx, nk, aligned);
    } else {
      const uint32_t k = e / (BX / G), xq = e % (BX / G);
      gr.g[it] = fetch_group<T>(base, s_k, k0 + k, x0 + xq * G, nk, nx, aligned);
    }
  }
}

template <int BX, bool KC>
__device__ __forceinline__ void stash_tile(const GroupRegs<Groups<float, BX>::N>& gr, float* tile) {
  const uint4* g = gr.g;
  constexpr int G = 4, BK = 16, STRIDE = Tile<float, BX>::STRIDE, NG = Groups<float, BX>::N;
  const uint32_t t = threadIdx.x;
#pragma unroll
  for (int it = 0; it < NG; ++it) {
    const uint32_t e = it * kGemmThreads + t;
    if (KC) {   // transposing: four scalar writes
      const uint32_t x = e / (BK / G), kq = e % (BK / G);
      tile[(kq * G + 0) * STRIDE + x] = __uint_as_float(g[it].x);
      tile[(kq * G + 1) * STRIDE + x] = __uint_as_float(g[it].y);
      tile[(kq * G + 2) * STRIDE + x] = __uint_as_float(g[it].z);
      tile[(kq * G + 3) * STRIDE + x] = __uint_as_float(g[it].w);
    } else {
      const uint32_t k = e / (BX / G), xq = e % (BX / G);
      *(uint4*)&tile[k * STRIDE + xq * G] = g[it];
    }
  }
}

// MFMAs of one k-slice.
template <int BM, int BN, int MB, int NB>
__device__ __forceinline__ void mma_slice(v16f (&acc)[MB][NB], const float* As, const float* Bs, uint32_t wave_m, uint32_t wave_n,
                                          uint32_t lane) {
  constexpr int SA = Tile<float, BM>::STRIDE, SB = Tile<float, BN>::STRIDE;
#pragma unroll
  for (int kk = 0; kk < 16; kk += 2) {
    const uint32_t kl = kk + (lane >> 5);
    float af[MB], bf[NB];
#pragma unroll
    for (int i = 0; i < MB; ++i) af[i] = As[kl * SA + wave_m * (MB * 32) + i * 32 + (lane & 31)];
#pragma unroll
    for (int j = 0; j < NB; ++j) bf[j] = Bs[kl * SB + wave_n * (NB * 32) + j * 32 + (lane & 31)];
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int j = 0; j < NB; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
  }
}

template <typename T, int BM, int BN> struct Smem {
  static constexpr size_t kOperands = 2 * (Tile<T, BM>::ELEMS + Tile<T, BN>::ELEMS) * sizeof(T);   // double buffered
  static constexpr size_t kC = (size_t)BM * (BN + kCPad) * sizeof(float);
  static constexpr size_t kBytes = kOperands > kC ? kOperands : kC;
};

// T: float.  AKC / BKC: the operand's contiguous dimension is k.
template <typename T, int BM, int BN, bool AKC, bool BKC>
__global__ __launch_bounds__(kGemmThreads) void lt_gemm_kernel(const GemmArgs a) {
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
  v16f acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  GroupRegs<Groups<T, BM>::N> ga;
  GroupRegs<Groups<T, BN>::N> gb;
  if (k_begin < k_end) {
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
      mma_slice<BM, BN, MB, NB>(acc, As(cur), Bs(cur), wave_m, wave_n, lane);
      if (more) {
        stash_tile<BM, AKC>(ga, As(cur ^ 1));
        stash_tile<BN, BKC>(gb, Bs(cur ^ 1));
      }
      __syncthreads();
      cur ^= 1;
    }
  }
  // split-K: this workgroup's partial product goes to its own fp32 copy of the output, row major
  float* const raw = a.splits > 1u ? a.split_ws + (size_t)split * ((size_t)a.batch0 * a.batch1 * a.m * a.n) : nullptr;
  epilogue<BM, BN, MB, NB>(a, acc, (float*)smem, tile_m, tile_n, wave_m, wave_n, lane, batch, raw);
}

template <typename T, int BM, int BN>
static void launch_variant(const GemmArgs& a, const dim3 grid, hipStream_t s) {
  const bool akc = a.a.s_col == 1, bkc = a.b.s_row == 1;
  if (akc && bkc) hipLaunchKernelGGL((lt_gemm_kernel<T, BM, BN, true, true>), grid, dim3(kGemmThreads), 0, s, a);
  else if (akc) hipLaunchKernelGGL((lt_gemm_kernel<T, BM, BN, true, false>), grid, dim3(kGemmThreads), 0, s, a);
  else if (bkc) hipLaunchKernelGGL((lt_gemm_kernel<T, BM, BN, false, true>), grid, dim3(kGemmThreads), 0, s, a);
  else hipLaunchKernelGGL((lt_gemm_kernel<T, BM, BN, false, false>), grid, dim3(kGemmThreads), 0, s, a);
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  // an operand must have unit stride along one of its two dimensions
  if ((a.a.s_col != 1 && a.a.s_row != 1) || (a.b.s_col != 1 && a.b.s_row != 1)) return hipErrorInvalidValue;
  if (a.in_dtype == kBF16) return launch_gemm_bf16(a, s);
  const uint32_t batch = a.batch0 * a.batch1;
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
