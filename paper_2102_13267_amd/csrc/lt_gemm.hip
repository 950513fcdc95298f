// Contraction region: C = post(A * B) on the MFMA matrix cores (gfx950), fp32 or bf16 operands,
// fp32 accumulation.  Operands are addressed through element strides, so transposed, batched and
// head-split layouts need no copies.  The elementwise chain that consumes the product (bias,
// activation, residual, optimiser update, cast ...) is interpreted on the accumulator tile in
// registers before anything is written: the product itself never travels to HBM unless asked for.
//
// Workgroup tile 128 x 128, four wavefronts in a 2 x 2 arrangement, each owning 64 x 64 as 2 x 2
// MFMA 32x32 blocks.  K is staged through LDS in slices of 16 (fp32) or 32 (bf16).
#include <hip/hip_runtime.h>

#include "lt_interp.h"
#include "lt_launch.h"

namespace ltk {

constexpr int kBM = 128, kBN = 128;
constexpr int kGemmThreads = 256;

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

// One accumulator quad = four consecutive rows of one column (the MFMA 32x32 result layout).
// Runs the post program for it.
__device__ __forceinline__ void post_quad(const EwProg& p, const ProgRegs pr, Quad acc, uint32_t row0, uint32_t col,
                                          uint32_t rows_valid, uint64_t out_base_row, uint32_t n) {
  // flat index of element e of the quad in the [rows, n] output space: i0 + e*n
  const uint64_t i0 = (out_base_row + row0) * (uint64_t)n + col;
  RF<16> f = rf_zero<16>();
  const uint32_t n_in = p.n_in;
#pragma unroll
  for (int k = 0; k < kMaxIn; ++k) {
    Quad q = splat(0.0f);
    if ((uint32_t)k < n_in) {
      const EwIn& in = p.in[k];
      if (in.mode == kScalar) {
        q = splat(load_elem(in.ptr, in.dtype, 0));
      } else if (in.mode == kRowVec) {
        q = splat(load_elem(in.ptr, in.dtype, col));
      } else {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
          if ((uint32_t)e < rows_valid) {
            const uint64_t i = i0 + (uint64_t)e * n;
            const uint64_t off = in.mode == kFull ? i : in.mode == kColVec ? out_base_row + row0 + e : strided_index(p, in, i);
            q.v[e] = load_elem(in.ptr, in.dtype, off);
          }
        }
      }
    }
#pragma unroll
    for (int v = 0; v < kVec; ++v) f.e[v][k] = q.v[v];
  }
  f = rf_set<16>(f, p.anchor_slot, acc);
  f = interp<16>(f, pr, p.n_code);
  const uint32_t n_out = p.n_out;
#pragma unroll
  for (int o = 0; o < kMaxOut; ++o) {
    if ((uint32_t)o < n_out) {
      const EwOut& out = p.out[o];
      const Quad q = rf_get<16>(f, out.slot);
#pragma unroll
      for (int e = 0; e < kVec; ++e)
        if ((uint32_t)e < rows_valid) store_elem(out.ptr, out.dtype, i0 + (uint64_t)e * n, q.v[e]);
    }
  }
}

__device__ __forceinline__ void epilogue(const GemmArgs& a, const v16f (&acc)[2][2], uint32_t tile_m, uint32_t tile_n,
                                         uint32_t wave_m, uint32_t wave_n, uint32_t lane, uint32_t batch) {
  const uint64_t base_row = (uint64_t)batch * a.m;
  const ProgRegs pr = load_prog_regs(a.post);
#pragma unroll
  for (int bm = 0; bm < 2; ++bm) {
#pragma unroll
    for (int bn = 0; bn < 2; ++bn) {
      const uint32_t col = tile_n + wave_n * 64 + bn * 32 + (lane & 31);
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const uint32_t row0 = tile_m + wave_m * 64 + bm * 32 + g * 8 + (lane >> 5) * 4;
        if (col < a.n && row0 < a.m) {
          const uint32_t rv = min(4u, a.m - row0);
          Quad q;
#pragma unroll
          for (int e = 0; e < kVec; ++e) q.v[e] = acc[bm][bn][g * 4 + e];
          post_quad(a.post, pr, q, row0, col, rv, base_row, a.n);
        }
      }
    }
  }
}

// ---- fp32: v_mfma_f32_32x32x2_f32; LDS holds A as [k][m] and B as [k][n] ----------------------------
constexpr int kBK32 = 16;
constexpr int kPad32 = 4;

__global__ __launch_bounds__(kGemmThreads) void lt_gemm_f32_kernel(const GemmArgs a) {
  __shared__ float As[kBK32][kBM + kPad32];
  __shared__ float Bs[kBK32][kBN + kPad32];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t wave_m = wave >> 1, wave_n = wave & 1;
  const uint32_t tile_m = blockIdx.y * kBM, tile_n = blockIdx.x * kBN, batch = blockIdx.z;
  const float* A = (const float*)a.a.ptr + (int64_t)batch * a.a.s_b0;
  const float* B = (const float*)a.b.ptr + (int64_t)batch * a.b.s_b0;
  v16f acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  for (uint32_t k0 = 0; k0 < a.k; k0 += kBK32) {
    // stage A[tile_m .. +128][k0 .. +16] and B[k0 .. +16][tile_n .. +128]; 2048 elements each,
    // 8 per thread; the thread's fast index follows the operand's unit stride for coalescing
#pragma unroll
    for (int it = 0; it < 8; ++it) {
      const uint32_t e = it * kGemmThreads + tid;
      uint32_t m, k;
      if (a.a.s_col == 1) { k = e % kBK32; m = e / kBK32; } else { m = e % kBM; k = e / kBM; }
      const uint32_t gm = tile_m + m, gk = k0 + k;
      As[k][m] = (gm < a.m && gk < a.k) ? A[(int64_t)gm * a.a.s_row + (int64_t)gk * a.a.s_col] : 0.0f;
      uint32_t n, kb;
      if (a.b.s_col == 1) { n = e % kBN; kb = e / kBN; } else { kb = e % kBK32; n = e / kBK32; }
      const uint32_t gn = tile_n + n, gkb = k0 + kb;
      Bs[kb][n] = (gn < a.n && gkb < a.k) ? B[(int64_t)gkb * a.b.s_row + (int64_t)gn * a.b.s_col] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kBK32; kk += 2) {
      const uint32_t kl = kk + (lane >> 5);
      float af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) af[i] = As[kl][wave_m * 64 + i * 32 + (lane & 31)];
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[j] = Bs[kl][wave_n * 64 + j * 32 + (lane & 31)];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  epilogue(a, acc, tile_m, tile_n, wave_m, wave_n, lane, batch);
}

// ---- bf16: v_mfma_f32_32x32x16_bf16; LDS holds A as [m][k] and B as [n][k] ---------------------------
constexpr int kBK16 = 32;
constexpr int kPad16 = 8;

__global__ __launch_bounds__(kGemmThreads) void lt_gemm_bf16_kernel(const GemmArgs a) {
  __shared__ __attribute__((aligned(16))) uint16_t As[kBM][kBK16 + kPad16];
  __shared__ __attribute__((aligned(16))) uint16_t Bs[kBN][kBK16 + kPad16];
  const uint32_t tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const uint32_t wave_m = wave >> 1, wave_n = wave & 1;
  const uint32_t tile_m = blockIdx.y * kBM, tile_n = blockIdx.x * kBN, batch = blockIdx.z;
  const uint16_t* A = (const uint16_t*)a.a.ptr + (int64_t)batch * a.a.s_b0;
  const uint16_t* B = (const uint16_t*)a.b.ptr + (int64_t)batch * a.b.s_b0;
  v16f acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // 128 x 32 elements per operand and slice = 512 groups of 8; two groups per thread
  const bool a_k_contig = a.a.s_col == 1, b_k_contig = a.b.s_row == 1;
  const bool a_vec = a_k_contig ? ((a.a.s_row % 8) == 0 && (a.k % 8) == 0) : ((a.a.s_col % 8) == 0 && (a.m % 8) == 0);
  const bool b_vec = b_k_contig ? ((a.b.s_col % 8) == 0 && (a.k % 8) == 0) : ((a.b.s_row % 8) == 0 && (a.n % 8) == 0);
  const bool a_al = (((uintptr_t)A) & 15u) == 0, b_al = (((uintptr_t)B) & 15u) == 0;
  for (uint32_t k0 = 0; k0 < a.k; k0 += kBK16) {
#pragma unroll
    for (int it = 0; it < 2; ++it) {
      const uint32_t g = it * kGemmThreads + tid;
      // ---- A
      if (a_k_contig) {
        const uint32_t m = g >> 2, k = (g & 3) * 8;
        const uint32_t gm = tile_m + m, gk = k0 + k;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (gm < a.m && gk < a.k) {
          const uint16_t* src = A + (int64_t)gm * a.a.s_row + gk;
          if (a_vec && a_al) v = *(const uint4*)src;
          else {
            uint16_t t[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = (gk + j < a.k) ? src[j] : (uint16_t)0;
            v = make_uint4(t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16));
          }
        }
        *(uint4*)&As[m][k] = v;
      } else {
        const uint32_t k = g >> 4, m = (g & 15) * 8;
        const uint32_t gm = tile_m + m, gk = k0 + k;
        uint16_t t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = 0;
        if (gk < a.k && gm < a.m) {
          const uint16_t* src = A + (int64_t)gk * a.a.s_col + gm;
          if (a_vec && a_al) {
            const uint4 v = *(const uint4*)src;
            t[0] = v.x & 0xffff; t[1] = v.x >> 16; t[2] = v.y & 0xffff; t[3] = v.y >> 16;
            t[4] = v.z & 0xffff; t[5] = v.z >> 16; t[6] = v.w & 0xffff; t[7] = v.w >> 16;
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = (gm + j < a.m) ? src[j] : (uint16_t)0;
          }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) As[m + j][k] = t[j];
      }
      // ---- B
      if (b_k_contig) {
        const uint32_t n = g >> 2, k = (g & 3) * 8;
        const uint32_t gn = tile_n + n, gk = k0 + k;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (gn < a.n && gk < a.k) {
          const uint16_t* src = B + (int64_t)gn * a.b.s_col + gk;
          if (b_vec && b_al) v = *(const uint4*)src;
          else {
            uint16_t t[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = (gk + j < a.k) ? src[j] : (uint16_t)0;
            v = make_uint4(t[0] | (t[1] << 16), t[2] | (t[3] << 16), t[4] | (t[5] << 16), t[6] | (t[7] << 16));
          }
        }
        *(uint4*)&Bs[n][k] = v;
      } else {
        const uint32_t k = g >> 4, n = (g & 15) * 8;
        const uint32_t gn = tile_n + n, gk = k0 + k;
        uint16_t t[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) t[j] = 0;
        if (gk < a.k && gn < a.n) {
          const uint16_t* src = B + (int64_t)gk * a.b.s_row + gn;
          if (b_vec && b_al) {
            const uint4 v = *(const uint4*)src;
            t[0] = v.x & 0xffff; t[1] = v.x >> 16; t[2] = v.y & 0xffff; t[3] = v.y >> 16;
            t[4] = v.z & 0xffff; t[5] = v.z >> 16; t[6] = v.w & 0xffff; t[7] = v.w >> 16;
          } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) t[j] = (gn + j < a.n) ? src[j] : (uint16_t)0;
          }
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) Bs[n + j][k] = t[j];
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < kBK16; kk += 16) {
      const uint32_t kl = kk + (lane >> 5) * 8;
      v8bf af[2], bf[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) af[i] = *(const v8bf*)&As[wave_m * 64 + i * 32 + (lane & 31)][kl];
#pragma unroll
      for (int j = 0; j < 2; ++j) bf[j] = *(const v8bf*)&Bs[wave_n * 64 + j * 32 + (lane & 31)][kl];
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    __syncthreads();
  }
  epilogue(a, acc, tile_m, tile_n, wave_m, wave_n, lane, batch);
}

hipError_t launch_gemm(const GemmArgs& a, hipStream_t s) {
  const dim3 grid((a.n + kBN - 1) / kBN, (a.m + kBM - 1) / kBM, a.batch0 * a.batch1);
  if (grid.y > 65535u || grid.z > 65535u) return hipErrorInvalidValue;
  if (a.in_dtype == kBF16) hipLaunchKernelGGL(lt_gemm_bf16_kernel, grid, dim3(kGemmThreads), 0, s, a);
  else hipLaunchKernelGGL(lt_gemm_f32_kernel, grid, dim3(kGemmThreads), 0, s, a);
  return hipGetLastError();
}

}  // namespace ltk
