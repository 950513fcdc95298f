// Elementwise fused region: one coalesced HBM pass; the whole chain is interpreted in registers.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "lt_interp.h"
#include "lt_launch.h"

namespace ltk {

constexpr int kBlock = 256;
// ---- elementwise region: one coalesced pass, 16 bytes per lane and input ------------------
// A workgroup walks tiles of kBlock * kVec = 1024 consecutive elements with a grid stride.  The
// tile base is wave-uniform (scalar registers); lanes differ only by a constant 32-bit offset.
template <int NS, int MAXIN, bool FAST, bool F32>
__global__ __launch_bounds__(kBlock) void lt_ew_kernel(const EwArgs a) {
  const EwProg& p = a.prog;
  const uint64_t n = p.n;
  constexpr uint64_t kTile = (uint64_t)kBlock * kVec;
  const uint64_t ntiles = (n + kTile - 1) / kTile;
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t lane = threadIdx.x * kVec;
  // (Prefetching the next tile's inputs during interpretation was measured and lost to the
  // occupancy it costs: 4 resident waves per SIMD hide HBM latency better than 3 pipelined ones.)
  for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint64_t base = tile * kTile;
    const uint64_t left = n - base;                       // >= 1
    if ((uint64_t)lane >= left) continue;
    const uint32_t nvalid = left - lane >= (uint64_t)kVec ? (uint32_t)kVec : (uint32_t)(left - lane);
    RF<NS> f = load_inputs<NS, MAXIN, FAST, F32>(rf_zero<NS>(), p, base, lane, nvalid);
    f = interp<NS>(f, pr, n_code);
    store_outputs<NS, FAST, F32>(f, p, base, lane, nvalid);
  }
}

// ---- streamed elementwise region --------------------------------------------------------------
// For fp32 programs of at most eight slots whose inputs are whole 4-vectors addressed like the
// output, plus at most two device scalars (a clipping factor, say).  Which input is which is
// sorted out on the host (EwStreamArgs), so that the kernel's loads are unconditional: a workgroup
// takes two tiles per trip, the NV vector inputs of both are fetched back to back, and the
// interpreter runs once for both (register file = 8 slots x 2).  A program with fewer than NV
// vector inputs loads one of them again (same slot, same data).  Tiles without a partner -- an odd
// one, a last one that not every lane takes part in -- go through the same code with both halves
// on the same tile: they load the same values before either stores, and store the same results.
struct EwStreamArgs {
  EwProg prog;
  uint32_t vin[4];    // input numbers of the vector inputs (padded with the first)
  uint32_t sin[2];    // input numbers of the device scalars
  uint32_t n_sin, pad;
  uint32_t vrow[4];   // bf16 kernel: 1 = vector input j is a row vector (indexed by column), 0 = a full tensor
};

// NT: non-temporal loads and stores, for regions larger than the last-level cache (what they read
// is not there and what they write will not be when it is needed): 5.6 -> 6.0 TB/s on 1 GiB operands.
template <int NV, bool NT>
__global__ __launch_bounds__(kBlock) void lt_ew_stream_kernel(const EwStreamArgs a) {
  const EwProg& p = a.prog;
  const uint64_t n = p.n;
  constexpr uint64_t kTile = (uint64_t)kBlock * kVec;
  const uint64_t ntiles = (n + kTile - 1) / kTile;
  const uint64_t npairs = (n / kTile) / 2;            // pairs of tiles that every lane takes part in
  const uint64_t ntrips = npairs + (ntiles - 2 * npairs);
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t lane = threadIdx.x * kVec;
  const char* vp[NV];
  uint32_t vslot[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    vslot[j] = a.vin[j];
    vp[j] = (const char*)p.in[vslot[j]].ptr;
  }
  float sval[2] = {0.0f, 0.0f};
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if ((uint32_t)j < a.n_sin) sval[j] = *(const float*)p.in[a.sin[j]].ptr;
  for (uint64_t trip = blockIdx.x; trip < ntrips; trip += gridDim.x) {
    const bool pair = trip < npairs;
    const uint64_t t0 = pair ? 2 * trip : npairs + trip, t1 = pair ? t0 + 1 : t0;
    const uint64_t base0 = t0 * kTile, base1 = t1 * kTile;
    if ((uint64_t)lane >= n - base0) continue;   // (only in the last tile, which is its own partner)
    RawVec v0[NV], v1[NV];
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const RawVec* s0 = (const RawVec*)(vp[j] + (base0 + lane) * 4u);
      const RawVec* s1 = (const RawVec*)(vp[j] + (base1 + lane) * 4u);
      v0[j] = NT ? __builtin_nontemporal_load(s0) : *s0;
      v1[j] = NT ? __builtin_nontemporal_load(s1) : *s1;
    }
    RF<16> f = rf_zero<16>();
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      Quad q;
      q.v[0] = v0[j].x; q.v[1] = v0[j].y; q.v[2] = v0[j].z; q.v[3] = v0[j].w;
      f = rf_set<16>(f, vslot[j], q);
      q.v[0] = v1[j].x; q.v[1] = v1[j].y; q.v[2] = v1[j].z; q.v[3] = v1[j].w;
      f = rf_set<16>(f, vslot[j] + 8u, q);
    }
    for (uint32_t j = 0; j < a.n_sin; ++j) {
      const Quad q = splat(j == 0u ? sval[0] : sval[1]);
      f = rf_set<16>(f, a.sin[j], q);
      f = rf_set<16>(f, a.sin[j] + 8u, q);
    }
    f = interp<16, 2>(f, pr, n_code);
    store_outputs<16, true, true, 0, NT>(f, p, base0, lane, kVec);
    store_outputs<16, true, true, 8, NT>(f, p, base1, lane, kVec);
  }
}

// The same for programs whose plain inputs are all bf16 (outputs of any type): a lane takes 8
// consecutive elements -- one 16-byte load per input, one 16-byte store per bf16 output -- which
// are the two 4-vectors of one interpreter dispatch; a tile is 2048 elements.  An interpreted
// wave retires an instruction every 10 to 12 cycles (scalar decode, branches, relative register
// addressing), so what bounds this kernel is instructions per tile divided by waves per SIMD, not
// memory latency: a 134 MB multiply ran at 2.6 TB/s with one short-lived wave per tile (every
// wave paid the set-up of the program's scalars and pointers, and padded input lists were
// loaded and converted twice).  Hence: NV is the exact number of vector inputs; a workgroup walks
// its tiles with a grid stride and asks for the next tile's inputs as soon as this tile's are in
// the register file, so the loads fly while the program is interpreted; 8 values of an output
// leave in one store.
template <int NV>
__global__ __launch_bounds__(kBlock, 4) void lt_ew_stream_bf16_kernel(const EwStreamArgs a) {
  const EwProg& p = a.prog;
  const uint64_t n = p.n;   // a multiple of 8: a lane is either wholly inside or wholly outside
  constexpr uint64_t kTile = (uint64_t)kBlock * 2 * kVec;
  const uint64_t ntiles = (n + kTile - 1) / kTile;
  uint64_t tile = blockIdx.x;
  if (tile >= ntiles) return;
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t lane = threadIdx.x * 2 * kVec;
  const char* vp[NV];
  uint32_t vslot[NV];
  bool vrow[NV];
#pragma unroll
  for (int j = 0; j < NV; ++j) {
    vslot[j] = a.vin[j];
    vp[j] = (const char*)p.in[vslot[j]].ptr;
    vrow[j] = a.vrow[j] != 0u;
  }
  float sval[2] = {0.0f, 0.0f};
#pragma unroll
  for (int j = 0; j < 2; ++j)
    if ((uint32_t)j < a.n_sin) sval[j] = *(const float*)p.in[a.sin[j]].ptr;
  typedef uint32_t U32x4 __attribute__((ext_vector_type(4)));
  // a row vector (a bias) is read at the column of the lane's first element: the host takes this
  // kernel only when rows are whole 8-element groups, so the 8 columns are consecutive.  The
  // column moves on by the grid stride modulo the row length, without a division per tile.
  const uint32_t cols = p.cols;
  const uint32_t col_step = (uint32_t)(((uint64_t)gridDim.x * kTile) % cols);
  uint32_t col = (uint32_t)((tile * kTile + lane) % cols);
  U32x4 v[NV];
  bool live = (uint64_t)lane < n - tile * kTile;
#pragma unroll
  for (int j = 0; j < NV; ++j) v[j] = live ? *(const U32x4*)(vp[j] + (vrow[j] ? (uint64_t)col : tile * kTile + lane) * 2u) : U32x4{0u, 0u, 0u, 0u};
  for (;;) {
    RF<16> f = rf_zero<16>();
#pragma unroll
    for (int j = 0; j < NV; ++j) {
      const U32x4 w = v[j];
      Quad q;
      q.v[0] = __uint_as_float(w.x << 16); q.v[1] = __uint_as_float(w.x & 0xffff0000u);
      q.v[2] = __uint_as_float(w.y << 16); q.v[3] = __uint_as_float(w.y & 0xffff0000u);
      f = rf_set<16>(f, vslot[j], q);
      q.v[0] = __uint_as_float(w.z << 16); q.v[1] = __uint_as_float(w.z & 0xffff0000u);
      q.v[2] = __uint_as_float(w.w << 16); q.v[3] = __uint_as_float(w.w & 0xffff0000u);
      f = rf_set<16>(f, vslot[j] + 8u, q);
    }
    for (uint32_t j = 0; j < a.n_sin; ++j) {
      const Quad q = splat(j == 0u ? sval[0] : sval[1]);
      f = rf_set<16>(f, a.sin[j], q);
      f = rf_set<16>(f, a.sin[j] + 8u, q);
    }
    // this tile's inputs are in the register file: ask for the next tile's.  A program that
    // updates an input in place is safe: tiles are disjoint and a lane stores where it loaded.
    const uint64_t cur = tile * kTile;
    const bool cur_live = live;
    tile += gridDim.x;
    const bool more = tile < ntiles;
    if (more) {
      live = (uint64_t)lane < n - tile * kTile;
      col += col_step;
      col = col >= cols ? col - cols : col;
#pragma unroll
      for (int j = 0; j < NV; ++j) v[j] = live ? *(const U32x4*)(vp[j] + (vrow[j] ? (uint64_t)col : tile * kTile + lane) * 2u) : U32x4{0u, 0u, 0u, 0u};
    }
    f = interp<16, 2>(f, pr, n_code);
    if (cur_live) {
#pragma unroll
      for (int o = 0; o < kMaxOut; ++o) {
        if ((uint32_t)o < p.n_out) {
          const EwOut& out = p.out[o];
          const Quad q0 = rf_get<16>(f, out.slot), q1 = rf_get<16>(f, out.slot + 8u);
          if (out.scalar) {
            if (cur + lane == 0) store_elem<false>(out.ptr, out.dtype, 0, q0.v[0]);
          } else if (out.dtype == kBF16) {
            const U32x4 u = {f32_to_bf16_pair(q0.v[0], q0.v[1]), f32_to_bf16_pair(q0.v[2], q0.v[3]),
                             f32_to_bf16_pair(q1.v[0], q1.v[1]), f32_to_bf16_pair(q1.v[2], q1.v[3])};
            *(U32x4*)((char*)out.ptr + (cur + lane) * 2u) = u;
          } else {
            store_vec4<false>(out.ptr, out.dtype, cur, lane, q0);
            store_vec4<false>(out.ptr, out.dtype, cur, lane + (uint32_t)kVec, q1);
          }
        }
      }
    }
    if (!more) break;
  }
}

// Host side: fill in EwStreamArgs if the program qualifies.
// vec_dtype: element type the vector inputs must have (kF32: everything fp32; kBF16: bf16 vector
// inputs, fp32 device scalars, outputs of any type, n a multiple of 8).
static bool make_stream_args(const EwProg& p, uint32_t vec_dtype, EwStreamArgs* out) {
  if (!p.fast || p.n_slots > 8u || p.n_in == 0u) return false;
  if (vec_dtype == kF32 ? !p.all_f32 : (p.n % 8u) != 0u) return false;
  uint32_t nv = 0, ns = 0;
  for (uint32_t k = 0; k < p.n_in; ++k) {
    const EwIn& in = p.in[k];
    if (in.fetch == kFetchVec4 && in.mode == kFull && in.dtype == vec_dtype) {
      if (nv == 4u) return false;
      out->vrow[nv] = 0u;
      out->vin[nv++] = k;
    } else if (vec_dtype == kBF16 && in.fetch == kFetchVec4 && in.mode == kRowVec && in.dtype == kBF16 && (p.cols % 8u) == 0u &&
               ((uintptr_t)in.ptr & 15u) == 0u) {
      if (nv == 4u) return false;   // (8 consecutive columns of a row vector: one aligned 16-byte load)
      out->vrow[nv] = 1u;
      out->vin[nv++] = k;
    } else if (in.fetch == kFetchBcast && in.mode == kScalar && in.dtype == kF32) {
      if (ns == 2u) return false;
      out->sin[ns++] = k;
    } else {
      return false;
    }
  }
  if (nv == 0u) return false;
  for (uint32_t j = nv; j < 4u; ++j) {
    out->vin[j] = out->vin[0];
    out->vrow[j] = out->vrow[0];
  }
  for (uint32_t j = ns; j < 2u; ++j) out->sin[j] = 0u;
  out->n_sin = ns;
  out->pad = nv;
  out->prog = p;
  return true;
}

// Second half of a split-K contraction: add the splits' partial products (fixed order, so the
// sum does not depend on scheduling) and run the contraction's post program on the result.
template <int MAXIN, bool FAST>
__global__ __launch_bounds__(kBlock) void lt_split_post_kernel(const SplitPostArgs a) {
  const EwProg& p = a.prog;
  const uint64_t n = p.n;
  constexpr uint64_t kTile = (uint64_t)kBlock * kVec;
  const uint64_t ntiles = (n + kTile - 1) / kTile;
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t lane = threadIdx.x * kVec;
  const bool vec = (a.stride % 4u) == 0u;
  for (uint64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
    const uint64_t base = tile * kTile;
    const uint64_t left = n - base;
    if ((uint64_t)lane >= left) continue;
    const uint32_t nvalid = left - lane >= (uint64_t)kVec ? (uint32_t)kVec : (uint32_t)(left - lane);
    Quad anchor = splat(0.0f);
    for (uint32_t s = 0; s < a.splits; ++s) {
      const float* src = a.ws + (uint64_t)s * a.stride + base + lane;
      if (FAST || (vec && nvalid == (uint32_t)kVec)) {   // 16-byte aligned: every split starts at a multiple of 4 floats
        const float4 t = *(const float4*)src;
        anchor.v[0] += t.x; anchor.v[1] += t.y; anchor.v[2] += t.z; anchor.v[3] += t.w;
      } else {
        for (uint32_t e = 0; e < nvalid; ++e) anchor.v[e] += src[e];
      }
    }
    RF<16> f = load_inputs<16, MAXIN, FAST, false>(rf_zero<16>(), p, base, lane, nvalid);
    f = rf_set<16>(f, p.anchor_slot, anchor);
    f = interp<16>(f, pr, n_code);
    store_outputs<16, FAST, false>(f, p, base, lane, nvalid);
  }
}

// The same with the loads sorted out on the host, for post programs of at most eight slots whose
// inputs are plain (same shape as the product): at most two fp32 ones and one bf16 one -- an
// optimiser update of bf16 parameters with fp32 moments.  Two tiles per trip and workgroup, one
// trip per workgroup; the partial products of four splits at a time and every input of both tiles
// are fetched before anything is used, and the interpreter runs once for both tiles.
struct SplitStreamArgs {
  SplitPostArgs base;
  uint32_t fin[2];    // input numbers of the fp32 inputs (padded with the first)
  uint32_t bin;       // input number of the bf16 input
  uint32_t n_fin, n_bin, pad;
};

template <int NVF, int NVB>
__global__ __launch_bounds__(kBlock) void lt_split_post_stream_kernel(const SplitStreamArgs sa) {
  const SplitPostArgs& a = sa.base;
  const EwProg& p = a.prog;
  const uint64_t n = p.n;
  constexpr uint64_t kTile = (uint64_t)kBlock * kVec;
  const uint64_t ntiles = (n + kTile - 1) / kTile;
  const uint64_t npairs = (n / kTile) / 2;
  const uint64_t ntrips = npairs + (ntiles - 2 * npairs);
  const ProgRegs pr = load_prog_regs(p);
  const uint32_t n_code = p.n_code;
  const uint32_t lane = threadIdx.x * kVec;
  const char* fp[NVF > 0 ? NVF : 1];
  uint32_t fslot[NVF > 0 ? NVF : 1];
#pragma unroll
  for (int j = 0; j < NVF; ++j) {
    fslot[j] = sa.fin[j];
    fp[j] = (const char*)p.in[fslot[j]].ptr;
  }
  const char* bp = NVB ? (const char*)p.in[sa.bin].ptr : nullptr;
  for (uint64_t trip = blockIdx.x; trip < ntrips; trip += gridDim.x) {
    const bool pair = trip < npairs;
    const uint64_t t0 = pair ? 2 * trip : npairs + trip, t1 = pair ? t0 + 1 : t0;
    const uint64_t e0 = t0 * kTile + lane, e1 = t1 * kTile + lane;   // first element of this lane's two quads
    if (e0 >= n) continue;   // (only in the last tile, which is its own partner)
    RawVec vf0[NVF > 0 ? NVF : 1], vf1[NVF > 0 ? NVF : 1];
    typedef uint32_t U32x2 __attribute__((ext_vector_type(2)));
    U32x2 vb0 = {0, 0}, vb1 = {0, 0};
#pragma unroll
    for (int j = 0; j < NVF; ++j) {
      vf0[j] = *(const RawVec*)(fp[j] + e0 * 4u);
      vf1[j] = *(const RawVec*)(fp[j] + e1 * 4u);
    }
    if (NVB) {
      vb0 = *(const U32x2*)(bp + e0 * 2u);
      vb1 = *(const U32x2*)(bp + e1 * 2u);
    }
    // partial products, summed in split order (the result does not depend on scheduling)
    RawVec s0 = {0, 0, 0, 0}, s1 = {0, 0, 0, 0};
    uint32_t sp = 0;
    for (; sp + 2u <= a.splits; sp += 2u) {
      RawVec t0v[2], t1v[2];
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        const float* src = a.ws + (uint64_t)(sp + j) * a.stride;
        t0v[j] = *(const RawVec*)(src + e0);
        t1v[j] = *(const RawVec*)(src + e1);
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        s0 += t0v[j];
        s1 += t1v[j];
      }
    }
    for (; sp < a.splits; ++sp) {
      const float* src = a.ws + (uint64_t)sp * a.stride;
      const RawVec u0 = *(const RawVec*)(src + e0), u1 = *(const RawVec*)(src + e1);
      s0 += u0;
      s1 += u1;
    }
    RF<16> f = rf_zero<16>();
    Quad q;
#pragma unroll
    for (int j = 0; j < NVF; ++j) {
      q.v[0] = vf0[j].x; q.v[1] = vf0[j].y; q.v[2] = vf0[j].z; q.v[3] = vf0[j].w;
      f = rf_set<16>(f, fslot[j], q);
      q.v[0] = vf1[j].x; q.v[1] = vf1[j].y; q.v[2] = vf1[j].z; q.v[3] = vf1[j].w;
      f = rf_set<16>(f, fslot[j] + 8u, q);
    }
    if (NVB) {
      q.v[0] = __uint_as_float(vb0.x << 16); q.v[1] = __uint_as_float(vb0.x & 0xffff0000u);
      q.v[2] = __uint_as_float(vb0.y << 16); q.v[3] = __uint_as_float(vb0.y & 0xffff0000u);
      f = rf_set<16>(f, sa.bin, q);
      q.v[0] = __uint_as_float(vb1.x << 16); q.v[1] = __uint_as_float(vb1.x & 0xffff0000u);
      q.v[2] = __uint_as_float(vb1.y << 16); q.v[3] = __uint_as_float(vb1.y & 0xffff0000u);
      f = rf_set<16>(f, sa.bin + 8u, q);
    }
    q.v[0] = s0.x; q.v[1] = s0.y; q.v[2] = s0.z; q.v[3] = s0.w;
    f = rf_set<16>(f, p.anchor_slot, q);
    q.v[0] = s1.x; q.v[1] = s1.y; q.v[2] = s1.z; q.v[3] = s1.w;
    f = rf_set<16>(f, p.anchor_slot + 8u, q);
    f = interp<16, 2>(f, pr, n_code);
    store_outputs<16, true, false, 0>(f, p, t0 * kTile, lane, kVec);
    store_outputs<16, true, false, 8>(f, p, t1 * kTile, lane, kVec);
  }
}

static bool make_split_stream_args(const SplitPostArgs& a, SplitStreamArgs* out) {
  const EwProg& p = a.prog;
  if (!p.fast || p.n_slots > 8u || (a.stride % 4u) != 0u) return false;
  uint32_t nf = 0, nb = 0;
  out->fin[0] = out->fin[1] = out->bin = 0u;
  for (uint32_t k = 0; k < p.n_in; ++k) {
    const EwIn& in = p.in[k];
    if (in.fetch != kFetchVec4 || in.mode != kFull) return false;
    if (in.dtype == kF32) {
      if (nf == 2u) return false;
      out->fin[nf++] = k;
    } else if (in.dtype == kBF16) {
      if (nb == 1u) return false;
      out->bin = k;
      ++nb;
    } else {
      return false;
    }
  }
  if (nf == 1u) out->fin[1] = out->fin[0];
  out->n_fin = nf;
  out->n_bin = nb;
  out->pad = 0;
  out->base = a;
  return true;
}

hipError_t launch_split_post(const SplitPostArgs& a, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kBlock);
  SplitStreamArgs sa;
  if (make_split_stream_args(a, &sa)) {
    const uint64_t tiles = (a.prog.n + 1023) / 1024;
    const dim3 g2((uint32_t)std::max<uint64_t>(1, std::min<uint64_t>((tiles + 1) / 2, 0x7fffffffull)));
    if (sa.n_fin == 0u && sa.n_bin == 0u) LT_LAUNCH((lt_split_post_stream_kernel<0, 0>), g2, b, s, sa);
    else if (sa.n_fin == 0u) LT_LAUNCH((lt_split_post_stream_kernel<0, 1>), g2, b, s, sa);
    else if (sa.n_bin == 0u) LT_LAUNCH((lt_split_post_stream_kernel<2, 0>), g2, b, s, sa);
    else LT_LAUNCH((lt_split_post_stream_kernel<2, 1>), g2, b, s, sa);
    return hipGetLastError();
  }
  // whole 4-vectors of partials need 16-byte aligned splits
  const bool fast = a.prog.fast && a.prog.n_in <= 4u && (a.stride % 4u) == 0u;
  if (fast) LT_LAUNCH((lt_split_post_kernel<4, true>), g, b, s, a);
  else LT_LAUNCH((lt_split_post_kernel<8, false>), g, b, s, a);
  return hipGetLastError();
}

static constexpr uint64_t kStreamGroups = 1024;   // 256 compute units x 4

hipError_t launch_ew(const EwArgs& a, uint32_t grid, hipStream_t s) {
  const EwProg& p = a.prog;
  const dim3 g(grid), b(kBlock);
  const bool f16 = p.fast && p.n_slots <= 16u;
  EwStreamArgs sa;
  if (make_stream_args(p, kBF16, &sa)) {
    const uint64_t tiles = (p.n + 2047) / 2048;
    // at most four workgroups per compute unit (what the registers allow to be resident): each
    // walks its share of the tiles
    const dim3 g2((uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(tiles, kStreamGroups)));
    if (sa.pad == 1u) LT_LAUNCH(lt_ew_stream_bf16_kernel<1>, g2, b, s, sa);
    else if (sa.pad == 2u) LT_LAUNCH(lt_ew_stream_bf16_kernel<2>, g2, b, s, sa);
    else if (sa.pad == 3u) LT_LAUNCH(lt_ew_stream_bf16_kernel<3>, g2, b, s, sa);
    else LT_LAUNCH(lt_ew_stream_bf16_kernel<4>, g2, b, s, sa);
    return hipGetLastError();
  }
  if (make_stream_args(p, kF32, &sa)) {
    const uint64_t tiles = (p.n + 1023) / 1024;
    // one trip per workgroup: measured 5.27 TB/s on 1 GiB operands against 4.3 with 8192 workgroups
    // walking the same tiles with a grid stride (the loop stays for spaces beyond 2^31 trips)
    const dim3 g2((uint32_t)std::max<uint64_t>(1, std::min<uint64_t>((tiles + 1) / 2, 0x7fffffffull)));
    const bool nt = p.n * 4u * (uint64_t)(p.n_in + p.n_out) > (256ull << 20);   // beyond the 256 MiB last-level cache
    if (sa.pad <= 2u && nt) LT_LAUNCH((lt_ew_stream_kernel<2, true>), g2, b, s, sa);
    else if (sa.pad <= 2u) LT_LAUNCH((lt_ew_stream_kernel<2, false>), g2, b, s, sa);
    else if (nt) LT_LAUNCH((lt_ew_stream_kernel<4, true>), g2, b, s, sa);
    else LT_LAUNCH((lt_ew_stream_kernel<4, false>), g2, b, s, sa);
    return hipGetLastError();
  }
  if (f16 && p.all_f32 && p.n_in <= 4u) LT_LAUNCH((lt_ew_kernel<16, 4, true, true>), g, b, s, a);
  else if (f16 && p.all_f32 && p.n_in <= 6u) LT_LAUNCH((lt_ew_kernel<16, 6, true, true>), g, b, s, a);
  else if (f16 && p.all_f32) LT_LAUNCH((lt_ew_kernel<16, 8, true, true>), g, b, s, a);
  else if (f16) LT_LAUNCH((lt_ew_kernel<16, 8, true, false>), g, b, s, a);
  else LT_LAUNCH((lt_ew_kernel<32, 8, false, false>), g, b, s, a);
  return hipGetLastError();
}

// ---- window update (the inverse of a narrow view, section 4.4 of the paper) ---------------------
// One element per lane and trip, any element size: a copy, bound by HBM.  In place only the
// window is touched.
template <typename T>
__global__ __launch_bounds__(kBlock) void lt_slice_update_kernel(const SliceArgs a) {
  const T* base = (const T*)a.base;
  const T* upd = (const T*)a.upd;
  T* out = (T*)a.out;
  const uint64_t stride = (uint64_t)gridDim.x * kBlock;
  const uint64_t win = a.len * a.inner, row = a.dim * a.inner, lo = a.start * a.inner;
  for (uint64_t i = (uint64_t)blockIdx.x * kBlock + threadIdx.x; i < a.n; i += stride) {
    if (a.window_only) {
      const uint64_t o = i / win, r = i % win;
      out[o * row + lo + r] = upd[i];
    } else {
      const uint64_t o = i / row, r = i % row;
      out[i] = (r >= lo && r < lo + win) ? upd[o * win + (r - lo)] : base[i];
    }
  }
}

hipError_t launch_slice_update(const SliceArgs& a, uint32_t grid, hipStream_t s) {
  if (a.n == 0) return hipSuccess;
  if (!a.upd || !a.out || (!a.window_only && !a.base) || a.start + a.len > a.dim || grid == 0) return hipErrorInvalidValue;
  if (a.elem_bytes == 4) LT_LAUNCH(lt_slice_update_kernel<uint32_t>, dim3(grid), dim3(kBlock), s, a);
  else if (a.elem_bytes == 2) LT_LAUNCH(lt_slice_update_kernel<uint16_t>, dim3(grid), dim3(kBlock), s, a);
  else if (a.elem_bytes == 8) LT_LAUNCH(lt_slice_update_kernel<uint64_t>, dim3(grid), dim3(kBlock), s, a);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

}  // namespace ltk
