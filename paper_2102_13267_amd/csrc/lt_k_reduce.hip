// Reduction regions: row, global (single launch) and column reductions, each with an interpreted
// elementwise prologue and an interpreted post program (epilogue / finaliser).
#include <hip/hip_runtime.h>

#include "lt_launch.h"
#include "lt_reduce.h"

namespace ltk {

// Run the post program of an anchored region for the flat elements i .. i+nvalid-1 of its
// space, with the anchor's value(s) already placed in slot post.anchor_slot.
__device__ __forceinline__ void run_post(const EwProg& post, const ProgRegs post_regs, Quad anchor, uint64_t i,
                                         uint32_t nvalid) {
  RF<16> f = load_inputs<16>(rf_zero<16>(), post, 0, (uint32_t)i, nvalid);
  f = rf_set(f, post.anchor_slot, anchor);
  f = interp<16>(f, post_regs, post.n_code);
  store_outputs<16>(f, post, 0, (uint32_t)i, nvalid);
}

// Streamed row reduction: fp32 programs of at most eight slots whose inputs are one or two whole
// tensors and at most one vector broadcast along rows, rows of a multiple of 16 x threads_per_row
// columns.  A lane takes four 4-vectors of its row per trip (threads_per_row x 4 columns apart):
// their loads go out together and the interpreter runs once for the four (8 slots x 4 vectors) --
// what bounds a cache-resident row reduction with a long prologue is the interpreter's dispatch,
// not memory.  NV, NR: whole inputs, row-vector inputs (the host sorts out which is which).
template <int NV, int NR>
__global__ __launch_bounds__(kBlock) void lt_row_reduce_stream_kernel(const RowArgs a) {
  __shared__ float lds[kBlock / 64];
  const EwProg& pro = a.pro;
  const ProgRegs pro_regs = load_prog_regs(a.pro), post_regs = load_prog_regs(a.post);
  const uint32_t pro_n = a.pro.n_code;
  const uint32_t tpr = a.threads_per_row;
  const uint32_t rows_per_block = kBlock / tpr;
  const uint32_t lane = threadIdx.x % tpr;
  const uint32_t sub = threadIdx.x / tpr;
  const uint32_t nblocks = (a.rows + rows_per_block - 1) / rows_per_block;
  const uint32_t step = tpr * kVec;   // columns between a lane's consecutive 4-vectors
  const char* vp[NV];
  uint32_t vslot[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    vslot[k] = a.vin[k];
    vp[k] = (const char*)pro.in[vslot[k]].ptr;
  }
  const char* rp = NR ? (const char*)pro.in[a.rin].ptr : nullptr;
  for (uint32_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const uint32_t row = blk * rows_per_block + sub;
    float acc = red_identity(a.red);
    if (row < a.rows) {
      for (uint32_t c = lane * kVec; c < a.cols; c += 4u * step) {   // (cols is a multiple of 4 * step)
        RawVec v[NV][4], rv[NR ? 4 : 1];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint64_t e = (uint64_t)row * a.cols + c + (uint32_t)j * step;
#pragma unroll
          for (int k = 0; k < NV; ++k) v[k][j] = *(const RawVec*)(vp[k] + e * 4u);
          if (NR) rv[j] = *(const RawVec*)(rp + (size_t)(c + (uint32_t)j * step) * 4u);
        }
        RF<32> f = rf_zero<32>();
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          Quad q;
#pragma unroll
          for (int k = 0; k < NV; ++k) {
            q.v[0] = v[k][j].x; q.v[1] = v[k][j].y; q.v[2] = v[k][j].z; q.v[3] = v[k][j].w;
            f = rf_set<32>(f, vslot[k] + (uint32_t)(8 * j), q);
          }
          if (NR) {
            q.v[0] = rv[j].x; q.v[1] = rv[j].y; q.v[2] = rv[j].z; q.v[3] = rv[j].w;
            f = rf_set<32>(f, a.rin + (uint32_t)(8 * j), q);
          }
        }
        f = interp<32, 4>(f, pro_regs, pro_n);
#pragma unroll
        for (int j = 0; j < 4; ++j) acc = fold_vec(a.red, acc, rf_get<32>(f, pro.anchor_slot + (uint32_t)(8 * j)), kVec);
      }
    }
    float r;
    if (tpr == 64u) r = wave_reduce(a.red, acc);
    else r = block_reduce(a.red, acc, lds);
    if (a.red == kRedMean) r = r / (float)a.cols;
    if (lane == 0 && row < a.rows) run_post(a.post, post_regs, splat(r), row, 1u);
  }
}

// Row reduction.  threads_per_row is 64 (one wave per row, four rows per workgroup) or 256.
__global__ __launch_bounds__(kBlock) void lt_row_reduce_kernel(const RowArgs a) {
  __shared__ float lds[kBlock / 64];
  const EwProg& pro = a.pro;
  const ProgRegs pro_regs = load_prog_regs(a.pro), post_regs = load_prog_regs(a.post);
  const uint32_t pro_n = a.pro.n_code;
  const uint32_t tpr = a.threads_per_row;
  const uint32_t rows_per_block = kBlock / tpr;
  const uint32_t lane = threadIdx.x % tpr;
  const uint32_t sub = threadIdx.x / tpr;
  const uint32_t nblocks = (a.rows + rows_per_block - 1) / rows_per_block;
  for (uint32_t blk = blockIdx.x; blk < nblocks; blk += gridDim.x) {
    const uint32_t row = blk * rows_per_block + sub;
    float acc = red_identity(a.red);
    if (row < a.rows) {
      for (uint32_t c = lane * kVec; c < a.cols; c += tpr * kVec) {
        const uint32_t nvalid = (a.cols - c >= (uint32_t)kVec) ? (uint32_t)kVec : a.cols - c;
        const uint32_t i = row * a.cols + c;
        // (the compact general path: measured faster here than the unrolled loads, whose code the
        // typical small, cache-resident row reduction would have to fetch first)
        RF<16> f = load_inputs<16>(rf_zero<16>(), pro, 0, i, nvalid);
        f = interp<16>(f, pro_regs, pro_n);
        acc = fold_vec(a.red, acc, rf_get(f, pro.anchor_slot), nvalid);
      }
    }
    float r;
    if (tpr == 64u) r = wave_reduce(a.red, acc);
    else r = block_reduce(a.red, acc, lds);
    if (a.red == kRedMean) r = r / (float)a.cols;
    if (lane == 0 && row < a.rows) run_post(a.post, post_regs, splat(r), row, 1u);
  }
}

// Global reduction in one launch.  NIN > 0: streamed (U 4-vectors per lane and trip fetched
// together, a workgroup reading U consecutive tiles); NIN == 0: general path.
// Q = 2, 4: so many 4-vectors per interpreter dispatch (programs of at most NS/Q slots).
template <int NS, int NIN, int U, bool BF, int Q>
__global__ __launch_bounds__(kBlock) void lt_all_reduce_kernel(const AllArgs a) {
  __shared__ float lds[kBlock / 64];
  __shared__ uint32_t is_last;
  const EwProg& pro = a.pro;
  const ProgRegs pro_regs = load_prog_regs(a.pro), post_regs = load_prog_regs(a.post);
  const uint32_t pro_n = a.pro.n_code;
  const uint64_t n = pro.n;
  const uint64_t nvec = (n + kVec - 1) / kVec;
  float acc = red_identity(a.red);
  uint64_t tail_from = 0;   // first 4-vector the general loop below has to cover
  if (NIN > 0) {
    // a trip of the grid covers gridDim.x * U tiles of kBlock vectors; workgroup b takes tiles
    // b*U .. b*U+U-1 of each trip, i.e. U * 4 KiB (fp32) of consecutive memory
    constexpr int UU = NIN > 0 ? U : 1, NN = NIN > 0 ? NIN : 1;
    const uint64_t per_trip = (uint64_t)gridDim.x * UU * kBlock;
    const uint64_t trips = nvec / per_trip;
    // A prologue of one instruction, square or abs of the operand, is applied in place (same
    // values, same order of additions as the interpreter's): the interpreter's dispatch is what
    // keeps such a reduction from the memory system's rate, and these two are every norm.
    uint32_t lone = 0;
    if (NN == 1 && pro_n == 1u) {
      const uint32_t w = pro.code[0], op = w & 0xffu;
      if ((op == kSquare || op == kAbs) && ((w >> 13) & 63u) == 0u && ((w >> 8) & 31u) == pro.anchor_slot) lone = op;
    }
    for (uint64_t t = 0; t < trips; ++t) {
      const uint64_t v0 = t * per_trip + (uint64_t)blockIdx.x * UU * kBlock;   // wave-uniform
      Stream<NN, UU, BF> st;
#pragma unroll
      for (int u = 0; u < UU; ++u) stream_fetch<NN, UU, BF>(st, u, pro, (v0 + (uint64_t)u * kBlock) * kVec, threadIdx.x * kVec);
      if (NN == 1 && pro_n == 0u) {   // the operand itself is reduced: nothing to interpret
#pragma unroll
        for (int u = 0; u < UU; ++u) acc = fold_vec(a.red, acc, stream_quad<NN, UU, BF>(st, 0, u), kVec);
      } else if (NN == 1 && lone != 0u) {   // one unary instruction on the operand (a norm: sum of squares, of magnitudes)
#pragma unroll
        for (int u = 0; u < UU; ++u) {
          Quad q = stream_quad<NN, UU, BF>(st, 0, u);
#pragma unroll
          for (int v = 0; v < kVec; ++v) q.v[v] = lone == kSquare ? q.v[v] * q.v[v] : fabsf(q.v[v]);
          acc = fold_vec(a.red, acc, q, kVec);
        }
      } else {
#pragma unroll 1
        for (uint32_t u = 0; u < (uint32_t)UU; u += Q) {
          RF<NS> f = stream_place<NS, NN, UU, BF>(rf_zero<NS>(), st, u);
          if (Q >= 2) f = stream_place<NS, NN, UU, BF, NS / Q>(f, st, u + 1u);
          if (Q == 4) {
            f = stream_place<NS, NN, UU, BF, 2 * (NS / Q)>(f, st, u + 2u);
            f = stream_place<NS, NN, UU, BF, 3 * (NS / Q)>(f, st, u + 3u);
          }
          f = interp<NS, Q>(f, pro_regs, pro_n);
#pragma unroll
          for (int j = 0; j < Q; ++j) acc = fold_vec(a.red, acc, rf_get(f, pro.anchor_slot + j * (NS / Q)), kVec);
        }
      }
    }
    tail_from = trips * per_trip;
  }
  for (uint64_t v = tail_from + (uint64_t)blockIdx.x * kBlock + threadIdx.x; v < nvec; v += (uint64_t)gridDim.x * kBlock) {
    const uint64_t i = v * kVec;
    const uint32_t nvalid = (n - i >= (uint64_t)kVec) ? (uint32_t)kVec : (uint32_t)(n - i);
    RF<NS> f = load_inputs<NS, kMaxIn, false, false>(rf_zero<NS>(), pro, 0, (uint32_t)i, nvalid);
    f = interp<NS>(f, pro_regs, pro_n);
    acc = fold_vec(a.red, acc, rf_get(f, pro.anchor_slot), nvalid);
  }
  float r = block_reduce(a.red, acc, lds);
  if (gridDim.x > 1u) {   // (a single workgroup is its own last one: no partials, no ticket)
    if (threadIdx.x == 0) {
      publish(&a.partials[blockIdx.x], r);
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // (the store has been performed before the ticket is taken)
      uint32_t t = atomicAdd(a.ticket, 1u);
      is_last = (t == gridDim.x - 1) ? 1u : 0u;
    }
    __syncthreads();
    if (!is_last) return;
    // the last workgroup combines the partials in a fixed order (deterministic for a given grid)
    acc = red_identity(a.red);
    for (uint32_t g = threadIdx.x; g < gridDim.x; g += kBlock) acc = red_combine(a.red, acc, published(&a.partials[g]));
    r = block_reduce(a.red, acc, lds);
    if (threadIdx.x == 0) *a.ticket = 0u;
  }
  if (a.red == kRedMean) r = r / (float)a.count;
  const EwProg& post = a.post;
  const uint64_t pn = post.n;
  const uint64_t pvec = (pn + kVec - 1) / kVec;
  for (uint64_t v = threadIdx.x; v < pvec; v += kBlock) {
    const uint64_t i = v * kVec;
    const uint32_t nvalid = (pn - i >= (uint64_t)kVec) ? (uint32_t)kVec : (uint32_t)(pn - i);
    run_post(post, post_regs, splat(r), i, nvalid);
  }
}

constexpr int kColBlock = 512;

// Column reduction over axis 0 of [rows, cols].  blockIdx.x: strip of 256 columns (64 lanes x 4);
// the eight waves of a workgroup take interleaved rows; blockIdx.y: slab of rows.  A lane owns four
// columns, so nothing crosses lanes until the waves meet in LDS.  FAST (whole aligned 4-vectors,
// no strided input): U rows per wave are fetched together before any is interpreted.
__device__ __forceinline__ void col_fold(uint32_t red, float4& acc, const Quad& q) {
  acc.x = red_combine(red, acc.x, q.v[0]);
  acc.y = red_combine(red, acc.y, q.v[1]);
  acc.z = red_combine(red, acc.z, q.v[2]);
  acc.w = red_combine(red, acc.w, q.v[3]);
}

// NC > 0: besides the NIN inputs read in full (input numbers a.vin) the program has per-row inputs
// (a.cin: a mean, a reciprocal deviation), which a wave reads as one broadcast element per row.
template <int NS, int NIN, int U, bool BF, int NC = 0>
__global__ __launch_bounds__(kColBlock) void lt_col_reduce_kernel(const ColArgs a) {
  constexpr uint32_t kWaves = kColBlock / 64;
  __shared__ float4 lds[kColBlock];
  __shared__ uint32_t is_last;
  const EwProg& pro = a.pro;
  const ProgRegs pro_regs = load_prog_regs(a.pro), post_regs = load_prog_regs(a.post);
  const uint32_t pro_n = a.pro.n_code;
  const uint32_t lane = threadIdx.x & 63;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint32_t c = blockIdx.x * 256u + lane * kVec;
  const uint32_t nvalid = c >= a.cols ? 0u : ((a.cols - c >= (uint32_t)kVec) ? (uint32_t)kVec : a.cols - c);
  const uint32_t rows_per_slab = (a.rows + gridDim.y - 1) / gridDim.y;
  const uint32_t r0 = min(a.rows, blockIdx.y * rows_per_slab);
  const uint32_t r1 = min(a.rows, r0 + rows_per_slab);
  const float id = red_identity(a.red);
  const uint32_t pstride = (a.cols + 3u) & ~3u;   // floats between slabs of partials
  if (NIN == 0 && a.narrow) {
    // Narrow and small (at most 64 columns, at most 65536 elements; one workgroup): a strip of 256
    // columns would leave all but a few lanes idle and walk the rows one by one.  Instead thread
    // t < S, S the largest multiple of cols within the workgroup, takes the elements t, t + S,
    // t + 2 S, ... -- all of column t % cols -- four of them per interpreter dispatch; the threads
    // of a column then meet in LDS.
    float* lf = (float*)lds;   // kColBlock x 4 floats
    const uint32_t cols = a.cols, S = ((uint32_t)kColBlock / cols) * cols, n = a.rows * cols;
    float part = id;
    if (threadIdx.x < S) {
      for (uint32_t i0 = threadIdx.x; i0 < n; i0 += 4u * S) {
        uint32_t nv = 1u;
#pragma unroll
        for (uint32_t e = 1; e < (uint32_t)kVec; ++e) nv += (i0 + e * S < n) ? 1u : 0u;
        RF<16> f = rf_zero<16>();
#pragma unroll 1
        for (uint32_t k = 0; k < pro.n_in; ++k) {
          const EwIn& in = pro.in[k];
          Quad q;
#pragma unroll
          for (uint32_t e = 0; e < (uint32_t)kVec; ++e) {
            const uint32_t ee = e < nv ? e : nv - 1u;   // (past the end: the last valid one again, no load behind a branch)
            q.v[e] = load_elem<false>(in.ptr, in.dtype, elem_offset(pro, in, i0 + ee * S));
          }
          f = rf_set<16>(f, k, q);
        }
        f = interp<16>(f, pro_regs, pro_n);
        const Quad r = rf_get(f, pro.anchor_slot);
        part = red_combine(a.red, part, r.v[0]);
        if (nv > 1u) part = red_combine(a.red, part, r.v[1]);
        if (nv > 2u) part = red_combine(a.red, part, r.v[2]);
        if (nv > 3u) part = red_combine(a.red, part, r.v[3]);
      }
    }
    lf[threadIdx.x] = part;
    __syncthreads();
    float colv = id;
    if (threadIdx.x < cols)
      for (uint32_t j = threadIdx.x; j < S; j += cols) colv = red_combine(a.red, colv, lf[j]);   // fixed order
    if (a.red == kRedMean) colv = colv / (float)a.rows;
    __syncthreads();
    if (threadIdx.x < cols) lf[threadIdx.x] = colv;
    __syncthreads();
    const uint32_t c4 = threadIdx.x * (uint32_t)kVec;
    if (c4 < cols) {
      const uint32_t nvp = cols - c4 >= (uint32_t)kVec ? (uint32_t)kVec : cols - c4;
      Quad accq;
#pragma unroll
      for (uint32_t e = 0; e < (uint32_t)kVec; ++e) accq.v[e] = e < nvp ? lf[c4 + e] : 0.0f;
      run_post(a.post, post_regs, accq, c4, nvp);
    }
    return;
  }
  float4 acc = make_float4(id, id, id, id);
  if (nvalid) {
    uint32_t r = r0 + wave;
    if (NIN > 0) {   // streamed: cols is a multiple of 4, so this lane's vector is whole
      constexpr int UU = NIN > 0 ? U : 1, NN = NIN > 0 ? NIN : 1;
      for (; r + (UU - 1) * kWaves < r1; r += UU * kWaves) {
        Stream<NN, UU, BF> st;
        typename WideVec<UU>::type cw[NC > 0 ? NC : 1];   // per-row inputs of the UU rows
        if (NC > 0) {
#pragma unroll
          for (int u = 0; u < UU; ++u) {
            const uint64_t e = (uint64_t)(r + u * kWaves) * a.cols + blockIdx.x * 256u + lane * kVec;
#pragma unroll
            for (int k = 0; k < NN; ++k) {
              const char* src = (const char*)pro.in[a.vin[k]].ptr;
              if (BF) {
                typedef uint32_t U32x2 __attribute__((ext_vector_type(2)));
                const U32x2 t = *(const U32x2*)(src + e * 2u);
                st.s[k][2 * u] = __uint_as_float(t.x);
                st.s[k][2 * u + 1] = __uint_as_float(t.y);
              } else {
                const RawVec t = *(const RawVec*)(src + e * 4u);
                st.s[k][4 * u] = t.x; st.s[k][4 * u + 1] = t.y; st.s[k][4 * u + 2] = t.z; st.s[k][4 * u + 3] = t.w;
              }
            }
#pragma unroll
            for (int j = 0; j < NC; ++j) {
              const EwIn& in = pro.in[a.cin[j]];
              cw[j][u] = load_elem<false>(in.ptr, in.dtype, r + u * kWaves);
            }
          }
          // NS = 32: four rows per interpreter dispatch (8 slots x 4 rows), programs of at most 8 slots
          constexpr int QQ = NS == 32 ? 4 : 1;
          constexpr uint32_t SL = NS / QQ;
#pragma unroll 1
          for (uint32_t u = 0; u < (uint32_t)UU; u += QQ) {
            RF<NS> f = rf_zero<NS>();
#pragma unroll
            for (int j = 0; j < QQ; ++j) {
              const RF<NS> one = stream_place<NS, NN, UU, BF>(rf_zero<NS>(), st, u + (uint32_t)j);   // (row u + j in slots 0 .. NN-1)
#pragma unroll
              for (int k = 0; k < NN; ++k) f = rf_set<NS>(f, a.vin[k] + (uint32_t)j * SL, rf_get<NS>(one, (uint32_t)k));
#pragma unroll
              for (int c = 0; c < NC; ++c) f = rf_set<NS>(f, a.cin[c] + (uint32_t)j * SL, splat(cw[c][u + (uint32_t)j]));
            }
            f = interp<NS, QQ>(f, pro_regs, pro_n);
#pragma unroll
            for (int j = 0; j < QQ; ++j) col_fold(a.red, acc, rf_get(f, pro.anchor_slot + (uint32_t)j * SL));
          }
          continue;
        }
#pragma unroll
        for (int u = 0; u < UU; ++u)
          stream_fetch<NN, UU, BF>(st, u, pro, (uint64_t)(r + u * kWaves) * a.cols + blockIdx.x * 256u, lane * kVec);
        if (NN == 1 && pro_n == 0u) {   // the operand itself is reduced: nothing to interpret
#pragma unroll
          for (int u = 0; u < UU; ++u) col_fold(a.red, acc, stream_quad<NN, UU, BF>(st, 0, u));
        } else {
#pragma unroll 1
          for (uint32_t u = 0; u < (uint32_t)UU; ++u) {
            RF<NS> f = stream_place<NS, NN, UU, BF>(rf_zero<NS>(), st, u);
            f = interp<NS>(f, pro_regs, pro_n);
            col_fold(a.red, acc, rf_get(f, pro.anchor_slot));
          }
        }
      }
    }
    for (; r < r1; r += kWaves) {
      const uint64_t rb = (uint64_t)r * a.cols + blockIdx.x * 256u;
      RF<NS> f = (pro.fast && nvalid == (uint32_t)kVec) ? load_inputs<NS, kMaxIn, true, false>(rf_zero<NS>(), pro, rb, lane * kVec, nvalid)
                                                        : load_inputs<NS, kMaxIn, false, false>(rf_zero<NS>(), pro, rb, lane * kVec, nvalid);
      f = interp<NS>(f, pro_regs, pro_n);
      col_fold(a.red, acc, rf_get(f, pro.anchor_slot));
    }
  }
  lds[threadIdx.x] = acc;
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int w = 1; w < (int)kWaves; ++w) {
      const float4 o = lds[w * 64 + lane];
      acc.x = red_combine(a.red, acc.x, o.x);
      acc.y = red_combine(a.red, acc.y, o.y);
      acc.z = red_combine(a.red, acc.z, o.z);
      acc.w = red_combine(a.red, acc.w, o.w);
    }
    if (gridDim.y == 1u) {   // one slab: this is the result, no partials, no tickets
      if (!nvalid) return;
      if (a.red == kRedMean) {
        const float inv = 1.0f / (float)a.rows;
        acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
      }
      Quad accq;
      accq.v[0] = acc.x; accq.v[1] = acc.y; accq.v[2] = acc.z; accq.v[3] = acc.w;
      run_post(a.post, post_regs, accq, c, nvalid);
      return;
    }
    // The slab stride is padded to a multiple of four floats so that whole vectors stay 16-byte
    // aligned.
    if (nvalid == (uint32_t)kVec) {
      publish4(a.partials + (uint64_t)blockIdx.y * pstride + c, acc);
    } else if (nvalid) {
      float* dst = a.partials + (uint64_t)blockIdx.y * pstride + c;
      publish(dst, acc.x);
      if (nvalid > 1u) publish(dst + 1, acc.y);
      if (nvalid > 2u) publish(dst + 2, acc.z);
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");   // (this wave's stores have been performed before its ticket is taken)
    if (lane == 0) {
      uint32_t t = atomicAdd(&a.tickets[blockIdx.x], 1u);
      is_last = (t == gridDim.y - 1) ? 1u : 0u;
    }
  }
  if (gridDim.y == 1u) return;   // (uniform: wave 0 has finished the strip above)
  __syncthreads();
  if (!is_last) return;
  if (threadIdx.x == 0) a.tickets[blockIdx.x] = 0u;
  // the last workgroup of a strip combines the slabs: each wave a contiguous share, eight loads in
  // flight, fixed order (deterministic for a given grid)
  acc = make_float4(id, id, id, id);
  if (nvalid) {
    const uint32_t per_wave = (gridDim.y + kWaves - 1) / kWaves;
    const uint32_t s0 = min(gridDim.y, wave * per_wave), s1 = min(gridDim.y, s0 + per_wave);
    for (uint32_t sb = s0; sb < s1; sb += 8) {
      float4 t[8];
#pragma unroll
      for (uint32_t j = 0; j < 8; ++j) {
        t[j] = make_float4(id, id, id, id);
        if (sb + j < s1) {
          const float* src = a.partials + (uint64_t)(sb + j) * pstride + c;
          if (nvalid == (uint32_t)kVec) {
            t[j] = published4(src);
          } else {
            t[j].x = published(src);
            if (nvalid > 1u) t[j].y = published(src + 1);
            if (nvalid > 2u) t[j].z = published(src + 2);
          }
        }
      }
#pragma unroll
      for (uint32_t j = 0; j < 8; ++j) {
        acc.x = red_combine(a.red, acc.x, t[j].x);
        acc.y = red_combine(a.red, acc.y, t[j].y);
        acc.z = red_combine(a.red, acc.z, t[j].z);
        acc.w = red_combine(a.red, acc.w, t[j].w);
      }
    }
  }
  __syncthreads();   // every wave has read its slot of the first exchange
  lds[threadIdx.x] = acc;
  __syncthreads();
  if (wave != 0 || !nvalid) return;
#pragma unroll
  for (int w = 1; w < (int)kWaves; ++w) {
    const float4 o = lds[w * 64 + lane];
    acc.x = red_combine(a.red, acc.x, o.x);
    acc.y = red_combine(a.red, acc.y, o.y);
    acc.z = red_combine(a.red, acc.z, o.z);
    acc.w = red_combine(a.red, acc.w, o.w);
  }
  if (a.red == kRedMean) {
    const float inv = 1.0f / (float)a.rows;
    acc.x *= inv; acc.y *= inv; acc.z *= inv; acc.w *= inv;
  }
  Quad accq;
  accq.v[0] = acc.x; accq.v[1] = acc.y; accq.v[2] = acc.z; accq.v[3] = acc.w;
  run_post(a.post, post_regs, accq, c, nvalid);
}


// Host side: does the program qualify for the streamed row reduction?  Fills in a->vin, a->rin and,
// when rows are a multiple of 1024 columns only, narrows threads_per_row to 64 (one wave per row)
// so that a lane has four 4-vectors to take together.
static bool row_stream_args(RowArgs* a, uint32_t* grid) {
  const EwProg& p = a->pro;
  if (!p.fast || !p.all_f32 || p.n_slots > 8u || p.n_in == 0u) return false;
  uint32_t nv = 0, nr = 0;
  for (uint32_t k = 0; k < p.n_in; ++k) {
    const EwIn& in = p.in[k];
    if (in.fetch != kFetchVec4 || in.dtype != kF32) return false;
    if (in.mode == kFull && nv < 2u) a->vin[nv++] = k;
    else if (in.mode == kRowVec && nr < 1u) { a->rin = k; ++nr; }
    else return false;
  }
  if (nv == 0u) return false;
  uint32_t tpr = a->threads_per_row;
  if (a->cols % (16u * tpr) != 0u) {
    tpr = 64u;
    if (a->cols % (16u * tpr) != 0u) return false;
  }
  if (tpr != a->threads_per_row) {
    a->threads_per_row = tpr;
    const uint32_t rpb = (uint32_t)kBlock / tpr;
    *grid = (a->rows + rpb - 1) / rpb < 4096u ? (a->rows + rpb - 1) / rpb : 4096u;
    if (*grid == 0u) *grid = 1u;
  }
  a->n_vin = nv;
  a->n_rin = nr;
  for (uint32_t j = nv; j < 2u; ++j) a->vin[j] = a->vin[0];
  return true;
}

hipError_t launch_row_reduce(const RowArgs& args, uint32_t grid, hipStream_t s) {
  RowArgs a = args;
  a.vin[0] = a.vin[1] = a.rin = a.n_vin = a.n_rin = 0u;
  if (row_stream_args(&a, &grid)) {
    const dim3 g(grid), b(kBlock);
    if (a.n_vin == 1u && a.n_rin == 0u) LT_LAUNCH((lt_row_reduce_stream_kernel<1, 0>), g, b, s, a);
    else if (a.n_vin == 1u) LT_LAUNCH((lt_row_reduce_stream_kernel<1, 1>), g, b, s, a);
    else if (a.n_rin == 0u) LT_LAUNCH((lt_row_reduce_stream_kernel<2, 0>), g, b, s, a);
    else LT_LAUNCH((lt_row_reduce_stream_kernel<2, 1>), g, b, s, a);
    return hipGetLastError();
  }
  LT_LAUNCH(lt_row_reduce_kernel, dim3(grid), dim3(kBlock), s, args);
  return hipGetLastError();
}
hipError_t launch_all_reduce(const AllArgs& a, uint32_t grid, hipStream_t s) {
  const dim3 g(grid), b(kBlock);
  const int kind = stream_kind(a.pro);
  const uint32_t n_in = a.pro.n_in;
  const bool two = a.pro.n_slots <= 8u;   // the program fits half a register file: two 4-vectors per dispatch
  if (kind == 1 && n_in == 1u && two) LT_LAUNCH((lt_all_reduce_kernel<32, 1, 8, false, 4>), g, b, s, a);
  else if (kind == 1 && n_in == 1u) LT_LAUNCH((lt_all_reduce_kernel<16, 1, 8, false, 1>), g, b, s, a);
  else if (kind == 1 && n_in == 2u && two) LT_LAUNCH((lt_all_reduce_kernel<32, 2, 4, false, 4>), g, b, s, a);
  else if (kind == 1 && n_in == 2u) LT_LAUNCH((lt_all_reduce_kernel<16, 2, 4, false, 1>), g, b, s, a);
  else if (kind == 2 && n_in == 1u && two) LT_LAUNCH((lt_all_reduce_kernel<32, 1, 8, true, 4>), g, b, s, a);
  else if (kind == 2 && n_in == 1u) LT_LAUNCH((lt_all_reduce_kernel<16, 1, 8, true, 1>), g, b, s, a);
  else if (kind == 2 && n_in == 2u && two) LT_LAUNCH((lt_all_reduce_kernel<32, 2, 8, true, 4>), g, b, s, a);
  else if (kind == 2 && n_in == 2u) LT_LAUNCH((lt_all_reduce_kernel<16, 2, 8, true, 1>), g, b, s, a);
  else LT_LAUNCH((lt_all_reduce_kernel<16, 0, 1, false, 1>), g, b, s, a);
  return hipGetLastError();
}
// Host side: a program whose inputs are one or two whole tensors of one element type plus one or
// two per-row vectors (the weight gradient of a layer norm: sum over rows of dy * (x - mean) * rstd).
// Returns 0 (no), 1 (fp32) or 2 (bf16) and fills in a->vin, a->cin.
static int mixed_kind(ColArgs* a) {
  const EwProg& p = a->pro;
  if (!p.fast || (a->cols % 4u) != 0u || p.n_slots > 16u) return 0;
  uint32_t nv = 0, nc = 0, dt = 0;
  for (uint32_t k = 0; k < p.n_in; ++k) {
    const EwIn& in = p.in[k];
    if (in.mode == kFull && in.fetch == kFetchVec4 && (nv == 0u || in.dtype == dt) && nv < 2u) {
      dt = in.dtype;
      a->vin[nv++] = k;
    } else if (in.mode == kColVec && nc < 2u && (in.dtype == kF32 || in.dtype == kBF16)) {
      a->cin[nc++] = k;
    } else {
      return 0;
    }
  }
  if (nv == 0u || nc == 0u || (dt != kF32 && dt != kBF16)) return 0;
  for (uint32_t j = nv; j < 2u; ++j) a->vin[j] = a->vin[0];
  for (uint32_t j = nc; j < 2u; ++j) a->cin[j] = a->cin[0];
  return dt == kF32 ? 1 : 2;
}

hipError_t launch_col_reduce(const ColArgs& args, uint32_t grid_x, uint32_t grid_y, hipStream_t s) {
  const dim3 g(grid_x, grid_y), b(kColBlock);
  ColArgs a = args;
  a.vin[0] = 0u; a.vin[1] = 1u; a.cin[0] = a.cin[1] = 0u;
  const int kind = (a.cols % 4u) == 0u ? stream_kind(a.pro) : 0;
  const uint32_t n_in = a.pro.n_in;
  if (kind == 1 && n_in == 1u) LT_LAUNCH((lt_col_reduce_kernel<16, 1, 8, false>), g, b, s, a);
  else if (kind == 1 && n_in == 2u) LT_LAUNCH((lt_col_reduce_kernel<16, 2, 4, false>), g, b, s, a);
  else if (kind == 2 && n_in == 1u) LT_LAUNCH((lt_col_reduce_kernel<16, 1, 8, true>), g, b, s, a);
  else if (kind == 2 && n_in == 2u) LT_LAUNCH((lt_col_reduce_kernel<16, 2, 8, true>), g, b, s, a);
  else {
    const int mk = mixed_kind(&a);
    const bool four = a.pro.n_slots <= 8u;   // the program fits a quarter of a 32-wide register file
    if (mk == 1 && four) LT_LAUNCH((lt_col_reduce_kernel<32, 2, 4, false, 2>), g, b, s, a);
    else if (mk == 1) LT_LAUNCH((lt_col_reduce_kernel<16, 2, 4, false, 2>), g, b, s, a);
    else if (mk == 2 && four) LT_LAUNCH((lt_col_reduce_kernel<32, 2, 8, true, 2>), g, b, s, a);
    else if (mk == 2) LT_LAUNCH((lt_col_reduce_kernel<16, 2, 8, true, 2>), g, b, s, a);
    else if (a.cols <= 64u && (uint64_t)a.rows * a.cols <= 65536u) {
      a.narrow = 1u;   // narrow and small: one workgroup, a thread per (column, row residue)
      LT_LAUNCH((lt_col_reduce_kernel<16, 0, 1, false>), dim3(1, 1), b, s, a);
    } else LT_LAUNCH((lt_col_reduce_kernel<16, 0, 1, false>), g, b, s, a);
  }
  return hipGetLastError();
}

}  // namespace ltk
