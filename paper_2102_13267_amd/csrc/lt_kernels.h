// Kernel argument blocks shared by the host lowering pass and the HIP kernels.
//
// Every fused region is run by one kernel family.  What varies per region -- the
// elementwise chain -- is not compiled: it is a small bytecode program that lives in
// the kernel-argument segment (read through scalar loads) and is interpreted with the
// value slots held in vector registers.  The paper leaves code generation to its
// backend compiler (section 4, "lowering"); this build replaces that compiler with an
// interpreter so that a cache miss costs microseconds, not a JIT run.
#ifndef LT_KERNELS_H_
#define LT_KERNELS_H_

#include <stdint.h>

namespace ltk {

constexpr int kMaxIn = 8;       // array inputs of one program
constexpr int kMaxOut = 8;      // outputs of one program
constexpr int kMaxScal = 32;    // scalar table: dynamic scalars and immediates
constexpr int kMaxCode = 48;    // instructions
constexpr int kSlots = 32;      // value slots a program may name (kernels hold 16 or 32)
constexpr int kVec = 4;         // elements handled per lane and interpreted instruction

// device dtypes of loads / stores
enum : uint32_t { kF32 = 0, kBF16 = 1, kI32 = 2, kI64 = 3 };

// how an input is addressed from the flat index i of the iteration space [rows, cols]
enum : uint32_t {
  kFull = 0,     // element i
  kRowVec = 1,   // element i % cols   (a vector broadcast along rows, e.g. a bias)
  kColVec = 2,   // element i / cols   (one value per row)
  kScalar = 3,   // element 0
  kStrided = 4   // sum_k coord_k(i) * stride[k] over the (<= 4-d) iteration space
};

// interpreter opcodes.  Unary ops come first: the interpreter reads operand b only for
// op >= kAdd.  Operand a is always a value slot; a scalar-table operand can only be b (or c of
// kFma), so non-commutative ops have a reversed form ("kRsub": b - a).
enum : uint32_t {
  kMov = 0, kNeg, kAbs, kExp, kLog, kTanh, kSqrt, kRsqrt, kRecip, kRelu, kGelu, kSquare,
  kSigmoid, kRoundBf16,
  kAdd, kSub, kRsub, kMul, kDiv, kRdiv, kMax, kMin,
  kReluGrad,     // b > 0 ? a : 0     (a = dy, b = x)
  kRreluGrad,    // a > 0 ? b : 0
  kGeluGrad,     // a * gelu'(b)
  kRgeluGrad,    // b * gelu'(a)
  kFma,          // a*b + c
  kSplat,        // b (a scalar-table entry) replicated
  kNumOps
};

// instruction word: op[7:0] dst[12:8] a[18:13] b[24:19] c[30:25];
// operand < 32: value slot; operand >= 32: scal[operand - 32]
inline uint32_t encode(uint32_t op, uint32_t dst, uint32_t a, uint32_t b = 0, uint32_t c = 0) {
  return op | (dst << 8) | (a << 13) | (b << 19) | (c << 25);
}

// how the kernels fetch an input on their fast path (full 4-vectors)
enum : uint32_t {
  kFetchVec4 = 0,   // one 16-byte (8-byte for bf16) load of four consecutive elements
  kFetchBcast = 1,  // one element, replicated to the four lanes
  kFetchSlow = 2    // element by element through the general addressing code
};

struct EwIn {
  const void* ptr;
  uint32_t mode;
  uint32_t dtype;
  uint32_t fetch;      // kFetch*: decided by the host from mode, cols and alignment
  uint32_t pad;
  int64_t stride[4];   // kStrided only, in elements
};

struct EwOut {
  void* ptr;
  uint32_t dtype;
  uint32_t slot;       // value slot stored
  uint32_t scalar;     // 1: a rank-0 result, written once (by flat index 0)
  uint32_t pad;
};

struct EwProg {
  uint32_t n_in, n_out, n_code, anchor_slot;  // anchor_slot: where a reduction / GEMM result enters
  uint32_t vec_ok;     // 1: cols % 4 == 0, so a 4-vector never straddles a row
  uint32_t full_vec_ok;  // 1: every 4-vector of the flat space starts at a multiple of 4
  uint32_t cols;       // last dimension of the iteration space (>= 1)
  uint32_t n_slots;    // value slots the program uses (selects the 16- or 32-slot kernel)
  uint32_t needs_divmod;  // 1: some input is addressed by i / cols or i % cols
  uint32_t fast;       // 1: n % 4 == 0, every input fetches as vec4 / broadcast, outputs contiguous
  uint32_t all_f32;    // 1: every input and output is fp32
  uint32_t pad2;
  uint64_t n;          // elements of the iteration space
  uint32_t dims[4];    // iteration space collapsed to 4 dims (kStrided addressing)
  EwIn in[kMaxIn];
  EwOut out[kMaxOut];
  float scal[kMaxScal];
  uint32_t code[kMaxCode];
};

// ---- elementwise region -----------------------------------------------------------
struct EwArgs {
  EwProg prog;
};

// ---- reductions ---------------------------------------------------------------------
enum : uint32_t { kRedSum = 0, kRedMax = 1, kRedMean = 2 };

// row reduction: out[r] = post(reduce_c pro(x[r, c]))
struct RowArgs {
  EwProg pro;          // iteration space [rows, cols]; its result is slot pro.anchor_slot
  EwProg post;         // iteration space [rows]
  uint32_t rows, cols, red, threads_per_row;
  // filled in by launch_row_reduce for the streamed variant: input numbers of the (up to two) fp32
  // inputs read in full and of the (up to one) fp32 vector broadcast along rows; counts
  uint32_t vin[2], rin, n_vin, n_rin, pad;
};

// global reduction, single launch: per-workgroup partials, the last workgroup to finish
// combines them, then runs the post program (scalar epilogue and optional finaliser)
struct AllArgs {
  EwProg pro;          // iteration space = the reduced tensor, flat
  EwProg post;         // iteration space: 1 element, or the finaliser's shape
  float* partials;     // [gridDim.x]
  uint32_t* ticket;    // zero before launch; reset by the kernel
  uint32_t red, pad;
  uint64_t count;      // elements reduced (for mean)
};

// column reduction over axis 0 of [rows, cols]
struct ColArgs {
  EwProg pro;          // iteration space [rows, cols]
  EwProg post;         // iteration space [cols]
  float* partials;     // [gridDim.y, cols]
  uint32_t* tickets;   // [gridDim.x], zero before launch; reset by the kernel
  uint32_t rows, cols, red;
  uint32_t narrow;     // set by launch_col_reduce: at most 64 columns and 65536 elements, one workgroup (see the kernel)
  // filled in by launch_col_reduce for the streamed variants: input numbers of the (up to two)
  // inputs read in full and of the (up to two) per-row inputs (kColVec), padded with the first
  uint32_t vin[2], cin[2];
};

// ---- row operators with a fixed body ---------------------------------------------------
enum : uint32_t { kSoftmax = 0, kSoftmaxGrad, kLayerNorm, kLayerNormGrad, kXent, kXentGrad };

struct RowOpArgs {
  uint32_t op, rows, cols, threads_per_row;
  const void* in[5];
  uint32_t in_dtype[5];
  void* out[3];
  uint32_t out_dtype[3];
  float eps;           // layer norm
  float scale;         // xent_grad
};

// ---- contraction ------------------------------------------------------------------------
// C[b] = post(A[b] * B[b]); A is M x K, B is K x N, element (i, j) of an operand is at
// base + b0*sb0 + b1*sb1 + i*s_row + j*s_col (element strides), so transposes, batched
// operands and head-split layouts are all addressing, never copies.
struct GemmOperand {
  const void* ptr;
  int64_t s_row, s_col, s_b0, s_b1;
};

struct GemmArgs {
  GemmOperand a, b;
  uint32_t m, n, k;
  uint32_t batch0, batch1;   // batch = batch0 * batch1 (b = b0 * batch1 + b1)
  uint32_t in_dtype;         // kF32 or kBF16 (both operands)
  uint32_t tiles_m, tiles_n;
  // where output element (b0, b1, row, col) goes: b0*o_b0 + b1*o_b1 + row*o_row + col (elements).
  // Contiguous [batch, m, n] by default; a permuted layout when the product's only reader is a
  // permutation (head merge), which then costs nothing.
  int64_t o_b0, o_b1, o_row;
  // Split-K (the LDS-staged kernels): `splits` workgroups share an output tile, each contracting a
  // slice of k and leaving its fp32 partial product, row major, in split_ws[split]; the post
  // program then runs in a second launch (SplitPostArgs) that adds the partials up in split order.
  uint32_t splits, tile_m, tile_n;   // workgroup tile: 128 rows, 128 or 64 columns
  uint32_t direct;           // 1: the one-launch kernel for small fp32 products (tiles of 32 x 32 or 64 x 32)
  float* split_ws;           // [splits][batch * m * n] floats
  // The one-launch small kernel (direct = 1) with splits > 1: `splits` workgroups share a tile;
  // split_ws then holds [tile][split][tile_m x tile_n] partial tiles and tickets[tile]
  // counts the workgroups that have left theirs (zero before the launch; the last one adds the
  // partials up in split order, runs the post program and resets the ticket).
  uint32_t* tickets;
  EwProg post;               // iteration space = the output
  // The one-launch small kernel can carry the column sums of its B operand ([k, n], rows
  // contiguous) along: a weight gradient x^T dy and the bias gradient sum_rows(dy) read the same
  // dy.  col_sum = 1: the workgroups of the first tile row add up the columns of B they fetch
  // anyway (col_red: kRedSum or kRedMean) and run col_post on them, iteration space [n].
  uint32_t col_sum, col_red;
  EwProg col_post;
};

// second launch of a split-K contraction: anchor = sum over splits of ws[split][i], then the
// contraction's post program over the flat output, exactly like an elementwise region
struct SplitPostArgs {
  EwProg prog;
  const float* ws;
  uint32_t splits, pad;
  uint64_t stride;           // floats between consecutive splits (= elements of the output)
};

// ---- window update -------------------------------------------------------------------------
// out = base with the window [start, start + len) along one axis replaced by upd.  The tensors are
// seen as [outer, dim, inner] (base, out) and [outer, len, inner] (upd), dense.  window_only: out
// is base's own buffer (updated in place), so only the window is written.
struct SliceArgs {
  const void* base;
  const void* upd;
  void* out;
  uint64_t n;              // elements this launch walks: the window (window_only) or all of out
  uint64_t dim, inner, start, len;
  uint32_t elem_bytes;     // 2, 4 or 8
  uint32_t window_only;
};

// Argument blocks travel by value in the kernel argument segment, which holds 4 KiB.
static_assert(sizeof(EwArgs) <= 4096 && sizeof(RowArgs) <= 4096 && sizeof(AllArgs) <= 4096 && sizeof(ColArgs) <= 4096 &&
                  sizeof(GemmArgs) <= 4096 && sizeof(SplitPostArgs) <= 4096 && sizeof(SliceArgs) <= 4096,
              "a kernel's argument block must fit the kernel argument segment");

}  // namespace ltk
#endif  // LT_KERNELS_H_
