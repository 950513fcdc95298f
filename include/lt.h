/*
 * lt.h -- C ABI of the LazyTensor fused-execution library for AMD MI355X (gfx950).
 *
 * The library implements the hot path of the LazyTensor method (Suhan et al.,
 * "LazyTensor: combining eager execution with domain-specific compilers"):
 * tensor operations are recorded into an IR graph instead of being run
 * (section 3); a barrier cuts the trace of all live tensors (section 4,
 * barrier and DeviceContextArena paragraphs), canonicalises and hashes it,
 * looks it up in a compiled-program cache (section 4, caching paragraph) and
 * runs it as a small number of fused device kernels.
 *
 * Conventions
 *  - Every function returns lt_status (LT_OK = 0).  Nothing throws or aborts.
 *    On error no state changes and lt_last_error() describes the failure.
 *  - "device pointer" = address in the HBM of the context's GPU.
 *    "host pointer"   = ordinary process memory.
 *  - One thread per lt_ctx.  All operands of an op must belong to the same
 *    context (no implicit transfers between devices, section 4.1).
 *  - Tensors are row-major and contiguous.  Shapes have rank <= LT_MAX_RANK.
 */
#ifndef LT_H_
#define LT_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LT_MAX_RANK 6

typedef struct lt_ctx lt_ctx;   /* one per device: the paper's DeviceContextArena       */
typedef uint64_t lt_tensor;     /* unique tensor id (section 4); 0 = invalid; never reused */

typedef enum { LT_F32 = 0, LT_BF16 = 1, LT_I32 = 2, LT_I64 = 3 } lt_dtype;

typedef enum {
  LT_OK = 0,
  LT_ERR_ARG = 1,          /* null pointer, bad rank, bad attribute                      */
  LT_ERR_HANDLE = 2,       /* unknown or released tensor id                              */
  LT_ERR_SHAPE = 3,        /* operand shapes do not fit the op                           */
  LT_ERR_DTYPE = 4,        /* operand dtypes do not fit the op                           */
  LT_ERR_UNSUPPORTED = 5,  /* op or pattern has no lowering (section 4.5 fallback hook)  */
  LT_ERR_OOM = 6,          /* workspace arena exhausted                                  */
  LT_ERR_DEVICE = 7        /* HIP runtime error, or compute requested on a null device   */
} lt_status;

/* Opcodes: the IR stays at framework-op level like the aten:: nodes of figure 1. */
typedef enum {
  LT_OP_NEG = 16, LT_OP_ABS, LT_OP_EXP, LT_OP_LOG, LT_OP_TANH, LT_OP_SQRT, LT_OP_RSQRT,
  LT_OP_RECIP, LT_OP_RELU, LT_OP_GELU, LT_OP_SQUARE, LT_OP_CAST, LT_OP_SIGMOID,
  LT_OP_ADD = 32,          /* inputs (a, b) or (a, b, alpha): a + alpha*b, alpha rank 0    */
  LT_OP_SUB, LT_OP_MUL, LT_OP_DIV, LT_OP_MAXIMUM, LT_OP_MINIMUM,
  LT_OP_RELU_GRAD,         /* (dy, x): dy where x > 0 else 0                                */
  LT_OP_GELU_GRAD,         /* (dy, x): dy * d gelu(x)/dx, exact (erf) form                  */
  LT_OP_EXPAND = 48,       /* attrs LT_ATTR_DIM0+i = output dims                             */
  LT_OP_RESHAPE,           /* attrs LT_ATTR_DIM0+i = output dims                             */
  LT_OP_PERMUTE,           /* attrs LT_ATTR_DIM0+i = source axis of output axis i            */
  LT_OP_NARROW,            /* attrs LT_ATTR_AXIS, _START, _LENGTH: a window along one axis   */
  LT_OP_SLICE_UPDATE,      /* (base, update), attrs LT_ATTR_AXIS, _START: base with that window replaced */
  LT_OP_SUM = 64, LT_OP_AMAX, LT_OP_MEAN, /* attr LT_ATTR_AXIS (last or first axis); none = all */
  LT_OP_SOFTMAX = 80,      /* (x): softmax over the last axis                                */
  LT_OP_SOFTMAX_GRAD,      /* (dy, y): y * (dy - sum(dy*y))                                  */
  LT_OP_LAYER_NORM,        /* (x, gamma, beta), attr LT_ATTR_EPS -> 3 outputs (y, mean, rstd) */
  LT_OP_LAYER_NORM_GRAD,   /* (dy, x, gamma, mean, rstd) -> dx                               */
  LT_OP_XENT,              /* (logits[B,C], labels i32[B]) -> f32[B]: logsumexp - picked     */
  LT_OP_XENT_GRAD,         /* (logits, labels, scale rank 0) -> (softmax - onehot) * scale   */
  LT_OP_MATMUL = 96        /* (a, b), attrs LT_ATTR_TRANS_A/B, optional LT_ATTR_DTYPE;        */
                           /* leading axes of a and b equal, or b a plain matrix             */
} lt_opcode;

typedef enum {
  LT_ATTR_VALUE = 1, LT_ATTR_DTYPE = 2, LT_ATTR_AXIS = 3, LT_ATTR_EPS = 4,
  LT_ATTR_TRANS_A = 5, LT_ATTR_TRANS_B = 6, LT_ATTR_START = 7, LT_ATTR_LENGTH = 8, LT_ATTR_DIM0 = 16
} lt_attr_key;

typedef struct {
  uint16_t key;        /* lt_attr_key                                  */
  uint8_t is_float;    /* 1: use f, 0: use i                           */
  union { int64_t i; double f; } v;
} lt_attr;

/* flags of lt_tensor_from_device */
#define LT_DONATABLE 1u /* a barrier may overwrite this buffer in place (section 4.3)    */

typedef struct {
  uint64_t hash;        /* FNV-1a-64 of the canonical byte string of the cut trace      */
  uint64_t key_bytes;   /* length of that string (second half of the cache key)         */
  int32_t cache_hit;    /* 1 if a cached plan was reused                                */
  int32_t n_nodes;      /* nodes in the cut trace                                       */
  int32_t n_roots;      /* live tensors that were evaluated                             */
  int32_t n_regions;    /* fused regions in the plan                                    */
  int32_t n_launches;   /* kernels launched                                             */
  uint64_t bytes_planned;  /* algorithmic HBM bytes of the plan (inputs once + outputs once) */
  uint64_t flops_planned;  /* 2*M*N*K summed over the plan's contractions               */
  uint64_t ns_collect, ns_hash, ns_lower, ns_launch; /* host time per phase             */
} lt_barrier_info;

typedef struct {
  uint64_t barriers, cache_hits, cache_misses;
  uint64_t nodes_recorded, regions_launched, kernels_launched;
  uint64_t ns_lowering_total;
  uint64_t arena_bytes_in_use, arena_bytes_peak;
  uint64_t live_tensors;
  uint64_t fallback_ops;   /* ops that went through the registered fallback (section 4.5) */
  uint64_t replays;        /* lt_step_replay calls that ran (not counted as barriers)          */
  uint64_t graph_launches; /* steps enqueued as one HIP graph (lt_set_graphs)                  */
  uint64_t graphs_built;   /* HIP graphs captured and instantiated                             */
  uint64_t quick_hits;     /* barriers whose plan was found by the record-time fingerprint      */
} lt_stats_t;

/*
 * Create the context of one device (section 4: one DeviceContextArena per device, alive for
 * the process).  device >= 0: HIP device ordinal; kernels are launched on `hip_stream`
 * (a hipStream_t, may be NULL = default stream).  device = -1: a null device named "CPU:0":
 * it records, hashes, caches and lowers exactly like a real one but launches nothing
 * (lt_fetch fails with LT_ERR_DEVICE); used to test host logic without a GPU.
 * workspace: device pointer to `workspace_bytes` of caller-owned memory in which the library
 * places every tensor a barrier produces and its reduction scratch; BORROWED, must outlive the
 * context.  For a null device it may be NULL with any size (addresses are then only planned).
 */
lt_status lt_init(int device, void* hip_stream, void* workspace, size_t workspace_bytes, lt_ctx** out);
lt_status lt_shutdown(lt_ctx* ctx);

/*
 * Factory: wrap existing device data (section 3: every graph starts at a factory method).
 * dptr: device pointer to a contiguous row-major tensor; BORROWED -- never freed by the
 * library; the caller keeps it valid until every handle bound to it is released or rebound.
 * With LT_DONATABLE the buffer may be overwritten in place when the handle is the destination
 * of lt_assign and nothing else can observe the old value (section 4.3).
 */
lt_status lt_tensor_from_device(lt_ctx* ctx, void* dptr, lt_dtype dtype, int rank,
                                const int64_t* dims, uint32_t flags, lt_tensor* out);

/*
 * Factory: rank-0 scalar.  Exactly +0 and 1 become constants that are part of the graph's
 * identity; every other value (including -0.0) is a dynamic parameter that does not change the
 * hash (section 4.1, special-scalar heuristic).
 */
lt_status lt_scalar(lt_ctx* ctx, lt_dtype dtype, double value, lt_tensor* out);

/*
 * Record one IR-compatible op (section 3): appends a node, runs nothing.  inputs: n_in live
 * handles; attrs: n_attr attributes; outputs: receives n_out new handles (n_out must equal the
 * op's output count: 3 for LT_OP_LAYER_NORM, else 1).  Binary ops broadcast like NumPy.
 */
lt_status lt_op(lt_ctx* ctx, uint16_t opcode, const lt_tensor* inputs, int n_in,
                const lt_attr* attrs, int n_attr, lt_tensor* outputs, int n_out);

/* In-place update as substitution (section 4.3): dst now denotes src's computation. */
lt_status lt_assign(lt_ctx* ctx, lt_tensor dst, lt_tensor src);

/*
 * A view of `base` (section 4.4, in-place operations on views): view_op is LT_OP_PERMUTE,
 * LT_OP_RESHAPE or LT_OP_NARROW with the attributes lt_op takes for it.  The new tensor shares
 * storage with its base as far as a program can tell:
 *  - read as an operand, fetched or evaluated at a barrier, it is the view op applied to the base's
 *    current value (the paper's forward sequence; derived again whenever the base was replaced);
 *  - lt_assign(view, src) gives the view the value src AND rebuilds the base from it with the
 *    inverse of the view op -- the inverse permutation, the reshape back, the base with the window
 *    replaced (the backward sequence) -- through every level when the base is itself a view; other
 *    views of the same base see the change.  src must have the view's dtype and shape (LT_ERR_SHAPE).
 * Everything is recorded in the one IR graph: no memory is shared, nothing runs.  A base released
 * while views of it are alive stays evaluated at barriers until its last view is released.
 */
lt_status lt_view(lt_ctx* ctx, lt_tensor base, uint16_t view_op, const lt_attr* attrs, int n_attr, lt_tensor* out);

/* UnregisterTensor (section 4): the handle dies; its pending computation is no longer a root. */
lt_status lt_release(lt_ctx* ctx, lt_tensor t);

/*
 * The same for n handles at once (ts: host array of n ids).  A front end that learns of dead
 * tensors one by one (a garbage collector) can hand them over in one call before the next
 * barrier: liveness only matters when the trace is cut.  Every valid id is released; an unknown
 * one is skipped and reported as LT_ERR_HANDLE after the others have been released.
 */
lt_status lt_release_many(lt_ctx* ctx, const lt_tensor* ts, size_t n);

/*
 * Barrier (section 4: mark_step / LazyTensorBarrier).  Evaluates the pending computation of
 * every live tensor: cut, canonical order, hash, cache lookup, lowering on a miss, kernel
 * launches on the context's stream, then every evaluated handle is rebound to its data.
 * blocking != 0 waits for the stream.  info may be NULL.
 * Errors: LT_ERR_UNSUPPORTED (an op pattern of the trace has no lowering), LT_ERR_OOM (the plan's
 * results and temporaries do not fit the workspace; found before anything is launched).  Either way
 * nothing ran and the trace stays pending.  LT_ERR_DEVICE: a HIP call failed; launches already
 * enqueued may have updated donated buffers, side streams have been joined, the trace stays pending.
 */
lt_status lt_barrier(lt_ctx* ctx, int blocking, lt_barrier_info* info);

/*
 * lt_barrier for callers that cannot allocate device memory or create runtime objects while they
 * run it: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same contract as lt_barrier, except that
 *  - the reduction scratch (partial results, tickets) and every temporary of the plan (region
 *    outputs that are not results, partial products of split contractions) live in a 16 MiB
 *    array in the library's own device image instead of the workspace: 4 MiB + 4 KiB of it are the
 *    reduction scratch, 12,578,816 bytes are handed to the plan's temporaries front to back
 *    (each rounded up to 256 bytes, none reused inside a step).  A plan that needs more fails
 *    with LT_ERR_OOM before anything is launched (the trace stays pending: lt_barrier can
 *    still run it).  Results that are not written in place over a donated input are placed in the
 *    workspace given to lt_init, as always -- host-side bookkeeping over caller-owned memory;
 *  - every launch goes to the context's stream: no side streams, no events, no per-launch timing;
 *  - it calls no hipMalloc / hipFree, no allocating library routine, and no hipMemsetAsync (the
 *    tickets are cleared by a small kernel).  With blocking = 0 it makes no synchronising call either.
 * The array's device address is looked up once per device in lt_init; if that failed, this call
 * returns LT_ERR_DEVICE with the reason.  Every context on a GPU shares that GPU's array, which
 * keeps the contents of the last call: calls that overlap in time on one GPU (two contexts, or
 * two streams) race.  The array stays allocated on every GPU the library has run on until the
 * process ends.
 */
lt_status lt_barrier_static(lt_ctx* ctx, int blocking, lt_barrier_info* info);

/*
 * IR-incompatible op (section 3): blocking barrier if `t` is pending, then copy its data to
 * host_dst (host pointer, nbytes must equal the tensor's byte size).
 */
lt_status lt_fetch(lt_ctx* ctx, lt_tensor t, void* host_dst, size_t nbytes);

/* Device pointer of a materialised tensor; LT_ERR_HANDLE while it is still pending. */
lt_status lt_device_ptr(lt_ctx* ctx, lt_tensor t, void** dptr);

/* dtype / rank / dims (dims must have room for LT_MAX_RANK entries); any argument may be NULL. */
lt_status lt_shape(lt_ctx* ctx, lt_tensor t, lt_dtype* dtype, int* rank, int64_t* dims);

/*
 * Running a step again without tracing it (section 7 of the paper lists this as future work: when
 * the user guarantees that the computation has not changed, recording it can be skipped).
 *
 * lt_step_capture: a handle on the step that the LAST barrier of ctx ran -- its compiled plan, the
 * tensors whose data were the plan's inputs (the trace's device_data leaves, in the order of the
 * canonical numbering), the values of its non-special scalars (same order) and the tensors that
 * received its results.  It holds no device memory and stays valid until lt_step_free, the
 * context's shutdown, or a call that clears the plan cache (lt_set_fusion), after which
 * lt_step_replay returns LT_ERR_ARG.  Errors: LT_ERR_ARG no barrier has run; LT_ERR_HANDLE an
 * input tensor of the step has been released (it could not be named again);
 * LT_ERR_UNSUPPORTED the plan writes over an input's buffer and the result does not belong to
 * that same tensor (only x <- f(x) may be repeated in place), or during the step lt_assign gave
 * a tensor the plain data or scalar of another tensor (src not pending: the tensor only becomes a
 * second name of src's buffer, which leaves nothing in the trace for the plan to repeat).
 *
 * lt_step_replay: runs the plan on the CURRENT data of the same input tensors and binds the
 * results to the same result tensors, exactly as the barrier did (donated inputs are updated in
 * place, other results get fresh workspace memory, the tensors' previous results are released).
 * scalars: NULL = the captured values, else n_scalars doubles in canonical order (lt_step_scalars
 * gives the captured ones, e.g. to find the learning rate among them).  Nothing is recorded,
 * cut, hashed or looked up.  The caller guarantees that tracing the step again would give the
 * same trace; checked are only: no trace is pending (LT_ERR_ARG), every input still exists
 * (LT_ERR_HANDLE) as plain data of the captured dtype, shape and donation flag (LT_ERR_SHAPE), an
 * input updated in place is not shared with another tensor (LT_ERR_ARG).  On an error nothing has
 * run.  Views of result tensors are brought up to date when they are next used, as after a
 * barrier.  info may be NULL (hash, key_bytes, n_nodes, ns_hash and ns_lower are 0).
 *
 * lt_step_scalars: number of scalars of the step; copies up to cap captured values to out (out
 * may be NULL).  -1 for a NULL step.
 *
 * lt_tensor_rebind: a data tensor made by lt_tensor_from_device now names other device memory of
 * the same dtype and shape (the next batch), keeping its id, so that a captured step reads it.
 * Ownership as for lt_tensor_from_device.  LT_ERR_ARG: a result tensor (library memory), a view,
 * a tensor the pending trace has read, a misaligned or null pointer.
 */
typedef struct lt_step lt_step;
lt_status lt_step_capture(lt_ctx* ctx, lt_step** out);
lt_status lt_step_replay(lt_ctx* ctx, lt_step* step, const double* scalars, int n_scalars, int blocking,
                         lt_barrier_info* info);
int lt_step_scalars(const lt_step* step, double* out, int cap);
void lt_step_free(lt_step* step);
lt_status lt_tensor_rebind(lt_ctx* ctx, lt_tensor t, void* device_ptr);

/*
 * Text form of the pending trace in the layout of figure 1(a) of the paper.  Writes at most
 * cap bytes (NUL-terminated when cap > 0) and always stores the full length in *len.
 */
lt_status lt_dump_ir(lt_ctx* ctx, char* buf, size_t cap, size_t* len);

/* Region list of the plan used by the last barrier, one region per line. Same buffer rules. */
lt_status lt_dump_plan(lt_ctx* ctx, char* buf, size_t cap, size_t* len);

/*
 * Stream schedule of the plan used by the last barrier, one launch per line in enqueue order:
 * "L<i> <kind> R<region> stream=<0..3> slot=<quarter of the reduction scratch> record=<0|1>
 * waits=[<earlier launches on other streams>] reads=[<storages>] writes=[<storages>]".  Stream 0
 * is the caller's; a storage is p<n> (the caller's buffer number n of the trace, a donated output
 * included) or t<n> (temporary number n of the plan).  Same buffer rules.
 */
lt_status lt_dump_schedule(lt_ctx* ctx, char* buf, size_t cap, size_t* len);

/* Canonical byte string of the last barrier's trace (what was hashed).  Same buffer rules. */
lt_status lt_dump_key(lt_ctx* ctx, uint8_t* buf, size_t cap, size_t* len);

lt_status lt_stats(lt_ctx* ctx, lt_stats_t* out);

/*
 * Per-kernel timing of the last barrier, measured with HIP events on the context's stream
 * when profiling is on.  lt_set_profiling(ctx, 1) makes every following barrier record events
 * around each launch; lt_last_launches returns up to cap entries.
 */
typedef struct {
  char kernel[48];       /* kernel family name                              */
  int32_t region;        /* index of the region in the plan                 */
  float ms;              /* elapsed device time                             */
  uint64_t bytes;        /* algorithmic bytes of the region                 */
  uint64_t flops;        /* 2MNK of the region's contraction (0 otherwise)  */
} lt_launch_record;
lt_status lt_set_profiling(lt_ctx* ctx, int on);
lt_status lt_last_launches(lt_ctx* ctx, lt_launch_record* out, int cap, int* n);

/*
 * Streams a barrier may spread its launches over (1 .. 4, default 4).  Launches of a plan that
 * do not depend on each other (section 4: the barrier hands the device a whole graph, not a
 * sequence) run on up to n - 1 side streams of the library's own next to the caller's stream;
 * every barrier forks them from the caller's stream and joins them into it again before it
 * returns, so the caller sees the ordering of a single stream.  n = 1 keeps every launch on the
 * caller's stream.  A plan whose temporaries do not fit the workspace without being recycled
 * inside the step also runs on one stream.  Barriers that record per-launch timings
 * (lt_set_profiling) run on one stream so that the timings are those of the kernels alone.
 * Errors: LT_ERR_ARG (n out of range).
 */
lt_status lt_set_streams(lt_ctx* ctx, int n);

/*
 * Ops without a lowering (section 4.5: every tensor op must give a correct program, if a slower
 * one).  A registered fallback makes lt_op handle such an op -- an opcode at or above
 * LT_OP_CUSTOM, or a reduction over an axis pattern the kernels do not cover (a middle axis; axis 0
 * of a tensor of rank > 2) -- in the paper's three steps, at the moment it is recorded:
 *   1. the pending trace is evaluated (a blocking barrier), so every input is plain data;
 *   2. fn is called with run = 0 to state the outputs' dtype and shape (opcodes the library knows
 *      skip this), then, with output buffers taken from the workspace, with run = 1 to compute
 *      them by whatever eager implementation the caller has, on `hip_stream` or synchronously;
 *   3. the results are new tensors holding data: a new IR graph starts from them.
 * inputs / outputs: host arrays of descriptors; dptr is a device pointer (NULL for a rank-0 scalar
 * input, whose value is in `scalar`).  fn returns 0 on success; anything else makes lt_op fail
 * with LT_ERR_UNSUPPORTED and leaves no trace of the op.  Without a fallback such ops fail with
 * LT_ERR_UNSUPPORTED (unknown opcodes when recorded, the reductions at the barrier).
 */
#define LT_OP_CUSTOM 1024
typedef struct {
  void* dptr;
  int32_t dtype;            /* lt_dtype */
  int32_t rank;
  int64_t dims[LT_MAX_RANK];
  int32_t is_scalar;        /* 1: a rank-0 scalar that lives on the host: use `scalar` */
  double scalar;
} lt_tensor_desc;
typedef int (*lt_fallback_fn)(void* user, uint16_t opcode, const lt_tensor_desc* inputs, int n_in, const lt_attr* attrs,
                              int n_attr, lt_tensor_desc* outputs, int n_out, int run, void* hip_stream);
lt_status lt_set_fallback(lt_ctx* ctx, lt_fallback_fn fn, void* user);

/*
 * Hashing while recording (section 7 of the paper: graph hashing is part of the per-step overhead
 * that is paid even on a cache hit).  Every recorded node is taken into a 128-bit fingerprint of
 * the pending trace as it is appended (opcode, type, shape, attributes, operands by record index,
 * which earlier leaf shares a leaf's buffer).  At a barrier the fingerprint, the live roots and
 * what each root could donate identify the canonical form of the cut, so a trace that this
 * context has seen before finds its plan without the canonical walk, serialisation and FNV hash;
 * a trace seen for the first time takes the canonical path (hash and key bit-exact as specified)
 * and is then remembered by fingerprint.  The fingerprint is not the cache key: lt_barrier_info
 * still reports the canonical hash, and lt_dump_key the canonical string.  mode 0: off; 1: on
 * (default); 2: on, and every fingerprint hit is checked against the canonical key (a
 * disagreement fails the barrier with LT_ERR_ARG and a message that says so) -- the tests run
 * in this mode.  A wrong hit needs a collision of two independent 64-bit lanes.  lt_stats counts
 * quick_hits.
 */
lt_status lt_set_quick_lookup(lt_ctx* ctx, int mode);

/*
 * One HIP graph per cached plan and set of addresses (section 7 of the paper: the cost that is
 * left on a cache hit is per-operation host work; here that is one launch and up to two events
 * per kernel).  With on != 0, a barrier or lt_step_replay whose plan, storage addresses and
 * scalars are those of an earlier step of this context enqueues that step's instantiated graph
 * with one call.  The arguments of a plan's launches depend on nothing else, so the graph is the
 * same work; a set of addresses is captured when it is seen for the second time (a training loop
 * that updates its parameters in place alternates between two sets, because a step's results are
 * placed before the previous step's are released), and a plan keeps at most four graphs, least
 * recently used out first.  Captures run on a stream of the library's own (default priority) and
 * contain kernel nodes only -- no memset, no copy.  Not used by lt_barrier_static, under
 * lt_set_profiling, or when the workspace cannot hold a plan's temporaries all at once.  If a
 * capture or instantiation fails the plan goes back to kernel-by-kernel launches for good and
 * the step still runs.  Default: off.  lt_stats counts graph_launches and graphs_built.
 */
lt_status lt_set_graphs(lt_ctx* ctx, int on);

/*
 * Debugging switch for the invariant of section 3 (a compiled trace is equivalent to running the
 * recorded operations one by one): with on = 0 every recorded op is lowered to a region, hence a
 * kernel, of its own -- views stay addressing, special scalars are still folded, in-place updates
 * still happen -- and the results must agree with those of the fused plans to rounding.  Changing
 * the setting waits for the stream and empties the plan cache.  Default: on.
 */
lt_status lt_set_fusion(lt_ctx* ctx, int on);

/* Message of the last failure on this context (or of lt_init when ctx is NULL). */
const char* lt_last_error(lt_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* LT_H_ */
