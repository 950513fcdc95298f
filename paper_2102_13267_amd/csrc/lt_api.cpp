// C ABI, part 1: context, factories, op recording (shape / dtype inference), in-place
// substitution, release and the figure-1 style IR dump.  Host only; nothing here touches the GPU
// except lt_init / lt_shutdown.
#include <hip/hip_runtime_api.h>

#include <algorithm>
#include <cmath>
#include <cstdio>

#include "lt_core.h"
#include "lt_launch.h"

namespace lt {

static thread_local std::string g_init_error;

lt_status fail(lt_ctx* ctx, lt_status code, const std::string& msg) {
  if (ctx) ctx->err = msg;
  else g_init_error = msg;
  return code;
}

size_t dtype_size(uint8_t d) { return d == LT_F32 ? 4 : d == LT_BF16 ? 2 : d == LT_I32 ? 4 : 8; }
const char* dtype_name(uint8_t d) { return d == LT_F32 ? "f32" : d == LT_BF16 ? "bf16" : d == LT_I32 ? "s32" : "s64"; }
static bool is_float(uint8_t d) { return d == LT_F32 || d == LT_BF16; }

int64_t numel(const int64_t* dims, int rank) {
  int64_t n = 1;
  for (int i = 0; i < rank; ++i) n *= dims[i];
  return n;
}

const char* op_name(uint16_t op) {
  switch (op) {
    case OP_DEVICE_DATA: case OP_SCALAR_PARAM: return "xla::device_data";
    case OP_CONSTANT: return "prim::Constant";
    case LT_OP_NEG: return "aten::neg"; case LT_OP_ABS: return "aten::abs"; case LT_OP_EXP: return "aten::exp";
    case LT_OP_LOG: return "aten::log"; case LT_OP_TANH: return "aten::tanh"; case LT_OP_SQRT: return "aten::sqrt";
    case LT_OP_RSQRT: return "aten::rsqrt"; case LT_OP_RECIP: return "aten::reciprocal";
    case LT_OP_RELU: return "aten::relu"; case LT_OP_GELU: return "aten::gelu"; case LT_OP_SQUARE: return "aten::square";
    case LT_OP_CAST: return "aten::to"; case LT_OP_SIGMOID: return "aten::sigmoid";
    case LT_OP_ADD: return "aten::add"; case LT_OP_SUB: return "aten::sub"; case LT_OP_MUL: return "aten::mul";
    case LT_OP_DIV: return "aten::div"; case LT_OP_MAXIMUM: return "aten::maximum"; case LT_OP_MINIMUM: return "aten::minimum";
    case LT_OP_RELU_GRAD: return "aten::threshold_backward"; case LT_OP_GELU_GRAD: return "aten::gelu_backward";
    case LT_OP_EXPAND: return "aten::expand"; case LT_OP_RESHAPE: return "aten::view"; case LT_OP_PERMUTE: return "aten::permute";
    case LT_OP_NARROW: return "aten::narrow"; case LT_OP_SLICE_UPDATE: return "aten::slice_scatter";
    case LT_OP_SUM: return "aten::sum"; case LT_OP_AMAX: return "aten::amax"; case LT_OP_MEAN: return "aten::mean";
    case LT_OP_SOFTMAX: return "aten::_softmax"; case LT_OP_SOFTMAX_GRAD: return "aten::_softmax_backward_data";
    case LT_OP_LAYER_NORM: return "aten::native_layer_norm";
    case LT_OP_LAYER_NORM_GRAD: return "aten::native_layer_norm_backward";
    case LT_OP_XENT: return "aten::nll_loss_of_log_softmax";
    case LT_OP_XENT_GRAD: return "aten::nll_loss_of_log_softmax_backward";
    case LT_OP_MATMUL: return "aten::matmul";
    default: return "?";
  }
}

Buffer::~Buffer() {
  if (owned && arena && ptr) arena->release(ptr);
}

void Arena::init(void* p, size_t bytes) {
  base = p ? (uintptr_t)p : (uintptr_t)0x100000;   // a null device plans addresses it never touches
  size = bytes & ~(size_t)255;
  free_blocks.clear();
  used.clear();
  if (size) free_blocks[0] = size;
  in_use = peak = 0;
}

void* Arena::alloc(size_t bytes) {
  size_t need = (std::max<size_t>(bytes, 1) + 255) & ~(size_t)255;
  for (auto it = free_blocks.begin(); it != free_blocks.end(); ++it) {
    if (it->second >= need) {
      uintptr_t off = it->first;
      size_t len = it->second;
      free_blocks.erase(it);
      if (len > need) free_blocks[off + need] = len - need;
      used[off] = need;
      in_use += need;
      peak = std::max(peak, in_use);
      return (void*)(base + off);
    }
  }
  return nullptr;
}

void Arena::release(void* p) {
  uintptr_t off = (uintptr_t)p - base;
  auto u = used.find(off);
  if (u == used.end()) return;
  size_t len = u->second;
  used.erase(u);
  in_use -= len;
  auto next = free_blocks.lower_bound(off);
  if (next != free_blocks.end() && off + len == next->first) {
    len += next->second;
    next = free_blocks.erase(next);
  }
  if (next != free_blocks.begin()) {
    auto prev = std::prev(next);
    if (prev->first + prev->second == off) {
      prev->second += len;
      return;
    }
  }
  free_blocks[off] = len;
}

// `hidden`: also find a handle that its owner has released but that lives on as the base of views
static Handle* find(lt_ctx* ctx, lt_tensor t, bool hidden = false) {
  auto it = ctx->handles.find(t);
  if (it == ctx->handles.end() || (it->second.released && !hidden)) return nullptr;
  return &it->second;
}

static void unbind(Handle* h) {
  if (h->kind == H_DATA && h->buf) h->buf->data_refs -= 1;
  h->buf.reset();
}

static Handle* new_handle(lt_ctx* ctx) {
  uint64_t id = ctx->next_id++;
  Handle& h = ctx->handles[id];
  h.id = id;
  return &h;
}

static lt_status record_op(lt_ctx* ctx, uint16_t opcode, const lt_tensor* inputs, int n_in, const lt_attr* attrs, int n_attr,
                           lt_tensor* outputs, int n_out, bool hidden);
static lt_status assign(lt_ctx* ctx, lt_tensor dst_id, lt_tensor src_id, bool hidden);
static lt_status run_fallback(lt_ctx* ctx, uint16_t opcode, const lt_tensor* inputs, int n_in, const lt_attr* attrs, int n_attr,
                              lt_tensor* outputs, int n_out, const Node* inferred);

// Drop a handle for good.  A view gives up its hold on its base; a base that its owner had
// already released goes with its last view.
static void erase_handle(lt_ctx* ctx, Handle* h) {
  const uint64_t base = h->view_base;
  unbind(h);
  ctx->handles.erase(h->id);
  if (base) {
    Handle* b = find(ctx, base, true);
    if (b && --b->view_refs == 0 && b->released) erase_handle(ctx, b);
  }
}

static lt_status release_one(lt_ctx* ctx, Handle* h) {
  if (h->view_refs > 0) {   // still the storage behind live views: hidden, not gone
    h->released = true;
    return LT_OK;
  }
  erase_handle(ctx, h);
  return LT_OK;
}

// A view's value is its view op applied to the CURRENT value of its base (section 4.4, the
// "forward sequence"): derive it again if the base has been replaced since it was last derived.
static lt_status refresh(lt_ctx* ctx, Handle* h) {
  if (!h->view_base) return LT_OK;
  Handle* b = find(ctx, h->view_base, true);
  if (!b) return fail(ctx, LT_ERR_HANDLE, "internal: a view has lost its base");
  lt_status st = refresh(ctx, b);
  if (st != LT_OK || h->seen == b->version) return st;
  lt_tensor tid = 0;
  const lt_tensor bid = b->id;
  st = record_op(ctx, h->view_op, &bid, 1, h->view_attrs, h->view_n_attr, &tid, 1, true);
  if (st != LT_OK) return st;
  Handle* t = find(ctx, tid, true);
  unbind(h);
  h->kind = H_PENDING;
  h->node = t->node;
  h->slot = 0;
  h->donor.reset();
  h->memo_epoch = ~0ull;
  h->version++;
  h->seen = b->version;
  ctx->handles.erase(tid);
  return LT_OK;
}

// Before the trace is cut, and before anything reads a view from outside: every live view holds
// the value its base has now.
lt_status refresh_views(lt_ctx* ctx) {
  std::vector<uint64_t> ids;
  for (auto& kv : ctx->handles)
    if (kv.second.view_base) ids.push_back(kv.first);
  for (uint64_t id : ids) {
    Handle* h = find(ctx, id, true);
    if (!h) continue;
    const lt_status st = refresh(ctx, h);
    if (st != LT_OK) return st;
  }
  return LT_OK;
}

// Append a node to the trace and take it into the trace's fingerprint.
static void push_node(lt_ctx* ctx, Node&& n) {
  Fingerprint& f = ctx->trace_fp;
  f.mix((uint64_t)n.op | ((uint64_t)n.dtype << 16) | ((uint64_t)n.rank << 24) | ((uint64_t)n.n_attr << 32) | ((uint64_t)n.n_in << 40) |
        ((uint64_t)n.n_out << 48));
  for (int d = 0; d < n.rank; ++d) f.mix((uint64_t)n.dims[d]);
  for (int k = 0; k < n.n_attr; ++k) {
    f.mix((uint64_t)n.attrs[k].key | ((uint64_t)n.attrs[k].is_float << 16));
    uint64_t payload;
    if (n.attrs[k].is_float) std::memcpy(&payload, &n.attrs[k].v.f, 8);
    else payload = (uint64_t)n.attrs[k].v.i;
    f.mix(payload);
  }
  for (int k = 0; k < n.n_in; ++k) f.mix(((uint64_t)(uint32_t)n.ins[k].node << 8) | (uint64_t)(uint8_t)n.ins[k].slot);
  if (n.op == OP_DEVICE_DATA) {
    // which earlier leaf names the same buffer (itself: none) -- the alias class of the cache key
    const int32_t self = (int32_t)ctx->nodes.size();
    f.mix((uint64_t)(uint32_t)ctx->leaf_of_buffer.emplace(n.buffer.get(), self).first->second);
  }
  ctx->nodes.push_back(std::move(n));
}

// operand reference of a handle in the trace being recorded; leaves are created on first use
static Val use(lt_ctx* ctx, Handle* h) {
  if (h->kind == H_PENDING) return Val{h->node, h->slot};
  if (h->memo_epoch != ctx->epoch || h->memo_node < 0) {
    Node n;
    n.dtype = h->dtype;
    n.rank = h->rank;
    n.src = h->id;
    std::memcpy(n.dims, h->dims, sizeof(n.dims));
    if (h->kind == H_DATA) {
      n.op = OP_DEVICE_DATA;
      n.buffer = h->buf;
    } else {
      const double v = h->value;
      const bool special = (v == 1.0) || (v == 0.0 && !std::signbit(v));
      if (special) {
        n.op = OP_CONSTANT;
        n.n_attr = 1;
        n.attrs[0].key = LT_ATTR_VALUE;
        n.attrs[0].is_float = is_float(h->dtype) ? 1 : 0;
        if (n.attrs[0].is_float) n.attrs[0].v.f = v;
        else n.attrs[0].v.i = (int64_t)v;
      } else {
        n.op = OP_SCALAR_PARAM;
        n.value = v;
      }
    }
    push_node(ctx, std::move(n));
    h->memo_epoch = ctx->epoch;
    h->memo_node = (int32_t)ctx->nodes.size() - 1;
    ctx->stats.nodes_recorded++;
  }
  return Val{h->memo_node, 0};
}

static bool broadcast(const int64_t* a, int ra, const int64_t* b, int rb, int64_t* out, int* rout) {
  int r = std::max(ra, rb);
  for (int i = 0; i < r; ++i) {
    int64_t da = i < ra ? a[ra - 1 - i] : 1, db = i < rb ? b[rb - 1 - i] : 1;
    if (da != db && da != 1 && db != 1) return false;
    out[r - 1 - i] = (da == 0 || db == 0) ? 0 : std::max(da, db);
  }
  *rout = r;
  return true;
}

static uint8_t promote(const Handle* a, const Handle* b) {
  if (a->dtype == b->dtype) return a->dtype;
  if (a->rank == 0 && b->rank > 0) return b->dtype;
  if (b->rank == 0 && a->rank > 0) return a->dtype;
  bool fa = is_float(a->dtype), fb = is_float(b->dtype);
  if (fa && fb) return LT_F32;
  if (fa) return a->dtype;
  if (fb) return b->dtype;
  return LT_I64;
}

static const lt_attr* find_attr(const lt_attr* attrs, int n, uint16_t key) {
  for (int i = 0; i < n; ++i)
    if (attrs[i].key == key) return &attrs[i];
  return nullptr;
}

static int dim_list(const lt_attr* attrs, int n, int64_t* out) {
  int count = 0;
  for (int i = 0; i < LT_MAX_RANK; ++i) {
    const lt_attr* a = find_attr(attrs, n, (uint16_t)(LT_ATTR_DIM0 + i));
    if (!a) break;
    out[count++] = a->v.i;
  }
  return count;
}

static void push_attr(Node* n, uint16_t key, bool isf, int64_t i, double f) {
  Attr& a = n->attrs[n->n_attr++];
  a.key = key;
  a.is_float = isf ? 1 : 0;
  if (isf) a.v.f = f;
  else a.v.i = i;
}

}  // namespace lt

using namespace lt;

extern "C" {

lt_status lt_init(int device, void* hip_stream, void* workspace, size_t workspace_bytes, lt_ctx** out) {
  if (!out) return fail(nullptr, LT_ERR_ARG, "lt_init: out is null");
  *out = nullptr;
  if (device < -1) return fail(nullptr, LT_ERR_ARG, "lt_init: bad device ordinal");
  std::unique_ptr<lt_ctx> ctx(new lt_ctx());
  ctx->device = device;
  ctx->stream = (hipStream_t)hip_stream;
  if (device >= 0) {
    if (!workspace || workspace_bytes < (8u << 20))
      return fail(nullptr, LT_ERR_ARG, "lt_init: a device context needs a workspace of at least 8 MiB");
    hipError_t e = hipSetDevice(device);
    if (e != hipSuccess) return fail(nullptr, LT_ERR_DEVICE, std::string("hipSetDevice: ") + hipGetErrorString(e));
    ctx->device_name = "HIP:" + std::to_string(device);
  } else {
    ctx->device_name = "CPU:0";
    if (!workspace && workspace_bytes == 0) workspace_bytes = (size_t)1 << 40;   // (addresses are only planned)
  }
  ctx->arena.init(workspace, workspace_bytes);
  ctx->red_partials = (float*)ctx->arena.alloc(kPartialFloats * sizeof(float));
  ctx->red_tickets = (uint32_t*)ctx->arena.alloc(kTickets * sizeof(uint32_t));
  if (!ctx->red_partials || !ctx->red_tickets) return fail(nullptr, LT_ERR_OOM, "lt_init: workspace too small");
  if (device >= 0) {
    hipError_t e = hipMemsetAsync(ctx->red_tickets, 0, kTickets * sizeof(uint32_t), ctx->stream);
    if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
    // side streams for independent launches: default priority, no implicit ordering against the
    // null stream (every edge to the caller's stream is an explicit event)
    for (int i = 0; i < kMaxStreams - 1 && e == hipSuccess; ++i) {
      e = hipStreamCreateWithFlags(&ctx->side[i], hipStreamNonBlocking);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->join_event[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->fork_event, hipEventDisableTiming);
    // the library's static scratch on this device: its address is looked up here, once per device,
    // so that lt_barrier_static itself neither allocates nor asks the runtime for anything
    if (e != hipSuccess) return fail(nullptr, LT_ERR_DEVICE, std::string("lt_init: ") + hipGetErrorString(e));
    void* p = nullptr;
    const hipError_t es = ltk::static_scratch(device, &p, &ctx->static_scratch_bytes);
    if (es == hipSuccess) ctx->static_scratch = (uint8_t*)p;
    else ctx->static_scratch_error = std::string("hipGetSymbolAddress of the static scratch: ") + hipGetErrorString(es);   // (lt_barrier_static reports it)
  } else {
    ctx->static_scratch = (uint8_t*)(uintptr_t)0x40000000;   // a null device only plans addresses
    ctx->static_scratch_bytes = ltk::kStaticScratchBytes;
  }
  *out = ctx.release();
  return LT_OK;
}

lt_status lt_shutdown(lt_ctx* ctx) {
  if (!ctx) return LT_ERR_ARG;
  if (ctx->device >= 0) {
    (void)hipStreamSynchronize(ctx->stream);
    for (hipEvent_t e : ctx->events) (void)hipEventDestroy(e);
    for (auto& bucket : ctx->cache)
      for (auto& plan : bucket.second) destroy_device_objects(plan.get());
    if (ctx->graph_stream) (void)hipStreamDestroy(ctx->graph_stream);
    for (int i = 0; i < kMaxStreams - 1; ++i) {
      if (ctx->side[i]) (void)hipStreamSynchronize(ctx->side[i]);
      if (ctx->side[i]) (void)hipStreamDestroy(ctx->side[i]);
      if (ctx->join_event[i]) (void)hipEventDestroy(ctx->join_event[i]);
    }
    if (ctx->fork_event) (void)hipEventDestroy(ctx->fork_event);
  }
  ctx->handles.clear();
  ctx->nodes.clear();
  delete ctx;
  return LT_OK;
}

const char* lt_last_error(lt_ctx* ctx) { return ctx ? ctx->err.c_str() : g_init_error.c_str(); }

lt_status lt_tensor_from_device(lt_ctx* ctx, void* dptr, lt_dtype dtype, int rank, const int64_t* dims,
                                uint32_t flags, lt_tensor* out) {
  if (!ctx || !out) return LT_ERR_ARG;
  if (rank < 0 || rank > LT_MAX_RANK || (rank > 0 && !dims)) return fail(ctx, LT_ERR_ARG, "tensor_from_device: bad rank");
  if ((int)dtype < 0 || (int)dtype > LT_I64) return fail(ctx, LT_ERR_DTYPE, "tensor_from_device: bad dtype");
  for (int i = 0; i < rank; ++i)
    if (dims[i] < 0) return fail(ctx, LT_ERR_SHAPE, "tensor_from_device: negative dimension");
  if (!dptr && ctx->device >= 0 && numel(dims, rank) > 0) return fail(ctx, LT_ERR_ARG, "tensor_from_device: null device pointer");
  if (ctx->device >= 0 && ((uintptr_t)dptr & 15u)) return fail(ctx, LT_ERR_ARG, "tensor_from_device: pointer must be 16-byte aligned");
  Handle* h = new_handle(ctx);
  h->kind = H_DATA;
  h->dtype = (uint8_t)dtype;
  h->rank = (uint8_t)rank;
  for (int i = 0; i < rank; ++i) h->dims[i] = dims[i];
  h->buf = std::make_shared<Buffer>();
  h->buf->ptr = dptr;
  h->buf->bytes = (size_t)numel(dims, rank) * dtype_size((uint8_t)dtype);
  h->buf->donatable = (flags & LT_DONATABLE) != 0;
  h->buf->data_refs = 1;
  *out = h->id;
  return LT_OK;
}

lt_status lt_tensor_rebind(lt_ctx* ctx, lt_tensor t, void* dptr) {
  if (!ctx) return LT_ERR_ARG;
  Handle* h = find(ctx, t, false);
  if (!h) return fail(ctx, LT_ERR_HANDLE, "lt_tensor_rebind: unknown or released tensor id");
  if (h->kind != H_DATA || !h->buf || h->view_base) return fail(ctx, LT_ERR_ARG, "lt_tensor_rebind: only a plain data tensor names device memory");
  if (h->buf->owned) return fail(ctx, LT_ERR_ARG, "lt_tensor_rebind: the tensor's memory belongs to the library (a result), not to the caller");
  if (h->memo_epoch == ctx->epoch && h->memo_node >= 0) return fail(ctx, LT_ERR_ARG, "lt_tensor_rebind: the pending trace reads this tensor: run a barrier first");
  if (!dptr && ctx->device >= 0 && h->buf->bytes > 0) return fail(ctx, LT_ERR_ARG, "lt_tensor_rebind: null device pointer");
  if (ctx->device >= 0 && ((uintptr_t)dptr & 15u)) return fail(ctx, LT_ERR_ARG, "lt_tensor_rebind: pointer must be 16-byte aligned");
  // a buffer of its own: other tensors that share the old one (lt_assign) keep the old memory
  auto nb = std::make_shared<Buffer>();
  nb->ptr = dptr;
  nb->bytes = h->buf->bytes;
  nb->donatable = h->buf->donatable;
  nb->data_refs = 1;
  h->buf->data_refs -= 1;
  h->buf = nb;
  h->donor.reset();
  h->version++;
  return LT_OK;
}

lt_status lt_scalar(lt_ctx* ctx, lt_dtype dtype, double value, lt_tensor* out) {
  if (!ctx || !out) return LT_ERR_ARG;
  if ((int)dtype < 0 || (int)dtype > LT_I64) return fail(ctx, LT_ERR_DTYPE, "lt_scalar: bad dtype");
  Handle* h = new_handle(ctx);
  h->kind = H_SCALAR;
  h->dtype = (uint8_t)dtype;
  h->rank = 0;
  h->value = value;
  *out = h->id;
  return LT_OK;
}

lt_status lt_op(lt_ctx* ctx, uint16_t opcode, const lt_tensor* inputs, int n_in, const lt_attr* attrs, int n_attr,
                lt_tensor* outputs, int n_out) {
  return record_op(ctx, opcode, inputs, n_in, attrs, n_attr, outputs, n_out, false);
}

}  // extern "C"

namespace lt {

static lt_status record_op(lt_ctx* ctx, uint16_t opcode, const lt_tensor* inputs, int n_in, const lt_attr* attrs, int n_attr,
                           lt_tensor* outputs, int n_out, bool hidden) {
  if (!ctx || !inputs || !outputs || n_in < 1 || n_in > kMaxIns || n_attr < 0 || (n_attr > 0 && !attrs))
    return fail(ctx, LT_ERR_ARG, "lt_op: bad arguments");
  Handle* in[kMaxIns];
  for (int i = 0; i < n_in; ++i) {
    in[i] = find(ctx, inputs[i], hidden);
    if (!in[i]) return fail(ctx, LT_ERR_HANDLE, "lt_op: unknown or released tensor id");
    if (in[i]->view_base) {   // a view is read at its base's current value
      const lt_status st = refresh(ctx, in[i]);
      if (st != LT_OK) return st;
    }
  }
  Node n;
  n.op = opcode;
  n.n_in = (uint8_t)n_in;
  n.n_out = 1;
  auto set_shape = [&](const int64_t* dims, int rank) {
    n.rank = (uint8_t)rank;
    for (int i = 0; i < rank; ++i) n.dims[i] = dims[i];
  };
  auto need = [&](int k) { return n_in == k; };
  const Handle* a = in[0];
  switch (opcode) {
    case LT_OP_NEG: case LT_OP_ABS: case LT_OP_EXP: case LT_OP_LOG: case LT_OP_TANH: case LT_OP_SQRT:
    case LT_OP_RSQRT: case LT_OP_RECIP: case LT_OP_RELU: case LT_OP_GELU: case LT_OP_SQUARE: case LT_OP_SIGMOID:
      if (!need(1)) return fail(ctx, LT_ERR_ARG, "unary op takes one input");
      n.dtype = a->dtype;
      set_shape(a->dims, a->rank);
      break;
    case LT_OP_CAST: {
      const lt_attr* d = find_attr(attrs, n_attr, LT_ATTR_DTYPE);
      if (!need(1) || !d || d->v.i < 0 || d->v.i > LT_I64) return fail(ctx, LT_ERR_ARG, "cast needs LT_ATTR_DTYPE");
      n.dtype = (uint8_t)d->v.i;
      set_shape(a->dims, a->rank);
      push_attr(&n, LT_ATTR_DTYPE, false, d->v.i, 0);
    } break;
    case LT_OP_ADD: case LT_OP_SUB: case LT_OP_MUL: case LT_OP_DIV: case LT_OP_MAXIMUM: case LT_OP_MINIMUM:
    case LT_OP_RELU_GRAD: case LT_OP_GELU_GRAD: {
      const bool alpha = opcode == LT_OP_ADD && n_in == 3;
      if (!need(2) && !alpha) return fail(ctx, LT_ERR_ARG, "binary op takes two inputs (add: optional alpha)");
      if (alpha && in[2]->rank != 0) return fail(ctx, LT_ERR_SHAPE, "add: alpha must be rank 0");
      int64_t dims[LT_MAX_RANK];
      int rank;
      if (!broadcast(a->dims, a->rank, in[1]->dims, in[1]->rank, dims, &rank))
        return fail(ctx, LT_ERR_SHAPE, "operand shapes do not broadcast");
      n.dtype = promote(a, in[1]);
      set_shape(dims, rank);
    } break;
    case LT_OP_EXPAND: case LT_OP_RESHAPE: {
      int64_t dims[LT_MAX_RANK];
      int rank = dim_list(attrs, n_attr, dims);
      if (!need(1)) return fail(ctx, LT_ERR_ARG, "expand / reshape take one input");
      if (opcode == LT_OP_EXPAND) {
        int64_t chk[LT_MAX_RANK];
        int cr;
        if (!broadcast(a->dims, a->rank, dims, rank, chk, &cr) || cr != rank || std::memcmp(chk, dims, rank * sizeof(int64_t)))
          return fail(ctx, LT_ERR_SHAPE, "expand: input does not broadcast to the requested size");
      } else if (numel(dims, rank) != numel(a->dims, a->rank)) {
        return fail(ctx, LT_ERR_SHAPE, "reshape: element count differs");
      }
      n.dtype = a->dtype;
      set_shape(dims, rank);
      for (int i = 0; i < rank; ++i) push_attr(&n, (uint16_t)(LT_ATTR_DIM0 + i), false, dims[i], 0);
    } break;
    case LT_OP_PERMUTE: {
      int64_t perm[LT_MAX_RANK];
      int rank = dim_list(attrs, n_attr, perm);
      if (!need(1) || rank != a->rank) return fail(ctx, LT_ERR_ARG, "permute: dims must list every axis");
      bool seen[LT_MAX_RANK] = {false};
      int64_t dims[LT_MAX_RANK];
      for (int i = 0; i < rank; ++i) {
        if (perm[i] < 0 || perm[i] >= rank || seen[perm[i]]) return fail(ctx, LT_ERR_ARG, "permute: not a permutation");
        seen[perm[i]] = true;
        dims[i] = a->dims[perm[i]];
      }
      n.dtype = a->dtype;
      set_shape(dims, rank);
      for (int i = 0; i < rank; ++i) push_attr(&n, (uint16_t)(LT_ATTR_DIM0 + i), false, perm[i], 0);
    } break;
    case LT_OP_SUM: case LT_OP_AMAX: case LT_OP_MEAN: {
      if (!need(1)) return fail(ctx, LT_ERR_ARG, "reduction takes one input");
      const lt_attr* ax = find_attr(attrs, n_attr, LT_ATTR_AXIS);
      n.dtype = a->dtype;
      if (!ax) {
        n.rank = 0;
      } else {
        int64_t axis = ax->v.i < 0 ? ax->v.i + a->rank : ax->v.i;
        if (axis < 0 || axis >= a->rank) return fail(ctx, LT_ERR_ARG, "reduction: axis out of range");
        int r = 0;
        for (int i = 0; i < a->rank; ++i)
          if (i != axis) n.dims[r++] = a->dims[i];
        n.rank = (uint8_t)r;
        push_attr(&n, LT_ATTR_AXIS, false, axis, 0);
        // the reduction kernels cover the last axis and axis 0 of a matrix: everything else is an
        // op without a lowering, which a registered fallback computes eagerly (section 4.5)
        const bool lowered = a->rank <= 1 || axis == a->rank - 1 || (axis == 0 && a->rank == 2);
        if (!lowered && ctx->fallback && n_out == 1) {
          const lt_attr ax_attr{LT_ATTR_AXIS, 0, {axis}};
          return run_fallback(ctx, opcode, inputs, n_in, &ax_attr, 1, outputs, n_out, &n);
        }
      }
    } break;
    case LT_OP_SOFTMAX:
      if (!need(1) || a->rank < 1) return fail(ctx, LT_ERR_ARG, "softmax takes one input of rank >= 1");
      n.dtype = a->dtype;
      set_shape(a->dims, a->rank);
      break;
    case LT_OP_SOFTMAX_GRAD: {
      if (!need(2)) return fail(ctx, LT_ERR_ARG, "softmax_grad takes (dy, y)");
      const Handle* y = in[1];
      if (y->rank < 1 || y->rank != a->rank || std::memcmp(y->dims, a->dims, y->rank * sizeof(int64_t)))
        return fail(ctx, LT_ERR_SHAPE, "softmax_grad: dy and y differ in shape");
      n.dtype = y->dtype;
      set_shape(y->dims, y->rank);
    } break;
    case LT_OP_LAYER_NORM: {
      if (!need(3) || a->rank < 1) return fail(ctx, LT_ERR_ARG, "layer_norm takes (x, gamma, beta)");
      const int64_t c = a->dims[a->rank - 1];
      for (int k = 1; k < 3; ++k)
        if (in[k]->rank != 1 || in[k]->dims[0] != c) return fail(ctx, LT_ERR_SHAPE, "layer_norm: gamma / beta must be [cols]");
      const lt_attr* e = find_attr(attrs, n_attr, LT_ATTR_EPS);
      n.dtype = a->dtype;
      set_shape(a->dims, a->rank);
      n.n_out = 3;
      push_attr(&n, LT_ATTR_EPS, true, 0, e ? e->v.f : 1e-5);
    } break;
    case LT_OP_LAYER_NORM_GRAD: {
      if (!need(5)) return fail(ctx, LT_ERR_ARG, "layer_norm_grad takes (dy, x, gamma, mean, rstd)");
      const Handle* x = in[1];
      if (x->rank < 1 || a->rank != x->rank || std::memcmp(a->dims, x->dims, x->rank * sizeof(int64_t)))
        return fail(ctx, LT_ERR_SHAPE, "layer_norm_grad: dy and x differ in shape");
      if (in[2]->rank != 1 || in[2]->dims[0] != x->dims[x->rank - 1]) return fail(ctx, LT_ERR_SHAPE, "layer_norm_grad: gamma must be [cols]");
      for (int k = 3; k < 5; ++k)
        if (in[k]->rank != x->rank - 1 || std::memcmp(in[k]->dims, x->dims, (x->rank - 1) * sizeof(int64_t)))
          return fail(ctx, LT_ERR_SHAPE, "layer_norm_grad: mean / rstd must be x.shape[:-1]");
      n.dtype = x->dtype;
      set_shape(x->dims, x->rank);
    } break;
    case LT_OP_XENT: case LT_OP_XENT_GRAD: {
      const bool grad = opcode == LT_OP_XENT_GRAD;
      if (!need(grad ? 3 : 2) || a->rank < 1) return fail(ctx, LT_ERR_ARG, "xent takes (logits, labels[, scale])");
      const Handle* lab = in[1];
      if (lab->dtype != LT_I32) return fail(ctx, LT_ERR_DTYPE, "xent: labels must be int32");
      if (lab->rank != a->rank - 1 || std::memcmp(lab->dims, a->dims, lab->rank * sizeof(int64_t)))
        return fail(ctx, LT_ERR_SHAPE, "xent: labels must be logits.shape[:-1]");
      if (grad && in[2]->rank != 0) return fail(ctx, LT_ERR_SHAPE, "xent_grad: scale must be rank 0");
      if (grad) {
        n.dtype = a->dtype;
        set_shape(a->dims, a->rank);
      } else {
        n.dtype = LT_F32;
        set_shape(a->dims, a->rank - 1);
      }
    } break;
    case LT_OP_MATMUL: {
      if (!need(2)) return fail(ctx, LT_ERR_ARG, "matmul takes two inputs");
      const Handle* b = in[1];
      const lt_attr* ta = find_attr(attrs, n_attr, LT_ATTR_TRANS_A);
      const lt_attr* tb = find_attr(attrs, n_attr, LT_ATTR_TRANS_B);
      const lt_attr* od = find_attr(attrs, n_attr, LT_ATTR_DTYPE);
      const bool tra = ta && ta->v.i, trb = tb && tb->v.i;
      if (a->rank < 2 || b->rank < 2) return fail(ctx, LT_ERR_SHAPE, "matmul: operands must have rank >= 2");
      const int64_t m = tra ? a->dims[a->rank - 1] : a->dims[a->rank - 2];
      const int64_t k = tra ? a->dims[a->rank - 2] : a->dims[a->rank - 1];
      const int64_t k2 = trb ? b->dims[b->rank - 1] : b->dims[b->rank - 2];
      const int64_t nn = trb ? b->dims[b->rank - 2] : b->dims[b->rank - 1];
      if (k != k2) return fail(ctx, LT_ERR_SHAPE, "matmul: inner dimensions differ");
      if (b->rank > 2 && (b->rank != a->rank || std::memcmp(a->dims, b->dims, (a->rank - 2) * sizeof(int64_t))))
        return fail(ctx, LT_ERR_SHAPE, "matmul: leading axes of a and b differ");
      if (!is_float(a->dtype) || !is_float(b->dtype)) return fail(ctx, LT_ERR_DTYPE, "matmul: float operands only");
      if (od && (od->v.i < 0 || od->v.i > LT_BF16)) return fail(ctx, LT_ERR_DTYPE, "matmul: output dtype must be f32 or bf16");
      n.dtype = od ? (uint8_t)od->v.i : (a->dtype == b->dtype ? a->dtype : (uint8_t)LT_F32);
      for (int i = 0; i < a->rank - 2; ++i) n.dims[i] = a->dims[i];
      n.dims[a->rank - 2] = m;
      n.dims[a->rank - 1] = nn;
      n.rank = a->rank;
      push_attr(&n, LT_ATTR_DTYPE, false, n.dtype, 0);
      push_attr(&n, LT_ATTR_TRANS_A, false, tra ? 1 : 0, 0);
      push_attr(&n, LT_ATTR_TRANS_B, false, trb ? 1 : 0, 0);
    } break;
    case LT_OP_NARROW: {
      const lt_attr* ax = find_attr(attrs, n_attr, LT_ATTR_AXIS);
      const lt_attr* st = find_attr(attrs, n_attr, LT_ATTR_START);
      const lt_attr* ln = find_attr(attrs, n_attr, LT_ATTR_LENGTH);
      if (!need(1) || !ax || !st || !ln) return fail(ctx, LT_ERR_ARG, "narrow takes one input and LT_ATTR_AXIS, _START, _LENGTH");
      const int64_t axis = ax->v.i < 0 ? ax->v.i + a->rank : ax->v.i;
      if (axis < 0 || axis >= a->rank) return fail(ctx, LT_ERR_ARG, "narrow: axis out of range");
      if (st->v.i < 0 || ln->v.i < 0 || st->v.i + ln->v.i > a->dims[axis]) return fail(ctx, LT_ERR_SHAPE, "narrow: window exceeds the axis");
      n.dtype = a->dtype;
      set_shape(a->dims, a->rank);
      n.dims[axis] = ln->v.i;
      push_attr(&n, LT_ATTR_AXIS, false, axis, 0);
      push_attr(&n, LT_ATTR_START, false, st->v.i, 0);
      push_attr(&n, LT_ATTR_LENGTH, false, ln->v.i, 0);
    } break;
    case LT_OP_SLICE_UPDATE: {
      const lt_attr* ax = find_attr(attrs, n_attr, LT_ATTR_AXIS);
      const lt_attr* st = find_attr(attrs, n_attr, LT_ATTR_START);
      if (!need(2) || !ax || !st) return fail(ctx, LT_ERR_ARG, "slice_update takes (base, update) and LT_ATTR_AXIS, _START");
      const Handle* u = in[1];
      const int64_t axis = ax->v.i < 0 ? ax->v.i + a->rank : ax->v.i;
      if (axis < 0 || axis >= a->rank) return fail(ctx, LT_ERR_ARG, "slice_update: axis out of range");
      if (u->rank != a->rank || u->dtype != a->dtype) return fail(ctx, LT_ERR_SHAPE, "slice_update: update must have the base's rank and dtype");
      for (int i = 0; i < a->rank; ++i)
        if (i != axis && u->dims[i] != a->dims[i]) return fail(ctx, LT_ERR_SHAPE, "slice_update: update differs from the base off the axis");
      if (st->v.i < 0 || st->v.i + u->dims[axis] > a->dims[axis]) return fail(ctx, LT_ERR_SHAPE, "slice_update: window exceeds the axis");
      n.dtype = a->dtype;
      set_shape(a->dims, a->rank);
      push_attr(&n, LT_ATTR_AXIS, false, axis, 0);
      push_attr(&n, LT_ATTR_START, false, st->v.i, 0);
    } break;
    default:
      if (ctx->fallback && opcode >= LT_OP_CUSTOM) return run_fallback(ctx, opcode, inputs, n_in, attrs, n_attr, outputs, n_out, nullptr);
      return fail(ctx, LT_ERR_UNSUPPORTED, "lt_op: opcode " + std::to_string(opcode) + " has no lowering");
  }
  if (n_out != n.n_out) return fail(ctx, LT_ERR_ARG, "lt_op: wrong number of outputs for this opcode");
  std::sort(n.attrs, n.attrs + n.n_attr, [](const Attr& x, const Attr& y) { return x.key < y.key; });
  // operands are resolved last so that a failed call leaves the trace untouched
  for (int i = 0; i < n_in; ++i) n.ins[i] = use(ctx, in[i]);
  push_node(ctx, std::move(n));
  ctx->stats.nodes_recorded++;
  const int32_t idx = (int32_t)ctx->nodes.size() - 1;
  const Node& nn = ctx->nodes[idx];
  for (int s = 0; s < nn.n_out; ++s) {
    Handle* h = new_handle(ctx);
    h->kind = H_PENDING;
    h->node = idx;
    h->slot = s;
    if (nn.op == LT_OP_LAYER_NORM && s > 0) {
      h->dtype = LT_F32;
      h->rank = nn.rank - 1;
    } else {
      h->dtype = nn.dtype;
      h->rank = nn.rank;
    }
    for (int i = 0; i < h->rank; ++i) h->dims[i] = nn.dims[i];
    outputs[s] = h->id;
  }
  return LT_OK;
}

// Section 4.5: evaluate the inputs, call the eager implementation, start a new graph from its result.
static lt_status run_fallback(lt_ctx* ctx, uint16_t opcode, const lt_tensor* inputs, int n_in, const lt_attr* attrs, int n_attr,
                              lt_tensor* outputs, int n_out, const Node* inferred) {
  if (n_out < 1 || n_out > 4) return fail(ctx, LT_ERR_ARG, "lt_op: an op without a lowering has 1 to 4 results");
  // 1. every input becomes plain data (the barrier evaluates all live tensors, the inputs among them)
  bool pending = false;
  for (int i = 0; i < n_in; ++i) {
    const Handle* h = find(ctx, inputs[i]);
    pending |= h->kind == H_PENDING;
  }
  if (pending) {
    const lt_status st = lt_barrier(ctx, 1, nullptr);
    if (st != LT_OK) return st;
  }
  lt_tensor_desc in[kMaxIns];
  for (int i = 0; i < n_in; ++i) {
    const Handle* h = find(ctx, inputs[i]);
    in[i] = lt_tensor_desc{};
    in[i].dtype = h->dtype;
    in[i].rank = h->rank;
    for (int d = 0; d < h->rank; ++d) in[i].dims[d] = h->dims[d];
    if (h->kind == H_SCALAR) {
      in[i].is_scalar = 1;
      in[i].scalar = h->value;
    } else {
      in[i].dptr = h->buf->ptr;
    }
  }
  // 2. result types: the library's own inference, or the callback's
  lt_tensor_desc out[4];
  for (int s = 0; s < n_out; ++s) out[s] = lt_tensor_desc{};
  if (inferred) {
    out[0].dtype = inferred->dtype;
    out[0].rank = inferred->rank;
    for (int d = 0; d < inferred->rank; ++d) out[0].dims[d] = inferred->dims[d];
  } else {
    if (ctx->fallback(ctx->fallback_user, opcode, in, n_in, attrs, n_attr, out, n_out, 0, ctx->stream) != 0)
      return fail(ctx, LT_ERR_UNSUPPORTED, "lt_op: opcode " + std::to_string(opcode) + " has no lowering and the fallback declined it");
    for (int s = 0; s < n_out; ++s) {
      bool ok = out[s].dtype >= 0 && out[s].dtype <= LT_I64 && out[s].rank >= 0 && out[s].rank <= LT_MAX_RANK;
      for (int d = 0; ok && d < out[s].rank; ++d) ok = out[s].dims[d] >= 0;
      if (!ok) return fail(ctx, LT_ERR_ARG, "fallback: bad result descriptor");
    }
  }
  BufRef bufs[4];
  for (int s = 0; s < n_out; ++s) {
    const size_t bytes = (size_t)numel(out[s].dims, out[s].rank) * dtype_size((uint8_t)out[s].dtype);
    bufs[s] = std::make_shared<Buffer>();
    bufs[s]->ptr = ctx->arena.alloc(bytes);
    if (!bufs[s]->ptr) return fail(ctx, LT_ERR_OOM, "workspace arena exhausted by the result of a fallback op");
    bufs[s]->bytes = bytes;
    bufs[s]->owned = true;
    bufs[s]->donatable = true;
    bufs[s]->arena = &ctx->arena;
    out[s].dptr = bufs[s]->ptr;
  }
  // the eager implementation
  if (ctx->fallback(ctx->fallback_user, opcode, in, n_in, attrs, n_attr, out, n_out, 1, ctx->stream) != 0)
    return fail(ctx, LT_ERR_UNSUPPORTED, "lt_op: the fallback failed on opcode " + std::to_string(opcode));
  // 3. a new IR graph starts from the results
  for (int s = 0; s < n_out; ++s) {
    Handle* h = new_handle(ctx);
    h->kind = H_DATA;
    h->dtype = (uint8_t)out[s].dtype;
    h->rank = (uint8_t)out[s].rank;
    for (int d = 0; d < h->rank; ++d) h->dims[d] = out[s].dims[d];
    h->buf = bufs[s];
    h->buf->data_refs = 1;
    outputs[s] = h->id;
  }
  ctx->stats.fallback_ops++;
  return LT_OK;
}

// In-place update as substitution (section 4.3).  Through a view (section 4.4): the view takes the
// new value, and the base is rebuilt from it by the inverse of the view op (the "backward
// sequence"), through every level of a chain of views.
static lt_status assign(lt_ctx* ctx, lt_tensor dst_id, lt_tensor src_id, bool hidden) {
  Handle* dst = find(ctx, dst_id, hidden);
  Handle* src = find(ctx, src_id, hidden);
  if (!dst || !src) return fail(ctx, LT_ERR_HANDLE, "lt_assign: unknown or released tensor id");
  if (dst == src) return LT_OK;
  if (src->view_base) {
    const lt_status st = refresh(ctx, src);
    if (st != LT_OK) return st;
  }
  if (dst->view_base) {
    bool same = dst->dtype == src->dtype && dst->rank == src->rank;
    for (int i = 0; same && i < dst->rank; ++i) same = dst->dims[i] == src->dims[i];
    if (!same) return fail(ctx, LT_ERR_SHAPE, "lt_assign: a view can only take a value of its own dtype and shape");
  }
  BufRef donor = dst->donor;
  if (dst->kind == H_DATA && dst->buf && dst->buf->donatable) donor = dst->buf;
  // dst becomes a second name of src's buffer (or scalar): host bookkeeping that leaves no node in
  // the trace, so a captured step could not repeat it
  if (src->kind != H_PENDING) ctx->bound_plain = true;
  unbind(dst);
  dst->kind = src->kind;
  dst->dtype = src->dtype;
  dst->rank = src->rank;
  std::memcpy(dst->dims, src->dims, sizeof(dst->dims));
  dst->node = src->node;
  dst->slot = src->slot;
  dst->buf = src->buf;
  dst->value = src->value;
  dst->memo_epoch = src->memo_epoch;
  dst->memo_node = src->memo_node;
  if (dst->kind == H_DATA && dst->buf) dst->buf->data_refs += 1;
  dst->donor = donor;
  dst->version++;
  if (!dst->view_base) return LT_OK;
  Handle* b = find(ctx, dst->view_base, true);
  if (!b) return fail(ctx, LT_ERR_HANDLE, "internal: a view has lost its base");
  lt_status st = refresh(ctx, b);   // (a base that is itself a stale view)
  if (st != LT_OK) return st;
  dst->seen = b->version;           // the view now holds its new value, not one to derive again
  lt_attr inv[kMaxAttrs];
  int n_inv = 0;
  lt_tensor tid = 0;
  const lt_tensor bid = b->id;
  if (dst->view_op == LT_OP_PERMUTE) {
    for (int i = 0; i < dst->view_n_attr; ++i) {   // inverse permutation: view axis j shows base axis p[j], so base axis p[j] is view axis j
      const int64_t j = dst->view_attrs[i].key - LT_ATTR_DIM0, src_axis = dst->view_attrs[i].v.i;
      inv[src_axis].key = (uint16_t)(LT_ATTR_DIM0 + src_axis);
      inv[src_axis].is_float = 0;
      inv[src_axis].v.i = j;
    }
    n_inv = dst->view_n_attr;
    st = record_op(ctx, LT_OP_PERMUTE, &dst_id, 1, inv, n_inv, &tid, 1, true);
  } else if (dst->view_op == LT_OP_RESHAPE) {
    for (int i = 0; i < b->rank; ++i) inv[n_inv++] = lt_attr{(uint16_t)(LT_ATTR_DIM0 + i), 0, {b->dims[i]}};
    st = record_op(ctx, LT_OP_RESHAPE, &dst_id, 1, inv, n_inv, &tid, 1, true);
  } else {
    for (int i = 0; i < dst->view_n_attr; ++i)
      if (dst->view_attrs[i].key == LT_ATTR_AXIS || dst->view_attrs[i].key == LT_ATTR_START) inv[n_inv++] = dst->view_attrs[i];
    const lt_tensor ins[2] = {bid, dst_id};
    st = record_op(ctx, LT_OP_SLICE_UPDATE, ins, 2, inv, n_inv, &tid, 1, true);
  }
  if (st != LT_OK) return st;
  st = assign(ctx, bid, tid, true);
  Handle* t = find(ctx, tid, true);
  if (t) erase_handle(ctx, t);
  dst = find(ctx, dst_id, true);
  b = find(ctx, bid, true);
  if (dst && b) dst->seen = b->version;
  return st;
}

}  // namespace lt

extern "C" {

lt_status lt_assign(lt_ctx* ctx, lt_tensor dst_id, lt_tensor src_id) {
  if (!ctx) return LT_ERR_ARG;
  return assign(ctx, dst_id, src_id, false);
}

lt_status lt_view(lt_ctx* ctx, lt_tensor base, uint16_t view_op, const lt_attr* attrs, int n_attr, lt_tensor* out) {
  if (!ctx || !out) return LT_ERR_ARG;
  if (view_op != LT_OP_PERMUTE && view_op != LT_OP_RESHAPE && view_op != LT_OP_NARROW)
    return fail(ctx, LT_ERR_ARG, "lt_view: the view ops are permute, reshape and narrow");
  if (n_attr < 0 || n_attr > kMaxAttrs) return fail(ctx, LT_ERR_ARG, "lt_view: bad attributes");
  lt_status st = record_op(ctx, view_op, &base, 1, attrs, n_attr, out, 1, false);
  if (st != LT_OK) return st;
  Handle* h = find(ctx, *out);
  Handle* b = find(ctx, base);
  h->view_base = base;
  h->view_op = view_op;
  h->view_n_attr = (uint8_t)n_attr;
  for (int i = 0; i < n_attr; ++i) h->view_attrs[i] = attrs[i];
  h->seen = b->version;
  b->view_refs++;
  return LT_OK;
}

lt_status lt_release(lt_ctx* ctx, lt_tensor t) {
  if (!ctx) return LT_ERR_ARG;
  Handle* h = find(ctx, t);
  if (!h) return fail(ctx, LT_ERR_HANDLE, "lt_release: unknown or released tensor id");
  return release_one(ctx, h);
}

lt_status lt_release_many(lt_ctx* ctx, const lt_tensor* ts, size_t n) {
  if (!ctx || (n && !ts)) return LT_ERR_ARG;
  lt_status st = LT_OK;
  for (size_t i = 0; i < n; ++i) {
    Handle* h = find(ctx, ts[i]);
    if (!h) {
      st = fail(ctx, LT_ERR_HANDLE, "lt_release_many: unknown or released tensor id");
      continue;
    }
    (void)release_one(ctx, h);
  }
  return st;
}

lt_status lt_shape(lt_ctx* ctx, lt_tensor t, lt_dtype* dtype, int* rank, int64_t* dims) {
  if (!ctx) return LT_ERR_ARG;
  Handle* h = find(ctx, t);
  if (!h) return fail(ctx, LT_ERR_HANDLE, "lt_shape: unknown or released tensor id");
  if (dtype) *dtype = (lt_dtype)h->dtype;
  if (rank) *rank = h->rank;
  if (dims)
    for (int i = 0; i < h->rank; ++i) dims[i] = h->dims[i];
  return LT_OK;
}

lt_status lt_device_ptr(lt_ctx* ctx, lt_tensor t, void** dptr) {
  if (!ctx || !dptr) return LT_ERR_ARG;
  Handle* h = find(ctx, t);
  if (!h) return fail(ctx, LT_ERR_HANDLE, "lt_device_ptr: unknown or released tensor id");
  if (h->view_base && refresh(ctx, h) != LT_OK) return LT_ERR_HANDLE;
  if (h->kind != H_DATA) return fail(ctx, LT_ERR_HANDLE, "lt_device_ptr: tensor is not materialised (barrier first)");
  *dptr = h->buf->ptr;
  return LT_OK;
}

static lt_status copy_out(const std::string& s, char* buf, size_t cap, size_t* len) {
  if (len) *len = s.size();
  if (buf && cap) {
    size_t n = std::min(cap - 1, s.size());
    std::memcpy(buf, s.data(), n);
    buf[n] = 0;
  }
  return LT_OK;
}

lt_status lt_dump_ir(lt_ctx* ctx, char* buf, size_t cap, size_t* len) {
  if (!ctx) return LT_ERR_ARG;
  lt_status vs = refresh_views(ctx);   // what the next barrier would cut
  if (vs != LT_OK) return vs;
  Cut cut;
  collect_cut(ctx, &cut);
  std::string s = "IR {\n";
  char tmp[96];
  for (size_t i = 0; i < cut.order.size(); ++i) {
    const Node& n = ctx->nodes[cut.order[i]];
    s += "    %" + std::to_string(i) + " = " + dtype_name(n.dtype) + "[";
    for (int d = 0; d < n.rank; ++d) s += (d ? "," : "") + std::to_string(n.dims[d]);
    s += std::string("] ") + op_name(n.op) + "(";
    for (int k = 0; k < n.n_in; ++k) {
      s += (k ? ", %" : "%") + std::to_string(cut.index_of[n.ins[k].node]);
      if (n.ins[k].slot) s += "." + std::to_string(n.ins[k].slot);
    }
    s += ")";
    if (n.op == OP_DEVICE_DATA || n.op == OP_SCALAR_PARAM) {
      s += ", device=" + ctx->device_name;
    } else if (n.op == OP_CONSTANT) {
      const double v = n.attrs[0].is_float ? n.attrs[0].v.f : (double)n.attrs[0].v.i;
      s += ", value=" + std::to_string((long long)v);
    } else if (n.op == LT_OP_EXPAND || n.op == LT_OP_RESHAPE || n.op == LT_OP_PERMUTE) {
      s += n.op == LT_OP_PERMUTE ? ", dims=(" : ", size=(";
      for (int k = 0; k < n.n_attr; ++k) s += (k ? ", " : "") + std::to_string(n.attrs[k].v.i);
      s += ")";
    } else {
      for (int k = 0; k < n.n_attr; ++k) {
        const Attr& a = n.attrs[k];
        const char* name = a.key == LT_ATTR_DTYPE ? "dtype" : a.key == LT_ATTR_AXIS ? "axis" : a.key == LT_ATTR_EPS ? "eps"
                           : a.key == LT_ATTR_TRANS_A ? "trans_a" : a.key == LT_ATTR_TRANS_B ? "trans_b"
                           : a.key == LT_ATTR_START ? "start" : a.key == LT_ATTR_LENGTH ? "length" : "attr";
        if (a.key == LT_ATTR_DTYPE) std::snprintf(tmp, sizeof(tmp), ", %s=%s", name, dtype_name((uint8_t)a.v.i));
        else if (a.is_float) std::snprintf(tmp, sizeof(tmp), ", %s=%g", name, a.v.f);
        else std::snprintf(tmp, sizeof(tmp), ", %s=%lld", name, (long long)a.v.i);
        s += tmp;
      }
    }
    for (size_t r = 0; r < cut.roots.size(); ++r) {
      if (cut.roots[r]->node == cut.order[i]) {
        s += ", ROOT=" + std::to_string(r);
        if (cut.roots[r]->slot) s += "." + std::to_string(cut.roots[r]->slot);
      }
    }
    s += "\n";
  }
  s += "}";
  return copy_out(s, buf, cap, len);
}

lt_status lt_dump_plan(lt_ctx* ctx, char* buf, size_t cap, size_t* len) {
  if (!ctx) return LT_ERR_ARG;
  return copy_out(ctx->last_plan ? ctx->last_plan->text : std::string(), buf, cap, len);
}

lt_status lt_dump_schedule(lt_ctx* ctx, char* buf, size_t cap, size_t* len) {
  if (!ctx) return LT_ERR_ARG;
  std::string s;
  if (ctx->last_plan) {
    static const char* const kinds[] = {"EW", "ROW", "ALL", "COL", "ROWOP", "MM", "SPLITPOST", "SLICE"};
    const Plan& p = *ctx->last_plan;
    for (size_t i = 0; i < p.launches.size(); ++i) {
      const Launch& l = p.launches[i];
      s += "L" + std::to_string(i) + " " + kinds[l.kind] + " R" + std::to_string(l.region) + " stream=" + std::to_string(l.stream) +
           " slot=" + std::to_string(l.scratch_slot) + " record=" + std::to_string(l.record) + " waits=[";
      for (size_t w = 0; w < l.waits.size(); ++w) s += (w ? "," : "") + std::to_string(l.waits[w]);
      s += "]";
      // what the launch reads and writes, from the plan's pointer patches (p<n>: caller's buffer
      // number n, donated outputs included; t<n>: temporary storage n)
      for (int wr = 0; wr < 2; ++wr) {
        s += wr ? " writes=[" : " reads=[";
        bool first = true;
        for (const PtrPatch& pp : p.ptr_patches) {
          if (pp.launch != i || pp.storage < 0 || (int)pp.write != wr) continue;
          const Storage& st = p.storages[pp.storage];
          s += (first ? "" : ",") + (st.param >= 0 ? "p" + std::to_string(st.param) : "t" + std::to_string(pp.storage));
          first = false;
        }
        s += "]";
      }
      s += "\n";
    }
  }
  return copy_out(s, buf, cap, len);
}

lt_status lt_dump_key(lt_ctx* ctx, uint8_t* buf, size_t cap, size_t* len) {
  if (!ctx) return LT_ERR_ARG;
  static const std::vector<uint8_t> none;
  const std::vector<uint8_t>& key = ctx->last_plan ? ctx->last_plan->key : none;
  if (len) *len = key.size();
  if (buf && cap) std::memcpy(buf, key.data(), std::min(cap, key.size()));
  return LT_OK;
}

lt_status lt_stats(lt_ctx* ctx, lt_stats_t* out) {
  if (!ctx || !out) return LT_ERR_ARG;
  ctx->stats.arena_bytes_in_use = ctx->arena.in_use;
  ctx->stats.arena_bytes_peak = ctx->arena.peak;
  ctx->stats.live_tensors = ctx->handles.size();
  *out = ctx->stats;
  return LT_OK;
}

lt_status lt_set_streams(lt_ctx* ctx, int n) {
  if (!ctx) return LT_ERR_ARG;
  if (n < 1 || n > kMaxStreams) return fail(ctx, LT_ERR_ARG, "lt_set_streams: between 1 and 4 streams");
  ctx->max_streams = n;
  return LT_OK;
}

lt_status lt_set_fusion(lt_ctx* ctx, int on) {
  if (!ctx) return LT_ERR_ARG;
  if (ctx->fusion == (on != 0)) return LT_OK;
  ctx->fusion = on != 0;
  // plans are lowered under one setting: the cache starts over
  if (ctx->device >= 0) {
    (void)hipStreamSynchronize(ctx->stream);
    for (auto& bucket : ctx->cache)
      for (auto& plan : bucket.second) destroy_device_objects(plan.get());
  }
  ctx->cache.clear();
  ctx->quick.clear();
  ctx->cache_generation++;
  ctx->last_plan = nullptr;
  ctx->last_step = lt::StepRecord{};
  return LT_OK;
}

lt_status lt_set_quick_lookup(lt_ctx* ctx, int mode) {
  if (!ctx || mode < 0 || mode > 2) return LT_ERR_ARG;
  ctx->quick_lookup = mode;
  return LT_OK;
}

lt_status lt_set_graphs(lt_ctx* ctx, int on) {
  if (!ctx) return LT_ERR_ARG;
  ctx->graphs = on != 0;
  return LT_OK;
}

lt_status lt_set_fallback(lt_ctx* ctx, lt_fallback_fn fn, void* user) {
  if (!ctx) return LT_ERR_ARG;
  ctx->fallback = fn;
  ctx->fallback_user = user;
  return LT_OK;
}

lt_status lt_set_profiling(lt_ctx* ctx, int on) {
  if (!ctx) return LT_ERR_ARG;
  ctx->profiling = on != 0;
  return LT_OK;
}

lt_status lt_last_launches(lt_ctx* ctx, lt_launch_record* out, int cap, int* n) {
  if (!ctx || !n) return LT_ERR_ARG;
  *n = (int)ctx->last_launches.size();
  if (out)
    for (int i = 0; i < std::min(cap, *n); ++i) out[i] = ctx->last_launches[i];
  return LT_OK;
}

}  // extern "C"
