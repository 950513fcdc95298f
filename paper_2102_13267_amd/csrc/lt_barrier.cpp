// C ABI, part 2: the barrier (section 4 of the paper: mark_step / LazyTensorBarrier) and fetch.
// Cut the trace of all live tensors, number it canonically, serialise, hash, look up the plan
// cache, lower on a miss, patch the cached launch arguments with this step's pointers and
// scalars, launch, and rebind every evaluated handle to its data.
#include <hip/hip_runtime_api.h>

#include <chrono>
#include <cmath>
#include <cstdio>

#include "lt_core.h"
#include "lt_launch.h"

namespace ltk {
static thread_local char g_kernel_name[48] = "";
void note_kernel(const char* name) {
  // "(lt_ew_stream_kernel<4, true>)" -> "lt_ew_stream_kernel<4, true>"
  size_t n = 0;
  for (const char* c = name; *c && n + 1 < sizeof(g_kernel_name); ++c)
    if (*c != '(' && *c != ')') g_kernel_name[n++] = *c;
  g_kernel_name[n] = 0;
}
const char* last_kernel() { return g_kernel_name; }
}  // namespace ltk

namespace lt {

static uint64_t now_ns() {
  return (uint64_t)std::chrono::duration_cast<std::chrono::nanoseconds>(
             std::chrono::steady_clock::now().time_since_epoch())
      .count();
}

uint64_t fnv1a64(const uint8_t* p, size_t n) {
  uint64_t h = 0xcbf29ce484222325ull;
  for (size_t i = 0; i < n; ++i) {
    h ^= p[i];
    h *= 0x100000001b3ull;
  }
  return h;
}

// Roots: live handles with a pending computation, ascending tensor id.  Canonical order:
// post-order from each root in turn, operands visited from last to first, every node once --
// the numbering that reproduces figures 1, 2 and 3 of the paper.
void collect_cut(lt_ctx* ctx, Cut* cut) {
  cut->roots.clear();
  cut->order.clear();
  cut->index_of.assign(ctx->nodes.size(), -1);
  for (auto& kv : ctx->handles)
    if (kv.second.kind == H_PENDING) cut->roots.push_back(&kv.second);
  std::vector<std::pair<int32_t, bool>> stack;
  for (Handle* r : cut->roots) {
    if (cut->index_of[r->node] >= 0) continue;
    stack.push_back({r->node, false});
    while (!stack.empty()) {
      auto [n, expanded] = stack.back();
      stack.pop_back();
      if (cut->index_of[n] >= 0) continue;
      if (expanded) {
        cut->index_of[n] = (int32_t)cut->order.size();
        cut->order.push_back(n);
        continue;
      }
      stack.push_back({n, true});
      const Node& node = ctx->nodes[n];
      for (int k = 0; k < node.n_in; ++k)   // pushed first to last => popped last to first
        if (cut->index_of[node.ins[k].node] < 0) stack.push_back({node.ins[k].node, false});
    }
  }
}

template <class T>
static void put(std::vector<uint8_t>* out, T v) {
  const uint8_t* p = (const uint8_t*)&v;   // gfx950 hosts are little-endian x86-64
  out->insert(out->end(), p, p + sizeof(T));
}

// Canonical little-endian byte string.  Buffer addresses and the values of dynamic scalars are
// left out; shapes, dtypes, attributes, operand indices, parameter ordinals, the root list and
// the donation pattern are in.
void serialise_cut(lt_ctx* ctx, Cut* cut, std::vector<uint8_t>* out) {
  out->clear();
  cut->param_nodes.clear();
  cut->scalar_nodes.clear();
  std::unordered_map<const Buffer*, uint32_t> param_of_buffer;
  for (int32_t idx : cut->order) {
    const Node& n = ctx->nodes[idx];
    put<uint16_t>(out, n.op);
    put<uint8_t>(out, n.dtype);
    put<uint8_t>(out, n.rank);
    for (int d = 0; d < n.rank; ++d) put<int64_t>(out, n.dims[d]);
    put<uint8_t>(out, n.n_attr);
    for (int k = 0; k < n.n_attr; ++k) {
      put<uint16_t>(out, n.attrs[k].key);
      put<uint8_t>(out, n.attrs[k].is_float);
      if (n.attrs[k].is_float) put<double>(out, n.attrs[k].v.f);
      else put<int64_t>(out, n.attrs[k].v.i);
    }
    put<uint8_t>(out, n.n_in);
    for (int k = 0; k < n.n_in; ++k) {
      put<uint32_t>(out, (uint32_t)cut->index_of[n.ins[k].node]);
      put<uint8_t>(out, (uint8_t)n.ins[k].slot);
    }
    if (n.op == OP_DEVICE_DATA) {
      // ordinal, then the ordinal of the first leaf bound to the same buffer: whether two leaves
      // alias decides what may be updated in place, so it is part of the program's identity
      const uint32_t ordinal = (uint32_t)cut->param_nodes.size();
      put<uint32_t>(out, ordinal);
      put<uint32_t>(out, param_of_buffer.emplace(n.buffer.get(), ordinal).first->second);
      cut->param_nodes.push_back(idx);
    } else if (n.op == OP_SCALAR_PARAM) {
      put<uint32_t>(out, (uint32_t)cut->scalar_nodes.size());
      cut->scalar_nodes.push_back(idx);
    }
  }
  put<uint32_t>(out, (uint32_t)cut->roots.size());
  cut->donors.assign(cut->roots.size(), 0xFFFFFFFFu);
  std::vector<const Buffer*> claimed;
  for (size_t r = 0; r < cut->roots.size(); ++r) {
    const Handle* h = cut->roots[r];
    uint32_t d = 0xFFFFFFFFu;
    const Buffer* b = h->donor.get();
    if (b) {
      auto it = param_of_buffer.find(b);
      bool taken = false;
      for (const Buffer* c : claimed) taken |= (c == b);
      const size_t bytes = (size_t)numel(h->dims, h->rank) * dtype_size(h->dtype);
      // the donor must be a parameter of this graph, seen by no live handle, of the same
      // dtype and shape (hence byte size) as the value that replaces it
      const Node* leaf = it != param_of_buffer.end() ? &ctx->nodes[cut->param_nodes[it->second]] : nullptr;
      bool same = leaf && leaf->dtype == h->dtype && leaf->rank == h->rank && b->bytes == bytes;
      if (same)
        for (int i = 0; i < h->rank; ++i) same &= leaf->dims[i] == h->dims[i];
      if (same && !taken && b->data_refs == 0) {
        d = it->second;
        claimed.push_back(b);
      }
    }
    cut->donors[r] = d;
    put<uint32_t>(out, (uint32_t)cut->index_of[h->node]);
    put<uint8_t>(out, (uint8_t)h->slot);
    put<uint32_t>(out, d);
  }
}

static lt_status hip_fail(lt_ctx* ctx, const char* what, hipError_t e) {
  return fail(ctx, LT_ERR_DEVICE, std::string(what) + ": " + hipGetErrorString(e));
}

static hipError_t launch_one(const Launch& l, const uint8_t* args, hipStream_t s) {
  switch (l.kind) {
    case L_EW: return ltk::launch_ew(*(const ltk::EwArgs*)args, l.grid_x, s);
    case L_ROW: return ltk::launch_row_reduce(*(const ltk::RowArgs*)args, l.grid_x, s);
    case L_ALL: return ltk::launch_all_reduce(*(const ltk::AllArgs*)args, l.grid_x, s);
    case L_COL: return ltk::launch_col_reduce(*(const ltk::ColArgs*)args, l.grid_x, l.grid_y, s);
    case L_ROWOP: return ltk::launch_row_op(*(const ltk::RowOpArgs*)args, l.grid_x, s);
    case L_GEMM: return ltk::launch_gemm(*(const ltk::GemmArgs*)args, s);
    case L_SPLITPOST: return ltk::launch_split_post(*(const ltk::SplitPostArgs*)args, l.grid_x, s);
    case L_SLICE: return ltk::launch_slice_update(*(const ltk::SliceArgs*)args, l.grid_x, s);
  }
  return hipErrorInvalidValue;
}

static const char* kind_name(LaunchKind k) {
  switch (k) {
    case L_EW: return "lt_ew_kernel";
    case L_ROW: return "lt_row_reduce_kernel";
    case L_ALL: return "lt_all_reduce_kernel";
    case L_COL: return "lt_col_reduce_kernel";
    case L_ROWOP: return "lt_row_op_kernel";
    case L_GEMM: return "lt_gemm_kernel";
    case L_SPLITPOST: return "lt_split_post_kernel";
    case L_SLICE: return "lt_slice_update_kernel";
  }
  return "?";
}

void destroy_device_objects(Plan* plan) {
  for (hipEvent_t& e : plan->events) {
    if (e) (void)hipEventDestroy(e);
    e = nullptr;
  }
  for (GraphEntry& g : plan->graphs.entries)
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
  plan->graphs.entries.clear();
}

// Bind this step's buffers and scalars into the cached plan and launch it.
// use_static: reduction scratch and temporaries live in the library's static device scratch, only
// results are placed in the caller's workspace; one stream, no events, nothing is created.
// params / scalars: the buffers of the plan's device parameters and the values of its
// non-special scalars, in the order of the canonical numbering.
static lt_status execute(lt_ctx* ctx, Plan* plan, const std::vector<BufRef>& params, const std::vector<double>& scalars,
                         std::vector<BufRef>* storage_bufs, bool use_static) {
  const size_t ns = plan->storages.size();
  storage_bufs->assign(ns, nullptr);
  std::vector<void*> ptr(ns, nullptr);
  for (size_t s = 0; s < ns; ++s) {
    const Storage& st = plan->storages[s];
    if (st.param >= 0) {
      (*storage_bufs)[s] = params[st.param];
      ptr[s] = (*storage_bufs)[s]->ptr;
    }
  }
  // fresh storages are taken from the arena for their whole plan lifetime; temporaries go back
  // as soon as the last launch that touches them is enqueued (one stream: reuse is ordered)
  std::vector<std::vector<size_t>> born(plan->launches.size() + 1), dies(plan->launches.size() + 1);
  for (size_t s = 0; s < ns; ++s) {
    const Storage& st = plan->storages[s];
    if (st.param >= 0) continue;
    born[st.first_launch].push_back(s);
    if (!st.bound_to_root) dies[st.last_launch].push_back(s);
  }
  const bool real = ctx->device >= 0;
  const bool prof = real && ctx->profiling && !use_static;
  auto fresh = [&](size_t s) -> bool {
    auto b = std::make_shared<Buffer>();
    b->ptr = ctx->arena.alloc(plan->storages[s].bytes);
    if (!b->ptr) return false;
    b->bytes = plan->storages[s].bytes;
    b->owned = true;
    b->donatable = true;   // library-owned memory may always be reused in place
    b->arena = &ctx->arena;
    (*storage_bufs)[s] = b;
    ptr[s] = b->ptr;
    return true;
  };
  // Memory is settled before the first launch, so that a step either runs whole or not at all (a
  // launch that has run may have updated a donated buffer in place: no second try after that).
  // Normally every fresh storage of the plan fits the workspace at once and is taken up front.
  // Otherwise the storages are taken when their first launch comes and given back behind their
  // last one -- after the same sequence has been tried on a copy of the arena's free list.
  bool upfront = true;
  float* red_partials = ctx->red_partials;
  uint32_t* red_tickets = ctx->red_tickets;
  if (use_static) {
    // layout of the static scratch: partials, tickets, then temporaries handed out front to back
    red_partials = (float*)ctx->static_scratch;
    red_tickets = (uint32_t*)(ctx->static_scratch + kPartialFloats * sizeof(float));
    size_t top = kPartialFloats * sizeof(float) + kTickets * sizeof(uint32_t);
    for (size_t s = 0; s < ns; ++s) {
      const Storage& st = plan->storages[s];
      if (st.param >= 0 || st.bound_to_root) continue;
      const size_t need = (std::max<size_t>(st.bytes, 1) + 255) & ~(size_t)255;
      if (need > ctx->static_scratch_bytes - top)
        return fail(ctx, LT_ERR_OOM, "lt_barrier_static: the plan's temporaries need more than the " +
                                         std::to_string((ctx->static_scratch_bytes - kPartialFloats * sizeof(float) - kTickets * sizeof(uint32_t)) >> 10) +
                                         " KiB that the library's static scratch holds for them");
      auto b = std::make_shared<Buffer>();
      b->ptr = ctx->static_scratch + top;
      b->bytes = st.bytes;
      (*storage_bufs)[s] = b;
      ptr[s] = b->ptr;
      top += need;
    }
    for (size_t s = 0; s < ns; ++s)
      if (plan->storages[s].param < 0 && plan->storages[s].bound_to_root && !fresh(s))
        return fail(ctx, LT_ERR_OOM, "workspace arena exhausted: the plan's results do not fit");
  } else {
    for (size_t s = 0; s < ns && upfront; ++s)
      if (plan->storages[s].param < 0) upfront = fresh(s);
  }
  if (!upfront) {
    for (size_t s = 0; s < ns; ++s)
      if (plan->storages[s].param < 0) {
        (*storage_bufs)[s].reset();
        ptr[s] = nullptr;
      }
    Arena trial = ctx->arena;
    std::vector<void*> tp(ns, nullptr);
    for (size_t li = 0; li < plan->launches.size(); ++li) {
      for (size_t s : born[li])
        if (!(tp[s] = trial.alloc(plan->storages[s].bytes)))
          return fail(ctx, LT_ERR_OOM, "workspace arena exhausted: the plan's temporaries and results do not fit");
      for (size_t s : dies[li]) trial.release(tp[s]);
    }
  }
  // Several streams: only when the schedule found independent work, no per-launch timing is
  // asked for, and the workspace holds every temporary at once (memory given back while the step
  // is still being enqueued could be handed to a launch that runs next to its last reader).
  const bool multi = real && !prof && !use_static && ctx->max_streams > 1 && plan->n_streams > 1 && upfront;
  ctx->last_launches.clear();
  if (prof) {
    while (ctx->events.size() < 2 * plan->launches.size()) {
      hipEvent_t e;
      hipError_t err = hipEventCreate(&e);
      if (err != hipSuccess) return hip_fail(ctx, "hipEventCreate", err);
      ctx->events.push_back(e);
    }
  }
  if (use_static && real) {
    // every call on a GPU shares that GPU's array, which keeps the last call's contents: the
    // tickets must start at zero (a kernel, not a memset: the caller may be capturing a graph)
    hipError_t e = ltk::launch_fill_u32(red_tickets, (uint32_t)kTickets, 0u, ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, "lt_fill_u32_kernel", e);
  }
  // ---- one HIP graph per plan and set of addresses (lt_set_graphs) ------------------------------
  // The launches' arguments are a function of the storages' addresses and the scalars.  When the
  // same ones come back (a training loop whose parameters are updated in place and whose results
  // alternate between the same workspace blocks), the step that was captured then is launched
  // again as a whole.  A signature is captured when it is seen for the second time.
  GraphSlots& gs = plan->graphs;
  const bool may_graph = real && ctx->graphs && !gs.disabled && !prof && !use_static && upfront && !plan->launches.empty();
  uint64_t sig = 0;
  bool capture = false;
  if (may_graph) {
    sig = fnv1a64((const uint8_t*)ptr.data(), ptr.size() * sizeof(void*));
    sig ^= fnv1a64((const uint8_t*)scalars.data(), scalars.size() * sizeof(double)) * 0x9e3779b97f4a7c15ull;
    sig ^= (uint64_t)(multi ? ctx->max_streams : 1) << 56;
    sig |= 1ull;   // (0 marks an empty slot of `seen`)
    for (GraphEntry& g : gs.entries) {
      if (g.sig != sig) continue;
      hipError_t e = hipGraphLaunch(g.exec, ctx->stream);
      if (e != hipSuccess) return hip_fail(ctx, "hipGraphLaunch", e);
      g.used = ++gs.clock;
      for (size_t li = 0; li < plan->launches.size(); ++li)
        for (size_t s : dies[li]) (*storage_bufs)[s].reset();   // behind the graph on the caller's stream
      ctx->stats.kernels_launched += plan->launches.size();
      ctx->stats.graph_launches++;
      return LT_OK;
    }
    for (size_t i = 0; i < GraphSlots::kSeen; ++i) capture |= gs.seen[i] == sig;
    gs.seen[gs.n_seen++ % GraphSlots::kSeen] = sig;
  }
  hipStream_t const caller_stream = ctx->stream;
  if (capture) {
    hipError_t e = hipSuccess;
    if (!ctx->graph_stream) e = hipStreamCreateWithFlags(&ctx->graph_stream, hipStreamNonBlocking);
    if (e == hipSuccess) e = hipStreamBeginCapture(ctx->graph_stream, hipStreamCaptureModeThreadLocal);
    if (e != hipSuccess) {
      (void)hipGetLastError();
      gs.disabled = true;
      capture = false;
    } else {
      ctx->stream = ctx->graph_stream;   // everything below is recorded, not run
    }
  }
  // Ends a capture on every way out: the caller's stream is the context's again, and the
  // recorded work becomes a graph (ok) or is dropped.
  auto end_capture = [&](bool ok) -> hipError_t {
    if (!capture) return hipSuccess;
    capture = false;
    ctx->stream = caller_stream;
    hipGraph_t graph = nullptr;
    hipError_t e = hipStreamEndCapture(ctx->graph_stream, &graph);
    hipGraphExec_t exec = nullptr;
    if (e == hipSuccess && ok) e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (graph) (void)hipGraphDestroy(graph);
    if (e != hipSuccess || !ok) {
      (void)hipGetLastError();
      gs.disabled = true;
      return e != hipSuccess ? e : hipErrorUnknown;
    }
    if (gs.entries.size() >= GraphSlots::kMax) {
      size_t victim = 0;
      for (size_t i = 1; i < gs.entries.size(); ++i)
        if (gs.entries[i].used < gs.entries[victim].used) victim = i;
      (void)hipGraphExecDestroy(gs.entries[victim].exec);
      gs.entries.erase(gs.entries.begin() + victim);
    }
    GraphEntry g;
    g.sig = sig;
    g.exec = exec;
    g.used = ++gs.clock;
    gs.entries.push_back(g);
    return hipSuccess;
  };
  bool forked[kMaxStreams] = {true, false, false, false};
  if (multi) {
    plan->events.resize(plan->launches.size(), nullptr);
    hipError_t e = hipEventRecord(ctx->fork_event, ctx->stream);
    if (e != hipSuccess) {
      (void)end_capture(false);
      return hip_fail(ctx, "hipEventRecord", e);
    }
  }
  const bool was_capturing = capture;
  std::vector<size_t> deferred;
  std::vector<uint8_t> args;
  std::vector<std::string> launch_names;   // kernel instances, when per-launch records are asked for
  size_t pp = 0, sp = 0;
  // join: whatever follows on the caller's stream comes after every side stream's work.  Runs on
  // every way out once a side stream may hold work -- a failed launch included, so that memory the
  // caller gets back (the arena blocks of this step) is never reused under a side stream's kernel.
  auto join_streams = [&]() -> hipError_t {
    hipError_t first = hipSuccess;
    for (int s = 1; s < kMaxStreams; ++s) {
      if (!forked[s]) continue;
      hipError_t e = hipEventRecord(ctx->join_event[s - 1], ctx->side[s - 1]);
      if (e == hipSuccess) e = hipStreamWaitEvent(ctx->stream, ctx->join_event[s - 1], 0);
      if (e != hipSuccess && first == hipSuccess) first = e;
      forked[s] = false;
    }
    return first;
  };
  auto give_up = [&](lt_status st) {
    if (multi) (void)join_streams();
    (void)end_capture(false);
    return st;
  };
  for (size_t li = 0; li < plan->launches.size(); ++li) {
    const Launch& l = plan->launches[li];
    if (!upfront)
      for (size_t s : born[li])
        if (!fresh(s)) return give_up(fail(ctx, LT_ERR_OOM, "internal: the arena differs from its trial run"));
    args = l.args;
    for (; pp < plan->ptr_patches.size() && plan->ptr_patches[pp].launch == li; ++pp) {
      const PtrPatch& p = plan->ptr_patches[pp];
      void* v = (uint8_t*)ptr[p.storage] + p.byte_offset;
      std::memcpy(args.data() + p.offset, &v, sizeof(void*));
    }
    for (; sp < plan->scal_patches.size() && plan->scal_patches[sp].launch == li; ++sp) {
      const ScalPatch& p = plan->scal_patches[sp];
      double v = scalars[p.scalar];
      float f = (float)(p.reciprocal ? 1.0 / v : v);
      std::memcpy(args.data() + p.offset, &f, sizeof(float));
    }
    if (real) {
      // reductions that may run next to each other work in different quarters of the scratch
      if (l.kind == L_ALL) {
        ltk::AllArgs* a = (ltk::AllArgs*)args.data();
        a->partials = red_partials + l.scratch_slot * (kPartialFloats / kScratchSlots);
        a->ticket = red_tickets + l.scratch_slot * (kTickets / kScratchSlots);
      } else if (l.kind == L_COL) {
        ltk::ColArgs* a = (ltk::ColArgs*)args.data();
        a->partials = red_partials + l.scratch_slot * (kPartialFloats / kScratchSlots);
        a->tickets = red_tickets + l.scratch_slot * (kTickets / kScratchSlots);
      } else if (gemm_shared_tiles(l) != 0) {
        ltk::GemmArgs* a = (ltk::GemmArgs*)args.data();
        a->split_ws = red_partials + l.scratch_slot * (kPartialFloats / kScratchSlots);
        a->tickets = red_tickets + l.scratch_slot * (kTickets / kScratchSlots);
      }
      hipStream_t stream = ctx->stream;
      if (multi) {
        if (l.stream > 0) stream = ctx->side[l.stream - 1];
        hipError_t e = hipSuccess;
        if (!forked[l.stream]) {   // the side stream starts behind everything the caller's stream holds
          e = hipStreamWaitEvent(stream, ctx->fork_event, 0);
          forked[l.stream] = true;
        }
        for (size_t w = 0; w < l.waits.size() && e == hipSuccess; ++w) e = hipStreamWaitEvent(stream, plan->events[l.waits[w]], 0);
        if (e != hipSuccess) return give_up(hip_fail(ctx, "hipStreamWaitEvent", e));
      }
      if (prof) (void)hipEventRecord(ctx->events[2 * li], ctx->stream);
      hipError_t e = launch_one(l, args.data(), stream);
      if (e != hipSuccess) return give_up(hip_fail(ctx, kind_name(l.kind), e));
      if (prof) {
        if (launch_names.size() <= li) launch_names.resize(plan->launches.size());
        launch_names[li] = ltk::last_kernel();
      }
      if (prof) (void)hipEventRecord(ctx->events[2 * li + 1], ctx->stream);
      if (multi && l.record) {
        if (!plan->events[li]) e = hipEventCreateWithFlags(&plan->events[li], hipEventDisableTiming);
        if (e == hipSuccess) e = hipEventRecord(plan->events[li], stream);
        if (e != hipSuccess) return give_up(hip_fail(ctx, "hipEventRecord", e));
      }
    }
    for (size_t s : dies[li]) {
      if (multi || was_capturing) {   // (a recorded step has not run yet)
        deferred.push_back(s);
        continue;
      }
      (*storage_bufs)[s].reset();
      ptr[s] = nullptr;
    }
    ctx->stats.kernels_launched++;
  }
  if (multi) {
    hipError_t e = join_streams();
    if (e != hipSuccess) {
      (void)end_capture(false);
      return hip_fail(ctx, "stream join", e);
    }
  }
  if (was_capturing) {
    // nothing has run yet.  The recorded step becomes a graph and is launched; if that cannot be
    // had, this plan gives graphs up and the step is enqueued kernel by kernel after all.
    hipError_t e = end_capture(true);
    if (e == hipSuccess) {
      e = hipGraphLaunch(gs.entries.back().exec, ctx->stream);
      if (e != hipSuccess) return hip_fail(ctx, "hipGraphLaunch", e);
      ctx->stats.graph_launches++;
      ctx->stats.graphs_built++;
    } else {
      ctx->stats.kernels_launched -= plan->launches.size();
      for (size_t s : deferred) (*storage_bufs)[s].reset();
      for (size_t s = 0; s < ns; ++s)
        if (plan->storages[s].param < 0) (*storage_bufs)[s].reset();
      storage_bufs->clear();
      return execute(ctx, plan, params, scalars, storage_bufs, use_static);   // (gs.disabled is set now)
    }
  }
  for (size_t s : deferred) (*storage_bufs)[s].reset();
  if (prof) {
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return hip_fail(ctx, "hipStreamSynchronize", e);
    for (size_t li = 0; li < plan->launches.size(); ++li) {
      lt_launch_record r{};
      std::snprintf(r.kernel, sizeof(r.kernel), "%s", li < launch_names.size() && !launch_names[li].empty() ? launch_names[li].c_str()
                                                                                                        : kind_name(plan->launches[li].kind));
      r.region = plan->launches[li].region;
      (void)hipEventElapsedTime(&r.ms, ctx->events[2 * li], ctx->events[2 * li + 1]);
      r.bytes = plan->launches[li].bytes;
      r.flops = plan->launches[li].flops;
      ctx->last_launches.push_back(r);
    }
  }
  return LT_OK;
}

}  // namespace lt

using namespace lt;

extern "C" {

static lt_status barrier_impl(lt_ctx* ctx, int blocking, lt_barrier_info* info, bool use_static) {
  const uint64_t t0 = now_ns();
  lt_status vs = refresh_views(ctx);   // (section 4.4) a live view is evaluated at its base's current value
  if (vs != LT_OK) return vs;
  Cut cut;
  std::vector<uint8_t> key;
  // Quick lookup (section 7 of the paper: hash while recording): the trace's fingerprint was
  // kept up to date by every recorded node; with the live roots and what each would donate it
  // identifies the canonical form, so a trace seen before needs no walk, no serialisation and
  // no hash -- only the roots (the live pending tensors, ascending id).
  Fingerprint fp = ctx->trace_fp;
  const QuickEntry* quick = nullptr;
  if (ctx->quick_lookup) {
    for (auto& kv : ctx->handles)
      if (kv.second.kind == H_PENDING) cut.roots.push_back(&kv.second);
    fp.mix((uint64_t)ctx->nodes.size());
    for (const Handle* r : cut.roots) {
      fp.mix(((uint64_t)(uint32_t)r->node << 8) | (uint64_t)(uint8_t)r->slot);
      // what the root could donate: the leaf of this trace that reads the buffer the tensor gave
      // up, and whether a live tensor still names that buffer
      const Buffer* b = r->donor.get();
      uint64_t d = 0;
      if (b) {
        auto it = ctx->leaf_of_buffer.find(b);
        d = it == ctx->leaf_of_buffer.end() ? 1 : (((uint64_t)(uint32_t)it->second << 2) | (b->data_refs == 0 ? 3u : 2u));
      }
      fp.mix(d);
    }
    auto it = ctx->quick.find(fp);
    if (it != ctx->quick.end() && it->second.generation == ctx->cache_generation) quick = &it->second;
  }
  uint64_t h = 0;
  Plan* plan = nullptr;
  uint64_t t1, t2;
  if (quick && ctx->quick_lookup == 1) {
    plan = quick->plan;
    h = quick->hash;
    cut.param_nodes = quick->param_nodes;
    cut.scalar_nodes = quick->scalar_nodes;
    cut.order.resize(quick->n_nodes);   // (only its length is looked at on a hit)
    t1 = t2 = now_ns();
    ctx->stats.quick_hits++;
  } else {
    collect_cut(ctx, &cut);
    serialise_cut(ctx, &cut, &key);
    t1 = now_ns();
    h = fnv1a64(key.data(), key.size());
    auto& bucket = ctx->cache[h];
    for (auto& p : bucket)
      if (p->key.size() == key.size() && std::memcmp(p->key.data(), key.data(), key.size()) == 0) plan = p.get();
    t2 = now_ns();
    if (quick) {   // checking mode: the fingerprint's answer must be the canonical key's
      if (quick->plan != plan || quick->param_nodes != cut.param_nodes || quick->scalar_nodes != cut.scalar_nodes)
        return fail(ctx, LT_ERR_ARG, "internal: the record-time fingerprint and the canonical key disagree");
      ctx->stats.quick_hits++;
    }
  }
  const bool hit = plan != nullptr;
  if (!hit) {
    lt_status st = LT_OK;
    std::unique_ptr<Plan> fresh = lower(ctx, cut, &st);
    if (!fresh) {
      auto b = ctx->cache.find(h);
      if (b != ctx->cache.end() && b->second.empty()) ctx->cache.erase(b);
      return st;
    }
    fresh->key = key;
    plan = fresh.get();
    ctx->cache[h].push_back(std::move(fresh));
  }
  if (ctx->quick_lookup && !quick) {
    QuickEntry& e = ctx->quick[fp];
    e.plan = plan;
    e.generation = ctx->cache_generation;
    e.hash = h;
    e.n_nodes = (int32_t)cut.order.size();
    e.param_nodes = cut.param_nodes;
    e.scalar_nodes = cut.scalar_nodes;
  }
  const uint64_t t3 = now_ns();
  std::vector<BufRef> bufs, params(cut.param_nodes.size());
  std::vector<double> scalars(cut.scalar_nodes.size());
  for (size_t k = 0; k < params.size(); ++k) params[k] = ctx->nodes[cut.param_nodes[k]].buffer;
  for (size_t k = 0; k < scalars.size(); ++k) scalars[k] = ctx->nodes[cut.scalar_nodes[k]].value;
  lt_status st = execute(ctx, plan, params, scalars, &bufs, use_static);
  if (st != LT_OK) return st;
  // what a captured step needs of this barrier (lt_step_capture)
  StepRecord& rec = ctx->last_step;
  rec.plan = plan;
  rec.generation = ctx->cache_generation;
  rec.params.resize(params.size());
  for (size_t k = 0; k < params.size(); ++k) {
    const Node& n = ctx->nodes[cut.param_nodes[k]];
    StepParam& sp = rec.params[k];
    sp.tensor = n.src;
    sp.dtype = n.dtype;
    sp.rank = n.rank;
    std::memcpy(sp.dims, n.dims, sizeof(sp.dims));
    sp.donatable = params[k] && params[k]->donatable;
  }
  rec.scalars = scalars;
  rec.roots.resize(cut.roots.size());
  for (size_t r = 0; r < cut.roots.size(); ++r) rec.roots[r] = cut.roots[r]->id;
  rec.bound_plain = ctx->bound_plain;
  ctx->bound_plain = false;
  // result binding: after the barrier every evaluated handle is plain data (or a scalar when
  // folding reduced it to one); a new IR graph starts (section 3)
  for (size_t r = 0; r < cut.roots.size(); ++r) {
    Handle* hd = cut.roots[r];
    const RootBind& rb = plan->roots[r];
    hd->node = -1;
    hd->slot = 0;
    if (rb.kind == RootBind::SCALAR || rb.kind == RootBind::CONST) {
      hd->kind = H_SCALAR;
      hd->value = rb.kind == RootBind::CONST ? rb.value : ctx->nodes[cut.scalar_nodes[rb.index]].value;
      continue;
    }
    hd->kind = H_DATA;
    hd->buf = rb.kind == RootBind::PARAM_ALIAS ? ctx->nodes[cut.param_nodes[rb.index]].buffer : bufs[rb.index];
    hd->buf->data_refs += 1;
  }
  for (auto& kv : ctx->handles) kv.second.donor.reset();
  bufs.clear();
  ctx->nodes.clear();
  ctx->trace_fp = Fingerprint{};
  ctx->leaf_of_buffer.clear();
  ctx->epoch++;
  const uint64_t t4 = now_ns();
  if (blocking && ctx->device >= 0) {
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, LT_ERR_DEVICE, std::string("hipStreamSynchronize: ") + hipGetErrorString(e));
  }
  ctx->last_plan = plan;
  ctx->stats.barriers++;
  (hit ? ctx->stats.cache_hits : ctx->stats.cache_misses)++;
  ctx->stats.regions_launched += plan->n_regions;
  if (!hit) ctx->stats.ns_lowering_total += t3 - t2;
  if (info) {
    info->hash = h;
    info->key_bytes = plan->key.size();
    info->cache_hit = hit ? 1 : 0;
    info->n_nodes = (int32_t)cut.order.size();
    info->n_roots = (int32_t)cut.roots.size();
    info->n_regions = plan->n_regions;
    info->n_launches = (int32_t)plan->launches.size();
    info->bytes_planned = plan->bytes_planned;
    info->flops_planned = plan->flops_planned;
    info->ns_collect = t1 - t0;
    info->ns_hash = t2 - t1;
    info->ns_lower = t3 - t2;
    info->ns_launch = t4 - t3;
  }
  return LT_OK;
}

lt_status lt_barrier(lt_ctx* ctx, int blocking, lt_barrier_info* info) {
  if (!ctx) return LT_ERR_ARG;
  return barrier_impl(ctx, blocking, info, false);
}

lt_status lt_barrier_static(lt_ctx* ctx, int blocking, lt_barrier_info* info) {
  if (!ctx) return LT_ERR_ARG;
  if (!ctx->static_scratch) return fail(ctx, LT_ERR_DEVICE, "lt_barrier_static: " + ctx->static_scratch_error);
  return barrier_impl(ctx, blocking, info, true);
}

// ---- a captured step (section 7 of the paper: skip tracing when the caller guarantees the same
// computation) ---------------------------------------------------------------------------------

lt_status lt_step_capture(lt_ctx* ctx, lt_step** out) {
  if (!ctx || !out) return LT_ERR_ARG;
  const StepRecord& rec = ctx->last_step;
  if (!rec.plan || rec.generation != ctx->cache_generation) return fail(ctx, LT_ERR_ARG, "lt_step_capture: no barrier has run (or its plan is gone)");
  std::unique_ptr<lt_step> step(new lt_step);
  step->ctx = ctx;
  step->rec = rec;
  const Plan* plan = rec.plan;
  step->written.assign(rec.params.size(), 0);
  for (const PtrPatch& p : plan->ptr_patches)
    if (p.write && p.storage >= 0 && plan->storages[p.storage].param >= 0) step->written[plan->storages[p.storage].param] = 1;
  if (rec.bound_plain)
    return fail(ctx, LT_ERR_UNSUPPORTED, "lt_step_capture: during the step lt_assign gave a tensor the plain data (or scalar) of another tensor; "
                                         "that leaves no node in the trace, so running the plan again would not repeat it");
  // every input must be a tensor that can be named again
  for (size_t k = 0; k < rec.params.size(); ++k) {
    auto it = ctx->handles.find(rec.params[k].tensor);
    if (it == ctx->handles.end() || it->second.released)
      return fail(ctx, LT_ERR_HANDLE, "lt_step_capture: input " + std::to_string(k) + " of the step was a tensor that has been released since: keep a step's inputs alive");
  }
  // a buffer the plan overwrites must come back as the value of the tensor it was taken from
  // (x <- f(x)): any other tensor would see its data change under it on the next run
  for (size_t r = 0; r < plan->roots.size(); ++r) {
    const RootBind& rb = plan->roots[r];
    if (rb.kind != RootBind::STORAGE) continue;
    const int param = plan->storages[rb.index].param;
    if (param >= 0 && rec.roots[r] != rec.params[param].tensor)
      return fail(ctx, LT_ERR_UNSUPPORTED, "lt_step_capture: the step writes a result over the buffer of input " + std::to_string(param) +
                                               ", and the result belongs to another tensor");
  }
  for (size_t k = 0; k < rec.params.size(); ++k) {
    if (!step->written[k]) continue;
    bool back = false;
    for (size_t r = 0; r < plan->roots.size(); ++r)
      back |= plan->roots[r].kind == RootBind::STORAGE && plan->storages[plan->roots[r].index].param == (int)k;
    if (!back) return fail(ctx, LT_ERR_UNSUPPORTED, "lt_step_capture: the step uses the buffer of input " + std::to_string(k) + " as scratch");
  }
  *out = step.release();
  return LT_OK;
}

int lt_step_scalars(const lt_step* step, double* out, int cap) {
  if (!step) return -1;
  const int n = (int)step->rec.scalars.size();
  for (int i = 0; i < n && i < cap && out; ++i) out[i] = step->rec.scalars[i];
  return n;
}

void lt_step_free(lt_step* step) { delete step; }

lt_status lt_step_replay(lt_ctx* ctx, lt_step* step, const double* scalars, int n_scalars, int blocking, lt_barrier_info* info) {
  if (!ctx || !step || step->ctx != ctx) return LT_ERR_ARG;
  const uint64_t t0 = now_ns();
  StepRecord& rec = step->rec;
  if (rec.generation != ctx->cache_generation) return fail(ctx, LT_ERR_ARG, "lt_step_replay: the plan cache has been cleared since the step was captured");
  if (!ctx->nodes.empty()) return fail(ctx, LT_ERR_ARG, "lt_step_replay: a trace is pending: run a barrier first");
  if (scalars && n_scalars != (int)rec.scalars.size())
    return fail(ctx, LT_ERR_ARG, "lt_step_replay: the step has " + std::to_string(rec.scalars.size()) + " scalars");
  Plan* plan = rec.plan;
  std::vector<BufRef> params(rec.params.size());
  for (size_t k = 0; k < params.size(); ++k) {
    const StepParam& sp = rec.params[k];
    auto it = ctx->handles.find(sp.tensor);
    if (it == ctx->handles.end() || it->second.released)
      return fail(ctx, LT_ERR_HANDLE, "lt_step_replay: input " + std::to_string(k) + " has been released");
    const Handle& h = it->second;
    bool same = h.kind == H_DATA && h.buf && h.dtype == sp.dtype && h.rank == sp.rank && h.buf->donatable == sp.donatable;
    for (int d = 0; same && d < sp.rank; ++d) same = h.dims[d] == sp.dims[d];
    if (!same) return fail(ctx, LT_ERR_SHAPE, "lt_step_replay: input " + std::to_string(k) + " is not plain data of the captured dtype, shape and donation flag any more");
    if (step->written[k] && h.buf->data_refs != 1)
      return fail(ctx, LT_ERR_ARG, "lt_step_replay: input " + std::to_string(k) + " is updated in place and shares its buffer with another tensor now");
    params[k] = h.buf;
  }
  std::vector<double> vals = rec.scalars;
  if (scalars) vals.assign(scalars, scalars + n_scalars);
  const uint64_t t1 = now_ns();
  std::vector<BufRef> bufs;
  lt_status st = execute(ctx, plan, params, vals, &bufs, false);
  if (st != LT_OK) return st;
  for (size_t r = 0; r < rec.roots.size(); ++r) {
    auto it = ctx->handles.find(rec.roots[r]);
    if (it == ctx->handles.end()) continue;   // released since: the value is dropped
    Handle* hd = &it->second;
    const RootBind& rb = plan->roots[r];
    BufRef nb;
    if (rb.kind == RootBind::STORAGE) nb = bufs[rb.index];
    else if (rb.kind == RootBind::PARAM_ALIAS) nb = params[rb.index];
    if (nb) nb->data_refs += 1;
    if (hd->kind == H_DATA && hd->buf) hd->buf->data_refs -= 1;
    hd->buf = nb;
    hd->node = -1;
    hd->slot = 0;
    hd->donor.reset();
    hd->version++;
    if (nb) {
      hd->kind = H_DATA;
    } else {
      hd->kind = H_SCALAR;
      hd->value = rb.kind == RootBind::CONST ? rb.value : vals[rb.index];
    }
  }
  bufs.clear();
  const uint64_t t2 = now_ns();
  if (blocking && ctx->device >= 0) {
    hipError_t e = hipStreamSynchronize(ctx->stream);
    if (e != hipSuccess) return fail(ctx, LT_ERR_DEVICE, std::string("hipStreamSynchronize: ") + hipGetErrorString(e));
  }
  ctx->last_plan = plan;
  ctx->stats.replays++;
  ctx->stats.regions_launched += plan->n_regions;
  if (info) {
    *info = lt_barrier_info{};
    info->cache_hit = 1;
    info->n_roots = (int32_t)rec.roots.size();
    info->n_regions = plan->n_regions;
    info->n_launches = (int32_t)plan->launches.size();
    info->bytes_planned = plan->bytes_planned;
    info->flops_planned = plan->flops_planned;
    info->ns_collect = t1 - t0;
    info->ns_launch = t2 - t1;
  }
  return LT_OK;
}

lt_status lt_fetch(lt_ctx* ctx, lt_tensor t, void* host_dst, size_t nbytes) {
  if (!ctx || !host_dst) return LT_ERR_ARG;
  auto it = ctx->handles.find(t);
  if (it == ctx->handles.end() || it->second.released) return fail(ctx, LT_ERR_HANDLE, "lt_fetch: unknown or released tensor id");
  if (it->second.view_base) {
    lt_status vs = refresh_views(ctx);
    if (vs != LT_OK) return vs;
  }
  if (it->second.kind == H_PENDING) {
    lt_status st = lt_barrier(ctx, 1, nullptr);
    if (st != LT_OK) return st;
    it = ctx->handles.find(t);
  }
  Handle& h = it->second;
  const size_t bytes = (size_t)numel(h.dims, h.rank) * dtype_size(h.dtype);
  if (nbytes != bytes) return fail(ctx, LT_ERR_ARG, "lt_fetch: nbytes does not match the tensor");
  if (h.kind == H_SCALAR) {
    if (h.dtype == LT_F32) { float v = (float)h.value; std::memcpy(host_dst, &v, 4); }
    else if (h.dtype == LT_I32) { int32_t v = (int32_t)h.value; std::memcpy(host_dst, &v, 4); }
    else if (h.dtype == LT_I64) { int64_t v = (int64_t)h.value; std::memcpy(host_dst, &v, 8); }
    else { float f = (float)h.value; uint32_t u; std::memcpy(&u, &f, 4); uint16_t b = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16); std::memcpy(host_dst, &b, 2); }
    return LT_OK;
  }
  if (ctx->device < 0) return fail(ctx, LT_ERR_DEVICE, "lt_fetch: a null device holds no data");
  hipError_t e = hipMemcpyAsync(host_dst, h.buf->ptr, bytes, hipMemcpyDeviceToHost, ctx->stream);
  if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
  if (e != hipSuccess) return fail(ctx, LT_ERR_DEVICE, std::string("lt_fetch: ") + hipGetErrorString(e));
  return LT_OK;
}

}  // extern "C"
