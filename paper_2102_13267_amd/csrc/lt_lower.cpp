// Lowering of a cut trace into a cached plan (runs on a cache miss only).
//
// The paper hands the trace to a domain-specific compiler (section 4: op lowerings, compile,
// cache).  Here the "compiler" is: fold the special scalars 0 and 1 (section 4.1), partition the
// DAG into fused regions, emit one bytecode program per elementwise chain, plan buffers with
// input/output donation (section 4.3) and pre-build the kernel argument blocks.  No code is
// generated, so a miss costs microseconds.
//
// Partition rules (deterministic; an independent implementation must produce the same list):
//   classes   LEAF (device_data, scalar, constant), VIEW (expand / reshape that is not a root),
//             EW (elementwise, permute, root views), ROW / COL / ALL (reductions by axis; the
//             fixed row operators are ROW), MM (matmul).
//   pass 0    every live EW / ROW / COL / ALL / MM node is a region of its own.
//   pass 1    plain reductions absorb, walking down from the anchor, every elementwise node of the
//             reduced tensor's shape whose users all lie inside the region (prologue).
//   pass 2    in canonical order each still-single elementwise node joins the region of one of
//             its producers: an anchored region as epilogue (same shape as the anchor's result;
//             a global reduction also takes a "finaliser" of <= 65536 elements), else elementwise
//             regions of equal shape are merged; never through a view, never if the region graph
//             would get a cycle, never beyond the caps (8 inputs, 8 outputs, inputs + members <= 32).
//   pass 3    donation: a root may overwrite its donated input when all other readers can be
//             ordered first (ordering edges are added) and the writer reads it index-aligned.
//   pass 4    regions run in topological order, smallest id (anchor, else first member) first.
#include <algorithm>
#include <cstdlib>
#include <cmath>
#include <cstdio>
#include <functional>
#include <set>

#include "lt_core.h"

namespace lt {
namespace {

enum Class : uint8_t { C_DEAD, C_LEAF, C_VIEW, C_EW, C_ROW, C_COL, C_ALL, C_MM, C_SLICE };

struct Region {
  Class kind;
  int32_t anchor;                 // canonical index or -1
  std::vector<int32_t> members;   // sorted canonical indices
  bool has_fin = false;
  bool sealed = false;              // ends in a layout permute: takes no further members
  std::vector<int64_t> fin_shape;
  std::vector<Region*> extra_succ;   // ordering-only edges added by donation
  bool alive = true;
  int32_t id() const { return anchor >= 0 ? anchor : members.front(); }
  bool has(int32_t m) const { return std::binary_search(members.begin(), members.end(), m); }
};

struct Lowering {
  lt_ctx* ctx;
  const Cut& cut;
  int32_t N;
  std::vector<const Node*> nd;
  std::vector<std::vector<Val>> rins;       // operands after folding (canonical indices)
  std::vector<Val> fwd;                     // node -> replacement (node == -1: none)
  std::vector<Val> root_vals;
  std::vector<Class> cls;
  std::vector<char> live, is_root;
  std::vector<std::vector<int32_t>> users;
  std::vector<std::unique_ptr<Region>> pool;
  std::vector<Region*> region_of;
  std::vector<Region*> ordered;
  std::string err;
  lt_status status = LT_OK;

  explicit Lowering(lt_ctx* c, const Cut& k) : ctx(c), cut(k), N((int32_t)k.order.size()) {}

  bool bad(lt_status s, const std::string& m) {
    if (status == LT_OK) {
      status = s;
      err = m;
    }
    return false;
  }

  // ---- value helpers -----------------------------------------------------------------------
  int out_rank(Val v) const {
    const Node* n = nd[v.node];
    return (n->op == LT_OP_LAYER_NORM && v.slot > 0) ? n->rank - 1 : n->rank;
  }
  std::vector<int64_t> out_shape(Val v) const {
    const Node* n = nd[v.node];
    return std::vector<int64_t>(n->dims, n->dims + out_rank(v));
  }
  uint8_t out_dtype(Val v) const {
    const Node* n = nd[v.node];
    return (n->op == LT_OP_LAYER_NORM && v.slot > 0) ? (uint8_t)LT_F32 : n->dtype;
  }
  std::vector<int64_t> shape_of(int32_t i) const { return std::vector<int64_t>(nd[i]->dims, nd[i]->dims + nd[i]->rank); }
  static int64_t count(const std::vector<int64_t>& s) {
    int64_t n = 1;
    for (int64_t d : s) n *= d;
    return n;
  }
  Val res(Val v) const {
    while (v.slot == 0 && fwd[v.node].node >= 0) v = fwd[v.node];
    return v;
  }
  static bool plain_reduce(uint16_t op) { return op == LT_OP_SUM || op == LT_OP_AMAX || op == LT_OP_MEAN; }
  static bool is_unary(uint16_t op) { return op >= LT_OP_NEG && op <= LT_OP_SIGMOID; }
  static bool is_binary(uint16_t op) { return op >= LT_OP_ADD && op <= LT_OP_GELU_GRAD; }
  static bool is_row_op(uint16_t op) { return op >= LT_OP_SOFTMAX && op <= LT_OP_XENT_GRAD; }

  // value of a node known at lowering time (constants 0 / 1, seen through views)
  bool const_of(Val v, double* out, const std::vector<std::vector<Val>>& ins) const {
    v = res(v);
    const Node* n = nd[v.node];
    if (n->op == OP_CONSTANT) {
      *out = n->attrs[0].is_float ? n->attrs[0].v.f : (double)n->attrs[0].v.i;
      return true;
    }
    if (n->op == LT_OP_EXPAND || n->op == LT_OP_RESHAPE) return const_of(ins[v.node][0], out, ins);
    return false;
  }
  bool is_imm(Val v) const {
    const Node* n = nd[v.node];
    if (n->op == OP_CONSTANT || n->op == OP_SCALAR_PARAM) return true;
    if (n->op == LT_OP_EXPAND || n->op == LT_OP_RESHAPE) return is_imm(rins[v.node][0]);
    return false;
  }
  Val base(Val v) const {
    while (cls[v.node] == C_VIEW) v = rins[v.node][0];
    return v;
  }

  // ---- step 1: special-scalar folding ------------------------------------------------------------
  void fold() {
    std::vector<std::vector<Val>> ins(N);
    for (int32_t i = 0; i < N; ++i)
      for (int k = 0; k < nd[i]->n_in; ++k)
        ins[i].push_back(Val{cut.index_of[nd[i]->ins[k].node], nd[i]->ins[k].slot});
    fwd.assign(N, Val{-1, 0});
    std::vector<char> drop_alpha(N, 0);
    for (int32_t i = 0; i < N; ++i) {
      const Node* n = nd[i];
      auto same = [&](Val v) {
        v = res(v);
        return out_shape(v) == shape_of(i) && out_dtype(v) == n->dtype;
      };
      const auto& o = ins[i];
      double c;
      if (n->op == LT_OP_ADD && o.size() == 3 && const_of(o[2], &c, ins) && c == 1.0) drop_alpha[i] = 1;
      const bool two = o.size() == 2 || drop_alpha[i];
      if (n->op == LT_OP_MUL) {
        if (const_of(o[1], &c, ins) && c == 1.0 && same(o[0])) fwd[i] = res(o[0]);
        else if (const_of(o[0], &c, ins) && c == 1.0 && same(o[1])) fwd[i] = res(o[1]);
      } else if (n->op == LT_OP_ADD && two) {
        if (const_of(o[1], &c, ins) && c == 0.0 && same(o[0])) fwd[i] = res(o[0]);
        else if (const_of(o[0], &c, ins) && c == 0.0 && same(o[1])) fwd[i] = res(o[1]);
      } else if (n->op == LT_OP_SUB) {
        if (const_of(o[1], &c, ins) && c == 0.0 && same(o[0])) fwd[i] = res(o[0]);
      } else if (n->op == LT_OP_DIV) {
        if (const_of(o[1], &c, ins) && c == 1.0 && same(o[0])) fwd[i] = res(o[0]);
      }
    }
    rins.assign(N, {});
    for (int32_t i = 0; i < N; ++i) {
      for (Val v : ins[i]) rins[i].push_back(res(v));
      if (drop_alpha[i]) rins[i].resize(2);
    }
    for (const Handle* h : cut.roots) root_vals.push_back(res(Val{cut.index_of[h->node], h->slot}));
    live.assign(N, 0);
    std::vector<int32_t> stack;
    for (Val v : root_vals) stack.push_back(v.node);
    while (!stack.empty()) {
      int32_t i = stack.back();
      stack.pop_back();
      if (live[i]) continue;
      live[i] = 1;
      for (Val v : rins[i]) stack.push_back(v.node);
    }
    is_root.assign(N, 0);
    for (Val v : root_vals) is_root[v.node] = 1;
  }

  // ---- step 2: classes and users ------------------------------------------------------------------
  bool classify() {
    users.assign(N, {});
    for (int32_t j = 0; j < N; ++j) {
      if (!live[j]) continue;
      for (Val v : rins[j])
        if (std::find(users[v.node].begin(), users[v.node].end(), j) == users[v.node].end()) users[v.node].push_back(j);
    }
    cls.assign(N, C_DEAD);
    for (int32_t i = 0; i < N; ++i) {
      if (!live[i]) continue;
      const uint16_t op = nd[i]->op;
      if (op == OP_DEVICE_DATA || op == OP_SCALAR_PARAM || op == OP_CONSTANT) cls[i] = C_LEAF;
      else if (op == LT_OP_EXPAND || op == LT_OP_RESHAPE) cls[i] = is_root[i] ? C_EW : C_VIEW;
      else if (op == LT_OP_PERMUTE) {
        // a permutation that only feeds contractions is addressing (operand strides), not a copy
        bool only_mm = !is_root[i] && !users[i].empty();
        for (int32_t u : users[i]) only_mm = only_mm && nd[u]->op == LT_OP_MATMUL;
        cls[i] = only_mm ? C_VIEW : C_EW;
      } else if (op == LT_OP_NARROW) {
        // a window is addressing (an offset and the base's strides) for the consumers that can
        // address it: elementwise ops, contractions, permutations; otherwise a copy
        bool addr = !is_root[i] && !users[i].empty();
        for (int32_t u : users[i])
          addr = addr && (is_unary(nd[u]->op) || is_binary(nd[u]->op) || nd[u]->op == LT_OP_MATMUL || nd[u]->op == LT_OP_PERMUTE);
        cls[i] = addr ? C_VIEW : C_EW;
      } else if (op == LT_OP_SLICE_UPDATE) cls[i] = C_SLICE;
      else if (is_unary(op) || is_binary(op)) cls[i] = C_EW;
      else if (plain_reduce(op)) {
        const int in_rank = out_rank(rins[i][0]);
        if (nd[i]->n_attr == 0 || in_rank <= 1) cls[i] = C_ALL;
        else if (nd[i]->attrs[0].v.i == in_rank - 1) cls[i] = C_ROW;
        else if (nd[i]->attrs[0].v.i == 0) cls[i] = C_COL;
        else return bad(LT_ERR_UNSUPPORTED, "reduction over a middle axis has no lowering");
      } else if (is_row_op(op)) cls[i] = C_ROW;
      else if (op == LT_OP_MATMUL) cls[i] = C_MM;
      else return bad(LT_ERR_UNSUPPORTED, "opcode has no lowering");
    }
    return true;
  }

  std::vector<int32_t> eff_users(int32_t i) const {
    std::vector<int32_t> out, stack(users[i]);
    while (!stack.empty()) {
      int32_t u = stack.back();
      stack.pop_back();
      if (cls[u] == C_VIEW) stack.insert(stack.end(), users[u].begin(), users[u].end());
      else if (std::find(out.begin(), out.end(), u) == out.end()) out.push_back(u);
    }
    return out;
  }

  // ---- region bookkeeping ----------------------------------------------------------------------------
  void region_io(const std::vector<int32_t>& members, std::vector<Val>* inputs, std::vector<Val>* outputs) const {
    auto in_set = [&](int32_t m) { return std::binary_search(members.begin(), members.end(), m); };
    inputs->clear();
    outputs->clear();
    for (int32_t m : members)
      for (Val v : rins[m]) {
        if (in_set(v.node) || is_imm(v)) continue;
        if (std::find(inputs->begin(), inputs->end(), v) == inputs->end()) inputs->push_back(v);
      }
    for (int32_t m : members) {
      const int n_out = nd[m]->op == LT_OP_LAYER_NORM ? 3 : 1;
      for (int s = 0; s < n_out; ++s) {
        const Val v{m, s};
        bool ext = std::find(root_vals.begin(), root_vals.end(), v) != root_vals.end();
        for (int32_t u : users[m])
          if (!in_set(u) && std::find(rins[u].begin(), rins[u].end(), v) != rins[u].end()) ext = true;
        if (ext) outputs->push_back(v);
      }
    }
  }

  bool caps_ok(const std::vector<int32_t>& members) const {
    std::vector<Val> in, out;
    region_io(members, &in, &out);
    // a permutation reads its operand at other positions than it writes: the operand has to be
    // in memory, so its producer never shares a region with the permutation
    for (int32_t m : members)
      if (nd[m]->op == LT_OP_PERMUTE && std::binary_search(members.begin(), members.end(), rins[m][0].node)) return false;
    // the same for anything read through a view (a window, a broadcast, a reshape): the value
    // under the view must be in memory, so it is never computed by the region that reads the view
    for (int32_t m : members)
      for (Val v : rins[m])
        if (cls[v.node] == C_VIEW && std::binary_search(members.begin(), members.end(), base(v).node)) return false;
    return (int)in.size() <= kMaxRegionInputs && (int)out.size() <= kMaxRegionOutputs &&
           (int)(in.size() + members.size()) <= kMaxRegionSlots;
  }

  static std::vector<int32_t> merged(const std::vector<int32_t>& a, const std::vector<int32_t>& b) {
    std::vector<int32_t> out(a.size() + b.size());
    std::merge(a.begin(), a.end(), b.begin(), b.end(), out.begin());
    return out;
  }

  void unite(Region* home, Region* other) {
    for (int32_t m : other->members) region_of[m] = home;
    home->members = merged(home->members, other->members);
    other->alive = false;
    other->members.clear();
  }

  std::vector<Region*> successors(const Region* r) const {
    std::vector<Region*> out(r->extra_succ);
    for (int32_t m : r->members)
      for (int32_t u : eff_users(m)) {
        Region* ru = region_of[u];
        if (ru != r && std::find(out.begin(), out.end(), ru) == out.end()) out.push_back(ru);
      }
    return out;
  }

  bool reachable(const Region* src, const Region* dst) const {
    std::vector<const Region*> stack{src}, seen;
    while (!stack.empty()) {
      const Region* x = stack.back();
      stack.pop_back();
      if (x == dst) return true;
      if (std::find(seen.begin(), seen.end(), x) != seen.end()) continue;
      seen.push_back(x);
      for (Region* s : successors(x)) stack.push_back(s);
    }
    return false;
  }

  bool can_union(const Region* a, const Region* b) const {
    for (Region* x : successors(a))
      if (x != b && reachable(x, b)) return false;
    for (Region* x : successors(b))
      if (x != a && reachable(x, a)) return false;
    return true;
  }

  bool compatible(const Region* r, int32_t i) const {
    if (r->sealed) return false;
    const std::vector<int64_t> shape = shape_of(i);
    if (r->kind == C_EW) return shape == shape_of(r->members.front());
    const int32_t a = r->anchor;
    if (r->kind == C_MM) return shape == shape_of(a);
    if (plain_reduce(nd[a]->op)) {
      if (shape == shape_of(a)) return true;
      if (r->kind == C_ALL && !shape.empty() && count(shape) <= kMaxFinaliserElems &&
          (!r->has_fin || r->fin_shape == shape))
        return true;
    }
    return false;
  }

  // ---- step 3: partition ------------------------------------------------------------------------------
  void partition() {
    region_of.assign(N, nullptr);
    for (int32_t i = 0; i < N; ++i) {
      if (cls[i] < C_EW) continue;
      pool.emplace_back(new Region{cls[i], cls[i] == C_EW ? -1 : i, {i}});
      region_of[i] = pool.back().get();
    }
    if (!ctx->fusion) return;   // debugging switch: every op runs as a kernel of its own
    // pass 1: prologue absorption into plain reductions
    for (int32_t a = 0; a < N; ++a) {
      if (!(cls[a] == C_ROW || cls[a] == C_COL || cls[a] == C_ALL) || !plain_reduce(nd[a]->op)) continue;
      Region* r = region_of[a];
      const std::vector<int64_t> in_shape = out_shape(rins[a][0]);
      for (int32_t i = a - 1; i >= 0; --i) {
        if (cls[i] != C_EW || region_of[i]->members.size() != 1 || is_root[i]) continue;
        if (shape_of(i) != in_shape || users[i].empty()) continue;
        bool inside = true;
        for (int32_t u : users[i]) inside &= r->has(u);
        if (!inside) continue;
        if (!caps_ok(merged(r->members, {i}))) continue;
        unite(r, region_of[i]);
      }
    }
    // pass 2: epilogue / finaliser / elementwise grouping
    for (int32_t i = 0; i < N; ++i) {
      if (cls[i] != C_EW || region_of[i]->members.size() != 1) continue;
      if (nd[i]->op == LT_OP_PERMUTE) {
        // a permutation of a bare contraction result that nothing else reads becomes the
        // contraction's output layout
        const Val v = rins[i][0];
        const int32_t a = v.node;
        if (cls[a] == C_MM && v.slot == 0 && region_of[a]->members.size() == 1 && users[a].size() == 1 && users[a][0] == i &&
            !is_root[a]) {
          Region* r = region_of[a];
          unite(r, region_of[i]);
          r->sealed = true;
        }
        continue;
      }
      std::vector<Region*> cand;
      for (Val v : rins[i]) {
        Region* r = region_of[v.node];
        if (r && std::find(cand.begin(), cand.end(), r) == cand.end()) cand.push_back(r);
      }
      std::stable_sort(cand.begin(), cand.end(), [](const Region* x, const Region* y) {
        const int kx = x->kind != C_EW ? 0 : 1, ky = y->kind != C_EW ? 0 : 1;
        if (kx != ky) return kx < ky;
        return x->id() > y->id();
      });
      Region* home = region_of[i];
      for (Region* r : cand) {
        if (!r->alive || r == home) continue;
        if (r->kind != C_EW) {
          if (home->members.size() != 1) continue;
          if (!compatible(r, i) || !caps_ok(merged(r->members, {i})) || !can_union(r, home)) continue;
          if (r->kind == C_ALL && shape_of(i) != shape_of(r->anchor)) {
            r->has_fin = true;
            r->fin_shape = shape_of(i);
          }
          unite(r, home);
          home = r;
          // elementwise producers of i that feed nothing but this region (e.g. beta*m of an
          // optimiser update) are computed by the region's post program too
          for (Val v : rins[i]) {
            Region* q = region_of[v.node];
            if (!q || q == home || q->kind != C_EW || !q->alive) continue;
            if (shape_of(q->members.front()) != shape_of(i)) continue;
            bool ok = true;
            for (int32_t m : q->members) {
              ok = ok && !is_root[m];
              // (what the anchor itself reads -- a contraction's operand -- must exist in memory)
              for (int32_t u : users[m]) ok = ok && (q->has(u) || home->has(u)) && u != home->anchor;
            }
            if (!ok) continue;
            if (!caps_ok(merged(home->members, q->members)) || !can_union(home, q)) continue;
            unite(home, q);
          }
        } else if (home->kind == C_EW) {
          if (!compatible(r, i) || !caps_ok(merged(r->members, home->members))) continue;
          if (!can_union(r, home)) continue;
          unite(r, home);
          home = r;
        }
      }
    }
  }

  // ---- step 4: donation and order ---------------------------------------------------------------------
  struct InPlace { Val v; uint32_t param; };
  std::vector<std::vector<InPlace>> inplace_of_region;   // parallel to `alive_regions`
  std::vector<Region*> alive_regions;                    // sorted by id
  std::vector<int32_t> inplace_root;                     // per root: param ordinal or -1

  int region_pos(const Region* r) const {
    return (int)(std::find(alive_regions.begin(), alive_regions.end(), r) - alive_regions.begin());
  }

  void donate_and_order() {
    for (auto& r : pool)
      if (r->alive) alive_regions.push_back(r.get());
    std::sort(alive_regions.begin(), alive_regions.end(), [](const Region* x, const Region* y) { return x->id() < y->id(); });
    inplace_of_region.assign(alive_regions.size(), {});
    inplace_root.assign(cut.roots.size(), -1);
    // canonical index of every device parameter
    std::vector<int32_t> pnode;
    for (int32_t idx : cut.param_nodes) pnode.push_back(cut.index_of[idx]);
    for (size_t k = 0; k < cut.roots.size(); ++k) {
      const uint32_t d = cut.donors[k];
      const Val v = root_vals[k];
      if (d == 0xFFFFFFFFu || !region_of[v.node]) continue;
      Region* rw = region_of[v.node];
      auto& mine = inplace_of_region[region_pos(rw)];
      bool dup = false;
      for (const InPlace& ip : mine) dup |= (ip.v == v);
      if (dup) continue;
      const Buffer* buf = nd[pnode[d]]->buffer.get();
      auto names_donor = [&](Val x) {
        return nd[x.node]->op == OP_DEVICE_DATA && x.slot == 0 && nd[x.node]->buffer.get() == buf;
      };
      bool ok = true;
      // another live tensor that folding resolved to the donor leaf itself (b = a * 1) is bound
      // to the donor's buffer after the barrier and must keep seeing the old value (section 4.3)
      for (size_t j = 0; j < root_vals.size(); ++j)
        if (j != k && names_donor(root_vals[j])) ok = false;
      // two leaves on one buffer (a second handle made by lt_assign): the launch schedule tracks
      // hazards per parameter, so a buffer known under two parameter numbers is never written
      int leaves = 0;
      for (int32_t pi : pnode) leaves += live[pi] && nd[pi]->buffer.get() == buf;
      if (leaves > 1) ok = false;
      std::vector<Region*> readers;
      for (Region* r : alive_regions) {
        bool reads = false;
        for (int32_t m : r->members)
          for (Val x : rins[m]) reads |= names_donor(base(x));
        if (!reads) continue;
        if (r == rw) {
          for (int32_t m : r->members)
            for (Val x : rins[m])
              if (names_donor(base(x))) {
                // a window update may overwrite its own base (operand 0, read in place) ...
                if (m == rw->anchor && nd[m]->op == LT_OP_SLICE_UPDATE && names_donor(x) && x == rins[m][0] && !names_donor(base(rins[m][1]))) continue;
                // ... everything else must read the donor position by position
                if (m == rw->anchor || !names_donor(x) || nd[m]->op == LT_OP_PERMUTE || nd[m]->op == LT_OP_EXPAND ||
                    nd[m]->op == LT_OP_RESHAPE || nd[m]->op == LT_OP_NARROW)
                  ok = false;
              }
        } else {
          readers.push_back(r);
        }
      }
      if (ok)
        for (Region* r : readers) ok &= !reachable(rw, r);
      if (!ok) continue;
      for (Region* r : readers)
        if (std::find(r->extra_succ.begin(), r->extra_succ.end(), rw) == r->extra_succ.end()) r->extra_succ.push_back(rw);
      mine.push_back(InPlace{v, d});
      inplace_root[k] = (int32_t)d;
    }
    // Kahn, smallest id first
    std::vector<std::vector<Region*>> succ(alive_regions.size());
    std::vector<int> indeg(alive_regions.size(), 0);
    for (size_t i = 0; i < alive_regions.size(); ++i) {
      succ[i] = successors(alive_regions[i]);
      for (Region* s : succ[i]) indeg[region_pos(s)]++;
    }
    std::vector<char> done(alive_regions.size(), 0);
    while (ordered.size() < alive_regions.size()) {
      size_t pick = alive_regions.size();
      for (size_t i = 0; i < alive_regions.size(); ++i)
        if (!done[i] && indeg[i] == 0) {
          pick = i;   // alive_regions is sorted by id, so the first ready one is the smallest
          break;
        }
      if (pick == alive_regions.size()) {
        bad(LT_ERR_UNSUPPORTED, "internal: region graph has a cycle");
        return;
      }
      done[pick] = 1;
      ordered.push_back(alive_regions[pick]);
      for (Region* s : succ[pick]) indeg[region_pos(s)]--;
    }
  }

  std::string plan_text() const {
    std::string out;
    char tmp[64];
    for (size_t k = 0; k < ordered.size(); ++k) {
      const Region* r = ordered[k];
      static const char* names[] = {"DEAD", "LEAF", "VIEW", "EW", "ROW", "COL", "ALL", "MM", "SLICE"};
      std::vector<Val> in, o;
      region_io(r->members, &in, &o);
      if (k) out += "\n";
      out += "R" + std::to_string(k) + " " + names[r->kind] + " anchor=" + (r->anchor < 0 ? "-" : std::to_string(r->anchor)) + " members=[";
      for (size_t i = 0; i < r->members.size(); ++i) out += (i ? "," : "") + std::to_string(r->members[i]);
      out += "] inputs=[";
      for (size_t i = 0; i < in.size(); ++i) {
        std::snprintf(tmp, sizeof(tmp), "%s%d.%d", i ? "," : "", in[i].node, in[i].slot);
        out += tmp;
      }
      out += "] outputs=[";
      for (size_t i = 0; i < o.size(); ++i) {
        std::snprintf(tmp, sizeof(tmp), "%s%d.%d", i ? "," : "", o[i].node, o[i].slot);
        out += tmp;
      }
      out += "] inplace=[";
      const auto& ips = inplace_of_region[region_pos(r)];
      for (size_t i = 0; i < ips.size(); ++i) {
        std::snprintf(tmp, sizeof(tmp), "%s%d.%d->p%u", i ? "," : "", ips[i].v.node, ips[i].v.slot, ips[i].param);
        out += tmp;
      }
      out += "]";
    }
    return out;
  }

  // ================= code generation =================================================================
  Plan* plan = nullptr;
  std::vector<std::vector<int32_t>> storage_of;   // [node][slot] -> storage index or -1
  std::vector<int32_t> param_ordinal;             // canonical node -> device parameter ordinal or -1
  std::vector<int32_t> scalar_ordinal;            // canonical node -> scalar ordinal or -1

  // Addressing of a value relative to an iteration space: the storage that holds it, the element
  // offset of its first element and the element stride along every dimension of the space (0 where
  // it is broadcast).
  struct Access {
    int32_t storage = -1;
    uint8_t dtype = 0;
    int64_t offset = 0;
    std::vector<int64_t> stride;
  };

  static std::vector<int64_t> contiguous(const std::vector<int64_t>& shape) {
    std::vector<int64_t> s(shape.size(), 1);
    for (int i = (int)shape.size() - 2; i >= 0; --i) s[i] = s[i + 1] * shape[i + 1];
    return s;
  }

  // A value as an address pattern: storage, shape, element strides, element offset.
  struct Pattern {
    int32_t storage = -1;
    int64_t offset = 0;
    std::vector<int64_t> shape, stride;
  };

  // The result of view node i (expand / reshape / permute / narrow) as a pattern over the pattern
  // of its operand: views move no data.
  bool apply_view(int32_t i, const Pattern& in, Pattern* out) {
    const Node* n = nd[i];
    const std::vector<int64_t> oshape = shape_of(i);
    out->storage = in.storage;
    out->offset = in.offset;
    out->shape = oshape;
    if (n->op == LT_OP_EXPAND) {
      out->stride.assign(oshape.size(), 0);
      const int off = (int)oshape.size() - (int)in.shape.size();
      for (size_t d = 0; d < in.shape.size(); ++d) out->stride[d + off] = in.shape[d] == 1 ? 0 : in.stride[d];
      return true;
    }
    if (n->op == LT_OP_PERMUTE) {
      out->stride.resize(oshape.size());
      for (size_t d = 0; d < oshape.size(); ++d) out->stride[d] = in.stride[n->attrs[d].v.i];
      return true;
    }
    if (n->op == LT_OP_NARROW) {
      int64_t axis = 0, start = 0;
      for (int k = 0; k < n->n_attr; ++k) {
        if (n->attrs[k].key == LT_ATTR_AXIS) axis = n->attrs[k].v.i;
        if (n->attrs[k].key == LT_ATTR_START) start = n->attrs[k].v.i;
      }
      out->stride = in.stride;
      out->offset += start * in.stride[axis];
      return true;
    }
    // reshape: only of a dense row-major value (an offset is fine)
    if (in.stride != contiguous(in.shape)) return bad(LT_ERR_UNSUPPORTED, "reshape of a strided or broadcast view has no lowering");
    out->stride = contiguous(oshape);
    return true;
  }

  // pattern of value v, seen through its chain of view nodes
  bool pattern_of(Val v, Pattern* out) {
    if (cls[v.node] != C_VIEW) {
      const int32_t s = storage_of[v.node][v.slot];
      if (s < 0) return bad(LT_ERR_UNSUPPORTED, "internal: operand has no storage");
      out->storage = s;
      out->offset = 0;
      out->shape = out_shape(v);
      out->stride = contiguous(out->shape);
      return true;
    }
    Pattern in;
    if (!pattern_of(rins[v.node][0], &in)) return false;
    return apply_view(v.node, in, out);
  }

  // access of operand v from iteration space `space`; via >= 0: as seen through member `via`, a
  // view op that is materialised by this region (a copy) and addresses its operand in its own way
  bool make_access(Val v, const std::vector<int64_t>& space, int32_t via, Access* out) {
    Pattern pat;
    if (!pattern_of(v, &pat)) return false;
    if (via >= 0) {
      Pattern seen;
      if (!apply_view(via, pat, &seen)) return false;
      pat = seen;
    }
    out->storage = pat.storage;
    out->offset = pat.offset;
    out->dtype = out_dtype(base(v));
    out->stride.assign(space.size(), 0);
    const int off = (int)space.size() - (int)pat.shape.size();
    if (off < 0) return bad(LT_ERR_UNSUPPORTED, "internal: operand rank exceeds its iteration space");
    for (size_t d = 0; d < pat.shape.size(); ++d) out->stride[d + off] = (pat.shape[d] == 1 && space[d + off] != 1) ? 0 : pat.stride[d];
    for (size_t d = 0; d < space.size(); ++d)
      if (space[d] == 1) out->stride[d] = 0;
    return true;
  }

  struct ProgBuild {
    ltk::EwProg prog{};
    struct In { uint32_t first; int32_t second; int64_t byte_offset; };
    std::vector<In> in_storage;                               // (input index, storage, offset into it)
    std::vector<std::pair<uint32_t, int32_t>> out_storage;   // (output index, storage)
    struct SP { uint32_t index; int32_t scalar; bool recip; };
    std::vector<SP> scal_patch;
    uint64_t bytes = 0;
  };

  // Build the bytecode program for `members` (sorted) over iteration space `space`.
  // anchor: value entering through prog.anchor_slot (node -1: none).
  // outputs: values the program must store.
  bool build_prog(const std::vector<int32_t>& members, const std::vector<int64_t>& space, Val anchor,
                  const std::vector<Val>& outputs, bool full_vec, ProgBuild* pb) {
    ltk::EwProg& p = pb->prog;
    const int64_t n = count(space);
    if (n >= ((int64_t)1 << 32)) return bad(LT_ERR_UNSUPPORTED, "iteration space of 2^32 or more elements");
    p.n = (uint64_t)n;
    p.cols = (uint32_t)(space.empty() ? 1 : std::max<int64_t>(space.back(), 1));
    p.vec_ok = (p.cols % 4u == 0u) ? 1u : 0u;
    p.full_vec_ok = (full_vec || p.vec_ok) ? 1u : 0u;
    // --- inputs and immediates
    struct ValInfo { int slot = -1; int last_use = -1; bool is_output = false; };
    std::vector<Val> vals;            // values that live in slots
    std::vector<ValInfo> info;
    auto find_val = [&](Val v) {
      for (size_t i = 0; i < vals.size(); ++i)
        if (vals[i] == v) return (int)i;
      return -1;
    };
    auto in_members = [&](int32_t m) { return std::binary_search(members.begin(), members.end(), m); };
    std::vector<float> scal;
    std::vector<int> scal_src;   // scalar ordinal or -1 (immediate), with recip flag in scal_rec
    std::vector<char> scal_rec;
    auto scal_index = [&](double value, int ordinal, bool recip) -> int {
      for (size_t i = 0; i < scal.size(); ++i) {
        if (ordinal >= 0 && scal_src[i] == ordinal && scal_rec[i] == (char)recip) return (int)i;
        if (ordinal < 0 && scal_src[i] < 0 && scal[i] == (float)value && std::signbit(scal[i]) == std::signbit((float)value)) return (int)i;
      }
      scal.push_back((float)(recip ? 1.0 / value : value));
      scal_src.push_back(ordinal);
      scal_rec.push_back((char)recip);
      return (int)scal.size() - 1;
    };
    // inputs, in first-use order (operand order inside each member); a permute member reads
    // its operand through a private input with permuted strides
    std::vector<Val> input_vals;
    std::vector<int32_t> input_perm;   // permute member that owns the input, or -1
    for (int32_t m : members) {
      if (m == anchor.node) continue;
      for (Val v : rins[m]) {
        if (in_members(v.node) || is_imm(v) || v == anchor) continue;
        // a view op that this region materialises (a permutation, or an expand / reshape / narrow
        // that is itself a result) addresses its operand in its own way: through a private input
        const bool perm = nd[m]->op == LT_OP_PERMUTE || nd[m]->op == LT_OP_RESHAPE || nd[m]->op == LT_OP_NARROW;
        bool have = false;
        for (size_t q = 0; q < input_vals.size(); ++q) have |= (input_vals[q] == v && input_perm[q] < 0);
        if (perm || !have) {
          input_vals.push_back(v);
          input_perm.push_back(perm ? m : -1);
        }
      }
    }
    if ((int)input_vals.size() > ltk::kMaxIn) return bad(LT_ERR_UNSUPPORTED, "internal: region has too many inputs");
    p.n_in = (uint32_t)input_vals.size();
    std::vector<int> permute_input(N, -1);
    for (size_t k = 0; k < input_vals.size(); ++k) {
      Access acc;
      if (input_perm[k] >= 0) permute_input[input_perm[k]] = (int)k;
      if (!make_access(input_vals[k], space, input_perm[k], &acc)) return false;
      ltk::EwIn& in = p.in[k];
      in.ptr = nullptr;
      in.dtype = acc.dtype;
      // classify the access
      const std::vector<int64_t> cs = contiguous(space);
      bool full = true, zero = true, rowvec = !space.empty(), colvec = !space.empty();
      for (size_t d = 0; d < space.size(); ++d) {
        const int64_t want = space[d] == 1 ? 0 : cs[d];
        if (acc.stride[d] != want) full = false;
        if (acc.stride[d] != 0) zero = false;
        if (d + 1 < space.size()) {
          if (acc.stride[d] != 0) rowvec = false;
          const int64_t lead = space[d] == 1 ? 0 : cs[d] / std::max<int64_t>(space.back(), 1);
          if (acc.stride[d] != lead) colvec = false;
        } else {
          if (acc.stride[d] != (space[d] == 1 ? 0 : 1)) rowvec = false;
          if (acc.stride[d] != 0) colvec = false;
        }
      }
      if (n <= 1 || zero) in.mode = ltk::kScalar;
      else if (full) in.mode = ltk::kFull;
      else if (rowvec) in.mode = ltk::kRowVec;
      else if (colvec) in.mode = ltk::kColVec;
      else {
        if (space.size() > 4) return bad(LT_ERR_UNSUPPORTED, "strided operand in an iteration space of rank > 4");
        in.mode = ltk::kStrided;
        const int off = 4 - (int)space.size();
        for (int d = 0; d < 4; ++d) {
          p.dims[d] = d < off ? 1u : (uint32_t)space[d - off];
          in.stride[d] = d < off ? 0 : acc.stride[d - off];
        }
      }
      // (a window that starts off a 16-byte boundary is read element by element)
      const bool aligned = (acc.offset * (int64_t)dtype_size(acc.dtype)) % 16 == 0;
      in.fetch = ltk::kFetchSlow;
      if (in.mode == ltk::kScalar) in.fetch = ltk::kFetchBcast;
      else if (in.mode == ltk::kFull && p.full_vec_ok && aligned) in.fetch = ltk::kFetchVec4;
      else if (in.mode == ltk::kRowVec && p.vec_ok && aligned) in.fetch = ltk::kFetchVec4;
      else if (in.mode == ltk::kColVec && p.vec_ok) in.fetch = ltk::kFetchBcast;
      if (in.mode == ltk::kRowVec || in.mode == ltk::kColVec) p.needs_divmod = 1;
      if (in.mode != ltk::kStrided && space.size() <= 4) {
        const int off = 4 - (int)space.size();
        for (int d = 0; d < 4; ++d) p.dims[d] = d < off ? 1u : (uint32_t)space[d - off];
      }
      pb->in_storage.push_back({(uint32_t)k, acc.storage, acc.offset * (int64_t)dtype_size(acc.dtype)});
      // algorithmic bytes: the un-broadcast operand is read once
      int64_t elems = 1;
      for (size_t d = 0; d < space.size(); ++d)
        if (acc.stride[d] != 0) elems *= space[d];
      pb->bytes += (uint64_t)elems * dtype_size(acc.dtype);
      if (input_perm[k] < 0) {
        vals.push_back(input_vals[k]);
        info.push_back(ValInfo{(int)k, -1, false});
      }
    }
    for (size_t d = 0; d < 4; ++d)
      if (p.dims[d] == 0) p.dims[d] = 1;
    // --- liveness: last use of every value, by member position
    if (anchor.node >= 0) {
      vals.push_back(anchor);
      info.push_back(ValInfo{-1, -1, false});
    }
    for (size_t pos = 0; pos < members.size(); ++pos) {
      const int32_t m = members[pos];
      if (m == anchor.node) continue;
      for (Val v : rins[m]) {
        const int vi = find_val(v);
        if (vi >= 0) info[vi].last_use = (int)pos;
      }
      const int n_out = 1;
      for (int s = 0; s < n_out; ++s) {
        vals.push_back(Val{m, s});
        info.push_back(ValInfo{-1, -1, false});
      }
    }
    for (Val o : outputs) {
      const int vi = find_val(o);
      if (vi < 0) return bad(LT_ERR_UNSUPPORTED, "internal: region output is not computed by the region");
      info[vi].is_output = true;
    }
    // --- slot allocation (inputs sit in slots 0 .. n_in-1 when the program starts)
    std::vector<char> slot_used(ltk::kSlots, 0);
    for (uint32_t k = 0; k < p.n_in; ++k) slot_used[k] = 1;
    int max_slot = (int)p.n_in;
    auto take_slot = [&]() {
      for (int s = 0; s < ltk::kSlots; ++s)
        if (!slot_used[s]) {
          slot_used[s] = 1;
          max_slot = std::max(max_slot, s + 1);
          return s;
        }
      return -1;
    };
    // permuted private inputs hold their slot until their permute member has copied them
    if (anchor.node >= 0) {
      const int s = take_slot();
      if (s < 0) return bad(LT_ERR_UNSUPPORTED, "region needs more than 32 value slots");
      info[find_val(anchor)].slot = s;
      p.anchor_slot = (uint32_t)s;
    }
    auto operand = [&](Val v, bool recip, uint32_t* enc) -> bool {
      const Node* n = nd[v.node];
      if (is_imm(v)) {
        Val b = v;
        while (nd[b.node]->op == LT_OP_EXPAND || nd[b.node]->op == LT_OP_RESHAPE) b = rins[b.node][0];
        int idx;
        if (nd[b.node]->op == OP_CONSTANT) {
          const double c = nd[b.node]->attrs[0].is_float ? nd[b.node]->attrs[0].v.f : (double)nd[b.node]->attrs[0].v.i;
          idx = scal_index(c, -1, recip);
        } else {
          idx = scal_index(nd[b.node]->value, scalar_ordinal[b.node], recip);
        }
        if (idx >= ltk::kMaxScal) return bad(LT_ERR_UNSUPPORTED, "region uses more than 32 distinct scalars");
        *enc = 32u + (uint32_t)idx;
        return true;
      }
      (void)n;
      const int vi = find_val(v);
      if (vi < 0 || info[vi].slot < 0) return bad(LT_ERR_UNSUPPORTED, "internal: operand value has no slot");
      *enc = (uint32_t)info[vi].slot;
      return true;
    };
    uint32_t n_code = 0;
    auto emit = [&](uint32_t op, uint32_t dst, uint32_t a, uint32_t b = 0, uint32_t c = 0) -> bool {
      if (n_code >= (uint32_t)ltk::kMaxCode) return bad(LT_ERR_UNSUPPORTED, "region program exceeds 48 instructions");
      p.code[n_code++] = ltk::encode(op, dst, a, b, c);
      return true;
    };
    for (size_t pos = 0; pos < members.size(); ++pos) {
      const int32_t m = members[pos];
      if (m == anchor.node) continue;
      const Node* n = nd[m];
      const auto& o = rins[m];
      if (n->dtype != LT_F32 && n->dtype != LT_BF16) return bad(LT_ERR_UNSUPPORTED, "integer elementwise arithmetic has no lowering");
      uint32_t enc[3] = {0, 0, 0};
      const bool private_in = permute_input[m] >= 0;
      if (private_in) {
        enc[0] = (uint32_t)permute_input[m];
      } else {
        const bool recip_b = n->op == LT_OP_DIV && nd[o[1].node]->op == OP_SCALAR_PARAM;
        for (size_t q = 0; q < o.size(); ++q)
          if (!operand(o[q], q == 1 && recip_b, &enc[q])) return false;
      }
      // operands whose last use is this member free their slots before the result is placed
      for (Val v : o) {
        const int vi = find_val(v);
        if (vi >= 0 && info[vi].last_use == (int)pos && !info[vi].is_output && info[vi].slot >= 0) {
          slot_used[info[vi].slot] = 0;
        }
      }
      if (private_in) slot_used[permute_input[m]] = 0;
      const int dst = take_slot();
      if (dst < 0) return bad(LT_ERR_UNSUPPORTED, "region needs more than 32 value slots");
      info[find_val(Val{m, 0})].slot = dst;
      uint32_t op, rop = ltk::kNumOps;     // rop: the form with operands a and b exchanged
      switch (n->op) {
        case LT_OP_NEG: op = ltk::kNeg; break;
        case LT_OP_ABS: op = ltk::kAbs; break;
        case LT_OP_EXP: op = ltk::kExp; break;
        case LT_OP_LOG: op = ltk::kLog; break;
        case LT_OP_TANH: op = ltk::kTanh; break;
        case LT_OP_SQRT: op = ltk::kSqrt; break;
        case LT_OP_RSQRT: op = ltk::kRsqrt; break;
        case LT_OP_RECIP: op = ltk::kRecip; break;
        case LT_OP_RELU: op = ltk::kRelu; break;
        case LT_OP_GELU: op = ltk::kGelu; break;
        case LT_OP_SQUARE: op = ltk::kSquare; break;
        case LT_OP_SIGMOID: op = ltk::kSigmoid; break;
        case LT_OP_CAST: op = n->dtype == LT_BF16 ? ltk::kRoundBf16 : ltk::kMov; break;
        case LT_OP_EXPAND: case LT_OP_RESHAPE: case LT_OP_PERMUTE: case LT_OP_NARROW: op = ltk::kMov; break;
        case LT_OP_ADD: op = o.size() == 3 ? ltk::kFma : ltk::kAdd; rop = ltk::kAdd; break;
        case LT_OP_SUB: op = ltk::kSub; rop = ltk::kRsub; break;
        case LT_OP_MUL: op = rop = ltk::kMul; break;
        case LT_OP_DIV:
          if (nd[o[1].node]->op == OP_SCALAR_PARAM) op = rop = ltk::kMul;   // times the reciprocal
          else { op = ltk::kDiv; rop = ltk::kRdiv; }
          break;
        case LT_OP_MAXIMUM: op = rop = ltk::kMax; break;
        case LT_OP_MINIMUM: op = rop = ltk::kMin; break;
        case LT_OP_RELU_GRAD: op = ltk::kReluGrad; rop = ltk::kRreluGrad; break;
        case LT_OP_GELU_GRAD: op = ltk::kGeluGrad; rop = ltk::kRgeluGrad; break;
        default: return bad(LT_ERR_UNSUPPORTED, "opcode cannot be a member of an elementwise program");
      }
      // operand a of an instruction must be a slot: a scalar there is exchanged with b when b
      // is a slot, else copied into the destination slot first
      auto splat_into_dst = [&](uint32_t scalar_enc) { return emit(ltk::kSplat, (uint32_t)dst, 0, scalar_enc); };
      bool okk;
      if (op == ltk::kFma) {
        // a + alpha*b  ->  fma(x = b, y = alpha, z = a); x must be a slot
        uint32_t x = enc[1], y = enc[2], z = enc[0];
        if (x >= 32u && y < 32u) std::swap(x, y);
        if (x >= 32u) {
          if (!splat_into_dst(x)) return false;
          x = (uint32_t)dst;
        }
        okk = emit(op, (uint32_t)dst, x, y, z);
      } else if (op >= ltk::kAdd) {
        uint32_t a = enc[0], b = enc[1];
        if (a >= 32u && b < 32u) {
          std::swap(a, b);
          op = rop;
        } else if (a >= 32u) {
          if (!splat_into_dst(a)) return false;
          a = (uint32_t)dst;
        }
        okk = emit(op, (uint32_t)dst, a, b);
      } else {
        uint32_t a = enc[0];
        if (a >= 32u) {
          if (!splat_into_dst(a)) return false;
          a = (uint32_t)dst;
        }
        okk = emit(op, (uint32_t)dst, a);
      }
      if (!okk) return false;
    }
    p.n_code = n_code;
    p.n_slots = (uint32_t)max_slot;
    for (size_t i = 0; i < scal.size(); ++i) {
      p.scal[i] = scal[i];
      if (scal_src[i] >= 0) pb->scal_patch.push_back({(uint32_t)i, scal_src[i], (bool)scal_rec[i]});
    }
    // --- outputs
    if ((int)outputs.size() > ltk::kMaxOut) return bad(LT_ERR_UNSUPPORTED, "internal: region has too many outputs");
    p.n_out = (uint32_t)outputs.size();
    for (size_t k = 0; k < outputs.size(); ++k) {
      const Val v = outputs[k];
      ltk::EwOut& out = p.out[k];
      out.ptr = nullptr;
      out.dtype = out_dtype(v);
      out.slot = (uint32_t)info[find_val(v)].slot;
      const int64_t on = count(out_shape(v));
      out.scalar = (on == 1 && n > 1) ? 1u : 0u;
      if (on != n && on != 1) return bad(LT_ERR_UNSUPPORTED, "internal: output shape differs from its iteration space");
      pb->out_storage.push_back({(uint32_t)k, storage_of[v.node][v.slot]});
      pb->bytes += (uint64_t)on * dtype_size(out.dtype);
    }
    finish_flags(&p);
    return true;
  }

  // Flags for the kernels' fast variants: whole 4-vectors only (n % 4 == 0, no element-wise
  // input), and "everything is fp32".
  static void finish_flags(ltk::EwProg* q) {
    bool fast = (q->n % 4u) == 0u, f32 = true;
    for (uint32_t i = 0; i < q->n_in; ++i) {
      fast = fast && q->in[i].fetch != ltk::kFetchSlow;
      f32 = f32 && q->in[i].dtype == ltk::kF32;
    }
    for (uint32_t i = 0; i < q->n_out; ++i) {
      f32 = f32 && q->out[i].dtype == ltk::kF32;
      fast = fast && (q->out[i].scalar || q->full_vec_ok);
    }
    q->fast = fast ? 1u : 0u;
    q->all_f32 = f32 ? 1u : 0u;
  }

  // append one program's patches to the plan; `offset` = byte offset of the EwProg inside the args
  void add_prog_patches(uint32_t launch, size_t offset, const ProgBuild& pb) {
    for (auto& is : pb.in_storage)
      plan->ptr_patches.push_back(PtrPatch{launch, (uint32_t)(offset + offsetof(ltk::EwProg, in) + is.first * sizeof(ltk::EwIn) + offsetof(ltk::EwIn, ptr)), is.second, is.byte_offset});
    for (auto& os : pb.out_storage)
      plan->ptr_patches.push_back(PtrPatch{launch, (uint32_t)(offset + offsetof(ltk::EwProg, out) + os.first * sizeof(ltk::EwOut) + offsetof(ltk::EwOut, ptr)), os.second, 0, 1});
    for (auto& sp : pb.scal_patch)
      plan->scal_patches.push_back(ScalPatch{launch, (uint32_t)(offset + offsetof(ltk::EwProg, scal) + sp.index * sizeof(float)), sp.scalar, (uint8_t)(sp.recip ? 1 : 0)});
  }

  void touch(int32_t storage, int launch) {
    if (storage < 0) return;
    Storage& s = plan->storages[storage];
    if (s.first_launch < 0) s.first_launch = launch;
    s.last_launch = launch;
  }

  template <class T>
  Launch make_launch(LaunchKind kind, int region, const T& args) {
    Launch l;
    l.kind = kind;
    l.region = region;
    l.args.resize(sizeof(T));
    std::memcpy(l.args.data(), &args, sizeof(T));
    return l;
  }

  static uint32_t ew_grid(uint64_t n) {
    const uint64_t tiles = (n + 1023) / 1024;
    return (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>(tiles, 256 * 32));
  }

  // A contraction operand seen through its views: strides of the two matrix dimensions and of the
  // (non-unit) leading dimensions.
  struct MatView {
    int32_t storage;
    uint8_t dtype;
    int64_t rows, cols, s_row, s_col, byte_offset;
    std::vector<int64_t> lead, s_lead;
  };

  bool operand_gemm(Val v, bool trans, MatView* mv) {
    Pattern pat;
    if (!pattern_of(v, &pat)) return false;
    const std::vector<int64_t>&shape = pat.shape, &stride = pat.stride;
    mv->storage = pat.storage;
    mv->dtype = out_dtype(base(v));
    mv->byte_offset = pat.offset * (int64_t)dtype_size(mv->dtype);
    const size_t r = shape.size();
    mv->rows = trans ? shape[r - 1] : shape[r - 2];
    mv->cols = trans ? shape[r - 2] : shape[r - 1];
    mv->s_row = trans ? stride[r - 1] : stride[r - 2];
    mv->s_col = trans ? stride[r - 2] : stride[r - 1];
    if (mv->rows == 1) mv->s_row = mv->s_col == 1 ? mv->cols : 1;   // any stride serves a single row / column
    if (mv->cols == 1) mv->s_col = mv->s_row == 1 ? mv->rows : 1;
    mv->lead.clear();
    mv->s_lead.clear();
    for (size_t d = 0; d + 2 < r; ++d)
      if (shape[d] != 1) {
        mv->lead.push_back(shape[d]);
        mv->s_lead.push_back(stride[d]);
      }
    return true;
  }

  bool codegen() {
    storage_of.assign(N, {});
    param_ordinal.assign(N, -1);
    scalar_ordinal.assign(N, -1);
    for (size_t k = 0; k < cut.param_nodes.size(); ++k) param_ordinal[cut.index_of[cut.param_nodes[k]]] = (int32_t)k;
    for (size_t k = 0; k < cut.scalar_nodes.size(); ++k) scalar_ordinal[cut.index_of[cut.scalar_nodes[k]]] = (int32_t)k;
    plan->n_params = (int)cut.param_nodes.size();
    plan->n_scalars = (int)cut.scalar_nodes.size();
    // storages: every live device parameter, then every region output
    for (int32_t i = 0; i < N; ++i) {
      storage_of[i].assign(nd[i]->op == LT_OP_LAYER_NORM ? 3 : 1, -1);
      if (live[i] && nd[i]->op == OP_DEVICE_DATA) {
        Storage s;
        s.param = param_ordinal[i];
        s.first_launch = s.last_launch = 0;
        plan->storages.push_back(s);
        storage_of[i][0] = (int32_t)plan->storages.size() - 1;
      }
    }
    for (size_t k = 0; k < ordered.size(); ++k) {
      std::vector<Val> in, out;
      region_io(ordered[k]->members, &in, &out);
      const auto& ips = inplace_of_region[region_pos(ordered[k])];
      for (Val v : out) {
        Storage s;
        s.first_launch = -1;
        for (const InPlace& ip : ips)
          if (ip.v == v) s.param = (int)ip.param;
        if (s.param < 0) s.bytes = (size_t)count(out_shape(v)) * dtype_size(out_dtype(v));
        else s.first_launch = s.last_launch = 0;
        plan->storages.push_back(s);
        storage_of[v.node][v.slot] = (int32_t)plan->storages.size() - 1;
      }
    }
    // roots
    for (size_t r = 0; r < root_vals.size(); ++r) {
      const Val v = root_vals[r];
      RootBind rb;
      const Node* n = nd[v.node];
      if (n->op == OP_DEVICE_DATA) {
        rb.kind = RootBind::PARAM_ALIAS;
        rb.index = param_ordinal[v.node];
      } else if (n->op == OP_SCALAR_PARAM) {
        rb.kind = RootBind::SCALAR;
        rb.index = scalar_ordinal[v.node];
      } else if (n->op == OP_CONSTANT) {
        rb.kind = RootBind::CONST;
        rb.value = n->attrs[0].is_float ? n->attrs[0].v.f : (double)n->attrs[0].v.i;
      } else {
        rb.kind = RootBind::STORAGE;
        rb.index = storage_of[v.node][v.slot];
        if (rb.index < 0) return bad(LT_ERR_UNSUPPORTED, "internal: root has no storage");
        plan->storages[rb.index].bound_to_root = true;
      }
      plan->roots.push_back(rb);
    }
    // launches
    for (size_t k = 0; k < ordered.size(); ++k) {
      if (!emit_region((int)k, ordered[k])) return false;
    }
    for (Storage& s : plan->storages)
      if (s.first_launch < 0) s.first_launch = s.last_launch = 0;
    plan->n_regions = (int)ordered.size();
    for (const Launch& l : plan->launches) {
      plan->bytes_planned += l.bytes;
      plan->flops_planned += l.flops;
    }
    return true;
  }

  void note_prog_storages(const ProgBuild& pb, int launch) {
    for (auto& is : pb.in_storage) touch(is.second, launch);
    for (auto& os : pb.out_storage) touch(os.second, launch);
  }

  bool emit_region(int k, Region* r) {
    std::vector<Val> in, out;
    region_io(r->members, &in, &out);
    const int launch = (int)plan->launches.size();
    if (r->kind == C_EW) {
      ProgBuild pb;
      if (!build_prog(r->members, shape_of(r->members.front()), Val{-1, 0}, out, true, &pb)) return false;
      ltk::EwArgs a{};
      a.prog = pb.prog;
      Launch l = make_launch(L_EW, k, a);
      l.grid_x = ew_grid(pb.prog.n);
      l.bytes = pb.bytes;
      plan->launches.push_back(std::move(l));
      add_prog_patches(launch, offsetof(ltk::EwArgs, prog), pb);
      note_prog_storages(pb, launch);
      return true;
    }
    const int32_t a = r->anchor;
    const Node* an = nd[a];
    // split members: the prologue is what the anchor depends on, everything else runs after it
    std::vector<char> feeds(N, 0);
    {
      std::vector<int32_t> stack{a};
      while (!stack.empty()) {
        const int32_t x = stack.back();
        stack.pop_back();
        for (Val v : rins[x])
          if (r->has(v.node) && !feeds[v.node]) {
            feeds[v.node] = 1;
            stack.push_back(v.node);
          }
      }
    }
    std::vector<int32_t> pro_m, post_m;
    for (int32_t m : r->members) {
      if (m == a) continue;
      if (feeds[m]) pro_m.push_back(m);
      else post_m.push_back(m);
    }
    if (r->kind == C_MM) return emit_gemm(k, r, post_m, out);
    if (r->kind == C_SLICE) return emit_slice(k, r);
    if (!plain_reduce(an->op)) return emit_row_op(k, r, out);
    // ---- plain reduction
    const Val src = rins[a][0];
    const std::vector<int64_t> in_shape = out_shape(src);
    // prologue program: members below the anchor plus a final value = the reduced operand
    ProgBuild pro;
    {
      if (!build_prologue(pro_m, in_shape, src, r->kind == C_ALL, &pro)) return false;
    }
    std::vector<int64_t> post_space = shape_of(a);
    if (r->has_fin) post_space = r->fin_shape;
    ProgBuild post;
    std::vector<int32_t> post_members = post_m;
    post_members.push_back(a);
    // canonical (= topological) order; a member that only the epilogue reads may well have been
    // numbered before the anchor (x - 0.5 * v: the operands are numbered last to first)
    std::sort(post_members.begin(), post_members.end());
    if (!build_prog(post_members, post_space, Val{a, 0}, out, r->kind == C_ALL, &post)) return false;
    const uint32_t red = an->op == LT_OP_SUM ? ltk::kRedSum : an->op == LT_OP_AMAX ? ltk::kRedMax : ltk::kRedMean;
    if (r->kind == C_ROW) {
      ltk::RowArgs args{};
      args.pro = pro.prog;
      args.post = post.prog;
      args.cols = (uint32_t)in_shape.back();
      args.rows = (uint32_t)(count(in_shape) / std::max<int64_t>(1, in_shape.back()));
      args.red = red;
      args.threads_per_row = args.cols >= 512 ? 256u : 64u;
      Launch l = make_launch(L_ROW, k, args);
      const uint32_t rpb = 256u / args.threads_per_row;
      l.grid_x = std::max<uint32_t>(1, std::min<uint32_t>((args.rows + rpb - 1) / rpb, 256 * 16));
      l.bytes = pro.bytes + post.bytes;
      plan->launches.push_back(std::move(l));
      add_prog_patches(launch, offsetof(ltk::RowArgs, pro), pro);
      add_prog_patches(launch, offsetof(ltk::RowArgs, post), post);
    } else if (r->kind == C_ALL) {
      ltk::AllArgs args{};
      args.pro = pro.prog;
      args.post = post.prog;
      args.red = red;
      args.count = (uint64_t)count(in_shape);
      Launch l = make_launch(L_ALL, k, args);
      l.grid_x = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>((args.count + 4095) / 4096, 256 * 2));
      l.bytes = pro.bytes + post.bytes;
      plan->launches.push_back(std::move(l));
      add_prog_patches(launch, offsetof(ltk::AllArgs, pro), pro);
      add_prog_patches(launch, offsetof(ltk::AllArgs, post), post);
    } else {
      if (in_shape.size() != 2) return bad(LT_ERR_UNSUPPORTED, "axis-0 reduction needs a rank-2 operand (reshape first)");
      if (ride_with_contraction(r, red, in_shape, pro, post)) return true;
      ltk::ColArgs args{};
      args.pro = pro.prog;
      args.post = post.prog;
      args.rows = (uint32_t)in_shape[0];
      args.cols = (uint32_t)in_shape[1];
      args.red = red;
      Launch l = make_launch(L_COL, k, args);
      l.grid_x = (args.cols + 255) / 256;
      if (l.grid_x > kTickets) return bad(LT_ERR_UNSUPPORTED, "axis-0 reduction wider than 262144 columns");
      // a slab of 64 rows gives each of a workgroup's 8 waves one 8-row trip
      uint32_t gy = std::max<uint32_t>(1, std::min<uint32_t>(args.rows / 64, 64));
      // small: one slab per strip and no cross-workgroup step -- unless the rows are not whole
      // 4-vectors, where the element-wise path is slow enough to want the rows spread out
      if ((uint64_t)args.rows * args.cols <= 65536) gy = (args.cols % 4u) == 0u ? 1u : std::max<uint32_t>(1, std::min<uint32_t>(args.rows / 8, 32));
      while (gy > 1 && (uint64_t)gy * (args.cols + 3) > kPartialFloats) gy /= 2;
      if ((uint64_t)gy * (args.cols + 3) > kPartialFloats) return bad(LT_ERR_UNSUPPORTED, "axis-0 reduction wider than 1048576 columns");
      while (gy > 1 && (uint64_t)gy * l.grid_x > 256) gy /= 2;
      l.grid_y = gy;
      l.bytes = pro.bytes + post.bytes;
      plan->launches.push_back(std::move(l));
      add_prog_patches(launch, offsetof(ltk::ColArgs, pro), pro);
      add_prog_patches(launch, offsetof(ltk::ColArgs, post), post);
    }
    note_prog_storages(pro, launch);
    note_prog_storages(post, launch);
    return true;
  }

  // A bias gradient next to its weight gradient: dW = x^T dy and db = sum over the rows of dy read
  // the same dy, and the small one-launch contraction fetches every column of its B operand anyway.
  // When the launch emitted just before this column sum is such a contraction with this sum's
  // operand as its B ([k, n], rows contiguous, fp32, no prologue), the sum and its post program
  // ride along in that launch (GemmArgs::col_sum) and this region gets no launch of its own.
  // Nothing the column program writes may be touched by the contraction, and nothing it reads
  // may be written by it.
  bool ride_with_contraction(const Region* r, uint32_t red, const std::vector<int64_t>& in_shape, const ProgBuild& pro, const ProgBuild& post) {
    if (plan->launches.empty() || r->has_fin || (red != ltk::kRedSum && red != ltk::kRedMean)) return false;
    const uint32_t prev = (uint32_t)plan->launches.size() - 1;
    Launch& pl = plan->launches[prev];
    if (pl.kind != L_GEMM || pl.args.size() != sizeof(ltk::GemmArgs)) return false;
    ltk::GemmArgs* ga = (ltk::GemmArgs*)pl.args.data();
    if (!ga->direct || ga->tile_m != 32u || ga->tile_n != 32u || ga->splits != 1u || ga->col_sum || ga->batch0 * ga->batch1 != 1u || ga->in_dtype != ltk::kF32) return false;
    if (ga->k != (uint32_t)in_shape[0] || ga->n != (uint32_t)in_shape[1] || ga->b.s_col != 1 || ga->b.s_row != in_shape[1]) return false;
    if (pro.prog.n_code != 0u || pro.prog.n_in != 1u || pro.in_storage.size() != 1 || pro.prog.in[0].mode != ltk::kFull ||
        pro.prog.in[0].dtype != ltk::kF32 || !pro.scal_patch.empty() || post.prog.n_slots > 16u)
      return false;
    // the contraction's B operand is this sum's operand; collect what the contraction reads and writes
    const uint32_t b_off = (uint32_t)(offsetof(ltk::GemmArgs, b) + offsetof(ltk::GemmOperand, ptr));
    bool same_b = false;
    // (a donated output and the parameter it overwrites are two storages of one buffer: compare buffers)
    auto buffer_of = [&](int32_t st) -> int64_t {
      if (st < 0) return INT64_MIN;
      return plan->storages[st].param >= 0 ? -(int64_t)plan->storages[st].param - 1 : (int64_t)st;
    };
    std::vector<int64_t> reads, writes;
    for (const PtrPatch& pp : plan->ptr_patches) {
      if (pp.launch != prev) continue;
      if (pp.offset == b_off) same_b = pp.storage == pro.in_storage[0].second && pp.byte_offset == pro.in_storage[0].byte_offset;
      (pp.write ? writes : reads).push_back(buffer_of(pp.storage));
    }
    if (!same_b) return false;
    auto among = [](const std::vector<int64_t>& v, int64_t x) { return std::find(v.begin(), v.end(), x) != v.end(); };
    for (auto& is : post.in_storage)
      if (among(writes, buffer_of(is.second))) return false;
    for (auto& os : post.out_storage)
      if (among(writes, buffer_of(os.second)) || among(reads, buffer_of(os.second))) return false;
    ga->col_sum = 1u;
    ga->col_red = red;
    ga->col_post = post.prog;
    pl.bytes += post.bytes;
    add_prog_patches(prev, offsetof(ltk::GemmArgs, col_post), post);
    note_prog_storages(pro, (int)prev);
    note_prog_storages(post, (int)prev);
    return true;
  }

  // Prologue of a reduction: the members below the anchor, producing `src` in slot anchor_slot.
  // When `src` is not computed by a member it is simply the program's only input.
  bool build_prologue(const std::vector<int32_t>& members, const std::vector<int64_t>& space, Val src, bool full_vec,
                      ProgBuild* pb) {
    const bool computed = std::binary_search(members.begin(), members.end(), src.node);
    if (computed) {
      // treat src as an "output" so that its slot stays live; it is not stored
      std::vector<Val> outs{src};
      storage_of[src.node][src.slot] = -2;   // placeholder, removed below
      if (!build_prog(members, space, Val{-1, 0}, outs, full_vec, pb)) return false;
      storage_of[src.node][src.slot] = -1;
      pb->prog.anchor_slot = pb->prog.out[0].slot;
      pb->prog.n_out = 0;
      finish_flags(&pb->prog);
      pb->out_storage.clear();
      pb->bytes -= (uint64_t)count(space) * dtype_size(out_dtype(src));
      return true;
    }
    // identity prologue: load src into slot 0
    ltk::EwProg& p = pb->prog;
    p = ltk::EwProg{};
    Access acc;
    if (!make_access(src, space, -1, &acc)) return false;
    if (acc.offset != 0) return bad(LT_ERR_UNSUPPORTED, "reduction of a window has no lowering");
    // reuse build_prog's classification by building a one-member copy program is overkill:
    // a reduction operand that is not computed in the region is always read in full
    const std::vector<int64_t> cs = contiguous(space);
    bool full = true;
    for (size_t d = 0; d < space.size(); ++d)
      if (acc.stride[d] != (space[d] == 1 ? 0 : cs[d])) full = false;
    if (!full) return bad(LT_ERR_UNSUPPORTED, "reduction of a broadcast view has no lowering");
    p.n = (uint64_t)count(space);
    p.cols = (uint32_t)(space.empty() ? 1 : std::max<int64_t>(space.back(), 1));
    p.vec_ok = (p.cols % 4u == 0u) ? 1u : 0u;
    p.full_vec_ok = (full_vec || p.vec_ok) ? 1u : 0u;
    p.n_in = 1;
    p.in[0].mode = p.n <= 1 ? ltk::kScalar : ltk::kFull;
    p.in[0].dtype = acc.dtype;
    p.in[0].fetch = p.n <= 1 ? ltk::kFetchBcast : (p.full_vec_ok ? ltk::kFetchVec4 : ltk::kFetchSlow);
    p.anchor_slot = 0;
    p.n_slots = 1;
    for (int d = 0; d < 4; ++d) p.dims[d] = 1;
    pb->in_storage.push_back({0u, acc.storage, acc.offset * (int64_t)dtype_size(acc.dtype)});
    pb->bytes += p.n * dtype_size(acc.dtype);
    finish_flags(&p);
    return true;
  }

  // Window update: base and update must be dense in memory; written in place when the result
  // replaces the base's own (donated) buffer.
  bool emit_slice(int k, Region* r) {
    const int32_t a = r->anchor;
    const Node* an = nd[a];
    if (r->members.size() != 1) return bad(LT_ERR_UNSUPPORTED, "internal: window update with fused members");
    const int launch = (int)plan->launches.size();
    int64_t axis = 0, start = 0;
    for (int i = 0; i < an->n_attr; ++i) {
      if (an->attrs[i].key == LT_ATTR_AXIS) axis = an->attrs[i].v.i;
      if (an->attrs[i].key == LT_ATTR_START) start = an->attrs[i].v.i;
    }
    const std::vector<int64_t> bs = shape_of(a), us = out_shape(rins[a][1]);
    Access ab, au;
    if (!make_access(rins[a][0], bs, -1, &ab) || !make_access(rins[a][1], us, -1, &au)) return false;
    auto dense = [&](const Access& acc, const std::vector<int64_t>& shp) {
      const std::vector<int64_t> cs = contiguous(shp);
      for (size_t d = 0; d < shp.size(); ++d)
        if (shp[d] != 1 && acc.stride[d] != cs[d]) return false;
      return true;
    };
    if (!dense(ab, bs) || !dense(au, us)) return bad(LT_ERR_UNSUPPORTED, "window update of a strided or broadcast operand has no lowering");
    const int32_t so = storage_of[a][0];
    if (so < 0) return bad(LT_ERR_UNSUPPORTED, "internal: window update without storage");
    const bool in_place = plan->storages[so].param >= 0 && plan->storages[ab.storage].param == plan->storages[so].param && ab.offset == 0;
    ltk::SliceArgs args{};
    uint64_t outer = 1, inner = 1;
    for (int64_t d = 0; d < axis; ++d) outer *= (uint64_t)bs[d];
    for (size_t d = (size_t)axis + 1; d < bs.size(); ++d) inner *= (uint64_t)bs[d];
    args.dim = (uint64_t)bs[axis];
    args.inner = inner;
    args.start = (uint64_t)start;
    args.len = (uint64_t)us[axis];
    args.elem_bytes = (uint32_t)dtype_size(an->dtype);
    args.window_only = in_place ? 1u : 0u;
    args.n = in_place ? outer * args.len * inner : outer * args.dim * inner;
    Launch l = make_launch(L_SLICE, k, args);
    l.grid_x = (uint32_t)std::max<uint64_t>(1, std::min<uint64_t>((args.n + 255) / 256, 256 * 64));
    const uint64_t win_bytes = outer * args.len * inner * args.elem_bytes, all_bytes = outer * args.dim * inner * args.elem_bytes;
    l.bytes = in_place ? 2 * win_bytes : 2 * all_bytes;
    plan->launches.push_back(std::move(l));
    if (!in_place) {
      plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)offsetof(ltk::SliceArgs, base), ab.storage, ab.offset * (int64_t)args.elem_bytes});
      touch(ab.storage, launch);
    }
    plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)offsetof(ltk::SliceArgs, upd), au.storage, au.offset * (int64_t)args.elem_bytes});
    plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)offsetof(ltk::SliceArgs, out), so, 0, 1});
    touch(au.storage, launch);
    touch(so, launch);
    return true;
  }

  bool emit_row_op(int k, Region* r, const std::vector<Val>& out) {
    const int32_t a = r->anchor;
    const Node* an = nd[a];
    if (r->members.size() != 1) return bad(LT_ERR_UNSUPPORTED, "internal: fixed row operator with fused members");
    const int launch = (int)plan->launches.size();
    ltk::RowOpArgs args{};
    const std::vector<int64_t> xs = out_shape(rins[a][an->op == LT_OP_LAYER_NORM_GRAD ? 1 : 0]);
    args.cols = (uint32_t)xs.back();
    args.rows = (uint32_t)(count(xs) / std::max<int64_t>(1, xs.back()));
    args.threads_per_row = args.cols > 1024 ? 256u : args.cols > 256 ? 64u : 16u;   // a lane holds up to 16 columns
    if (args.cols > args.threads_per_row * 16u) return bad(LT_ERR_UNSUPPORTED, "row operator on rows longer than 4096 elements");
    switch (an->op) {
      case LT_OP_SOFTMAX: args.op = ltk::kSoftmax; break;
      case LT_OP_SOFTMAX_GRAD: args.op = ltk::kSoftmaxGrad; break;
      case LT_OP_LAYER_NORM: args.op = ltk::kLayerNorm; args.eps = (float)an->attrs[0].v.f; break;
      case LT_OP_LAYER_NORM_GRAD: args.op = ltk::kLayerNormGrad; break;
      case LT_OP_XENT: args.op = ltk::kXent; break;
      default: args.op = ltk::kXentGrad; break;
    }
    Launch l = make_launch(L_ROWOP, k, args);
    const uint32_t rpb = 256u / args.threads_per_row;
    l.grid_x = std::max<uint32_t>(1, std::min<uint32_t>((args.rows + rpb - 1) / rpb, 256 * 16));
    uint64_t bytes = 0;
    const size_t n_arr = an->op == LT_OP_XENT_GRAD ? 2 : rins[a].size();
    for (size_t i = 0; i < n_arr; ++i) {
      Access acc;
      const std::vector<int64_t> vs = out_shape(rins[a][i]);
      if (!make_access(rins[a][i], vs, -1, &acc)) return false;
      if (acc.offset != 0) return bad(LT_ERR_UNSUPPORTED, "row operator on a window has no lowering");
      if (acc.stride != contiguous(vs) && count(vs) > 1) {
        bool dense = true;
        const std::vector<int64_t> cs = contiguous(vs);
        for (size_t d = 0; d < vs.size(); ++d) dense &= (vs[d] == 1 || acc.stride[d] == cs[d]);
        if (!dense) return bad(LT_ERR_UNSUPPORTED, "row operator on a broadcast view has no lowering");
      }
      ((ltk::RowOpArgs*)l.args.data())->in_dtype[i] = acc.dtype;
      plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)(offsetof(ltk::RowOpArgs, in) + i * sizeof(void*)), acc.storage, 0});
      touch(acc.storage, launch);
      bytes += (uint64_t)count(vs) * dtype_size(acc.dtype);
    }
    if (an->op == LT_OP_XENT_GRAD) {
      // the scale is a rank-0 operand: an immediate or a dynamic scalar
      const Val s = rins[a][2];
      if (!is_imm(s)) return bad(LT_ERR_UNSUPPORTED, "xent_grad: scale must be a scalar constant or parameter");
      Val b = s;
      while (nd[b.node]->op == LT_OP_EXPAND || nd[b.node]->op == LT_OP_RESHAPE) b = rins[b.node][0];
      if (nd[b.node]->op == OP_CONSTANT) {
        ((ltk::RowOpArgs*)l.args.data())->scale = (float)(nd[b.node]->attrs[0].is_float ? nd[b.node]->attrs[0].v.f : (double)nd[b.node]->attrs[0].v.i);
      } else {
        plan->scal_patches.push_back(ScalPatch{(uint32_t)launch, (uint32_t)offsetof(ltk::RowOpArgs, scale), scalar_ordinal[b.node], 0});
      }
    }
    // outputs: every slot of the anchor that is needed; unneeded layer-norm statistics still
    // need somewhere to go, so they get storage as well
    const int n_out = an->op == LT_OP_LAYER_NORM ? 3 : 1;
    for (int s = 0; s < n_out; ++s) {
      int32_t st = storage_of[a][s];
      if (st < 0) {
        Storage ns;
        ns.first_launch = -1;
        ns.bytes = (size_t)count(out_shape(Val{a, s})) * dtype_size(out_dtype(Val{a, s}));
        plan->storages.push_back(ns);
        st = storage_of[a][s] = (int32_t)plan->storages.size() - 1;
      }
      ((ltk::RowOpArgs*)l.args.data())->out_dtype[s] = out_dtype(Val{a, s});
      plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)(offsetof(ltk::RowOpArgs, out) + s * sizeof(void*)), st, 0, 1});
      touch(st, launch);
      bytes += (uint64_t)count(out_shape(Val{a, s})) * dtype_size(out_dtype(Val{a, s}));
    }
    (void)out;
    l.bytes = bytes;
    plan->launches.push_back(std::move(l));
    return true;
  }

  bool emit_gemm(int k, Region* r, const std::vector<int32_t>& post_m_in, const std::vector<Val>& out_in) {
    const int32_t a = r->anchor;
    const Node* an = nd[a];
    const int launch = (int)plan->launches.size();
    bool tra = false, trb = false;
    for (int i = 0; i < an->n_attr; ++i) {
      if (an->attrs[i].key == LT_ATTR_TRANS_A) tra = an->attrs[i].v.i != 0;
      if (an->attrs[i].key == LT_ATTR_TRANS_B) trb = an->attrs[i].v.i != 0;
    }
    ltk::GemmArgs args{};
    MatView A, B;
    if (!operand_gemm(rins[a][0], tra, &A)) return false;
    if (!operand_gemm(rins[a][1], trb, &B)) return false;
    if (A.dtype != B.dtype) return bad(LT_ERR_UNSUPPORTED, "matmul of operands with different dtypes has no lowering");
    if ((A.s_row != 1 && A.s_col != 1) || (B.s_row != 1 && B.s_col != 1))
      return bad(LT_ERR_UNSUPPORTED, "matmul operand without a unit-stride matrix dimension");
    const std::vector<int64_t> os = shape_of(a);
    int64_t m = A.rows, n = B.cols;
    const int64_t kk = A.cols;
    std::vector<int64_t> lead = A.lead;
    if (B.lead.empty() && !A.lead.empty()) {
      // a plain matrix on the right: fold the (dense) leading axes of a into its rows
      if (tra) return bad(LT_ERR_UNSUPPORTED, "transposed batched a with an unbatched b has no lowering");
      int64_t expect = A.s_row * A.rows;
      for (int d = (int)A.lead.size() - 1; d >= 0; --d) {
        if (A.s_lead[d] != expect) return bad(LT_ERR_UNSUPPORTED, "matmul: leading axes of a are not dense over its rows");
        expect *= A.lead[d];
      }
      for (int64_t d : A.lead) m *= d;
      lead.clear();
      A.lead.clear();
      A.s_lead.clear();
    }
    if (lead.size() > 2) return bad(LT_ERR_UNSUPPORTED, "matmul with more than two batch axes has no lowering");
    if (B.lead != lead) return bad(LT_ERR_UNSUPPORTED, "matmul: batch axes of a and b differ after views");
    args.m = (uint32_t)m;
    args.n = (uint32_t)n;
    args.k = (uint32_t)kk;
    args.batch0 = lead.size() == 2 ? (uint32_t)lead[0] : lead.size() == 1 ? (uint32_t)lead[0] : 1u;
    args.batch1 = lead.size() == 2 ? (uint32_t)lead[1] : 1u;
    auto fill = [&](ltk::GemmOperand* g, const MatView& mv) {
      g->ptr = nullptr;
      g->s_row = mv.s_row;
      g->s_col = mv.s_col;
      g->s_b0 = mv.s_lead.size() >= 1 ? mv.s_lead[0] : 0;
      g->s_b1 = mv.s_lead.size() == 2 ? mv.s_lead[1] : 0;
    };
    fill(&args.a, A);
    fill(&args.b, B);
    args.in_dtype = A.dtype;
    const int64_t batch = (int64_t)args.batch0 * args.batch1;
    // output layout: contiguous [batch0, batch1, m, n] unless the region ends in a layout permute
    args.o_row = n;
    args.o_b1 = m * n;
    args.o_b0 = (int64_t)args.batch1 * m * n;
    std::vector<int32_t> post_m = post_m_in;
    std::vector<Val> out = out_in;
    if (r->sealed) {
      const int32_t pm = post_m.back();   // the permute member
      if (post_m.size() != 1 || nd[pm]->op != LT_OP_PERMUTE) return bad(LT_ERR_UNSUPPORTED, "internal: sealed region shape");
      // stride of anchor dimension d in the permuted, dense result
      const std::vector<int64_t> pshape = shape_of(pm), pcs = contiguous(pshape);
      std::vector<int64_t> sd(os.size(), 0);
      for (size_t j = 0; j < pshape.size(); ++j) sd[nd[pm]->attrs[j].v.i] = pcs[j];
      const size_t rr = os.size();
      if (sd[rr - 1] != 1) return bad(LT_ERR_UNSUPPORTED, "permuted matmul result must keep its last axis last");
      std::vector<int64_t> ol;
      for (size_t d = 0; d + 2 < rr; ++d)
        if (os[d] != 1) ol.push_back(sd[d]);
      if (ol.size() != lead.size()) return bad(LT_ERR_UNSUPPORTED, "permuted matmul result: batch axes do not match");
      args.o_row = sd[rr - 2];
      args.o_b0 = ol.size() >= 1 ? ol[0] : 0;
      args.o_b1 = ol.size() == 2 ? ol[1] : 0;
      // the region's output is the permute's value; the program only stores the accumulator
      storage_of[a][0] = storage_of[pm][0];
      post_m.clear();
      out.assign(1, Val{a, 0});
    }
    ProgBuild post;
    std::vector<int32_t> post_members = post_m;
    post_members.push_back(a);
    // canonical (= topological) order; a member that only the epilogue reads may well have been
    // numbered before the anchor (x - 0.5 * v: the operands are numbered last to first)
    std::sort(post_members.begin(), post_members.end());
    if (!build_prog(post_members, os, Val{a, 0}, out, false, &post)) return false;
    if (r->sealed) {
      storage_of[a][0] = -1;
      // quads are 16-byte aligned in the permuted layout only if every stride is a multiple of 4
      const bool al = (args.o_row % 4) == 0 && (args.o_b0 % 4) == 0 && (args.o_b1 % 4) == 0 && (n % 4) == 0;
      post.prog.vec_ok = post.prog.full_vec_ok = al ? 1u : 0u;
    }
    args.post = post.prog;
    args.splits = 1;
    int32_t ws_storage = -1;
    if (A.dtype == LT_BF16) {
      // the bf16 kernel works on 128 x 128 tiles; few tiles and a long k: split k so that about
      // two workgroups per compute unit exist, each keeping at least four 64-wide slices
      const uint32_t bm = 128u;
      const uint32_t bn = n <= 64 ? 64u : 128u;   // narrow outputs (attention heads): no half-empty tiles
      args.tile_m = bm;
      args.tile_n = bn;
      args.tiles_m = (uint32_t)((m + bm - 1) / bm);
      args.tiles_n = (uint32_t)((n + bn - 1) / bn);
      const uint64_t tiles = (uint64_t)args.tiles_m * args.tiles_n * (uint64_t)batch;
      const uint64_t slices = (uint64_t)(kk + 63) / 64;
      uint64_t splits = std::min<uint64_t>({512 / std::max<uint64_t>(tiles, 1), slices / 4, 16});
      if (r->sealed) splits = 1;   // the second launch writes the dense layout only
      if (splits > 1) {
        args.splits = (uint32_t)splits;
        Storage ws;
        ws.param = -1;
        ws.bytes = (size_t)((uint64_t)splits * (uint64_t)batch * m * n * sizeof(float));
        ws.first_launch = launch;
        ws.last_launch = launch + 1;
        ws_storage = (int32_t)plan->storages.size();
        plan->storages.push_back(ws);
      }
    }
    if (A.dtype == LT_F32) {
      // 64 x 64 tiles unless 128 x 128 ones still give every compute unit a workgroup; a long k
      // over few tiles is split until about two workgroups per compute unit exist (one hides the
      // other's slice boundaries: loads landing, the barrier), each with >= 4 slices of 16.
      // Measured on [B, 2048] x [2048, 2048]: B = 1024 as 512 unsplit tiles of 64 x 64 runs at
      // 85 TFLOP/s (128 x 128 tiles split in two: 78); B = 256 at 54 split in four, 37 unsplit.
      const uint64_t big_tiles = (uint64_t)((m + 127) / 128) * ((n + 127) / 128) * (uint64_t)batch;
      const uint32_t ts = big_tiles >= 256 ? 128u : 64u;
      args.tile_m = args.tile_n = ts;
      const uint64_t tiles = (uint64_t)((m + ts - 1) / ts) * ((n + ts - 1) / ts) * (uint64_t)batch;
      const uint64_t slices = (uint64_t)(kk + 15) / 16;
      uint64_t splits = r->sealed ? 1 : std::min<uint64_t>({512 / std::max<uint64_t>(tiles, 1), slices / 4, 16});
      // Small products (a layer of a small MLP: 128 x 512 x 784) go to the kernel that splits k
      // inside a workgroup of eight waves over a 32 x 32 tile: one launch where the split costs
      // two.  Measured, HIP events around each launch included: 128 x 512 x 784 18.5 -> 14.4 us,
      // 128 x 512 x 512 16.8 -> 11.0, 784 x 512 x 128 (400 tiles) 15.9 -> 12.5.
      // A long k over few tiles (a small batch against a wide weight matrix) is shared by up to
      // eight workgroups per tile, each with at least 256 of k, which exchange their partial tiles
      // inside the same launch (reduction scratch and tickets) -- as long as all of them fit the
      // chip at once, one workgroup per compute unit (a second round costs more than the split
      // pair): [B, 2048] x [2048, 2048] with B = 8 .. 32 23.4 -> 13.1 us (four per tile), B = 64
      // 26.2 -> 17.6 (two per tile); from B = 256 on the split pair is faster.
      {
        const uint64_t tiles32 = (uint64_t)((m + 31) / 32) * ((n + 31) / 32) * (uint64_t)batch;
        if (tiles32 <= 512 && 2.0 * (double)batch * m * n * kk <= 2.5e8 && kk >= 32 && kk <= 1024) {
          args.tile_m = args.tile_n = 32u;
          args.direct = 1u;
          splits = 1;
        } else if (!r->sealed && tiles32 >= 1 && tiles32 <= 256 && kk > 1024) {
          // (above 128 tiles of 32 x 32: tiles of 64 x 32, two blocks times four shares of k per
          // workgroup; B = 128: 30.0 -> 26.2 us.  Tiles of 64 x 64 lose to the split pair everywhere.)
          const uint32_t tm = tiles32 <= 128 ? 32u : 64u;
          const uint64_t tiles = (uint64_t)((m + tm - 1) / tm) * ((n + 31) / 32) * (uint64_t)batch;
          const uint64_t share = std::min<uint64_t>({8, 256 / std::max<uint64_t>(tiles, 1), (uint64_t)kk / 256});
          if (share >= 2) {
            args.tile_m = tm;
            args.tile_n = 32u;
            args.direct = 1u;
            args.splits = (uint32_t)share;   // (workgroups per tile of the one launch, not a second launch)
            splits = 1;
          }
        }
      }
      if (splits > 1) {
        args.splits = (uint32_t)splits;
        Storage ws;
        ws.param = -1;
        ws.bytes = (size_t)(splits * (uint64_t)batch * m * n * sizeof(float));
        ws.first_launch = launch;
        ws.last_launch = launch + 1;
        ws_storage = (int32_t)plan->storages.size();
        plan->storages.push_back(ws);
      }
    }
    if (ws_storage >= 0) {
      // two launches: the contraction proper (no post program), then partial sums + post program
      args.post = ltk::EwProg{};
      Launch l = make_launch(L_GEMM, k, args);
      l.flops = 2ull * (uint64_t)batch * m * n * kk;
      l.bytes = (uint64_t)batch * ((uint64_t)m * kk + (uint64_t)kk * n) * dtype_size(A.dtype);
      plan->launches.push_back(std::move(l));
      plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)(offsetof(ltk::GemmArgs, a) + offsetof(ltk::GemmOperand, ptr)), A.storage, A.byte_offset});
      plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)(offsetof(ltk::GemmArgs, b) + offsetof(ltk::GemmOperand, ptr)), B.storage, B.byte_offset});
      plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)offsetof(ltk::GemmArgs, split_ws), ws_storage, 0, 1});
      touch(A.storage, launch);
      touch(B.storage, launch);
      ltk::SplitPostArgs pa{};
      pa.prog = post.prog;
      pa.splits = args.splits;
      pa.stride = (uint64_t)batch * m * n;
      Launch l2 = make_launch(L_SPLITPOST, k, pa);
      l2.grid_x = ew_grid(post.prog.n);
      l2.bytes = post.bytes;
      plan->launches.push_back(std::move(l2));
      plan->ptr_patches.push_back(PtrPatch{(uint32_t)(launch + 1), (uint32_t)offsetof(ltk::SplitPostArgs, ws), ws_storage, 0});
      add_prog_patches(launch + 1, offsetof(ltk::SplitPostArgs, prog), post);
      note_prog_storages(post, launch + 1);
      return true;
    }
    Launch l = make_launch(L_GEMM, k, args);
    l.flops = 2ull * (uint64_t)batch * m * n * kk;
    l.bytes = post.bytes + (uint64_t)batch * ((uint64_t)m * kk + (uint64_t)kk * n) * dtype_size(A.dtype);
    plan->launches.push_back(std::move(l));
    plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)(offsetof(ltk::GemmArgs, a) + offsetof(ltk::GemmOperand, ptr)), A.storage, A.byte_offset});
    plan->ptr_patches.push_back(PtrPatch{(uint32_t)launch, (uint32_t)(offsetof(ltk::GemmArgs, b) + offsetof(ltk::GemmOperand, ptr)), B.storage, B.byte_offset});
    touch(A.storage, launch);
    touch(B.storage, launch);
    add_prog_patches(launch, offsetof(ltk::GemmArgs, post), post);
    note_prog_storages(post, launch);
    return true;
  }
};

}  // namespace

std::unique_ptr<Plan> lower(lt_ctx* ctx, const Cut& cut, lt_status* status) {
  Lowering L(ctx, cut);
  for (int32_t idx : cut.order) L.nd.push_back(&ctx->nodes[idx]);
  std::unique_ptr<Plan> plan(new Plan());
  L.plan = plan.get();
  L.fold();
  bool ok = L.classify();
  if (ok) {
    L.partition();
    L.donate_and_order();
    ok = L.status == LT_OK;
  }
  if (ok) {
    plan->text = L.plan_text();
    ok = L.codegen();
  }
  if (ok) {
    // patches must be sorted by launch for the single forward sweep of the executor
    std::stable_sort(plan->ptr_patches.begin(), plan->ptr_patches.end(), [](const PtrPatch& x, const PtrPatch& y) { return x.launch < y.launch; });
    std::stable_sort(plan->scal_patches.begin(), plan->scal_patches.end(), [](const ScalPatch& x, const ScalPatch& y) { return x.launch < y.launch; });
    schedule_streams(plan.get());
  }
  if (!ok) {
    *status = L.status == LT_OK ? LT_ERR_UNSUPPORTED : L.status;
    ctx->err = L.err;
    return nullptr;
  }
  *status = LT_OK;
  return plan;
}

}  // namespace lt
