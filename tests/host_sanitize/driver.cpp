// Host-side exercise of the C ABI on the null device, built with -fsanitize=address,undefined
// (tests/test_host_sanitized.py): recording, folding, views, in-place updates, barriers with cache
// hits and misses, every dump, the error paths, arena exhaustion, the fallback hook, the fusion
// switch, release of bases under views.  Exit code 0 = every expectation held; the sanitizers
// abort on their own findings.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/lt.h"

#define CHECK(cond)                                                         \
  do {                                                                      \
    if (!(cond)) {                                                          \
      std::fprintf(stderr, "%s:%d: CHECK failed: %s\n", __FILE__, __LINE__, #cond); \
      std::exit(1);                                                         \
    }                                                                       \
  } while (0)

static lt_ctx* ctx;

static lt_tensor dev(std::vector<int64_t> dims, lt_dtype dt = LT_F32, bool donatable = false) {
  lt_tensor t = 0;
  CHECK(lt_tensor_from_device(ctx, nullptr, dt, (int)dims.size(), dims.data(), donatable ? LT_DONATABLE : 0, &t) == LT_OK);
  return t;
}
static lt_tensor scal(double v) {
  lt_tensor t = 0;
  CHECK(lt_scalar(ctx, LT_F32, v, &t) == LT_OK);
  return t;
}
static lt_tensor op(uint16_t code, std::vector<lt_tensor> in, std::vector<lt_attr> attrs = {}) {
  lt_tensor out = 0;
  CHECK(lt_op(ctx, code, in.data(), (int)in.size(), attrs.data(), (int)attrs.size(), &out, 1) == LT_OK);
  return out;
}
static lt_attr iattr(uint16_t key, int64_t v) {
  lt_attr a{};
  a.key = key;
  a.is_float = 0;
  a.v.i = v;
  return a;
}
static std::string dump(lt_status (*fn)(lt_ctx*, char*, size_t, size_t*)) {
  size_t n = 0;
  CHECK(fn(ctx, nullptr, 0, &n) == LT_OK);
  std::string s(n + 1, '\0');
  CHECK(fn(ctx, &s[0], n + 1, &n) == LT_OK);
  s.resize(n);
  return s;
}
static void rel(std::vector<lt_tensor> ts) { CHECK(lt_release_many(ctx, ts.data(), ts.size()) == LT_OK); }

static int fallback(void*, uint16_t opcode, const lt_tensor_desc* in, int n_in, const lt_attr*, int, lt_tensor_desc* out, int n_out, int run,
                    void*) {
  if (opcode == LT_OP_CUSTOM + 1) return 1;
  if (!run) {
    for (int s = 0; s < n_out; ++s) {
      out[s].dtype = in[0].dtype;
      out[s].rank = in[0].rank;
      for (int d = 0; d < in[0].rank; ++d) out[s].dims[d] = in[0].dims[d];
    }
  }
  return n_in >= 1 ? 0 : 1;
}

int main() {
  CHECK(lt_init(-1, nullptr, nullptr, 0, &ctx) == LT_OK);
  lt_barrier_info info{};
  // the elementwise + reduce trace of the first configuration, ten times: one miss, nine hits
  lt_tensor x = dev({64, 48}), y = dev({64, 48}), bias = dev({48});
  for (int it = 0; it < 10; ++it) {
    lt_tensor half = scal(0.5);
    lt_tensor t = op(LT_OP_TANH, {op(LT_OP_ADD, {op(LT_OP_MUL, {x, y}), bias})});
    lt_tensor e = op(LT_OP_EXP, {op(LT_OP_NEG, {op(LT_OP_SQUARE, {x})})});
    lt_tensor z = op(LT_OP_ADD, {op(LT_OP_MUL, {t, e}), y, half});
    lt_tensor s = op(LT_OP_SUM, {z}, {iattr(LT_ATTR_AXIS, 1)});
    lt_tensor out = op(LT_OP_DIV, {s, op(LT_OP_AMAX, {op(LT_OP_ABS, {s})})});
    lt_stats_t st{};
    CHECK(lt_stats(ctx, &st) == LT_OK);
    // everything but `out` dies before the cut (ids are consecutive: release all in between)
    std::vector<lt_tensor> dead;
    for (lt_tensor id = half; id < out; ++id) dead.push_back(id);
    (void)lt_release_many(ctx, dead.data(), dead.size());   // (some ids in the range belong to nobody: reported, skipped)
    if (it == 0) CHECK(dump(lt_dump_ir).find("ROOT=0") != std::string::npos);
    CHECK(lt_barrier(ctx, 1, &info) == LT_OK);
    CHECK(info.cache_hit == (it > 0) && info.n_regions == 2 && info.n_roots == 1);
    CHECK(lt_release(ctx, out) == LT_OK);
  }
  CHECK(dump(lt_dump_plan).find("R1 ALL") != std::string::npos);
  CHECK(!dump(lt_dump_schedule).empty());
  std::vector<uint8_t> key(info.key_bytes);
  size_t klen = 0;
  CHECK(lt_dump_key(ctx, key.data(), key.size(), &klen) == LT_OK && klen == info.key_bytes);
  // an optimiser-like update in place, special scalars folded away, then the same step again
  lt_tensor p = dev({1 << 12}, LT_F32, true), g = dev({1 << 12});
  for (int it = 0; it < 2; ++it) {
    lt_tensor lr = scal(0.01 * (it + 1)), one = scal(1.0), zero = scal(0.0);
    lt_tensor upd = op(LT_OP_SUB, {op(LT_OP_MUL, {p, one}), op(LT_OP_ADD, {op(LT_OP_MUL, {g, lr}), zero})});
    CHECK(lt_assign(ctx, p, upd) == LT_OK);
    std::vector<lt_tensor> dead;
    for (lt_tensor id = lr; id <= upd; ++id) dead.push_back(id);
    (void)lt_release_many(ctx, dead.data(), dead.size());
    CHECK(lt_barrier(ctx, 0, &info) == LT_OK);
    CHECK(info.cache_hit == it && dump(lt_dump_plan).find("->p") != std::string::npos);
  }
  // a contraction with epilogue, a column reduction, a row operator with three results
  lt_tensor a = dev({128, 64}), w = dev({64, 32}), b2 = dev({32}), lab = dev({128}, LT_I32);
  lt_tensor h = op(LT_OP_RELU, {op(LT_OP_ADD, {op(LT_OP_MATMUL, {a, w}), b2})});
  lt_tensor col = op(LT_OP_SUM, {h}, {iattr(LT_ATTR_AXIS, 0)});
  lt_tensor loss = op(LT_OP_MEAN, {op(LT_OP_XENT, {h, lab})});
  lt_tensor ln[3];
  lt_attr eps{};
  eps.key = LT_ATTR_EPS;
  eps.is_float = 1;
  eps.v.f = 1e-5;
  lt_tensor ln_in[3] = {h, b2, b2};
  CHECK(lt_op(ctx, LT_OP_LAYER_NORM, ln_in, 3, &eps, 1, ln, 3) == LT_OK);
  CHECK(lt_barrier(ctx, 1, &info) == LT_OK && info.n_regions >= 4 && info.flops_planned == 2ull * 128 * 64 * 32);
  (void)col; (void)loss;
  // a weight gradient and the bias gradient next to it (the column sum rides in the contraction's
  // launch: two regions, one launch), a long k over few tiles (workgroups share tiles), and a pair
  // that must not share a launch (the column program reads what the contraction writes)
  {
    lt_tensor gx = dev({128, 96}), gdy = dev({128, 64}), gw = dev({96, 64}, LT_F32, true), gb = dev({64}, LT_F32, true);
    lt_tensor dw = op(LT_OP_MATMUL, {gx, gdy}, {iattr(LT_ATTR_TRANS_A, 1)});
    lt_tensor db = op(LT_OP_SUM, {gdy}, {iattr(LT_ATTR_AXIS, 0)});
    CHECK(lt_assign(ctx, gw, op(LT_OP_SUB, {gw, op(LT_OP_MUL, {dw, scal(0.01)})})) == LT_OK);
    CHECK(lt_assign(ctx, gb, op(LT_OP_SUB, {gb, op(LT_OP_MUL, {db, scal(0.01)})})) == LT_OK);
    CHECK(lt_barrier(ctx, 1, &info) == LT_OK && info.n_regions == 2 && info.n_launches == 1);
    lt_tensor lx = dev({8, 2048}), lw = dev({2048, 512});
    lt_tensor ly = op(LT_OP_MATMUL, {lx, lw});
    CHECK(lt_barrier(ctx, 1, &info) == LT_OK && info.n_launches == 1);
    lt_tensor dw2 = op(LT_OP_MATMUL, {gx, gdy}, {iattr(LT_ATTR_TRANS_A, 1)});
    CHECK(lt_assign(ctx, gw, op(LT_OP_SUB, {gw, op(LT_OP_MUL, {dw2, scal(0.01)})})) == LT_OK);
    lt_attr first[3] = {iattr(LT_ATTR_AXIS, 0), iattr(LT_ATTR_START, 0), iattr(LT_ATTR_LENGTH, 1)};
    lt_attr to_vec[1] = {iattr(LT_ATTR_DIM0, 64)};
    lt_tensor row0 = op(LT_OP_RESHAPE, {op(LT_OP_NARROW, {gw}, {first[0], first[1], first[2]})}, {to_vec[0]});
    lt_tensor db2 = op(LT_OP_ADD, {op(LT_OP_SUM, {gdy}, {iattr(LT_ATTR_AXIS, 0)}), row0});
    CHECK(lt_barrier(ctx, 1, &info) == LT_OK && info.n_launches >= 2);
    (void)ly; (void)db2;
  }
  // views: the program of the paper's figure 3, a window, a view of a view, a released base
  lt_tensor vx = dev({2, 3, 4}, LT_F32, true);
  lt_attr perm[3] = {iattr(LT_ATTR_DIM0, 1), iattr(LT_ATTR_DIM0 + 1, 2), iattr(LT_ATTR_DIM0 + 2, 0)};
  lt_tensor v = 0;
  CHECK(lt_view(ctx, vx, LT_OP_PERMUTE, perm, 3, &v) == LT_OK);
  CHECK(lt_assign(ctx, v, op(LT_OP_ADD, {v, scal(42.0)})) == LT_OK);
  lt_attr win[3] = {iattr(LT_ATTR_AXIS, 1), iattr(LT_ATTR_START, 1), iattr(LT_ATTR_LENGTH, 2)};
  lt_tensor wv = 0;
  CHECK(lt_view(ctx, vx, LT_OP_NARROW, win, 3, &wv) == LT_OK);
  CHECK(lt_assign(ctx, wv, op(LT_OP_MUL, {wv, scal(2.0)})) == LT_OK);
  lt_attr flat[2] = {iattr(LT_ATTR_DIM0, 6), iattr(LT_ATTR_DIM0 + 1, 4)};
  lt_tensor rv = 0, cv = 0;
  CHECK(lt_view(ctx, vx, LT_OP_RESHAPE, flat, 2, &rv) == LT_OK);
  lt_attr win2[3] = {iattr(LT_ATTR_AXIS, 0), iattr(LT_ATTR_START, 2), iattr(LT_ATTR_LENGTH, 3)};
  CHECK(lt_view(ctx, rv, LT_OP_NARROW, win2, 3, &cv) == LT_OK);
  CHECK(lt_assign(ctx, cv, op(LT_OP_NEG, {cv})) == LT_OK);
  CHECK(lt_assign(ctx, wv, vx) == LT_ERR_SHAPE);
  CHECK(lt_release(ctx, vx) == LT_OK);              // hidden: views still name it
  CHECK(lt_release(ctx, vx) == LT_ERR_HANDLE);
  CHECK(lt_barrier(ctx, 1, &info) == LT_OK && dump(lt_dump_plan).find(" SLICE ") != std::string::npos);
  CHECK(lt_assign(ctx, v, op(LT_OP_MUL, {v, scal(3.0)})) == LT_OK);
  CHECK(lt_barrier(ctx, 1, &info) == LT_OK);
  rel({cv, rv, wv, v});
  // error paths
  lt_tensor bad = 0;
  lt_tensor two[2] = {a, w};
  CHECK(lt_op(ctx, LT_OP_ADD, two, 2, nullptr, 0, &bad, 1) == LT_ERR_SHAPE);
  CHECK(std::strstr(lt_last_error(ctx), "broadcast") != nullptr);
  CHECK(lt_op(ctx, 999, two, 1, nullptr, 0, &bad, 1) == LT_ERR_UNSUPPORTED);
  CHECK(lt_op(ctx, LT_OP_CUSTOM, two, 1, nullptr, 0, &bad, 1) == LT_ERR_UNSUPPORTED);
  float hostbuf[4];
  CHECK(lt_fetch(ctx, b2, hostbuf, 32 * 4) == LT_ERR_DEVICE);
  CHECK(lt_fetch(ctx, 123456, hostbuf, 4) == LT_ERR_HANDLE);
  void* dp = nullptr;
  CHECK(lt_device_ptr(ctx, col, &dp) == LT_OK);
  lt_dtype dt;
  int rank;
  int64_t dims[LT_MAX_RANK];
  CHECK(lt_shape(ctx, ln[1], &dt, &rank, dims) == LT_OK && rank == 1 && dims[0] == 128 && dt == LT_F32);
  // the fallback hook and the fusion switch
  CHECK(lt_set_fallback(ctx, fallback, nullptr) == LT_OK);
  lt_tensor r3 = dev({2, 3, 4});
  lt_tensor mid = op(LT_OP_SUM, {op(LT_OP_EXP, {r3})}, {iattr(LT_ATTR_AXIS, 1)});
  CHECK(lt_device_ptr(ctx, mid, &dp) == LT_OK);
  lt_tensor cu = op(LT_OP_CUSTOM, {mid});
  CHECK(lt_shape(ctx, cu, &dt, &rank, dims) == LT_OK && rank == 2 && dims[1] == 4);
  CHECK(lt_op(ctx, LT_OP_CUSTOM + 1, &mid, 1, nullptr, 0, &bad, 1) == LT_ERR_UNSUPPORTED);
  CHECK(lt_set_fallback(ctx, nullptr, nullptr) == LT_OK);
  CHECK(lt_set_fusion(ctx, 0) == LT_OK);
  lt_tensor f1 = op(LT_OP_TANH, {op(LT_OP_EXP, {op(LT_OP_NEG, {r3})})});
  CHECK(lt_barrier(ctx, 1, &info) == LT_OK && info.n_regions >= 3);
  CHECK(lt_set_fusion(ctx, 1) == LT_OK);
  (void)f1;
  CHECK(lt_barrier_static(ctx, 1, &info) == LT_OK);
  CHECK(lt_set_streams(ctx, 9) == LT_ERR_ARG && lt_set_streams(ctx, 1) == LT_OK && lt_set_profiling(ctx, 1) == LT_OK);
  lt_launch_record recs[4];
  int nrec = 0;
  CHECK(lt_last_launches(ctx, recs, 4, &nrec) == LT_OK);
  CHECK(lt_shutdown(ctx) == LT_OK);
  // hashing while recording (every fingerprint hit checked against the canonical key), captured
  // steps, re-pointed inputs
  CHECK(lt_init(-1, nullptr, nullptr, 0, &ctx) == LT_OK);
  CHECK(lt_set_quick_lookup(ctx, 3) == LT_ERR_ARG && lt_set_quick_lookup(ctx, 2) == LT_OK && lt_set_graphs(ctx, 1) == LT_OK);
  lt_step* none = nullptr;
  CHECK(lt_step_capture(ctx, &none) == LT_ERR_ARG && none == nullptr);
  lt_tensor sp = dev({512}, LT_F32, true), sg = dev({512});
  lt_tensor snorm = 0;
  for (int it = 0; it < 3; ++it) {
    lt_tensor lr = scal(0.125 * (it + 1));
    lt_tensor upd = op(LT_OP_SUB, {sp, op(LT_OP_MUL, {sg, lr})});
    lt_tensor nn = op(LT_OP_SUM, {op(LT_OP_SQUARE, {upd})});
    CHECK(lt_assign(ctx, sp, upd) == LT_OK);
    if (snorm) CHECK(lt_release(ctx, snorm) == LT_OK);
    snorm = nn;
    rel({lr, upd});
    CHECK(lt_barrier(ctx, 1, &info) == LT_OK && info.cache_hit == (it > 0));
  }
  lt_stats_t qs{};
  CHECK(lt_stats(ctx, &qs) == LT_OK && qs.quick_hits == 2 && qs.cache_hits == 2);
  lt_step* step = nullptr;
  CHECK(lt_step_capture(ctx, &step) == LT_OK && step != nullptr);
  double sv[4];
  CHECK(lt_step_scalars(step, sv, 4) == 1 && sv[0] == 0.375 && lt_step_scalars(nullptr, sv, 4) == -1);
  CHECK(lt_step_replay(ctx, step, nullptr, 0, 1, &info) == LT_OK && info.cache_hit == 1 && info.n_regions >= 1);
  sv[0] = 0.5;
  CHECK(lt_step_replay(ctx, step, sv, 1, 0, nullptr) == LT_OK);
  CHECK(lt_step_replay(ctx, step, sv, 2, 0, nullptr) == LT_ERR_ARG);
  CHECK(lt_tensor_rebind(ctx, sg, nullptr) == LT_OK);                 // (a null device: any pointer)
  CHECK(lt_tensor_rebind(ctx, snorm, nullptr) == LT_ERR_ARG);         // a result: library memory
  CHECK(lt_step_replay(ctx, step, nullptr, 0, 1, nullptr) == LT_OK);
  lt_tensor pend = op(LT_OP_EXP, {sg});
  CHECK(lt_tensor_rebind(ctx, sg, nullptr) == LT_ERR_ARG);            // read by the pending trace
  CHECK(lt_step_replay(ctx, step, nullptr, 0, 1, nullptr) == LT_ERR_ARG);
  CHECK(lt_barrier(ctx, 1, nullptr) == LT_OK);
  rel({pend});
  CHECK(lt_stats(ctx, &qs) == LT_OK && qs.replays == 3);
  CHECK(lt_release(ctx, sg) == LT_OK);
  CHECK(lt_step_replay(ctx, step, nullptr, 0, 1, nullptr) == LT_ERR_HANDLE);
  CHECK(lt_set_fusion(ctx, 0) == LT_OK);
  CHECK(lt_step_replay(ctx, step, nullptr, 0, 1, nullptr) == LT_ERR_ARG);   // the plan is gone with the cache
  lt_step_free(step);
  lt_step_free(nullptr);
  CHECK(lt_shutdown(ctx) == LT_OK);
  // arena exhaustion on a small workspace: found before anything runs, trace stays pending
  CHECK(lt_init(-1, nullptr, nullptr, 13u << 20, &ctx) == LT_OK);
  lt_tensor big = dev({1 << 20});
  lt_tensor e1 = op(LT_OP_EXP, {big});
  CHECK(lt_barrier(ctx, 1, nullptr) == LT_OK);
  lt_tensor e2 = op(LT_OP_EXP, {e1}), e3 = op(LT_OP_TANH, {big});
  CHECK(lt_barrier(ctx, 1, nullptr) == LT_ERR_OOM);
  CHECK(lt_release(ctx, e1) == LT_OK);
  (void)e2; (void)e3;
  CHECK(lt_shutdown(ctx) == LT_OK);
  CHECK(lt_init(-2, nullptr, nullptr, 0, &ctx) == LT_ERR_ARG && lt_last_error(nullptr)[0] != 0);
  std::puts("host sanitizer driver: ok");
  return 0;
}
