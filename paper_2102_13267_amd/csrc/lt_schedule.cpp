// Stream schedule of a lowered plan.
//
// The launches of a plan form a DAG (a launch depends on the earlier launches whose storages it
// reads or overwrites), but one stream runs them as a chain.  Backward passes are full of
// independent work -- a weight gradient, the bias gradient next to it and the gradient that flows
// on all read the same tensor -- and the small launches among it (column reductions, the second
// halves of split contractions) leave most of the chip idle.  So every launch is given one of up
// to kMaxStreams streams by list scheduling with a crude duration model, and the cross-stream
// edges of the DAG become events.  Launch order inside a stream stays plan order.
//
// Hazards handled here: read-after-write, write-after-read and write-after-write on storages
// (donated outputs alias their parameter: both are keyed by the parameter ordinal), and the
// reduction scratch (partials and tickets), which is cut into kScratchSlots quarters so that up to
// that many reductions can be in flight.  Not handled here: reuse of arena memory inside a step;
// the executor does not recycle temporaries of a multi-stream plan before the streams have joined.
//
// Measured on the transformer-layer step (48 launches): spreading every launch by earliest start
// gains there but costs a step of twenty 6-microsecond kernels 5 % (40 % with non-blocking
// barriers): two events per edge are dearer than such a kernel.  So what may leave the caller's
// stream is what is long enough to pay for its events: column reductions of a few megabytes and
// more, and any other launch estimated at kSpreadUs or more (consecutive independent contractions
// then overlap one's epilogue and tail with the next one's start: +5 % on that step on top of the
// reductions' +3 %); the small step is left alone.
#include <algorithm>
#include <map>
#include <set>

#include "lt_core.h"

namespace lt {

namespace {

struct MemState {
  int last_writer = -1;
  std::vector<int> readers;   // since the last write
};

// microseconds, only good enough to balance streams
double estimate_us(const Launch& l) {
  const double mem = (double)l.bytes / 3.0e6;   // 3 TB/s
  if (l.kind == L_GEMM) return 8.0 + std::max(mem, (double)l.flops / 4.0e8);   // 400 TFLOP/s
  if (l.kind == L_COL) return 12.0 + mem;       // latency bound: dependent trips, ticket, last-workgroup pass
  return 6.0 + mem;
}

}  // namespace

uint64_t gemm_shared_tiles(const Launch& l) {
  if (l.kind != L_GEMM) return 0;
  const ltk::GemmArgs* a = (const ltk::GemmArgs*)l.args.data();
  if (!a->direct || a->splits <= 1u) return 0;
  return (uint64_t)((a->m + a->tile_m - 1u) / a->tile_m) * ((a->n + a->tile_n - 1u) / a->tile_n) * a->batch0 * a->batch1;
}

void schedule_streams(Plan* plan) {
  const size_t n = plan->launches.size();
  plan->n_streams = 1;
  plan->temp_bytes = 0;
  for (const Storage& st : plan->storages)
    if (st.param < 0) plan->temp_bytes += (st.bytes + 255) & ~(size_t)255;
  if (n == 0) return;

  // what each launch reads and writes
  std::vector<std::vector<int64_t>> reads(n), writes(n);
  auto key_of = [&](int32_t s) -> int64_t {
    const Storage& st = plan->storages[s];
    return st.param >= 0 ? -(int64_t)st.param - 1 : (int64_t)s;
  };
  for (const PtrPatch& p : plan->ptr_patches) {
    if (p.storage < 0) continue;
    (p.write ? writes : reads)[p.launch].push_back(key_of(p.storage));
  }
  // reduction scratch: a quarter each while it fits, otherwise all of it
  constexpr int64_t kScratchKey = INT64_MIN / 2;
  int next_slot = 0;
  for (size_t i = 0; i < n; ++i) {
    Launch& l = plan->launches[i];
    l.stream = 0;
    l.record = 0;
    l.scratch_slot = 0;
    l.waits.clear();
    const uint64_t shared_tiles = gemm_shared_tiles(l);   // (a small contraction whose workgroups share tiles)
    if (l.kind != L_ALL && l.kind != L_COL && shared_tiles == 0) continue;
    uint64_t floats = l.grid_x, tickets = 1;
    if (l.kind == L_COL) {
      const ltk::ColArgs* a = (const ltk::ColArgs*)l.args.data();
      floats = (uint64_t)l.grid_y * ((a->cols + 3u) & ~3u);
      tickets = l.grid_x;
    } else if (l.kind == L_GEMM) {
      {
        const ltk::GemmArgs* a = (const ltk::GemmArgs*)l.args.data();
        floats = shared_tiles * a->splits * a->tile_m * a->tile_n;
      }
      tickets = shared_tiles;
    }
    if (floats <= kPartialFloats / kScratchSlots && tickets <= kTickets / kScratchSlots) {
      l.scratch_slot = (uint8_t)next_slot;
      writes[i].push_back(kScratchKey + next_slot);
      next_slot = (next_slot + 1) % kScratchSlots;
    } else {
      for (int s = 0; s < kScratchSlots; ++s) writes[i].push_back(kScratchKey + s);
    }
  }

  std::map<int64_t, MemState> mem;
  std::vector<double> finish(n, 0.0);
  double avail[kMaxStreams] = {0, 0, 0, 0};
  int waited[kMaxStreams][kMaxStreams];   // [waiting stream][other stream]: last launch of it already waited for
  for (auto& row : waited)
    for (int& w : row) w = -1;
  constexpr double kSyncUs = 4.0;   // what a cross-stream edge costs
  constexpr double kSpreadUs = 10.0;   // launches at least this long may start early on a side stream

  for (size_t i = 0; i < n; ++i) {
    Launch& l = plan->launches[i];
    std::set<int> deps;
    for (int64_t k : reads[i]) {
      auto it = mem.find(k);
      if (it != mem.end() && it->second.last_writer >= 0) deps.insert(it->second.last_writer);
    }
    for (int64_t k : writes[i]) {
      auto it = mem.find(k);
      if (it == mem.end()) continue;
      if (it->second.last_writer >= 0) deps.insert(it->second.last_writer);
      for (int r : it->second.readers) deps.insert(r);
    }
    deps.erase((int)i);
    // Stream choice: the stream on which the launch can start first, among those it may use.
    // Short launches stay on the caller's stream, in plan order (an event costs more than they
    // do).  What may move: column reductions of a few megabytes and more (a chain of dependent
    // trips, a ticket and a last-workgroup pass, at most 256 workgroups: most of the chip is idle
    // under them), and launches of kSpreadUs and more (workgroups of the next independent launch
    // fill the chip while this one's last workgroups run their epilogues).  A narrow launch that
    // depends on side stream work follows it there, so that the caller's stream never stalls
    // behind a side stream for the sake of a small kernel.
    const bool narrow = l.kind == L_COL || (l.kind != L_GEMM && l.bytes < (4u << 20));
    const bool movable = l.kind == L_COL ? l.bytes >= (4u << 20) : estimate_us(l) >= kSpreadUs;
    int best = 0;
    double best_start = 0;
    for (int s = 0; s < kMaxStreams; ++s) {
      double start = avail[s];
      bool follows = false;
      for (int d : deps) {
        const bool same = plan->launches[d].stream == s;
        follows |= same && s > 0;
        start = std::max(start, finish[d] + (same ? 0.0 : kSyncUs));
      }
      if (s > 0 && avail[s] == 0.0) start = std::max(start, kSyncUs);   // a side stream first has to be forked
      if (s > 0 && !(movable || (narrow && follows))) continue;
      if (s == 0 || start + 1e-9 < best_start) {
        best = s;
        best_start = start;
      }
    }
    l.stream = (uint8_t)best;
    finish[i] = best_start + estimate_us(l);
    avail[best] = finish[i];
    plan->n_streams = std::max(plan->n_streams, best + 1);
    for (auto it = deps.rbegin(); it != deps.rend(); ++it) {   // latest first: it covers the earlier ones of its stream
      const int d = *it;
      const int sd = plan->launches[d].stream;
      if (sd == best || waited[best][sd] >= d) continue;
      waited[best][sd] = d;
      l.waits.push_back((uint32_t)d);
      plan->launches[d].record = 1;
    }
    for (int64_t k : writes[i]) {
      MemState& m = mem[k];
      m.last_writer = (int)i;
      m.readers.clear();
    }
    for (int64_t k : reads[i]) {
      MemState& m = mem[k];
      if (m.last_writer != (int)i) m.readers.push_back((int)i);
    }
  }
}

}  // namespace lt
