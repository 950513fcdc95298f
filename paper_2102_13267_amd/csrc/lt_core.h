// Internal host-side data structures of the LazyTensor library: IR nodes, tensor handles,
// device buffers, the workspace arena, cached plans and the context (the paper's
// DeviceContextArena, section 4).
#ifndef LT_CORE_H_
#define LT_CORE_H_

#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <cstring>
#include <map>
#include <memory>
#include <string>
#include <unordered_map>
#include <vector>

#include "../../include/lt.h"
#include "lt_kernels.h"

namespace lt {

// node kinds that the public opcode enum does not list (leaves)
enum : uint16_t { OP_DEVICE_DATA = 1, OP_SCALAR_PARAM = 2, OP_CONSTANT = 3 };

constexpr int kMaxAttrs = 8;
constexpr int kMaxIns = 5;

// caps on one fused region (part of the partition rules)
constexpr int kMaxRegionInputs = 8;
constexpr int kMaxRegionOutputs = 8;
constexpr int kMaxRegionSlots = 32;
constexpr int64_t kMaxFinaliserElems = 65536;

constexpr int kMaxStreams = 4;     // the caller's stream + three side streams
constexpr int kScratchSlots = 4;   // quarters of the reduction scratch, one per concurrent reduction

struct Arena;

// A device buffer.  Borrowed buffers belong to the caller; owned ones are carved out of the
// workspace arena and return to it when the last reference goes away.
struct Buffer {
  void* ptr = nullptr;
  size_t bytes = 0;
  bool owned = false;
  bool donatable = false;
  int data_refs = 0;   // live handles currently bound to this buffer
  Arena* arena = nullptr;
  ~Buffer();
};
using BufRef = std::shared_ptr<Buffer>;

// First-fit free-list allocator over the caller's workspace (256-byte granules).
struct Arena {
  uintptr_t base = 0;
  size_t size = 0;
  std::map<uintptr_t, size_t> free_blocks;   // offset -> length
  std::unordered_map<uintptr_t, size_t> used;  // offset -> length
  size_t in_use = 0, peak = 0;
  void init(void* p, size_t bytes);
  void* alloc(size_t bytes);   // nullptr when exhausted
  void release(void* p);
};

struct Attr {
  uint16_t key;
  uint8_t is_float;
  union { int64_t i; double f; } v;
};

struct Val {
  int32_t node;
  int32_t slot;
  bool operator==(const Val& o) const { return node == o.node && slot == o.slot; }
  bool operator!=(const Val& o) const { return !(*this == o); }
};

struct Node {
  uint16_t op = 0;
  uint8_t dtype = 0, rank = 0, n_attr = 0, n_in = 0, n_out = 1;
  int64_t dims[LT_MAX_RANK] = {0};
  Attr attrs[kMaxAttrs];
  Val ins[kMaxIns];
  BufRef buffer;       // OP_DEVICE_DATA
  double value = 0;    // OP_SCALAR_PARAM: the dynamic value (not part of the graph's identity)
  uint64_t src = 0;    // leaves: id of the tensor the leaf was made from (a captured step names its inputs by it)
};

enum HandleKind : uint8_t { H_PENDING = 0, H_DATA = 1, H_SCALAR = 2 };

struct Handle {
  uint64_t id = 0;
  HandleKind kind = H_DATA;
  uint8_t dtype = 0, rank = 0;
  int64_t dims[LT_MAX_RANK] = {0};
  int32_t node = -1, slot = 0;    // H_PENDING
  BufRef buf;                     // H_DATA
  double value = 0;               // H_SCALAR
  BufRef donor;                   // buffer this handle gave up through lt_assign
  uint64_t memo_epoch = ~0ull;    // leaf node created for this handle in the current trace
  int32_t memo_node = -1;
  // views (section 4.4): a view handle names its base and the view op; its value is that op
  // applied to the base's CURRENT value, recomputed when the base has changed since (`seen`)
  uint64_t version = 0;           // bumped whenever the handle's value is replaced
  uint64_t view_base = 0;         // tensor id of the base (0: not a view)
  uint16_t view_op = 0;           // LT_OP_PERMUTE / LT_OP_RESHAPE / LT_OP_NARROW
  uint8_t view_n_attr = 0;
  lt_attr view_attrs[kMaxAttrs];
  uint64_t seen = 0;              // base's version that the current value was derived from
  int32_t view_refs = 0;          // views that name this handle as their base
  bool released = false;          // released by the caller, kept while views still name it
};

// ---- a lowered, cached program ------------------------------------------------------------

enum LaunchKind : uint8_t { L_EW, L_ROW, L_ALL, L_COL, L_ROWOP, L_GEMM, L_SPLITPOST, L_SLICE };

struct Storage {
  int param = -1;        // >= 0: the buffer of device parameter `param` (input, or donated output)
  size_t bytes = 0;      // param < 0: a fresh arena allocation of this size
  int first_launch = 0, last_launch = 0;
  bool bound_to_root = false;
};

struct PtrPatch {
  uint32_t launch, offset;   // byte offset of a pointer field inside the launch's argument block
  int32_t storage;
  int64_t byte_offset;
  uint8_t write = 0;         // 1: the launch writes this storage (0: it only reads it)
};

struct ScalPatch {
  uint32_t launch, offset;   // byte offset of a float inside the argument block
  int32_t scalar;            // scalar parameter ordinal
  uint8_t reciprocal;        // 1: store 1/value
};

struct Launch {
  LaunchKind kind;
  int32_t region;
  uint32_t grid_x = 1, grid_y = 1;
  std::vector<uint8_t> args;
  uint64_t bytes = 0, flops = 0;
  // stream schedule (schedule_streams): which of the context's streams runs the launch, the
  // earlier launches on OTHER streams it has to wait for, whether a later launch on another
  // stream waits for it, and its quarter of the reduction scratch
  uint8_t stream = 0, record = 0, scratch_slot = 0;
  std::vector<uint32_t> waits;
};

struct RootBind {
  enum Kind : uint8_t { STORAGE, PARAM_ALIAS, SCALAR, CONST } kind = STORAGE;
  int32_t index = -1;        // storage / param ordinal / scalar ordinal
  double value = 0;          // CONST
};

// Instantiated HIP graphs of a plan, by the signature of everything that goes into its launches'
// arguments (the address of every storage, the scalars): a step whose buffers sit where they sat
// before is enqueued as one graph launch instead of one launch and up to two events per kernel.
struct GraphEntry {
  uint64_t sig = 0;
  hipGraphExec_t exec = nullptr;
  uint64_t used = 0;     // (for least-recently-used replacement)
};
struct GraphSlots {
  static constexpr size_t kMax = 4, kSeen = 8;
  std::vector<GraphEntry> entries;
  uint64_t seen[kSeen] = {0};   // signatures of recent steps: a graph is built for one that comes back
  size_t n_seen = 0;
  uint64_t clock = 0;
  bool disabled = false;        // a capture failed: this plan is launched kernel by kernel from now on
};

struct Plan {
  std::vector<uint8_t> key;
  std::string text;
  int n_params = 0, n_scalars = 0, n_regions = 0;
  std::vector<Storage> storages;
  std::vector<Launch> launches;
  std::vector<PtrPatch> ptr_patches;
  std::vector<ScalPatch> scal_patches;
  std::vector<RootBind> roots;
  uint64_t bytes_planned = 0, flops_planned = 0;
  int n_streams = 1;                 // streams the schedule uses (1: everything on the caller's stream)
  size_t temp_bytes = 0;             // arena bytes when no temporary is reused inside the step
  std::vector<hipEvent_t> events;    // one per launch with `record` set (created on first use)
  GraphSlots graphs;                 // lt_set_graphs
};

// Fingerprint of the trace as it is being recorded (section 7 of the paper: hashing while the graph
// is built, instead of walking it again at the barrier): two independent 64-bit lanes, one word
// at a time.  It covers every recorded node in record order -- opcode, type, shape, attributes,
// operands by record index, which earlier leaf shares a leaf's buffer -- so two traces with the
// same fingerprint and the same live roots have the same canonical form.
struct Fingerprint {
  uint64_t a = 0x9e3779b97f4a7c15ull, b = 0xc2b2ae3d27d4eb4full;
  void mix(uint64_t w) {
    a = (a ^ w) * 0xff51afd7ed558ccdull;
    a ^= a >> 29;
    b = (b + w) * 0xc4ceb9fe1a85ec53ull;
    b ^= b >> 31;
  }
  bool operator==(const Fingerprint& o) const { return a == o.a && b == o.b; }
};
struct FingerprintHash {
  size_t operator()(const Fingerprint& f) const { return (size_t)(f.a ^ (f.b * 0x9e3779b97f4a7c15ull)); }
};

// What the barrier needs of a trace it has seen before, by fingerprint: the plan, and where in the
// recorded trace the plan's parameters and scalars are (record indices, canonical order).
struct QuickEntry {
  Plan* plan = nullptr;
  uint64_t generation = 0, hash = 0;
  int32_t n_nodes = 0;                       // nodes of the canonical cut
  std::vector<int32_t> param_nodes, scalar_nodes;
};

// What a captured step has to know about the barrier it repeats: the plan, the tensors whose
// data were the plan's device parameters (canonical order) with what the plan assumed of them,
// the non-special scalars, and the tensors that received the roots.
struct StepParam {
  uint64_t tensor = 0;
  uint8_t dtype = 0, rank = 0;
  int64_t dims[LT_MAX_RANK] = {0};
  bool donatable = false;
};
struct StepRecord {
  Plan* plan = nullptr;
  uint64_t generation = 0;           // of the plan cache (plans die when the cache is cleared)
  std::vector<StepParam> params;
  std::vector<double> scalars;
  std::vector<uint64_t> roots;       // tensor ids, in the plan's root order
  bool bound_plain = false;          // a tensor took another's plain data or scalar (no node): not repeatable
};

}  // namespace lt

struct lt_step {
  lt_ctx* ctx = nullptr;
  lt::StepRecord rec;
  std::vector<uint8_t> written;      // per parameter: the plan writes its buffer (a donated input)
};

struct lt_ctx {
  int device = -1;
  hipStream_t stream = nullptr;
  std::string device_name;
  lt::Arena arena;
  std::vector<lt::Node> nodes;               // the trace being recorded (flat arena, indices not pointers)
  std::map<uint64_t, lt::Handle> handles;    // live tensors by id
  uint64_t next_id = 1, epoch = 0;
  std::unordered_map<uint64_t, std::vector<std::unique_ptr<lt::Plan>>> cache;
  lt::Plan* last_plan = nullptr;
  uint64_t cache_generation = 0;             // bumped whenever the plan cache is cleared
  // record-time fingerprint of the pending trace, the first leaf of every buffer it reads, and
  // the plans by fingerprint (lt_set_quick_lookup)
  lt::Fingerprint trace_fp;
  std::unordered_map<const lt::Buffer*, int32_t> leaf_of_buffer;
  std::unordered_map<lt::Fingerprint, lt::QuickEntry, lt::FingerprintHash> quick;
  int quick_lookup = 1;                      // 0: off, 1: on, 2: on, and every hit is checked against the canonical key
  lt::StepRecord last_step;                  // the last barrier, for lt_step_capture
  bool bound_plain = false;                  // since the last barrier, lt_assign gave a tensor plain data or a scalar
  lt_stats_t stats{};
  std::string err;
  float* red_partials = nullptr;             // reduction scratch inside the workspace
  uint32_t* red_tickets = nullptr;
  bool profiling = false;
  std::vector<lt_launch_record> last_launches;
  std::vector<hipEvent_t> events;
  // side streams for launches that do not depend on each other (default priority, created by
  // lt_init), and the events that fork them from / join them into the caller's stream
  hipStream_t side[lt::kMaxStreams - 1] = {};
  hipEvent_t fork_event = nullptr, join_event[lt::kMaxStreams - 1] = {};
  int max_streams = lt::kMaxStreams;   // lt_set_streams
  bool graphs = false;                 // lt_set_graphs: steps with unchanged addresses run as one HIP graph
  hipStream_t graph_stream = nullptr;  // the stream that graph captures are made on (created on first use)
  bool fusion = true;                  // lt_set_fusion: off = one region per recorded op
  lt_fallback_fn fallback = nullptr;   // lt_set_fallback: eager implementation of ops without a lowering
  void* fallback_user = nullptr;
  // the library's static device scratch on this device (lt_barrier_static): reduction partials,
  // tickets, then room for a plan's temporaries
  uint8_t* static_scratch = nullptr;
  size_t static_scratch_bytes = 0;
  std::string static_scratch_error;    // why the array's address could not be had (empty: it could)
};

namespace lt {

constexpr size_t kPartialFloats = 1 << 20;   // reduction partials (4 MiB of the workspace)
constexpr size_t kTickets = 1024;


lt_status fail(lt_ctx* ctx, lt_status code, const std::string& msg);
size_t dtype_size(uint8_t dtype);
const char* dtype_name(uint8_t dtype);
const char* op_name(uint16_t op);
int64_t numel(const int64_t* dims, int rank);

// destroys the events and graphs that a plan owns on the device (lt_barrier.cpp)
void destroy_device_objects(Plan* plan);

// views (lt_api.cpp): bring every live view up to date with its base
lt_status refresh_views(lt_ctx* ctx);

// barrier pieces (lt_barrier.cpp)
struct Cut {
  std::vector<Handle*> roots;
  std::vector<int32_t> order;       // canonical position -> node index
  std::vector<int32_t> index_of;    // node index -> canonical position (-1: not in the cut)
  std::vector<uint32_t> donors;     // per root: donated parameter ordinal or 0xFFFFFFFF
  std::vector<int32_t> param_nodes, scalar_nodes;   // ordinal -> node index
};
void collect_cut(lt_ctx* ctx, Cut* cut);
void serialise_cut(lt_ctx* ctx, Cut* cut, std::vector<uint8_t>* out);
uint64_t fnv1a64(const uint8_t* p, size_t n);

// lowering (lt_lower.cpp): returns nullptr and sets ctx->err / *status on failure
std::unique_ptr<Plan> lower(lt_ctx* ctx, const Cut& cut, lt_status* status);
// stream schedule of a lowered plan (lt_schedule.cpp)
void schedule_streams(Plan* plan);
// 32 x 32 tiles of a one-launch small contraction whose workgroups share tiles (they exchange partial
// tiles through the reduction scratch and take tickets); 0 for every other launch
uint64_t gemm_shared_tiles(const Launch& l);

}  // namespace lt
#endif  // LT_CORE_H_
