// fs_internal.h - host-side data structures of the stitched-kernel executor.
#ifndef FS_INTERNAL_H_
#define FS_INTERNAL_H_

#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <array>
#include <map>
#include <set>
#include <mutex>
#include <string>
#include <vector>

#include "fs.h"

namespace fs {

// ---- errors --------------------------------------------------------------------------------
void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));
std::string& error_buffer();
#define FS_FAIL(status, ...)       \
  do {                             \
    ::fs::set_error(__VA_ARGS__);  \
    return (status);               \
  } while (0)

// ---- device figures --------------------------------------------------------------------------
// What the planner needs to know about the machine.  Read once per process from the current
// device; the published MI355X figures stand in when planning runs without one (kernels are
// compiled ahead of time on machines that have no GPU).
struct DeviceLimits {
  int cus = 256;                      // compute units (8 XCDs x 32)
  int lds_per_workgroup = 163840;     // LDS bytes one workgroup may allocate (all of a compute unit's 160 KB)
  int64_t resident_lanes = 524288;    // lanes resident on the whole device (2048 per compute unit)
  int64_t l2_bytes = 4ll << 20;       // L2 of one XCD
  bool from_device = false;
};
const DeviceLimits& device_limits();

// ---- graph -----------------------------------------------------------------------------------
inline bool op_is_view(int op) { return op == FS_RESHAPE || op == FS_BITCAST; }  // the operand's bytes under another shape
inline bool op_is_free(int op) {  // never materialised, never a launch: inlined into consumers
  return op == FS_INPUT || op == FS_CONST || op == FS_BCAST_ROWVEC || op == FS_BCAST_COLVEC || op_is_view(op);
}
inline bool op_is_unary(int op) { return op >= FS_NEG && op <= FS_CONVERT; }
inline bool op_is_binary(int op) { return op >= FS_ADD && op <= FS_MIN; }
inline bool op_is_approx(int op) {  // not bit-reproducible against a correctly rounded reference
  return op == FS_EXP || op == FS_LOG || op == FS_TANH || op == FS_SIGMOID || op == FS_RSQRT || op == FS_RCP ||
         op == FS_GELU_TANH;
}
int op_arity(int op);
const char* op_name(int op);
inline int dtype_size(int dt) { return dt == FS_F32 ? 4 : dt == FS_BF16 ? 2 : 1; }

struct Graph {
  std::vector<fs_node> nodes;
  std::vector<int> outputs;              // plan outputs (node ids)
  std::vector<int> input_ids;            // FS_INPUT nodes in id order
  std::vector<int> input_index;          // node id -> index into inputs[] or -1
  std::vector<int> output_index;         // node id -> index into outputs[] or -1
  std::vector<std::vector<int>> users;   // direct users of each node
  std::vector<char> exact;               // node feeds a predicate: its bits must be reproducible (no contraction)
  std::vector<int> root_of;              // the node whose buffer a node's bytes live in: itself, or what its chain of views starts from
  std::vector<int> family_output;        // root -> index of the plan output (the root itself or a view of it) whose buffer holds it, or -1
  // flat_in[node][k]: operand k is a tensor in memory whose row-major element sequence the node reads under its own
  // [rows, cols] (set by absorb_views: an elementwise region re-labelled with the shape on the other side of a view)
  std::vector<std::array<unsigned char, 3>> flat_in;
  int views_absorbed = 0;                // views that absorb_views made transparent
  int n() const { return (int)nodes.size(); }
};

// Validates desc and fills g.  (Section 2.1: the op classes; this is the receiving end of a fusion plan.)
fs_status build_graph(const fs_graph_desc* desc, Graph* g);

// ---- groups ----------------------------------------------------------------------------------
// How a tensor relates to its group's work space [R,C] (Section 4.1: the schedule is defined on
// the root's output shape; operands get theirs by back-propagation, Section 4.2).
enum Kind : int {
  KIND_NONE = 0,
  KIND_FULL = 1,  // [R,C]: E elements per lane, in VGPRs
  KIND_COLV = 2,  // [R,1]: one value per row, replicated in the row's lanes
  KIND_ROWV = 3,  // [1,C]: one value per column, the lane's slice loaded once per workgroup
  KIND_PART = 4   // an operand of a concat member: covers part of the work space, read through that member's two-source load
};

// Bounds of one fused group.  kMaxGroupTensors: pointers in a kernel's argument block (8 bytes each; the block and the
// kernel's scalar registers hold them all, and a body that touches more tensors than this is bound by their traffic,
// not by launches).  kMaxGroupMembers: compute nodes in one generated body (code size and compile time grow with it;
// the 200-node benchmark DAG's largest group has 46).
constexpr int kMaxGroupTensors = 48;
constexpr int kMaxGroupMembers = 96;

struct ExtTensor {
  int node = -1;
  Kind kind = KIND_NONE;
  int dtype = 0;
  bool transposed = false;  // output only: stored as [C,R]
  bool deferred = false;    // output only: column-reduction result written by the last workgroup
  bool streaming = false;   // large tensor touched once: non-temporal loads / stores
  int arg = -1;             // index into the kernel's pointer table
};

struct Schedule {
  int V = 4;        // elements per vector access
  int NV = 0;       // vectors per row = C / V
  int L = 64;       // lanes per row (power of two)
  int NVL = 1;      // vectors per lane = ceil(NV / L)
  int E = 4;        // elements per lane = NVL * V
  int WG = 256;     // workgroup size
  int G = 4;        // row-groups per workgroup = WG / L
  int U = 1;        // row tiles per loop trip in looping kernels (loads of all U issued first)
  int CT = 1;       // column tiles per row (> 1 only for groups without reductions: very long rows)
  int n_iters = 0;  // ceil(R * CT / G): loop trips over the whole grid
  int grid = 0;     // workgroups (`blocks` of Section 4.1)
  bool ragged = false;  // some lane's vector index can fall beyond NV
  int lds_bytes = 0;    // static LDS of the generated kernel
  int lds_planned = 0;  // ... as planned before code generation (an upper bound of lds_bytes)
  int fan_in = 32;  // column-reduction tree fan-in
  int fold_piece = 0;  // columns that pass through the in-workgroup fold area at a time
  bool stage_rowv = false;  // [1,C] inputs are staged once per workgroup in LDS
  // Looping workgroups that stage their [1,C] operands before the loop ask for the first trip's rows before the staging
  // and for the next trip's at the end of a trip (the same registers: the rows are dead by then), so the first memory
  // round trip overlaps the staging.  Rows of one wavefront and a handful of trips only.
  bool rotate_loop = false;
  bool tile_transpose = false;  // transposed roots leave through a padded LDS tile
  // Reduction-free groups with transposed roots over wide rows: 2-D tiles.  A workgroup owns G
  // consecutive rows of one column tile of NVL*L*V columns (unit = column tile fastest), so both
  // the reads and the transposed writes are runs of consecutive elements.
  bool tiled_transpose = false;
  // Order in which the workgroups walk those tiles.  Workgroups that run at the same time should
  // cover a block of the tensor that is wide both ways: a band of `tt_col_band` column tiles is
  // walked row tile by row tile (column tiles fastest inside the band) before the next band starts,
  // so the few hundred tiles in flight read runs of tt_col_band tiles' width and write, between
  // them, long runs of every transposed row they touch.  0 = rows of tiles in plain order (the
  // bands would be as wide as the tensor anyway).
  int tt_col_band = 0;
  // A few very long rows (few_long_rows) leave most CUs idle with one workgroup per row.  When all
  // row reductions are in the first stage and every other result is an [R,1] value or needs no
  // reduction result (split_rows), each row is cut into S segments of CPS chunks, one workgroup per
  // segment, and the segments' partial results are folded across workgroups with the ticket scheme
  // of the column reductions.
  int min_waves = 0;  // amdgpu_waves_per_eu attribute of the kernel, 0 = none
  bool few_long_rows = false;
  bool split_rows = false;
  int S = 1, CPS = 0;
  // Rows too long for the registers of one workgroup, with row reductions: the row is walked in CT
  // column chunks once per stage, and each stage recomputes the elementwise values it needs from
  // the inputs instead of keeping them (space traded for recomputation, Section 5.1.2).
  bool chunked = false;
  // ... optionally with the first RESV vectors of the row resident in registers for the whole
  // body (64 elements per lane), so only the rest is walked, NVLC vectors per lane per chunk.
  bool resident = false;
  int NVLC = 0, RESV = 0;
  bool ragged_chunks = false;
  // ... and with the first `stage_chunks` chunks of every value that more than one pass needs and that got an LDS
  // slot (GroupPlan::stage_slots) kept in LDS in the value's own dtype: written by the first pass that loads or
  // computes it, read back by the later ones, so the row crosses HBM once instead of once per stage (Section 5.1.1:
  // values needed by several loops of the kernel are the ones shared memory is allocated for).  stage_avail: LDS
  // bytes the planner leaves for it.
  int stage_avail = 0, stage_chunks = 0;
  // Column reductions over rows too wide for one workgroup: CT column tiles, each folded by its own
  // RB = grid / CT workgroups (tile = block % CT).  Strides of one tile's scratch in the workspace:
  bool col_tiled = false;
  int RB = 0;
  size_t part_stride_floats = 0;
  int ticket_stride = 0;
};

// One LDS buffer of a kernel that walks its rows in chunks (Section 5.1): it holds the first stage_chunks chunks of one row
// value at a time, stored in that value's dtype.  `owners` are the values that occupy it one after the other (space
// sharing, Section 5.1.3): each later owner dominates its predecessor in the group's data flow seen from the roots, so
// once it exists nothing needs the predecessor any more, and it overwrites it in place, lane by lane.
struct StageSlot {
  int elem_bytes = 0;
  std::vector<int> owners;
};

struct GroupPlan {
  std::vector<int> members;  // compute nodes, ascending id
  int R = 0, C = 0;          // work space
  std::map<int, Kind> kind;  // members and external tensors -> kind
  std::map<int, int> level;  // members -> stage (number of row reductions upstream)
  std::map<int, bool> tflag; // members -> lives in the transposed orientation of the work space
  std::vector<ExtTensor> ext_in, ext_out;
  std::vector<int> row_reduces;  // REDUCE_ROW members that need a cross-lane exchange
  std::vector<int> col_reduces;  // REDUCE_COL members finished by the grid-wide fold
  // chunked kernels: the LDS buffers for values that several passes over the row need (filled by generate_kernel)
  std::vector<StageSlot> stage_slots;
  std::map<int, int> stage_slot_of;             // buffered value (input or member) -> slot
  std::vector<std::pair<int, int>> stage_given_up;  // candidates that are recomputed instead (Section 5.1.2): (member, 1 = inexpensive op | 2 = expensive op)
  std::string lds_plan_text;                    // the above in words (a comment in the kernel source)
  int max_batched_reduces = 0;   // largest number of row reductions sharing one exchange
  Schedule s;
  // workspace scratch (byte offsets inside the plan workspace)
  size_t part_offset = 0, part_bytes = 0;
  size_t ticket_offset = 0;
  int n_tickets = 0;
  uint64_t min_hbm_bytes = 0;
  // generated kernel
  std::string kernel_name, source;
  std::string perf_key;  // filled on demand by fs_plan_group_perf_key
};

// Values that more than one kernel computes.  A cheap elementwise result that a later kernel needs is
// computed again there, from operands that exist in memory anyway, instead of passing through memory
// itself: group_of holds the (first) kernel of every node in launch order, extra the other kernels
// that hold a copy of it.
struct CloneInfo {
  std::vector<int> group_of;
  std::map<int, std::set<int>> extra;
  bool computed_in(int node, int grp) const {
    if (group_of[node] == grp) return true;
    auto it = extra.find(node);
    return it != extra.end() && it->second.count(grp) != 0;
  }
};

struct PlanOptions {
  uint32_t mode = FS_MODE_STITCHED;
  int lds_budget = 65536;
  bool lds_budget_given = false;  // the caller set it: rows staged in LDS stay inside it too (else they may take what the device allows)
  fs_sched_hint hint = {0, 0, 0, 0};
  bool has_hint = false;
  // How much of a row longer than 32 elements per lane may stay in registers: 2 = up to 64 elements
  // per lane (or 48 resident ones plus chunks), 1 = 32 resident ones plus chunks, 0 = chunks only.
  // Plan creation steps down while the compiled kernel spills.
  int wide_level = 2;
  int min_waves = 0;  // > 0: the kernel asks the compiler for that many wavefronts per SIMD (occupancy feedback at plan creation)
  bool layered = false;  // group with the layered planner of Section 3.2 instead of the default one
  // set once the groups are final: whether a value leaves a kernel then depends on which kernels compute it themselves
  const CloneInfo* clones = nullptr;
};

// Analyse a candidate member set: work space, kinds, stages, external tensors, schedule, LDS plan.
// Returns FS_OK, FS_ERR_UNSUPPORTED (cannot be one stitched kernel) or FS_ERR_LDS_BUDGET.
// This is the schedule-consistency check of Section 3.2 (third condition of SchdConsistent)
// together with the schedule and shared-memory planning of Sections 4 and 5.1.
fs_status analyse_group(const Graph& g, const std::vector<int>& members, const std::vector<int>& group_of,
                        int self_group, const PlanOptions& opt, GroupPlan* out);

// Assign every compute node to a group.  group_of[node] = group id or -1 for free nodes.
fs_status form_groups(const Graph& g, const fs_graph_desc* desc, const PlanOptions& opt, std::vector<int>* group_of,
                      std::vector<std::vector<int>>* groups_in_launch_order);

// After grouping: elementwise values that cross a kernel boundary are computed again by the consuming
// kernel where that moves fewer bytes (the consumer reads the producer's operands, which exist in
// memory anyway, instead of the value; the producer no longer stores it when nobody else reads it).
// Adds the copies to the consumers' member lists and records them in `clones`.
void recompute_across_kernels(const Graph& g, const PlanOptions& opt, std::vector<int>* group_of,
                              std::vector<std::vector<int>>* groups_in_launch_order, CloneInfo* clones);

// Work/Span analysis (Section 3.1): span per node, -1 for inlined and dead nodes.
void work_span(const Graph& g, std::vector<int>* span);

// Emit the HIP source of one group's kernel (Section 5.2, Algorithm 2 realised as a
// straight-line body over hand-written device building blocks).
fs_status generate_kernel(const Graph& g, GroupPlan* gp, int group_index);

// Compile `source` for gfx950 (disk-cached).  No GPU needed.
fs_status compile_kernel(const std::string& source, const std::string& name, std::vector<char>* code);

const char* device_header_source();  // text of fs_device.h, embedded at build time

// ---- schedule tuning and the performance library (Sections 4.3, 4.4) ---------------------------
// Schedules worth trying for a group besides the one the analytic rules picked (`base`): the
// neighbourhood of the base schedule in lanes per row, workgroup size and grid.
std::vector<fs_sched_hint> candidate_hints(const GroupPlan& base);
// Library key of one kernel under one launch, lookups and inserts (persistent, see fs_perflib.cpp).
std::string perf_key(const GroupPlan& gp);
size_t perflib_size();
bool perflib_lookup(const std::string& key, double* usec);
bool perflib_insert(const std::string& key, double usec, const std::string& note);
// Re-plans `members` under every candidate schedule, looks the kernels up in the library and
// replaces *gp by the fastest recorded one.  Returns true when *gp changed.
bool choose_from_library(const Graph& g, const std::vector<int>& members, const std::vector<int>& group_of, int self_group,
                         const PlanOptions& opt, GroupPlan* gp);

}  // namespace fs

struct fs_plan {
  fs::Graph graph;
  fs::PlanOptions opt;
  std::vector<int> group_of;
  fs::CloneInfo clones;               // values computed by more than one kernel (opt.clones points here)
  std::vector<fs::GroupPlan> groups;  // in launch order
  // workspace layout
  std::map<int, size_t> ws_tensor_offset;  // node materialised in the workspace -> byte offset
  size_t ticket_bytes = 0;                 // tickets live at the start of the workspace
  size_t workspace_bytes = 0;
  uint64_t min_hbm_bytes = 0, launched_hbm_bytes = 0, unfused_hbm_bytes = 0;
  std::vector<char> code;  // one gfx950 code object holding every kernel of the plan
  // per-device loaded code
  struct Loaded {
    std::vector<void*> modules;    // hipModule_t per group
    std::vector<void*> functions;  // hipFunction_t per group
  };
  std::mutex mu;
  std::map<int, Loaded> loaded;
};

#endif  // FS_INTERNAL_H_
