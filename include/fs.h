/*
 * fs.h — C ABI of the stitched-kernel executor for AMD MI355X (gfx950).
 *
 * The library executes a *fusion plan*: a DAG of typed, fine-grained, memory-bound
 * tensor ops (elementwise, broadcast, transpose, row/column reduction) on 2-D
 * row-major tensors.  Each fused group of the plan runs as ONE stitched GPU kernel:
 * elementwise producers are composed into their consumers in registers (the paper's
 * "thread composition", Section 1 / Figure 2(a)), and ops that need a different
 * parallel loop - reductions and the ops that consume a reduction result - are
 * composed through on-chip shared memory inside the same kernel ("block
 * composition" / stitching, Section 1 / Figure 2(b), Section 5.2 / Algorithm 2).
 *
 * Conventions
 *   - Every function returns fs_status.  Nothing throws or aborts across the ABI.
 *     fs_last_error() returns a thread-local, human-readable message for the last
 *     non-FS_OK status returned on the calling thread.
 *   - "host" pointers are ordinary CPU memory; "device" pointers are HIP device
 *     memory of the current device.  The caller owns every device buffer (inputs,
 *     outputs, workspace) and the stream; the library owns only fs_plan objects
 *     (host memory plus loaded code objects).
 *   - Tensors are dense, contiguous, row-major [rows, cols].  FS_F32 is IEEE
 *     binary32, FS_BF16 is bfloat16 (raw uint16 bits), FS_U8 is a predicate byte
 *     holding 0 or 1.  Every device tensor pointer must be 16-byte aligned.
 *   - A plan is immutable after fs_plan_create.  fs_plan_run may be called
 *     concurrently on one plan only with distinct workspaces.
 *
 * Environment (all optional)
 *   FS_KERNEL_CACHE        directory of the compiled-kernel cache (default: kcache/
 *                          beside the shared library); kernels are keyed by source,
 *                          compile options and compiler version
 *   FS_PERF_LIBRARY        file of the performance library (see fs_plan_tune)
 *   FS_LOG_PLAN            when set, plan creation reports on stderr every kernel it
 *                          plans again because the compiled code spills registers or
 *                          sits just above an occupancy step, and the registers and
 *                          scratch bytes of every kernel it ends up with
 *   FS_DUMP_FAILED_SOURCE  file that receives the generated source when its
 *                          compilation fails
 */
#ifndef FS_H_
#define FS_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FS_ABI_VERSION 2u

typedef struct fs_plan fs_plan; /* opaque */

typedef enum {
  FS_OK = 0,
  FS_ERR_INVALID_ARG = 1, /* null pointer, bad abi_version, misaligned device pointer ... */
  FS_ERR_BAD_GRAPH = 2,   /* operand id >= node id (cycle / dangling id), bad arity, bad output id */
  FS_ERR_SHAPE = 3,       /* operand / result shapes inconsistent with the opcode */
  FS_ERR_DTYPE = 4,       /* operand / result dtypes inconsistent with the opcode */
  FS_ERR_UNSUPPORTED = 5, /* valid graph, but a caller-given grouping cannot be one stitched kernel */
  FS_ERR_LDS_BUDGET = 6,  /* a caller-given group needs more LDS than lds_budget_bytes */
  FS_ERR_WORKSPACE = 7,   /* workspace null, misaligned or smaller than fs_plan_workspace_bytes */
  FS_ERR_COMPILE = 8,     /* run-time compilation of a group's kernel failed */
  FS_ERR_HIP = 9,         /* a HIP runtime call failed (message holds the HIP error string) */
  FS_ERR_OOM = 10         /* host allocation failed */
} fs_status;

typedef enum { FS_F32 = 0, FS_BF16 = 1, FS_U8 = 2 } fs_dtype;

/*
 * Opcodes.  The four op classes of the paper's problem statement (Section 2.1):
 * elementwise, shape modulation (the two broadcasts, Transpose, Reshape / Bitcast; Concat,
 * which Section 6.3 names), Reduction (sum/max/min/mean, Section 1) and - deliberately
 * absent - BatchMatMul.
 *
 * Tensors of any rank enter the plan as [rows, cols] = [product of the leading dims, product
 * of the trailing dims] of their dense row-major layout; FS_RESHAPE moves that split (or
 * regroups the element sequence in any other way that keeps the element count).  In the
 * schedule terms of Section 4.1 / Table 1 this is the split_dim of a Row schedule, which a Reshape
 * passes through when the split dimension survives.  Here a Reshape / Bitcast next to an elementwise
 * region (no broadcast, no reduction, no transpose on that side) is passed through: the region is
 * computed under the shape of the other side and shares its kernel.  Between two computations that
 * both have a row structure it is a zero-cost view at a boundary between kernels: producer and
 * consumer address the same bytes.
 */
typedef enum {
  FS_INPUT = 0,  /* external tensor; the k-th FS_INPUT node (in id order) is inputs[k] of fs_plan_run */
  FS_CONST = 1,  /* tensor of the declared shape filled with attr_f; never materialised */
  /* unary elementwise, shape and arity (1): out[i,j] = f(in0[i,j]) */
  FS_NEG = 2,
  FS_ABS = 3,
  FS_EXP = 4,
  FS_LOG = 5,
  FS_TANH = 6,
  FS_SIGMOID = 7,   /* 1 / (1 + exp(-x)) */
  FS_SQRT = 8,
  FS_RSQRT = 9,     /* 1 / sqrt(x) */
  FS_RCP = 10,      /* 1 / x */
  FS_GELU_TANH = 11,/* 0.5 x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) */
  FS_CONVERT = 12,  /* value-preserving change of dtype (round to nearest even when narrowing) */
  /* binary elementwise, arity 2, all three shapes equal */
  FS_ADD = 13,
  FS_SUB = 14,
  FS_MUL = 15,
  FS_DIV = 16,
  FS_MAX = 17,      /* IEEE maxNum */
  FS_MIN = 18,      /* IEEE minNum */
  /* predicates */
  FS_CMP = 19,      /* arity 2, result FS_U8: attr_i is an fs_cmp */
  FS_SELECT = 20,   /* arity 3: in0 is FS_U8; out = in0 ? in1 : in2 (bits of the chosen operand) */
  /* shape modulation; broadcasts are never materialised (the paper inlines such
   * trivial ops by thread composition, Section 4.3) */
  FS_BCAST_ROWVEC = 21, /* in0 [1,C] -> out [R,C]: out[i,j] = in0[0,j] */
  FS_BCAST_COLVEC = 22, /* in0 [R,1] -> out [R,C]: out[i,j] = in0[i,0] */
  FS_TRANSPOSE = 23,    /* in0 [R,C] -> out [C,R]: out[j,i] = in0[i,j] */
  /* reductions; attr_i is an fs_reduce_kind */
  FS_REDUCE_ROW = 24,   /* in0 [R,C] -> out [R,1], reduces over the columns of each row */
  FS_REDUCE_COL = 25,   /* in0 [R,C] -> out [1,C], reduces over the rows of each column */
  /* more shape modulation.  RESHAPE / BITCAST: out.flat[i] = in0.flat[i], same dtype, rows*cols unchanged;
   * never materialised and never a launch: the result is a view of in0's buffer (in0: an FS_INPUT, a compute
   * node or another view; not a broadcast or constant).  The two names denote the same map: in the source
   * framework a Bitcast is a Reshape known not to move data, and with dense row-major tensors every Reshape is.
   * As a plan output a view makes its producer write straight into the caller's buffer; a view of an FS_INPUT
   * cannot be a plan output (nothing would be computed), nor can two members of one view family both be. */
  FS_RESHAPE = 26,
  FS_BITCAST = 27,
  /* CONCAT: attr_i is an fs_concat_axis; in0 and in1 have the result's dtype.  FS_CONCAT_COLS: in0 [R,C0],
   * in1 [R,C1] -> out [R,C0+C1], row i = in0's row i followed by in1's; FS_CONCAT_ROWS: in0 [R0,C], in1 [R1,C]
   * -> out [R0+R1,C].  The operands are read from memory by the kernel that holds the concat (a consumer
   * fused with it reads two tensors as one row and nothing is copied); an operand computed by the same group
   * is materialised first. */
  FS_CONCAT = 28,
  FS_NUM_OPCODES = 29
} fs_opcode;

typedef enum { FS_CMP_GT = 0, FS_CMP_GE = 1, FS_CMP_LT = 2, FS_CMP_LE = 3, FS_CMP_EQ = 4, FS_CMP_NE = 5 } fs_cmp;
typedef enum { FS_RED_SUM = 0, FS_RED_MAX = 1, FS_RED_MIN = 2, FS_RED_MEAN = 3 } fs_reduce_kind;
typedef enum { FS_CONCAT_ROWS = 0, FS_CONCAT_COLS = 1 } fs_concat_axis;

/*
 * One node of the DAG.  The node id is its index in fs_graph_desc.nodes, and the
 * array must be topologically ordered: every in[k] < id.  rows/cols/dtype declare
 * the node's OUTPUT tensor and are checked against the opcode's rule.
 * Arithmetic is done in fp32 and the value is rounded once to the node's dtype, so
 * a FS_BF16 node holds a bf16-representable value even when it never leaves registers.
 */
typedef struct {
  int32_t opcode; /* fs_opcode */
  int32_t dtype;  /* fs_dtype of the result */
  int32_t rows;
  int32_t cols;
  int32_t num_in; /* 0..3 */
  int32_t in[3];  /* operand node ids; unused entries ignored */
  int32_t attr_i; /* fs_cmp for FS_CMP, fs_reduce_kind for FS_REDUCE_*, fs_concat_axis for FS_CONCAT, else 0 */
  float attr_f;   /* value of FS_CONST, else 0 */
} fs_node;

/* Execution mode. */
#define FS_MODE_STITCHED 0u /* fused groups, one kernel launch per group */
#define FS_MODE_UNFUSED 1u  /* one launch per compute node, every intermediate in HBM; the
                               comparison executor for launch count and HBM traffic
                               (the role of the per-op baseline in Section 6.3) */
#define FS_MODE_LAYERED 4u /* flag, may be or-ed in: form groups with the layered planner exactly as
                              Section 3.2 describes it (Work/Span layers, intra-layer ElementwiseFusion,
                              Algorithm 1 from every fusion root) instead of the default planner, which
                              visits nodes in the same order but joins a node to any consistent user
                              group and then merges sibling groups across layers */
#define FS_MODE_NO_PERFLIB 2u /* flag, may be or-ed in: ignore the performance library and keep the
                                 schedules of the analytic rules */

/*
 * Optional schedule override, applied to every group it is legal for (0 = let the
 * scheduler decide).  In the paper's terms (Section 4.1) every group runs a Row
 * schedule with split_dim = 0: `max_workgroups` bounds `blocks`; lanes_per_row
 * says how many lanes cooperate on one row (a power of two, 1..1024, the analogue
 * of reduce_warps in Section 4.4); wg_threads is the workgroup size (multiple of 64,
 * <= 1024).  max_workgroups = 1 gives the always-valid single-block schedule of
 * Section 4.3.  For a group over a handful of very long rows that are split over
 * workgroups, max_workgroups is the number of row segments in all (lanes_per_row and
 * wg_threads are fixed at 256 there).
 */
typedef struct {
  int32_t lanes_per_row;
  int32_t wg_threads;
  int32_t max_workgroups;
  int32_t tiles_per_trip; /* looping kernels: row tiles handled per loop trip (1..4), the loads of all of
                             them issued before the first is used */
} fs_sched_hint;

typedef struct {
  uint32_t abi_version;          /* FS_ABI_VERSION */
  int32_t num_nodes;
  const fs_node* nodes;          /* host; copied by fs_plan_create */
  int32_t num_outputs;
  const int32_t* outputs;        /* host; node ids that are plan outputs (not INPUT/CONST/BCAST_*; a RESHAPE/BITCAST only
                                    as a view of a computed value), distinct */
  const int32_t* group_of_node;  /* host; NULL => the library groups greedily.  Else one group id >= 0 per
                                    node (ignored for INPUT/CONST/BCAST_* nodes, which are inlined into
                                    each consumer): the caller's fusion plan.  Ignored in FS_MODE_UNFUSED. */
  uint32_t mode;                 /* FS_MODE_* */
  int32_t lds_budget_bytes;      /* per-workgroup LDS limit for one group; at most what fs_device_limits reports for
                                    one workgroup.  0 => the library's own choice: 65536 (of 160 KB per CU) for most
                                    kernels; up to half a CU's LDS for the transpose tile of large 2-byte tensors; all
                                    a workgroup may use for rows walked in chunks with their head kept in LDS (one
                                    workgroup per CU runs such a kernel).  A value given here binds all of them. */
  const fs_sched_hint* hint;     /* host; may be NULL */
} fs_graph_desc;

/* What the scheduler decided for one group (one kernel launch). */
typedef struct {
  int32_t num_nodes;        /* compute nodes executed by this kernel */
  int32_t dom_rows;         /* the group's work space [dom_rows, dom_cols] (Section 4.1: output shape of the root) */
  int32_t dom_cols;
  int32_t lanes_per_row;    /* lanes that share one row */
  int32_t vec_elems;        /* elements per vector memory access (16 bytes when shapes allow) */
  int32_t elems_per_lane;   /* columns held by one lane for each [R,C] value */
  int32_t wg_threads;       /* workgroup size */
  int32_t rows_per_iter;    /* rows a workgroup processes per loop trip = wg_threads / lanes_per_row */
  int32_t grid;             /* workgroups launched = `blocks` of Section 4.1 */
  int32_t lds_bytes;        /* static LDS the kernel uses */
  int32_t num_row_reduces;  /* stitched row reductions */
  int32_t num_col_reduces;  /* two-stage column reductions */
  int32_t num_ext_inputs;   /* tensors read from HBM */
  int32_t num_ext_outputs;  /* tensors written to HBM */
  uint64_t min_hbm_bytes;   /* external inputs once + outputs once */
  uint64_t scratch_bytes;   /* column-reduction partials + tickets inside the plan workspace */
} fs_group_info;

/*
 * fs_plan_create: validate the DAG (ids, arity, shapes, dtypes), form groups
 * (given or greedy; a cut-down of the paper's Algorithm 1 with its SchdConsistent
 * checks, Section 3.2), pick each group's schedule (Section 4) and LDS plan
 * (Section 5.1), generate and compile each group's kernel for gfx950
 * (Section 5.2 / Algorithm 2).  Host-only: needs no GPU.  desc and everything it points
 * to may be freed after the call.  *out_plan is set only on FS_OK.
 */
fs_status fs_plan_create(const fs_graph_desc* desc, fs_plan** out_plan);

/*
 * fs_plan_destroy: frees the plan and unloads its code objects from every device it was loaded
 * on (the end of the life of a fused computation's compiled form, Section 5.2).  NULL is FS_OK.
 * No launch of the plan may still be in flight.
 */
fs_status fs_plan_destroy(fs_plan* plan);

/*
 * fs_plan_workspace_bytes: bytes of device workspace fs_plan_run needs.  The workspace is the
 * off-chip side of the plan's memory planning (Section 5.1 plans the on-chip side per kernel): tensors
 * that cross group boundaries (what fusion could not keep on chip), the per-workgroup partials of
 * two-stage column reductions and their ticket counters.  May be 0.
 */
fs_status fs_plan_workspace_bytes(const fs_plan* plan, size_t* bytes);

/*
 * fs_plan_load: load the plan's code objects onto the CURRENT device now (hipModuleLoadData; it
 * allocates device memory for the code and may synchronise).  fs_plan_run does this by itself on
 * its first call on a device; a caller that wants the first fs_plan_run to be free of allocation -
 * stream capture, a serving loop - calls fs_plan_load (or makes one warm fs_plan_run) beforehand.
 * Idempotent per device.  FS_ERR_HIP without a usable device.
 */
fs_status fs_plan_load(fs_plan* plan);

/*
 * fs_plan_run: execute the fusion plan - ONE kernel launch per fused computation (Section 1: the
 * ops of a fused computation are composed inside a single kernel, by thread composition in
 * registers and by block composition through on-chip memory; Section 2.2: the stitched kernel) -
 * enqueued in dependence order on `hip_stream` (a hipStream_t; NULL = the null stream) of the
 * current device.  Asynchronous.  Once the plan is loaded on the device (fs_plan_load, or an
 * earlier fs_plan_run) it makes no allocation, no synchronisation and no host<->device copy.
 *   inputs   host array of device pointers, one per FS_INPUT node in id order; caller-owned,
 *            16-byte aligned, dense row-major; read only
 *   outputs  host array of device pointers, one per entry of desc.outputs, same order; caller-
 *            owned, 16-byte aligned; every element is overwritten
 *   workspace / workspace_bytes  caller-owned device buffer of >= fs_plan_workspace_bytes bytes,
 *            256-byte aligned; may be NULL when 0 bytes are needed.  The ticket counters inside
 *            it must be zero before the FIRST run on that buffer (fs_plan_workspace_init does
 *            it); every run leaves them zero again.  A run that is killed half-way may leave
 *            them non-zero: initialise again (fs_plan_workspace_check tells).
 * Errors: FS_ERR_INVALID_ARG for a NULL or misaligned pointer and when an output's byte range
 * overlaps an input's, another output's or the workspace's, or an input's overlaps the
 * workspace's (inputs may alias each other: they are only read); FS_ERR_WORKSPACE for a NULL,
 * misaligned or undersized workspace; FS_ERR_HIP when loading or a launch fails.  Nothing has
 * been enqueued when the status is FS_ERR_INVALID_ARG or FS_ERR_WORKSPACE.
 */
fs_status fs_plan_run(fs_plan* plan, const void* const* inputs, void* const* outputs,
                      void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fs_plan_run_static: fs_plan_run for callers that cannot allocate or provide a workspace - code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The workspace is
 * a static device array inside the library, FS_STATIC_SCRATCH_BYTES per GPU (held by every GPU the
 * library runs on until the process ends); the caller still passes inputs and outputs.  The call
 * itself makes no allocation of any kind: the plan must already be loaded on the current device
 * (fs_plan_load, which also resolves the array's address on that device; FS_ERR_INVALID_ARG
 * otherwise), and a plan whose fs_plan_workspace_bytes exceeds FS_STATIC_SCRATCH_BYTES is refused
 * with FS_ERR_WORKSPACE.  All calls on one GPU share the one array, which keeps the previous
 * call's contents: each call first zeroes its plan's ticket counters with a fill kernel on
 * `hip_stream` (a kernel, not a memset), then enqueues the plan's launches.  Calls that overlap
 * in time on one GPU - different streams, or different plans - race on the array: serialise them.
 * Results are those of fs_plan_run, bit for bit.  Other errors as for fs_plan_run.
 */
#define FS_STATIC_SCRATCH_BYTES (8u << 20)
fs_status fs_plan_run_static(fs_plan* plan, const void* const* inputs, void* const* outputs, void* hip_stream);

/* Enqueue a fill kernel on `hip_stream` that zeroes the ticket counters of a fresh workspace
 * (a kernel, not a memset: it may be recorded into a HIP graph). */
fs_status fs_plan_workspace_init(fs_plan* plan, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fs_plan_workspace_check: a debugging aid for the one precondition fs_plan_run cannot see from
 * the host.  SYNCHRONISES `hip_stream`, copies the ticket counters back and returns
 * FS_ERR_WORKSPACE when any of them is non-zero (a workspace that was never initialised, was
 * recycled from other use, or belongs to a run that was killed inside a fold: with such tickets
 * the last-arriver test of the grid-wide fold never fires and column-reduction outputs are not
 * written).  FS_OK for a plan without tickets.
 */
fs_status fs_plan_workspace_check(fs_plan* plan, const void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * fs_plan_stats: plan-level figures for the metric.  num_groups = fused computations;
 * num_launches = kernel launches per run (equal to num_groups: one launch per group).  Their
 * ratio between a stitched and an unfused plan of the same DAG is the paper's fusion ratio
 * (Section 6.3: kernels after fusion / kernels of the baseline).  min_hbm_bytes = every plan
 * input read once + every plan output written once (the memory footprint fusion aims at,
 * Section 4.1); unfused_hbm_bytes = what one launch per compute node moves for this DAG, every
 * intermediate written and read back, whatever mode this plan was created in (broadcasts and
 * constants are never materialised, Section 4.3).  Any out pointer may be NULL.
 */
fs_status fs_plan_stats(const fs_plan* plan, int32_t* num_groups, int32_t* num_launches,
                        uint64_t* min_hbm_bytes, uint64_t* unfused_hbm_bytes);

/* Bytes THIS plan's launches move: the sum over its groups of external inputs + outputs (equals
 * min_hbm_bytes for a single-group plan, unfused_hbm_bytes for an unfused one). */
fs_status fs_plan_launched_hbm_bytes(const fs_plan* plan, uint64_t* bytes);

/*
 * The device figures the planner works with: compute units, LDS bytes one workgroup may use,
 * lanes resident on the whole device, last-level cache bytes.  Read from the current device once
 * per process (hipDeviceGetAttribute); without a device (planning ahead of time on a build
 * machine) the published MI355X figures stand in and *from_device is 0.  Any out pointer may be NULL.
 */
fs_status fs_device_limits(int32_t* compute_units, int32_t* lds_bytes_per_workgroup, int32_t* resident_lanes,
                           int64_t* l2_bytes, int32_t* from_device);

fs_status fs_plan_group_info(const fs_plan* plan, int32_t group, fs_group_info* out_info);

/* The group each node was assigned to (-1 for INPUT/CONST/BCAST_*). out has room for num_nodes entries.
 * In the library's own plans an elementwise value that a later kernel needs may be computed by that kernel
 * as well (from operands that are in memory anyway) instead of being stored and read back: this reports the
 * first kernel that computes the node, and fs_group_info's num_nodes counts such copies in each kernel. */
fs_status fs_plan_node_groups(const fs_plan* plan, int32_t* out, int32_t num_nodes);

/* Work/Span analysis (Section 3.1): the span of every node: 0 for a node no live node consumes,
 * else 1 + the largest span of its users; -1 for INPUT/CONST/BCAST_* and dead nodes.  Nodes of
 * equal span are one layer.  out has room for num_nodes entries. */
fs_status fs_plan_node_spans(const fs_plan* plan, int32_t* out, int32_t num_nodes);

/* The generated HIP source of one group's kernel (owned by the plan; valid until destroy). */
fs_status fs_plan_group_source(const fs_plan* plan, int32_t group, const char** out_src);

/* Name of the kernel symbol of one group (for matching profiler output). */
fs_status fs_plan_group_kernel_name(const fs_plan* plan, int32_t group, const char** out_name);

/*
 * Schedule tuning with the performance library (Sections 4.3 and 4.4).
 *
 * The library is a persistent key-value store of measured kernel times: key = one generated
 * kernel (its structure and every schedule constant: lanes per row, elements per lane,
 * workgroup size) under one launch (rows, loop trips, grid); value = microseconds.  It lives
 * in the text file named by the environment variable FS_PERF_LIBRARY, else in perflib.tsv beside
 * the shared library.  fs_plan_create consults it for every group unless the caller passes a
 * schedule hint or FS_MODE_NO_PERFLIB: it enumerates the group's candidate schedules, looks
 * each candidate's kernel up and keeps the fastest recorded one.
 *
 * fs_plan_tune is the measure-on-miss half: for every group of `plan`, in launch order, it
 * builds each candidate schedule's kernel, and for every key the library does not hold yet it
 * runs that kernel on the caller's buffers `reps` times (HIP events on `hip_stream`, the
 * last-level cache flushed before each timed launch when the group moves more than 1 MiB),
 * and inserts the median.  It does not change `plan`: create the plan again to use what was
 * learned.  Unlike fs_plan_run it SYNCHRONISES and ALLOCATES (private scratch for the
 * candidates' partials and a flush buffer, freed before it returns); the outputs and the
 * workspace hold the results of a normal run afterwards.  inputs / outputs / workspace as for
 * fs_plan_run.  reps <= 0 means 9.  report may be NULL.
 */
typedef struct {
  int32_t groups;           /* groups visited */
  int32_t candidates;       /* candidate kernels considered (the current schedules included) */
  int32_t measured;         /* of those, measured now and inserted */
  int32_t hits;             /* of those, already in the library */
  int32_t improvable;       /* groups for which some candidate is recorded faster than the current schedule */
  int32_t reserved;
  double current_usec;      /* sum over groups of the recorded time of the plan's current schedules */
  double best_usec;         /* sum over groups of the fastest recorded candidate */
} fs_tune_report;

/* The performance-library key of one group's kernel under its launch (owned by the plan). */
fs_status fs_plan_group_perf_key(const fs_plan* plan, int32_t group, const char** out_key);

fs_status fs_plan_tune(fs_plan* plan, const void* const* inputs, void* const* outputs, void* workspace,
                       size_t workspace_bytes, void* hip_stream, int32_t reps, fs_tune_report* report);

/*
 * fs_copy_probe: a plain streaming copy of `bytes` bytes (multiple of 16) from src
 * to dst (both device, 16-byte aligned) with 128-bit accesses, enqueued on
 * `hip_stream`.  It exists to measure the achievable HBM streaming rate of the
 * device (the practical ceiling under the 8 TB/s datasheet peak) and to calibrate
 * profiler byte counters against a kernel of known traffic.
 */
fs_status fs_copy_probe(const void* src, void* dst, size_t bytes, void* hip_stream);

/*
 * fs_copy_probe_shape: the same copy in a chosen launch shape - `vectors_in_flight` (1, 2, 4 or 8)
 * 16-byte vectors per lane per loop trip, `workgroups` workgroups of 256 lanes that loop with a grid
 * stride (0 = one trip per workgroup) - for finding what the fastest plain copy of a given size
 * reaches on the device, i.e. what a kernel that moves that many bytes can be held against.
 */
fs_status fs_copy_probe_shape(const void* src, void* dst, size_t bytes, int32_t vectors_in_flight, int32_t workgroups,
                              void* hip_stream);

/*
 * fs_alu_probe: `workgroups` workgroups of 256 lanes, each lane running 8 independent chains of `iters` * 16
 * dependent fp32 fused multiply-adds (iters * 128 FMAs per lane) and writing one float to `out` (device,
 * workgroups * 256 floats), enqueued on `hip_stream`.  It measures what the vector ALUs sustain when nothing
 * else is used - the clock a kernel bound by ordinary fp32 arithmetic can count on, and the "alu" peak the
 * stitched kernels' instruction counts are held against (packed fp32 instructions are not used).
 */
fs_status fs_alu_probe(void* out, int32_t workgroups, int32_t iters, void* hip_stream);

/* fs_launch_probe: enqueue an empty kernel (one wavefront) on `hip_stream`: what a launch costs when
 * nothing is computed, the floor under the launch-bound workloads. */
fs_status fs_launch_probe(void* hip_stream);

const char* fs_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* FS_H_ */
