// fs_group.cpp - fused-group analysis, schedule and LDS planning, and group formation.
#include <algorithm>
#include <functional>
#include <set>
#include <cstdlib>

#include "fs_internal.h"

namespace fs {

namespace {

int pow2_floor(int x) {
  int p = 1;
  while (p * 2 <= x) p *= 2;
  return p;
}
int pow2_ceil(int x) {
  int p = 1;
  while (p < x) p <<= 1;
  return p;
}

struct Resolved {
  bool literal = false;  // FS_CONST: no tensor behind it
  int node = -1;         // the tensor actually read (bcasts looked through)
  Kind kind = KIND_NONE; // its kind in the group's work space
};

struct Analyser {
  const Graph& g;
  GroupPlan& gp;
  std::vector<char> in_set;
  int R = 1, C = 1;

  Analyser(const Graph& g_, GroupPlan& gp_) : g(g_), gp(gp_), in_set(g_.n(), 0) {}

  Kind classify(int rows, int cols) const {
    if (rows == R && cols == C) return KIND_FULL;
    if (rows == R && cols == 1) return KIND_COLV;
    if (rows == 1 && cols == C) return KIND_ROWV;
    return KIND_NONE;
  }
  // t: the tensor lives in the transposed orientation of the work space (its [r,c] is the work
  // space's [c,r]).  A [C,1] tensor of that orientation is one value per work-space column and has
  // the memory layout of a [1,C] tensor, so vectors need no data movement at all.
  Kind classify(const fs_node& n, bool t) const { return t ? classify(n.cols, n.rows) : classify(n.rows, n.cols); }

  int source_of(int o) const {
    const fs_node& n = g.nodes[o];
    return (n.opcode == FS_BCAST_ROWVEC || n.opcode == FS_BCAST_COLVEC) ? n.in[0] : o;
  }

  // What a consumer working in orientation t and expecting kind `want` sees when it reads operand `o`.
  bool resolve(int o, Kind want, bool t, Resolved* r) const {
    const fs_node& n = g.nodes[o];
    if (classify(n, t) != want) return false;
    if (n.opcode == FS_CONST) {
      r->literal = true;
      return true;
    }
    if (n.opcode == FS_BCAST_ROWVEC || n.opcode == FS_BCAST_COLVEC) {
      const int x = n.in[0];
      const fs_node& xn = g.nodes[x];
      if (xn.opcode == FS_CONST) {
        r->literal = true;
        return true;
      }
      const Kind kx = classify(xn, t);
      if (kx == KIND_NONE) return false;
      // a broadcast either widens a vector to the full work space or is the identity
      const Kind vec = ((n.opcode == FS_BCAST_ROWVEC) != t) ? KIND_ROWV : KIND_COLV;
      if (!(kx == want || (want == KIND_FULL && kx == vec))) return false;
      r->node = x;
      r->kind = kx;
      return true;
    }
    r->node = o;
    r->kind = want;
    return true;
  }
};

void add_ext_in(GroupPlan& gp, int node, Kind k, int dtype) {
  for (const ExtTensor& e : gp.ext_in)
    if (e.node == node) return;
  ExtTensor e;
  e.node = node;
  e.kind = k;
  e.dtype = dtype;
  gp.ext_in.push_back(e);
}

}  // namespace

// -------------------------------------------------------------------------------------------
// Schedule and LDS plan of one group.
//
// Every group runs a Row schedule with split_dim = 0 (Section 4.1): the work space [R,C] is
// cut along rows into `grid` blocks.  What is tuned is how many lanes cooperate on a row (L,
// the role of reduce_warps in Section 4.4), the workgroup size and the block count.  Row
// reductions want a row inside one wavefront (no LDS, no barrier); very long rows are spread
// over several wavefronts and folded through LDS; small problems trade elements per lane
// for more wavefronts so that the 256 CUs all get work.
// -------------------------------------------------------------------------------------------
namespace {
// The decisions of one group's schedule, taken in a fixed order; every step reads what the steps before it decided.
struct Scheduler {
  const Graph& g;
  const PlanOptions& opt;
  GroupPlan* gp;
  Schedule& s;
  const int R, C;
  // the machine: compute units and resident lanes as the device reports them (256 and 524288 on MI355X)
  int CUS = 0;
  int64_t RES = 0;
  // what the group is made of
  int max_es = 0, V = 4, NV = 0;
  bool has_concat = false, rowred = false, colred = false, has_transposed = false, tileable = false;
  // the form its rows take
  int ecap = 8, l_min = 1, l_max = 1;
  bool few_long_rows = false, split_rows = false, resident = false, chunked = false, col_tiled = false, tiled_transpose = false;
  // lanes, vectors, workgroup
  int L = 64, tt_rows = 64, NVL = 1, CT = 1, NVLC = 0, RESV = 0, WG = 256;
  bool staged_loop = false;
  int fold_width = 0;

  Scheduler(const Graph& g_, const PlanOptions& opt_, GroupPlan* gp_) : g(g_), opt(opt_), gp(gp_), s(gp_->s), R(gp_->R), C(gp_->C) {}

  // lanes per row are a power of two: when half as many lanes would hold the row with at most
  // 1.5 x a cap below 32, take them (5120 bf16 columns under a cap of 16: 256 lanes x 24 elements,
  // not 512 x 16 with 37 % of the lanes idle)
  int lanes_for(int e) const {
    const int l = pow2_ceil((NV + e / V - 1) / (e / V));
    if (rowred && l >= 2 && e < 32 && ((NV + l / 2 - 1) / (l / 2)) * V * 2 <= e * 3) return l / 2;
    return l;
  }

  // element size, vector width, which reductions the group holds
  fs_status measure_group() {
    // the machine: compute units and resident lanes as the device reports them (256 and 524288 on MI355X)
    CUS = device_limits().cus;
    RES = device_limits().resident_lanes;
    max_es = 0;
    for (const ExtTensor& e : gp->ext_in)
      if (e.kind == KIND_FULL || e.kind == KIND_PART) max_es = std::max(max_es, dtype_size(e.dtype));
    for (const ExtTensor& e : gp->ext_out)
      if (e.kind == KIND_FULL) max_es = std::max(max_es, dtype_size(e.dtype));
    if (max_es == 0) max_es = 4;
    V = 16 / max_es;
    while (C % V) V /= 2;
    has_concat = false;
    for (int m : gp->members)
      if (g.nodes[m].opcode == FS_CONCAT) {
        has_concat = true;
        if (g.nodes[m].attr_i == FS_CONCAT_COLS)  // a vector access must not straddle the seam
          while (g.nodes[g.nodes[m].in[0]].cols % V) V /= 2;
      }
    NV = C / V;
    rowred = !gp->row_reduces.empty();
    colred = !gp->col_reduces.empty();
    return FS_OK;
  }

  // how a row is held: registers (16, 32, 64 elements per lane), a resident part plus chunks, chunks only, split over workgroups, column tiles, 2-D transpose tiles
  fs_status pick_row_form() {
    // Elements of one [R,C] value a lane may hold.  With row reductions the row stays in registers
    // across the stages together with everything else that is live: the other [R,C] inputs and the
    // lane's slices of the [1,C] operands (E registers each).  128 registers per lane keep four
    // wavefronts per SIMD in flight; 16 elements per lane is the most that pays even when more would
    // fit (measured over 26 row-reduction cases: 16 beats 32 by 3-10 %: more wavefronts per row, more
    // rows in flight); rows too long for that take 32 and 64 below.
    int n_live = 1;
    for (const ExtTensor& e : gp->ext_in) n_live += e.kind == KIND_FULL || e.kind == KIND_ROWV;
    n_live += (int)gp->col_reduces.size();  // a column accumulator per element
    ecap = rowred ? std::max(8, std::min(16, pow2_floor(128 / n_live))) : 8;
    if (colred && !rowred) ecap = 32 / max_es;  // 32 bytes per lane per tile (bf16 sums: 30.2 -> 25.4 us on [65536,1024])
    ecap = std::max(ecap, V);
    l_min = lanes_for(ecap);
    l_max = std::min(1024, pow2_ceil(NV));
    // Groups without reductions do not need a whole row in one workgroup: very long rows are cut
    // into column tiles, each handled like a row of its own.
    tileable = !rowred && !colred;
    has_transposed = false;
    for (const ExtTensor& e : gp->ext_out) has_transposed |= e.transposed;
    // A few very long rows occupy as many CUs as there are rows ([4, 4M] row sums: 263 us on 4 CUs).
    // When every row reduction of the group is in its first stage and everything else that leaves the
    // group is either a per-row value or computed before any reduction result, each row is split
    // over many workgroups; other such groups are better cut into kernels of that form and
    // reduction-free ones (worth_fusing).
    few_long_rows = rowred && !colred && !has_transposed && R <= 128 && (int64_t)C * max_es >= (1 << 18) && (int64_t)R * C * max_es >= (1 << 20);
    split_rows = few_long_rows;
    if (split_rows) {
      for (const ExtTensor& e : gp->ext_out) split_rows &= e.kind == KIND_COLV || gp->level.at(e.node) == 0;
      for (int m : gp->row_reduces) split_rows &= gp->level.at(m) == 0;
    }
    // Rows too long for that: first more elements per lane (32, then 64: one workgroup per CU, but the
    // row is still read once instead of once per stage); beyond that the first 48 (or 32) elements
    // per lane stay resident and the rest of the row is walked in chunks; last, chunks only.  Plan
    // creation steps `wide_level` down while the compiled kernel spills.
    // Rows whose [1,C] operands weigh at least as much per column as the rows themselves (LayerNorm with gamma, beta and a
    // bias over bf16 rows: 12 bytes against 4) keep nothing resident: their last stage needs the registers for the operands,
    // and the whole row fits LDS in its own dtype more often than not.  Measured, LayerNorm+GeLU bf16: [4096,65536] 323 us
    // with a resident part, 282 us chunks only; [4096,49152] 287 -> 207 us; [2049,100000] 267 -> 239 us.
    resident = false;
    if (rowred && l_min > 1024 && !split_rows) {
      const int e32 = std::max(32, V), e64 = std::max(64, V);
      const bool may_chunk = !colred && !has_transposed;
      int64_t rowv_bytes = 0, full_bytes = 0;
      for (const ExtTensor& e : gp->ext_in) {
        if (e.kind == KIND_ROWV) rowv_bytes += dtype_size(e.dtype);
        if (e.kind == KIND_FULL) full_bytes += dtype_size(e.dtype);
      }
      for (const ExtTensor& e : gp->ext_out)
        if (e.kind == KIND_FULL) full_bytes += dtype_size(e.dtype);
      const bool keep_registers = rowv_bytes < full_bytes;
      if (ecap < e32 && lanes_for(e32) <= 1024 && (opt.wide_level >= 1 || !may_chunk)) ecap = e32, l_min = lanes_for(e32);
      else if (may_chunk && keep_registers && opt.wide_level >= 2 && lanes_for(e64) <= 1024) ecap = e64, l_min = lanes_for(e64);
      else if (may_chunk && keep_registers && opt.wide_level >= 1) resident = true;
    }
    // Row reductions over rows that do not fit the registers of one workgroup: the workgroup walks
    // its row in column chunks, once per stage, recomputing what each stage needs.
    chunked = (l_min > 1024 && rowred && !colred && !has_transposed) || split_rows;
    // Column reductions alone do not need whole rows either: column tiles, each with its own fold.
    // Tiles of 64 lanes x 16 elements, whatever the row length: every tile has its own, small fold (a workgroup's
    // partial is 4 KB, the folds of different tiles run side by side), where one tile as wide as the row makes the last
    // arrivers of the grid fold read 16 x C floats each.  Column sums of f32: [8192,8192] 58 -> 78 % of peak,
    // [16384,4096] 65 -> 69 %, [4096,16384] 71 -> 78 % (tiles of 256 lanes before), narrower rows unchanged.
    col_tiled = colred && !rowred && !has_transposed && (l_min > 1024 || (l_min > 64 && !has_concat));
    if (l_min > 1024 && !tileable && !chunked && !col_tiled)
      FS_FAIL(FS_ERR_UNSUPPORTED, "rows of %d columns are too long for one workgroup in a group with %s", C,
              colred ? "row and column reductions" : "transposed outputs");
    if (has_concat && (chunked || col_tiled))
      FS_FAIL(FS_ERR_UNSUPPORTED, "a concat cannot be read by a kernel that walks rows of %d columns in chunks", C);
    if (tileable) l_min = std::min(l_min, 256);
    // wide transposes: 2-D tiles through LDS
    tiled_transpose = has_transposed && tileable && C > 256 && R > 1;
    if (split_rows) l_min = 256;
    else if (chunked) l_min = 1024;  // (measured: the largest workgroup keeps the fewest rows in flight, so re-reads hit the caches more often)
    if (col_tiled) l_min = std::min(64, l_max);
    return FS_OK;
  }

  // lanes per row
  fs_status pick_lanes() {
    L = rowred ? std::min(64, l_max) : std::min(256, l_max);
    // Very narrow rows: a row of at most 32 bytes belongs to one lane (no cross-lane step at all;
    // [4M,3] L2-normalise: 34.8 -> 17.6 us); rows that can only be read element by element (odd
    // widths) get at least two elements per lane.
    // A row that leaves part of a wavefront's last vector slots empty (768 bf16 columns: 96 vectors
    // on 64 lanes x 2) is better served by fewer lanes that it fills exactly, several rows per
    // wavefront (32 lanes x 3: LayerNorm+GeLU bf16 [32768,768] 24.0 -> 20.9 us).
    // Below a quarter of the slots empty it does not pay (softmax fp32 [32768,640]: 27.7 us on 64 lanes
    // x 3 vectors with 17 % empty, 29.4 us on 32 x 5).
    if (rowred && !colred && L > l_min && l_min >= 1) {
      const auto waste = [&](int lanes) { return (int64_t)((NV + lanes - 1) / lanes) * lanes - NV; };
      if (waste(L) * 4 >= NV + waste(L))
        for (int l = L; l >= l_min; l /= 2)
          if (waste(l) < waste(L)) L = l;
    }
    if (rowred && !colred && C * max_es <= 32) L = 1;
    else if (rowred && !colred && V == 1 && NV >= 4) L = std::min(L, pow2_ceil(NV) / 2);
    // a transposed root leaves as runs of G = WG/L consecutive elements: at least 16 rows per workgroup
    if (has_transposed && !rowred) L = std::min(L, std::max(l_min, 16));
    // looping (column-reduction) kernels want more bytes in flight per lane: 16 elements per lane
    if (colred) L = std::min(L, std::max(1, pow2_ceil((NV * V + 15) / 16)));
    L = std::max(L, l_min);
    if (col_tiled) L = l_min;
    // tile = tt_rows rows (128 bytes of the narrowest transposed output: the length of a run in the
    // transposed tensor) by 1024 / tt_rows lanes x one 16-byte vector; measured best among 14 shapes
    tt_rows = 64;
    if (tiled_transpose) {
      int es = 4;
      for (const ExtTensor& e : gp->ext_out)
        if (e.transposed) es = std::min(es, dtype_size(e.dtype));
      tt_rows = std::max(16, std::min(64, 128 / es));
      L = std::min(1024 / tt_rows, l_max);
      // the tile holds one float per element: 16-element vectors (u8 alone) need narrower tiles to fit the budget
      while (L > 4 && (int64_t)L * V * (tt_rows + 1) * 4 > opt.lds_budget) L /= 2;
    }
    // small problems: more lanes per row until the device has ~8 wavefronts per CU
    // (a row that will be cut into column tiles anyway is not a small problem)
    const bool col_tiles_anyway = tileable && (int64_t)NV * V > (int64_t)L * ecap;
    while ((int64_t)R * L / 64 < 8 * CUS && L < l_max && !(has_transposed && !rowred) && !chunked && !col_tiled && !col_tiles_anyway) L *= 2;
    if (split_rows) L = 256;
    if (opt.has_hint && opt.hint.lanes_per_row > 0 && !tiled_transpose && !split_rows) {
      const int h = opt.hint.lanes_per_row;
      if ((h & (h - 1)) == 0 && h >= ((chunked || col_tiled) ? 64 : l_min) && h <= 1024) L = h;
    }
    return FS_OK;
  }

  // vectors per lane, column tiles / chunks per row
  fs_status pick_vectors() {
    NVL = (NV + L - 1) / L, CT = 1;
    if (NVL * V > ecap && tileable) {
      NVL = std::max(1, ecap / V);
      CT = (NV + NVL * L - 1) / (NVL * L);
    }
    if (tiled_transpose) {
      NVL = 1;
      // 2-byte elements: two vectors per lane make the tile's rows 512-byte runs like those of f32 tiles; the tile
      // (one float per element) then takes 66.5 KB, which two workgroups per CU still fit -- unless the caller set a budget
      // (bf16 transposes: [32768,8192] 198 -> 182 us, [16384,4096] 49.0 -> 46.9 us; f32 with two vectors: slower; so are
      // bf16 tensors with few tiles either way: [65536,1024] 49.9 -> 51.5 us, [1000,30000] 37.0 -> 38.0 us, [2048,2048])
      int es_in = 4;
      for (const ExtTensor& e : gp->ext_in)
        if (e.kind == KIND_FULL) es_in = std::min(es_in, dtype_size(e.dtype));
      if (es_in == 2 && V == 8 && !opt.lds_budget_given && (int64_t)2 * L * V * (tt_rows + 1) * 4 + 1024 <= device_limits().lds_per_workgroup / 2 &&
          NV >= 16 * L && R >= 4096 && (int64_t)R * C * 2 >= (32ll << 20))
        NVL = 2;
      CT = (NV + NVL * L - 1) / (NVL * L);
    }
    NVLC = 0, RESV = 0;
    if (chunked || col_tiled) {
      NVLC = std::max(1, 16 / V);
      // column tiles: 64 bytes of the narrowest input per lane and trip (bf16: 32 elements), not beyond the row
      // (bf16 column sums of [16384,4096]: 30.5 -> 26.7 us); 32 accumulators per column reduction at most
      if (col_tiled && gp->col_reduces.size() <= 2) NVLC = std::max(1, std::min(std::min(4, 32 / V), (NV + L - 1) / L));
      NVL = resident ? std::max(1, (opt.wide_level >= 2 ? 48 : 32) / V) : NVLC;  // (64 resident elements plus a chunk in flight spill)
      RESV = resident ? NVL * L : 0;
      CT = (NV - RESV + NVLC * L - 1) / (NVLC * L);
    }
    return FS_OK;
  }

  // workgroup size; whether workgroups loop with their [1,C] operands staged once
  fs_status pick_workgroup() {
    const int64_t total_waves = std::max<int64_t>(1, (int64_t)R * CT * L / 64);
    if (col_tiled) {
      WG = std::max(64, L);
      for (int w = 512; w >= 128; w /= 2)
        if (w >= L && (int64_t)R * L / w >= 8) {
          WG = w;
          break;
        }
    } else if (colred) {
      // large workgroups (few partials, many rows per trip) as long as every CU still gets a workgroup
      // and the in-workgroup fold area (one row of C floats per wavefront or row-group) fits the budget
      WG = std::max(64, L);
      for (int w = 512; w >= 128; w /= 2)
        if (w >= L && (int64_t)R * L / w >= CUS) {
          WG = w;
          break;
        }
      if (rowred && L >= 256) WG = std::max(WG, std::min(1024, 4 * L));  // rows across several wavefronts: 16 wavefronts per CU
    }
    else if (total_waves > 4 * CUS || has_transposed) WG = std::max(256, L);
    else WG = std::max(64, L);
    // Rows with [1,C] operands, above all operands that outweigh the row's own traffic (LayerNorm with
    // gamma, beta and a bias over bf16 rows: 12 bytes per column against 4).  Re-reading the operands for every row, or for
    // every few rows of a one-trip workgroup, costs L2 bandwidth; keeping them in registers costs
    // occupancy (48 of 84 registers).  When they fit the LDS budget and there is work for more than
    // two rounds of resident workgroups, the workgroups loop instead, 32 wavefronts per CU, and stage
    // the operands in LDS once, before the loop.  LayerNorm+GeLU bf16 [8192,4096]: 35.3 us re-reading,
    // 31.2 us from registers, 27.6 us staged; [16384,2048]: 29.3 -> 26.5 us; [16384,1024]: 14.7 ->
    // 13.1 us (one trip: staged once per 4 rows); no gain without such operands (softmax: 3-7 % slower),
    // nor for one-wavefront rows with fewer than 16 elements per lane or a half-empty last vector
    // ([16384,512]: 9.2 -> 9.7 us, [32768,768]: 22.6 -> 24.1 us), which keep the one-trip form.
    staged_loop = false;
    if (rowred && !colred && !chunked && !has_transposed && CT == 1 && R > 1) {
      int64_t rowv_bytes = 0, full_bytes = 0;
      int n_rowv_in = 0;
      for (const ExtTensor& e : gp->ext_in) {  // bytes per column
        if (e.kind == KIND_ROWV) rowv_bytes += dtype_size(e.dtype), ++n_rowv_in;
        if (e.kind == KIND_FULL) full_bytes += dtype_size(e.dtype);
      }
      for (const ExtTensor& e : gp->ext_out)
        if (e.kind == KIND_FULL) full_bytes += dtype_size(e.dtype);
      const int wg = L >= 128 ? std::min(1024, 4 * L) : std::max(256, std::min(1024, 16 * L));  // 4 rows, or 16 one-wavefront rows, per trip
      // (one-wavefront rows: beyond ~8 rounds of resident workgroups the one-trip form catches up and
      // passes: [65536,1024] 48.9 against 49.5 us, [262144,1024] 203 against 210 us)
      const bool full_slices = NVL * V >= 16 && (int64_t)NVL * L == NV && (int64_t)R * L <= 8 * RES;
      // rows across several wavefronts gain with any [1,C] operand (RMSNorm bf16 [8192,4096]: 24.5 ->
      // 23.6 us, residual+LayerNorm: 50.5 -> 45.8 us); one-wavefront rows only with heavy ones
      // (up to ~4 rounds of work: at [32768,2048] the one-trip form is 2-5 % faster again)
      const bool heavy = rowv_bytes * 2 >= full_bytes * 3;
      // from two rounds of resident workgroups on; from one round where heavy operands meet rows of one or two wavefronts
      // (LayerNorm+GeLU bf16 [8192,1024]: 9.0 -> 8.0 us, [12288,1024]: 11.7 -> 10.6 us, [6000,2048]: 12.4 -> 10.3 us; rows over
      // four wavefronts and light operands lose there: [2048,4096] 9.9 -> 10.6 us, RMSNorm [1024,8192] 6.7 -> 7.7 us)
      const int rounds = heavy && L <= 128 ? 1 : 2;
      const bool pays = L >= 128 ? heavy || (n_rowv_in > 0 && (int64_t)R * L <= 4 * RES) : full_slices && heavy;
      if (pays && (int64_t)n_rowv_in * NVL * L * V * 4 + 1024 <= opt.lds_budget && (int64_t)R * L / wg >= rounds * (RES / wg)) {
        staged_loop = true;
        WG = wg;
      }
    }
    if (chunked) WG = L;  // one row per workgroup
    if (tiled_transpose) WG = std::max(64, L * std::min(tt_rows, std::max(4, pow2_ceil(R))));
    if (opt.has_hint && opt.hint.wg_threads > 0 && !chunked && !tiled_transpose) {
      const int h = opt.hint.wg_threads;
      if (h % 64 == 0 && h >= L && h <= 1024) WG = h;
    }
    return FS_OK;
  }

  // the schedule record, row segments of split rows, loop trips
  fs_status fill_schedule() {
    s.V = V;
    s.NV = NV;
    s.L = L;
    s.NVL = NVL;
    s.CT = CT;
    s.E = s.NVL * V;
    s.WG = WG;
    s.G = WG / L;
    s.ragged = resident ? false : (int64_t)CT * NVL * L != NV;
    s.resident = resident;
    s.NVLC = NVLC;
    s.RESV = RESV;
    s.ragged_chunks = chunked && (int64_t)RESV + (int64_t)CT * NVLC * L != NV;
    s.chunked = chunked;
    s.col_tiled = col_tiled;
    s.tiled_transpose = tiled_transpose;
    // Bands whose rows are 4 KB runs of the narrowest input (8 tiles of f32, 16 of bf16), twice that when the tensor has
    // so few row tiles that a band would not fill the device.  Against plain order, f32: [8192,8192] 60 -> 75 % of peak,
    // [1024,65536] 51 -> 72 %, [8192,28672] 58 -> 70 %, [300,100000] 34 -> 63 %; bf16: [32768,8192] 56 -> 66 %,
    // [1000,30000] 30 -> 46 %; never slower on 24 shapes.  (Bands of 2 or 4 tiles are slower than none; the best
    // width varies by a few per cent with the row pitch, [16384,16384] f32: 66 % with 8, 61 % with 16, 68 % with 24.)
    s.tt_col_band = 0;
    if (tiled_transpose) {
      int es = 4;
      for (const ExtTensor& e : gp->ext_in)
        if (e.kind == KIND_FULL) es = std::min(es, dtype_size(e.dtype));
      const int row_tiles = (R + s.G - 1) / s.G;
      int band = std::max(1, 4096 / (NVL * L * V * es));
      if (row_tiles <= 32) band *= 2;
      if (CT > band) s.tt_col_band = band;
    }
    s.split_rows = split_rows;
    s.min_waves = opt.min_waves;
    s.few_long_rows = few_long_rows;
    s.S = 1;
    s.CPS = CT;
    if (split_rows) {  // at least 2 chunks per workgroup, about `target` workgroups in all
      const int target = opt.has_hint && opt.hint.max_workgroups > 0 ? opt.hint.max_workgroups : 512;
      s.S = std::max(1, std::min((CT + 1) / 2, std::max(1, target / R)));
      s.CPS = (CT + s.S - 1) / s.S;
      s.S = (CT + s.CPS - 1) / s.CPS;  // no empty segment
    }
    s.n_iters = split_rows ? R * s.S : chunked ? R : col_tiled ? (R + s.G - 1) / s.G : tiled_transpose ? (int)((int64_t)CT * ((R + s.G - 1) / s.G))
                                                                               : (int)(((int64_t)R * CT + s.G - 1) / s.G);
    return FS_OK;
  }

  // workgroups launched, row tiles per trip, fold fan-in
  fs_status pick_grid() {
    // Streaming groups launch one workgroup per row tile: the hardware hands tiles out in memory
    // order and a fresh wavefront issues its loads at once, which measures faster on this device
    // than persistent workgroups looping with a grid stride.  Column reductions keep a bounded
    // grid because every workgroup leaves a partial to fold.
    int cap = colred ? CUS : (1 << 30);
    // Exception: [1,C] operands that cannot be shared through LDS (fewer than 4 rows per workgroup)
    // are read again from L2 for every row of a one-shot grid.  When those reads outweigh the row's
    // own traffic (LayerNorm with gamma, beta and a bias over rows of 4096+ elements: 12 bytes per
    // column against 4), the workgroups loop instead, 16 wavefronts per CU, and keep their slices of
    // the operands in registers (measured on [8192,4096] bf16: 35.3 -> 29.4 us).
    if (staged_loop && s.G >= 2) {
      cap = std::max(CUS, (int)(RES / WG));
    } else if (!colred && !chunked && CT == 1 && s.G < 4 && R > 1) {
      int64_t rowv_bytes = 0, full_bytes = 0;
      for (const ExtTensor& e : gp->ext_in) {  // bytes per column
        if (e.kind == KIND_ROWV) rowv_bytes += dtype_size(e.dtype);
        if (e.kind == KIND_FULL) full_bytes += dtype_size(e.dtype);
      }
      for (const ExtTensor& e : gp->ext_out)
        if (e.kind == KIND_FULL) full_bytes += dtype_size(e.dtype);
      if (rowv_bytes * 2 >= full_bytes * 3) cap = std::max(CUS, (int)(RES / 2 / WG));
    }
    if (opt.has_hint && opt.hint.max_workgroups > 0) cap = opt.hint.max_workgroups;
    cap = std::min(cap, (int)(0x7fffffff / WG));  // a launch holds fewer than 2^31 lanes: beyond that the workgroups loop
    s.grid = std::max(1, std::min(s.n_iters, cap));
    // workload 2 (2 trips): 13.5 -> 13.0 us; LayerNorm+GeLU bf16 [12288,1024]: 10.7 -> 10.2 us; 4 trips: +0.4 %, 8 trips: -0.8 %;
    // rows over several wavefronts lose 3-16 % ([6000,2048]: 10.5 -> 12.3 us)
    s.rotate_loop = staged_loop && L <= 64 && s.grid < s.n_iters && s.n_iters <= 4 * (int64_t)s.grid;
    s.RB = s.grid;
    if (split_rows) {
      s.grid = R * s.S;
      s.RB = s.S;
    }
    if (col_tiled) {  // RB workgroups per column tile, about `cap` workgroups in all
      s.RB = std::max(1, std::min(s.n_iters, std::max(1, cap / CT)));
      s.grid = s.RB * CT;
    }
    // Looping kernels that only fold columns have almost no arithmetic per trip: their rate is set by
    // the bytes in flight, and two row tiles per trip measured 13 % faster (28.1 -> 24.5 us on
    // [65536,512]).  With a row reduction in the body one tile per trip is the faster form.
    s.U = (colred && !rowred && s.grid < s.n_iters && CT == 1) ? 2 : 1;
    if (opt.has_hint && opt.hint.tiles_per_trip >= 1 && opt.hint.tiles_per_trip <= 4) s.U = opt.hint.tiles_per_trip;
    if (has_concat) s.U = 1;
    // two fold levels at most: the smallest fan-in whose square covers the grid
    // (64 workgroups per fold: 16 measured 9 % faster than 8 on column sums of [16384,4096], 44.6 against 48.8 us)
    s.fan_in = s.RB <= 32 ? 8 : s.RB <= 256 ? 16 : 32;
    return FS_OK;
  }

  // LDS plan of the kernel
  fs_status plan_lds() {
    // LDS plan (Section 5.1).  Size requirements: cross-wave row-reduction partials (the "direct
    // allocation" for a non-root Reduce) and the column-partial fold area.  Space sharing: all row
    // reductions of the kernel reuse one ping-pong pair of slots instead of one buffer each (the
    // Reduce.2-reuses-Reduce.1 case of Section 5.1.3); the column fold area is shared by all column
    // reductions in turn.
    // Space sharing by lifetime (the idea of Section 5.1.3 applied to the kernel's two phases): what
    // the row loop uses (transpose tile, staged [1,C] operands) is dead when the epilogue folds the
    // column partials, so both live in one pool of max(loop bytes, fold bytes).
    int fixed = 0, loop_bytes = 0, fold_bytes = 0;
    if (rowred && L > 64) fixed += 2 * s.G * (L / 64) * gp->max_batched_reduces * 4;
    if (split_rows) fixed += 16 + (int)gp->row_reduces.size() * 4;
    fold_width = col_tiled ? NVL * L * V : C;  // columns one workgroup folds
    s.fold_piece = fold_width;
    if (colred) {
      // the fold area takes at most half of the budget: wide rows pass through it in pieces
      fixed += 16;
      const int fold_rows = L < 64 ? WG / 64 : s.G;
      const int piece_cap = std::max(8, (opt.lds_budget / 2 / (fold_rows * 4)) / 8 * 8);
      if (fold_width > piece_cap) s.fold_piece = piece_cap;
      fold_bytes = fold_rows * s.fold_piece * 4;
    }
    auto total = [&]() { return fixed + std::max(loop_bytes, fold_bytes); };
    // [1,C] inputs shared by all rows of a workgroup are staged in LDS by the whole workgroup (once,
    // before the loop, when the workgroup loops) when several rows share them and the budget allows
    int n_rowv = 0;
    for (const ExtTensor& e : gp->ext_in) n_rowv += e.kind == KIND_ROWV;
    s.stage_rowv = false;
    s.tile_transpose = false;
    const int tile_bytes = (tiled_transpose ? NVL * L * V : C) * (s.G + 1) * 4;
    // (the wider tiles of 2-byte transposes may pass the default budget: half of what a CU has, so that two workgroups fit)
    const int tile_cap = tiled_transpose && NVL == 2 ? device_limits().lds_per_workgroup / 2 : opt.lds_budget;
    if (has_transposed && (CT == 1 || tiled_transpose) && s.G >= 4 && fixed + std::max(loop_bytes + tile_bytes, fold_bytes) <= tile_cap) {
      s.tile_transpose = true;
      loop_bytes += tile_bytes;
    }
    const int slot_bytes = s.NVL * s.L * V * 4;
    if (n_rowv > 0 && CT == 1 && (s.G >= 4 || (staged_loop && s.G >= 2)) && R > 1 &&
        fixed + std::max(loop_bytes + n_rowv * slot_bytes, fold_bytes) <= opt.lds_budget) {
      s.stage_rowv = true;
      loop_bytes += n_rowv * slot_bytes;
    }
    const int lds = total();
    s.lds_bytes = s.lds_planned = lds;
    if (lds > (s.tile_transpose ? tile_cap : opt.lds_budget))
      FS_FAIL(FS_ERR_LDS_BUDGET, "group needs %d bytes of LDS, budget is %d", lds, opt.lds_budget);
    // Rows walked in chunks: what is left of the workgroup's LDS may hold the head of the row in its input dtype
    // (one 1024-lane workgroup per compute unit runs such a kernel, so it may take all a workgroup is allowed
    // unless the caller set a budget); code generation decides which inputs are worth it.
    s.stage_avail = 0;
    if (chunked && !split_rows) {
      const int cap = opt.lds_budget_given ? opt.lds_budget : device_limits().lds_per_workgroup;
      s.stage_avail = std::max(0, cap - lds - 512);
    }
    return FS_OK;
  }

  // workspace scratch of grid-wide folds
  fs_status plan_scratch() {
    // grid-wide fold scratch
    gp->n_tickets = 0;
    gp->part_bytes = 0;
    s.part_stride_floats = 0;
    s.ticket_stride = 0;
    if (split_rows) {  // per row: S partials of one float per reduction
      const size_t k = gp->row_reduces.size();
      int n = s.S;
      while (n > 1) {
        s.part_stride_floats += (size_t)n * k;
        n = (n + s.fan_in - 1) / s.fan_in;
        s.ticket_stride += n;
      }
      gp->n_tickets = s.ticket_stride * R;
      gp->part_bytes = s.part_stride_floats * R * 4;
    }
    if (colred) {
      const size_t kc = gp->col_reduces.size() * (size_t)fold_width;
      int n = s.RB;
      while (n > 1) {
        s.part_stride_floats += (size_t)n * kc;
        n = (n + s.fan_in - 1) / s.fan_in;
        s.ticket_stride += n;
      }
      const int tiles = col_tiled ? CT : 1;
      gp->n_tickets = s.ticket_stride * tiles;
      gp->part_bytes = s.part_stride_floats * tiles * 4;
    }
    return FS_OK;
  }

  fs_status run() {
    fs_status st;
    if ((st = measure_group()) != FS_OK) return st;
    if ((st = pick_row_form()) != FS_OK) return st;
    if ((st = pick_lanes()) != FS_OK) return st;
    if ((st = pick_vectors()) != FS_OK) return st;
    if ((st = pick_workgroup()) != FS_OK) return st;
    if ((st = fill_schedule()) != FS_OK) return st;
    if ((st = pick_grid()) != FS_OK) return st;
    if ((st = plan_lds()) != FS_OK) return st;
    return plan_scratch();
  }
};
}  // namespace

static fs_status choose_schedule(const Graph& g, const PlanOptions& opt, GroupPlan* gp) { return Scheduler(g, opt, gp).run(); }

fs_status analyse_group(const Graph& g, const std::vector<int>& members, const std::vector<int>& /*group_of*/,
                        int self_group, const PlanOptions& opt, GroupPlan* out) {
  GroupPlan& gp = *out;
  gp = GroupPlan();
  gp.members = members;
  std::sort(gp.members.begin(), gp.members.end());
  Analyser a(g, gp);
  for (int m : gp.members) a.in_set[m] = 1;

  // Orientation of every member.  A transpose inside a group moves no data: it flips the flag,
  // and everything downstream is computed in the producer's register layout (the paper inlines
  // such shape modulation by thread composition, Section 4.3).  Only a value that LEAVES the
  // kernel in the flipped orientation is stored transposed.
  std::map<int, bool>& tf = gp.tflag;
  for (int m : gp.members) {
    const fs_node& n = g.nodes[m];
    bool t = n.opcode == FS_TRANSPOSE;  // operands outside the group are read as they lie in memory
    for (int k = 0; k < n.num_in; ++k) {
      const int src = a.source_of(n.in[k]);
      if (a.in_set[src]) {
        t = (n.opcode == FS_TRANSPOSE) ? !tf[src] : tf[src];
        break;
      }
    }
    tf[m] = t;
  }
  // work space: the largest extents seen, every shape taken in its orientation
  int R = 1, C = 1;
  for (int m : gp.members) {
    const fs_node& n = g.nodes[m];
    const bool t = tf[m], t_op = n.opcode == FS_TRANSPOSE ? !t : t;
    R = std::max(R, t ? n.cols : n.rows), C = std::max(C, t ? n.rows : n.cols);
    for (int k = 0; k < n.num_in; ++k) {
      if (g.flat_in[m][k]) continue;  // read as an element sequence under this node's own shape: its label says nothing here
      const fs_node& o = g.nodes[n.in[k]];
      R = std::max(R, t_op ? o.cols : o.rows), C = std::max(C, t_op ? o.rows : o.cols);
    }
  }
  a.R = gp.R = R;
  a.C = gp.C = C;

  auto is_reduce = [&](int id) { return g.nodes[id].opcode == FS_REDUCE_ROW || g.nodes[id].opcode == FS_REDUCE_COL; };
  // reductions by their direction in the work space (a row reduction of a flipped tensor runs down the columns)
  auto reduces_rows = [&](int id) { return is_reduce(id) && gp.kind[id] == KIND_COLV && C > 1; };   // lanes exchange values
  auto reduces_cols = [&](int id) { return is_reduce(id) && gp.kind[id] == KIND_ROWV && R > 1; };   // finished by the grid fold

  for (int m : gp.members) {
    const fs_node& n = g.nodes[m];
    const bool t = tf[m], t_op = n.opcode == FS_TRANSPOSE ? !t : t;
    const Kind result_kind = a.classify(n, t);
    if (n.opcode == FS_CONCAT) {
      // read from memory as one row out of two tensors; nothing is computed, so nothing is fused INTO a concat:
      // an operand produced by this group would have to exist in memory first
      if (t || result_kind != KIND_FULL) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d (concat) does not fit the group's work space [%d,%d]", m, R, C);
      for (int k = 0; k < 2; ++k) {
        const int o = n.in[k];
        if (a.in_set[g.root_of[o]]) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d (concat): operand %d is computed by the same kernel", m, o);
        for (const ExtTensor& e : gp.ext_in)
          if (e.node == o && e.kind != KIND_PART) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d is read both whole and as part of a concat", o);
        add_ext_in(gp, o, KIND_PART, g.nodes[o].dtype);
        gp.kind[o] = KIND_PART;
      }
      gp.kind[m] = KIND_FULL;
      gp.level[m] = 0;
    }
    Kind operand_kind = result_kind;
    if (is_reduce(m) || n.opcode == FS_TRANSPOSE) operand_kind = KIND_FULL;
    if (result_kind == KIND_NONE || (n.opcode == FS_TRANSPOSE && result_kind != KIND_FULL))
      FS_FAIL(FS_ERR_UNSUPPORTED, "node %d [%d,%d] does not fit the group's work space [%d,%d]", m, n.rows, n.cols, R, C);
    gp.kind[m] = result_kind;
    const bool deferred = reduces_cols(m);
    int lvl = result_kind == KIND_ROWV && !deferred ? -1 : 0;
    for (int k = 0; k < n.num_in && n.opcode != FS_CONCAT; ++k) {
      Resolved r;
      if (g.flat_in[m][k]) {
        // a tensor in memory under another [rows, cols] label: the same elements at row * C + column of this work space.
        // It cannot come from this kernel's registers (another label means another assignment of elements to lanes).
        const int o = n.in[k];
        if (g.nodes[o].opcode == FS_CONST) continue;
        if (a.in_set[o] || a.in_set[g.root_of[o]])
          FS_FAIL(FS_ERR_UNSUPPORTED, "node %d reads node %d under another shape: it has to exist in memory first", m, o);
        if (t_op || operand_kind != KIND_FULL || (int64_t)g.nodes[o].rows * g.nodes[o].cols != (int64_t)R * C)
          FS_FAIL(FS_ERR_UNSUPPORTED, "node %d: operand %d (read as a flat element sequence) does not fill the work space [%d,%d]", m, o, R, C);
        for (const ExtTensor& e : gp.ext_in)
          if (e.node == o && e.kind != KIND_FULL) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d is read in two ways", o);
        add_ext_in(gp, o, KIND_FULL, g.nodes[o].dtype);
        gp.kind[o] = KIND_FULL;
        continue;
      }
      if (!a.resolve(n.in[k], operand_kind, t_op, &r))
        FS_FAIL(FS_ERR_UNSUPPORTED, "node %d: operand %d does not fit the group's work space [%d,%d]", m, n.in[k], R, C);
      if (r.literal) continue;
      if (a.in_set[r.node]) {
        if (tf[r.node] != t_op) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d mixes orientations", m);
        if (reduces_cols(r.node))
          FS_FAIL(FS_ERR_UNSUPPORTED, "node %d consumes node %d, whose value only exists after the whole grid has run", m, r.node);
        lvl = std::max(lvl, gp.level[r.node] + (reduces_rows(r.node) ? 1 : 0));
      } else {
        // a view of a value this kernel computes would have to exist in memory first
        if (a.in_set[g.root_of[r.node]]) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d reads node %d, a view of a value computed by the same kernel", m, r.node);
        // tensors from memory: a full tensor can only be read in the orientation it is stored in
        if (r.kind == KIND_FULL && t_op) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d would need a transposing load of node %d", m, r.node);
        for (const ExtTensor& e : gp.ext_in)
          if (e.node == r.node && e.kind != r.kind) FS_FAIL(FS_ERR_UNSUPPORTED, "node %d is read in two orientations", r.node);
        add_ext_in(gp, r.node, r.kind, g.nodes[r.node].dtype);
        gp.kind[r.node] = r.kind;
      }
    }
    gp.level[m] = lvl;
    if (reduces_rows(m)) gp.row_reduces.push_back(m);
    if (reduces_cols(m)) gp.col_reduces.push_back(m);

    // does the value leave the kernel?
    bool leaves = g.output_index[m] >= 0;
    std::function<void(int)> scan_users = [&](int id) {
      for (int u : g.users[id]) {
        const int uop = g.nodes[u].opcode;
        if (uop == FS_BCAST_ROWVEC || uop == FS_BCAST_COLVEC) scan_users(u);
        else if (op_is_view(uop)) leaves = true;  // a view is read from memory (or is a plan output): the value must exist there
        else if (!opt.clones) leaves |= !a.in_set[u];
        else {
          // every kernel that computes u reads m from memory unless it computes m itself
          const CloneInfo& ci = *opt.clones;
          auto needs = [&](int h) { return h == self_group ? !a.in_set[u] : (h >= 0 && !ci.computed_in(m, h)); };
          leaves |= needs(ci.group_of[u]);
          auto it = ci.extra.find(u);
          if (it != ci.extra.end())
            for (int h : it->second) leaves |= needs(h);
        }
      }
    };
    scan_users(m);
    // (a copy: the first kernel that computes the value is the one that stores it)
    if (opt.clones && opt.clones->group_of[m] != self_group) leaves = false;
    if (leaves) {
      ExtTensor e;
      e.node = m;
      e.kind = result_kind;
      e.dtype = n.dtype;
      e.transposed = t && result_kind == KIND_FULL && R > 1 && C > 1;
      e.deferred = deferred;
      if (t && result_kind == KIND_FULL && !e.transposed && (R > 1 || C > 1)) {
        // a flipped vector-shaped work space ([R,1] <-> [1,R]) has the same memory layout: plain store
      }
      gp.ext_out.push_back(e);
    }
  }
  if (gp.ext_out.empty()) FS_FAIL(FS_ERR_UNSUPPORTED, "group produces nothing");
  if ((int)(gp.ext_in.size() + gp.ext_out.size()) > kMaxGroupTensors) FS_FAIL(FS_ERR_UNSUPPORTED, "group touches too many tensors");

  // row reductions of one stage share one exchange
  std::map<int, int> per_level;
  for (int m : gp.row_reduces) gp.max_batched_reduces = std::max(gp.max_batched_reduces, ++per_level[gp.level[m]]);

  int arg = 0;
  for (ExtTensor& e : gp.ext_in) e.arg = arg++;
  for (ExtTensor& e : gp.ext_out) e.arg = arg++;
  // Tensors far larger than the caches are read / written once: keep them out of the way (non-temporal accesses).
  // So are smaller ones that no other kernel of the plan touches -- a plan input only this kernel reads, a plan output
  // nothing else in the plan consumes: what is written normally stays in the L2 until the end of the kernel and is
  // written back then, after the last wavefront, which costs a microsecond or two that a kernel of 5-10 us notices
  // (softmax f32 [4096,1024]: 8.0 -> 6.6 us, [2048,1024]: 5.8 -> 4.6 us; LayerNorm+GeLU bf16 [4096,1024]: 6.0 -> 5.1 us;
  // Adam [2048,2048]: 23.8 -> 21.2 us; 1 MB tensors: no difference).  Values that pass between kernels stay cacheable.
  constexpr uint64_t kStreamBytes = 32ull << 20, kStreamOnceBytes = 2ull << 20;
  auto bytes_of = [&](const ExtTensor& e) { return (uint64_t)g.nodes[e.node].rows * g.nodes[e.node].cols * dtype_size(e.dtype); };
  std::function<bool(int)> used_only_here = [&](int id) {
    for (int u : g.users[id]) {
      const int uop = g.nodes[u].opcode;
      if (uop == FS_BCAST_ROWVEC || uop == FS_BCAST_COLVEC || op_is_view(uop)) {
        if (!used_only_here(u)) return false;  // (a view that is a plan output consumes nothing)
      } else if (!a.in_set[u]) {
        return false;
      }
    }
    return true;
  };
  for (ExtTensor& e : gp.ext_in) {
    const int root = g.root_of[e.node];
    const bool once = g.nodes[root].opcode == FS_INPUT && used_only_here(root);
    e.streaming = e.kind == KIND_FULL && bytes_of(e) >= (once ? kStreamOnceBytes : kStreamBytes);
  }
  for (ExtTensor& e : gp.ext_out) {
    const bool once = g.family_output[e.node] >= 0 && used_only_here(e.node);
    e.streaming = e.kind == KIND_FULL && !e.transposed && bytes_of(e) >= (once ? kStreamOnceBytes : kStreamBytes);
  }

  gp.min_hbm_bytes = 0;
  for (const ExtTensor& e : gp.ext_in) gp.min_hbm_bytes += (uint64_t)g.nodes[e.node].rows * g.nodes[e.node].cols * dtype_size(e.dtype);
  for (const ExtTensor& e : gp.ext_out) gp.min_hbm_bytes += (uint64_t)g.nodes[e.node].rows * g.nodes[e.node].cols * dtype_size(e.dtype);

  const fs_status st = choose_schedule(g, opt, &gp);
  if (st == FS_OK && gp.s.chunked)  // every stage reads the row again: keep it in the caches
    for (ExtTensor& e : gp.ext_in) e.streaming = false;
  return st;
}

// -------------------------------------------------------------------------------------------
// Schedule tuning (Section 4.3): candidates and the library-driven choice.
// -------------------------------------------------------------------------------------------
std::vector<fs_sched_hint> candidate_hints(const GroupPlan& base) {
  const Schedule& s = base.s;
  std::vector<fs_sched_hint> out;
  if (s.chunked) return out;  // one row per 1024-lane workgroup: nothing to vary
  std::vector<int> Ls, WGs, caps;
  for (int L : {s.L / 2, s.L, s.L * 2})
    if (L >= 1 && L <= 1024) Ls.push_back(L);
  for (int WG : {s.WG / 2, s.WG, s.WG * 2})
    if (WG >= 64 && WG <= 1024) WGs.push_back(WG);
  caps.push_back(0);
  if (!base.col_reduces.empty() && s.grid > 1)  // every workgroup leaves a partial: the grid is a real trade-off
    for (int c : {s.grid / 2, s.grid * 2})
      if (c >= 1 && c <= 2048) caps.push_back(c);
  for (int L : Ls)
    for (int WG : WGs)
      for (int cap : caps) {
        if (WG < L) continue;
        if (L == s.L && WG == s.WG && cap == 0) continue;  // the base schedule itself
        out.push_back(fs_sched_hint{L, WG, cap, 0});
      }
  // looping kernels: the other number of row tiles per trip with the base shape
  if (s.grid < s.n_iters && s.CT == 1) out.push_back(fs_sched_hint{s.L, s.WG, 0, s.U == 1 ? 2 : 1});
  // row-reduction groups with [1,C] operands staged in LDS: one trip per workgroup against looping
  // workgroups that stage once (32 wavefronts per CU), whichever the base is not
  if (s.stage_rowv && base.col_reduces.empty() && s.CT == 1 && s.L <= 256) {
    const int wg_loop = s.L >= 128 ? std::min(1024, 4 * s.L) : 1024, wg_once = std::max(256, 4 * s.L);
    if (s.grid >= s.n_iters) out.push_back(fs_sched_hint{s.L, wg_loop, (int)(device_limits().resident_lanes / wg_loop), 0});
    else if (wg_once <= 1024) out.push_back(fs_sched_hint{s.L, wg_once, 1 << 20, 0});
  }
  return out;
}

bool choose_from_library(const Graph& g, const std::vector<int>& members, const std::vector<int>& group_of, int self_group,
                         const PlanOptions& opt, GroupPlan* gp) {
  // a candidate has to beat the analytic schedule by more than the noise of the measurement
  constexpr double kMargin = 0.95;
  double best = 0.0;
  const bool base_known = perflib_lookup(perf_key(*gp), &best);
  best *= kMargin;
  bool changed = false;
  GroupPlan cand;
  const std::vector<fs_sched_hint> hints = candidate_hints(*gp);
  for (const fs_sched_hint& h : hints) {
    PlanOptions o = opt;
    o.hint = h;
    o.has_hint = true;
    if (analyse_group(g, members, group_of, self_group, o, &cand) != FS_OK) continue;
    if (cand.s.L != h.lanes_per_row || cand.s.WG != h.wg_threads) continue;  // the hint was not legal for this group
    if (generate_kernel(g, &cand, self_group) != FS_OK) continue;
    double us = 0.0;
    if (!perflib_lookup(perf_key(cand), &us)) continue;
    // an unmeasured base schedule is not displaced: only compare within the library
    if (!base_known) continue;
    if (us < best) {
      best = us;
      *gp = cand;
      changed = true;
    }
  }
  return changed;
}

// -------------------------------------------------------------------------------------------
// Group formation.
//
// Unfused mode: one group per compute node.  Caller-given plan: checked, not changed.
// Otherwise a greedy producer/consumer fusion in the spirit of Algorithm 1 (Section 3.2):
// nodes are visited from the outputs upwards (the order of decreasing span); a node joins the
// group of one of its users when the three conditions of SchdConsistent hold:
//   1. no dependence cycle between groups would appear (the paper's `giveup` test),
//   2. it has a user in that group (producer/consumer fusion only),
//   3. the merged group still has a valid schedule and fits the LDS budget (analyse_group).
// -------------------------------------------------------------------------------------------
namespace {

// Performance feedback to the fusion decision (the role of the schedule planner's feedback edge,
// Section 2.2): a column reduction finished inside a kernel costs a ticketed grid-wide fold, a few
// microseconds of latency.  That is hidden behind the streaming of a large group, but for a
// launch-bound group it is dearer than the launch it saves, so small groups do not take one in.
bool worth_fusing(const GroupPlan& merged) {
  constexpr uint64_t kFoldWorthBytes = 16ull << 20;
  // A transposed root that cannot leave through an LDS tile (rows spread over a whole workgroup)
  // is written element by element, R elements apart: an order of magnitude slower than handing
  // the value to a kernel of its own that transposes in 2-D tiles (softmax + transpose of
  // [8192,4096]: 408 us fused, 95 us as two kernels); launch-bound groups keep it (one launch less).
  if (merged.members.size() > 1 && !merged.s.tile_transpose && !merged.s.tiled_transpose && merged.min_hbm_bytes >= kFoldWorthBytes)
    for (const ExtTensor& e : merged.ext_out)
      if (e.transposed) return false;
  // A handful of very long rows: one workgroup per row leaves most of the device idle, so such a
  // group, if its rows do not fit one workgroup's registers either, is only formed when its rows can
  // be split over workgroups.  Softmax of [8, 1M]: 286 us as
  // one kernel on 8 CUs, 38 us as three kernels that each fill the device; [32, 256K]: 73 -> 37 us;
  // from 64 rows on the single kernel is as fast or faster ([128, 64K]: 20 against 35 us).
  if (merged.members.size() > 1 && merged.s.few_long_rows && !merged.s.split_rows && merged.s.chunked && merged.R <= 32) return false;
  return merged.col_reduces.empty() || merged.members.size() == 1 || merged.s.grid == 1 || merged.min_hbm_bytes >= kFoldWorthBytes;
}

struct Former {
  const Graph& g;
  const PlanOptions& opt;
  std::vector<int> group_of;              // node -> group id, -1 unassigned/free
  std::vector<std::vector<int>> members;  // group id -> nodes
  std::vector<char> live;

  Former(const Graph& g_, const PlanOptions& o) : g(g_), opt(o), group_of(g_.n(), -1), live(g_.n(), 0) {}

  void mark_live() {
    std::vector<int> stack(g.outputs.begin(), g.outputs.end());
    while (!stack.empty()) {
      const int id = stack.back();
      stack.pop_back();
      if (live[id]) continue;
      live[id] = 1;
      for (int k = 0; k < g.nodes[id].num_in; ++k) stack.push_back(g.nodes[id].in[k]);
    }
  }

  // compute-node users of `id`, looking through broadcasts
  void real_users(int id, std::vector<int>* out) const {
    for (int u : g.users[id]) {
      if (!live[u]) continue;
      const int uop = g.nodes[u].opcode;
      if (uop == FS_BCAST_ROWVEC || uop == FS_BCAST_COLVEC || op_is_view(uop)) real_users(u, out);
      else out->push_back(u);
    }
  }

  // is group `to` reachable from group `from` along producer -> consumer edges?
  bool reaches(int from, int to) const {
    std::vector<char> seen(members.size(), 0);
    std::vector<int> stack{from};
    while (!stack.empty()) {
      const int grp = stack.back();
      stack.pop_back();
      if (grp == to) return true;
      if (seen[grp]) continue;
      seen[grp] = 1;
      for (int m : members[grp]) {
        std::vector<int> us;
        real_users(m, &us);
        for (int u : us)
          if (group_of[u] >= 0 && group_of[u] != grp && !seen[group_of[u]]) stack.push_back(group_of[u]);
      }
    }
    return false;
  }

  // direct producer -> consumer successors of a group
  std::set<int> successors(int grp) const {
    std::set<int> out;
    for (int m : members[grp]) {
      std::vector<int> us;
      real_users(m, &us);
      for (int u : us)
        if (group_of[u] >= 0 && group_of[u] != grp) out.insert(group_of[u]);
    }
    return out;
  }

  // Second pass: fuse groups that are not (only) producer and consumer of each other.  This is
  // the role of the paper's intra-layer ElementwiseFusion and of its multi-root computations
  // (Sections 3.2 and 4.3): kernels over the same work space are merged when they read a common
  // [R,C] tensor (one read instead of two) or when they are so small that the launch, not the
  // traffic, is what they cost (the tunable footprint threshold of Section 3.2).
  void merge_siblings() {
    constexpr uint64_t kFootprintThreshold = 16ull << 20;
    std::vector<GroupPlan> plan(members.size());
    std::vector<char> valid(members.size(), 0);
    auto analyse = [&](int grp) {
      valid[grp] = !members[grp].empty() && analyse_group(g, members[grp], group_of, grp, opt, &plan[grp]) == FS_OK;
    };
    for (size_t grp = 0; grp < members.size(); ++grp) analyse((int)grp);
    // The scan restarts from the first pair after every merge (which merge comes first decides the result: merging
    // is not confluent), but a pair whose merged group was analysed and refused is not analysed again until one of
    // the two groups has changed: the analysis is the expensive part, and it depends on the two member sets only.
    std::vector<int> version(members.size(), 0);
    std::map<std::pair<size_t, size_t>, std::pair<int, int>> refused;
    bool changed = true;
    GroupPlan merged_plan;
    while (changed) {
      changed = false;
      for (size_t a = 0; a < members.size() && !changed; ++a) {
        if (!valid[a]) continue;
        for (size_t b = a + 1; b < members.size() && !changed; ++b) {
          if (!valid[b]) continue;
          // work spaces must nest: equal, or one of them is a vector ([R,1] / [1,C]) of the other
          auto fits = [](int x, int y) { return x == y || x == 1 || y == 1; };
          // ... or do so after a flip (a transpose inside the merged group reorients one side)
          const bool straight = fits(plan[a].R, plan[b].R) && fits(plan[a].C, plan[b].C);
          const bool flipped = fits(plan[a].R, plan[b].C) && fits(plan[a].C, plan[b].R);
          if (!straight && !flipped) continue;
          if ((int)(members[a].size() + members[b].size()) > kMaxGroupMembers) continue;
          // profitable?
          bool share_full = false;
          for (const ExtTensor& x : plan[a].ext_in)
            for (const ExtTensor& y : plan[b].ext_in) share_full |= x.node == y.node && x.kind == KIND_FULL && y.kind == KIND_FULL;
          for (const ExtTensor& x : plan[a].ext_out)
            for (const ExtTensor& y : plan[b].ext_in) share_full |= x.node == y.node && y.kind == KIND_FULL;
          for (const ExtTensor& x : plan[b].ext_out)
            for (const ExtTensor& y : plan[a].ext_in) share_full |= x.node == y.node && y.kind == KIND_FULL;
          const bool small = plan[a].min_hbm_bytes + plan[b].min_hbm_bytes <= kFootprintThreshold;
          if (!share_full && !small) continue;
          // a path a -> c -> ... -> b through a third group would become a cycle
          bool cycle = false;
          for (int c : successors((int)a)) cycle |= c != (int)b && reaches(c, (int)b);
          for (int c : successors((int)b)) cycle |= c != (int)a && reaches(c, (int)a);
          if (cycle) continue;
          auto seen = refused.find({a, b});
          if (seen != refused.end() && seen->second == std::make_pair(version[a], version[b])) continue;
          std::vector<int> merged = members[a];
          merged.insert(merged.end(), members[b].begin(), members[b].end());
          if (analyse_group(g, merged, group_of, (int)a, opt, &merged_plan) != FS_OK || !worth_fusing(merged_plan)) {
            refused[{a, b}] = {version[a], version[b]};
            continue;
          }
          ++version[a];
          for (int m : members[b]) group_of[m] = (int)a;
          members[a] = merged;
          members[b].clear();
          valid[b] = 0;
          plan[a] = merged_plan;
          changed = true;
        }
      }
    }
  }

  // ---- Work/Span analysis (Section 3.1) --------------------------------------------------------
  // span = 0 for a node nothing live consumes (a root); otherwise 1 + the largest span among its
  // users (broadcasts are looked through: they are inlined, not instructions of their own).
  // Nodes of equal span form a layer and do not depend on each other.
  std::vector<int> spans() const {
    std::vector<int> span(g.n(), -1);
    for (int id = g.n() - 1; id >= 0; --id) {
      if (!live[id] || op_is_free(g.nodes[id].opcode)) continue;
      std::vector<int> us;
      real_users(id, &us);
      int sp = 0;
      for (int u : us) sp = std::max(sp, span[u] + 1);
      span[id] = sp;
    }
    return span;
  }

  static bool is_elementwise(int op) { return op_is_unary(op) || op_is_binary(op) || op == FS_CMP || op == FS_SELECT; }

  // ---- the layered planner: Section 3.2 as written ----------------------------------------------
  // For every layer from the roots upwards: (1) intra-layer ElementwiseFusion of the layer's still
  // unassigned elementwise nodes (schedule-compatible, fused footprint under the threshold);
  // (2) for every fusion root of the layer, Algorithm 1: walk the layers above it, fuse a node
  // when SchdConsistent holds, otherwise put it in `giveup`.
  void plan_layered() {
    constexpr uint64_t kFootprintThreshold = 16ull << 20;
    const std::vector<int> span = spans();
    int max_span = -1;
    for (int sp : span) max_span = std::max(max_span, sp);
    std::vector<std::vector<int>> layer(max_span + 1);
    for (int id = 0; id < g.n(); ++id)
      if (span[id] >= 0) layer[span[id]].push_back(id);
    GroupPlan scratch;
    for (int s = 0; s <= max_span; ++s) {
      // (1) ElementwiseFusion among the unassigned nodes of this layer
      std::vector<int> roots;  // group ids created in this layer
      for (int id : layer[s]) {
        if (group_of[id] >= 0) continue;
        int joined = -1;
        if (is_elementwise(g.nodes[id].opcode)) {
          for (int grp : roots) {
            if (!is_elementwise(g.nodes[members[grp][0]].opcode)) continue;
            std::vector<int> merged = members[grp];
            merged.push_back(id);
            if (analyse_group(g, merged, group_of, grp, opt, &scratch) != FS_OK) continue;
            if (scratch.min_hbm_bytes > kFootprintThreshold) continue;
            joined = grp;
            break;
          }
        }
        if (joined < 0) {
          joined = (int)members.size();
          members.push_back({});
          roots.push_back(joined);
        }
        group_of[id] = joined;
        members[joined].push_back(id);
      }
      // (2) Algorithm 1 from every fusion root of this layer
      for (int grp : roots) {
        std::set<int> giveup;
        for (int l = s + 1; l <= max_span; ++l) {
          for (int hlo : layer[l]) {
            if (group_of[hlo] >= 0) continue;
            std::vector<int> us;
            real_users(hlo, &us);
            bool user_gave_up = false, user_fused = false;
            for (int u : us) {
              user_gave_up |= giveup.count(u) != 0;
              user_fused |= group_of[u] == grp;
            }
            bool ok = !user_gave_up && user_fused;  // SchdConsistent, tests 1 and 2
            if (ok) {
              // (exact form of test 1 for users that already belong to other fused computations)
              for (int u : us) {
                const int h = group_of[u];
                if (h >= 0 && h != grp && reaches(h, grp)) ok = false;
              }
            }
            if (ok) {  // test 3: an optimised schedule (and LDS plan) for the fused computation exists
              std::vector<int> merged = members[grp];
              merged.push_back(hlo);
              ok = (int)merged.size() <= 96 && analyse_group(g, merged, group_of, grp, opt, &scratch) == FS_OK && worth_fusing(scratch);
            }
            if (ok) {
              group_of[hlo] = grp;
              members[grp].push_back(hlo);
            } else {
              giveup.insert(hlo);
            }
          }
        }
      }
    }
  }

  fs_status topo_order(std::vector<std::vector<int>>* ordered) const {
    const int NG = (int)members.size();
    std::vector<std::set<int>> succ(NG);
    std::vector<int> indeg(NG, 0);
    for (int grp = 0; grp < NG; ++grp)
      for (int m : members[grp]) {
        std::vector<int> us;
        real_users(m, &us);
        for (int u : us) {
          const int h = group_of[u];
          if (h >= 0 && h != grp && succ[grp].insert(h).second) ++indeg[h];
        }
      }
    // Kahn, smallest first-member id first (stable, close to the caller's order)
    auto key = [&](int grp) { return *std::min_element(members[grp].begin(), members[grp].end()); };
    std::set<std::pair<int, int>> ready;
    for (int grp = 0; grp < NG; ++grp)
      if (!members[grp].empty() && indeg[grp] == 0) ready.insert({key(grp), grp});
    size_t placed = 0, nonempty = 0;
    for (int grp = 0; grp < NG; ++grp) nonempty += !members[grp].empty();
    while (!ready.empty()) {
      const int grp = ready.begin()->second;
      ready.erase(ready.begin());
      ordered->push_back(members[grp]);
      ++placed;
      for (int h : succ[grp])
        if (--indeg[h] == 0) ready.insert({key(h), h});
    }
    if (placed != nonempty) FS_FAIL(FS_ERR_UNSUPPORTED, "the grouping has a dependence cycle between groups");
    return FS_OK;
  }
};

}  // namespace

fs_status form_groups(const Graph& g, const fs_graph_desc* desc, const PlanOptions& opt, std::vector<int>* group_of,
                      std::vector<std::vector<int>>* ordered) {
  Former f(g, opt);
  f.mark_live();
  const int N = g.n();
  GroupPlan scratch;

  if (opt.mode == FS_MODE_UNFUSED) {
    for (int id = 0; id < N; ++id)
      if (f.live[id] && !op_is_free(g.nodes[id].opcode)) {
        f.group_of[id] = (int)f.members.size();
        f.members.push_back({id});
      }
  } else if (desc->group_of_node) {
    std::map<int, int> remap;
    for (int id = 0; id < N; ++id) {
      if (!f.live[id] || op_is_free(g.nodes[id].opcode)) continue;
      const int want = desc->group_of_node[id];
      if (want < 0) FS_FAIL(FS_ERR_INVALID_ARG, "group_of_node[%d] = %d", id, want);
      auto it = remap.find(want);
      if (it == remap.end()) {
        it = remap.insert({want, (int)f.members.size()}).first;
        f.members.push_back({});
      }
      f.group_of[id] = it->second;
      f.members[it->second].push_back(id);
    }
  } else if (opt.layered) {
    f.plan_layered();
  } else {
    for (int id = N - 1; id >= 0; --id) {
      if (!f.live[id] || op_is_free(g.nodes[id].opcode)) continue;
      std::vector<int> us;
      f.real_users(id, &us);
      // candidate groups: those of its users, most users first
      std::map<int, int> votes;
      for (int u : us)
        if (f.group_of[u] >= 0) ++votes[f.group_of[u]];
      std::vector<std::pair<int, int>> cands;
      for (auto& kv : votes) cands.push_back({-kv.second, kv.first});
      std::sort(cands.begin(), cands.end());
      int joined = -1;
      for (auto& cand : cands) {
        const int grp = cand.second;
        // condition 1: joining must not close a cycle through a user left outside
        bool cycle = false;
        for (int u : us) {
          const int h = f.group_of[u];
          if (h >= 0 && h != grp && f.reaches(h, grp)) {
            cycle = true;
            break;
          }
        }
        if (cycle) continue;
        // condition 3: schedule and LDS plan of the merged group
        std::vector<int> merged = f.members[grp];
        merged.push_back(id);
        if ((int)merged.size() > kMaxGroupMembers) continue;
        if (analyse_group(g, merged, f.group_of, grp, opt, &scratch) != FS_OK) continue;
        if (!worth_fusing(scratch)) continue;
        joined = grp;
        break;
      }
      if (joined < 0) {
        joined = (int)f.members.size();
        f.members.push_back({});
      }
      f.group_of[id] = joined;
      f.members[joined].push_back(id);
    }
    f.merge_siblings();
  }
  *group_of = f.group_of;
  return f.topo_order(ordered);
}

void recompute_across_kernels(const Graph& g, const PlanOptions& opt, std::vector<int>* group_of,
                              std::vector<std::vector<int>>* ordered, CloneInfo* ci) {
  const int NG = (int)ordered->size();
  ci->group_of = *group_of;
  ci->extra.clear();
  if (NG < 2) return;
  PlanOptions o = opt;
  o.clones = ci;
  std::vector<GroupPlan> gps(NG);
  for (int gi = 0; gi < NG; ++gi)
    if (analyse_group(g, (*ordered)[gi], *group_of, gi, o, &gps[gi]) != FS_OK) return;  // (plan creation reports it)
  auto elementwise = [&](int op) { return op_is_unary(op) || op_is_binary(op) || op == FS_CMP || op == FS_SELECT; };
  auto in_list = [](const std::vector<ExtTensor>& l, int node) {
    for (const ExtTensor& e : l)
      if (e.node == node) return true;
    return false;
  };
  for (int b = 1; b < NG; ++b) {
    for (int round = 0; round < 16; ++round) {  // a copy may expose its own producer
      bool changed = false;
      const std::vector<ExtTensor> reads = gps[b].ext_in;
      for (const ExtTensor& e : reads) {
        const int t = e.node;
        const fs_node& n = g.nodes[t];
        if (e.kind != KIND_FULL || ci->group_of[t] < 0 || !elementwise(n.opcode) || ci->computed_in(t, b)) continue;
        if (g.family_output[t] >= 0) continue;  // a plan output exists in memory anyway: reading it is as cheap as its operands
        // every reader inside b takes it as a plain operand (not under another shape), and nobody views it
        bool plain = true;
        for (int u : g.users[t]) plain &= !op_is_view(g.nodes[u].opcode);
        for (int m : (*ordered)[b])
          for (int k = 0; k < g.nodes[m].num_in; ++k) plain &= !(g.nodes[m].in[k] == t && g.flat_in[m][k]);
        if (!plain) continue;
        // the value and, with it, those of its elementwise producers that exist in no memory: everything else they read has to
        // be there already (plan inputs, values some kernel stores anyway, vectors)
        std::vector<int> T, stack{t};
        bool available = true;
        while (!stack.empty() && available) {
          const int x = stack.back();
          stack.pop_back();
          if (std::find(T.begin(), T.end(), x) != T.end()) continue;
          T.push_back(x);
          if (T.size() > 8) available = false;
          const fs_node& xn = g.nodes[x];
          for (int k = 0; k < xn.num_in && available; ++k) {
            int src = xn.in[k];
            if (g.flat_in[x][k]) available = false;
            while (g.nodes[src].opcode == FS_BCAST_ROWVEC || g.nodes[src].opcode == FS_BCAST_COLVEC) src = g.nodes[src].in[0];
            const fs_node& sn = g.nodes[src];
            if (sn.opcode == FS_CONST || sn.opcode == FS_INPUT) continue;
            const int h = ci->group_of[src];
            if (h >= 0 && ci->computed_in(src, b)) continue;
            if (h < 0 || h >= b) available = false;  // (a view; or not a value of an earlier kernel)
            else if (in_list(gps[h].ext_out, src)) continue;
            else if ((int64_t)sn.rows * sn.cols < (int64_t)n.rows * n.cols) continue;  // a vector: storing it costs next to nothing
            else if (elementwise(sn.opcode)) stack.push_back(src);
            else available = false;
          }
        }
        // (bytes are what is scarce, but not free of charge: at most two transcendental or division-like operations are
        // computed a second time for one value)
        int dear = 0;
        for (int x : T) dear += op_is_approx(g.nodes[x].opcode) || g.nodes[x].opcode == FS_DIV || g.nodes[x].opcode == FS_SQRT;
        if (!available || dear > 2) continue;
        // every producer keeps what it still uses itself
        CloneInfo trial = *ci;
        std::map<int, std::vector<int>> mm;  // member lists of the kernels that change
        mm[b] = (*ordered)[b];
        std::sort(T.begin(), T.end());
        for (int i = (int)T.size() - 1; i >= 0; --i) {  // consumers before producers
          const int x = T[i], a = trial.group_of[x];
          if (!mm.count(a)) mm[a] = (*ordered)[a];
          std::vector<int>& ma = mm[a];
          // it stays in its kernel while something there uses it, or while a third kernel reads it from memory
          // (the first kernel that computes a value is the one that stores it, and that one runs before every reader)
          bool stays = false;
          for (int u : g.users[x]) {
            std::vector<int> chain{u};
            while (!chain.empty()) {
              const int y = chain.back();
              chain.pop_back();
              const int yop = g.nodes[y].opcode;
              if (yop == FS_BCAST_ROWVEC || yop == FS_BCAST_COLVEC) {
                chain.insert(chain.end(), g.users[y].begin(), g.users[y].end());
                continue;
              }
              stays |= std::find(ma.begin(), ma.end(), y) != ma.end() || op_is_view(yop);
              auto other = [&](int h) { return h >= 0 && h != a && h != b && !trial.computed_in(x, h); };
              stays |= other(trial.group_of[y]);
              auto it = trial.extra.find(y);
              if (it != trial.extra.end())
                for (int h : it->second) stays |= other(h);
            }
          }
          mm[b].push_back(x);
          if (stays) {
            trial.extra[x].insert(b);
          } else {
            ma.erase(std::find(ma.begin(), ma.end(), x));
            trial.group_of[x] = b;
            trial.extra[x].erase(b);
          }
        }
        bool fits = (int)mm[b].size() <= kMaxGroupMembers;
        for (auto& kv : mm) fits &= !kv.second.empty();
        if (!fits) continue;
        PlanOptions ot = opt;
        ot.clones = &trial;
        std::map<int, GroupPlan> np;
        uint64_t before = 0, after = 0;
        for (auto& kv : mm) {
          fits = fits && analyse_group(g, kv.second, trial.group_of, kv.first, ot, &np[kv.first]) == FS_OK;
          if (!fits) break;
          before += gps[kv.first].min_hbm_bytes;
          after += np[kv.first].min_hbm_bytes;
        }
        if (!fits || after >= before || !worth_fusing(np[b])) continue;
        // a kernel that changes its form for the copy (rows no longer held in registers, another launch shape class) is not worth it
        if (np[b].s.chunked != gps[b].s.chunked || np[b].s.split_rows != gps[b].s.split_rows || np[b].s.col_tiled != gps[b].s.col_tiled) continue;
        for (auto& kv : mm) {
          (*ordered)[kv.first] = kv.second;
          gps[kv.first] = np[kv.first];
        }
        *ci = trial;
        changed = true;
        break;
      }
      if (!changed) break;
    }
  }
  *group_of = ci->group_of;
}

void work_span(const Graph& g, std::vector<int>* span) {
  PlanOptions opt;
  Former f(g, opt);
  f.mark_live();
  *span = f.spans();
}

}  // namespace fs
