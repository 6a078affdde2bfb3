// fs_codegen.cpp - emits the HIP source of one fused group's stitched kernel.
//
// Structure of the emitted kernel (the realisation of Algorithm 2, Section 5.2):
//   - an op that is neither a root, nor a reduction, nor kept in shared memory is emitted
//     inline, element by element, into the registers of the lane that owns the element
//     (the ElementalIrEmitter branch: thread composition);
//   - a row reduction ends a stage: lanes fold their own elements, the wavefront folds by
//     lane permutes, wavefronts of one row meet in LDS (EmitWriteSharedArray), and the
//     consumers of the result continue in the same kernel (block composition);
//   - roots are written to global memory as soon as they exist (EmitWriteOutputArray).
// The body is straight-line code over the building blocks of fs_device.h; names are local
// indices, so two groups with the same structure produce the same text and share a binary.
//
// Two peephole rules keep the instruction count down (on this device 4 bytes of HBM traffic
// pay for only ~20 scalar fp32 instructions, so arithmetic is never free):
//   - a multiply whose only consumer is an add/sub (or a sum reduction) is contracted into an
//     fma, unless one of the two feeds a predicate: predicates must see exactly the roundings
//     the graph spells out;
//   - a value that is only stored is not rounded to its dtype in registers first (the store
//     rounds);
//   - two per-column operands ([1,C] tensors from memory) that enter a chain of additions one
//     after the other, (p + beta) + bias, are added to each other once per workgroup instead of
//     once per element: p + (beta + bias).  This reassociates, so it is not done on predicate
//     paths either; elsewhere the result moves by one rounding, as with the fma contraction.
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <functional>
#include <set>
#include <sstream>

#include "fs_internal.h"

namespace fs {

namespace {

struct Emitter {
  const Graph& g;
  GroupPlan& gp;
  std::ostringstream os;
  std::map<int, int> local;  // node id -> local index
  std::vector<char> in_set;
  std::vector<int> uses;      // in-group operand slots reading each member (looking through broadcasts)
  std::vector<char> folded;   // multiply emitted inside its single consumer
  // z = (p +- Ra) +- Rb with Ra, Rb per-column tensors from memory used nowhere else: emitted as +-p + (+-Ra +- Rb)
  struct Comb {
    int z, m, p;      // the outer add/sub, the inner one (absorbed: never emitted), the remaining operand (as m names it)
    int ra, rb;       // the two [1,C] tensors
    bool neg_a, neg_b, neg_p;
  };
  std::vector<Comb> combs;
  std::map<int, int> comb_of;      // z -> index into combs
  std::vector<char> absorbed;      // inner add/sub of a comb
  std::map<int, int> ext_uses;     // [1,C] tensor from memory -> operand slots reading it
  std::map<int, int> slot_of_ext;  // staged [1,C] tensor -> LDS slot
  std::vector<int> slot_of_comb;   // comb -> LDS slot
  int n_slots = 0;

  Emitter(const Graph& g_, GroupPlan& gp_)
      : g(g_), gp(gp_), in_set(g_.n(), 0), uses(g_.n(), 0), folded(g_.n(), 0), absorbed(g_.n(), 0) {}

  int loc(int node) {
    auto it = local.find(node);
    if (it != local.end()) return it->second;
    const int idx = (int)local.size();
    local[node] = idx;
    return idx;
  }
  static const char* prefix(Kind k) { return k == KIND_FULL ? "v" : k == KIND_COLV ? "s" : "r"; }
  std::string name(int node, Kind k) { return std::string(prefix(k)) + std::to_string(loc(node)); }

  static std::string literal(float f, int dtype) {
    uint32_t u;
    memcpy(&u, &f, 4);
    char buf[96];
    snprintf(buf, sizeof(buf), "fs_round<%d>(fs_lit(0x%08xu /* %.9g */))", dtype, u, (double)f);
    return buf;
  }

  // the tensor behind an operand: looks through a broadcast, and through transposes that are
  // members of the group (they only flip the orientation flag; the registers are the producer's)
  int source_of(int o) const {
    const fs_node* n = &g.nodes[o];
    if (n->opcode == FS_BCAST_ROWVEC || n->opcode == FS_BCAST_COLVEC) {
      o = n->in[0];
      n = &g.nodes[o];
    }
    while (n->opcode == FS_TRANSPOSE && in_set[o] && in_set[n->in[0]]) {
      o = n->in[0];
      n = &g.nodes[o];
    }
    return o;
  }
  // a member transpose of an in-group value has no registers of its own
  bool is_alias(int m) const { return g.nodes[m].opcode == FS_TRANSPOSE && in_set[g.nodes[m].in[0]]; }
  bool is_col_reduce(int m) const { return std::find(gp.col_reduces.begin(), gp.col_reduces.end(), m) != gp.col_reduces.end(); }

  const ExtTensor* find_out(int node) const {
    for (const ExtTensor& e : gp.ext_out)
      if (e.node == node) return &e;
    return nullptr;
  }

  // may multiply `m` be emitted inside consumer `u` as part of an fma?
  bool can_fold_mul(int m, int u) const {
    if (m < 0 || !in_set[m]) return false;
    const fs_node& mn = g.nodes[m];
    const fs_node& un = g.nodes[u];
    const bool reduce = un.opcode == FS_REDUCE_ROW || un.opcode == FS_REDUCE_COL;
    return mn.opcode == FS_MUL && uses[m] == 1 && !find_out(m) && mn.dtype == FS_F32 && un.dtype == FS_F32 && !g.exact[m] &&
           !g.exact[u] && gp.kind.at(m) == (reduce ? KIND_FULL : gp.kind.at(u));
  }

  // expression for element e of operand `o` (indexable by `e` inside an unrolled loop)
  std::string ref(int o) {
    const fs_node& n = g.nodes[o];
    if (n.opcode == FS_CONST) return literal(n.attr_f, n.dtype);
    const int src = source_of(o);
    if (g.nodes[src].opcode == FS_CONST) return literal(g.nodes[src].attr_f, g.nodes[src].dtype);
    const Kind k = gp.kind.at(src);
    if (k == KIND_COLV) return name(src, k);
    return name(src, k) + "[e]";
  }

  std::string expr(int id) {
    const fs_node& n = g.nodes[id];
    auto A = [&]() { return ref(n.in[0]); };
    auto B = [&]() { return ref(n.in[1]); };
    auto Cc = [&]() { return ref(n.in[2]); };
    switch (n.opcode) {
      case FS_NEG: return "-(" + A() + ")";
      case FS_ABS: return "__builtin_fabsf(" + A() + ")";
      case FS_EXP: return "fs_exp(" + A() + ")";
      case FS_LOG: return "fs_log(" + A() + ")";
      case FS_TANH: return "fs_tanh(" + A() + ")";
      case FS_SIGMOID: return "fs_sigmoid(" + A() + ")";
      case FS_SQRT: return "fs_sqrt(" + A() + ")";
      case FS_RSQRT: return "fs_rsqrt(" + A() + ")";
      case FS_RCP: return "fs_rcp(" + A() + ")";
      case FS_GELU_TANH: return "fs_gelu_tanh(" + A() + ")";
      case FS_CONVERT: return "(" + A() + ")";
      case FS_ADD:
      case FS_SUB: {
        const bool sub = n.opcode == FS_SUB;
        if (comb_of.count(id)) {
          const Comb& c = combs[comb_of.at(id)];
          const std::string rc = "rc" + std::to_string(loc(c.z)) + "[e]";
          if (folded[c.p]) {
            const fs_node& mn = g.nodes[c.p];
            return "__builtin_fmaf(" + std::string(c.neg_p ? "-(" : "(") + ref(mn.in[0]) + "), " + ref(mn.in[1]) + ", " + rc + ")";
          }
          return c.neg_p ? "(" + rc + " - " + ref(c.p) + ")" : "(" + ref(c.p) + " + " + rc + ")";
        }
        for (int side = 0; side < 2; ++side) {
          const int m = n.in[side];
          if (!folded[m]) continue;
          const fs_node& mn = g.nodes[m];
          const std::string x = ref(mn.in[0]), y = ref(mn.in[1]), other = ref(n.in[1 - side]);
          if (!sub) return "__builtin_fmaf(" + x + ", " + y + ", " + other + ")";
          if (side == 0) return "__builtin_fmaf(" + x + ", " + y + ", -(" + other + "))";  // m - c
          return "__builtin_fmaf(-(" + x + "), " + y + ", " + other + ")";                 // c - m
        }
        return "(" + A() + (sub ? " - " : " + ") + B() + ")";
      }
      case FS_MUL: return "(" + A() + " * " + B() + ")";
      case FS_DIV: return "fs_div(" + A() + ", " + B() + ")";
      case FS_MAX: return "fs_max(" + A() + ", " + B() + ")";
      case FS_MIN: return "fs_min(" + A() + ", " + B() + ")";
      case FS_CMP: {
        static const char* ops[] = {">", ">=", "<", "<=", "==", "!="};
        return "((" + A() + " " + ops[n.attr_i] + " " + B() + ") ? 1.0f : 0.0f)";
      }
      case FS_SELECT: return "((" + A() + " != 0.0f) ? " + B() + " : " + Cc() + ")";
      case FS_REDUCE_ROW:  // degenerate (one column): the value itself
      case FS_REDUCE_COL:  // degenerate (one row)
        return "(" + A() + ")";
    }
    return "0.0f";
  }

  // value of node `id` rounded to its dtype, unless it is only stored (the store rounds)
  std::string rounded(int id, const std::string& e) {
    const fs_node& n = g.nodes[id];
    if (n.dtype != FS_BF16 || (uses[id] == 0 && find_out(id))) return e;
    return "fs_round<" + std::to_string(n.dtype) + ">(" + e + ")";
  }

  static std::string tmpl_row() { return "V, NVL, L, NV, RAGGED"; }

  // The last stage of a row-reduction body (everything after the last exchange: normalise, scale,
  // activation, stores) can be emitted vector by vector: the same statements inside a loop over
  // the lane's NVL vectors, each touching the V elements of vector j only.  Operands that are read
  // where they are used (staged or reloaded [1,C] tensors) and the values on their way to a store
  // are then live for one vector at a time instead of the whole slice (LayerNorm+bias+GeLU with
  // 16 elements per lane: 66 -> 61 registers, i.e. 8 instead of 7 wavefronts per SIMD).
  bool strip = false;
  std::ostringstream pre;  // while `strip`: array declarations and per-row scalars, placed before the loop
  std::string eloop() const {
    return strip ? "_Pragma(\"unroll\") for (int e = j * V; e < (j + 1) * V; ++e) " : "_Pragma(\"unroll\") for (int e = 0; e < E; ++e) ";
  }
  void declare(const std::string& nm, const std::string& ind) { (strip ? pre : os) << ind << "float " << nm << "[E];\n"; }
  // row-slice calls: whole slice, or vector j of it
  std::string vec_fn(const char* fn) const { return std::string(fn) + (strip ? "_vec" : ""); }
  std::string vec_arg() const { return strip ? ", j" : ""; }

  // an array holding operand `o` as a full slice (needed by max/min reductions / transposed stores)
  std::string as_array(int o, const std::string& tag) {
    o = source_of(o) == o || !op_is_free(g.nodes[o].opcode) ? source_of(o) : o;
    const fs_node& n = g.nodes[o];
    if ((!op_is_free(n.opcode) || n.opcode == FS_INPUT) && !folded[o]) {
      const Kind k = gp.kind.at(o);
      if (k != KIND_COLV) return name(o, k);
    }
    const std::string t = "t" + tag;
    os << "    float " << t << "[E];\n    _Pragma(\"unroll\") for (int e = 0; e < E; ++e) " << t << "[e] = "
       << (folded[o] ? expr(o) : ref(o)) << ";\n";
    return t;
  }

  void emit_store(const ExtTensor& e, const std::string& indent) {
    const int holder = source_of(e.node);  // an aliasing transpose stores its producer's registers
    const std::string nm = name(holder, gp.kind.at(holder));
    if (e.transposed) {
      // the value leaves in the flipped orientation: through a padded LDS tile when the plan has one
      if (gp.s.tile_transpose) {
        // tensors far larger than the caches leave with non-temporal stores, like the plain row stores
        // (transposes of 256-512 MB: 2-5 % faster; 16 MB and u8: not)
        const bool nt = dtype_size(e.dtype) >= 2 && (uint64_t)g.nodes[e.node].rows * g.nodes[e.node].cols * dtype_size(e.dtype) >= (32ull << 20);
        os << indent << "fs_store_tile_transposed<" << e.dtype << ", " << tmpl_row() << ", WG, TCW, C, " << (nt ? "true" : "false") << ">(" << nm << ", lds_tile, a.p[" << e.arg
           << "], R, row - rg, lir, rg, vbase);\n";
      } else
        os << indent << "fs_store_row_transposed<" << e.dtype << ", " << tmpl_row() << ">(" << nm << ", a.p[" << e.arg
           << "], R, row, lir, vbase, rok);\n";
      return;
    }
    if (e.kind == KIND_FULL)
      os << indent << vec_fn("fs_store_row") << "<" << e.dtype << ", " << tmpl_row() << ", " << (e.streaming ? "true" : "false") << ">(" << nm
         << ", a.p[" << e.arg << "], row0, lir, vbase, rok" << vec_arg() << ");\n";
    else if (e.kind == KIND_COLV)
      (strip ? pre : os) << indent << "if (rok && lir == 0 && vbase == 0) fs_store1<" << e.dtype << ">(a.p[" << e.arg << "], row, " << nm << ");\n";
  }

  // the [1,C] tensor from memory behind operand `o`, or -1
  int ext_rowv_of(int o) const {
    if (g.nodes[o].opcode == FS_CONST) return -1;
    const int src = source_of(o);
    if (g.nodes[src].opcode == FS_CONST || in_set[src]) return -1;
    auto it = gp.kind.find(src);
    return it != gp.kind.end() && it->second == KIND_ROWV ? src : -1;
  }

  void find_combs() {
    for (int z : gp.members) {
      const fs_node& zn = g.nodes[z];
      if ((zn.opcode != FS_ADD && zn.opcode != FS_SUB) || zn.dtype != FS_F32 || g.exact[z] || gp.kind.at(z) != KIND_FULL) continue;
      for (int side = 0; side < 2; ++side) {
        const int rb = ext_rowv_of(zn.in[side]), m = zn.in[1 - side];
        if (rb < 0 || !in_set[m] || absorbed[m] || folded[m] || comb_of.count(m)) continue;
        const fs_node& mn = g.nodes[m];
        if ((mn.opcode != FS_ADD && mn.opcode != FS_SUB) || mn.dtype != FS_F32 || g.exact[m] || uses[m] != 1 || find_out(m) ||
            gp.kind.at(m) != KIND_FULL || gp.level.at(m) != gp.level.at(z))
          continue;
        bool done = false;
        for (int side2 = 0; side2 < 2 && !done; ++side2) {
          const int ra = ext_rowv_of(mn.in[side2]), pp = mn.in[1 - side2];
          if (ra < 0 || ra == rb || ext_uses[ra] != 1 || ext_uses[rb] != 1 || ext_rowv_of(pp) >= 0) continue;
          // m = s1*p + t1*Ra, z = s2*m + t2*Rb  (s, t = +-1)
          const bool msub = mn.opcode == FS_SUB, zsub = zn.opcode == FS_SUB;
          const int s1 = (msub && side2 == 0) ? -1 : 1, t1 = (msub && side2 == 1) ? -1 : 1;   // operand `side2` is Ra
          const int s2 = (zsub && side == 0) ? -1 : 1, t2 = (zsub && side == 1) ? -1 : 1;     // operand `side` is Rb
          Comb c;
          c.z = z, c.m = m, c.p = pp, c.ra = ra, c.rb = rb;
          c.neg_p = s2 * s1 < 0, c.neg_a = s2 * t1 < 0, c.neg_b = t2 < 0;
          comb_of[z] = (int)combs.size();
          combs.push_back(c);
          absorbed[m] = 1;
          done = true;
        }
        if (done) break;
      }
    }
  }

  void count_uses() {
    for (int m : gp.members) {
      const fs_node& n = g.nodes[m];
      for (int k = 0; k < n.num_in; ++k) {
        const int src = source_of(n.in[k]);
        if (in_set[src]) ++uses[src];
        const int r = ext_rowv_of(n.in[k]);
        if (r >= 0) ++ext_uses[r];
      }
    }
    // decide which multiplies disappear into their consumer
    for (int u : gp.members) {
      const fs_node& un = g.nodes[u];
      if (un.opcode == FS_ADD || un.opcode == FS_SUB) {
        for (int side = 0; side < 2; ++side) {
          const int m = un.in[side];  // direct operand only (a broadcast in between changes the kind)
          if (can_fold_mul(m, u) && !folded[un.in[1 - side]]) {
            folded[m] = 1;
            break;
          }
        }
      } else if ((un.opcode == FS_REDUCE_ROW || un.opcode == FS_REDUCE_COL) && (un.attr_i == FS_RED_SUM || un.attr_i == FS_RED_MEAN) &&
                 gp.R > 1 && gp.C > 1) {
        if (can_fold_mul(un.in[0], u)) folded[un.in[0]] = 1;
      }
    }
  }

  // ---- rows walked in column chunks (Schedule::chunked) ----------------------------------------
  // [R,C] and [1,C] members (and tensors from memory) that `targets` depend on without crossing a
  // row reduction: what one pass over the row has to load and recompute.
  // `avail`: members whose chunk is read back from LDS instead (buffered by an earlier pass): the walk stops there
  // and lists them in `from_lds`.
  void needed_for(const std::vector<int>& targets, std::set<int>* mem, std::set<int>* ext, const std::set<int>* avail = nullptr,
                  std::set<int>* from_lds = nullptr) {
    std::vector<int> stack(targets);
    while (!stack.empty()) {
      const int id = stack.back();
      stack.pop_back();
      const fs_node& n = g.nodes[id];
      for (int k = 0; k < n.num_in; ++k) {
        if (g.nodes[n.in[k]].opcode == FS_CONST) continue;
        const int src = source_of(n.in[k]);
        if (g.nodes[src].opcode == FS_CONST) continue;
        const Kind kd = gp.kind.at(src);
        if (kd == KIND_COLV) continue;  // one value per row: exists before the pass starts
        if (!in_set[src]) ext->insert(src);
        else if (avail && avail->count(src)) from_lds->insert(src);
        else if (mem->insert(src).second) stack.push_back(src);
      }
    }
  }

  void emit_exchange(const std::vector<int>& batch, bool xwave, int WPR, int KB, const std::string& ind) {
    for (int b : batch)
      os << ind << "q" << loc(b) << " = fs_segment_allreduce<" << g.nodes[b].attr_i << ", (L < 64 ? L : 64)>(q" << loc(b) << ");\n";
    if (xwave) {
      os << ind << "{\n" << ind << "  const fs_xwave<" << KB << ", " << WPR << "> xw{lds_rr + (parity * G + rg) * " << WPR * KB
         << ", lir >> 6, (tid & 63) == 0};\n";
      for (size_t k = 0; k < batch.size(); ++k) os << ind << "  xw.put(" << k << ", q" << loc(batch[k]) << ");\n";
      os << ind << "  fs_lds_barrier();\n";
      for (size_t k = 0; k < batch.size(); ++k)
        os << ind << "  q" << loc(batch[k]) << " = xw.get<" << g.nodes[batch[k]].attr_i << ">(" << k << ");\n";
      os << ind << "  parity ^= 1;\n" << ind << "}\n";
    }
    for (int b : batch) {
      const fs_node& bn = g.nodes[b];
      const std::string q = "q" + std::to_string(loc(b));
      os << ind << "const float " << name(b, KIND_COLV) << " = " << rounded(b, bn.attr_i == FS_RED_MEAN ? q + " / (float)C" : q) << ";\n";
      if (const ExtTensor* e = find_out(b)) emit_store(*e, ind);
    }
  }

  // One pass over the row: loads, the members the targets need in id order, then `tail` per chunk.
  // Passes alternate their direction: a pass starts with the chunks its predecessor touched
  // last, the ones most likely still in the L2.
  //
  // Shared-memory planning (Section 5.1) for these kernels: a value that several passes need - an [R,C] input, or an
  // elementwise result - may keep the first STAGE_CHUNKS chunks of the row in an LDS slot (GroupPlan::stage_slots, chosen
  // by plan_stage_buffers below).  The first pass that loads / computes it writes the slot; later passes read it back
  // and compute only what lies between it and their targets.  Chunks beyond STAGE_CHUNKS are recomputed from memory,
  // as without the buffer: such a pass has two bodies, chosen per chunk.
  int n_passes = 0;
  std::map<int, int> pass_loads;     // [R,C] input -> passes that load it      } without buffers: the dry run's counts
  std::map<int, int> pass_computes;  // [R,C] member -> passes that compute it  } (see plan_stage_buffers)
  std::map<int, int> first_pass;     // ... and the first of them
  std::map<int, int> pass_loads_planned;  // [R,C] input -> passes that load it where the row is buffered, with the plan's buffers in place
  std::set<int> stage_written;       // buffered values whose slot has been written by an earlier pass
  bool staged(int node) const { return gp.s.stage_chunks > 0 && gp.stage_slot_of.count(node) > 0; }
  long chunk_bytes(int elem_bytes) const { return (long)gp.s.NVLC * gp.s.L * gp.s.V * elem_bytes; }
  // byte offset of `node`'s slot inside lds_stage, or -1
  long stage_offset(int node) const {
    auto it = gp.stage_slot_of.find(node);
    if (it == gp.stage_slot_of.end()) return -1;
    long off = 0;
    for (int k = 0; k < it->second; ++k) off += gp.s.stage_chunks * chunk_bytes(gp.stage_slots[k].elem_bytes);
    return off;
  }
  std::string stage_chunk(int node) const {
    return "lds_stage + " + std::to_string(stage_offset(node)) + " + (long)ch * " + std::to_string(chunk_bytes(dtype_size(g.nodes[node].dtype)));
  }

  template <class Tail>
  void emit_pass_body(const std::set<int>& mem, const std::set<int>& ext, const std::set<int>& from_lds, bool store_outputs, Tail tail) {
    for (const ExtTensor& e : gp.ext_in) {
      if (!ext.count(e.node)) continue;
      os << "      float " << name(e.node, e.kind) << "[E];\n";
      if (e.kind == KIND_FULL) {
        const std::string nm = name(e.node, e.kind);
        const std::string from_mem = "fs_load_row<" + std::to_string(e.dtype) + ", " + tmpl_row() + ", false>(" + nm + ", a.p[" + std::to_string(e.arg) +
                                     "], row0, lir, vbase);";
        if (!staged(e.node)) {
          os << "      " << from_mem << "\n";
        } else if (stage_written.count(e.node)) {  // a later pass: the head of the row comes back from LDS
          os << "      if (ch < STAGE_CHUNKS) fs_load_row_chunk_lds<" << e.dtype << ", V, NVL, L>(" << nm << ", " << stage_chunk(e.node) << ", lir);\n"
             << "      else " << from_mem << "\n";
        } else {  // the first pass that reads it: keep the head of the row, as it came from memory
          os << "      fs_load_row_staging<" << e.dtype << ", " << tmpl_row() << ", false>(" << nm << ", a.p[" << e.arg << "], row0, lir, vbase, "
             << stage_chunk(e.node) << ", ch < STAGE_CHUNKS);\n";
        }
      } else
        os << "      fs_load_row<" << e.dtype << ", " << tmpl_row() << ">(" << name(e.node, e.kind) << ", a.p[" << e.arg << "], 0, lir, vbase);\n";
    }
    for (int m : from_lds)  // buffered by an earlier pass (only emitted for chunks below STAGE_CHUNKS)
      os << "      float " << name(m, KIND_FULL) << "[E];\n      fs_load_row_chunk_lds<" << g.nodes[m].dtype << ", V, NVL, L>(" << name(m, KIND_FULL) << ", "
         << stage_chunk(m) << ", lir);\n";
    for (int m : gp.members) {
      if (!mem.count(m) || folded[m]) continue;
      const fs_node& n = g.nodes[m];
      const Kind k = gp.kind.at(m);
      if (!is_alias(m))
        os << "      float " << name(m, k) << "[E];\n      _Pragma(\"unroll\") for (int e = 0; e < E; ++e) " << name(m, k) << "[e] = "
           << (n.opcode == FS_TRANSPOSE ? ref(n.in[0]) : rounded(m, expr(m))) << ";\n";
      if (staged(m) && !stage_written.count(m))  // its first pass: the slot takes it over (from whatever it dominates)
        os << "      if (ch < STAGE_CHUNKS) fs_stage_row_chunk<" << n.dtype << ", V, NVL, L>(" << stage_chunk(m) << ", " << name(m, k) << ", lir);\n";
      if (!store_outputs) continue;
      if (const ExtTensor* e = find_out(m)) {
        if (k == KIND_ROWV)
          os << "      if (row == 0) fs_store_row<" << e->dtype << ", " << tmpl_row() << ">(" << name(source_of(m), k) << ", a.p[" << e->arg
             << "], 0, lir, vbase, true);\n";
        else
          emit_store(*e, "      ");
      }
    }
    tail();
  }

  // `targets`: what the pass is for (the stage's reductions, or the roots); `seed`: those of them the pass computes itself
  template <class Tail>
  void emit_pass(const std::vector<int>& targets, const std::set<int>& seed, bool store_outputs, Tail tail, const std::string& loop = "") {
    std::set<int> avail;
    for (int m : gp.members)
      if (staged(m) && stage_written.count(m) && !seed.count(m)) avail.insert(m);
    std::set<int> mem(seed), ext, mem_a(seed), ext_a, lds_a;
    needed_for(targets, &mem, &ext);
    if (!avail.empty()) needed_for(targets, &mem_a, &ext_a, &avail, &lds_a);
    for (int m : mem) {
      if (!first_pass.count(m)) first_pass[m] = n_passes;
      if (!folded[m] && gp.kind.at(m) == KIND_FULL) ++pass_computes[m];
    }
    for (int x : ext)
      if (gp.kind.at(x) == KIND_FULL) {
        ++pass_loads[x];
        if (!first_pass.count(x)) first_pass[x] = n_passes;
      }
    for (int t : targets)
      if (!first_pass.count(t)) first_pass[t] = n_passes;
    for (int x : lds_a.empty() ? ext : ext_a)  // what the pass loads for the chunks that are in LDS, under the current plan
      if (gp.kind.at(x) == KIND_FULL) ++pass_loads_planned[x];
    if (!loop.empty()) os << "    " << loop << " {\n";
    // (with a resident part the registers are nearly full: the chunk loop stays rolled, one chunk - 64 bytes per lane -
    // in flight at a time, instead of the compiler interleaving several chunks and spilling on some builds)
    else if (n_passes % 2 == 0) os << "    " << (gp.s.resident ? "_Pragma(\"unroll 1\") " : "") << "for (int ch = 0; ch < CT; ++ch) {\n";
    else os << "    " << (gp.s.resident ? "_Pragma(\"unroll 1\") " : "") << "for (int ch = CT - 1; ch >= 0; --ch) {\n";
    ++n_passes;
    // (inside a pass the chunk's own sizes shadow the body's: the building blocks read them by name)
    os << "      constexpr int NVL = NVLC, E = NVLC * V;\n      constexpr bool RAGGED = RAGC;\n"
       << "      const int vbase = RESV + ch * (NVL * L);\n      (void)RAGGED;\n";
    if (lds_a.empty()) {
      emit_pass_body(mem, ext, lds_a, store_outputs, tail);
    } else if (gp.s.stage_chunks >= gp.s.CT) {  // the whole row is buffered
      emit_pass_body(mem_a, ext_a, lds_a, store_outputs, tail);
    } else {
      os << "      if (ch < STAGE_CHUNKS) {\n";
      emit_pass_body(mem_a, ext_a, lds_a, store_outputs, tail);
      os << "      } else {\n";
      emit_pass_body(mem, ext, std::set<int>(), store_outputs, tail);
      os << "      }\n";
    }
    os << "    }\n";
    // (a lane reads back exactly the LDS positions it wrote itself, and a wavefront's LDS accesses complete in order:
    // no barrier between the pass that writes a slot and the passes that read it, nor before a value that dominates
    // the slot's previous owner overwrites it in place)
    for (int x : ext)
      if (staged(x)) stage_written.insert(x);
    for (int m : lds_a.empty() ? mem : mem_a)
      if (staged(m) && !folded[m]) stage_written.insert(m);
  }

  // inside a pass: fold the chunk's elements into the running lane partials q<b> of the stage's reductions
  void emit_chunk_accumulate(const std::vector<int>& batch) {
    const std::string col_ok = "(!RAGGED || (vbase + (e / V) * L + lir) < NV)";
    for (int b : batch) {
      const fs_node& bn = g.nodes[b];
      const std::string q = "q" + std::to_string(loc(b));
      if (folded[bn.in[0]]) {
        const fs_node& mn = g.nodes[bn.in[0]];
        os << "      _Pragma(\"unroll\") for (int e = 0; e < E; ++e) " << q << " = " << col_ok << " ? __builtin_fmaf(" << ref(mn.in[0]) << ", "
           << ref(mn.in[1]) << ", " << q << ") : " << q << ";\n";
      } else {
        os << "      {\n";
        const std::string arr = as_array(bn.in[0], std::to_string(loc(b)));
        os << "      " << q << " = fs_red_op<" << bn.attr_i << ">(" << q << ", fs_lane_reduce<" << bn.attr_i << ", " << tmpl_row() << ">(" << arr
           << ", lir, vbase));\n      }\n";
      }
    }
  }

  void run_chunked(bool xwave, int WPR, int KB) {
    auto is_rr = [&](int m) { return std::find(gp.row_reduces.begin(), gp.row_reduces.end(), m) != gp.row_reduces.end(); };
    int max_level = 0;
    for (int m : gp.members) max_level = std::max(max_level, gp.level.at(m));
    os << "  for (int it = (int)blockIdx.x; it < a.n_iters; it += (int)gridDim.x) {\n";
    os << "    const long row = it, row0 = row * C;\n    constexpr bool rok = true;\n    constexpr int vbase = 0;  // (outside the passes)\n"
       << "    (void)row0; (void)rok; (void)vbase;\n";
    for (const ExtTensor& e : gp.ext_in)
      if (e.kind == KIND_COLV) os << "    const float " << name(e.node, KIND_COLV) << " = fs_load1<" << e.dtype << ">(a.p[" << e.arg << "], row);\n";
    for (int lvl = 0; lvl <= max_level + 1; ++lvl) {
      // per-row values of this stage (they depend on earlier reductions only)
      for (int m : gp.members) {
        if (gp.level.at(m) != lvl || gp.kind.at(m) != KIND_COLV || is_rr(m) || folded[m]) continue;
        os << "    const float " << name(m, KIND_COLV) << " = " << rounded(m, expr(m)) << ";\n";
        if (const ExtTensor* e = find_out(m))
          os << "    if (lir == 0) fs_store1<" << e->dtype << ">(a.p[" << e->arg << "], row, " << name(m, KIND_COLV) << ");\n";
      }
      std::vector<int> batch;
      for (int m : gp.row_reduces)
        if (gp.level.at(m) == lvl) batch.push_back(m);
      if (batch.empty()) continue;
      for (int b : batch) os << "    float q" << loc(b) << " = fs_red_identity<" << g.nodes[b].attr_i << ">();\n";
      emit_pass(batch, std::set<int>(), false, [&]() { emit_chunk_accumulate(batch); });
      emit_exchange(batch, xwave, WPR, KB, "    ");
    }
    // last pass: everything that leaves the kernel as an [R,C] or [1,C] tensor
    std::vector<int> roots;
    for (const ExtTensor& e : gp.ext_out)
      if (e.kind != KIND_COLV) roots.push_back(e.node);
    if (!roots.empty()) emit_pass(roots, std::set<int>(roots.begin(), roots.end()), true, []() {});
    os << "  }\n}\n";
  }

  // ---- a few very long rows: one workgroup per row segment (Schedule::split_rows) ----------------
  // Every workgroup walks its segment's chunks once, storing what leaves the kernel as [R,C] or
  // [1,C] tensors and folding the reductions' operands into lane partials; the workgroup's lanes are
  // folded as for any row reduction, and the S segment results of a row meet through the ticketed
  // fold of the column reductions (a "vector" of one float per reduction).  The workgroup that
  // folds last also evaluates the per-row values that depend on the results, and stores.
  void run_split_rows(const std::string& kname, int WPR, int KB) {
    const Schedule& s = gp.s;
    const int K = (int)gp.row_reduces.size();
    auto is_rr = [&](int m) { return std::find(gp.row_reduces.begin(), gp.row_reduces.end(), m) != gp.row_reduces.end(); };
    os << "  constexpr int S = " << s.S << ", CPS = " << s.CPS << ";\n";
    os << "  __shared__ fs_u32 lds_flag;\n  __shared__ float lds_vals[" << K << "];\n";
    os << "  const long row = (int)blockIdx.x / S, row0 = row * C;\n  const int seg = (int)blockIdx.x % S;\n"
       << "  constexpr bool rok = true;\n  constexpr int vbase = 0;\n  (void)row0; (void)rok; (void)vbase;\n";
    for (const ExtTensor& e : gp.ext_in)
      if (e.kind == KIND_COLV) os << "  const float " << name(e.node, KIND_COLV) << " = fs_load1<" << e.dtype << ">(a.p[" << e.arg << "], row);\n";
    // per-row values that need no reduction result
    for (int m : gp.members)
      if (gp.level.at(m) == 0 && gp.kind.at(m) == KIND_COLV && !is_rr(m) && !folded[m])
        os << "  const float " << name(m, KIND_COLV) << " = " << rounded(m, expr(m)) << ";\n";
    // one pass over the segment: the reductions' operands, and what leaves the kernel as [R,C] or [1,C]
    // tensors (all of it computed before any reduction result)
    std::vector<int> targets(gp.row_reduces);
    std::set<int> seed;
    for (const ExtTensor& e : gp.ext_out)
      if (e.kind != KIND_COLV) targets.push_back(e.node), seed.insert(e.node);
    for (int b : gp.row_reduces) os << "  float q" << loc(b) << " = fs_red_identity<" << g.nodes[b].attr_i << ">();\n";
    os << "  {\n    const int ch_end = (seg + 1) * CPS < CT ? (seg + 1) * CPS : CT;\n";
    emit_pass(targets, seed, true, [&]() { emit_chunk_accumulate(gp.row_reduces); }, "for (int ch = seg * CPS; ch < ch_end; ++ch)");
    os << "  }\n";
    // fold the workgroup's lanes (the results are not rounded or divided yet: that happens once, at the end)
    for (int b : gp.row_reduces)
      os << "  q" << loc(b) << " = fs_segment_allreduce<" << g.nodes[b].attr_i << ", (L < 64 ? L : 64)>(q" << loc(b) << ");\n";
    if (s.L > 64) {
      os << "  {\n    const fs_xwave<" << KB << ", " << WPR << "> xw{lds_rr, lir >> 6, (tid & 63) == 0};\n";
      for (int k = 0; k < K; ++k) os << "    xw.put(" << k << ", q" << loc(gp.row_reduces[k]) << ");\n";
      os << "    fs_lds_barrier();\n";
      for (int k = 0; k < K; ++k)
        os << "    q" << loc(gp.row_reduces[k]) << " = xw.get<" << g.nodes[gp.row_reduces[k]].attr_i << ">(" << k << ");\n";
      os << "  }\n";
    }
    os << "  typedef fs_colfold<" << K << ", 1, WG, 1> SF;\n  float cv[SF::CPT][1];\n  cv[0][0] = 0.0f;\n";
    for (int k = 0; k < K; ++k) os << "  if (tid == " << k << ") cv[0][0] = q" << loc(gp.row_reduces[k]) << ";\n";
    os << "  if (fs_colred_fold_grid<" << K << ", 1, WG, 1, " << s.fan_in << ", " << kname << "_kinds>(cv, a.part + row * " << s.part_stride_floats
       << "L, a.tickets + row * " << s.ticket_stride << ", &lds_flag, (fs_u32)seg, (fs_u32)S)) {\n";
    os << "    if (tid < " << K << ") lds_vals[tid] = cv[0][0];\n    __syncthreads();\n    if (tid == 0) {\n";
    // thread 0 of the last workgroup: the results, what depends on them, and the stores
    std::vector<int> order;
    for (int m : gp.members)
      if (gp.kind.at(m) == KIND_COLV && !folded[m] && (is_rr(m) || gp.level.at(m) >= 1)) order.push_back(m);
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return gp.level.at(x) < gp.level.at(y); });
    for (int m : order) {
      if (is_rr(m)) {
        const int k = (int)(std::find(gp.row_reduces.begin(), gp.row_reduces.end(), m) - gp.row_reduces.begin());
        const std::string q = "lds_vals[" + std::to_string(k) + "]";
        os << "      const float " << name(m, KIND_COLV) << " = " << rounded(m, g.nodes[m].attr_i == FS_RED_MEAN ? q + " / (float)C" : q) << ";\n";
      } else {
        os << "      const float " << name(m, KIND_COLV) << " = " << rounded(m, expr(m)) << ";\n";
      }
    }
    for (const ExtTensor& e : gp.ext_out)
      if (e.kind == KIND_COLV)
        os << "      fs_store1<" << e.dtype << ">(a.p[" << e.arg << "], row, " << name(source_of(e.node), KIND_COLV) << ");\n";
    os << "    }\n  }\n}\n";
  }

  // ---- shared-memory planning for rows walked in chunks (Section 5.1) ----------------------------
  // Called on a dry run (no buffers yet), whose passes counted who needs what.
  //   size requirements (5.1.1)  candidates are the values several passes need: [R,C] inputs that more than one pass
  //                              loads, and elementwise results whose direct users belong to more than one pass
  //                              (multiple users, in different loops of the kernel); each would take one row in its
  //                              own dtype.
  //   space sharing (5.1.3)      dominance tree from the roots over the group's data flow: a candidate that dominates
  //                              a buffered value of the same element size, and is first computed no earlier, takes
  //                              over that value's slot - everything that still needs the old value gets it through
  //                              the new one (softmax: exp(x - max) overwrites x; LayerNorm on fp32 rows: x - mean
  //                              overwrites x).  Sharing costs nothing, so it is applied before anything is given up.
  //   size shrinking (5.1.2)     while the slots of a whole row exceed the budget, candidates that need a slot of their own
  //                              are given up - recomputed by every pass instead - in the paper's order: results of
  //                              inexpensive ops first, then of expensive ones (exp, log, tanh, sigmoid, gelu, divide,
  //                              sqrt, rsqrt, rcp), the one closest to the roots first within a class.  Inputs are
  //                              never given up (recomputing them means HBM traffic, the bound): if they alone exceed
  //                              the budget, all slots keep only the head of the row (stage_chunks < CT).
  static bool op_is_expensive(int op) {
    return op == FS_EXP || op == FS_LOG || op == FS_TANH || op == FS_SIGMOID || op == FS_GELU_TANH || op == FS_DIV || op == FS_SQRT ||
           op == FS_RSQRT || op == FS_RCP;
  }
  static const char* op_word(int op) {
    switch (op) {
      case FS_INPUT: return "input";
      case FS_NEG: return "neg";
      case FS_ABS: return "abs";
      case FS_EXP: return "exp";
      case FS_LOG: return "log";
      case FS_TANH: return "tanh";
      case FS_SIGMOID: return "sigmoid";
      case FS_SQRT: return "sqrt";
      case FS_RSQRT: return "rsqrt";
      case FS_RCP: return "rcp";
      case FS_GELU_TANH: return "gelu";
      case FS_CONVERT: return "convert";
      case FS_ADD: return "add";
      case FS_SUB: return "sub";
      case FS_MUL: return "mul";
      case FS_DIV: return "div";
      case FS_MAX: return "max";
      case FS_MIN: return "min";
      case FS_CMP: return "cmp";
      case FS_SELECT: return "select";
    }
    return "op";
  }
  void plan_stage_buffers(const std::set<int>& unbuffered_inputs) {
    gp.stage_slots.clear();
    gp.stage_slot_of.clear();
    gp.stage_given_up.clear();
    gp.lds_plan_text.clear();
    gp.s.stage_chunks = 0;
    const int ROOT = -1;
    // data flow seen from the roots: consumer -> operand edges, a virtual root above every output
    std::map<int, std::vector<int>> consumers;
    for (int u : gp.members) {
      const fs_node& n = g.nodes[u];
      for (int k = 0; k < n.num_in; ++k) {
        if (g.nodes[n.in[k]].opcode == FS_CONST) continue;
        const int src = source_of(n.in[k]);
        if (g.nodes[src].opcode == FS_CONST) continue;
        consumers[src].push_back(u);
      }
    }
    for (const ExtTensor& e : gp.ext_out) consumers[e.node].push_back(ROOT);
    // immediate dominators (node ids are topological: consumers have larger ids, so descending order visits them first)
    std::map<int, int> idom, depth, dist;
    depth[ROOT] = 0, dist[ROOT] = 0;
    std::vector<int> order;
    for (const auto& kv : consumers) order.push_back(kv.first);
    std::sort(order.rbegin(), order.rend());
    auto intersect = [&](int x, int y) {
      while (x != y) {
        if (depth.at(x) > depth.at(y)) x = idom.at(x);
        else y = idom.at(y);
      }
      return x;
    };
    for (int n : order) {
      int dom = -2, d = 1 << 30;
      for (int c : consumers[n]) {
        if (!depth.count(c)) continue;  // (a consumer nothing reaches from the roots)
        dom = dom == -2 ? c : intersect(dom, c);
        d = std::min(d, dist.at(c) + 1);
      }
      if (dom == -2) continue;
      idom[n] = dom, depth[n] = depth.at(dom) + 1, dist[n] = d;
    }
    auto dominates = [&](int b, int x) {  // b strictly above x in the dominance tree
      if (!depth.count(b) || !depth.count(x)) return false;
      while (depth.at(x) > depth.at(b)) x = idom.at(x);
      return x == b && depth.at(x) == depth.at(b) && b != ROOT;
    };
    // candidates in the order their first pass comes (inputs before what is computed from them)
    struct Cand { int node; bool input; int first; };
    std::vector<Cand> cands;
    for (const ExtTensor& e : gp.ext_in)
      if (e.kind == KIND_FULL && pass_loads[e.node] >= 2 && !unbuffered_inputs.count(e.node)) cands.push_back({e.node, true, first_pass[e.node]});
    for (int m : gp.members) {
      const fs_node& n = g.nodes[m];
      if (gp.kind.at(m) != KIND_FULL || folded[m] || find_out(m) || is_alias(m)) continue;
      std::set<int> homes;  // the passes its direct users belong to (where each is computed first)
      for (int u : consumers[m])
        if (u != ROOT && first_pass.count(u)) homes.insert(first_pass.at(u));
      if (homes.size() < 2) continue;
      if (n.opcode == FS_CONVERT || n.opcode == FS_TRANSPOSE || n.opcode == FS_CONCAT || (n.dtype != FS_F32 && n.dtype != FS_BF16)) continue;
      cands.push_back({m, false, first_pass[m]});
    }
    std::stable_sort(cands.begin(), cands.end(), [](const Cand& x, const Cand& y) { return x.first != y.first ? x.first < y.first : x.node < y.node; });
    std::vector<int> own;  // intermediates that would need a slot of their own
    for (const Cand& c : cands) {
      const int eb = dtype_size(g.nodes[c.node].dtype);
      int share = -1;
      if (!c.input)
        for (size_t k = 0; k < gp.stage_slots.size() && share < 0; ++k) {
          const int prev = gp.stage_slots[k].owners.back();
          if (gp.stage_slots[k].elem_bytes == eb && dominates(c.node, prev) && first_pass[prev] <= c.first) share = (int)k;
        }
      if (share >= 0) {
        gp.stage_slots[share].owners.push_back(c.node);
        gp.stage_slot_of[c.node] = share;
        continue;
      }
      if (!c.input) own.push_back(c.node);
      gp.stage_slot_of[c.node] = (int)gp.stage_slots.size();
      gp.stage_slots.push_back(StageSlot{eb, {c.node}});
    }
    auto row_bytes = [&]() {
      long b = 0;
      for (const StageSlot& sl : gp.stage_slots) b += gp.s.CT * chunk_bytes(sl.elem_bytes);
      return b;
    };
    // shrinking: give up own-slot intermediates while the whole row does not fit
    std::stable_sort(own.begin(), own.end(), [&](int x, int y) {
      const int cx = op_is_expensive(g.nodes[x].opcode), cy = op_is_expensive(g.nodes[y].opcode);
      if (cx != cy) return cx < cy;
      return dist.at(x) < dist.at(y);
    });
    for (size_t k = 0; k < own.size() && row_bytes() > gp.s.stage_avail; ++k) {
      const int slot = gp.stage_slot_of.at(own[k]);
      for (int o : gp.stage_slots[slot].owners) {
        gp.stage_given_up.push_back({o, op_is_expensive(g.nodes[o].opcode) ? 2 : 1});
        gp.stage_slot_of.erase(o);
      }
      gp.stage_slots.erase(gp.stage_slots.begin() + slot);
      for (auto& kv : gp.stage_slot_of)
        if (kv.second > slot) --kv.second;
    }
    long per_chunk = 0;
    for (const StageSlot& sl : gp.stage_slots) per_chunk += chunk_bytes(sl.elem_bytes);
    if (per_chunk > 0) gp.s.stage_chunks = (int)std::min<long>(gp.s.CT, gp.s.stage_avail / per_chunk);
    if (gp.s.stage_chunks <= 0) {
      gp.s.stage_chunks = 0;
      gp.stage_slots.clear();
      gp.stage_slot_of.clear();
    }
    // in words
    std::ostringstream t;
    t << "LDS plan: " << gp.s.stage_chunks << " of " << gp.s.CT << " chunks per row";
    for (size_t k = 0; k < gp.stage_slots.size(); ++k) {
      t << "; slot " << k << " (" << gp.stage_slots[k].elem_bytes << " B/element): ";
      for (size_t o = 0; o < gp.stage_slots[k].owners.size(); ++o) {
        const int node = gp.stage_slots[k].owners[o];
        t << (o ? ", then " : "") << name(node, KIND_FULL) << " " << op_word(g.nodes[node].opcode) << (o ? " (dominates it)" : "");
      }
    }
    for (const auto& gu : gp.stage_given_up)
      t << "; recomputed instead: " << name(gu.first, KIND_FULL) << " " << op_word(g.nodes[gu.first].opcode)
        << (gu.second == 2 ? " (expensive" : " (inexpensive") << ", its own slot would exceed the budget)";
    gp.lds_plan_text = t.str();
  }

  void run(const std::string& kname) {
    const Schedule& s = gp.s;
    for (int m : gp.members) in_set[m] = 1;
    count_uses();
    const int C = gp.C;
    const int NP = (int)(gp.ext_in.size() + gp.ext_out.size());
    const int K = (int)gp.col_reduces.size();
    const int WPR = s.L > 64 ? s.L / 64 : 1;
    const int KB = std::max(1, gp.max_batched_reduces);
    const bool xwave = !gp.row_reduces.empty() && s.L > 64;
    // Per-column values ([1,C] tensors) are loaded into registers once per workgroup when the
    // workgroup loops over many rows; with one trip per workgroup (or column tiles) they are
    // simply read where the loop body needs them.
    const bool ctile = s.col_tiled;  // column reductions by column tiles: a workgroup keeps its tile, RB workgroups share the rows
    const bool rowv_in_loop = !ctile && (s.CT > 1 || s.grid >= s.n_iters || s.stage_rowv);
    // per-column operands that can be added to each other once per workgroup (staged in LDS, or held in registers by
    // a looping workgroup); where they are read again for every row there is nothing to gain
    if (!s.chunked && !s.split_rows && !s.resident && s.CT == 1 && (s.stage_rowv || !rowv_in_loop)) find_combs();
    std::set<int> comb_only;  // [1,C] tensors that are only read through a comb
    for (const Comb& c : combs) comb_only.insert(c.ra), comb_only.insert(c.rb);
    for (const ExtTensor& e : gp.ext_in)
      if (e.kind == KIND_ROWV && !comb_only.count(e.node)) slot_of_ext[e.node] = n_slots++;
    for (size_t k = 0; k < combs.size(); ++k) slot_of_comb.push_back(n_slots++);

    // fixed local numbering: external inputs first, then members
    for (const ExtTensor& e : gp.ext_in) loc(e.node);
    for (int m : gp.members) loc(m);

    os << "// work space [R," << C << "], " << s.L << " lanes/row, " << s.E << " elements/lane, workgroup " << s.WG << "\n";
    os << "struct " << kname << "_args { void* p[" << NP << "]; float* part; fs_u32* tickets; int R; int n_iters; };\n";
    // the reductions that are folded across workgroups: column reductions, or the row reductions of split rows
    const std::vector<int>& folded_across = s.split_rows ? gp.row_reduces : gp.col_reduces;
    if (!folded_across.empty()) {
      os << "struct " << kname << "_kinds {\n  static FS_DEV float op(int k, float a, float b) { switch (k) {";
      for (size_t k = 0; k < folded_across.size(); ++k)
        os << " case " << k << ": return fs_red_op<" << g.nodes[folded_across[k]].attr_i << ">(a, b);";
      os << " } return a; }\n  static FS_DEV float identity(int k) { switch (k) {";
      for (size_t k = 0; k < folded_across.size(); ++k)
        os << " case " << k << ": return fs_red_identity<" << g.nodes[folded_across[k]].attr_i << ">();";
      os << " } return 0.0f; }\n};\n";
    }
    os << "extern \"C\" __global__ void __launch_bounds__(" << s.WG << ") ";
    if (s.min_waves > 0) os << "__attribute__((amdgpu_waves_per_eu(" << s.min_waves << "))) ";
    os << kname << "(const " << kname << "_args a) {\n";
    os << "  constexpr int V = " << s.V << ", NVL = " << s.NVL << ", L = " << s.L << ", NV = " << s.NV << ", E = NVL * V, WG = " << s.WG
       << ", G = WG / L, C = " << C << ", CT = " << s.CT << ";\n";
    os << "  constexpr bool RAGGED = " << (s.ragged ? "true" : "false") << ";\n";
    os << "  const int tid = (int)threadIdx.x, lir = tid & (L - 1), rg = tid / L;\n";
    os << "  const long R = a.R;\n";
    os << "  (void)lir; (void)rg; (void)R; (void)C; (void)G; (void)CT;\n";
    if (xwave) os << "  __shared__ float lds_rr[2 * G * " << WPR << " * " << KB << "];\n  int parity = 0;\n";
    if (s.chunked) {
      os << "  constexpr int NVLC = " << s.NVLC << ", RESV = " << s.RESV << ";\n  constexpr bool RAGC = " << (s.ragged_chunks ? "true" : "false")
         << ";\n";
      if (s.stage_chunks > 0 && !gp.stage_slots.empty()) {
        long bytes = 0;
        for (const StageSlot& sl : gp.stage_slots) bytes += s.stage_chunks * chunk_bytes(sl.elem_bytes);
        os << "  // " << gp.lds_plan_text << "\n";
        os << "  constexpr int STAGE_CHUNKS = " << s.stage_chunks << ";  // chunks of every buffered value kept in LDS\n"
           << "  __shared__ __attribute__((aligned(16))) unsigned char lds_stage[" << bytes << "];\n";
      }
      if (s.split_rows) {
        run_split_rows(kname, WPR, KB);
        return;
      }
      if (!s.resident) {
        run_chunked(xwave, WPR, KB);
        return;
      }
    }
    // CW columns are folded together: the whole row, or one column tile
    // (RB, the number of workgroups that fold together, only where something is folded: a kernel without column
    // reductions has the same text, hence the same compiled code, whatever the number of rows)
    os << "  constexpr int CW = " << (ctile ? "NVL * L * V" : "C") << ", NVF = CW / V, RB = " << (K > 0 || ctile ? s.RB : 1) << ";\n";
    if (ctile) os << "  const int tile = (int)blockIdx.x % CT, rb = (int)blockIdx.x / CT, vbase = tile * (NVL * L);\n";
    else os << "  const int tile = 0, rb = (int)blockIdx.x;\n";
    os << "  (void)tile; (void)rb; (void)CW; (void)NVF; (void)RB;\n";
    // One LDS pool, shared by lifetime: the row loop's buffers (transpose tile, staged [1,C]
    // operands) and the epilogue's column-fold area never live at the same time.
    if (K > 0 || s.tile_transpose || s.stage_rowv) {
      os << "  constexpr int TCW = " << (s.tiled_transpose ? "NVL * L * V" : "C") << ";  // columns of one transpose tile\n";
      os << "  constexpr int SLOT = NVL * L * V, TILE_FLOATS = " << (s.tile_transpose ? "TCW * (G + 1)" : "0") << ", LOOP_FLOATS = TILE_FLOATS + "
         << (s.stage_rowv ? n_slots : 0) << " * SLOT, PC = " << std::max(1, s.fold_piece) << ", FOLD_FLOATS = " << (K > 0 ? "(L < 64 ? WG / 64 : G) * PC" : "0") << ";\n";
      os << "  __shared__ float lds_pool[LOOP_FLOATS > FOLD_FLOATS ? LOOP_FLOATS : FOLD_FLOATS];\n";
      os << "  float* const lds_tile = lds_pool; float* const lds_rowv = lds_pool + TILE_FLOATS; float* const lds_col = lds_pool;\n";
      os << "  (void)lds_tile; (void)lds_rowv; (void)lds_col; (void)SLOT; (void)PC;\n";
    }
    if (K > 0) os << "  __shared__ fs_u32 lds_flag;\n";

    // ---- per-column values ----
    // (looping kernels without LDS staging: loaded into registers once per workgroup, before the loop)
    auto emit_rowv = [&](const std::string& ind, const std::string& vb, const std::string& store_cond) {
      for (const ExtTensor& e : gp.ext_in)
        if (e.kind == KIND_ROWV) {
          os << ind << "float " << name(e.node, KIND_ROWV) << "[E];\n";
          os << ind << "fs_load_row<" << e.dtype << ", " << tmpl_row() << ">(" << name(e.node, KIND_ROWV) << ", a.p[" << e.arg << "], 0, lir, " << vb
             << ");\n";
        }
      for (const Comb& c : combs)
        os << ind << "float rc" << loc(c.z) << "[E];\n" << ind << "_Pragma(\"unroll\") for (int e = 0; e < E; ++e) rc" << loc(c.z) << "[e] = "
           << (c.neg_a ? "-" : "") << name(c.ra, KIND_ROWV) << "[e] " << (c.neg_b ? "- " : "+ ") << name(c.rb, KIND_ROWV) << "[e];\n";
      for (int m : gp.members) {
        if (gp.level.at(m) >= 0 || folded[m]) continue;
        const std::string nm = name(m, KIND_ROWV);
        os << ind << "float " << nm << "[E];\n" << ind << "_Pragma(\"unroll\") for (int e = 0; e < E; ++e) " << nm << "[e] = "
           << rounded(m, expr(m)) << ";\n";
        if (const ExtTensor* e = find_out(m))
          os << ind << "if (" << store_cond << ") fs_store_row<" << e->dtype << ", " << tmpl_row() << ">(" << nm << ", a.p[" << e->arg
             << "], 0, lir, " << vb << ", true);\n";
      }
    };
    if (!rowv_in_loop) emit_rowv("  ", ctile ? "vbase" : "0", "rb == 0 && rg == 0");
    // staged [1,C] operands of a looping kernel: written to LDS once, before the loop
    const bool stage_before_loop = s.stage_rowv && s.grid < s.n_iters;
    auto ext_of = [&](int node) -> const ExtTensor& {
      for (const ExtTensor& e : gp.ext_in)
        if (e.node == node) return e;
      return gp.ext_in.front();
    };
    auto emit_staging = [&](const std::string& ind) {
      for (const ExtTensor& e : gp.ext_in)
        if (e.kind == KIND_ROWV && slot_of_ext.count(e.node))
          os << ind << "fs_stage_rowvec<" << e.dtype << ", V, L, C, WG>(lds_rowv + " << slot_of_ext.at(e.node) << " * SLOT, a.p[" << e.arg << "]);\n";
      for (size_t k = 0; k < combs.size(); ++k) {
        const ExtTensor &ea = ext_of(combs[k].ra), &eb = ext_of(combs[k].rb);
        os << ind << "fs_stage_rowvec_sum<" << ea.dtype << ", " << eb.dtype << ", " << (combs[k].neg_a ? "true" : "false") << ", "
           << (combs[k].neg_b ? "true" : "false") << ", V, L, C, WG>(lds_rowv + " << slot_of_comb[k] << " * SLOT, a.p[" << ea.arg << "], a.p[" << eb.arg
           << "]);\n";
      }
      os << ind << "__syncthreads();\n";
    };
    // rotated loop: the first trip's rows are requested before the operands are staged, the next trip's at the end of a trip
    bool rotate = s.rotate_loop && stage_before_loop && !ctile && !s.tiled_transpose && s.CT == 1 && !s.resident && s.U <= 1;
    for (int m : gp.members) rotate &= g.nodes[m].opcode != FS_CONCAT;
    if (rotate) {
      os << "  const long row_first = (long)blockIdx.x * G + rg, row_first_ld = row_first < R ? row_first : R - 1;\n";
      for (const ExtTensor& e : gp.ext_in)
        if (e.kind == KIND_FULL) {
          os << "  float " << name(e.node, KIND_FULL) << "[E];\n";
          os << "  fs_load_row<" << e.dtype << ", " << tmpl_row() << ", " << (e.streaming ? "true" : "false") << ">(" << name(e.node, KIND_FULL)
             << ", a.p[" << e.arg << "], row_first_ld * C, lir, 0);\n";
        }
    }
    if (stage_before_loop) emit_staging("  ");
    for (int k = 0; k < K; ++k) {
      const int m = gp.col_reduces[k];
      os << "  float ca" << loc(m) << "[E];\n  _Pragma(\"unroll\") for (int e = 0; e < E; ++e) ca" << loc(m) << "[e] = fs_red_identity<"
         << g.nodes[m].attr_i << ">();\n";
    }

    // ---- the row loop ----
    // A looping kernel handles U row tiles per trip: the loads of all U tiles are issued first,
    // then the U bodies run one after the other (more bytes in flight per wavefront).
    // (workgroups that stage their [1,C] operands before the loop read them from LDS inside each tile's body: they
    // may take several tiles per trip too)
    // ([1,C] values computed by the kernel inside the loop body are declared, and stored by the workgroup of row 0, under the
    // names of a single tile: such bodies take one tile per trip)
    bool rowv_member_in_loop = false;
    for (int m : gp.members) rowv_member_in_loop |= rowv_in_loop && gp.level.at(m) < 0;
    const int U = ((rowv_in_loop && !stage_before_loop) || s.CT > 1 || ctile || rowv_member_in_loop) ? 1 : std::max(1, s.U);
    if (ctile) {
      os << "  for (int it = rb; it < a.n_iters; it += RB) {\n";
    } else if (U == 1) {
      os << "  for (int it = (int)blockIdx.x; it < a.n_iters; it += (int)gridDim.x) {\n";
    } else {
      os << "  for (int it0 = (int)blockIdx.x * " << U << "; it0 < a.n_iters; it0 += (int)gridDim.x * " << U << ") {\n";
    }
    for (int u = 0; u < U; ++u) {
      const std::string x = U == 1 ? "" : "_" + std::to_string(u);
      if (U > 1) os << "    const int it" << x << " = it0 + " << u << ";\n";
      if (ctile) {
        os << "    const long row = (long)it * G + rg;\n";
      } else if (s.tiled_transpose) {
        // 2-D tiles: consecutive workgroups take consecutive column tiles of the same G rows
        if (s.tt_col_band > 0) {
          // bands of TCB column tiles, each walked row tile by row tile; the row-tile count is a constant of this
          // kernel so that every division below is one by a constant (a runtime divisor costs 2-3 % of a tile's time)
          const int trt = s.n_iters / s.CT, tcb = s.tt_col_band, last = s.CT % tcb;
          os << "    constexpr int TRT = " << trt << ", TCB = " << tcb << ", FULL_BANDS = CT / TCB, LAST_BAND = " << (last ? last : tcb) << ";\n"
             << "    const int band = it / (TCB * TRT), in_band = it - band * (TCB * TRT);\n"
             << "    const int rtile = band < FULL_BANDS ? in_band / TCB : in_band / LAST_BAND;\n"
             << "    const int ctile = band * TCB + in_band - rtile * (band < FULL_BANDS ? TCB : LAST_BAND);\n"
             << "    const long row = (long)rtile * G + rg;\n    const int vbase = ctile * (NVL * L);\n";
        } else {
          os << "    const long row = (long)(it / CT) * G + rg;\n    const int vbase = (it % CT) * (NVL * L);\n";
        }
      } else if (s.CT == 1 || s.resident) {
        os << "    const long row" << x << " = (long)it" << x << " * G + rg;\n    constexpr int vbase" << x << " = 0;\n";
      } else {
        os << "    const long unit = (long)it * G + rg;\n    const long row = unit / CT;\n    const int vbase = (int)(unit % CT) * (NVL * L);\n";
      }
      // rows beyond R are clamped for loads (never predicated) and masked at stores / accumulations
      os << "    const bool rok" << x << " = row" << x << " < R;\n    const long row_ld" << x << " = rok" << x << " ? row" << x
         << " : R - 1;\n    const long row0" << x << " = row_ld" << x << " * C;\n    (void)row0" << x << "; (void)vbase" << x << ";\n";
      for (const ExtTensor& e : gp.ext_in) {
        if (e.kind == KIND_FULL && rotate) {
          // (already in registers: requested before the loop or at the end of the previous trip)
        } else if (e.kind == KIND_FULL) {
          os << "    float " << name(e.node, KIND_FULL) << x << "[E];\n";
          os << "    fs_load_row<" << e.dtype << ", " << tmpl_row() << ", " << (e.streaming ? "true" : "false") << ">(" << name(e.node, KIND_FULL)
             << x << ", a.p[" << e.arg << "], row0" << x << ", lir, vbase" << x << ");\n";
        } else if (e.kind == KIND_COLV) {
          os << "    const float " << name(e.node, KIND_COLV) << x << " = fs_load1<" << e.dtype << ">(a.p[" << e.arg << "], row_ld" << x << ");\n";
        }
      }
      // concat members: one row out of two tensors, loaded with the other inputs (U is 1 in such groups)
      for (int m : gp.members) {
        const fs_node& cn = g.nodes[m];
        if (cn.opcode != FS_CONCAT) continue;
        const ExtTensor &ea = ext_of(cn.in[0]), &eb = ext_of(cn.in[1]);
        const long split = cn.attr_i == FS_CONCAT_COLS ? g.nodes[cn.in[0]].cols : g.nodes[cn.in[0]].rows;
        os << "    float " << name(m, KIND_FULL) << "[E];\n    fs_load_row_concat<" << cn.dtype << ", " << tmpl_row() << ", " << cn.attr_i << ", " << split
           << "L, " << g.nodes[cn.in[1]].cols << "L>(" << name(m, KIND_FULL) << ", a.p[" << ea.arg << "], a.p[" << eb.arg << "], row_ld, lir, vbase);\n";
      }
    }
    // Inside the loop body every per-column value is made available right before its first use,
    // one tensor at a time (a [1,C] operand costs E registers from its load to its last use; three
    // of them loaded at the top of a LayerNorm body with 32 elements per lane spill).  Staged
    // operands are written to LDS up front; only their reads into registers are lazy.
    std::set<int> rowv_ready;
    const bool lazy_rowv = rowv_in_loop;
    if (lazy_rowv && s.stage_rowv && !stage_before_loop) emit_staging("    ");
    std::function<void(int)> ensure_rowv = [&](int src) {
      if (!lazy_rowv || rowv_ready.count(src)) return;
      rowv_ready.insert(src);
      const std::string nm = name(src, KIND_ROWV);
      if (!in_set[src]) {
        for (const ExtTensor& e : gp.ext_in) {
          if (e.kind != KIND_ROWV || e.node != src) continue;
          declare(nm, "    ");
          if (s.stage_rowv)
            os << "    " << vec_fn("fs_read_staged") << "<" << tmpl_row() << ">(" << nm << ", lds_rowv + " << slot_of_ext.at(src) << " * SLOT, lir"
               << vec_arg() << ");\n";
          else
            os << "    " << vec_fn("fs_load_row") << "<" << e.dtype << ", " << tmpl_row() << ">(" << nm << ", a.p[" << e.arg << "], 0, lir, vbase"
               << vec_arg() << ");\n";
        }
        return;
      }
      // a [1,C] member: its own operands first
      const fs_node& n = g.nodes[src];
      for (int k = 0; k < n.num_in; ++k) {
        if (g.nodes[n.in[k]].opcode == FS_CONST) continue;
        const int o = source_of(n.in[k]);
        if (g.nodes[o].opcode != FS_CONST && gp.kind.at(o) == KIND_ROWV) ensure_rowv(o);
      }
      if (folded[src]) return;
      declare(nm, "    ");
      os << "    " << eloop() << nm << "[e] = " << rounded(src, expr(src)) << ";\n";
      if (const ExtTensor* e = find_out(src))
        os << "    if (row == 0 && rok) " << vec_fn("fs_store_row") << "<" << e->dtype << ", " << tmpl_row() << ">(" << nm << ", a.p[" << e->arg
           << "], 0, lir, vbase, true" << vec_arg() << ");\n";
    };
    std::set<int> comb_ready;
    std::function<void(int)> ensure_rowv_operands = [&](int m) {
      if (comb_of.count(m)) {  // reads its combined operand (staged) and whatever the remaining operand needs
        const Comb& c = combs[comb_of.at(m)];
        if (comb_ready.insert(c.z).second) {
          const std::string nm = "rc" + std::to_string(loc(c.z));
          declare(nm, "    ");
          os << "    " << vec_fn("fs_read_staged") << "<" << tmpl_row() << ">(" << nm << ", lds_rowv + " << slot_of_comb[comb_of.at(m)] << " * SLOT, lir"
             << vec_arg() << ");\n";
        }
        if (g.nodes[c.p].opcode != FS_CONST) {
          const int o = source_of(c.p);
          if (g.nodes[o].opcode != FS_CONST) {
            if (gp.kind.at(o) == KIND_ROWV) ensure_rowv(o);
            else if (in_set[o] && folded[o]) ensure_rowv_operands(o);
          }
        }
        return;
      }
      const fs_node& n = g.nodes[m];
      for (int k = 0; k < n.num_in; ++k) {
        if (g.nodes[n.in[k]].opcode == FS_CONST) continue;
        const int o = source_of(n.in[k]);
        if (g.nodes[o].opcode == FS_CONST) continue;
        if (gp.kind.at(o) == KIND_ROWV) ensure_rowv(o);
        else if (in_set[o] && folded[o]) ensure_rowv_operands(o);
      }
    };
    // members in stage order; the row reductions of a stage come last and share one exchange
    std::vector<int> order;
    for (int m : gp.members)
      if (gp.level.at(m) >= 0 && !folded[m] && !absorbed[m]) order.push_back(m);
    auto is_rr = [&](int m) { return std::find(gp.row_reduces.begin(), gp.row_reduces.end(), m) != gp.row_reduces.end(); };
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) {
      const int lx = gp.level.at(x), ly = gp.level.at(y);
      if (lx != ly) return lx < ly;
      return (int)is_rr(x) < (int)is_rr(y);
    });
    const std::string col_ok = "(!RAGGED || ((e / V) * L + lir) < NV)";
    // the statements after the last exchange are emitted vector by vector (see `strip`) when the
    // lane holds several vectors and they are plain elementwise work and stores
    size_t tail_start = 0;
    for (size_t k = 0; k < order.size(); ++k)
      if (is_rr(order[k])) tail_start = k + 1;
    bool strip_tail = tail_start > 0 && tail_start < order.size() && s.NVL >= 2 && !s.resident && !s.tile_transpose && !s.tiled_transpose;
    for (const ExtTensor& e : gp.ext_out) strip_tail &= !e.transposed;
    for (size_t k = tail_start; k < order.size() && strip_tail; ++k) strip_tail &= g.nodes[order[k]].opcode != FS_TRANSPOSE;
    std::ostringstream before_strip;

    for (int u = 0; u < U; ++u) {
      rowv_ready.clear();  // (each tile's body is a scope of its own: what it reads lazily it declares itself)
      comb_ready.clear();
      if (U > 1) {
        const std::string x = "_" + std::to_string(u);
        os << "    {\n    const long row = row" << x << "; const bool rok = rok" << x << "; const long row0 = row0" << x
           << "; constexpr int vbase = 0; (void)row; (void)rok; (void)row0; (void)vbase;\n";
        for (const ExtTensor& e : gp.ext_in) {
          if (e.kind == KIND_FULL) os << "    float (&" << name(e.node, KIND_FULL) << ")[E] = " << name(e.node, KIND_FULL) << x << ";\n";
          else if (e.kind == KIND_COLV) os << "    const float " << name(e.node, KIND_COLV) << " = " << name(e.node, KIND_COLV) << x << ";\n";
        }
      }
      size_t i = 0;
    while (i < order.size()) {
      if (i == tail_start && strip_tail) {
        strip = true;
        pre.str("");
        before_strip.str("");
        before_strip.swap(os);
      }
      const int m = order[i];
      const fs_node& n = g.nodes[m];
      if (lazy_rowv) {
        if (is_rr(m)) {  // the whole batch of this stage is emitted at once
          for (size_t k = i; k < order.size() && is_rr(order[k]) && gp.level.at(order[k]) == gp.level.at(m); ++k) ensure_rowv_operands(order[k]);
        } else {
          ensure_rowv_operands(m);
        }
      }
      if (is_rr(m)) {
        // batch: every row reduction of this stage
        std::vector<int> batch;
        const int lvl = gp.level.at(m);
        while (i < order.size() && is_rr(order[i]) && gp.level.at(order[i]) == lvl) batch.push_back(order[i++]);
        for (int b : batch) {
          const fs_node& bn = g.nodes[b];
          const std::string q = "q" + std::to_string(loc(b));
          if (folded[bn.in[0]]) {
            // sum of products: one fma per element
            const fs_node& mn = g.nodes[bn.in[0]];
            os << "    float " << q << " = 0.0f;\n    _Pragma(\"unroll\") for (int e = 0; e < E; ++e) " << q << " = " << col_ok
               << " ? __builtin_fmaf(" << ref(mn.in[0]) << ", " << ref(mn.in[1]) << ", " << q << ") : " << q << ";\n";
          } else {
            const std::string arr = as_array(bn.in[0], std::to_string(loc(b)));
            os << "    float " << q << " = fs_lane_reduce<" << bn.attr_i << ", " << tmpl_row() << ">(" << arr << ", lir);\n";
          }
        }
        if (s.resident)  // the part of the row that is not resident: walked in chunks, recomputed from the inputs or read back from LDS
          emit_pass(batch, std::set<int>(), false, [&]() { emit_chunk_accumulate(batch); });
        for (int b : batch) {
          const std::string q = "q" + std::to_string(loc(b));
          os << "    " << q << " = fs_segment_allreduce<" << g.nodes[b].attr_i << ", (L < 64 ? L : 64)>(" << q << ");\n";
        }
        if (xwave) {
          os << "    {\n      const fs_xwave<" << KB << ", " << WPR << "> xw{lds_rr + (parity * G + rg) * " << WPR * KB
             << ", lir >> 6, (tid & 63) == 0};\n";
          for (size_t k = 0; k < batch.size(); ++k) os << "      xw.put(" << k << ", q" << loc(batch[k]) << ");\n";
          os << "      fs_lds_barrier();\n";
          for (size_t k = 0; k < batch.size(); ++k)
            os << "      q" << loc(batch[k]) << " = xw.get<" << g.nodes[batch[k]].attr_i << ">(" << k << ");\n";
          os << "      parity ^= 1;\n    }\n";
        }
        for (int b : batch) {
          const fs_node& bn = g.nodes[b];
          const std::string q = "q" + std::to_string(loc(b));
          os << "    const float " << name(b, KIND_COLV) << " = " << rounded(b, bn.attr_i == FS_RED_MEAN ? q + " / (float)C" : q) << ";\n";
          if (const ExtTensor* e = find_out(b)) emit_store(*e, "    ");
        }
        continue;
      }
      ++i;
      if (is_col_reduce(m)) {
        const std::string ca = "ca" + std::to_string(loc(m));
        if (folded[n.in[0]]) {
          const fs_node& mn = g.nodes[n.in[0]];
          os << "    " << eloop() << ca << "[e] = rok ? __builtin_fmaf(" << ref(mn.in[0]) << ", " << ref(mn.in[1]) << ", " << ca << "[e]) : " << ca
             << "[e];\n";
        } else {
          os << "    " << eloop() << ca << "[e] = rok ? fs_red_op<" << n.attr_i << ">(" << ca << "[e], " << ref(n.in[0]) << ") : " << ca << "[e];\n";
        }
        continue;
      }
      if (n.opcode == FS_CONCAT) {  // loaded at the top of the body
        if (const ExtTensor* e = find_out(m)) emit_store(*e, "    ");
        continue;
      }
      if (n.opcode == FS_TRANSPOSE) {
        // no arithmetic: an in-group operand is aliased; an operand from memory is copied (it was loaded as it lies)
        if (!is_alias(m)) {
          declare(name(m, KIND_FULL), "    ");
          os << "    " << eloop() << name(m, KIND_FULL) << "[e] = " << ref(n.in[0]) << ";\n";
        }
        if (const ExtTensor* e = find_out(m)) emit_store(*e, "    ");
        continue;
      }
      const Kind k = gp.kind.at(m);
      if (k == KIND_COLV) {
        (strip ? pre : os) << "    const float " << name(m, k) << " = " << rounded(m, expr(m)) << ";\n";
      } else {
        declare(name(m, k), "    ");
        os << "    " << eloop() << name(m, k) << "[e] = " << rounded(m, expr(m)) << ";\n";
      }
      if (const ExtTensor* e = find_out(m)) emit_store(*e, "    ");
    }
      if (strip) {
        strip = false;
        const std::string body = os.str();
        os.swap(before_strip);
        os << pre.str() << "    _Pragma(\"unroll\") for (int j = 0; j < NVL; ++j) {\n" << body << "    }\n";
      }
      if (U > 1) os << "    }\n";
    }
    if (lazy_rowv)  // [1,C] members nothing in the body consumed (outputs only)
      for (int m : gp.members)
        if (gp.level.at(m) < 0) ensure_rowv(m);
    if (s.resident) {  // last pass over the non-resident part: everything that leaves as an [R,C] or [1,C] tensor
      std::vector<int> roots;
      for (const ExtTensor& e : gp.ext_out)
        if (e.kind != KIND_COLV) roots.push_back(e.node);
      if (!roots.empty()) emit_pass(roots, std::set<int>(roots.begin(), roots.end()), true, []() {});
    }
    if (rotate) {
      os << "    if (it + (int)gridDim.x < a.n_iters) {\n      const long rn = (long)(it + (int)gridDim.x) * G + rg, rnl = rn < R ? rn : R - 1;\n";
      for (const ExtTensor& e : gp.ext_in)
        if (e.kind == KIND_FULL)
          os << "      fs_load_row<" << e.dtype << ", " << tmpl_row() << ", " << (e.streaming ? "true" : "false") << ">(" << name(e.node, KIND_FULL)
             << ", a.p[" << e.arg << "], rnl * C, lir, 0);\n";
      os << "    }\n";
    }
    os << "  }\n";

    // ---- epilogue: finish the column reductions ----
    if (K > 0) {
      const int CW = ctile ? s.NVL * s.L * s.V : C;
      const int FV = CW % 4 == 0 ? 4 : CW % 2 == 0 ? 2 : 1;
      os << "  {\n    constexpr int FV = " << FV << ";\n    typedef fs_colfold<" << K << ", CW, WG, FV> S;\n    float cv[S::CPT][FV];\n";
      for (int k = 0; k < K; ++k) {
        const int m = gp.col_reduces[k];
        os << "    fs_colred_fold_wg<" << g.nodes[m].attr_i << ", " << k << ", " << K << ", V, NVL, L, NVF, CW, WG, FV, PC>(ca" << loc(m)
           << ", cv, lds_col, lir, rg);\n";
      }
      os << "    if (fs_colred_fold_grid<" << K << ", CW, WG, FV, " << s.fan_in << ", " << kname << "_kinds>(cv, a.part + (long)tile * "
         << s.part_stride_floats << "L, a.tickets + tile * " << s.ticket_stride << ", &lds_flag, (fs_u32)rb, (fs_u32)RB)) {\n";
      os << "      _Pragma(\"unroll\") for (int i = 0; i < S::CPT; ++i) {\n        const int c = tid + i * WG;\n"
         << "        if (c < S::NCH) {\n          const int k = c / S::CH, col0 = tile * CW + (c % S::CH) * FV;\n";
      for (int k = 0; k < K; ++k) {
        const int m = gp.col_reduces[k];
        const ExtTensor* e = find_out(m);
        if (!e) continue;
        const fs_node& n = g.nodes[m];
        os << "          if (k == " << k << ") { _Pragma(\"unroll\") for (int f = 0; f < FV; ++f) if (col0 + f < C) fs_store1<" << e->dtype
           << ">(a.p[" << e->arg << "], col0 + f, cv[i][f]" << (n.attr_i == FS_RED_MEAN ? " / (float)a.R" : "") << "); }\n";
      }
      os << "        }\n      }\n    }\n  }\n";
    }
    os << "}\n";
  }
};

uint64_t fnv1a(const std::string& s) {
  uint64_t h = 1469598103934665603ull;
  for (unsigned char c : s) {
    h ^= c;
    h *= 1099511628211ull;
  }
  return h;
}

}  // namespace

fs_status generate_kernel(const Graph& g, GroupPlan* gp, int /*group_index*/) {
  // Rows walked in chunks: a dry run counts which passes load each [R,C] input and compute each elementwise result;
  // plan_stage_buffers turns that into the kernel's LDS buffers (Section 5.1).
  gp->stage_slots.clear();
  gp->stage_slot_of.clear();
  gp->stage_given_up.clear();
  gp->lds_plan_text.clear();
  gp->s.stage_chunks = 0;
  long stage_bytes = 0;
  if (gp->s.chunked && !gp->s.split_rows && gp->s.stage_avail > 0) {
    Emitter dry(g, *gp);
    dry.run("FSK");
    dry.plan_stage_buffers(std::set<int>());
    // An input whose every later use now goes through a buffered result no longer needs a slot of its own (masked
    // softmax: once x * scale + mask is buffered, neither x nor the mask is read again): plan again without it.
    std::set<int> unbuffered;
    for (int round = 0; round < 8 && !gp->stage_slots.empty(); ++round) {
      Emitter check(g, *gp);
      check.run("FSK");
      bool changed = false;
      for (const StageSlot& sl : gp->stage_slots)
        if (sl.owners.size() == 1 && !check.in_set[sl.owners[0]] && check.pass_loads_planned[sl.owners[0]] < 2)
          changed |= unbuffered.insert(sl.owners[0]).second;
      if (!changed) break;
      dry.plan_stage_buffers(unbuffered);
    }
    for (const StageSlot& sl : gp->stage_slots) stage_bytes += gp->s.stage_chunks * dry.chunk_bytes(sl.elem_bytes);
  }
  // first pass with a placeholder name to hash the structure, second pass with the real name
  std::string text;
  {
    Emitter e(g, *gp);
    e.run("FSK");
    text = e.os.str();
  }
  char nm[64];
  snprintf(nm, sizeof(nm), "fs_k_%016llx", (unsigned long long)fnv1a(text));
  Emitter e(g, *gp);
  e.run(nm);
  gp->kernel_name = nm;
  gp->source = e.os.str();
  // staged per-column operands that were added to each other share one LDS slot
  gp->s.lds_bytes = gp->s.lds_planned - (gp->s.stage_rowv ? (int)e.combs.size() * gp->s.NVL * gp->s.L * gp->s.V * 4 : 0) + (int)stage_bytes;
  return FS_OK;
}

}  // namespace fs
