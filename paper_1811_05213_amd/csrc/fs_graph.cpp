// fs_graph.cpp - ingestion and validation of a fusion plan (ids, arity, shapes, dtypes).
#include <cstring>

#include "fs_internal.h"

namespace fs {

static thread_local std::string g_error;
std::string& error_buffer() { return g_error; }

void set_error(const char* fmt, ...) {
  char buf[1024];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_error = buf;
}

int op_arity(int op) {
  if (op == FS_INPUT || op == FS_CONST) return 0;
  if (op_is_unary(op)) return 1;
  if (op_is_binary(op) || op == FS_CMP) return 2;
  if (op == FS_SELECT) return 3;
  if (op == FS_BCAST_ROWVEC || op == FS_BCAST_COLVEC || op == FS_TRANSPOSE || op == FS_REDUCE_ROW || op == FS_REDUCE_COL)
    return 1;
  if (op == FS_RESHAPE || op == FS_BITCAST) return 1;
  if (op == FS_CONCAT) return 2;
  return -1;
}

const char* op_name(int op) {
  static const char* names[FS_NUM_OPCODES] = {
      "input", "const", "neg", "abs", "exp", "log", "tanh", "sigmoid", "sqrt", "rsqrt", "rcp", "gelu_tanh", "convert",
      "add", "sub", "mul", "div", "max", "min", "cmp", "select", "bcast_rowvec", "bcast_colvec", "transpose",
      "reduce_row", "reduce_col", "reshape", "bitcast", "concat"};
  return (op >= 0 && op < FS_NUM_OPCODES) ? names[op] : "?";
}

static bool is_float_dtype(int dt) { return dt == FS_F32 || dt == FS_BF16; }

// -------------------------------------------------------------------------------------------
// Reshape / Bitcast between elementwise regions (Table 1: the schedule passes through a Reshape when the split
// dimension survives).  Tensors are dense and row-major, so a Row schedule cut along dimension 0 owns a run of
// consecutive elements whatever [rows, cols] that run is labelled with: an elementwise region - unary, binary,
// compare and select ops whose operands are whole tensors or constants, no broadcast, no reduction, no transpose -
// computes the same thing under either label.  For a view v = reshape(p) the region on one side is therefore
// re-labelled with the shape of the other side and v becomes transparent (its users read p directly), so that
// both sides can share a kernel.  Tried in this order:
//   down  the users of v, and what follows them, are such a region ending in plan outputs: they take p's shape
//         (p's side keeps its row structure: a softmax followed, through a reshape, by a residual add is one kernel);
//   up    p and what it is computed from are such a region used by nothing else: they take v's shape (an activation
//         followed, through a reshape, by a reduction over the new rows is one kernel).
// Where a re-labelled node reads a tensor that keeps its own label (a plan input, another kernel's result), the
// operand slot is marked flat_in: the kernel addresses it by row * C + column of its own work space, which is the
// same element.  A concat or a transpose at the edge of a region stops the re-labelling (inside a kernel they are
// free, alone they would cost a launch).  Node ids, dtypes and values are untouched.
// -------------------------------------------------------------------------------------------
static bool is_elementwise_op(int op) { return op_is_unary(op) || op_is_binary(op) || op == FS_CMP || op == FS_SELECT; }

static void absorb_views(Graph* g) {
  const int N = g->n();
  g->flat_in.assign(N, {{0, 0, 0}});
  g->views_absorbed = 0;
  auto rebuild_users = [&]() {
    // a view nothing reads any more (and that is no plan output) is dead: it does not count as a user
    std::vector<char> live(N, 1);
    std::vector<int> n_users(N, 0);
    for (int id = 0; id < N; ++id)
      for (int k = 0; k < g->nodes[id].num_in; ++k) ++n_users[g->nodes[id].in[k]];
    for (int id = N - 1; id >= 0; --id)
      if (op_is_view(g->nodes[id].opcode) && n_users[id] == 0 && g->output_index[id] < 0) {
        live[id] = 0;
        --n_users[g->nodes[id].in[0]];
      }
    g->users.assign(N, {});
    for (int id = 0; id < N; ++id)
      if (live[id])
        for (int k = 0; k < g->nodes[id].num_in; ++k) g->users[g->nodes[id].in[k]].push_back(id);
  };
  auto same_shape = [&](int x, int rows, int cols) { return g->nodes[x].rows == rows && g->nodes[x].cols == cols; };
  // may `o` stay outside a re-labelled region and be read flat by it?
  auto flat_readable = [&](int o) {
    const int op = g->nodes[o].opcode;
    return op != FS_BCAST_ROWVEC && op != FS_BCAST_COLVEC && op != FS_CONCAT && op != FS_TRANSPOSE;
  };
  for (int v = 0; v < N; ++v) {
    if (!op_is_view(g->nodes[v].opcode)) continue;
    const int p = g->nodes[v].in[0];
    const fs_node pn = g->nodes[p], vn = g->nodes[v];
    if (op_is_free(pn.opcode) || g->users[v].empty()) continue;  // views of inputs and of views cost nothing as they are
    if (pn.rows == vn.rows && pn.cols == vn.cols) continue;
    std::vector<char> in_region(N, 0);
    std::vector<int> region;
    bool ok = true;
    // ---- down: everything downstream of v, up to plan outputs
    {
      std::vector<int> stack(g->users[v].begin(), g->users[v].end());
      while (!stack.empty() && ok) {
        const int u = stack.back();
        stack.pop_back();
        if (in_region[u]) continue;
        const fs_node& un = g->nodes[u];
        if (!is_elementwise_op(un.opcode) || !same_shape(u, vn.rows, vn.cols)) { ok = false; break; }
        in_region[u] = 1;
        region.push_back(u);
        for (int w : g->users[u]) stack.push_back(w);
      }
      // side inputs of the region that are elementwise work for it alone (a convert of a residual) come along
      for (bool grew = ok; grew;) {
        grew = false;
        for (size_t r = 0; r < region.size(); ++r) {
          const fs_node& rn = g->nodes[region[r]];
          for (int k = 0; k < rn.num_in; ++k) {
            const int o = rn.in[k];
            if (o == v || in_region[o] || !is_elementwise_op(g->nodes[o].opcode) || !same_shape(o, vn.rows, vn.cols) || g->output_index[o] >= 0) continue;
            bool all_inside = true, readable = true;
            for (int w : g->users[o]) all_inside &= (bool)in_region[w];
            for (int q = 0; q < g->nodes[o].num_in; ++q) {
              const int oo = g->nodes[o].in[q];
              readable &= g->nodes[oo].opcode == FS_CONST || (flat_readable(oo) && same_shape(oo, vn.rows, vn.cols));
            }
            if (all_inside && readable) in_region[o] = 1, region.push_back(o), grew = true;
          }
        }
      }
      for (int u : region)
        for (int k = 0; k < g->nodes[u].num_in && ok; ++k) {
          const int o = g->nodes[u].in[k];
          if (o != v && !in_region[o] && g->nodes[o].opcode != FS_CONST && !(flat_readable(o) && same_shape(o, vn.rows, vn.cols))) ok = false;
        }
      if (ok && !region.empty()) {
        for (int u : region) {
          fs_node& un = g->nodes[u];
          for (int k = 0; k < un.num_in; ++k) {
            if (un.in[k] == v) un.in[k] = p;
            else if (!in_region[un.in[k]]) g->flat_in[u][k] = 1;
          }
          un.rows = pn.rows, un.cols = pn.cols;
        }
        ++g->views_absorbed;
        rebuild_users();
        continue;
      }
    }
    // ---- up: p and what it is computed from, used by nothing but this view
    std::fill(in_region.begin(), in_region.end(), 0);
    region.clear();
    if (!is_elementwise_op(pn.opcode) || g->users[p].size() != 1 || g->output_index[p] >= 0) continue;
    in_region[p] = 1;
    region.push_back(p);
    for (bool grew = true; grew;) {  // an operand joins once every one of its users is inside
      grew = false;
      for (size_t r = 0; r < region.size(); ++r) {
        const fs_node& rn = g->nodes[region[r]];
        for (int k = 0; k < rn.num_in; ++k) {
          const int o = rn.in[k];
          if (in_region[o] || !is_elementwise_op(g->nodes[o].opcode) || !same_shape(o, pn.rows, pn.cols) || g->output_index[o] >= 0) continue;
          bool all_inside = true;
          for (int w : g->users[o]) all_inside &= (bool)in_region[w];
          if (all_inside) in_region[o] = 1, region.push_back(o), grew = true;
        }
      }
    }
    // drop members whose operands cannot be read flat, and whoever depends on having them inside, until it settles
    for (bool changed = true; changed && in_region[p];) {
      changed = false;
      for (int u : region) {
        if (!in_region[u]) continue;
        bool good = true;
        for (int k = 0; k < g->nodes[u].num_in; ++k) {
          const int o = g->nodes[u].in[k];
          if (!in_region[o] && g->nodes[o].opcode != FS_CONST && !(flat_readable(o) && same_shape(o, pn.rows, pn.cols))) good = false;
        }
        for (int w : g->users[u])
          if (w != v && !in_region[w]) good = false;
        if (!good) in_region[u] = 0, changed = true;
      }
    }
    if (!in_region[p]) continue;
    for (int u : region) {
      if (!in_region[u]) continue;
      fs_node& un = g->nodes[u];
      for (int k = 0; k < un.num_in; ++k)
        if (!in_region[un.in[k]]) g->flat_in[u][k] = 1;
      un.rows = vn.rows, un.cols = vn.cols;
    }
    for (int u : std::vector<int>(g->users[v]))
      for (int k = 0; k < g->nodes[u].num_in; ++k)
        if (g->nodes[u].in[k] == v) g->nodes[u].in[k] = p;
    ++g->views_absorbed;
    rebuild_users();
  }
}

fs_status build_graph(const fs_graph_desc* desc, Graph* g) {
  if (!desc) FS_FAIL(FS_ERR_INVALID_ARG, "desc is NULL");
  if (desc->abi_version != FS_ABI_VERSION)
    FS_FAIL(FS_ERR_INVALID_ARG, "abi_version %u, library speaks %u", desc->abi_version, FS_ABI_VERSION);
  if (desc->num_nodes <= 0 || !desc->nodes) FS_FAIL(FS_ERR_INVALID_ARG, "no nodes");
  if (desc->num_outputs <= 0 || !desc->outputs) FS_FAIL(FS_ERR_INVALID_ARG, "no outputs");
  if ((desc->mode & ~(uint32_t)(FS_MODE_UNFUSED | FS_MODE_NO_PERFLIB | FS_MODE_LAYERED)) != 0) FS_FAIL(FS_ERR_INVALID_ARG, "unknown mode %u", desc->mode);
  if (desc->lds_budget_bytes < 0 || desc->lds_budget_bytes > device_limits().lds_per_workgroup)
    FS_FAIL(FS_ERR_INVALID_ARG, "lds_budget_bytes %d outside [0, %d] (the most one workgroup may use on this device)", desc->lds_budget_bytes,
            device_limits().lds_per_workgroup);

  const int N = desc->num_nodes;
  g->nodes.assign(desc->nodes, desc->nodes + N);
  g->users.assign(N, {});
  g->input_index.assign(N, -1);
  g->output_index.assign(N, -1);
  g->input_ids.clear();

  for (int id = 0; id < N; ++id) {
    const fs_node& n = g->nodes[id];
    const int ar = op_arity(n.opcode);
    if (ar < 0) FS_FAIL(FS_ERR_BAD_GRAPH, "node %d: unknown opcode %d", id, n.opcode);
    if (n.num_in != ar) FS_FAIL(FS_ERR_BAD_GRAPH, "node %d (%s): arity %d, expected %d", id, op_name(n.opcode), n.num_in, ar);
    if (n.dtype != FS_F32 && n.dtype != FS_BF16 && n.dtype != FS_U8) FS_FAIL(FS_ERR_DTYPE, "node %d: unknown dtype %d", id, n.dtype);
    if (n.rows < 1 || n.cols < 1) FS_FAIL(FS_ERR_SHAPE, "node %d: shape [%d,%d]", id, n.rows, n.cols);
    if ((int64_t)n.rows * n.cols > ((int64_t)1 << 40)) FS_FAIL(FS_ERR_SHAPE, "node %d: too large", id);
    for (int k = 0; k < ar; ++k) {
      if (n.in[k] < 0 || n.in[k] >= id)
        FS_FAIL(FS_ERR_BAD_GRAPH, "node %d (%s): operand %d is node %d; ids must be topological (operand id < node id)", id,
                op_name(n.opcode), k, n.in[k]);
    }
    const fs_node* a = ar > 0 ? &g->nodes[n.in[0]] : nullptr;
    const fs_node* b = ar > 1 ? &g->nodes[n.in[1]] : nullptr;
    const fs_node* c = ar > 2 ? &g->nodes[n.in[2]] : nullptr;
    auto same_shape = [&](const fs_node* x) { return x->rows == n.rows && x->cols == n.cols; };
    const int op = n.opcode;

    if (op == FS_INPUT) {
      g->input_index[id] = (int)g->input_ids.size();
      g->input_ids.push_back(id);
    } else if (op == FS_CONST) {
      if (!is_float_dtype(n.dtype)) FS_FAIL(FS_ERR_DTYPE, "node %d (const): dtype must be f32 or bf16", id);
    } else if (op == FS_CONVERT) {
      if (!same_shape(a)) FS_FAIL(FS_ERR_SHAPE, "node %d (convert): shape differs from operand", id);
      if (!is_float_dtype(n.dtype)) FS_FAIL(FS_ERR_DTYPE, "node %d (convert): target must be f32 or bf16", id);
    } else if (op_is_unary(op)) {
      if (!same_shape(a)) FS_FAIL(FS_ERR_SHAPE, "node %d (%s): shape differs from operand", id, op_name(op));
      if (!is_float_dtype(n.dtype) || !is_float_dtype(a->dtype)) FS_FAIL(FS_ERR_DTYPE, "node %d (%s): needs f32/bf16", id, op_name(op));
    } else if (op_is_binary(op)) {
      if (!same_shape(a) || !same_shape(b)) FS_FAIL(FS_ERR_SHAPE, "node %d (%s): operand shapes differ from result", id, op_name(op));
      if (!is_float_dtype(n.dtype) || !is_float_dtype(a->dtype) || !is_float_dtype(b->dtype))
        FS_FAIL(FS_ERR_DTYPE, "node %d (%s): needs f32/bf16", id, op_name(op));
    } else if (op == FS_CMP) {
      if (!same_shape(a) || !same_shape(b)) FS_FAIL(FS_ERR_SHAPE, "node %d (cmp): operand shapes differ from result", id);
      if (n.dtype != FS_U8) FS_FAIL(FS_ERR_DTYPE, "node %d (cmp): result must be u8", id);
      if (!is_float_dtype(a->dtype) || !is_float_dtype(b->dtype)) FS_FAIL(FS_ERR_DTYPE, "node %d (cmp): operands must be f32/bf16", id);
      if (n.attr_i < FS_CMP_GT || n.attr_i > FS_CMP_NE) FS_FAIL(FS_ERR_BAD_GRAPH, "node %d (cmp): kind %d", id, n.attr_i);
    } else if (op == FS_SELECT) {
      if (!same_shape(a) || !same_shape(b) || !same_shape(c)) FS_FAIL(FS_ERR_SHAPE, "node %d (select): operand shapes differ", id);
      if (a->dtype != FS_U8) FS_FAIL(FS_ERR_DTYPE, "node %d (select): predicate must be u8", id);
      if (b->dtype != n.dtype || c->dtype != n.dtype) FS_FAIL(FS_ERR_DTYPE, "node %d (select): branches must have the result dtype", id);
    } else if (op == FS_BCAST_ROWVEC) {
      if (a->rows != 1 || a->cols != n.cols) FS_FAIL(FS_ERR_SHAPE, "node %d (bcast_rowvec): operand must be [1,%d]", id, n.cols);
      if (a->dtype != n.dtype) FS_FAIL(FS_ERR_DTYPE, "node %d (bcast_rowvec): dtype differs from operand", id);
      if (op_is_free(a->opcode) && a->opcode != FS_INPUT && a->opcode != FS_CONST && !op_is_view(a->opcode))
        FS_FAIL(FS_ERR_BAD_GRAPH, "node %d: broadcast of a broadcast", id);
    } else if (op == FS_BCAST_COLVEC) {
      if (a->cols != 1 || a->rows != n.rows) FS_FAIL(FS_ERR_SHAPE, "node %d (bcast_colvec): operand must be [%d,1]", id, n.rows);
      if (a->dtype != n.dtype) FS_FAIL(FS_ERR_DTYPE, "node %d (bcast_colvec): dtype differs from operand", id);
      if (op_is_free(a->opcode) && a->opcode != FS_INPUT && a->opcode != FS_CONST && !op_is_view(a->opcode))
        FS_FAIL(FS_ERR_BAD_GRAPH, "node %d: broadcast of a broadcast", id);
    } else if (op == FS_TRANSPOSE) {
      if (a->rows != n.cols || a->cols != n.rows) FS_FAIL(FS_ERR_SHAPE, "node %d (transpose): result must be [%d,%d]", id, a->cols, a->rows);
      if (a->dtype != n.dtype) FS_FAIL(FS_ERR_DTYPE, "node %d (transpose): dtype differs from operand", id);
    } else if (op_is_view(op)) {
      if ((int64_t)a->rows * a->cols != (int64_t)n.rows * n.cols)
        FS_FAIL(FS_ERR_SHAPE, "node %d (%s): [%d,%d] holds another number of elements than its operand [%d,%d]", id, op_name(op), n.rows, n.cols, a->rows, a->cols);
      if (a->dtype != n.dtype) FS_FAIL(FS_ERR_DTYPE, "node %d (%s): dtype differs from operand", id, op_name(op));
      if (a->opcode == FS_CONST || a->opcode == FS_BCAST_ROWVEC || a->opcode == FS_BCAST_COLVEC)
        FS_FAIL(FS_ERR_BAD_GRAPH, "node %d (%s): a view of node %d (%s), which is never materialised", id, op_name(op), n.in[0], op_name(a->opcode));
    } else if (op == FS_CONCAT) {
      if (n.attr_i == FS_CONCAT_COLS) {
        if (a->rows != n.rows || b->rows != n.rows || (int64_t)a->cols + b->cols != n.cols)
          FS_FAIL(FS_ERR_SHAPE, "node %d (concat along columns): [%d,%d] ++ [%d,%d] is not [%d,%d]", id, a->rows, a->cols, b->rows, b->cols, n.rows, n.cols);
      } else if (n.attr_i == FS_CONCAT_ROWS) {
        if (a->cols != n.cols || b->cols != n.cols || (int64_t)a->rows + b->rows != n.rows)
          FS_FAIL(FS_ERR_SHAPE, "node %d (concat along rows): [%d,%d] over [%d,%d] is not [%d,%d]", id, a->rows, a->cols, b->rows, b->cols, n.rows, n.cols);
      } else {
        FS_FAIL(FS_ERR_BAD_GRAPH, "node %d (concat): axis %d", id, n.attr_i);
      }
      if (a->dtype != n.dtype || b->dtype != n.dtype) FS_FAIL(FS_ERR_DTYPE, "node %d (concat): operands must have the result dtype", id);
      for (const fs_node* x : {a, b})
        if (x->opcode == FS_CONST || x->opcode == FS_BCAST_ROWVEC || x->opcode == FS_BCAST_COLVEC)
          FS_FAIL(FS_ERR_BAD_GRAPH, "node %d (concat): operands must be tensors in memory, not broadcasts or constants", id);
    } else if (op == FS_REDUCE_ROW || op == FS_REDUCE_COL) {
      if (op == FS_REDUCE_ROW && (a->rows != n.rows || n.cols != 1)) FS_FAIL(FS_ERR_SHAPE, "node %d (reduce_row): result must be [%d,1]", id, a->rows);
      if (op == FS_REDUCE_COL && (a->cols != n.cols || n.rows != 1)) FS_FAIL(FS_ERR_SHAPE, "node %d (reduce_col): result must be [1,%d]", id, a->cols);
      if (!is_float_dtype(n.dtype) || !is_float_dtype(a->dtype)) FS_FAIL(FS_ERR_DTYPE, "node %d (reduce): needs f32/bf16", id);
      if (n.attr_i < FS_RED_SUM || n.attr_i > FS_RED_MEAN) FS_FAIL(FS_ERR_BAD_GRAPH, "node %d (reduce): kind %d", id, n.attr_i);
    }
    for (int k = 0; k < ar; ++k) g->users[n.in[k]].push_back(id);
  }

  // every ancestor of a predicate operand must be computed with exactly the roundings the graph
  // spells out, or the predicate would not be reproducible bit for bit
  g->exact.assign(N, 0);
  for (int id = N - 1; id >= 0; --id) {
    const fs_node& n = g->nodes[id];
    if (n.opcode == FS_CMP || g->exact[id])
      for (int k = 0; k < n.num_in; ++k) g->exact[n.in[k]] = 1;
  }

  // a view's bytes are those of the node its chain of views starts from
  g->root_of.assign(N, 0);
  for (int id = 0; id < N; ++id) g->root_of[id] = op_is_view(g->nodes[id].opcode) ? g->root_of[g->nodes[id].in[0]] : id;

  g->outputs.clear();
  std::vector<int>& family_output = g->family_output;  // root -> the plan output that lives in its family's buffer
  family_output.assign(N, -1);
  for (int k = 0; k < desc->num_outputs; ++k) {
    const int o = desc->outputs[k];
    if (o < 0 || o >= N) FS_FAIL(FS_ERR_BAD_GRAPH, "output %d: node id %d out of range", k, o);
    const int root = g->root_of[o];
    if (op_is_free(g->nodes[root].opcode))
      FS_FAIL(FS_ERR_BAD_GRAPH, "output %d: node %d (%s) is never materialised%s", k, o, op_name(g->nodes[o].opcode),
              root != o ? " (a view of a plan input computes nothing)" : "");
    if (g->output_index[o] >= 0) FS_FAIL(FS_ERR_BAD_GRAPH, "output %d: node %d listed twice", k, o);
    if (family_output[root] >= 0)
      FS_FAIL(FS_ERR_BAD_GRAPH, "outputs %d and %d (nodes %d and %d) are views of the same value: list one of them", family_output[root], k,
              g->outputs[family_output[root]], o);
    family_output[root] = k;
    g->output_index[o] = k;
    g->outputs.push_back(o);
  }

  // views between elementwise regions become transparent (operand edges and shape labels change, ids do not);
  // what was derived from the edges is derived again
  absorb_views(g);
  if (g->views_absorbed > 0) {
    g->exact.assign(N, 0);
    for (int id = N - 1; id >= 0; --id) {
      const fs_node& n = g->nodes[id];
      if (n.opcode == FS_CMP || g->exact[id])
        for (int k = 0; k < n.num_in; ++k) g->exact[n.in[k]] = 1;
    }
  }
  return FS_OK;
}

}  // namespace fs
