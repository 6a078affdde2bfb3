/*
 * fso.c - CPU ORACLE (test infrastructure only; see fso.h).
 *
 * Evaluation rule, chosen because the paper inherits the numerical semantics of the
 * framework's ops without restating them (Section 1 names the op kinds only):
 *   - nodes are processed in id order, one op at a time, each one's whole tensor
 *     materialised before any consumer runs;
 *   - inside an op everything is fp64: operands are widened, transcendental functions
 *     come from the C math library, reductions accumulate sequentially in index order;
 *   - the result is rounded ONCE (nearest-even) to the node's declared dtype.  For
 *     + - * / sqrt this equals the correctly rounded fp32 operation (53 >= 2*24+2 bits
 *     makes the double rounding innocuous), which is what makes predicates reproducible
 *     bit for bit.
 * Every tensor is held as an array of double whose values are exactly representable
 * in the node's dtype.
 */
#include "fso.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

double fso_round_f32(double x) { return (double)(float)x; }

/* fp64 -> bfloat16 (8 significant bits, fp32's exponent range), nearest-even, as a double. */
double fso_round_bf16(double x) {
  if (x == 0.0 || isnan(x) || isinf(x)) return x;
  int e;
  double m = frexp(x, &e); /* x = m * 2^e, 0.5 <= |m| < 1 */
  double r;
  if (e - 1 < -126) {
    /* below the smallest normal 2^-126: fixed quantum 2^-133 (7 fraction bits) */
    r = ldexp(nearbyint(ldexp(x, 133)), -133);
  } else {
    r = ldexp(nearbyint(ldexp(m, 8)), e - 8); /* 8 significant bits */
  }
  if (fabs(r) >= ldexp(1.0, 128)) r = copysign(INFINITY, x);
  return r;
}

static double round_to(int dtype, double x) {
  switch (dtype) {
    case FSO_F32: return fso_round_f32(x);
    case FSO_BF16: return fso_round_bf16(x);
    default: return x; /* u8 values are already 0/1 */
  }
}

static double bf16_bits_to_double(uint16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return (double)f;
}

static uint16_t double_to_bf16_bits(double x) { /* x is already bf16-representable (or gets rounded here) */
  float f = (float)fso_round_bf16(x);
  uint32_t u;
  memcpy(&u, &f, 4);
  return (uint16_t)(u >> 16);
}

static int arity(int op) {
  if (op == FSO_INPUT || op == FSO_CONST) return 0;
  if (op >= FSO_NEG && op <= FSO_CONVERT) return 1;
  if (op >= FSO_ADD && op <= FSO_CMP) return 2;
  if (op == FSO_SELECT) return 3;
  if (op >= FSO_BCAST_ROWVEC && op <= FSO_REDUCE_COL) return 1;
  if (op == FSO_RESHAPE || op == FSO_BITCAST) return 1;
  if (op == FSO_CONCAT) return 2;
  return -1;
}

static double unary_f64(int op, double x) {
  switch (op) {
    case FSO_NEG: return -x;
    case FSO_ABS: return fabs(x);
    case FSO_EXP: return exp(x);
    case FSO_LOG: return log(x);
    case FSO_TANH: return tanh(x);
    case FSO_SIGMOID: return 1.0 / (1.0 + exp(-x));
    case FSO_SQRT: return sqrt(x);
    case FSO_RSQRT: return 1.0 / sqrt(x);
    case FSO_RCP: return 1.0 / x;
    case FSO_GELU_TANH: {
      const double k = 0.7978845608028654; /* sqrt(2/pi) */
      return 0.5 * x * (1.0 + tanh(k * (x + 0.044715 * x * x * x)));
    }
    case FSO_CONVERT: return x;
  }
  return NAN;
}

static double binary_f64(int op, double a, double b) {
  switch (op) {
    case FSO_ADD: return a + b;
    case FSO_SUB: return a - b;
    case FSO_MUL: return a * b;
    case FSO_DIV: return a / b;
    case FSO_MAX: return fmax(a, b);
    case FSO_MIN: return fmin(a, b);
  }
  return NAN;
}

static double cmp_f64(int kind, double a, double b) {
  switch (kind) {
    case FSO_GT: return a > b;
    case FSO_GE: return a >= b;
    case FSO_LT: return a < b;
    case FSO_LE: return a <= b;
    case FSO_EQ: return a == b;
    case FSO_NE: return a != b;
  }
  return 0.0;
}

/* ---- companion 3: the spread of a correct fp32 implementation around the reference, to first order ----------------
 * Model: every correctly rounded fp32 op errs by a value uniform in +-half a spacing, spread spacing/sqrt(12), the
 * spacing taken at its upper end 2^-23 |result|; exp, log, tanh, sigmoid, rsqrt, rcp and gelu, which a GPU builds on
 * hardware approximations good to 1-2 spacings, err by one spacing; a sum accumulated in fp32 rounds every partial sum
 * of a balanced pairwise summation.  Rounding errors are independent: they travel through each op's derivative and add
 * in quadrature.  The errors of approximated ops are not noise - an approximation leans one way over a range of
 * arguments - so they travel through the derivatives' absolute values and add linearly.  The spread of an element is
 * the sum of the two parts.  Inputs, constants and predicates are exact. */
static double spacing32(double x) { return ldexp(fabs(x), -23); }
#define FSO_SPREAD_ROUNDED 0.28867513459481287 /* 1/sqrt(12) */
static int is_approximated(int op) {
  return op == FSO_EXP || op == FSO_LOG || op == FSO_TANH || op == FSO_SIGMOID || op == FSO_RSQRT || op == FSO_RCP || op == FSO_GELU_TANH;
}
static double unary_f64(int op, double x);
/* |f'(x)| by a central difference in fp64 (one-sided at the edge of a domain) */
static double unary_slope(int op, double x) {
  if (op == FSO_NEG || op == FSO_ABS || op == FSO_CONVERT) return 1.0;
  const double h = 1e-6 * fmax(1.0, fabs(x));
  double lo = x - h, hi = x + h;
  if ((op == FSO_LOG || op == FSO_SQRT || op == FSO_RSQRT) && lo <= 0.0) lo = x;
  if (op == FSO_RCP && ((lo < 0.0) != (hi < 0.0))) lo = x;
  const double d = (unary_f64(op, hi) - unary_f64(op, lo)) / (hi - lo);
  return isfinite(d) ? fabs(d) : 0.0;
}
static double local_spread(const fso_node* n, double value) {
  if (n->dtype != FSO_F32) return 0.0; /* bf16 nodes: their rounding decisions are shared with the path under test by the tests */
  return spacing32(value) * (is_approximated(n->opcode) ? 1.0 : FSO_SPREAD_ROUNDED);
}
static double quad(double a, double b) { return sqrt(a * a + b * b); }
/* variance that rounding every partial sum of a balanced pairwise summation to fp32 adds to the total; *sum = the total */
static double pairwise_rounding_variance(const double* p, long n, long stride, double* sum) {
  if (n == 1) { *sum = p[0]; return 0.0; }
  double sl, sr;
  const long h = n / 2;
  const double v = pairwise_rounding_variance(p, h, stride, &sl) + pairwise_rounding_variance(p + h * stride, n - h, stride, &sr);
  *sum = sl + sr;
  const double e = FSO_SPREAD_ROUNDED * spacing32(*sum);
  return v + e * e;
}

/* sequential reduction of n values spaced `stride` apart; displaced: sums are moved by
 * 2^-24 * sum |terms| (the accumulation companion, see fso.h) */
static double reduce_f64(int kind, const double* p, long n, long stride, int acc32) {
  double acc;
  long i;
  switch (kind) {
    case FSO_SUM:
    case FSO_MEAN:
      acc = 0.0;
      for (i = 0; i < n; ++i) acc += p[i * stride];
      if (acc32) {
        double mag = 0.0;
        for (i = 0; i < n; ++i) mag += fabs(p[i * stride]);
        acc += ldexp(mag, -24);
      }
      return kind == FSO_MEAN ? acc / (double)n : acc;
    case FSO_MAX_:
      acc = p[0];
      for (i = 1; i < n; ++i) acc = fmax(acc, p[i * stride]);
      return acc;
    case FSO_MIN_:
      acc = p[0];
      for (i = 1; i < n; ++i) acc = fmin(acc, p[i * stride]);
      return acc;
  }
  return NAN;
}

int fso_run(const fso_graph* g, const void* const* host_in, void* const* host_out, int num_threads, int round_nodes) {
  if (!g || !g->nodes || g->num_nodes <= 0 || (g->num_outputs > 0 && (!g->outputs || !host_out))) return -1;
  if (num_threads < 1) num_threads = 1;
#ifdef _OPENMP
  omp_set_num_threads(num_threads);
#endif
  const int N = g->num_nodes;
  const int acc32 = round_nodes == 2;
  const int spread = round_nodes == 3;
  int id, k;

  /* structural checks: topological ids, arity, shapes */
  for (id = 0; id < N; ++id) {
    const fso_node* n = &g->nodes[id];
    if (arity(n->opcode) < 0 || n->num_in != arity(n->opcode) || n->rows < 1 || n->cols < 1) return -2;
    for (k = 0; k < n->num_in; ++k)
      if (n->in[k] < 0 || n->in[k] >= id) return -2;
    if (n->num_in >= 1) {
      const fso_node* a = &g->nodes[n->in[0]];
      switch (n->opcode) {
        case FSO_BCAST_ROWVEC: if (a->rows != 1 || a->cols != n->cols) return -2; break;
        case FSO_BCAST_COLVEC: if (a->cols != 1 || a->rows != n->rows) return -2; break;
        case FSO_TRANSPOSE: if (a->rows != n->cols || a->cols != n->rows) return -2; break;
        case FSO_REDUCE_ROW: if (a->rows != n->rows || n->cols != 1) return -2; break;
        case FSO_REDUCE_COL: if (a->cols != n->cols || n->rows != 1) return -2; break;
        case FSO_RESHAPE:
        case FSO_BITCAST: if ((long)a->rows * a->cols != (long)n->rows * n->cols) return -2; break;
        case FSO_CONCAT: {
          const fso_node* b = &g->nodes[n->in[1]];
          if (n->attr_i == 1) { if (a->rows != n->rows || b->rows != n->rows || a->cols + b->cols != n->cols) return -2; }
          else if (n->attr_i == 0) { if (a->cols != n->cols || b->cols != n->cols || a->rows + b->rows != n->rows) return -2; }
          else return -2;
          break;
        }
        default:
          for (k = 0; k < n->num_in; ++k) {
            const fso_node* b = &g->nodes[n->in[k]];
            if (b->rows != n->rows || b->cols != n->cols) return -2;
          }
      }
    }
  }
  for (k = 0; k < g->num_outputs; ++k)
    if (g->outputs[k] < 0 || g->outputs[k] >= N) return -2;

  /* last consumer of every node, so its buffer can be freed early */
  int* last_use = (int*)malloc(sizeof(int) * (size_t)N);
  double** val = (double**)calloc((size_t)N, sizeof(double*));
  double** sig = (double**)calloc((size_t)N, sizeof(double*)); /* companion 3: the spread of every node's elements */
  if (!last_use || !val || !sig) { free(last_use); free(val); free(sig); return -3; }
  for (id = 0; id < N; ++id) last_use[id] = id;
  for (id = 0; id < N; ++id)
    for (k = 0; k < g->nodes[id].num_in; ++k) last_use[g->nodes[id].in[k]] = id;
  for (k = 0; k < g->num_outputs; ++k) last_use[g->outputs[k]] = N; /* keep until the end */

  int rc = 0, in_idx = 0;
  for (id = 0; id < N && rc == 0; ++id) {
    const fso_node* n = &g->nodes[id];
    const long R = n->rows, C = n->cols, E = R * C;
    double* out = (double*)malloc(sizeof(double) * (size_t)E);
    if (!out) { rc = -3; break; }
    val[id] = out;
    const double* a = n->num_in > 0 ? val[n->in[0]] : NULL;
    const double* b = n->num_in > 1 ? val[n->in[1]] : NULL;
    const double* c = n->num_in > 2 ? val[n->in[2]] : NULL;
    const int dt = round_nodes ? n->dtype : FSO_U8 /* = leave untouched */;
    long i, j;

    switch (n->opcode) {
      case FSO_INPUT: {
        const void* src = host_in ? host_in[in_idx] : NULL;
        ++in_idx;
        if (!src) { rc = -1; break; }
        if (n->dtype == FSO_F32) {
          const float* s = (const float*)src;
#pragma omp parallel for
          for (i = 0; i < E; ++i) out[i] = (double)s[i];
        } else if (n->dtype == FSO_BF16) {
          const uint16_t* s = (const uint16_t*)src;
#pragma omp parallel for
          for (i = 0; i < E; ++i) out[i] = bf16_bits_to_double(s[i]);
        } else {
          const uint8_t* s = (const uint8_t*)src;
#pragma omp parallel for
          for (i = 0; i < E; ++i) out[i] = s[i] ? 1.0 : 0.0;
        }
        break;
      }
      case FSO_CONST: {
        const double v = round_to(dt, (double)n->attr_f);
        for (i = 0; i < E; ++i) out[i] = v;
        break;
      }
      case FSO_CMP:
#pragma omp parallel for private(j)
        for (i = 0; i < R; ++i)
          for (j = 0; j < C; ++j) out[i * C + j] = cmp_f64(n->attr_i, a[i * C + j], b[i * C + j]);
        break;
      case FSO_SELECT:
#pragma omp parallel for private(j)
        for (i = 0; i < R; ++i)
          for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, a[i * C + j] != 0.0 ? b[i * C + j] : c[i * C + j]);
        break;
      case FSO_BCAST_ROWVEC:
#pragma omp parallel for private(j)
        for (i = 0; i < R; ++i)
          for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, a[j]);
        break;
      case FSO_BCAST_COLVEC:
#pragma omp parallel for private(j)
        for (i = 0; i < R; ++i)
          for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, a[i]);
        break;
      case FSO_TRANSPOSE: /* out is [R,C], operand is [C,R] */
#pragma omp parallel for private(j)
        for (i = 0; i < R; ++i)
          for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, a[j * R + i]);
        break;
      case FSO_RESHAPE:
      case FSO_BITCAST: /* the same row-major element sequence under another [rows, cols] split */
#pragma omp parallel for
        for (i = 0; i < E; ++i) out[i] = round_to(dt, a[i]);
        break;
      case FSO_CONCAT:
        if (n->attr_i == 1) { /* along columns: row i is in0's row i followed by in1's row i */
          const long Ca = g->nodes[n->in[0]].cols, Cb = g->nodes[n->in[1]].cols;
#pragma omp parallel for private(j)
          for (i = 0; i < R; ++i)
            for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, j < Ca ? a[i * Ca + j] : b[i * Cb + (j - Ca)]);
        } else { /* along rows: in0's rows, then in1's */
          const long Ra = g->nodes[n->in[0]].rows;
#pragma omp parallel for private(j)
          for (i = 0; i < R; ++i)
            for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, i < Ra ? a[i * C + j] : b[(i - Ra) * C + j]);
        }
        break;
      case FSO_REDUCE_ROW: { /* operand [R, Ca] -> [R,1] */
        const long Ca = g->nodes[n->in[0]].cols;
#pragma omp parallel for
        for (i = 0; i < R; ++i) out[i] = round_to(dt, reduce_f64(n->attr_i, a + i * Ca, Ca, 1, acc32));
        break;
      }
      case FSO_REDUCE_COL: { /* operand [Ra, C] -> [1,C] */
        const long Ra = g->nodes[n->in[0]].rows;
#pragma omp parallel for
        for (j = 0; j < C; ++j) out[j] = round_to(dt, reduce_f64(n->attr_i, a + j, Ra, C, acc32));
        break;
      }
      default:
        if (n->num_in == 1) {
#pragma omp parallel for private(j)
          for (i = 0; i < R; ++i)
            for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, unary_f64(n->opcode, a[i * C + j]));
        } else if (n->num_in == 2) {
#pragma omp parallel for private(j)
          for (i = 0; i < R; ++i)
            for (j = 0; j < C; ++j) out[i * C + j] = round_to(dt, binary_f64(n->opcode, a[i * C + j], b[i * C + j]));
        } else {
          rc = -2;
        }
    }

    if (spread && rc == 0) {
      /* the same walk for the spreads.  Two parts per element: sg[0..E) rounding noise, independent from op to op and
       * element to element, added in quadrature; sg[E..2E) the error of approximated ops, which may lean one way
       * over many elements and is therefore added linearly, by absolute value. */
      double* sg = (double*)calloc((size_t)(2 * E), sizeof(double));
      if (!sg) { rc = -3; break; }
      sig[id] = sg;
      double* ch = sg + E;
      const long Ea = n->num_in > 0 ? (long)g->nodes[n->in[0]].rows * g->nodes[n->in[0]].cols : 0;
      const long Eb = n->num_in > 1 ? (long)g->nodes[n->in[1]].rows * g->nodes[n->in[1]].cols : 0;
      const long Ec = n->num_in > 2 ? (long)g->nodes[n->in[2]].rows * g->nodes[n->in[2]].cols : 0;
      const double* sa = n->num_in > 0 ? sig[n->in[0]] : NULL;
      const double* sb = n->num_in > 1 ? sig[n->in[1]] : NULL;
      const double* sc = n->num_in > 2 ? sig[n->in[2]] : NULL;
      const double* ca = sa ? sa + Ea : NULL;
      const double* cb = sb ? sb + Eb : NULL;
      const double* cc = sc ? sc + Ec : NULL;
#define FSO_MOVE(dst, src_a, src_c) do { sg[dst] = (src_a); ch[dst] = (src_c); } while (0)
      switch (n->opcode) {
        case FSO_INPUT: case FSO_CONST: case FSO_CMP: break; /* exact */
        case FSO_SELECT:
          for (i = 0; i < E; ++i) { if (a[i] != 0.0) FSO_MOVE(i, sb[i], cb[i]); else FSO_MOVE(i, sc[i], cc[i]); }
          break;
        case FSO_BCAST_ROWVEC:
          for (i = 0; i < R; ++i) for (j = 0; j < C; ++j) FSO_MOVE(i * C + j, sa[j], ca[j]);
          break;
        case FSO_BCAST_COLVEC:
          for (i = 0; i < R; ++i) for (j = 0; j < C; ++j) FSO_MOVE(i * C + j, sa[i], ca[i]);
          break;
        case FSO_TRANSPOSE:
          for (i = 0; i < R; ++i) for (j = 0; j < C; ++j) FSO_MOVE(i * C + j, sa[j * R + i], ca[j * R + i]);
          break;
        case FSO_RESHAPE: case FSO_BITCAST:
          for (i = 0; i < E; ++i) FSO_MOVE(i, sa[i], ca[i]);
          break;
        case FSO_CONCAT:
          if (n->attr_i == 1) {
            const long Ca = g->nodes[n->in[0]].cols, Cb = g->nodes[n->in[1]].cols;
            for (i = 0; i < R; ++i) for (j = 0; j < C; ++j) {
              if (j < Ca) FSO_MOVE(i * C + j, sa[i * Ca + j], ca[i * Ca + j]); else FSO_MOVE(i * C + j, sb[i * Cb + (j - Ca)], cb[i * Cb + (j - Ca)]);
            }
          } else {
            const long Ra = g->nodes[n->in[0]].rows;
            for (i = 0; i < R; ++i) for (j = 0; j < C; ++j) {
              if (i < Ra) FSO_MOVE(i * C + j, sa[i * C + j], ca[i * C + j]); else FSO_MOVE(i * C + j, sb[(i - Ra) * C + j], cb[(i - Ra) * C + j]);
            }
          }
          break;
        case FSO_REDUCE_ROW: case FSO_REDUCE_COL: {
          const int rowwise = n->opcode == FSO_REDUCE_ROW;
          const long cnt = rowwise ? g->nodes[n->in[0]].cols : g->nodes[n->in[0]].rows;
          const long outs = rowwise ? R : C, step = rowwise ? 1 : C;
          long t;
          for (i = 0; i < outs; ++i) {
            const long base = rowwise ? i * cnt : i;
            const double* p = a + base;
            if (n->attr_i == FSO_SUM || n->attr_i == FSO_MEAN) {
              double var = 0.0, lin = 0.0, total;
              for (t = 0; t < cnt; ++t) var += sa[base + t * step] * sa[base + t * step], lin += ca[base + t * step];
              double sd = sqrt(var + pairwise_rounding_variance(p, cnt, step, &total));
              if (n->attr_i == FSO_MEAN) sd = quad(sd / (double)cnt, local_spread(n, out[i])), lin /= (double)cnt;
              FSO_MOVE(i, sd, lin);
            } else { /* max / min: the spread of the element that was picked */
              long pick = 0;
              for (t = 1; t < cnt; ++t)
                if (n->attr_i == FSO_MAX_ ? p[t * step] > p[pick * step] : p[t * step] < p[pick * step]) pick = t;
              FSO_MOVE(i, sa[base + pick * step], ca[base + pick * step]);
            }
          }
          break;
        }
        default:
          if (n->num_in == 1) {
            const int approx = is_approximated(n->opcode), moves = n->opcode == FSO_NEG || n->opcode == FSO_ABS;
#pragma omp parallel for
            for (i = 0; i < E; ++i) {
              const double slope = unary_slope(n->opcode, a[i]), own = moves ? 0.0 : local_spread(n, out[i]);
              sg[i] = approx ? slope * sa[i] : quad(slope * sa[i], own);
              ch[i] = slope * ca[i] + (approx ? own : 0.0);
            }
          } else if (n->num_in == 2) {
#pragma omp parallel for
            for (i = 0; i < E; ++i) {
              double sd, lin;
              switch (n->opcode) {
                case FSO_ADD: case FSO_SUB: sd = quad(sa[i], sb[i]), lin = ca[i] + cb[i]; break;
                case FSO_MUL: sd = quad(b[i] * sa[i], a[i] * sb[i]), lin = fabs(b[i]) * ca[i] + fabs(a[i]) * cb[i]; break;
                case FSO_DIV: sd = quad(sa[i] / b[i], a[i] * sb[i] / (b[i] * b[i])), lin = ca[i] / fabs(b[i]) + fabs(a[i]) * cb[i] / (b[i] * b[i]); break;
                case FSO_MAX: sd = a[i] >= b[i] ? sa[i] : sb[i], lin = a[i] >= b[i] ? ca[i] : cb[i]; break;
                default: sd = a[i] <= b[i] ? sa[i] : sb[i], lin = a[i] <= b[i] ? ca[i] : cb[i]; break; /* FSO_MIN */
              }
              sg[i] = (n->opcode == FSO_MAX || n->opcode == FSO_MIN) ? sd : quad(sd, local_spread(n, out[i]));
              ch[i] = lin;
            }
          }
      }
#undef FSO_MOVE
    }

    /* free operands whose last consumer this was */
    for (k = 0; k < n->num_in; ++k) {
      int o = n->in[k];
      if (last_use[o] == id && val[o]) { free(val[o]); val[o] = NULL; free(sig[o]); sig[o] = NULL; }
    }
    if (last_use[id] == id && val[id]) { free(val[id]); val[id] = NULL; free(sig[id]); sig[id] = NULL; } /* dead node */
  }

  /* write plan outputs in their dtype (fp64-through mode rounds here) */
  for (k = 0; k < g->num_outputs && rc == 0; ++k) {
    const int o = g->outputs[k];
    const fso_node* n = &g->nodes[o];
    const long E = (long)n->rows * n->cols;
    const double* v = val[o];
    long i;
    if (!v || !host_out[k]) { rc = -1; break; }
    if (spread) { /* companion 3 hands back the spreads, as doubles, whatever the output's dtype */
      double* d = (double*)host_out[k];
      for (i = 0; i < E; ++i) d[i] = sig[o] ? sig[o][i] + sig[o][E + i] : 0.0; /* noise + lean */
      continue;
    }
    if (n->dtype == FSO_F32) {
      float* d = (float*)host_out[k];
      for (i = 0; i < E; ++i) d[i] = (float)v[i];
    } else if (n->dtype == FSO_BF16) {
      uint16_t* d = (uint16_t*)host_out[k];
      for (i = 0; i < E; ++i) d[i] = double_to_bf16_bits(v[i]);
    } else {
      uint8_t* d = (uint8_t*)host_out[k];
      for (i = 0; i < E; ++i) d[i] = v[i] != 0.0;
    }
  }

  for (id = 0; id < N; ++id) free(val[id]), free(sig[id]);
  free(val);
  free(sig);
  free(last_use);
  return rc;
}
