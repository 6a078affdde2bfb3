/*
 * fso.h - CPU ORACLE for the stitched-kernel executor.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, one-op-at-a-time interpreter of a fusion plan (a DAG of
 * elementwise / broadcast / transpose / reduction ops on 2-D row-major tensors, the
 * op classes of the paper's Section 2.1).  Fusion changes where intermediates live, not
 * what is computed (Section 4.1 names footprint and launch count as the objectives;
 * Section 5.1.1 recomputes "to ensure correctness"), so the reference result of a fused
 * kernel is simply the op-by-op evaluation of its DAG: that is all this file does.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header or table with the GPU library: the structs below are
 * this library's own declaration of the plan layout.
 *
 * Parity pins (tests/test_oracle_pins.py): closed forms, invariants, brute force
 * in pure Python, numpy.float32 bit-equality of the basic arithmetic, torch CPU
 * fp64 softmax / layer_norm / gelu.  The paper prints no numerical example, so no
 * pin comes from paper-printed values.
 */
#ifndef FSO_H_
#define FSO_H_
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { FSO_F32 = 0, FSO_BF16 = 1, FSO_U8 = 2 };

enum {
  FSO_INPUT = 0, FSO_CONST = 1,
  FSO_NEG = 2, FSO_ABS = 3, FSO_EXP = 4, FSO_LOG = 5, FSO_TANH = 6, FSO_SIGMOID = 7, FSO_SQRT = 8,
  FSO_RSQRT = 9, FSO_RCP = 10, FSO_GELU_TANH = 11, FSO_CONVERT = 12,
  FSO_ADD = 13, FSO_SUB = 14, FSO_MUL = 15, FSO_DIV = 16, FSO_MAX = 17, FSO_MIN = 18,
  FSO_CMP = 19, FSO_SELECT = 20,
  FSO_BCAST_ROWVEC = 21, FSO_BCAST_COLVEC = 22, FSO_TRANSPOSE = 23,
  FSO_REDUCE_ROW = 24, FSO_REDUCE_COL = 25,
  /* shape modulation beyond transpose (Section 2.1 names Reshape and Bitcast; Section 6.3 Concat).  A tensor of any
   * rank is presented to the plan as [rows, cols] = [product of its leading dims, product of its trailing dims];
   * RESHAPE re-splits the same row-major element sequence: out.flat[i] = in.flat[i].  BITCAST is the same map
   * (in the source framework a Bitcast is a Reshape known not to move data; with dense row-major tensors every
   * Reshape is).  CONCAT joins two tensors along columns (attr_i = 1: out[i, :] = in0[i, :] ++ in1[i, :]) or
   * along rows (attr_i = 0: in0's rows, then in1's). */
  FSO_RESHAPE = 26, FSO_BITCAST = 27, FSO_CONCAT = 28
};
enum { FSO_GT = 0, FSO_GE = 1, FSO_LT = 2, FSO_LE = 3, FSO_EQ = 4, FSO_NE = 5 };
enum { FSO_SUM = 0, FSO_MAX_ = 1, FSO_MIN_ = 2, FSO_MEAN = 3 };

typedef struct {
  int32_t opcode, dtype, rows, cols, num_in, in[3], attr_i;
  float attr_f;
} fso_node;

typedef struct {
  int32_t num_nodes;
  const fso_node* nodes;   /* topological: every operand id < node id */
  int32_t num_outputs;
  const int32_t* outputs;
} fso_graph;

/*
 * Evaluate the DAG on host buffers.
 *   host_in[k]   the k-th FSO_INPUT node's tensor in its dtype (f32 / bf16 bits as uint16 / u8)
 *   host_out[k]  buffer for outputs[k] in that node's dtype
 *   num_threads  OpenMP threads for the independent outer loop of each op (>= 1)
 *   round_nodes  1: every node is rounded to its declared dtype before any consumer
 *                   reads it (the reference of record);
 *                0: nodes stay in fp64, rounding only at plan outputs (a companion
 *                   used to flag ill-conditioned elements, never the pass/fail reference);
 *                2: as 1, but every sum (and the sum inside a mean) is displaced by
 *                   2^-24 * sum |terms|: one fp32 rounding unit per term, the first-order
 *                   size of what accumulating in fp32 can do to a sum in ANY order.  The path
 *                   under test accumulates in fp32, in a tree order of its own; this second
 *                   companion shows, element by element, how far that choice can move an
 *                   output (a sum of positive terms hardly moves; a sum whose terms cancel
 *                   moves by many times its own size).  Never the pass/fail reference either.
 *                3: no values at all: host_out[k] receives, as DOUBLES (rows*cols of them, whatever the
 *                   output's dtype), the first-order spread (standard deviation) of a correct fp32
 *                   implementation's result around the reference, element by element.  Model: a correctly
 *                   rounded fp32 op errs uniformly within half a spacing (spread spacing/sqrt(12), the
 *                   spacing taken as 2^-23 |result|); exp, log, tanh, sigmoid, rsqrt, rcp and gelu, which
 *                   a GPU builds on hardware approximations good to 1-2 spacings, have a spread of one
 *                   spacing; a sum accumulated in fp32 rounds every partial sum of a balanced pairwise
 *                   summation.  Rounding errors are independent, travel through each op's derivative and
 *                   add in quadrature; the errors of approximated ops may lean one way over many elements
 *                   (an approximation is a fixed function, not noise), so they travel through the
 *                   derivatives' absolute values and add linearly; an element's spread is the sum of the
 *                   two parts.  Inputs, constants, predicates and bf16 roundings are exact.  Where
 *                   companions 0 and 2 each show ONE realisation of rounding noise (which can be small at
 *                   an element by chance), this one gives its scale.  Never the pass/fail reference.
 * Returns 0, or a negative code: -1 bad argument, -2 bad graph, -3 out of memory.
 */
int fso_run(const fso_graph* g, const void* const* host_in, void* const* host_out, int num_threads, int round_nodes);

/* The two roundings, exported so tests can pin them on their own. */
double fso_round_f32(double x);
double fso_round_bf16(double x);

#ifdef __cplusplus
}
#endif
#endif
