/* A fusion plan as a flat text file, written by tests/test_sanitizers.py and read by the two sanitizer drivers:
 *   line 1:  num_nodes num_outputs
 *   then one line per node:  opcode dtype rows cols num_in in0 in1 in2 attr_i attr_f
 *   last line: the output node ids
 * Enum values are the ones of the library under test (the test writes one file per library). */
#ifndef PLAN_FILE_H_
#define PLAN_FILE_H_
#include <stdio.h>
#include <stdlib.h>

typedef struct { int opcode, dtype, rows, cols, num_in, in[3], attr_i; float attr_f; } pf_node;

static int pf_read(const char* path, pf_node** nodes, int* num_nodes, int** outputs, int* num_outputs) {
  FILE* f = fopen(path, "r");
  if (!f) return -1;
  if (fscanf(f, "%d %d", num_nodes, num_outputs) != 2 || *num_nodes <= 0 || *num_outputs <= 0) { fclose(f); return -2; }
  *nodes = (pf_node*)calloc((size_t)*num_nodes, sizeof(pf_node));
  *outputs = (int*)calloc((size_t)*num_outputs, sizeof(int));
  for (int i = 0; i < *num_nodes; ++i) {
    pf_node* n = &(*nodes)[i];
    if (fscanf(f, "%d %d %d %d %d %d %d %d %d %f", &n->opcode, &n->dtype, &n->rows, &n->cols, &n->num_in, &n->in[0], &n->in[1], &n->in[2],
               &n->attr_i, &n->attr_f) != 10) { fclose(f); return -3; }
  }
  for (int k = 0; k < *num_outputs; ++k)
    if (fscanf(f, "%d", &(*outputs)[k]) != 1) { fclose(f); return -4; }
  fclose(f);
  return 0;
}
#endif
