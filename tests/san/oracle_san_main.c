/* Runs the CPU oracle on plans read from files, under AddressSanitizer / UndefinedBehaviorSanitizer.
 * Inputs are filled with a fixed pattern; all three evaluation modes are run; a checksum is printed. */
#include <stdint.h>
#include <string.h>

#include "../../oracle/fso.h"
#include "plan_file.h"

int main(int argc, char** argv) {
  double checksum = 0.0;
  for (int a = 1; a < argc; ++a) {
    pf_node* pn; int N, K; int* outs;
    if (pf_read(argv[a], &pn, &N, &outs, &K) != 0) { fprintf(stderr, "cannot read %s\n", argv[a]); return 2; }
    fso_node* nodes = (fso_node*)calloc((size_t)N, sizeof(fso_node));
    int n_in = 0;
    for (int i = 0; i < N; ++i) {
      nodes[i].opcode = pn[i].opcode; nodes[i].dtype = pn[i].dtype; nodes[i].rows = pn[i].rows; nodes[i].cols = pn[i].cols;
      nodes[i].num_in = pn[i].num_in; memcpy(nodes[i].in, pn[i].in, sizeof(pn[i].in)); nodes[i].attr_i = pn[i].attr_i; nodes[i].attr_f = pn[i].attr_f;
      n_in += pn[i].opcode == FSO_INPUT;
    }
    void** in = (void**)calloc((size_t)(n_in ? n_in : 1), sizeof(void*));
    void** out = (void**)calloc((size_t)K, sizeof(void*));
    int k = 0;
    for (int i = 0; i < N; ++i) {
      if (pn[i].opcode != FSO_INPUT) continue;
      const long E = (long)pn[i].rows * pn[i].cols;
      if (pn[i].dtype == FSO_F32) { float* p = (float*)malloc(4 * (size_t)E); for (long e = 0; e < E; ++e) p[e] = (float)((e * 37 + i * 11) % 201 - 100) / 64.0f; in[k] = p; }
      else if (pn[i].dtype == FSO_BF16) { uint16_t* p = (uint16_t*)malloc(2 * (size_t)E); for (long e = 0; e < E; ++e) p[e] = (uint16_t)(0x3F00 + (e * 13 + i) % 256 + ((e & 1) ? 0x8000 : 0)); in[k] = p; }
      else { uint8_t* p = (uint8_t*)malloc((size_t)E); for (long e = 0; e < E; ++e) p[e] = (uint8_t)((e + i) % 3 == 0); in[k] = p; }
      ++k;
    }
    fso_graph g = {N, nodes, K, outs};
    for (int mode = 0; mode <= 3; ++mode) {  /* the reference, its fp64 and accumulation companions, the spread */
      for (int o = 0; o < K; ++o) {
        const pf_node* n = &pn[outs[o]];
        const size_t es = mode == 3 ? 8 : n->dtype == FSO_F32 ? 4 : n->dtype == FSO_BF16 ? 2 : 1;   /* the spread comes back as doubles */
        out[o] = malloc(es * (size_t)n->rows * n->cols);   /* exact size: an overrun is caught */
      }
      const int rc = fso_run(&g, (const void* const*)in, out, mode == 1 ? 3 : 1, mode);
      if (rc != 0) { fprintf(stderr, "%s: fso_run mode %d returned %d\n", argv[a], mode, rc); return 3; }
      for (int o = 0; o < K; ++o) {
        const pf_node* n = &pn[outs[o]];
        if (mode != 3 && n->dtype == FSO_F32) checksum += ((float*)out[o])[(size_t)n->rows * n->cols - 1];
        free(out[o]);
      }
    }
    for (int i = 0; i < n_in; ++i) free(in[i]);
    free(in); free(out); free(nodes); free(pn); free(outs);
  }
  printf("oracle ok %.6g\n", checksum);
  return 0;
}
