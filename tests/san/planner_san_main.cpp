// Runs the host side of the library - plan ingestion, grouping, schedule and LDS planning, code generation - on
// plans read from files, under AddressSanitizer / UndefinedBehaviorSanitizer.  The device and the run-time compiler
// are stubbed: nothing here needs HIP.
#include <cstring>
#include <string>
#include <vector>

#include "fs_internal.h"
extern "C" {
#include "plan_file.h"
}

namespace fs {
const DeviceLimits& device_limits() {
  static DeviceLimits lim;
  return lim;
}
const char* device_header_source() { return ""; }
}  // namespace fs

static int plan_once(const char* path, uint32_t mode, int lds_budget, const fs_sched_hint* hint) {
  pf_node* pn; int N, K; int* outs;
  if (pf_read(path, &pn, &N, &outs, &K) != 0) { fprintf(stderr, "cannot read %s\n", path); return -1; }
  std::vector<fs_node> nodes((size_t)N);
  for (int i = 0; i < N; ++i) {
    nodes[i].opcode = pn[i].opcode; nodes[i].dtype = pn[i].dtype; nodes[i].rows = pn[i].rows; nodes[i].cols = pn[i].cols;
    nodes[i].num_in = pn[i].num_in; memcpy(nodes[i].in, pn[i].in, sizeof(pn[i].in)); nodes[i].attr_i = pn[i].attr_i; nodes[i].attr_f = pn[i].attr_f;
  }
  fs_graph_desc desc = {};
  desc.abi_version = FS_ABI_VERSION; desc.num_nodes = N; desc.nodes = nodes.data(); desc.num_outputs = K; desc.outputs = outs;
  desc.mode = mode; desc.lds_budget_bytes = lds_budget; desc.hint = hint;
  fs::Graph g;
  fs_status st = fs::build_graph(&desc, &g);
  size_t text = 0;
  int groups = -1;
  if (st == FS_OK) {
    fs::PlanOptions opt;
    opt.mode = mode & FS_MODE_UNFUSED; opt.layered = (mode & FS_MODE_LAYERED) != 0;
    opt.lds_budget = lds_budget > 0 ? lds_budget : 65536; opt.lds_budget_given = lds_budget > 0;
    if (hint) opt.hint = *hint, opt.has_hint = true;
    std::vector<int> group_of;
    std::vector<std::vector<int>> ordered;
    st = fs::form_groups(g, &desc, opt, &group_of, &ordered);
    if (st == FS_OK) {
      groups = (int)ordered.size();
      for (size_t gi = 0; gi < ordered.size(); ++gi)
        for (int m : ordered[gi]) group_of[m] = (int)gi;
      for (size_t gi = 0; gi < ordered.size() && st == FS_OK; ++gi) {
        fs::GroupPlan gp;
        st = fs::analyse_group(g, ordered[gi], group_of, (int)gi, opt, &gp);
        if (st == FS_OK) st = fs::generate_kernel(g, &gp, (int)gi);
        text += gp.source.size();
      }
    }
  }
  printf("%s mode %u budget %d: status %d, %d groups, %zu bytes of kernel text\n", path, mode, lds_budget, (int)st, groups, text);
  free(pn); free(outs);
  return (int)st;
}

int main(int argc, char** argv) {
  int worst = 0;
  const fs_sched_hint one_block = {0, 0, 1, 0};
  for (int a = 1; a < argc; ++a) {
    for (uint32_t mode : {FS_MODE_STITCHED, FS_MODE_UNFUSED, FS_MODE_LAYERED}) {
      const int st = plan_once(argv[a], mode, 0, nullptr);
      if (st != FS_OK && st != FS_ERR_UNSUPPORTED && st != FS_ERR_LDS_BUDGET) worst = 1;
    }
    plan_once(argv[a], FS_MODE_STITCHED, 256, nullptr);      // a tiny budget: the refusal paths
    plan_once(argv[a], FS_MODE_STITCHED, 0, &one_block);      // the single-block schedule
  }
  return worst;
}
