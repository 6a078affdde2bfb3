// fs_runtime.cpp - the C ABI: plan creation (group, schedule, generate, compile), launches,
// introspection.  Kernels are compiled at plan creation with the HIP run-time compiler for
// gfx950 only; compilation needs no GPU, loading and launching do.
#include <dlfcn.h>
#include <hip/hip_runtime_api.h>
#include <hip/hiprtc.h>
#include <sys/stat.h>
#include <unistd.h>

#include <algorithm>
#include <cstdlib>
#include <cstring>
#include <fstream>
#include <set>

#include "fs_internal.h"

namespace fs {
int launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream);
int launch_zero_u32(void* p, size_t count, hipStream_t stream);
int launch_copy_probe_shape(const void* src, void* dst, size_t bytes, int vectors_in_flight, int workgroups, hipStream_t stream);
int launch_empty(hipStream_t stream);
int launch_alu_probe(float* out, int workgroups, int iters, hipStream_t stream);
size_t static_scratch_bytes();
int static_scratch_resolve(int device, void** out);
void* static_scratch_lookup(int device);

namespace {

uint64_t fnv1a(const std::string& s, uint64_t h = 1469598103934665603ull) {
  for (unsigned char c : s) {
    h ^= c;
    h *= 1099511628211ull;
  }
  return h;
}

std::string cache_dir() {
  if (const char* e = getenv("FS_KERNEL_CACHE")) return e;
  Dl_info info;
  if (dladdr((void*)&cache_dir, &info) && info.dli_fname) {
    std::string p = info.dli_fname;
    const size_t slash = p.rfind('/');
    if (slash != std::string::npos) return p.substr(0, slash) + "/kcache";
  }
  return "";
}

const char* kCompileOptions[] = {"--offload-arch=gfx950", "-O3",      "-std=c++17",     "-ffp-contract=off",
                                 "-Xclang",               "-target-feature", "-Xclang", "-packed-fp32-ops"};
constexpr int kNumCompileOptions = 8;

bool read_file(const std::string& path, std::vector<char>* out) {
  std::ifstream f(path, std::ios::binary);
  if (!f) return false;
  f.seekg(0, std::ios::end);
  const std::streamoff n = f.tellg();
  if (n <= 0) return false;
  out->resize((size_t)n);
  f.seekg(0);
  f.read(out->data(), n);
  return (bool)f;
}

void write_file_atomic(const std::string& path, const std::vector<char>& data) {
  const std::string tmp = path + ".tmp" + std::to_string((long)getpid());
  {
    std::ofstream f(tmp, std::ios::binary);
    if (!f) return;
    f.write(data.data(), (std::streamsize)data.size());
    if (!f) {
      unlink(tmp.c_str());
      return;
    }
  }
  if (rename(tmp.c_str(), path.c_str()) != 0) unlink(tmp.c_str());
}

}  // namespace

const DeviceLimits& device_limits() {
  static DeviceLimits lim;
  static std::once_flag once;
  std::call_once(once, [] {
    int count = 0, dev = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || count <= 0 || hipGetDevice(&dev) != hipSuccess) {
      (void)hipGetLastError();  // no device: not an error of any later call
      return;
    }
    int cus = 0, lds = 0, lanes_per_cu = 0, l2 = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return;
    if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess || lds <= 0) return;
    if (hipDeviceGetAttribute(&lanes_per_cu, hipDeviceAttributeMaxThreadsPerMultiProcessor, dev) != hipSuccess || lanes_per_cu <= 0) return;
    if (hipDeviceGetAttribute(&l2, hipDeviceAttributeL2CacheSize, dev) != hipSuccess || l2 <= 0) l2 = 4 << 20;
    lim.cus = cus;
    lim.lds_per_workgroup = lds;
    lim.resident_lanes = (int64_t)cus * lanes_per_cu;
    lim.l2_bytes = l2;
    lim.from_device = true;
  });
  return lim;
}

fs_status compile_kernel(const std::string& source, const std::string& name, std::vector<char>* code) {
  std::string key_text = source;
  for (int i = 0; i < kNumCompileOptions; ++i) key_text += kCompileOptions[i];
  int rtc_major = 0, rtc_minor = 0;
  hiprtcVersion(&rtc_major, &rtc_minor);
  key_text += std::to_string(rtc_major) + "." + std::to_string(rtc_minor);
  char key[40];
  snprintf(key, sizeof(key), "%016llx%016llx", (unsigned long long)fnv1a(key_text),
           (unsigned long long)fnv1a(key_text, 0x9e3779b97f4a7c15ull));
  const std::string dir = cache_dir();
  const std::string path = dir.empty() ? "" : dir + "/" + key + ".hsaco";
  if (!path.empty() && read_file(path, code)) return FS_OK;

  hiprtcProgram prog;
  if (hiprtcCreateProgram(&prog, source.c_str(), (name + ".hip").c_str(), 0, nullptr, nullptr) != HIPRTC_SUCCESS)
    FS_FAIL(FS_ERR_COMPILE, "hiprtcCreateProgram failed");
  const hiprtcResult rc = hiprtcCompileProgram(prog, kNumCompileOptions, kCompileOptions);
  if (rc != HIPRTC_SUCCESS) {
    size_t n = 0;
    hiprtcGetProgramLogSize(prog, &n);
    std::string log(n, '\0');
    if (n) hiprtcGetProgramLog(prog, &log[0]);
    hiprtcDestroyProgram(&prog);
    if (const char* dump = getenv("FS_DUMP_FAILED_SOURCE")) {
      std::ofstream f(dump);
      f << source;
    }
    FS_FAIL(FS_ERR_COMPILE, "kernel compilation failed: %s\n%.800s", hiprtcGetErrorString(rc), log.c_str());
  }
  size_t n = 0;
  hiprtcGetCodeSize(prog, &n);
  code->resize(n);
  hiprtcGetCode(prog, code->data());
  hiprtcDestroyProgram(&prog);
  if (!path.empty()) {
    mkdir(dir.c_str(), 0755);
    write_file_atomic(path, *code);
  }
  return FS_OK;
}

// One integer field of every kernel of a code object (".private_segment_fixed_size": scratch, i.e. register spill,
// bytes; ".vgpr_count": vector registers), read from the code object's metadata: the ELF note named "AMDGPU" of type
// 32 holds a msgpack map whose "amdhsa.kernels" entry is an array of one map per kernel (".name", then the fields).
// A small msgpack reader walks it; anything malformed ends the walk and yields an empty result.
namespace {
struct MsgPack {
  const unsigned char* p;
  const unsigned char* end;
  bool ok = true;
  bool need(size_t n) {
    if ((size_t)(end - p) < n) ok = false;
    return ok;
  }
  uint64_t be(int n) {
    uint64_t v = 0;
    if (!need((size_t)n)) return 0;
    for (int i = 0; i < n; ++i) v = (v << 8) | *p++;
    return v;
  }
  // reads one value; strings and integers are reported, containers report their element count
  enum Type { NIL, BOOL, INT, STR, ARRAY, MAP, OTHER };
  Type next(std::string* str, int64_t* num, uint32_t* count) {
    if (!need(1)) return OTHER;
    const unsigned char b = *p++;
    auto take_str = [&](uint64_t n) {
      if (!need((size_t)n)) return OTHER;
      if (str) str->assign((const char*)p, (size_t)n);
      p += n;
      return STR;
    };
    auto skip = [&](uint64_t n) {
      if (need((size_t)n)) p += n;
      return OTHER;
    };
    if (b <= 0x7f) { if (num) *num = b; return INT; }
    if (b >= 0xe0) { if (num) *num = (int8_t)b; return INT; }
    if ((b & 0xe0) == 0xa0) return take_str(b & 0x1f);
    if ((b & 0xf0) == 0x90) { if (count) *count = b & 0x0f; return ARRAY; }
    if ((b & 0xf0) == 0x80) { if (count) *count = b & 0x0f; return MAP; }
    switch (b) {
      case 0xc0: return NIL;
      case 0xc2: case 0xc3: if (num) *num = b == 0xc3; return BOOL;
      case 0xc4: return skip(be(1));
      case 0xc5: return skip(be(2));
      case 0xc6: return skip(be(4));
      case 0xca: return skip(4);
      case 0xcb: return skip(8);
      case 0xcc: if (num) *num = (int64_t)be(1); else be(1); return INT;
      case 0xcd: if (num) *num = (int64_t)be(2); else be(2); return INT;
      case 0xce: if (num) *num = (int64_t)be(4); else be(4); return INT;
      case 0xcf: if (num) *num = (int64_t)be(8); else be(8); return INT;
      case 0xd0: { const int64_t v = (int8_t)be(1); if (num) *num = v; return INT; }
      case 0xd1: { const int64_t v = (int16_t)be(2); if (num) *num = v; return INT; }
      case 0xd2: { const int64_t v = (int32_t)be(4); if (num) *num = v; return INT; }
      case 0xd3: { const int64_t v = (int64_t)be(8); if (num) *num = v; return INT; }
      case 0xd9: return take_str(be(1));
      case 0xda: return take_str(be(2));
      case 0xdb: return take_str(be(4));
      case 0xdc: if (count) *count = (uint32_t)be(2); else be(2); return ARRAY;
      case 0xdd: if (count) *count = (uint32_t)be(4); else be(4); return ARRAY;
      case 0xde: if (count) *count = (uint32_t)be(2); else be(2); return MAP;
      case 0xdf: if (count) *count = (uint32_t)be(4); else be(4); return MAP;
    }
    ok = false;  // extension types do not occur in this metadata
    return OTHER;
  }
  void skip_value(int depth = 0) {
    uint32_t n = 0;
    const Type t = next(nullptr, nullptr, &n);
    if (!ok || depth > 32) { ok = false; return; }
    if (t == ARRAY) for (uint32_t i = 0; i < n && ok; ++i) skip_value(depth + 1);
    if (t == MAP) for (uint32_t i = 0; i < 2 * n && ok; ++i) skip_value(depth + 1);
  }
};

// the msgpack metadata of an AMDGPU code object (ELF64, little endian), or an empty range
bool amdgpu_metadata(const std::vector<char>& code, const unsigned char** begin, const unsigned char** end) {
  const unsigned char* d = (const unsigned char*)code.data();
  const size_t n = code.size();
  auto rd = [&](size_t off, int bytes) {
    uint64_t v = 0;
    for (int i = bytes - 1; i >= 0; --i) v = (v << 8) | d[off + i];
    return v;
  };
  if (n < 64 || memcmp(d, "\177ELF", 4) != 0 || d[4] != 2 || d[5] != 1) return false;
  const uint64_t shoff = rd(0x28, 8), shentsize = rd(0x3a, 2), shnum = rd(0x3c, 2);
  if (shentsize < 64 || shoff > n || shnum > (n - shoff) / shentsize) return false;
  for (uint64_t k = 0; k < shnum; ++k) {
    const size_t sh = (size_t)(shoff + k * shentsize);
    if (rd(sh + 4, 4) != 7 /* SHT_NOTE */) continue;
    const uint64_t off = rd(sh + 0x18, 8), size = rd(sh + 0x20, 8);
    if (off > n || size > n - off) continue;
    size_t q = (size_t)off;
    const size_t stop = (size_t)(off + size);
    while (q + 12 <= stop) {
      const uint64_t namesz = rd(q, 4), descsz = rd(q + 4, 4), type = rd(q + 8, 4);
      const size_t name = q + 12, desc = name + (size_t)((namesz + 3) & ~(uint64_t)3);
      if (desc > stop || descsz > stop - desc) break;
      if (type == 32 && namesz == 7 && memcmp(d + name, "AMDGPU", 6) == 0) {
        *begin = d + desc;
        *end = d + desc + descsz;
        return true;
      }
      q = desc + (size_t)((descsz + 3) & ~(uint64_t)3);
    }
  }
  return false;
}
}  // namespace

std::map<std::string, long> code_object_kernel_field(const std::vector<char>& code, const char* key) {
  std::map<std::string, long> out;
  MsgPack m{nullptr, nullptr};
  if (!amdgpu_metadata(code, &m.p, &m.end)) return out;
  uint32_t top = 0;
  if (m.next(nullptr, nullptr, &top) != MsgPack::MAP) return out;
  for (uint32_t e = 0; e < top && m.ok; ++e) {
    std::string k;
    if (m.next(&k, nullptr, nullptr) != MsgPack::STR) return out;
    if (k != "amdhsa.kernels") {
      m.skip_value();
      continue;
    }
    uint32_t kernels = 0;
    if (m.next(nullptr, nullptr, &kernels) != MsgPack::ARRAY) return out;
    for (uint32_t i = 0; i < kernels && m.ok; ++i) {
      uint32_t fields = 0;
      if (m.next(nullptr, nullptr, &fields) != MsgPack::MAP) return out;
      std::string name;
      long value = -1;
      for (uint32_t f = 0; f < fields && m.ok; ++f) {
        std::string fk;
        if (m.next(&fk, nullptr, nullptr) != MsgPack::STR) return out;
        if (fk == ".name") {
          if (m.next(&name, nullptr, nullptr) != MsgPack::STR) return out;
        } else if (fk == key) {
          int64_t v = -1;
          if (m.next(nullptr, &v, nullptr) != MsgPack::INT) return out;
          value = (long)v;
        } else {
          m.skip_value();
        }
      }
      if (m.ok && !name.empty() && value >= 0) out[name] = value;
    }
  }
  return out;
}

}  // namespace fs

using namespace fs;

static size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

extern "C" {

const char* fs_last_error(void) { return error_buffer().c_str(); }

fs_status fs_plan_create(const fs_graph_desc* desc, fs_plan** out_plan) {
  if (!out_plan) FS_FAIL(FS_ERR_INVALID_ARG, "out_plan is NULL");
  *out_plan = nullptr;
  fs_plan* plan = new (std::nothrow) fs_plan();
  if (!plan) FS_FAIL(FS_ERR_OOM, "out of host memory");
  fs_status st = build_graph(desc, &plan->graph);
  if (st != FS_OK) {
    delete plan;
    return st;
  }
  plan->opt.mode = desc->mode & FS_MODE_UNFUSED;
  plan->opt.layered = (desc->mode & FS_MODE_LAYERED) != 0;
  const bool use_library = !(desc->mode & FS_MODE_NO_PERFLIB) && !desc->hint && perflib_size() > 0;
  plan->opt.lds_budget = desc->lds_budget_bytes > 0 ? desc->lds_budget_bytes : std::min(65536, device_limits().lds_per_workgroup);
  plan->opt.lds_budget_given = desc->lds_budget_bytes > 0;
  if (desc->hint) {
    plan->opt.hint = *desc->hint;
    plan->opt.has_hint = true;
    const fs_sched_hint& h = plan->opt.hint;
    if (h.lanes_per_row < 0 || h.wg_threads < 0 || h.max_workgroups < 0 || h.tiles_per_trip < 0) {
      delete plan;
      FS_FAIL(FS_ERR_INVALID_ARG, "negative schedule hint");
    }
  }

  std::vector<std::vector<int>> ordered;
  st = form_groups(plan->graph, desc, plan->opt, &plan->group_of, &ordered);
  if (st != FS_OK) {
    delete plan;
    return st;
  }
  const Graph& g = plan->graph;
  plan->groups.resize(ordered.size());
  // group ids follow launch order
  for (size_t gi = 0; gi < ordered.size(); ++gi)
    for (int m : ordered[gi]) plan->group_of[m] = (int)gi;
  // the library's own grouping may compute a cheap value in two kernels rather than pass it through memory
  // (a caller's plan and the one-launch-per-op executor are taken as they are)
  if (plan->opt.mode != FS_MODE_UNFUSED && !desc->group_of_node) {
    recompute_across_kernels(g, plan->opt, &plan->group_of, &ordered, &plan->clones);
    plan->opt.clones = &plan->clones;
    plan->groups.resize(ordered.size());
  }
  for (size_t gi = 0; gi < ordered.size(); ++gi) {
    st = analyse_group(g, ordered[gi], plan->group_of, (int)gi, plan->opt, &plan->groups[gi]);
    if (st == FS_OK) st = generate_kernel(g, &plan->groups[gi], (int)gi);
    if (st != FS_OK) {
      delete plan;
      return st;
    }
    // schedule tuning: the fastest candidate the performance library knows (Sections 4.3, 4.4)
    if (use_library) choose_from_library(g, ordered[gi], plan->group_of, (int)gi, plan->opt, &plan->groups[gi]);
  }

  // One translation unit per plan: the building blocks once, then every distinct kernel body.
  // Spill feedback: a kernel whose code object reports scratch memory is planned again with less
  // register pressure -- rows held beyond 32 elements per lane step down towards chunks, otherwise
  // the workgroup is halved (the register file is shared by fewer wavefronts) -- and the unit is
  // compiled again; a few rounds at most.
  // Occupancy feedback: a 1024-lane workgroup is 4 wavefronts per SIMD, so a CU holds two of them
  // only at 64 vector registers or fewer.  A kernel that is up to 16 registers above that is compiled
  // once more with the compiler asked for 8 wavefronts per SIMD, and keeps that form if it then fits
  // without spilling (softmax over 32768 fp32 columns: 67 -> 56 registers, 105.5 -> 94.5 us; a
  // masked softmax of the same shape spills when forced and stays as it was).
  std::vector<PlanOptions> group_opt(plan->groups.size(), plan->opt);
  std::vector<GroupPlan> before_waves(plan->groups.size());  // the plan to return to when forcing the occupancy spills
  std::vector<char> waves_tried(plan->groups.size(), 0);
  for (int round = 0;; ++round) {
    std::string tu = device_header_source();
    std::set<std::string> seen;
    for (const GroupPlan& gp : plan->groups)
      if (seen.insert(gp.kernel_name).second) tu += "\n" + gp.source;
    st = compile_kernel(tu, "fs_plan", &plan->code);
    if (st != FS_OK) {
      delete plan;
      return st;
    }
    const std::map<std::string, long> scratch = code_object_kernel_field(plan->code, ".private_segment_fixed_size");
    const std::map<std::string, long> vgprs = code_object_kernel_field(plan->code, ".vgpr_count");
    bool changed = false;
    for (size_t gi = 0; gi < plan->groups.size(); ++gi) {
      GroupPlan& gp = plan->groups[gi];
      auto it = scratch.find(gp.kernel_name);
      if (gp.s.min_waves > 0) {  // a forced occupancy must come (nearly) for free: at most 8 spilled registers
        if (it != scratch.end() && it->second > 32) {
          if (getenv("FS_LOG_PLAN"))
            fprintf(stderr, "fs: group %zu kernel %s spills %ld bytes at %d wavefronts per SIMD: back to the plain form\n", gi,
                    gp.kernel_name.c_str(), it->second, gp.s.min_waves);
          gp = before_waves[gi];
          group_opt[gi].min_waves = 0;
          changed = true;
        }
        continue;
      }
      if (round >= 4) continue;  // (only returns to the plain form are still taken: the loop ends)
      // (a few spilled registers cost nothing measurable, and whether a borderline kernel gets them varies with what the
      // run-time compiler compiled before in the same process; hundreds of bytes are what ruins a kernel)
      if (it == scratch.end() || it->second <= 128) {
        auto vg = vgprs.find(gp.kernel_name);
        if (!waves_tried[gi] && gp.s.WG == 1024 && vg != vgprs.end() && vg->second > 64 && vg->second <= 80 && (it == scratch.end() || it->second == 0)) {
          waves_tried[gi] = 1;
          PlanOptions o = group_opt[gi];
          o.min_waves = 8;
          GroupPlan again;
          if (analyse_group(g, ordered[gi], plan->group_of, (int)gi, o, &again) == FS_OK && generate_kernel(g, &again, (int)gi) == FS_OK &&
              again.kernel_name != gp.kernel_name) {
            if (getenv("FS_LOG_PLAN"))
              fprintf(stderr, "fs: group %zu kernel %s uses %ld registers with 1024-lane workgroups: trying 8 wavefronts per SIMD\n", gi,
                      gp.kernel_name.c_str(), vg->second);
            before_waves[gi] = gp;
            group_opt[gi] = o;
            gp = again;
            changed = true;
          }
        }
        continue;
      }
      // the next milder plan that actually differs from the current one
      PlanOptions o = group_opt[gi];
      GroupPlan again;
      bool found = false;
      while (!found && !gp.row_reduces.empty() && (gp.s.E >= 32 || gp.s.resident) && o.wide_level > 0) {
        --o.wide_level;
        found = analyse_group(g, ordered[gi], plan->group_of, (int)gi, o, &again) == FS_OK &&
                generate_kernel(g, &again, (int)gi) == FS_OK && again.kernel_name != gp.kernel_name;
      }
      if (!found && gp.s.WG >= 2 * std::max(64, gp.s.L) && !gp.s.chunked && !gp.s.tiled_transpose) {
        o = group_opt[gi];
        if (!o.has_hint) o.hint = fs_sched_hint{0, 0, 0, 0};
        o.has_hint = true;
        o.hint.wg_threads = gp.s.WG / 2;
        found = analyse_group(g, ordered[gi], plan->group_of, (int)gi, o, &again) == FS_OK &&
                generate_kernel(g, &again, (int)gi) == FS_OK && again.kernel_name != gp.kernel_name;
      }
      if (getenv("FS_LOG_PLAN"))
        fprintf(stderr, "fs: group %zu kernel %s spills %ld bytes (%d lanes/row, %d elements/lane, workgroup %d): %s\n", gi, gp.kernel_name.c_str(),
                it->second, gp.s.L, gp.s.E, gp.s.WG, found ? "planned again" : "kept");
      if (!found) continue;
      group_opt[gi] = o;
      gp = again;
      changed = true;
    }
    if (!changed) {
      if (getenv("FS_LOG_PLAN"))
        for (size_t gi = 0; gi < plan->groups.size(); ++gi) {
          const GroupPlan& gp = plan->groups[gi];
          auto vg = vgprs.find(gp.kernel_name);
          auto sc = scratch.find(gp.kernel_name);
          fprintf(stderr, "fs: group %zu kernel %s: %ld vector registers, %ld bytes of scratch, workgroup %d, grid %d\n", gi, gp.kernel_name.c_str(),
                  vg == vgprs.end() ? -1 : vg->second, sc == scratch.end() ? -1 : sc->second, gp.s.WG, gp.s.grid);
        }
      break;
    }
  }

  // workspace: [tickets][tensors crossing group boundaries][column-reduction partials]
  size_t off = 0;
  for (GroupPlan& gp : plan->groups) {
    gp.ticket_offset = off;
    off += (size_t)gp.n_tickets * 4;
  }
  plan->ticket_bytes = align_up(off, 256);
  off = plan->ticket_bytes;
  for (GroupPlan& gp : plan->groups)
    for (const ExtTensor& e : gp.ext_out)
      // (a value a plan output is a view of is written straight into the caller's buffer)
      if (g.family_output[e.node] < 0 && !plan->ws_tensor_offset.count(e.node)) {
        plan->ws_tensor_offset[e.node] = off;
        off = align_up(off + (size_t)g.nodes[e.node].rows * g.nodes[e.node].cols * dtype_size(e.dtype), 256);
      }
  for (GroupPlan& gp : plan->groups)
    if (gp.part_bytes) {
      gp.part_offset = off;
      off = align_up(off + gp.part_bytes, 256);
    }
  plan->workspace_bytes = off;

  plan->min_hbm_bytes = 0;
  for (int id : g.input_ids) {
    bool used = false;  // only inputs some live node reads
    for (const GroupPlan& gp : plan->groups)
      for (const ExtTensor& e : gp.ext_in) used |= g.root_of[e.node] == id;
    if (used) plan->min_hbm_bytes += (uint64_t)g.nodes[id].rows * g.nodes[id].cols * dtype_size(g.nodes[id].dtype);
  }
  for (int o : g.outputs) plan->min_hbm_bytes += (uint64_t)g.nodes[o].rows * g.nodes[o].cols * dtype_size(g.nodes[o].dtype);
  plan->launched_hbm_bytes = 0;
  for (const GroupPlan& gp : plan->groups) plan->launched_hbm_bytes += gp.min_hbm_bytes;
  // what one launch per compute node would move: every live node as a group of its own
  plan->unfused_hbm_bytes = 0;
  if (plan->opt.mode == FS_MODE_UNFUSED) {
    plan->unfused_hbm_bytes = plan->launched_hbm_bytes;
  } else {
    PlanOptions uo;
    uo.mode = FS_MODE_UNFUSED;
    uo.lds_budget = plan->opt.lds_budget;
    GroupPlan single;
    for (int id = 0; id < g.n(); ++id)
      if (plan->group_of[id] >= 0 && analyse_group(g, std::vector<int>{id}, plan->group_of, 0, uo, &single) == FS_OK)
        plan->unfused_hbm_bytes += single.min_hbm_bytes;
  }

  *out_plan = plan;
  return FS_OK;
}

fs_status fs_plan_destroy(fs_plan* plan) {
  if (!plan) return FS_OK;
  for (auto& kv : plan->loaded)
    for (void* m : kv.second.modules)
      if (m) (void)hipModuleUnload((hipModule_t)m);
  delete plan;
  return FS_OK;
}

fs_status fs_plan_workspace_bytes(const fs_plan* plan, size_t* bytes) {
  if (!plan || !bytes) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  *bytes = plan->workspace_bytes;
  return FS_OK;
}

static fs_status load_on_device(fs_plan* plan, int device, fs_plan::Loaded** out) {
  std::lock_guard<std::mutex> lk(plan->mu);
  auto it = plan->loaded.find(device);
  if (it != plan->loaded.end()) {
    *out = &it->second;
    return FS_OK;
  }
  hipModule_t mod;
  hipError_t e = hipModuleLoadData(&mod, plan->code.data());
  if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "hipModuleLoadData: %s", hipGetErrorString(e));
  fs_plan::Loaded ld;
  ld.modules.push_back((void*)mod);
  for (const GroupPlan& gp : plan->groups) {
    hipFunction_t fn;
    e = hipModuleGetFunction(&fn, mod, gp.kernel_name.c_str());
    if (e != hipSuccess) {
      (void)hipModuleUnload(mod);
      FS_FAIL(FS_ERR_HIP, "hipModuleGetFunction(%s): %s", gp.kernel_name.c_str(), hipGetErrorString(e));
    }
    ld.functions.push_back((void*)fn);
  }
  *out = &(plan->loaded[device] = std::move(ld));
  return FS_OK;
}

namespace fs {
// kernarg block: { void* p[NP]; float* part; u32* tickets; int R; int n_iters; }
hipError_t launch_group(const GroupPlan& gp, void* function, void* const* tensors, void* part, void* tickets, hipStream_t stream) {
  alignas(8) char buf[8 * 48 + 32];
  size_t n = 0;
  auto push_ptr = [&](void* p) {
    memcpy(buf + n, &p, 8);
    n += 8;
  };
  const size_t np = gp.ext_in.size() + gp.ext_out.size();
  for (size_t k = 0; k < np; ++k) push_ptr(tensors[k]);
  push_ptr(part);
  push_ptr(tickets);
  const int R = gp.R, iters = gp.s.n_iters;
  memcpy(buf + n, &R, 4);
  memcpy(buf + n + 4, &iters, 4);
  n += 8;
  size_t size = n;
  void* config[] = {HIP_LAUNCH_PARAM_BUFFER_POINTER, buf, HIP_LAUNCH_PARAM_BUFFER_SIZE, &size, HIP_LAUNCH_PARAM_END};
  return hipModuleLaunchKernel((hipFunction_t)function, (unsigned)gp.s.grid, 1, 1, (unsigned)gp.s.WG, 1, 1, 0, stream, nullptr, config);
}
}  // namespace fs

static fs_status check_workspace(const fs_plan* plan, const void* workspace, size_t workspace_bytes) {
  if (plan->workspace_bytes == 0) return FS_OK;
  if (!workspace) FS_FAIL(FS_ERR_WORKSPACE, "workspace is NULL but the plan needs %zu bytes", plan->workspace_bytes);
  if (workspace_bytes < plan->workspace_bytes)
    FS_FAIL(FS_ERR_WORKSPACE, "workspace has %zu bytes, the plan needs %zu", workspace_bytes, plan->workspace_bytes);
  if (((uintptr_t)workspace & 255) != 0) FS_FAIL(FS_ERR_WORKSPACE, "workspace is not 256-byte aligned");
  return FS_OK;
}

fs_status fs_plan_workspace_init(fs_plan* plan, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!plan) FS_FAIL(FS_ERR_INVALID_ARG, "plan is NULL");
  fs_status st = check_workspace(plan, workspace, workspace_bytes);
  if (st != FS_OK) return st;
  if (plan->ticket_bytes == 0) return FS_OK;
  const int e = launch_zero_u32(workspace, plan->ticket_bytes / 4, (hipStream_t)hip_stream);
  if (e != 0) FS_FAIL(FS_ERR_HIP, "fill kernel launch: %s", hipGetErrorString((hipError_t)e));
  return FS_OK;
}

// One launch per group, in launch order, on `stream`; `workspace` holds tickets, boundary tensors and partials.
static fs_status enqueue_groups(const fs_plan* plan, const fs_plan::Loaded* ld, const void* const* inputs, void* const* outputs,
                                void* workspace, hipStream_t stream) {
  const Graph& g = plan->graph;
  char* ws = (char*)workspace;
  auto tensor_ptr = [&](int node) -> void* {  // a view addresses the buffer of the value it is a view of
    const int root = g.root_of[node];
    if (g.input_index[root] >= 0) return const_cast<void*>(inputs[g.input_index[root]]);
    if (g.family_output[root] >= 0) return outputs[g.family_output[root]];
    return ws + plan->ws_tensor_offset.at(root);
  };
  for (size_t gi = 0; gi < plan->groups.size(); ++gi) {
    const GroupPlan& gp = plan->groups[gi];
    void* tensors[48];
    size_t n = 0;
    for (const ExtTensor& t : gp.ext_in) tensors[n++] = tensor_ptr(t.node);
    for (const ExtTensor& t : gp.ext_out) tensors[n++] = tensor_ptr(t.node);
    const hipError_t e = launch_group(gp, ld->functions[gi], tensors, gp.part_bytes ? (void*)(ws + gp.part_offset) : nullptr,
                                      gp.n_tickets ? (void*)(ws + gp.ticket_offset) : nullptr, stream);
    if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "launch of group %zu (%s): %s", gi, gp.kernel_name.c_str(), hipGetErrorString(e));
  }
  return FS_OK;
}

// Pointer checks shared by fs_plan_run and fs_plan_tune: NULL, alignment, and byte ranges that
// overlap where one of the two is written (outputs against inputs, other outputs and the workspace;
// inputs against the workspace).  Inputs may alias each other: they are only read.
static fs_status check_buffers(const fs_plan* plan, const void* const* inputs, void* const* outputs, const void* workspace) {
  if (!outputs) FS_FAIL(FS_ERR_INVALID_ARG, "outputs is NULL");
  const Graph& g = plan->graph;
  if (!g.input_ids.empty() && !inputs) FS_FAIL(FS_ERR_INVALID_ARG, "inputs is NULL");
  for (size_t k = 0; k < g.input_ids.size(); ++k)
    if (!inputs[k] || ((uintptr_t)inputs[k] & 15)) FS_FAIL(FS_ERR_INVALID_ARG, "inputs[%zu] is NULL or not 16-byte aligned", k);
  for (size_t k = 0; k < g.outputs.size(); ++k)
    if (!outputs[k] || ((uintptr_t)outputs[k] & 15)) FS_FAIL(FS_ERR_INVALID_ARG, "outputs[%zu] is NULL or not 16-byte aligned", k);
  auto bytes_of = [&](int node) { return (uintptr_t)g.nodes[node].rows * (uintptr_t)g.nodes[node].cols * (uintptr_t)dtype_size(g.nodes[node].dtype); };
  auto overlap = [](uintptr_t a, uintptr_t an, uintptr_t b, uintptr_t bn) { return a < b + bn && b < a + an; };
  const uintptr_t ws = (uintptr_t)workspace, wsn = workspace ? plan->workspace_bytes : 0;
  for (size_t k = 0; k < g.outputs.size(); ++k) {
    const uintptr_t o = (uintptr_t)outputs[k], on = bytes_of(g.outputs[k]);
    for (size_t j = 0; j < g.input_ids.size(); ++j)
      if (overlap(o, on, (uintptr_t)inputs[j], bytes_of(g.input_ids[j]))) FS_FAIL(FS_ERR_INVALID_ARG, "outputs[%zu] overlaps inputs[%zu]", k, j);
    for (size_t j = 0; j < k; ++j)
      if (overlap(o, on, (uintptr_t)outputs[j], bytes_of(g.outputs[j]))) FS_FAIL(FS_ERR_INVALID_ARG, "outputs[%zu] overlaps outputs[%zu]", k, j);
    if (wsn && overlap(o, on, ws, wsn)) FS_FAIL(FS_ERR_INVALID_ARG, "outputs[%zu] overlaps the workspace", k);
  }
  for (size_t j = 0; j < g.input_ids.size(); ++j)
    if (wsn && overlap((uintptr_t)inputs[j], bytes_of(g.input_ids[j]), ws, wsn)) FS_FAIL(FS_ERR_INVALID_ARG, "inputs[%zu] overlaps the workspace", j);
  return FS_OK;
}

fs_status fs_plan_load(fs_plan* plan) {
  if (!plan) FS_FAIL(FS_ERR_INVALID_ARG, "plan is NULL");
  int device = 0;
  const hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  // (set-up of the allocation-free entry point: this device's address of the static scratch array)
  const int se = static_scratch_resolve(device, nullptr);
  if (se != 0) FS_FAIL(FS_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString((hipError_t)se));
  fs_plan::Loaded* ld = nullptr;
  return load_on_device(plan, device, &ld);
}

fs_status fs_plan_workspace_check(fs_plan* plan, const void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!plan) FS_FAIL(FS_ERR_INVALID_ARG, "plan is NULL");
  fs_status st = check_workspace(plan, workspace, workspace_bytes);
  if (st != FS_OK) return st;
  size_t n = 0;
  for (const GroupPlan& gp : plan->groups) n += (size_t)gp.n_tickets;
  if (n == 0) return FS_OK;
  hipError_t e = hipStreamSynchronize((hipStream_t)hip_stream);
  if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "hipStreamSynchronize: %s", hipGetErrorString(e));
  std::vector<uint32_t> host(n);
  e = hipMemcpy(host.data(), workspace, n * 4, hipMemcpyDeviceToHost);
  if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "hipMemcpy: %s", hipGetErrorString(e));
  for (size_t i = 0; i < n; ++i)
    if (host[i] != 0u)
      FS_FAIL(FS_ERR_WORKSPACE, "ticket %zu of %zu holds %u, not 0: the workspace was never initialised, or a run on it did not finish", i, n, host[i]);
  return FS_OK;
}

fs_status fs_plan_run(fs_plan* plan, const void* const* inputs, void* const* outputs, void* workspace,
                      size_t workspace_bytes, void* hip_stream) {
  if (!plan) FS_FAIL(FS_ERR_INVALID_ARG, "plan is NULL");
  fs_status st = check_workspace(plan, workspace, workspace_bytes);
  if (st != FS_OK) return st;
  st = check_buffers(plan, inputs, outputs, workspace);
  if (st != FS_OK) return st;

  int device = 0;
  const hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  fs_plan::Loaded* ld = nullptr;
  st = load_on_device(plan, device, &ld);
  if (st != FS_OK) return st;
  return enqueue_groups(plan, ld, inputs, outputs, workspace, (hipStream_t)hip_stream);
}

fs_status fs_plan_run_static(fs_plan* plan, const void* const* inputs, void* const* outputs, void* hip_stream) {
  if (!plan) FS_FAIL(FS_ERR_INVALID_ARG, "plan is NULL");
  if (plan->workspace_bytes > static_scratch_bytes())
    FS_FAIL(FS_ERR_WORKSPACE, "the plan needs %zu bytes of workspace, the static scratch holds %zu: use fs_plan_run with a workspace of your own",
            plan->workspace_bytes, static_scratch_bytes());
  int device = 0;
  const hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  // look-ups only: loading a code object or resolving the symbol would allocate
  fs_plan::Loaded* ld = nullptr;
  {
    std::lock_guard<std::mutex> lk(plan->mu);
    auto it = plan->loaded.find(device);
    if (it != plan->loaded.end()) ld = &it->second;
  }
  void* ws = static_scratch_lookup(device);
  if (!ld || !ws) FS_FAIL(FS_ERR_INVALID_ARG, "the plan is not loaded on device %d: call fs_plan_load first (this entry point allocates nothing)", device);
  const fs_status st = check_buffers(plan, inputs, outputs, plan->workspace_bytes ? ws : nullptr);
  if (st != FS_OK) return st;
  // the array keeps what the previous call (of any plan) left: this plan's tickets must start at zero
  if (plan->ticket_bytes) {
    const int ze = launch_zero_u32(ws, plan->ticket_bytes / 4, (hipStream_t)hip_stream);
    if (ze != 0) FS_FAIL(FS_ERR_HIP, "fill kernel launch: %s", hipGetErrorString((hipError_t)ze));
  }
  return enqueue_groups(plan, ld, inputs, outputs, ws, (hipStream_t)hip_stream);
}

fs_status fs_plan_stats(const fs_plan* plan, int32_t* num_groups, int32_t* num_launches, uint64_t* min_hbm_bytes,
                        uint64_t* unfused_hbm_bytes) {
  if (!plan) FS_FAIL(FS_ERR_INVALID_ARG, "plan is NULL");
  if (num_groups) *num_groups = (int32_t)plan->groups.size();
  if (num_launches) *num_launches = (int32_t)plan->groups.size();
  if (min_hbm_bytes) *min_hbm_bytes = plan->min_hbm_bytes;
  if (unfused_hbm_bytes) *unfused_hbm_bytes = plan->unfused_hbm_bytes;
  return FS_OK;
}

fs_status fs_plan_launched_hbm_bytes(const fs_plan* plan, uint64_t* bytes) {
  if (!plan || !bytes) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  *bytes = plan->launched_hbm_bytes;
  return FS_OK;
}

fs_status fs_device_limits(int32_t* compute_units, int32_t* lds_bytes_per_workgroup, int32_t* resident_lanes, int64_t* l2_bytes,
                           int32_t* from_device) {
  const DeviceLimits& lim = device_limits();
  if (compute_units) *compute_units = lim.cus;
  if (lds_bytes_per_workgroup) *lds_bytes_per_workgroup = lim.lds_per_workgroup;
  if (resident_lanes) *resident_lanes = (int32_t)lim.resident_lanes;
  if (l2_bytes) *l2_bytes = lim.l2_bytes;
  if (from_device) *from_device = lim.from_device ? 1 : 0;
  return FS_OK;
}

fs_status fs_plan_group_info(const fs_plan* plan, int32_t group, fs_group_info* o) {
  if (!plan || !o) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  if (group < 0 || group >= (int)plan->groups.size()) FS_FAIL(FS_ERR_INVALID_ARG, "group %d out of range", group);
  const GroupPlan& gp = plan->groups[group];
  o->num_nodes = (int32_t)gp.members.size();
  o->dom_rows = gp.R;
  o->dom_cols = gp.C;
  o->lanes_per_row = gp.s.L;
  o->vec_elems = gp.s.V;
  o->elems_per_lane = gp.s.E;
  o->wg_threads = gp.s.WG;
  o->rows_per_iter = gp.s.G;
  o->grid = gp.s.grid;
  o->lds_bytes = gp.s.lds_bytes;
  o->num_row_reduces = (int32_t)gp.row_reduces.size();
  o->num_col_reduces = (int32_t)gp.col_reduces.size();
  o->num_ext_inputs = (int32_t)gp.ext_in.size();
  o->num_ext_outputs = (int32_t)gp.ext_out.size();
  o->min_hbm_bytes = gp.min_hbm_bytes;
  o->scratch_bytes = gp.part_bytes + (uint64_t)gp.n_tickets * 4;
  return FS_OK;
}

fs_status fs_plan_node_groups(const fs_plan* plan, int32_t* out, int32_t num_nodes) {
  if (!plan || !out) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  if (num_nodes != plan->graph.n()) FS_FAIL(FS_ERR_INVALID_ARG, "num_nodes %d, plan has %d", num_nodes, plan->graph.n());
  for (int i = 0; i < num_nodes; ++i) out[i] = plan->group_of[i];
  return FS_OK;
}

fs_status fs_plan_node_spans(const fs_plan* plan, int32_t* out, int32_t num_nodes) {
  if (!plan || !out) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  if (num_nodes != plan->graph.n()) FS_FAIL(FS_ERR_INVALID_ARG, "num_nodes %d, plan has %d", num_nodes, plan->graph.n());
  std::vector<int> span;
  work_span(plan->graph, &span);
  for (int i = 0; i < num_nodes; ++i) out[i] = span[i];
  return FS_OK;
}

fs_status fs_plan_group_source(const fs_plan* plan, int32_t group, const char** out_src) {
  if (!plan || !out_src) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  if (group < 0 || group >= (int)plan->groups.size()) FS_FAIL(FS_ERR_INVALID_ARG, "group %d out of range", group);
  *out_src = plan->groups[group].source.c_str();
  return FS_OK;
}

fs_status fs_plan_group_kernel_name(const fs_plan* plan, int32_t group, const char** out_name) {
  if (!plan || !out_name) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  if (group < 0 || group >= (int)plan->groups.size()) FS_FAIL(FS_ERR_INVALID_ARG, "group %d out of range", group);
  *out_name = plan->groups[group].kernel_name.c_str();
  return FS_OK;
}

fs_status fs_plan_group_perf_key(const fs_plan* plan, int32_t group, const char** out_key) {
  if (!plan || !out_key) FS_FAIL(FS_ERR_INVALID_ARG, "NULL argument");
  if (group < 0 || group >= (int)plan->groups.size()) FS_FAIL(FS_ERR_INVALID_ARG, "group %d out of range", group);
  fs_plan* p = const_cast<fs_plan*>(plan);
  std::lock_guard<std::mutex> lk(p->mu);
  GroupPlan& gp = p->groups[group];
  if (gp.perf_key.empty()) gp.perf_key = perf_key(gp);
  *out_key = gp.perf_key.c_str();
  return FS_OK;
}

// ---- schedule tuning: measure-on-miss into the performance library (Sections 4.3, 4.4) ----------
namespace {

struct TuneScratch {  // everything fs_plan_tune allocates, released on every exit path
  void* flush = nullptr;
  void* scratch = nullptr;
  hipModule_t module = nullptr;
  std::vector<hipEvent_t> events;
  ~TuneScratch() {
    (void)hipDeviceSynchronize();  // nothing below may still be in use by a launch
    if (module) (void)hipModuleUnload(module);
    if (scratch) (void)hipFree(scratch);
    if (flush) (void)hipFree(flush);
    for (hipEvent_t e : events) (void)hipEventDestroy(e);
  }
};

}  // namespace

fs_status fs_plan_tune(fs_plan* plan, const void* const* inputs, void* const* outputs, void* workspace,
                       size_t workspace_bytes, void* hip_stream, int32_t reps, fs_tune_report* report) {
  if (!plan) FS_FAIL(FS_ERR_INVALID_ARG, "plan is NULL");
  const Graph& g = plan->graph;
  fs_status st = check_workspace(plan, workspace, workspace_bytes);
  if (st != FS_OK) return st;
  st = check_buffers(plan, inputs, outputs, workspace);
  if (st != FS_OK) return st;
  if (reps <= 0) reps = 9;
  if (reps > 101) reps = 101;
  hipStream_t stream = (hipStream_t)hip_stream;
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) FS_FAIL(FS_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
  fs_plan::Loaded* ld = nullptr;
  st = load_on_device(plan, device, &ld);
  if (st != FS_OK) return st;
#define FS_HIP(call)                                                                 \
  do {                                                                               \
    const hipError_t e_ = (call);                                                    \
    if (e_ != hipSuccess) FS_FAIL(FS_ERR_HIP, "%s: %s", #call, hipGetErrorString(e_)); \
  } while (0)

  char* ws = (char*)workspace;
  auto tensor_ptr = [&](int node) -> void* {  // a view addresses the buffer of the value it is a view of
    const int root = g.root_of[node];
    if (g.input_index[root] >= 0) return const_cast<void*>(inputs[g.input_index[root]]);
    if (g.family_output[root] >= 0) return outputs[g.family_output[root]];
    return ws + plan->ws_tensor_offset.at(root);
  };

  TuneScratch res;
  constexpr size_t kFlushBytes = 256ull << 20;  // one pass over 2 x 256 MiB evicts the last-level cache
  res.events.resize(2 * (size_t)reps);
  for (hipEvent_t& ev : res.events) {
    ev = nullptr;
    FS_HIP(hipEventCreate(&ev));
  }
  fs_tune_report rep = {};
  PlanOptions base_opt = plan->opt;
  base_opt.has_hint = false;

  for (size_t gi = 0; gi < plan->groups.size(); ++gi) {
    const GroupPlan& base = plan->groups[gi];
    void* tensors[48];
    size_t nt = 0;
    for (const ExtTensor& t : base.ext_in) tensors[nt++] = tensor_ptr(t.node);
    for (const ExtTensor& t : base.ext_out) tensors[nt++] = tensor_ptr(t.node);
    void* base_part = base.part_bytes ? (void*)(ws + base.part_offset) : nullptr;
    void* base_tickets = base.n_tickets ? (void*)(ws + base.ticket_offset) : nullptr;

    // the current schedule first, then its neighbourhood (distinct kernels only)
    std::vector<GroupPlan> cands;
    cands.push_back(base);
    std::set<std::string> keys{perf_key(base)};
    for (const fs_sched_hint& h : candidate_hints(base)) {
      PlanOptions o = base_opt;
      o.hint = h;
      o.has_hint = true;
      GroupPlan c;
      if (analyse_group(g, base.members, plan->group_of, (int)gi, o, &c) != FS_OK) continue;
      if (c.s.L != h.lanes_per_row || c.s.WG != h.wg_threads) continue;
      if (generate_kernel(g, &c, (int)gi) != FS_OK) continue;
      if (!keys.insert(perf_key(c)).second) continue;
      cands.push_back(std::move(c));
    }
    const bool cold = base.min_hbm_bytes > (1ull << 20);
    if (!res.flush) FS_HIP(hipMalloc(&res.flush, 2 * kFlushBytes));

    double cur_us = 0.0, best_us = 0.0;
    for (size_t k = 0; k < cands.size(); ++k) {
      const GroupPlan& c = cands[k];
      const std::string key = perf_key(c);
      double us = 0.0;
      ++rep.candidates;
      if (perflib_lookup(key, &us)) {
        ++rep.hits;
      } else {
        void* fn = ld->functions[gi];
        void* part = base_part;
        void* tickets = base_tickets;
        if (k > 0) {
          std::vector<char> code;
          st = compile_kernel(std::string(device_header_source()) + "\n" + c.source, c.kernel_name, &code);
          if (st != FS_OK) return st;
          FS_HIP(hipModuleLoadData(&res.module, code.data()));
          hipFunction_t f;
          FS_HIP(hipModuleGetFunction(&f, res.module, c.kernel_name.c_str()));
          fn = (void*)f;
          const size_t tbytes = align_up((size_t)c.n_tickets * 4, 256);
          if (tbytes + c.part_bytes > 0) {
            FS_HIP(hipMalloc(&res.scratch, tbytes + c.part_bytes));
            if (tbytes) {
              const int ze = launch_zero_u32(res.scratch, tbytes / 4, stream);
              if (ze != 0) FS_FAIL(FS_ERR_HIP, "fill kernel launch: %s", hipGetErrorString((hipError_t)ze));
            }
            tickets = c.n_tickets ? res.scratch : nullptr;
            part = c.part_bytes ? (void*)((char*)res.scratch + tbytes) : nullptr;
          } else {
            part = tickets = nullptr;
          }
        }
        // The device needs tens of milliseconds of work to reach its steady clocks, and it has idled
        // while this candidate was compiled: ~35 ms of copies first (a kernel measured right after an
        // idle period reads 5-10 % slow, more than most differences between candidates).
        for (int w = 0; w < 200; ++w) {
          const int ce = launch_copy_probe(res.flush, (char*)res.flush + kFlushBytes, kFlushBytes, stream);
          if (ce != 0) FS_FAIL(FS_ERR_HIP, "warm-up launch: %s", hipGetErrorString((hipError_t)ce));
        }
        for (int w = 0; w < 2; ++w) FS_HIP(launch_group(c, fn, tensors, part, tickets, stream));
        // a cold launch is timed on its own; launches that live in the caches anyway are timed in runs of 20
        const int inner = cold ? 1 : 20;
        for (int r = 0; r < reps; ++r) {
          if (cold) {
            const int ce = launch_copy_probe(res.flush, (char*)res.flush + kFlushBytes, kFlushBytes, stream);
            if (ce != 0) FS_FAIL(FS_ERR_HIP, "flush launch: %s", hipGetErrorString((hipError_t)ce));
          }
          FS_HIP(hipEventRecord(res.events[2 * r], stream));
          for (int i = 0; i < inner; ++i) FS_HIP(launch_group(c, fn, tensors, part, tickets, stream));
          FS_HIP(hipEventRecord(res.events[2 * r + 1], stream));
        }
        FS_HIP(hipStreamSynchronize(stream));
        std::vector<float> ms((size_t)reps);
        for (int r = 0; r < reps; ++r) FS_HIP(hipEventElapsedTime(&ms[r], res.events[2 * r], res.events[2 * r + 1]));
        std::sort(ms.begin(), ms.end());
        us = (double)ms[(size_t)reps / 2] * 1e3 / inner;
        char note[160];
        snprintf(note, sizeof(note), "%zu nodes on [%d,%d]: %d lanes/row, %d elements/lane, workgroup %d, grid %d, %s", c.members.size(), c.R,
                 c.C, c.s.L, c.s.E, c.s.WG, c.s.grid, cold ? "cold caches" : "warm caches");
        if (!perflib_insert(key, us, note)) FS_FAIL(FS_ERR_INVALID_ARG, "the performance library file cannot be written");
        ++rep.measured;
        if (res.module) {
          (void)hipModuleUnload(res.module);
          res.module = nullptr;
        }
        if (res.scratch) {
          (void)hipFree(res.scratch);
          res.scratch = nullptr;
        }
      }
      if (k == 0) cur_us = best_us = us;
      else if (us < best_us) best_us = us;
    }
    rep.current_usec += cur_us;
    rep.best_usec += best_us;
    if (best_us < cur_us) ++rep.improvable;
    ++rep.groups;
    // leave this group's results as a normal run would, for the groups that follow
    FS_HIP(launch_group(base, ld->functions[gi], tensors, base_part, base_tickets, stream));
  }
  FS_HIP(hipStreamSynchronize(stream));
#undef FS_HIP
  if (report) *report = rep;
  return FS_OK;
}

fs_status fs_copy_probe(const void* src, void* dst, size_t bytes, void* hip_stream) {
  if (!src || !dst || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
    FS_FAIL(FS_ERR_INVALID_ARG, "copy probe needs 16-byte aligned pointers and a multiple of 16 bytes");
  const int e = launch_copy_probe(src, dst, bytes, (hipStream_t)hip_stream);
  if (e != 0) FS_FAIL(FS_ERR_HIP, "copy probe launch: %s", hipGetErrorString((hipError_t)e));
  return FS_OK;
}

fs_status fs_copy_probe_shape(const void* src, void* dst, size_t bytes, int32_t vectors_in_flight, int32_t workgroups, void* hip_stream) {
  if (!src || !dst || (bytes & 15) || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15))
    FS_FAIL(FS_ERR_INVALID_ARG, "copy probe needs 16-byte aligned pointers and a multiple of 16 bytes");
  if (workgroups < 0 || (vectors_in_flight != 1 && vectors_in_flight != 2 && vectors_in_flight != 4 && vectors_in_flight != 8))
    FS_FAIL(FS_ERR_INVALID_ARG, "copy probe shape: vectors_in_flight must be 1, 2, 4 or 8 and workgroups >= 0");
  const int e = launch_copy_probe_shape(src, dst, bytes, vectors_in_flight, workgroups, (hipStream_t)hip_stream);
  if (e != 0) FS_FAIL(FS_ERR_HIP, "copy probe launch: %s", hipGetErrorString((hipError_t)e));
  return FS_OK;
}

fs_status fs_alu_probe(void* out, int32_t workgroups, int32_t iters, void* hip_stream) {
  if (!out || ((uintptr_t)out & 3) || workgroups < 1 || workgroups > (1 << 20) || iters < 1 || iters > (1 << 24))
    FS_FAIL(FS_ERR_INVALID_ARG, "alu probe needs an output buffer of workgroups * 256 floats, 1..2^20 workgroups and 1..2^24 trips");
  const int e = launch_alu_probe((float*)out, workgroups, iters, (hipStream_t)hip_stream);
  if (e != 0) FS_FAIL(FS_ERR_HIP, "alu probe launch: %s", hipGetErrorString((hipError_t)e));
  return FS_OK;
}

fs_status fs_launch_probe(void* hip_stream) {
  const int e = launch_empty((hipStream_t)hip_stream);
  if (e != 0) FS_FAIL(FS_ERR_HIP, "empty kernel launch: %s", hipGetErrorString((hipError_t)e));
  return FS_OK;
}

}  // extern "C"
