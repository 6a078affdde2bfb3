// fs_perflib.cpp - the performance library: a persistent key-value store of measured kernel
// times (Section 4.4).
//
// A key names one concrete kernel under one concrete launch: the kernel's structural hash (its
// generated source, which bakes in lanes per row, elements per lane, workgroup size and every
// other schedule constant), the number of rows, the loop trips and the grid.  The value is the
// measured time of that launch in microseconds.  Schedule tuning (Section 4.3) enumerates the
// candidate schedules of a group, looks each one up here and keeps the fastest; a key that
// misses is measured on the device by fs_plan_tune and inserted.
//
// Unlike the paper's library, which stores the time of every op of a computation on its own
// and scores a schedule by the sum, a record here is the time of the whole fused kernel: the
// kernel is generated and compiled in a fraction of a second, so the quantity being optimised
// can be measured directly instead of being approximated.
//
// Storage: a text file, one "key<TAB>microseconds" record per line, later records override
// earlier ones; '#' starts a comment.  The file named by FS_PERF_LIBRARY, else perflib.tsv
// beside the shared library.  Loaded on first use and re-read when the file changes.
#include <dlfcn.h>
#include <sys/stat.h>

#include <cstdlib>
#include <fstream>
#include <sstream>

#include "fs_internal.h"

namespace fs {

namespace {

struct Library {
  std::mutex mu;
  std::string path;
  std::map<std::string, double> kv;
  long long mtime_ns = -1;
  long long size = -1;
};

Library& library() {
  static Library lib;
  return lib;
}

std::string default_path() {
  if (const char* e = getenv("FS_PERF_LIBRARY")) return e;
  Dl_info info;
  if (dladdr((void*)&default_path, &info) && info.dli_fname) {
    std::string p = info.dli_fname;
    const size_t slash = p.rfind('/');
    if (slash != std::string::npos) return p.substr(0, slash) + "/perflib.tsv";
  }
  return "";
}

// (re)load when the path or the file changed; called with the lock held
void refresh(Library& lib) {
  const std::string path = default_path();
  struct stat st;
  const bool exists = !path.empty() && stat(path.c_str(), &st) == 0;
  const long long mt = exists ? (long long)st.st_mtim.tv_sec * 1000000000ll + st.st_mtim.tv_nsec : -1;
  const long long sz = exists ? (long long)st.st_size : -1;
  if (path == lib.path && mt == lib.mtime_ns && sz == lib.size) return;
  lib.path = path;
  lib.mtime_ns = mt;
  lib.size = sz;
  lib.kv.clear();
  if (!exists) return;
  std::ifstream f(path);
  std::string line;
  while (std::getline(f, line)) {
    if (line.empty() || line[0] == '#') continue;
    const size_t tab = line.find('\t');
    if (tab == std::string::npos) continue;
    char* end = nullptr;
    const double us = strtod(line.c_str() + tab + 1, &end);
    if (end == line.c_str() + tab + 1 || !(us > 0.0)) continue;
    lib.kv[line.substr(0, tab)] = us;
  }
}

}  // namespace

std::string perf_key(const GroupPlan& gp) {
  std::ostringstream os;
  os << gp.kernel_name << ":R" << gp.R << ":it" << gp.s.n_iters << ":g" << gp.s.grid << ":wg" << gp.s.WG;
  return os.str();
}

size_t perflib_size() {
  Library& lib = library();
  std::lock_guard<std::mutex> lk(lib.mu);
  refresh(lib);
  return lib.kv.size();
}

bool perflib_lookup(const std::string& key, double* usec) {
  Library& lib = library();
  std::lock_guard<std::mutex> lk(lib.mu);
  refresh(lib);
  auto it = lib.kv.find(key);
  if (it == lib.kv.end()) return false;
  if (usec) *usec = it->second;
  return true;
}

bool perflib_insert(const std::string& key, double usec, const std::string& note) {
  Library& lib = library();
  std::lock_guard<std::mutex> lk(lib.mu);
  refresh(lib);
  if (lib.path.empty()) return false;
  {
    std::ofstream f(lib.path, std::ios::app);
    if (!f) return false;
    char buf[64];
    snprintf(buf, sizeof(buf), "%.3f", usec);
    if (!note.empty()) f << "# " << note << "\n";
    f << key << "\t" << buf << "\n";
  }
  lib.mtime_ns = -1;  // our own write changed the file: read it back on the next use
  refresh(lib);
  return true;
}

}  // namespace fs
