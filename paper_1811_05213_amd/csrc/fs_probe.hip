// fs_probe.hip - ahead-of-time kernels: the streaming-copy probe and the workspace fill.
// Also instantiates the building blocks of fs_device.h once, so that a plain hipcc build
// checks the header that generated kernels are prefixed with.
#include <hip/hip_runtime.h>

#include <mutex>

#include "fs.h"
#include "fs_device.h"

typedef unsigned int fs_uint4 __attribute__((ext_vector_type(4)));

// Plain copy, 16 bytes per lane, one vector per lane, non-temporal: the reference point for
// "what fraction of the HBM roofline can a memory-bound kernel of this size reach on this device"
// (one workgroup per 4 KiB, no loop: the launch shape that measured fastest for streaming).
__global__ void __launch_bounds__(256) fs_copy_probe_kernel(const fs_uint4* __restrict__ src, fs_uint4* __restrict__ dst, long n_vec) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i < n_vec) __builtin_nontemporal_store(__builtin_nontemporal_load(&src[i]), &dst[i]);
}

// The same copy with U vectors in flight per lane and a chosen grid (workgroups loop with a grid stride
// when there are fewer of them than tiles): the shapes a streaming kernel could take, for finding the
// fastest plain copy of a given size on the device.  Indices beyond the end are clamped for the loads
// (never predicated, so all U loads are issued back to back) and masked at the stores.
template <int U> __global__ void __launch_bounds__(256) fs_copy_probe_shape_kernel(const fs_uint4* __restrict__ src, fs_uint4* __restrict__ dst, long n_vec) {
  const long stride = (long)gridDim.x * 256;
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n_vec; i += stride * U) {
    fs_uint4 t[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long j = i + u * stride;
      t[u] = __builtin_nontemporal_load(&src[j < n_vec ? j : n_vec - 1]);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long j = i + u * stride;
      if (j < n_vec) __builtin_nontemporal_store(t[u], &dst[j]);
    }
  }
}

// Nothing: the cost of a launch itself.
__global__ void fs_empty_kernel() {}

__global__ void __launch_bounds__(256) fs_zero_u32_kernel(unsigned int* p, long n) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// Exercises every building block (never launched by the library).
struct fs_selftest_kinds {
  static FS_DEV float op(int k, float a, float b) { return k == 0 ? fs_red_op<FS_K_SUM>(a, b) : fs_red_op<FS_K_MAX>(a, b); }
  static FS_DEV float identity(int k) { return k == 0 ? fs_red_identity<FS_K_SUM>() : fs_red_identity<FS_K_MAX>(); }
};
__global__ void __launch_bounds__(256) fs_device_selftest_kernel(const void* in, void* out, float* part, fs_u32* tickets, int R) {
  constexpr int V = 8, NVL = 2, L = 128, NV = 200, WG = 256, G = WG / L, C = NV * V, E = NVL * V;
  __shared__ float lds_rr[2 * G * 2 * 2];
  __shared__ float lds_col[(L < 64 ? WG / 64 : G) * C];
  __shared__ fs_u32 flag;
  const int tid = threadIdx.x, lir = tid & (L - 1), rg = tid / L;
  float ca[E], cb[E];
  for (int e = 0; e < E; ++e) ca[e] = 0.f, cb[e] = fs_red_identity<FS_K_MAX>();
  int parity = 0;
  for (int it = blockIdx.x; it * G < R; it += gridDim.x) {
    const long row = (long)it * G + rg;
    const bool rok = row < R;
    float v[E];
    fs_load_row<FS_DT_BF16, V, NVL, L, NV, true>(v, in, (rok ? row : 0) * C, lir, 0);
    float q = fs_segment_allreduce<FS_K_SUM, 64>(fs_lane_reduce<FS_K_SUM, V, NVL, L, NV, true>(v, lir));
    float m = fs_segment_allreduce<FS_K_MAX, 64>(fs_lane_reduce<FS_K_MAX, V, NVL, L, NV, true>(v, lir));
    const fs_xwave<2, 2> xw{lds_rr + (parity * G + rg) * 4, lir >> 6, (tid & 63) == 0};
    xw.put(0, q);
    xw.put(1, m);
    fs_lds_barrier();
    q = xw.get<FS_K_SUM>(0);
    m = xw.get<FS_K_MAX>(1);
    parity ^= 1;
    for (int e = 0; e < E; ++e) {
      v[e] = fs_round<FS_DT_BF16>(fs_gelu_tanh(fs_tanh(fs_exp(v[e] - m)) / q) + fs_sigmoid(fs_log(fs_rsqrt(fs_rcp(fs_sqrt(v[e]))))));
      ca[e] = rok ? ca[e] + v[e] : ca[e];
      cb[e] = rok ? fs_max(cb[e], v[e]) : cb[e];
    }
    fs_store_row<FS_DT_BF16, V, NVL, L, NV, true>(v, out, row * C, lir, 0, rok);
    fs_store_row_transposed<FS_DT_F32, V, NVL, L, NV, true>(v, out, R, row, lir, 0, rok);
  }
  constexpr int FV = 4;
  typedef fs_colfold<2, C, WG, FV> S;
  float cv[S::CPT][FV];
  fs_colred_fold_wg<FS_K_SUM, 0, 2, V, NVL, L, NV, C, WG, FV, C>(ca, cv, lds_col, lir, rg);
  fs_colred_fold_wg<FS_K_MAX, 1, 2, V, NVL, L, NV, C, WG, FV, C>(cb, cv, lds_col, lir, rg);
  if (fs_colred_fold_grid<2, C, WG, FV, 32, fs_selftest_kinds>(cv, part, tickets, &flag, blockIdx.x, gridDim.x))
    for (int i = 0; i < S::CPT; ++i)
      if (tid + i * WG < S::NCH) fs_store1<FS_DT_F32>(out, (tid + i * WG) * FV, cv[i][0] + cv[i][3]);
}

// Scratch of the allocation-free entry point (fs_plan_run_static): the plan workspace of callers that
// cannot provide one.  Every GPU the library runs on holds its own copy of this array, at its own
// address, until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress: kernels are given the per-device address that call returned, never the name.
static __device__ __align__(256) unsigned char scratch[FS_STATIC_SCRATCH_BYTES];

namespace fs {

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

size_t static_scratch_bytes() { return (size_t)FS_STATIC_SCRATCH_BYTES; }

// Set-up, once per device, with that device current: the device address of the scratch array.
int static_scratch_resolve(int device, void** out) {
  if (device < 0 || device >= kMaxDevices) return (int)hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (!g_scratch_ptr[device]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress((void**)&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return (int)e;
    if (!p) return (int)hipErrorInvalidSymbol;
    g_scratch_ptr[device] = p;
  }
  if (out) *out = g_scratch_ptr[device];
  return 0;
}

// The address resolved earlier for `device`, or NULL.  No HIP call.
void* static_scratch_lookup(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  return g_scratch_ptr[device];
}

int launch_copy_probe(const void* src, void* dst, size_t bytes, hipStream_t stream) {
  const long n_vec = (long)(bytes / 16);
  if (n_vec == 0) return 0;
  const long blocks = (n_vec + 255) / 256;
  if (blocks > 0x7fffffffL) return (int)hipErrorInvalidValue;
  hipLaunchKernelGGL(fs_copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const fs_uint4*)src, (fs_uint4*)dst, n_vec);
  return (int)hipGetLastError();
}

int launch_copy_probe_shape(const void* src, void* dst, size_t bytes, int vectors_in_flight, int workgroups, hipStream_t stream) {
  const long n_vec = (long)(bytes / 16);
  if (n_vec == 0) return 0;
  const int U = vectors_in_flight;
  if (U != 1 && U != 2 && U != 4 && U != 8) return (int)hipErrorInvalidValue;
  long blocks = (n_vec + 256L * U - 1) / (256L * U);  // one trip per workgroup
  if (workgroups > 0 && workgroups < blocks) blocks = workgroups;
  if (blocks > 0x7fffffffL) return (int)hipErrorInvalidValue;
  const dim3 grid((unsigned)blocks), wg(256);
  switch (U) {
    case 1: hipLaunchKernelGGL(fs_copy_probe_shape_kernel<1>, grid, wg, 0, stream, (const fs_uint4*)src, (fs_uint4*)dst, n_vec); break;
    case 2: hipLaunchKernelGGL(fs_copy_probe_shape_kernel<2>, grid, wg, 0, stream, (const fs_uint4*)src, (fs_uint4*)dst, n_vec); break;
    case 4: hipLaunchKernelGGL(fs_copy_probe_shape_kernel<4>, grid, wg, 0, stream, (const fs_uint4*)src, (fs_uint4*)dst, n_vec); break;
    default: hipLaunchKernelGGL(fs_copy_probe_shape_kernel<8>, grid, wg, 0, stream, (const fs_uint4*)src, (fs_uint4*)dst, n_vec); break;
  }
  return (int)hipGetLastError();
}

// Chains of dependent fp32 fused multiply-adds, 8 independent chains per lane, nothing else: what the vector ALUs
// sustain when they are the only thing a kernel uses.  `iters` trips of 128 FMAs per lane; the result is written so
// that nothing is optimised away.
__global__ void __launch_bounds__(256) fs_alu_probe_kernel(float* out, int iters, float a, float b) {
  float x0 = threadIdx.x * 1e-3f, x1 = x0 + 1, x2 = x0 + 2, x3 = x0 + 3, x4 = x0 + 4, x5 = x0 + 5, x6 = x0 + 6, x7 = x0 + 7;
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      x0 = __builtin_fmaf(x0, a, b), x1 = __builtin_fmaf(x1, a, b), x2 = __builtin_fmaf(x2, a, b), x3 = __builtin_fmaf(x3, a, b);
      x4 = __builtin_fmaf(x4, a, b), x5 = __builtin_fmaf(x5, a, b), x6 = __builtin_fmaf(x6, a, b), x7 = __builtin_fmaf(x7, a, b);
    }
  }
  out[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = ((x0 + x1) + (x2 + x3)) + ((x4 + x5) + (x6 + x7));
}

int launch_alu_probe(float* out, int workgroups, int iters, hipStream_t stream) {
  hipLaunchKernelGGL(fs_alu_probe_kernel, dim3((unsigned)workgroups), dim3(256), 0, stream, out, iters, 0.999f, 0.001f);
  return (int)hipGetLastError();
}

int launch_empty(hipStream_t stream) {
  hipLaunchKernelGGL(fs_empty_kernel, dim3(1), dim3(64), 0, stream);
  return (int)hipGetLastError();
}

int launch_zero_u32(void* p, size_t count, hipStream_t stream) {
  if (count == 0) return 0;
  hipLaunchKernelGGL(fs_zero_u32_kernel, dim3((unsigned)((count + 255) / 256)), dim3(256), 0, stream, (unsigned int*)p, (long)count);
  return (int)hipGetLastError();
}

}  // namespace fs
