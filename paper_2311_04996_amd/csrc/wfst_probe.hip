// Measured ceilings of the GPU the decoder runs on: what a plain device copy, random 128-byte
// line reads and random 64-bit global atomics reach.  The decoder's roofline is quoted against
// the published HBM bandwidth; these figures say what the chip delivers for the access patterns
// the decoder actually has (streams of records, one random line per token, and -- in the design
// that was measured and dropped -- one global atomic per candidate).
#include <hip/hip_runtime.h>

#include <cstdint>

#include "wfst_probe.h"

namespace {

constexpr int kThreads = 1024;

// dst[i] = src[i], 16 bytes per lane and step, grid-stride
__global__ __launch_bounds__(kThreads) void probe_copy(const int4 *src, int4 *dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * kThreads;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

__device__ __forceinline__ unsigned lcg(unsigned &s) { s = s * 1664525u + 1013904223u; return s; }

// every lane reads 16 bytes of a random 128-byte line, U independent loads in flight
template <int U>
__global__ __launch_bounds__(kThreads) void probe_lines(const int4 *a, unsigned line_mask, int iters, int *sink) {
  unsigned s = (blockIdx.x * kThreads + threadIdx.x) * 2654435761u + 12345u;
  int acc = 0;
  for (int it = 0; it < iters; ++it) {
    int4 v[U];
#pragma unroll
    for (int u = 0; u < U; ++u) v[u] = a[(size_t)((lcg(s) >> 4) & line_mask) * 8];   // 8 x 16 B = one line
#pragma unroll
    for (int u = 0; u < U; ++u) acc += v[u].x + v[u].w;
  }
  if (acc == 0x7fffffff) *sink = acc;          // never true: keeps the loads
}

// every lane does a 64-bit atomicMin on a random word, U in flight
template <int U>
__global__ __launch_bounds__(kThreads) void probe_atomics(unsigned long long *t, unsigned mask, int iters, int *sink) {
  unsigned s = (blockIdx.x * kThreads + threadIdx.x) * 2654435761u + 777u;
  unsigned long long acc = 0;
  for (int it = 0; it < iters; ++it) {
    unsigned long long r[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const unsigned x = lcg(s);
      r[u] = atomicMin(&t[(x >> 4) & mask], ((unsigned long long)x << 32) | u);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) acc += r[u];
  }
  if (acc == 0x7fffffffull) *sink = (int)acc;
}

struct Timer {
  hipEvent_t a = nullptr, b = nullptr;
  bool ok() { return hipEventCreate(&a) == hipSuccess && hipEventCreate(&b) == hipSuccess; }
  ~Timer() { if (a) (void)hipEventDestroy(a); if (b) (void)hipEventDestroy(b); }
};

#define PROBE_TRY(expr) do { if ((expr) != hipSuccess) { rc = -1; goto done; } } while (0)

}  // namespace

extern "C" {

int32_t wfst_probe_copy(int64_t bytes, int32_t reps, double *gb_per_s) {
  if (bytes < (1 << 20) || reps < 1 || !gb_per_s) return -1;
  int rc = 0; float ms = 0.0f;
  int4 *src = nullptr, *dst = nullptr;
  Timer t;
  const size_t n = (size_t)bytes / 16;
  if (!t.ok()) return -1;
  PROBE_TRY(hipMalloc(reinterpret_cast<void **>(&src), n * 16));
  PROBE_TRY(hipMalloc(reinterpret_cast<void **>(&dst), n * 16));
  PROBE_TRY(hipMemset(src, 1, n * 16));
  PROBE_TRY(hipMemset(dst, 0, n * 16));
  hipLaunchKernelGGL(probe_copy, dim3(2048), dim3(kThreads), 0, nullptr, src, dst, n);   // warm-up
  PROBE_TRY(hipDeviceSynchronize());
  PROBE_TRY(hipEventRecord(t.a, nullptr));
  for (int r = 0; r < reps; ++r) hipLaunchKernelGGL(probe_copy, dim3(2048), dim3(kThreads), 0, nullptr, src, dst, n);
  PROBE_TRY(hipEventRecord(t.b, nullptr));
  PROBE_TRY(hipEventSynchronize(t.b));
  PROBE_TRY(hipEventElapsedTime(&ms, t.a, t.b));
  *gb_per_s = 2.0 * (double)n * 16.0 * reps / (ms * 1e-3) / 1e9;       // bytes read + bytes written
done:
  if (src) (void)hipFree(src);
  if (dst) (void)hipFree(dst);
  return rc;
}

int32_t wfst_probe_random_lines(int64_t footprint_bytes, int32_t workgroups, int32_t loads_per_lane, double *lines_per_s) {
  if (footprint_bytes < (1 << 20) || workgroups < 1 || loads_per_lane < 8 || !lines_per_s) return -1;
  int rc = 0; float ms = 0.0f;
  int4 *a = nullptr; int *sink = nullptr;
  Timer t;
  size_t lines = 1;
  while (lines * 2 * 128 <= (size_t)footprint_bytes) lines *= 2;                 // a power of two of 128-byte lines
  if (!t.ok()) return -1;
  PROBE_TRY(hipMalloc(reinterpret_cast<void **>(&a), lines * 128));
  PROBE_TRY(hipMalloc(reinterpret_cast<void **>(&sink), sizeof(int)));
  PROBE_TRY(hipMemset(a, 1, lines * 128));
  hipLaunchKernelGGL(probe_lines<8>, dim3(workgroups), dim3(kThreads), 0, nullptr, a, (unsigned)(lines - 1), 8, sink);
  PROBE_TRY(hipDeviceSynchronize());
  PROBE_TRY(hipEventRecord(t.a, nullptr));
  hipLaunchKernelGGL(probe_lines<8>, dim3(workgroups), dim3(kThreads), 0, nullptr, a, (unsigned)(lines - 1), loads_per_lane / 8, sink);
  PROBE_TRY(hipEventRecord(t.b, nullptr));
  PROBE_TRY(hipEventSynchronize(t.b));
  PROBE_TRY(hipEventElapsedTime(&ms, t.a, t.b));
  *lines_per_s = (double)workgroups * kThreads * (loads_per_lane / 8 * 8) / (ms * 1e-3);
done:
  if (a) (void)hipFree(a);
  if (sink) (void)hipFree(sink);
  return rc;
}

int32_t wfst_probe_atomics(int64_t footprint_bytes, int32_t workgroups, int32_t atomics_per_lane, double *atomics_per_s) {
  if (footprint_bytes < (1 << 20) || workgroups < 1 || atomics_per_lane < 4 || !atomics_per_s) return -1;
  int rc = 0; float ms = 0.0f;
  unsigned long long *tab = nullptr; int *sink = nullptr;
  Timer t;
  size_t words = 1;
  while (words * 2 * 8 <= (size_t)footprint_bytes) words *= 2;
  if (!t.ok()) return -1;
  PROBE_TRY(hipMalloc(reinterpret_cast<void **>(&tab), words * 8));
  PROBE_TRY(hipMalloc(reinterpret_cast<void **>(&sink), sizeof(int)));
  PROBE_TRY(hipMemset(tab, 0xff, words * 8));
  hipLaunchKernelGGL(probe_atomics<4>, dim3(workgroups), dim3(kThreads), 0, nullptr, tab, (unsigned)(words - 1), 4, sink);
  PROBE_TRY(hipDeviceSynchronize());
  PROBE_TRY(hipEventRecord(t.a, nullptr));
  hipLaunchKernelGGL(probe_atomics<4>, dim3(workgroups), dim3(kThreads), 0, nullptr, tab, (unsigned)(words - 1), atomics_per_lane / 4, sink);
  PROBE_TRY(hipEventRecord(t.b, nullptr));
  PROBE_TRY(hipEventSynchronize(t.b));
  PROBE_TRY(hipEventElapsedTime(&ms, t.a, t.b));
  *atomics_per_s = (double)workgroups * kThreads * (atomics_per_lane / 4 * 4) / (ms * 1e-3);
done:
  if (tab) (void)hipFree(tab);
  if (sink) (void)hipFree(sink);
  return rc;
}

}  // extern "C"
