// Calibration probe for hardware-counter HBM traffic: a plain copy kernel of known size.
// `copy_probe <MiB> <reps>` copies <MiB> MiB (reads that much, writes that much) <reps> times.
// Profiling it with the same counters as the solver (FETCH_SIZE, WRITE_SIZE) gives the factor
// between counter units and bytes, which the solver's counter readings are scaled by.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef float f4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void copy_probe_kernel(const f4v* __restrict__ src, f4v* __restrict__ dst, size_t nvec) {
  const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
  if (e < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + e), dst + e);
}

int main(int argc, char** argv) {
  const size_t mib = argc > 1 ? (size_t)atoll(argv[1]) : 1024;
  const int reps = argc > 2 ? atoi(argv[2]) : 5;
  const size_t bytes = mib << 20, nvec = bytes / 16;
  f4v *src = nullptr, *dst = nullptr;
  if (hipMalloc(&src, bytes) != hipSuccess || hipMalloc(&dst, bytes) != hipSuccess) {
    fprintf(stderr, "copy_probe: allocation of 2 x %zu MiB failed\n", mib);
    return 1;
  }
  if (hipMemset(src, 1, bytes) != hipSuccess || hipMemset(dst, 0, bytes) != hipSuccess) return 1;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  (void)hipDeviceSynchronize();
  (void)hipEventRecord(e0);
  for (int r = 0; r < reps; ++r)
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)((nvec + 255) / 256)), dim3(256), 0, 0, src, dst, nvec);
  (void)hipEventRecord(e1);
  if (hipEventSynchronize(e1) != hipSuccess) return 1;
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  printf("copy_probe: %d launches, each reads %zu bytes and writes %zu bytes; %.4f ms per launch, %.0f GB/s\n", reps,
         bytes, bytes, ms / reps, 2.0 * bytes / (ms / reps) / 1e6);
  (void)hipFree(src);
  (void)hipFree(dst);
  return 0;
}
