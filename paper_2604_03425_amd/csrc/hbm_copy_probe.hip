// Plain copy kernel of known size: calibrates what rocprofv3's FETCH_SIZE / WRITE_SIZE counters read per byte moved.
// Usage: rocprofv3 --pmc FETCH_SIZE -- ./hbm_copy_probe   (copies 1 GiB three times)
#include <hip/hip_runtime.h>

#include <cstdio>

__global__ void copy_known(const ulonglong2* __restrict__ in, ulonglong2* __restrict__ out, size_t n) {
  size_t i = blockIdx.x * (size_t)blockDim.x + threadIdx.x;
  if (i < n) out[i] = in[i];
}

int main() {
  const size_t bytes = (size_t)1 << 30;
  ulonglong2 *a = nullptr, *b = nullptr;
  if (hipMalloc(&a, bytes) != hipSuccess || hipMalloc(&b, bytes) != hipSuccess) return 1;
  if (hipMemset(a, 1, bytes) != hipSuccess || hipMemset(b, 2, bytes) != hipSuccess) return 1;
  if (hipDeviceSynchronize() != hipSuccess) return 1;
  hipEvent_t e0, e1;
  hipEventCreate(&e0);
  hipEventCreate(&e1);
  hipEventRecord(e0);
  for (int i = 0; i < 3; i++) copy_known<<<bytes / 16 / 256, 256>>>(a, b, bytes / 16);
  hipEventRecord(e1);
  if (hipEventSynchronize(e1) != hipSuccess) return 1;
  float ms = 0;
  hipEventElapsedTime(&ms, e0, e1);
  printf("copied %zu bytes x3 in %.3f ms: %.1f GB/s (read+write)\n", bytes, ms, 3 * 2.0 * bytes / ms / 1e6);
  hipFree(a);
  hipFree(b);
  return 0;
}
