// Plain copy kernel of known size: the reference that rocprofv3's FETCH_SIZE / WRITE_SIZE counters
// are scaled by (1 GiB read, 1 GiB written per launch), and a stream-copy bandwidth figure.
#include <hip/hip_runtime.h>

#include <cstdio>

__global__ void k_copy_ref(const float4* a, float4* b, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x)
    b[i] = a[i];
}

int main() {
  const size_t n = (size_t)1 << 26;  // float4 elements = 1 GiB
  float4 *a, *b;
  if (hipMalloc(&a, n * 16) != hipSuccess || hipMalloc(&b, n * 16) != hipSuccess) return 1;
  if (hipMemset(a, 1, n * 16) != hipSuccess) return 1;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return 1;
  for (int r = 0; r < 4; ++r) {
    float ms = 0;
    bool ok = hipEventRecord(e0) == hipSuccess;
    k_copy_ref<<<8192, 256>>>(a, b, n);
    ok = ok && hipEventRecord(e1) == hipSuccess && hipEventSynchronize(e1) == hipSuccess &&
         hipEventElapsedTime(&ms, e0, e1) == hipSuccess;
    if (!ok) return 1;
    printf("copy %zu B read + %zu B written: %.3f ms, %.1f GB/s\n", n * 16, n * 16, ms, 2.0 * n * 16 / ms / 1e6);
  }
  return 0;
}
