// Rates of the memory operations the design rests on, measured on the box: dependent kernel
// launches, random 4-byte atomic adds (with and without return value, several footprints, one
// address, one compute unit), random 4-byte stores and gathers.  Every index is reduced modulo the
// array length; every loop has a fixed trip count.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

#define CK(x)                                                                       \
  do {                                                                              \
    hipError_t e_ = (x);                                                            \
    if (e_ != hipSuccess) { printf("%s failed: %s\n", #x, hipGetErrorString(e_)); return 1; } \
  } while (0)

__device__ __forceinline__ unsigned hash32(unsigned x) {
  x ^= x >> 16; x *= 0x7feb352dU; x ^= x >> 15; x *= 0x846ca68bU; x ^= x >> 16;
  return x;
}

// MODE 0: atomic add, no return value; 1: atomic add whose return value is used; 2: plain store;
// 3: gather; 4: atomic add on ONE address by every lane; 5: by one lane per wavefront
template <int MODE>
__global__ void k_random(int* arr, unsigned M, size_t n_ops, int per) {
  const size_t t = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  int acc = 0;
  for (int r = 0; r < per; ++r) {
    const size_t e = t + (size_t)r * gridDim.x * blockDim.x;
    if (e >= n_ops) break;
    const unsigned idx = MODE >= 4 ? 0u : hash32((unsigned)e * 2654435761u + 12345u) % M;
    if (MODE == 5) { if ((threadIdx.x & 63) == 0) atomicAdd(&arr[idx], 1); }
    else if (MODE == 0 || MODE == 4) atomicAdd(&arr[idx], 1);
    else if (MODE == 1) acc += atomicAdd(&arr[idx], 1);
    else if (MODE == 2) arr[idx] = (int)e;
    else acc += arr[idx];
  }
  if ((MODE == 1 || MODE == 3) && acc == 0x7fffffff) arr[0] = acc;
}

__global__ void k_empty(int* p) { if (p && threadIdx.x == 9999) p[0] = 1; }

template <int MODE>
static int run(const char* name, int* arr, unsigned M, size_t n_ops, unsigned grid_limit, hipEvent_t e0, hipEvent_t e1,
               int per = 16) {
  unsigned grid = (unsigned)((n_ops / per + 255) / 256);
  if (grid_limit && grid > grid_limit) grid = grid_limit;
  const size_t ops = (size_t)grid * 256 * per < n_ops ? (size_t)grid * 256 * per : n_ops;
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    k_random<MODE><<<grid, 256>>>(arr, M, ops, per);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  const double done = MODE == 5 ? (double)ops / 64.0 : (double)ops;
  printf("  %-44s %9.3f ms  %8.3f G ops/s\n", name, ms, done / ms / 1e6);
  return 0;
}

int main() {
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    for (int i = 0; i < 1000; ++i) k_empty<<<391, 256>>>(nullptr);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  printf("1000 empty launches of 391 x 256 threads on one stream: %.2f us each\n", ms);
  const size_t sizes[] = {100000, 1600000, 25100000, 251000000};
  for (size_t M : sizes) {
    int* arr = nullptr;
    CK(hipMalloc(&arr, M * 4)); CK(hipMemset(arr, 0, M * 4));
    const size_t n = (size_t)1 << 27;
    printf("array of %zu ints (%.1f MB), %zu random 4-byte operations:\n", M, M * 4 / 1e6, n);
    if (run<0>("atomic add, no return value", arr, (unsigned)M, n, 0, e0, e1)) return 1;
    if (run<1>("atomic add, return value used", arr, (unsigned)M, n, 0, e0, e1)) return 1;
    if (run<2>("store", arr, (unsigned)M, n, 0, e0, e1)) return 1;
    if (run<3>("gather", arr, (unsigned)M, n, 0, e0, e1)) return 1;
    if (M == 25100000) {
      if (run<0>("atomic add, no return, ONE workgroup", arr, (unsigned)M, (size_t)1 << 22, 1, e0, e1, 16384)) return 1;
      if (run<4>("atomic add on ONE address, every lane", arr, (unsigned)M, (size_t)1 << 24, 0, e0, e1)) return 1;
      if (run<5>("atomic add on ONE address, 1 lane per wave", arr, (unsigned)M, (size_t)1 << 24, 0, e0, e1)) return 1;
    }
    CK(hipFree(arr));
  }
  return 0;
}
