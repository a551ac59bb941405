// Rates of the memory operations the design rests on, measured on the box: dependent kernel
// launches, random 4-byte atomic adds (with and without return value, several footprints, one
// address, one compute unit), random 4-byte stores and gathers.  Every index is reduced modulo the
// array length; every loop has a fixed trip count.
//
// `chip_rates resident` measures instead what a kernel that stays resident over many time steps
// would pay for synchronising its blocks: which XCD (compute die, one L2 each) every block of a
// grid runs on, the hand-over of a word between two blocks on one XCD and on two (by kind of store
// and load), grid barriers (one counter, one counter per XCD under a top word, a flag per block;
// all blocks or the blocks of one XCD), whether data passed between blocks of one XCD arrives,
// dependent-access latencies, and what one XCD alone streams and scatters.  Every wait is a
// bounded spin: a wait that runs out sets an error word, and the blocks go on to the end.
#include <hip/hip_runtime.h>
#include <chrono>

#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

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

// Holds the stream for `ticks` of the 100 MHz wall clock (a bounded wait by construction).
__global__ void k_hold(unsigned long long ticks) {
  const unsigned long long t0 = wall_clock64();
  while (wall_clock64() - t0 < ticks) __builtin_amdgcn_s_sleep(32);
}
__global__ void k_empty(int* p) { if (p && threadIdx.x == 9999) p[0] = 1; }

// Dense neuron step as a stream: per neuron one cell (int) and one state (float) read, the state
// and a trace value written.  VEC = neurons per thread (1: 4-byte accesses, 4: 16-byte accesses).
template <int VEC>
__global__ void k_dense_step(const int* __restrict__ cell, float* __restrict__ state, float* __restrict__ trace, size_t n) {
  const size_t t = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) * VEC;
  if (t >= n) return;
  if (VEC == 1) {
    const float u = 0.995f * state[t] + (float)cell[t] * 0x1p-24f;
    state[t] = u >= 1.0f ? 0.0f : u;
    trace[t] = u;
  } else {
    const int4 c = *reinterpret_cast<const int4*>(cell + t);
    const float4 v = *reinterpret_cast<const float4*>(state + t);
    float4 u;
    u.x = 0.995f * v.x + (float)c.x * 0x1p-24f; u.y = 0.995f * v.y + (float)c.y * 0x1p-24f;
    u.z = 0.995f * v.z + (float)c.z * 0x1p-24f; u.w = 0.995f * v.w + (float)c.w * 0x1p-24f;
    *reinterpret_cast<float4*>(trace + t) = u;
    u.x = u.x >= 1.0f ? 0.0f : u.x; u.y = u.y >= 1.0f ? 0.0f : u.y;
    u.z = u.z >= 1.0f ? 0.0f : u.z; u.w = u.w >= 1.0f ? 0.0f : u.w;
    *reinterpret_cast<float4*>(state + t) = u;
  }
}

// The same step with four neurons per thread, 64 apart (4-byte accesses, a quarter of the wavefronts).
__global__ void k_dense_step_strided(const int* __restrict__ cell, float* __restrict__ state, float* __restrict__ trace, size_t n) {
  const size_t base = ((size_t)blockIdx.x * blockDim.x + (threadIdx.x & ~63u)) * 4 + (threadIdx.x & 63u);
  int c[4]; float v[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) { const size_t t = base + 64 * j; c[j] = t < n ? cell[t] : 0; v[j] = t < n ? state[t] : 0.0f; }
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const size_t t = base + 64 * j;
    const float u = 0.995f * v[j] + (float)c[j] * 0x1p-24f;
    if (t < n) { state[t] = u >= 1.0f ? 0.0f : u; trace[t] = u; }
  }
}

template <int VEC>
static int run_dense(size_t n, hipEvent_t e0, hipEvent_t e1) {
  const int steps = 256, rows = 16;
  int* cell = nullptr; float *state = nullptr, *trace = nullptr;
  CK(hipMalloc(&cell, n * 4 * rows)); CK(hipMalloc(&state, n * 4)); CK(hipMalloc(&trace, n * 4 * steps));
  CK(hipMemset(cell, 0, n * 4 * rows)); CK(hipMemset(state, 0, n * 4));
  const int per = VEC < 0 ? -VEC : VEC;
  const unsigned grid = (unsigned)((n / per + 255) / 256);
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    for (int i = 0; i < steps; ++i) {
      if (VEC < 0) k_dense_step_strided<<<grid, 256>>>(cell + (size_t)(i % rows) * n, state, trace + (size_t)i * n, n);
      else k_dense_step<(VEC < 0 ? 1 : VEC)><<<grid, 256>>>(cell + (size_t)(i % rows) * n, state, trace + (size_t)i * n, n);
    }
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  printf("  %8zu neurons, %2d-byte accesses, %d per thread: %6.2f us per launch, %6.0f GB/s (16 B per neuron)\n", n,
         VEC < 0 ? 4 : 4 * VEC, per,
         ms * 1e3 / steps, (double)n * 16.0 * steps / ms / 1e6);
  CK(hipFree(cell)); CK(hipFree(state)); CK(hipFree(trace));
  return 0;
}

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

#include "resident_rates.h"
#include "exchange_rates.h"

int main(int argc, char** argv) {
  if (argc > 1 && strcmp(argv[1], "resident") == 0) return resident_main();
  if (argc > 1 && strcmp(argv[1], "exchange") == 0) return exchange_main();
  hipEvent_t e0, e1;
  CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  float ms = 0;
  for (int rep = 0; rep < 2; ++rep) {
    CK(hipEventRecord(e0));
    for (int i = 0; i < 1000; ++i) k_empty<<<391, 256>>>(nullptr);
    CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
  }
  printf("1000 empty launches of 391 x 256 threads on one stream: %.2f us each\n", ms);
  // The same with the queue filled beforehand: a kernel that holds the stream for 6 ms goes first, the host
  // enqueues the 1000 launches behind it (2.4 ms of host time), and the events bracket what the GPU then
  // needs by itself -- so that the figure above can be told apart from the host's own rate of enqueueing.
  {
    double host_us = 0;
    for (int rep = 0; rep < 2; ++rep) {
      k_hold<<<1, 64>>>(600000ull);   // 6 ms in 10 ns ticks
      CK(hipEventRecord(e0));
      const auto t0 = std::chrono::steady_clock::now();
      for (int i = 0; i < 1000; ++i) k_empty<<<391, 256>>>(nullptr);
      host_us = std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count() / 1000.0;
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("1000 empty launches of 391 x 256 threads enqueued behind a kernel that holds the stream: %.2f us each on the GPU (the host enqueues one in %.2f us)\n", ms, host_us);
  }
  const int shapes[][2] = {{4096, 256}, {2048, 512}, {1024, 1024}, {16384, 64}};
  for (auto& sh : shapes) {
    for (int rep = 0; rep < 2; ++rep) {
      CK(hipEventRecord(e0));
      for (int i = 0; i < 1000; ++i) k_empty<<<sh[0], sh[1]>>>(nullptr);
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1)); CK(hipEventElapsedTime(&ms, e0, e1));
    }
    printf("1000 empty launches of %d x %d threads on one stream: %.2f us each\n", sh[0], sh[1], ms);
  }
  printf("dense neuron step as a stream (cell + state read, state + trace written), 256 launches on one stream:\n");
  for (size_t n : {(size_t)102400, (size_t)1048576, (size_t)4194304}) {
    if (run_dense<1>(n, e0, e1)) return 1;
    if (run_dense<4>(n, e0, e1)) return 1;
    if (run_dense<-4>(n, e0, e1)) return 1;
  }
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
