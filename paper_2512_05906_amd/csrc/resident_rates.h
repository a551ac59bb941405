// `chip_rates resident`: what a kernel that stays resident over many time steps pays for
// synchronising its blocks on this chip.  Included by chip_rates.hip.
//
// The chip has 8 XCDs with an L2 each.  Memory-scope bits of a vector access: none = wavefront
// scope (may hit in the compute unit's own cache), sc0 = workgroup scope, sc1 = agent scope
// (coherent over the whole chip), sc0 sc1 = system scope.  The accesses below are spelled out
// with their bits so that each combination can be timed; atomic read-modify-writes carry no scope
// bit below system scope and are the same instruction at every scope.
//
// Every wait is a bounded spin.  A wait that runs out sets Sync::err and the block stops
// waiting for the rest of the kernel, so every block reaches the end whatever happens.

#include <hip/hip_ext.h>
#include <chrono>

constexpr int kResThreads = 1024;
constexpr int kMaxSpins = 1 << 16;

__device__ __forceinline__ unsigned xcc_id() { return __builtin_amdgcn_s_getreg((3 << 11) | 20) & 15u; }   // HW_REG_XCC_ID
__device__ __forceinline__ unsigned hw_id() { return __builtin_amdgcn_s_getreg((31 << 11) | 4); }          // HW_REG_HW_ID

// loads and stores by scope bits: 0 none, 1 sc0, 2 sc1, 3 sc0 sc1, 4 nt
template <int F> __device__ __forceinline__ unsigned ld(const unsigned* p) {
  unsigned v;
  if (F == 0) asm volatile("global_load_dword %0, %1, off\n s_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  else if (F == 1) asm volatile("global_load_dword %0, %1, off sc0\n s_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  else if (F == 2) asm volatile("global_load_dword %0, %1, off sc1\n s_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  else if (F == 3) asm volatile("global_load_dword %0, %1, off sc0 sc1\n s_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  else asm volatile("global_load_dword %0, %1, off nt\n s_waitcnt vmcnt(0)" : "=v"(v) : "v"(p) : "memory");
  return v;
}
template <int F> __device__ __forceinline__ void st(unsigned* p, unsigned v) {
  if (F == 0) asm volatile("global_store_dword %0, %1, off" ::"v"(p), "v"(v) : "memory");
  else if (F == 1) asm volatile("global_store_dword %0, %1, off sc0" ::"v"(p), "v"(v) : "memory");
  else if (F == 2) asm volatile("global_store_dword %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
  else if (F == 3) asm volatile("global_store_dword %0, %1, off sc0 sc1" ::"v"(p), "v"(v) : "memory");
  else asm volatile("global_store_dword %0, %1, off nt" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void wait_vm() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

struct Sync {
  unsigned top; unsigned pad0[31];
  unsigned xc[8][32];        // one counter per XCD, a 128-byte line each
  unsigned packed[256];      // one flag per block, side by side
  unsigned err, ticket, mism, pad1[29];
  unsigned box[2][32];       // the two words of the hand-over test
  unsigned long long ticks[8];
  unsigned where[512];       // XCD / hardware id of every block
};

// ---------------------------------------------------------------- where blocks run
__global__ void k_where(Sync* s) {
  if (threadIdx.x == 0) { s->where[2 * blockIdx.x] = xcc_id(); s->where[2 * blockIdx.x + 1] = hw_id(); }
}

// ---------------------------------------------------------------- hand-over of one word between two blocks
template <int W, int R>
__global__ void k_pingpong(Sync* s, int a_id, int b_id, int iters) {
  if (threadIdx.x != 0) return;
  const bool a = (int)blockIdx.x == a_id, b = (int)blockIdx.x == b_id;
  if (!a && !b) return;
  s->where[a ? 0 : 1] = xcc_id();
  const unsigned long long t0 = wall_clock64();
  for (int k = 1; k <= iters; ++k) {
    if (a) st<W>(&s->box[0][0], (unsigned)k);
    unsigned* mine = a ? &s->box[1][0] : &s->box[0][0];
    int spins = 0;
    while (ld<R>(mine) != (unsigned)k) {
      if (++spins > kMaxSpins) { atomicOr(&s->err, 1u); return; }
    }
    if (b) st<W>(&s->box[1][0], (unsigned)k);
  }
  if (a) s->ticks[0] = wall_clock64() - t0;
}

// ---------------------------------------------------------------- grid barriers
// KIND 0: one counter (atomic add, then poll it); 1: one counter per XCD, the last arrival of an
// XCD adds to the top word, everybody polls the top word; 2: one flag per block (a store), the
// first lanes of the block poll all flags side by side.  W / R: scope bits of the flag store and
// of the polling load.  FENCE: agent-scope release before the arrival and acquire after the wait
// (write back / invalidate: what passing ordinary data through the barrier would need).
// only_xcc >= 0: bit mask of the XCDs whose blocks take part (P blocks in all); the others leave.
template <int KIND, int W, int R, bool FENCE>
__global__ __launch_bounds__(kResThreads) void k_barrier(Sync* s, int iters, int only_xcc, int P, int per_xcc, int nxcc) {
  __shared__ int s_rank;
  const unsigned x = xcc_id();
  if (only_xcc >= 0 && !((only_xcc >> x) & 1)) return;   // only_xcc: bit mask of the XCDs that take part
  if (threadIdx.x == 0) s_rank = (int)atomicAdd(&s->ticket, 1u);
  __syncthreads();
  const int rank = s_rank;
  if (rank >= P) return;
  bool dead = false;
  const unsigned long long t0 = wall_clock64();
  for (int k = 1; k <= iters; ++k) {
    __syncthreads();
    const int pollers = KIND == 2 ? ((P + 63) & ~63) : 64;
    if ((int)threadIdx.x < pollers && !dead) {
      if (FENCE) __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      if (KIND == 0) {
        if (threadIdx.x == 0) {
          atomicAdd(&s->top, 1u);
          int spins = 0;
          while ((int)(ld<R>(&s->top) - (unsigned)(k * P)) < 0)
            if (++spins > kMaxSpins) { atomicOr(&s->err, 1u); dead = true; break; }
        }
      } else if (KIND == 1) {
        if (threadIdx.x == 0) {
          const unsigned old = atomicAdd(&s->xc[x & 7][0], 1u);
          if (old + 1u == (unsigned)(k * per_xcc)) atomicAdd(&s->top, 1u);
          int spins = 0;
          while ((int)(ld<R>(&s->top) - (unsigned)(k * nxcc)) < 0)
            if (++spins > kMaxSpins) { atomicOr(&s->err, 1u); dead = true; break; }
        }
      } else {
        // every polling wavefront watches 64 flags, one per lane
        if (threadIdx.x == 0) st<W>(&s->packed[rank], (unsigned)k);
        const int f = (int)threadIdx.x < P ? (int)threadIdx.x : 0;
        int spins = 0;
        while (!__all((int)(ld<R>(&s->packed[f]) - (unsigned)k) >= 0))
          if (++spins > kMaxSpins) { if ((threadIdx.x & 63) == 0) atomicOr(&s->err, 1u); dead = true; break; }
      }
      if (FENCE) __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
    }
  }
  __syncthreads();
  if (rank == 0 && threadIdx.x == 0) s->ticks[0] = wall_clock64() - t0;
}

// ---------------------------------------------------------------- data through a barrier, one XCD
// Block r writes cell t of block (r + 1 + k) mod P (DW 0: store of the expected value with scope
// bits WF; DW 1: atomic add of the increment), waits for its own writes, passes a flag barrier,
// reads its own cells with scope bits RF and compares.  Counts the cells that differ.
template <int DW, int WF, int RF, int BW, int BR>
__global__ __launch_bounds__(kResThreads) void k_pass_data(Sync* s, unsigned* cells, int iters, int only_xcc, int P) {
  __shared__ int s_rank;
  if ((int)xcc_id() != only_xcc) return;
  if (threadIdx.x == 0) s_rank = (int)atomicAdd(&s->ticket, 1u);
  __syncthreads();
  const int rank = s_rank;
  if (rank >= P) return;
  bool dead = false;
  unsigned mism = 0;
  int phase = 0;
  auto barrier = [&]() {
    ++phase;
    __syncthreads();
    if (threadIdx.x < 64 && !dead) {
      if (threadIdx.x == 0) st<BW>(&s->packed[rank], (unsigned)phase);
      int spins = 0;
      for (;;) {
        bool ok = true;
        for (int f = threadIdx.x; f < P; f += 64) ok = ok && (int)(ld<BR>(&s->packed[f]) - (unsigned)phase) >= 0;
        if (__all(ok)) break;
        if (++spins > kMaxSpins) { if (threadIdx.x == 0) atomicOr(&s->err, 1u); dead = true; break; }
      }
    }
    __syncthreads();
  };
  const unsigned long long t0 = wall_clock64();
  unsigned expect = 0;
  for (int k = 1; k <= iters; ++k) {
    const int dst = (rank + 1 + k) % P;
    unsigned* c = &cells[(size_t)dst * kResThreads + threadIdx.x];
    const unsigned inc = (unsigned)k * 2654435761u + threadIdx.x;
    expect += inc;       // (the cell of thread t of every block receives the same increments)
    if (DW == 0) st<WF>(c, expect); else atomicAdd(c, inc);
    wait_vm();
    barrier();
    const unsigned got = ld<RF>(&cells[(size_t)rank * kResThreads + threadIdx.x]);
    if (got != expect) ++mism;
    barrier();
  }
  if (mism) atomicAdd(&s->mism, mism);
  if (rank == 0 && threadIdx.x == 0) s->ticks[0] = wall_clock64() - t0;
}

// ---------------------------------------------------------------- dependent accesses (one lane)
// arr holds a random cycle over its 128-byte lines (word 0 of a line = index of the next line's
// word 0).  KIND 0..4: load with those scope bits; 5: atomic add of `zero` with return value;
// 6: atomic add without return value, then wait for it (the next index comes from a hash).
template <int KIND>
__global__ void k_chase(unsigned* arr, unsigned lines, int warm, int timed, unsigned zero, Sync* s) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  unsigned idx = 0;
  auto hop = [&](int i) {
    if (KIND <= 4) idx = ld<(KIND <= 4 ? KIND : 0)>(&arr[idx]);
    else if (KIND == 5) idx = atomicAdd(&arr[idx], zero);
    else { atomicAdd(&arr[idx + 1], 1u); wait_vm(); idx = (hash32((unsigned)i * 2654435761u + 7u) % lines) * 32u; }
  };
  for (int i = 0; i < warm; ++i) hop(i);
  const unsigned long long t0 = wall_clock64();
  for (int i = 0; i < timed; ++i) hop(warm + i);
  s->ticks[0] = wall_clock64() - t0;
  s->ticks[1] = idx;
}

// ---------------------------------------------------------------- what one XCD streams and scatters
// Every taking-part block (those on the XCDs of the bit mask xmask) streams its share of rows of
// n cells, iters times over rotating rows, four cells per thread in flight.  MODE 0: read a row of
// ints, write a row of floats (non-temporal); 1: read only; 2: write only (non-temporal); 3: write
// only (ordinary stores); 4: read a row, write TWO rows (one non-temporal, one ordinary).
template <int MODE>
__global__ __launch_bounds__(kResThreads) void k_xcd_stream(Sync* s, int* __restrict__ src, float* __restrict__ dst, int n,
                                                           int rows, int iters, int xmask, int P) {
  __shared__ int s_rank;
  if (!((xmask >> xcc_id()) & 1)) return;
  if (threadIdx.x == 0) s_rank = (int)atomicAdd(&s->ticket, 1u);
  __syncthreads();
  const int rank = s_rank;
  if (rank >= P) return;
  const int per = ((n + P - 1) / P + 63) & ~63;
  const int lo = rank * per, hi = lo + per < n ? lo + per : n;
  int sink = 0;
  const unsigned long long t0 = wall_clock64();
  for (int k = 0; k < iters; ++k) {
    int* a = src + (size_t)((k * 7) % rows) * n;
    float* b = dst + (size_t)(k % rows) * n;
    for (int i0 = lo + threadIdx.x; i0 < hi; i0 += 4 * kResThreads) {
      int v[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = i0 + j * kResThreads;
        v[j] = (MODE != 2 && MODE != 3 && i < hi) ? a[i] : k;
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int i = i0 + j * kResThreads;
        if (i < hi) {
          if (MODE == 0 || MODE == 2 || MODE == 4) __builtin_nontemporal_store((float)v[j] * 0x1p-24f, &b[i]);
          if (MODE == 3) b[i] = (float)v[j];
          if (MODE == 4) a[i] = 0;
          if (MODE == 1) sink += v[j];
        }
      }
    }
  }
  if (sink == 0x7fffffff) dst[0] = 1.0f;
  __syncthreads();
  if (rank == 0 && threadIdx.x == 0) s->ticks[0] = wall_clock64() - t0;
}

// MODE 0: every block adds to random cells of the whole array.  MODE 1: the blocks of XCD x add to
// random cells of the x-th eighth only (no cell is touched by two XCDs).  (An atomic add of
// workgroup scope compiles to the same instruction as one of agent scope: there is no third case.)
template <int MODE>
__global__ __launch_bounds__(kResThreads) void k_xcd_atomics(Sync* s, int* cells, unsigned M, int per, int only_xcc, int P) {
  __shared__ int s_rank;
  if (only_xcc >= 0 && (int)xcc_id() != only_xcc) return;
  if (threadIdx.x == 0) s_rank = (int)atomicAdd(&s->ticket, 1u);
  __syncthreads();
  const int rank = s_rank;
  if (rank >= P) return;
  const unsigned slice = M / 8u, base = MODE ? (xcc_id() & 7u) * slice : 0u, span = MODE ? slice : M;
  const unsigned long long t0 = wall_clock64();
  for (int r = 0; r < per; ++r) {
    const unsigned e = ((unsigned)r * P + rank) * kResThreads + threadIdx.x;
    int* cell = &cells[base + hash32(e * 2654435761u + 12345u) % span];
    atomicAdd(cell, 1);
  }
  wait_vm();
  __syncthreads();
  if (threadIdx.x == 0) atomicMax((unsigned long long*)&s->ticks[0], (unsigned long long)(wall_clock64() - t0));
}

__global__ void k_sum_cells(const int* cells, unsigned M, unsigned long long* out) {
  unsigned long long t = 0;
  for (unsigned i = blockIdx.x * blockDim.x + threadIdx.x; i < M; i += gridDim.x * blockDim.x) t += (unsigned)cells[i];
  atomicAdd(out, t);
}

// ---------------------------------------------------------------- a chain of launches without the queue's barrier
// Kernel k of a chain: one thread per block waits (bounded, and not at all once a wait has run
// out) until all nblk blocks of kernel k - 1 have arrived on the per-XCD counters, then the block
// arrives itself.  Launched in stream order these waits are over at once; launched with
// hipExtAnyOrderLaunch the queue may start kernel k while k - 1 still runs, so that the launch
// overhead would hide behind the kernel before -- where the flag is honoured.
__global__ __launch_bounds__(256) void k_chain(Sync* s, unsigned k, unsigned nblk) {
  if (threadIdx.x == 0 && k > 0 && !__hip_atomic_load(&s->err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) {
    const unsigned target = k * nblk;
    int spins = 0;
    for (;;) {
      unsigned sum = 0;
#pragma unroll
      for (int x = 0; x < 8; ++x) sum += __hip_atomic_load(&s->xc[x][0], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if ((int)(sum - target) >= 0) break;
      if (++spins > kMaxSpins) { atomicOr(&s->err, 1u); break; }
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(&s->xc[xcc_id() & 7u][0], 1u);
}

// ---------------------------------------------------------------- host
static const char* kBits[] = {"none", "sc0", "sc1", "sc0 sc1", "nt"};

struct ResCtx {
  Sync* s;
  Sync h;
  hipEvent_t e0, e1;
};

static int res_reset(ResCtx& c) { CK(hipMemset(c.s, 0, sizeof(Sync))); return 0; }
static int res_read(ResCtx& c) { CK(hipMemcpy(&c.h, c.s, sizeof(Sync), hipMemcpyDeviceToHost)); return 0; }

template <int W, int R>
static int res_pingpong(ResCtx& c, int a, int b, const char* what) {
  const int iters = 2000;
  if (res_reset(c)) return 1;
  k_pingpong<W, R><<<16, 64>>>(c.s, a, b, iters);
  CK(hipDeviceSynchronize());
  if (res_read(c)) return 1;
  if (c.h.err) printf("  %-12s store %-8s load %-8s : does not arrive (wait ran out)\n", what, kBits[W], kBits[R]);
  else printf("  %-12s store %-8s load %-8s : %7.0f ns per hand-over (XCD %u -> XCD %u)\n", what, kBits[W], kBits[R],
              (double)c.h.ticks[0] * 10.0 / (2.0 * iters), c.h.where[0], c.h.where[1]);
  return 0;
}

template <int KIND, int W, int R, bool FENCE>
static int res_barrier(ResCtx& c, int grid, int only_xcc, int P, const char* what) {
  const int iters = 2000;
  float ms = 0;
  if (res_reset(c)) return 1;
  CK(hipEventRecord(c.e0));
  k_barrier<KIND, W, R, FENCE><<<grid, kResThreads>>>(c.s, iters, only_xcc, P, P / 8, 8);
  CK(hipEventRecord(c.e1)); CK(hipEventSynchronize(c.e1)); CK(hipEventElapsedTime(&ms, c.e0, c.e1));
  if (res_read(c)) return 1;
  if (c.h.err) printf("  %-58s: a wait ran out\n", what);
  else printf("  %-58s: %6.2f us per barrier (kernel %.2f ms)\n", what, (double)c.h.ticks[0] * 0.01 / iters, ms);
  return 0;
}

template <int DW, int WF, int RF, int BW, int BR>
static int res_pass(ResCtx& c, unsigned* cells, int P, const char* what) {
  const int iters = 1000;
  if (res_reset(c)) return 1;
  CK(hipMemset(cells, 0, (size_t)P * kResThreads * 4));
  k_pass_data<DW, WF, RF, BW, BR><<<256, kResThreads>>>(c.s, cells, iters, 0, P);
  CK(hipDeviceSynchronize());
  if (res_read(c)) return 1;
  if (c.h.err) printf("  %-64s: a wait ran out\n", what);
  else printf("  %-64s: %8u of %d cells differ, %6.2f us per round (write, barrier, read, barrier)\n", what, c.h.mism,
              iters * P * kResThreads, (double)c.h.ticks[0] * 0.01 / iters);
  return 0;
}

template <int KIND>
static int res_chase(ResCtx& c, unsigned* arr, unsigned lines, int warm, int timed, const char* what) {
  if (res_reset(c)) return 1;
  k_chase<KIND><<<1, 64>>>(arr, lines, warm, timed, 0u, c.s);
  CK(hipDeviceSynchronize());
  if (res_read(c)) return 1;
  printf("  %-60s: %7.0f ns per access\n", what, (double)c.h.ticks[0] * 10.0 / timed);
  return 0;
}

static int make_cycle(unsigned* d_arr, unsigned lines) {
  std::vector<unsigned> perm(lines), h((size_t)lines * 32, 0u);
  for (unsigned i = 0; i < lines; ++i) perm[i] = i;
  unsigned long long z = 88172645463325252ull;
  for (unsigned i = lines - 1; i > 0; --i) {
    z ^= z << 13; z ^= z >> 7; z ^= z << 17;
    const unsigned j = (unsigned)(z % (i + 1));
    const unsigned t = perm[i]; perm[i] = perm[j]; perm[j] = t;
  }
  for (unsigned i = 0; i < lines; ++i) h[(size_t)perm[i] * 32] = perm[(i + 1) % lines] * 32u;
  CK(hipMemcpy(d_arr, h.data(), (size_t)lines * 128, hipMemcpyHostToDevice));
  return 0;
}

static int resident_main() {
  ResCtx c;
  CK(hipMalloc(&c.s, sizeof(Sync)));
  CK(hipEventCreate(&c.e0)); CK(hipEventCreate(&c.e1));

  printf("where the blocks of a 256 x 1024-thread grid run (XCD of block b, by b mod 8):\n");
  if (res_reset(c)) return 1;
  k_where<<<256, kResThreads>>>(c.s);
  CK(hipDeviceSynchronize());
  if (res_read(c)) return 1;
  {
    int tab[8][8] = {};
    for (int b = 0; b < 256; ++b) tab[b & 7][c.h.where[2 * b] & 7] += 1;
    bool rr = true;
    for (int r = 0; r < 8; ++r)
      for (int x = 0; x < 8; ++x) if ((x == r) != (tab[r][x] == 32)) rr = false;
    for (int r = 0; r < 8; ++r) {
      printf("  b mod 8 = %d:", r);
      for (int x = 0; x < 8; ++x) printf(" %3d", tab[r][x]);
      printf("\n");
    }
    printf("  block b runs on XCD b mod 8: %s\n", rr ? "yes" : "NO");
  }

  printf("hand-over of one word between two single-wavefront blocks (store by one, polling load by the other):\n");
  // same XCD: blocks 0 and 8; two XCDs: blocks 0 and 1
  if (res_pingpong<0, 0>(c, 0, 8, "one XCD")) return 1;
  if (res_pingpong<0, 1>(c, 0, 8, "one XCD")) return 1;
  if (res_pingpong<1, 1>(c, 0, 8, "one XCD")) return 1;
  if (res_pingpong<0, 2>(c, 0, 8, "one XCD")) return 1;
  if (res_pingpong<2, 2>(c, 0, 8, "one XCD")) return 1;
  if (res_pingpong<3, 3>(c, 0, 8, "one XCD")) return 1;
  if (res_pingpong<0, 4>(c, 0, 8, "one XCD")) return 1;
  if (res_pingpong<1, 1>(c, 0, 1, "two XCDs")) return 1;
  if (res_pingpong<2, 2>(c, 0, 1, "two XCDs")) return 1;
  if (res_pingpong<0, 2>(c, 0, 1, "two XCDs")) return 1;
  if (res_pingpong<3, 3>(c, 0, 1, "two XCDs")) return 1;

  printf("grid barriers, 1024-thread blocks, 2000 in a row (time inside the kernel, per barrier):\n");
  if (res_barrier<0, 2, 2, false>(c, 64, -1, 64, "64 blocks, one counter, poll sc1")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 128, -1, 128, "128 blocks, one counter, poll sc1")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 256, -1, 256, "256 blocks, one counter, poll sc1")) return 1;
  if (res_barrier<0, 2, 2, true>(c, 256, -1, 256, "256 blocks, one counter, poll sc1, release/acquire fences")) return 1;
  if (res_barrier<1, 2, 2, false>(c, 64, -1, 64, "64 blocks, counter per XCD + top word, poll sc1")) return 1;
  if (res_barrier<1, 2, 2, false>(c, 256, -1, 256, "256 blocks, counter per XCD + top word, poll sc1")) return 1;
  if (res_barrier<1, 2, 2, true>(c, 256, -1, 256, "256 blocks, counter per XCD + top word, poll sc1, fences")) return 1;
  if (res_barrier<2, 2, 2, false>(c, 64, -1, 64, "64 blocks, flag per block, sc1 store / sc1 load")) return 1;
  if (res_barrier<2, 2, 2, false>(c, 256, -1, 256, "256 blocks, flag per block, sc1 store / sc1 load")) return 1;
  if (res_barrier<2, 2, 2, true>(c, 256, -1, 256, "256 blocks, flag per block, sc1 / sc1, fences")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 256, 1, 32, "32 blocks of ONE XCD, one counter, poll sc1")) return 1;
  if (res_barrier<2, 2, 2, false>(c, 256, 1, 32, "32 blocks of ONE XCD, flag per block, sc1 / sc1")) return 1;
  if (res_barrier<2, 1, 1, false>(c, 256, 1, 32, "32 blocks of ONE XCD, flag per block, sc0 / sc0")) return 1;
  if (res_barrier<2, 0, 1, false>(c, 256, 1, 32, "32 blocks of ONE XCD, flag per block, none / sc0")) return 1;
  if (res_barrier<2, 0, 0, false>(c, 256, 1, 32, "32 blocks of ONE XCD, flag per block, none / none")) return 1;
  if (res_barrier<2, 1, 1, false>(c, 128, 1, 16, "16 blocks of ONE XCD, flag per block, sc0 / sc0")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 128, 1, 16, "16 blocks of ONE XCD, one counter, poll sc1")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 64, 1, 8, "8 blocks of ONE XCD, one counter, poll sc1")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 256, 3, 64, "64 blocks of TWO XCDs, one counter, poll sc1")) return 1;
  if (res_barrier<2, 2, 2, false>(c, 256, 3, 64, "64 blocks of TWO XCDs, flag per block, sc1 / sc1")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 128, 3, 32, "32 blocks of TWO XCDs, one counter, poll sc1")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 256, 15, 128, "128 blocks of FOUR XCDs, one counter, poll sc1")) return 1;
  if (res_barrier<0, 2, 2, false>(c, 128, 15, 64, "64 blocks of FOUR XCDs, one counter, poll sc1")) return 1;

  printf("data through a flag barrier, 32 blocks of ONE XCD, 1024 cells each (1000 rounds):\n");
  {
    unsigned* cells = nullptr;
    CK(hipMalloc(&cells, 32 * kResThreads * 4));
    if (res_pass<0, 0, 0, 1, 1>(c, cells, 32, "store none, read none, barrier sc0/sc0")) return 1;
    if (res_pass<0, 0, 1, 1, 1>(c, cells, 32, "store none, read sc0, barrier sc0/sc0")) return 1;
    if (res_pass<0, 1, 1, 1, 1>(c, cells, 32, "store sc0, read sc0, barrier sc0/sc0")) return 1;
    if (res_pass<0, 0, 4, 1, 1>(c, cells, 32, "store none, read nt, barrier sc0/sc0")) return 1;
    if (res_pass<0, 2, 2, 2, 2>(c, cells, 32, "store sc1, read sc1, barrier sc1/sc1")) return 1;
    if (res_pass<1, 0, 0, 1, 1>(c, cells, 32, "atomic add, read none, barrier sc0/sc0")) return 1;
    if (res_pass<1, 0, 1, 1, 1>(c, cells, 32, "atomic add, read sc0, barrier sc0/sc0")) return 1;
    if (res_pass<1, 0, 2, 1, 1>(c, cells, 32, "atomic add, read sc1, barrier sc0/sc0")) return 1;
    if (res_pass<1, 0, 2, 2, 2>(c, cells, 32, "atomic add, read sc1, barrier sc1/sc1")) return 1;
    CK(hipFree(cells));
  }

  printf("dependent accesses of one lane (a random cycle over 128-byte lines):\n");
  {
    unsigned* arr = nullptr;
    const unsigned big = 1u << 23;   // 1 GiB of lines
    CK(hipMalloc(&arr, (size_t)big * 128));
    if (make_cycle(arr, 8192)) return 1;
    if (res_chase<0>(c, arr, 8192, 8192, 8192, "1 MB, load, second pass")) return 1;
    if (res_chase<1>(c, arr, 8192, 8192, 8192, "1 MB, load sc0, second pass")) return 1;
    if (res_chase<2>(c, arr, 8192, 8192, 8192, "1 MB, load sc1, second pass")) return 1;
    if (res_chase<3>(c, arr, 8192, 8192, 8192, "1 MB, load sc0 sc1, second pass")) return 1;
    if (res_chase<5>(c, arr, 8192, 8192, 8192, "1 MB, atomic add with return value, second pass")) return 1;
    if (res_chase<6>(c, arr, 8192, 8192, 8192, "1 MB, atomic add without return value + wait")) return 1;
    if (make_cycle(arr, 1u << 19)) return 1;
    if (res_chase<0>(c, arr, 1u << 19, 1 << 19, 8192, "64 MB, load, lines touched 64 MB ago")) return 1;
    if (res_chase<2>(c, arr, 1u << 19, 1 << 19, 8192, "64 MB, load sc1, lines touched 64 MB ago")) return 1;
    if (res_chase<5>(c, arr, 1u << 19, 1 << 19, 8192, "64 MB, atomic add with return value, touched 64 MB ago")) return 1;
    if (make_cycle(arr, big)) return 1;
    if (res_chase<0>(c, arr, big, 0, 8192, "1 GB, load, first touch")) return 1;
    if (res_chase<2>(c, arr, big, 0, 8192, "1 GB, load sc1, first touch")) return 1;
    if (res_chase<5>(c, arr, big, 0, 8192, "1 GB, atomic add with return value, first touch")) return 1;
    CK(hipFree(arr));
  }

  printf("streaming by the blocks of one, two, four and all XCDs (rows of 100,000 4-byte cells, 2000 rows, four cells per thread in flight):\n");
  {
    const int n = 100000, rows = 256, iters = 2000;
    int* src = nullptr; float* dst = nullptr;
    CK(hipMalloc(&src, (size_t)n * rows * 4)); CK(hipMalloc(&dst, (size_t)n * rows * 4));
    CK(hipMemset(src, 0, (size_t)n * rows * 4));
    const int cfgs[][3] = {{256, 0x1, 32}, {512, 0x1, 64}, {256, 0x3, 64}, {256, 0xf, 128}, {256, 0xff, 256}};
    const char* mode_name[] = {"read 4 B + write 4 B (nt)", "read 4 B", "write 4 B (nt)", "write 4 B", "read 4 B + write 4 B (nt) + write 4 B"};
    const double bytes[] = {8.0, 4.0, 4.0, 4.0, 12.0};
    for (int mode = 0; mode < 5; ++mode)
      for (auto& g : cfgs) {
        if (res_reset(c)) return 1;
        if (mode == 0) k_xcd_stream<0><<<g[0], kResThreads>>>(c.s, src, dst, n, rows, iters, g[1], g[2]);
        else if (mode == 1) k_xcd_stream<1><<<g[0], kResThreads>>>(c.s, src, dst, n, rows, iters, g[1], g[2]);
        else if (mode == 2) k_xcd_stream<2><<<g[0], kResThreads>>>(c.s, src, dst, n, rows, iters, g[1], g[2]);
        else if (mode == 3) k_xcd_stream<3><<<g[0], kResThreads>>>(c.s, src, dst, n, rows, iters, g[1], g[2]);
        else k_xcd_stream<4><<<g[0], kResThreads>>>(c.s, src, dst, n, rows, iters, g[1], g[2]);
        CK(hipDeviceSynchronize());
        if (res_read(c)) return 1;
        const double us = (double)c.h.ticks[0] * 0.01 / iters;
        int nx = 0; for (int b = 0; b < 8; ++b) nx += (g[1] >> b) & 1;
        printf("  %-40s %3d blocks on %d XCD(s): %6.2f us per row, %6.0f GB/s\n", mode_name[mode], g[2], nx, us,
               bytes[mode] * n / us / 1e3);
      }
    CK(hipFree(src)); CK(hipFree(dst));
  }

  printf("random atomic adds by the blocks of ONE XCD and of all (64 per thread; time of the slowest block):\n");
  {
    const unsigned Ms[] = {200000u, 1600000u};
    unsigned long long* total = nullptr;
    CK(hipMalloc(&total, 8));
    for (unsigned M : Ms) {
      int* cells = nullptr;
      CK(hipMalloc(&cells, (size_t)M * 4));
      const int cfgs[][4] = {{256, 0, 32, 0}, {256, 0, 32, 1}, {256, -1, 256, 0}, {256, -1, 256, 1}};
      const char* what[] = {"anywhere", "own eighth per XCD"};
      for (auto& g : cfgs) {
        if (res_reset(c)) return 1;
        CK(hipMemset(cells, 0, (size_t)M * 4)); CK(hipMemset(total, 0, 8));
        if (g[3] == 0) k_xcd_atomics<0><<<g[0], kResThreads>>>(c.s, cells, M, 64, g[1], g[2]);
        else k_xcd_atomics<1><<<g[0], kResThreads>>>(c.s, cells, M, 64, g[1], g[2]);
        CK(hipDeviceSynchronize());
        k_sum_cells<<<256, 256>>>(cells, M, total);
        CK(hipDeviceSynchronize());
        if (res_read(c)) return 1;
        unsigned long long got = 0;
        CK(hipMemcpy(&got, total, 8, hipMemcpyDeviceToHost));
        const unsigned long long want = 64ull * g[2] * kResThreads;
        const double us = (double)c.h.ticks[0] * 0.01;
        printf("  %.1f MB of cells, %3d blocks %-12s %-19s: %8.1f us, %6.2f G adds/s, sum of the cells %s\n", M * 4 / 1e6, g[2],
               g[1] >= 0 ? "of one XCD," : "(all XCDs),", what[g[3]], us, 64.0 * g[2] * kResThreads / us / 1e3,
               got == want ? "right" : "WRONG");
      }
      CK(hipFree(cells));
    }
    CK(hipFree(total));
  }
  printf("chain of 1000 dependent kernels, 391 x 256 threads, each waiting in its first thread for the arrivals of the one before:\n");
  for (int any = 0; any < 2; ++any) {
    if (res_reset(c)) return 1;
    const unsigned nblk = 391;
    for (int rep = 0; rep < 2; ++rep) {
      if (res_reset(c)) return 1;
      CK(hipEventRecord(c.e0));
      for (unsigned k = 0; k < 1000; ++k) {
        if (any) hipExtLaunchKernelGGL(k_chain, dim3(nblk), dim3(256), 0, 0, nullptr, nullptr, hipExtAnyOrderLaunch, c.s, k, nblk);
        else k_chain<<<nblk, 256>>>(c.s, k, nblk);
      }
      CK(hipEventRecord(c.e1));
      CK(hipDeviceSynchronize());
    }
    float ms = 0;
    CK(hipEventElapsedTime(&ms, c.e0, c.e1));
    if (res_read(c)) return 1;
    unsigned total = 0;
    for (int x = 0; x < 8; ++x) total += c.h.xc[x][0];
    printf("  %-44s: %6.2f us per kernel%s, arrivals %s\n", any ? "launched with hipExtAnyOrderLaunch" : "launched in stream order",
           ms, c.h.err ? " (A WAIT RAN OUT)" : "", total == 1000u * nblk ? "complete" : "INCOMPLETE");
  }
  printf("the same chain dealt out over two streams in turn (no barrier between the queues; the kernels' own waits order them):\n");
  {
    hipStream_t two[2];
    CK(hipStreamCreateWithFlags(&two[0], hipStreamNonBlocking));
    CK(hipStreamCreateWithFlags(&two[1], hipStreamNonBlocking));
    const unsigned nblk = 391;
    double us = 0, host_us = 0;
    for (int rep = 0; rep < 3; ++rep) {
      if (res_reset(c)) return 1;
      CK(hipDeviceSynchronize());
      const auto t0 = std::chrono::steady_clock::now();
      for (unsigned k = 0; k < 1000; ++k) k_chain<<<nblk, 256, 0, two[k & 1]>>>(c.s, k, nblk);
      const auto t1 = std::chrono::steady_clock::now();
      CK(hipStreamSynchronize(two[0])); CK(hipStreamSynchronize(two[1]));
      const auto t2 = std::chrono::steady_clock::now();
      host_us = std::chrono::duration<double, std::micro>(t1 - t0).count() / 1000.0;
      us = std::chrono::duration<double, std::micro>(t2 - t0).count() / 1000.0;
    }
    if (res_read(c)) return 1;
    unsigned total = 0;
    for (int x = 0; x < 8; ++x) total += c.h.xc[x][0];
    printf("  two streams in turn                         : %6.2f us per kernel by the host's clock (the host needs %.2f us to enqueue one)%s, arrivals %s\n",
           us, host_us, c.h.err ? " (A WAIT RAN OUT)" : "", total == 1000u * nblk ? "complete" : "INCOMPLETE");
    // the same with both queues filled beforehand: a kernel holds each stream for 8 ms in front of the chain, the host enqueues
    // everything meanwhile, and the events bracket what the GPU then needs by itself
    float ms = 0;
    for (int rep = 0; rep < 2; ++rep) {
      if (res_reset(c)) return 1;
      CK(hipDeviceSynchronize());
      k_hold<<<1, 64, 0, two[0]>>>(800000ull);
      k_hold<<<1, 64, 0, two[1]>>>(800000ull);
      CK(hipEventRecord(c.e0, two[1]));
      for (unsigned k = 0; k < 1000; ++k) k_chain<<<nblk, 256, 0, two[k & 1]>>>(c.s, k, nblk);
      CK(hipEventRecord(c.e1, two[1]));
      CK(hipStreamSynchronize(two[0])); CK(hipStreamSynchronize(two[1]));
      CK(hipEventElapsedTime(&ms, c.e0, c.e1));
    }
    if (res_read(c)) return 1;
    total = 0;
    for (int x = 0; x < 8; ++x) total += c.h.xc[x][0];
    printf("  two streams in turn, queues filled beforehand: %6.2f us per kernel on the GPU%s, arrivals %s\n", ms,
           c.h.err ? " (A WAIT RAN OUT)" : "", total == 1000u * nblk ? "complete" : "INCOMPLETE");
    // and one stream, in order, filled beforehand, for comparison
    for (int rep = 0; rep < 2; ++rep) {
      if (res_reset(c)) return 1;
      CK(hipDeviceSynchronize());
      k_hold<<<1, 64, 0, two[0]>>>(800000ull);
      CK(hipEventRecord(c.e0, two[0]));
      for (unsigned k = 0; k < 1000; ++k) k_chain<<<nblk, 256, 0, two[0]>>>(c.s, k, nblk);
      CK(hipEventRecord(c.e1, two[0]));
      CK(hipStreamSynchronize(two[0]));
      CK(hipEventElapsedTime(&ms, c.e0, c.e1));
    }
    printf("  one stream, queue filled beforehand          : %6.2f us per kernel on the GPU\n", ms);
    CK(hipStreamDestroy(two[0])); CK(hipStreamDestroy(two[1]));
  }
  CK(hipFree(c.s));
  return 0;
}
