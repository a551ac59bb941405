// `chip_rates exchange`: what one time step costs a kernel that stays resident on the WHOLE chip
// when the only thing that crosses blocks on the critical path is the step's spike words.
// Included by chip_rates.hip (after resident_rates.h, whose access helpers it uses).
//
// Per round every block stores its share of NW 32-bit words (agent-scope stores), waits for them,
// arrives on the counter of its XCD (an atomic add without return value), one wavefront polls the
// eight counters side by side (agent-scope loads, one counter per lane) until their sum says that
// everybody has arrived, and then all threads of the block read ALL the words (agent-scope 16-byte
// loads) and check them.  The words are double-buffered by round, so a block that is a round ahead
// never overwrites what a slower block still reads.  Every wait is a bounded spin.

template <int TPB>
__device__ __forceinline__ bool wait_arrivals(Sync* s, unsigned target, bool& dead) {
  // called by wavefront 0 of the block; lanes 0..7 each watch one counter
  if (dead) return false;
  const int lane = threadIdx.x & 63;
  int spins = 0;
  for (;;) {
    unsigned v = lane < 8 ? ld<2>(&s->xc[lane][0]) : 0u;
    v += __shfl_xor(v, 1); v += __shfl_xor(v, 2); v += __shfl_xor(v, 4);
    const unsigned sum = __shfl(v, 0);
    if ((int)(sum - target) >= 0) return true;
    if (++spins > kMaxSpins) { if (lane == 0) atomicOr(&s->err, 1u); dead = true; return false; }
  }
}

// MODE 0: arrival + wait only.  1: + the block's words stored before and all words read after.
// 2: as 1, and every thread also adds to 2 random cells (atomics without return, waited for before
// the arrival) and reads its own 4-byte cell after the wait (agent scope): the traffic of a step.
template <int TPB, int MODE>
__global__ __launch_bounds__(TPB) void k_exchange(Sync* s, unsigned* words, int NW, int* cells, int ncell, int iters, int P) {
  __shared__ int s_rank;
  if (threadIdx.x == 0) s_rank = (int)atomicAdd(&s->ticket, 1u);
  __syncthreads();
  const int rank = s_rank;
  if (rank >= P) return;
  const unsigned x = xcc_id() & 7u;
  const int per = (NW + P - 1) / P;
  const int lo = rank * per, hi = lo + per < NW ? lo + per : NW;
  bool dead = false;
  unsigned mism = 0, sink = 0;
  const unsigned long long t0 = wall_clock64();
  for (int k = 1; k <= iters; ++k) {
    unsigned* buf = words + (size_t)(k & 1) * NW;
    if (MODE >= 1) {
      const int i = lo + (int)threadIdx.x;
      if (i < hi) st<2>(&buf[i], hash32((unsigned)k * 0x9E3779B9u + (unsigned)i));
    }
    if (MODE == 2) {
      // 2 scattered adds per thread for the first 8 threads of every wavefront: ~6,000 per round over the chip
      if ((threadIdx.x & 63) < 8) {
        const unsigned e = ((unsigned)k * P + rank) * TPB + threadIdx.x;
        atomicAdd(&cells[hash32(e * 2654435761u + 1u) % (unsigned)ncell], 1);
        atomicAdd(&cells[hash32(e * 2654435761u + 2u) % (unsigned)ncell], 1);
      }
    }
    wait_vm();
    __syncthreads();
    if (threadIdx.x < 64) {
      if (threadIdx.x == 0) atomicAdd(&s->xc[x][0], 1u);
      wait_arrivals<TPB>(s, (unsigned)k * (unsigned)P, dead);
    }
    __syncthreads();
    if (MODE >= 1) {
      for (int i = 4 * (int)threadIdx.x; i < NW; i += 4 * TPB) {
        unsigned v0, v1, v2, v3;
        if (i + 3 < NW) {
          uint4 v;
          asm volatile("global_load_dwordx4 %0, %1, off sc1\n s_waitcnt vmcnt(0)" : "=v"(v) : "v"(&buf[i]) : "memory");
          v0 = v.x; v1 = v.y; v2 = v.z; v3 = v.w;
          if (v0 != hash32((unsigned)k * 0x9E3779B9u + (unsigned)i)) ++mism;
          if (v1 != hash32((unsigned)k * 0x9E3779B9u + (unsigned)i + 1u)) ++mism;
          if (v2 != hash32((unsigned)k * 0x9E3779B9u + (unsigned)i + 2u)) ++mism;
          if (v3 != hash32((unsigned)k * 0x9E3779B9u + (unsigned)i + 3u)) ++mism;
        } else {
          for (int j = i; j < NW; ++j)
            if (ld<2>(&buf[j]) != hash32((unsigned)k * 0x9E3779B9u + (unsigned)j)) ++mism;
        }
      }
    }
    if (MODE == 2) {
      const int c = rank * TPB + (int)threadIdx.x;
      if (c < ncell) sink += (unsigned)ld<2>((const unsigned*)&cells[c]);
    }
  }
  if (mism) atomicAdd(&s->mism, mism);
  if (sink == 0x7fffffffu) cells[0] = 1;
  __syncthreads();
  if (rank == 0 && threadIdx.x == 0) s->ticks[0] = wall_clock64() - t0;
}

template <int TPB, int MODE>
static int exch_run(ResCtx& c, unsigned* words, int NW, int* cells, int ncell, int P, const char* what) {
  const int iters = 2000;
  for (int rep = 0; rep < 2; ++rep) {
    if (res_reset(c)) return 1;
    k_exchange<TPB, MODE><<<P, TPB>>>(c.s, words, NW, cells, ncell, iters, P);
    CK(hipDeviceSynchronize());
  }
  if (res_read(c)) return 1;
  if (c.h.err) printf("  %4d blocks x %4d threads, %-52s: a wait ran out\n", P, TPB, what);
  else printf("  %4d blocks x %4d threads, %-52s: %6.2f us per round, %u words wrong\n", P, TPB, what,
              (double)c.h.ticks[0] * 0.01 / iters, c.h.mism);
  return 0;
}

static int exchange_main() {
  ResCtx c;
  CK(hipMalloc(&c.s, sizeof(Sync)));
  CK(hipEventCreate(&c.e0)); CK(hipEventCreate(&c.e1));
  const int NW = 3128, ncell = 100096;    // the spike words and the cells of 100,000 neurons
  unsigned* words = nullptr; int* cells = nullptr;
  CK(hipMalloc(&words, (size_t)2 * NW * 4)); CK(hipMalloc(&cells, (size_t)ncell * 4));
  CK(hipMemset(words, 0, (size_t)2 * NW * 4)); CK(hipMemset(cells, 0, (size_t)ncell * 4));
  printf("rounds of a kernel resident on the whole chip (arrive on the XCD's counter, one wavefront polls the 8 counters; 2000 rounds):\n");
  const char* names[] = {"arrival + wait only", "+ own words stored, all 3,128 words read", "+ 6,000 scattered adds, own cell read"};
#define EXCH(TPB, P) \
  if (exch_run<TPB, 0>(c, words, NW, cells, ncell, P, names[0])) return 1; \
  if (exch_run<TPB, 1>(c, words, NW, cells, ncell, P, names[1])) return 1; \
  if (exch_run<TPB, 2>(c, words, NW, cells, ncell, P, names[2])) return 1;
  EXCH(256, 64)
  EXCH(256, 128)
  EXCH(256, 256)
  EXCH(256, 391)
  EXCH(512, 196)
  EXCH(512, 256)
  EXCH(1024, 98)
  EXCH(1024, 256)
#undef EXCH
  CK(hipFree(words)); CK(hipFree(cells)); CK(hipFree(c.s));
  return 0;
}
