// Ring queue: the time steps of one window in ONE launch ("resident" step kernels).  Included by
// adseq.hip after ring_window.h.
//
// A launch per time step costs 4 us for 2 MB of work: 2.4 us of launch and, inside, a chain of
// dependent trips to memory.  What the chip offers instead (measured by `chip_rates resident`): a grid barrier over all 256 compute units costs as much as the launch it would
// replace (2.1 us at best), but the 32 compute units of ONE XCD, which share an L2, pass a barrier
// in 0.7 us and read each other's atomic adds and stores back from that L2 in 0.1 us.  So the steps
// of a window run in one launch on the blocks of one XCD: block b of the grid runs on XCD b mod 8,
// and only the blocks with b mod 8 = 0 take part (the others leave at once).  Each taking-part block
// owns a contiguous range of neurons for the whole launch and keeps what does not change, or only
// it changes, in registers: membrane state, row bounds, the step-independent half of the drive's
// hash.  Per step the cells of the window row are read with agent-scope loads (they hit in the
// shared L2; the adds of other blocks are atomics, which every scope sees), and a step ends with a
// barrier on one counter: the adds of a step's spikes are acknowledged before the block arrives.
// Nothing here depends on WHERE the blocks run for its results -- atomics, agent-scope loads and
// the counter are coherent over the whole chip -- only the speed does.
//
// Every wait is a bounded spin: a wait that runs out sets ERR_BARRIER in the device error word
// and the block stops waiting for the rest of the launch, so every block reaches the end of the
// kernel whatever happens (the results are then void, and the host reports the error).

constexpr int kResThreads = 1024;
constexpr int kResBlocks = 32;        // taking-part blocks at most: the compute units of one XCD
constexpr int kResStride = 8;         // XCDs: block b runs on XCD b mod 8
constexpr int kResMaxSpins = 1 << 22;

__device__ __forceinline__ int ld_agent(const int* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ unsigned ld_agent(const unsigned* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float ld_agent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_agent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void wait_all_memory() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

// Barrier number `target / P` of the launch sequence over the P taking-part blocks: every
// wavefront has waited for its own memory operations; thread 0 adds the block's arrival and polls
// the counter.  *dead (shared) is set when the wait runs out.
__device__ __forceinline__ void res_arrive(const Dev& d) {
  wait_all_memory();
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(&d.ctr->bar[0], 1u);
}
__device__ __forceinline__ void res_wait(const Dev& d, unsigned target, int* dead) {
  if (threadIdx.x == 0 && !*dead) {
    int spins = 0;
    while ((int)(ld_agent(&d.ctr->bar[0]) - target) < 0) {
      if (++spins > kResMaxSpins) { atomicOr(&d.ctr->err, ERR_BARRIER); *dead = 1; break; }
    }
  }
  __syncthreads();
}

// Steps n0 .. n0 + nsteps - 1 of the closed loop, all inside one window (no window boundary is
// crossed: the host expands the next window between two launches).  P taking-part blocks; block
// `rank` owns neurons [rank * chunk, rank * chunk + chunk) (chunk a multiple of 64, at most
// NPT * 1024), thread t the neurons rank * chunk + j * 1024 + t.  bar_base: value of the barrier
// counter when the launch begins.  Same arithmetic, in the same order, as k_step_win.
template <bool RECORD, int SYN, int NPT>
__global__ __launch_bounds__(kResThreads) void k_run_xcd(long long n0, int nsteps, unsigned bar_base, int P,
                                                         int chunk, Dev d) {
  __shared__ int s_dead;
  if (blockIdx.x % kResStride) return;
  const int rank = blockIdx.x / kResStride;
  if (rank >= P) return;
  if (threadIdx.x == 0) s_dead = 0;
  const int lane = threadIdx.x & 63;
  const int lo = rank * chunk;
  const int hi = lo + chunk < d.BN ? lo + chunk : d.BN;
  // what stays in registers for the whole launch
  int g[NPT], base[NPT], rlen[NPT];
  bool act[NPT];
  long long r0[NPT];
  unsigned long long h0[NPT];
  float V[NPT], J[NPT], Jf[NPT];
#pragma unroll
  for (int j = 0; j < NPT; ++j) {
    g[j] = lo + j * kResThreads + (int)threadIdx.x;
    act[j] = g[j] < hi;
    base[j] = 0; rlen[j] = 0; r0[j] = 0; h0[j] = 0; V[j] = 0.0f; J[j] = 0.0f; Jf[j] = 0.0f;
    if (act[j]) {
      const int b = trial_of(d, g[j]);
      const int i = g[j] - b * d.N;
      base[j] = b * d.N;
      r0[j] = d.row_ptr[i];
      rlen[j] = (int)(d.row_ptr[i + 1] - r0[j]);
      h0[j] = mix64(d.seed + 0x9E3779B97F4A7C15ull * ((unsigned long long)g[j] + 1ull));
      V[j] = d.V[g[j]];
      if (SYN) J[j] = d.J[g[j]];
      if (SYN == 2) Jf[j] = d.J[(size_t)d.BN + g[j]];
    }
  }
  __syncthreads();
  for (int k = 0; k < nsteps; ++k) {
    const long long n = n0 + k;
    const int phi = (int)(n & (long long)(d.W - 1));
    int near_h = d.W - 1 - phi;
    if (near_h > d.d_max) near_h = d.d_max;
    int* __restrict__ win = win_of(d, n);
    // the adds of step n - 1 are in place once every block has arrived
    if (k > 0) res_wait(d, bar_base + (unsigned)k * (unsigned)P, &s_dead);
    int acc[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) acc[j] = act[j] ? ld_agent(&win[(size_t)phi * d.BN + g[j]]) : 0;
    bool s[NPT];
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      s[j] = false;
      if (act[j]) {
        if (acc[j] != 0) win[(size_t)phi * d.BN + g[j]] = 0;
        float I = (float)acc[j] * 0x1p-24f;
        if (SYN) {
          const float jump = I;
          I = __fmaf_rn(d.alpha_s, J[j], jump);
          J[j] = I;
          if (SYN == 2) {
            const float fast = __fmaf_rn(d.alpha_r, Jf[j], jump);
            Jf[j] = fast;
            I = I - fast;
          }
        }
        if (d.p_thresh) {
          const unsigned long long z = mix64(h0[j] + 0x9E3779B97F4A7C15ull * ((unsigned long long)n + 1ull));
          const bool xi = (unsigned long long)(unsigned)(z >> 32) < d.p_thresh;
          I = I + (xi ? d.ext_w : 0.0f);
        }
        const float U = __fmaf_rn(d.alpha, V[j], I);
        s[j] = U >= d.theta;
        V[j] = s[j] ? d.v_reset : U;
        if (RECORD) {
          __builtin_nontemporal_store(U, &d.tapeU[(size_t)n * d.BN + g[j]]);
          if (s[j]) atomicAdd(&d.spk_count[g[j]], 1);
        }
      }
    }
    // spike words of the step, and the in-window events of the spikes: the front of the sorted
    // row, entries with arrival offset <= near_h (the rows are ascending in the offset, so a
    // wavefront reads 64 entries at a time until one lies beyond)
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      const unsigned long long bits = __ballot(s[j]);
      const int word = (lo >> 6) + j * (kResThreads / 64) + ((int)threadIdx.x >> 6);
      // (a thread's later neurons may lie beyond the block's range: those words are the next block's)
      if (lane == 0 && lo + j * kResThreads + ((int)threadIdx.x & ~63) < lo + chunk && word < d.words) {
        d.spike_bits[(size_t)(n % d.R) * d.words + word] = bits;
        if (RECORD) d.tape_bits[(size_t)n * d.words + word] = bits;
      }
      unsigned long long m = near_h >= 1 ? __ballot(s[j] && rlen[j] > 0) : 0ull;
      while (m) {
        const int L = __ffsll((long long)m) - 1;
        m &= m - 1;
        const long long pr = lane_get(r0[j], L);
        const int len = lane_get(rlen[j], L), bs = lane_get(base[j], L);
        for (int q0 = 0; q0 < len; q0 += 64) {
          bool more = false;
          if (q0 + lane < len) {
            const uint2 e = d.synf[pr + q0 + lane];
            const int D = (int)(e.x & d.dmask);
            if (D <= near_h) {
              atomicAdd(&win[(size_t)(phi + D) * d.BN + (size_t)bs + (e.x >> d.dbits)], (int)e.y);
              more = true;
            }
          }
          // the next 64 entries only if this group's last one was still inside the window
          if (!(__ballot(more) >> 63)) break;
        }
      }
    }
    if (k + 1 < nsteps) res_arrive(d);
  }
#pragma unroll
  for (int j = 0; j < NPT; ++j)
    if (act[j]) {
      d.V[g[j]] = V[j];
      if (SYN) d.J[g[j]] = J[j];
      if (SYN == 2) d.J[(size_t)d.BN + g[j]] = Jf[j];
    }
}
