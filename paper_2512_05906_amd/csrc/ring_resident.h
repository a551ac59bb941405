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

constexpr int kResThreads = 512;      // two wavefronts per SIMD: a step is bounded by the instructions a SIMD issues,
                                      // and by how many row loads of the step's spikes are in flight at once
constexpr int kResBlocks = 32;        // taking-part blocks at most: the compute units of one XCD
constexpr int kResStride = 8;         // XCDs: block b runs on XCD b mod 8
constexpr int kResMaxSpins = 1 << 16;  // polls of one wait before it gives up (tens of ms; a step takes microseconds); Dev::res_spins, lowered only by tests of the failure path
constexpr int kResLaunch = kResThreads + 64;   // one more wavefront per block that only synchronises: it
                                               // polls the barrier counter and adds the block's arrival, so that
                                               // a poll never waits behind the stores of a wavefront that has neurons

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
  if (threadIdx.x == kResThreads) atomicAdd(&d.ctr->bar[0], 1u);
}
__device__ __forceinline__ void res_wait(const Dev& d, unsigned target, int* dead) {
  if (threadIdx.x == kResThreads && !*dead) {
    int spins = 0;
    while ((int)(ld_agent(&d.ctr->bar[0]) - target) < 0) {
      if (++spins > d.res_spins) { atomicOr(&d.ctr->err, ERR_BARRIER); *dead = 1; break; }
    }
  }
  __syncthreads();
}

// The same barrier for many blocks on several XCDs (Dev::res_wide): arrivals at ONE counter queue up behind one another
// (11 ns each), so the blocks arrive on eight counters, a line each, and the synchronising wavefront polls all eight side
// by side (one per lane) until their sum reaches the target; the first poll waits a little, because polls are loads of
// the very lines the arrivals add to.
__device__ __forceinline__ void wide_arrive(const Dev& d, int rank) {
  wait_all_memory();
  __syncthreads();
  if (threadIdx.x == kResThreads) atomicAdd(&d.ctr->rev_arrivals[rank & (kArriveLines - 1)][0], 1u);
}
__device__ __forceinline__ void wide_wait(const Dev& d, unsigned target, int* dead) {
  if (threadIdx.x >= kResThreads && !*dead) {   // the synchronising wavefront, all lanes (the same way through for each)
    const int lane = threadIdx.x & 63;
    const unsigned* p = &d.ctr->rev_arrivals[lane & (kArriveLines - 1)][0];
    for (int k = 0; k < d.rev_delay; ++k) __builtin_amdgcn_s_sleep(16);
    int spins = 0;
    for (;;) {
      const unsigned v = lane < kArriveLines ? ld_agent(p) : 0u;
      unsigned sum = 0;
#pragma unroll
      for (int x = 0; x < kArriveLines; ++x) sum += (unsigned)__builtin_amdgcn_readlane((int)v, x);
      if ((int)(sum - target) >= 0) break;
      if (++spins > d.res_spins) { if (lane == 0) { atomicOr(&d.ctr->err, ERR_BARRIER); *dead = 1; } break; }
    }
  }
  __syncthreads();
}

// Layout of a taking-part block's neurons (ResMap): block `rank` owns neurons [rank * chunk,
// rank * chunk + chunk), chunk a multiple of 256 and at most NG * 1024; thread t of the block owns,
// in group q < NG, the four consecutive neurons rank * chunk + q * 1024 + 4 t + c, c < 4.  A
// wavefront's group thus covers 256 consecutive neurons = four spike words, and every access of a
// group moves 16 bytes per lane.
constexpr int kDriveSteps = 256;

// Drive bits of steps [n_lo, n_hi) in the layout the resident kernel reads: one 16-bit word per
// (step, taking-part block, thread), bit 4 q + c = neuron c of the thread's group q, at
// drive_words16[(n mod kDriveSteps) * P * 256 + rank * 256 + t].  The drive depends on (seed,
// neuron, step) only, so the whole chip hashes a stretch of steps ahead of the resident launches:
// their one XCD would spend a third of a step on the two 64-bit multiplications per neuron.
__global__ __launch_bounds__(kBlock) void k_drive_words(Dev d, long long n_lo, long long n_hi, int P, int chunk, int NG) {
  const long long per_step = (long long)P * kResThreads;
  const long long items = (n_hi - n_lo) * per_step;
  unsigned short* out = reinterpret_cast<unsigned short*>(d.drive_words);
  for (long long it = (long long)blockIdx.x * kBlock + threadIdx.x; it < items; it += (long long)gridDim.x * kBlock) {
    const long long n = n_lo + it / per_step;
    const int rt = (int)(it % per_step);
    const int rank = rt / kResThreads, t = rt % kResThreads;
    const int hi = rank * chunk + chunk < d.BN ? rank * chunk + chunk : d.BN;
    unsigned bits = 0;
    for (int q = 0; q < NG; ++q)
      for (int c = 0; c < 4; ++c) {
        const int g = rank * chunk + q * 4 * kResThreads + 4 * t + c;
        if (g < hi && (unsigned long long)drive_bits(d.seed, (unsigned long long)g, (unsigned long long)n) < d.p_thresh)
          bits |= 1u << (4 * q + c);
      }
    out[(size_t)(n & (kDriveSteps - 1)) * per_step + rt] = (unsigned short)bits;
  }
}

// A compute unit moves 64 bytes per cycle to or from its memory pipeline and takes a wavefront's
// memory instruction every few cycles whatever its width, so the rows are moved 16 bytes per lane.
// Agent-scope 16-byte loads exist only as buffer loads (the scope is the instruction's cache
// policy); a buffer access beyond the descriptor's length reads zero and writes nothing, which is
// how the lanes past the end of the block's range are switched off.
typedef int res_v4i __attribute__((ext_vector_type(4)));
typedef float res_v4f __attribute__((ext_vector_type(4)));
constexpr int kBufAgent = 16;         // cache policy bit sc1: agent scope
constexpr int kBufNonTemporal = 2;    // cache policy bit nt
__device__ __forceinline__ __amdgpu_buffer_rsrc_t res_rows(const void* p, int bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(p), 0, bytes, 0x00020000);
}

// A spike of the step being run, as the block's wavefronts share them out: bounds of its sorted
// row and the first state index of its trial.
struct ResSpike { long long r0; int len; int base; };

// Steps n0 .. n0 + nsteps - 1 of the closed loop, all inside one window (no window boundary is
// crossed: the host expands the next window between two launches).  P taking-part blocks of 256
// threads (one wavefront per SIMD: what bounds a step on one XCD is the number of instructions a
// SIMD has to issue, so few wavefronts with many neurons each, no per-neuron branches, and a
// common path -- no spike among the wavefront's neurons -- that is as short as it can be).
// Needs B N a multiple of 4 (16-byte aligned rows).  bar_base: value of the barrier counter when
// the launch begins.  Same arithmetic, in the same order, as k_step_win; the drive bits come from
// drive_words (k_drive_words has run for these steps with the same P, chunk, NG).
template <bool RECORD, int SYN, int NG>
__global__ __launch_bounds__(kResLaunch) void k_run_xcd(long long n0, int nsteps, unsigned bar_base, int P,
                                                         int chunk, int stride, Dev d) {
  __shared__ int s_dead, s_nspk;
  __shared__ ResSpike s_spk[NG * 4 * kResThreads];   // the block's spikes of the step (one entry per neuron at most)
  if (blockIdx.x % stride) return;
  const int rank = blockIdx.x / stride;
  if (rank >= P) return;
  // (a wait that ran out in an earlier launch stays on record: then nobody waits any more, the run is void anyway)
  if (threadIdx.x == 0) { s_dead = (ld_agent(&d.ctr->err) & ERR_BARRIER) ? 1 : 0; s_nspk = 0; }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool worker = threadIdx.x < kResThreads;   // uniform per wavefront; the last wavefront only synchronises
  const int lo = rank * chunk;
  const int hi = worker ? (lo + chunk < d.BN ? lo + chunk : d.BN) : 0;   // (no neuron lies below 0: the last wavefront owns none)
  constexpr int NPT = NG * 4;
  // what stays in registers for the whole launch (index j = 4 q + c)
  int g0[NG], rlen[NPT];
  long long r0[NPT];
  float V[NPT], J[NPT], Jf[NPT];
  unsigned actmask = 0;   // bit j: neuron j of this thread exists
  long long popped = 0;   // Q8.24 sum of what this thread has popped (counted for the whole launch at its end)
#pragma unroll
  for (int q = 0; q < NG; ++q) {
    g0[q] = lo + q * 4 * kResThreads + 4 * (int)threadIdx.x;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int j = 4 * q + c, g = g0[q] + c;
      rlen[j] = 0; r0[j] = 0; V[j] = 0.0f; J[j] = 0.0f; Jf[j] = 0.0f;
      if (g < hi) {
        actmask |= 1u << j;
        const int i = g - trial_of(d, g) * d.N;
        r0[j] = d.row_ptr[i];
        rlen[j] = (int)(d.row_ptr[i + 1] - r0[j]);
        V[j] = d.V[g];
        if (SYN) J[j] = d.J[g];
        if (SYN == 2) Jf[j] = d.J[(size_t)d.BN + g];
      }
    }
  }
  // lane 4 q + w of a wavefront stores word w of the wavefront's group q: its index, or -1
  int my_word = -1;
#pragma unroll
  for (int q = 0; q < NG; ++q) {
    const int gw = __builtin_amdgcn_readfirstlane(g0[q]);   // first neuron of the wavefront's group q
    if (worker && (lane >> 2) == q && gw < lo + chunk && (gw >> 6) + (lane & 3) < d.words) my_word = (gw >> 6) + (lane & 3);
  }
  int slot = (int)(n0 % d.R);   // row of the circular spike words that holds step n0 (one division per launch)
  const unsigned short* drive16 = reinterpret_cast<const unsigned short*>(d.drive_words) + (size_t)rank * kResThreads + threadIdx.x;
  const size_t drive_stride = (size_t)P * kResThreads;
  __syncthreads();
  // The chain a step cannot avoid is: barrier -> cells (L2) -> threshold -> row pieces of the
  // spikes -> their adds acknowledged -> arrival.  Everything else is taken off it: the drive bits
  // of a step are fetched, and the cells of its row touched (which brings them into the L2), while
  // the block waits for the barrier before it; the tape, the cleared cells and the spike words are
  // stored after the arrival, so that the wait for the adds does not wait for them.
#ifdef ADSEQ_PHASE_CLOCK
  unsigned long long pc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, pt = wall_clock64();
#define PHASE(i) { const unsigned long long t_ = wall_clock64(); pc[i] += t_ - pt; pt = t_; }
#else
#define PHASE(i) {}
#endif
#ifdef ADSEQ_ABLATE
#define DBG_SKIP(bit) (d.dbg & (bit))
#else
#define DBG_SKIP(bit) false
#endif
  unsigned dr = (d.p_thresh && worker) ? drive16[(size_t)(n0 & (kDriveSteps - 1)) * drive_stride] : 0u;
  res_v4i touch[NG];   // the touching loads of a later row: their values are never used
  {
    // the row of the launch's second step is touched now (later rows: two steps ahead, inside the loop)
    const int phi0 = (int)(n0 & (long long)(d.W - 1));
    const __amdgpu_buffer_rsrc_t second = res_rows(win_of(d, n0) + (size_t)(phi0 + 1) * d.BN, (nsteps > 1 && phi0 + 1 < d.W) ? hi * 4 : 0);
#pragma unroll
    for (int q = 0; q < NG; ++q) touch[q] = __builtin_amdgcn_raw_buffer_load_b128(second, g0[q] * 4, 0, kBufAgent);
  }
  for (int k = 0; k < nsteps; ++k) {
    const long long n = n0 + k;
    const int phi = (int)(n & (long long)(d.W - 1));
    int near_h = d.W - 1 - phi;
    if (near_h > d.d_max) near_h = d.d_max;
    int* __restrict__ win = win_of(d, n) + (size_t)phi * d.BN;   // row of this step
    const __amdgpu_buffer_rsrc_t cells = res_rows(win, hi * 4);
    PHASE(5)
    // the adds of step n - 1 are in place once every block has arrived
    if (k > 0) {
      if (d.res_wide) wide_wait(d, bar_base + (unsigned)k * (unsigned)P, &s_dead);
      else res_wait(d, bar_base + (unsigned)k * (unsigned)P, &s_dead);
    }
    PHASE(0)
#pragma unroll
    for (int q = 0; q < NG; ++q) asm volatile("" ::"v"(touch[q]));   // (the touching loads of the step before stay alive until here)
    res_v4i acc[NG];
#pragma unroll
    for (int q = 0; q < NG; ++q) acc[q] = __builtin_amdgcn_raw_buffer_load_b128(cells, g0[q] * 4, 0, kBufAgent);
#ifdef ADSEQ_PHASE_CLOCK
    wait_all_memory();
#endif
    PHASE(1)
    float U[NPT];
    unsigned smask = 0;   // bit j: neuron j spiked
#pragma unroll
    for (int j = 0; j < NPT; ++j) {
      popped += acc[j >> 2][j & 3];
      float I = (float)acc[j >> 2][j & 3] * 0x1p-24f;
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
      if (d.p_thresh) I = I + (((dr >> j) & 1u) ? d.ext_w : 0.0f);
      U[j] = __fmaf_rn(d.alpha, V[j], I);
      const bool sj = U[j] >= d.theta;
      V[j] = sj ? d.v_reset : U[j];
      smask |= sj ? 1u << j : 0u;
    }
    smask &= actmask;
    const bool wave_spiked = __ballot(smask != 0u) != 0ull;   // uniform: most wavefronts have no spike in a step
    PHASE(2)
    // The in-window events of the spikes: the front of the sorted row, entries with arrival
    // offset <= near_h (the rows are ascending in the offset).  A wavefront holds 1,024 neurons and
    // several of them spike in a step, so the block's spikes go into a list in LDS and the four
    // wavefronts share them out, four spikes at a time per wavefront: the leading 64 entries of
    // all four are requested before the first add (one trip to memory, not one per spike).
    if (near_h >= 1) {
      if (wave_spiked && !DBG_SKIP(128)) {
        unsigned long long m[NPT];
        int total = 0;
#pragma unroll
        for (int j = 0; j < NPT; ++j) {
          m[j] = __ballot(((smask >> j) & 1u) && rlen[j] > 0);
          total += __popcll(m[j]);
        }
        int at = 0;
        if (lane == 0 && total) at = atomicAdd(&s_nspk, total);
        at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
        for (int j = 0; j < NPT; ++j) {
          if (m[j] == 0ull) continue;   // uniform
          if ((m[j] >> lane) & 1ull) {
            ResSpike r;
            r.r0 = r0[j]; r.len = rlen[j]; r.base = trial_of(d, g0[j >> 2] + (j & 3)) * d.N;
            s_spk[at + __popcll(m[j] & ((1ull << lane) - 1ull))] = r;
          }
          at += __popcll(m[j]);
        }
      }
      __syncthreads();
      const int nspk = DBG_SKIP(64) ? 0 : s_nspk;
      for (int k0 = wave; worker && k0 < nspk; k0 += 4 * (kResThreads / 64)) {
        ResSpike r[4]; uint2 e[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int x = k0 + u * (kResThreads / 64);
          r[u].r0 = 0; r[u].len = 0; r[u].base = 0; e[u] = make_uint2(0u, 0u);
          if (x < nspk) {
            r[u] = s_spk[x];
            if (lane < r[u].len) e[u] = d.synf[r[u].r0 + lane];
          }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (r[u].len == 0) continue;   // uniform
          bool more = false;
          if (lane < r[u].len) {
            const int D = (int)(e[u].x & d.dmask);
            if (D <= near_h) {
              atomicAdd(&win[(size_t)D * d.BN + (size_t)r[u].base + (e[u].x >> d.dbits)], (int)e[u].y);
              more = true;
            }
          }
          // the next 64 entries only while a group's last one was still inside the window
          for (int q0 = 64; (__ballot(more) >> 63) && q0 < r[u].len; q0 += 64) {
            more = false;
            if (q0 + lane < r[u].len) {
              const uint2 x = d.synf[r[u].r0 + q0 + lane];
              const int D = (int)(x.x & d.dmask);
              if (D <= near_h) {
                atomicAdd(&win[(size_t)D * d.BN + (size_t)r[u].base + (x.x >> d.dbits)], (int)x.y);
                more = true;
              }
            }
          }
        }
      }
    }
#ifdef ADSEQ_PHASE_CLOCK
    wait_all_memory();
#endif
    PHASE(3)
    if (k + 1 < nsteps) {
      if (d.res_wide) wide_arrive(d, rank);
      else res_arrive(d);
    }
    if (threadIdx.x == 0) s_nspk = 0;   // (every wavefront has read the list: block barrier in res_arrive; the last step needs none)
    // touch the cells of the row two steps on (values that may still change are not used: the
    // loads only bring the lines into the L2, two steps before they are popped; issued after the
    // arrival, so that the wait for the adds does not wait for them)
    if (phi + 2 < d.W && k + 2 < nsteps && !DBG_SKIP(8)) {
      const __amdgpu_buffer_rsrc_t ahead = res_rows(win + 2 * (size_t)d.BN, hi * 4);
#pragma unroll
      for (int q = 0; q < NG; ++q) touch[q] = __builtin_amdgcn_raw_buffer_load_b128(ahead, g0[q] * 4, 0, kBufAgent);
    }
    PHASE(4)
    // off the chain: tape, spike words and counts of this step (the popped cells are not cleared
    // here: the expansion at the next window boundary zeroes the whole buffer, see k_win_bin)
    unsigned long long wbits = 0ull;   // lane 4 q + w: word w of group q
    const __amdgpu_buffer_rsrc_t tape = res_rows(d.tapeU + (size_t)n * d.BN, RECORD ? hi * 4 : 0);
#pragma unroll
    for (int q = 0; q < NG; ++q) {
      if (RECORD && !DBG_SKIP(2)) {
        const res_v4f u4 = {U[4 * q], U[4 * q + 1], U[4 * q + 2], U[4 * q + 3]};
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(res_v4i, u4), tape, g0[q] * 4, 0, kBufNonTemporal);
      }
      if (wave_spiked && !DBG_SKIP(4)) {
        const int s4 = (int)((smask >> (4 * q)) & 15u);
        if (RECORD && !DBG_SKIP(16)) {
#pragma unroll
          for (int c = 0; c < 4; ++c)
            if ((s4 >> c) & 1) atomicAdd(&d.spk_count[g0[q] + c], 1);
        }
        // spike words: lane 16 w + x holds neurons 4 x .. 4 x + 3 of word w; lane l of a ballot must
        // stand for neuron l of the word, i.e. for bit (l & 3) of lane 16 w + (l >> 2)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int v = __shfl(s4, 16 * w + (lane >> 2), 64);
          const unsigned long long b = __ballot((v >> (lane & 3)) & 1);
          if (lane == 4 * q + w) wbits = b;
        }
      }
    }
    if (my_word >= 0 && !DBG_SKIP(32)) {
      d.spike_bits[(size_t)slot * d.words + my_word] = wbits;
      if (RECORD) d.tape_bits[(size_t)n * d.words + my_word] = wbits;
    }
    if (++slot == d.R) slot = 0;
    PHASE(6)
    if (k + 1 < nsteps) {
      // drive bits of the next step
      if (d.p_thresh && worker) dr = drive16[(size_t)((n + 1) & (kDriveSteps - 1)) * drive_stride];
      PHASE(7)
    }
  }
#ifdef ADSEQ_PHASE_CLOCK
  if (threadIdx.x == 0 && rank == 0)
    for (int i = 0; i < 8; ++i) atomicAdd(&d.ctr->phase[i], pc[i]);
#endif
  if (d.count_pop) count_popped(d, popped);
#pragma unroll
  for (int j = 0; j < NPT; ++j)
    if ((actmask >> j) & 1u) {
      const int g = g0[j >> 2] + (j & 3);
      d.V[g] = V[j];
      if (SYN) d.J[g] = J[j];
      if (SYN == 2) d.J[(size_t)d.BN + g] = Jf[j];
    }
}
