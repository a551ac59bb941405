// Ring queue: step launches that wait for one another themselves ("chained" step kernels).
// Included by adseq.hip after ring_resident.h (whose agent-scope access helpers it uses).
// Experimental (ADSEQ_RING_CHAIN = 1), off by default: results identical, but slower than one
// stream on the headline network -- see the end of this comment.
//
// Two kernels that follow one another on ONE stream are separated by the queue's barrier: the
// second is set up only after the first has drained and its caches are written back, 1.5-2.4 us
// during which nothing runs.  Two kernels on TWO streams have no such barrier, so the host deals
// the step launches out over two streams in turn and the kernels order themselves: every block
// of step launch k first does what depends on nothing step k - 1 produces (argument fetch, row
// bounds, drive hash; in the reverse sweep the tape, the far queue terms, the rows of its spikes
// and every adjoint gather except those one step away), then waits until all blocks of launch
// k - 1 have ARRIVED -- their stores and atomic adds acknowledged -- and only then reads what launch
// k - 1 wrote, with agent-scope loads.  What crosses from one launch to the next is written with
// agent-scope stores or atomics (coherent over the chip without a fence: `chip_rates resident`).
// Launch k - 2 is the stream's own predecessor, so everything older than one step is ordered by
// the stream and visible to ordinary loads.  At a window boundary the two streams meet through
// events, so the window kernels are ordered after every step before them and before every step
// after them.
//
// Measured: a chain of EMPTY kernels of this shape runs at 1.3 us per kernel on two streams
// against 2.5 us on one (`chip_rates resident`), but the real steps do not (100,000 neurons,
// 1,000 steps, forward / reverse ms per run): one stream 6.04 / 7.11; chained, 391 blocks of 256
// threads 9.61 / 8.08; 98 blocks of 1,024 threads with a pause between polls 7.50 / 7.49.  What the
// queue's barrier costs between two launches, the hand-over inside the kernels costs again: the
// producer waits for the acknowledgement of its agent-scope stores and atomics, its arrival
// travels to the counter, the consumer's poll travels there and back, and its first loads go past
// the L2 -- each a trip over the fabric of 0.5-1 us -- while the polls of the waiting launch load the
// same fabric (`chip_rates exchange`: a round of a resident kernel that exchanges a step's spike
// words and 6,000 adds over the whole chip takes 3.8-9.2 us).
//
// Arrivals: one counter per residue of the block index mod 8 (the block's XCD), each on a line of
// its own, never reset during a run; launch k waits until their sum reaches what the host counted
// for all launches before it.  Every wait is a bounded spin (Dev::res_spins polls): a wait that
// runs out sets ERR_BARRIER, after which no launch waits any more, so every block of every launch
// reaches its end whatever happens; the run is then void and the host reports it.

// Waits (wavefront 0 polls, the block follows through the workgroup barrier) until the arrival
// counters add up to `target`.
__device__ __forceinline__ void chain_wait(const Dev& d, unsigned target) {
  if (threadIdx.x < 64) {
    // lanes 0..7 watch one counter each, lane 8 the error word (a wait that ran out earlier: nobody waits any more)
    const int lane = threadIdx.x;
    const unsigned* p = lane < 8 ? &d.ctr->arrive[lane][0] : &d.ctr->err;
    int spins = 0;
    for (;;) {
      const unsigned v = lane < 9 ? ld_agent(p) : 0u;
      unsigned sum = 0;
#pragma unroll
      for (int x = 0; x < 8; ++x) sum += (unsigned)__builtin_amdgcn_readlane((int)v, x);
      const unsigned err = (unsigned)__builtin_amdgcn_readlane((int)v, 8);
      if ((int)(sum - target) >= 0 || (err & ERR_BARRIER)) break;
      if (++spins > d.res_spins) { if (lane == 0) atomicOr(&d.ctr->err, ERR_BARRIER); break; }
      for (int k = 0; k < d.chain_sleep; ++k) __builtin_amdgcn_s_sleep(2);
    }
  }
  __syncthreads();
}

// The block's arrival: every wavefront has its stores and atomic adds acknowledged first.
__device__ __forceinline__ void chain_arrive(const Dev& d) {
  wait_all_memory();
  __syncthreads();
  if (threadIdx.x == 0) atomicAdd(&d.ctr->arrive[blockIdx.x & 7][0], 1u);
}

// Forward step n as k_step_win runs it (same arithmetic in the same order, delta synapse only),
// waiting for `target` arrivals before it pops.  The membrane state goes from launch to launch
// through agent-scope accesses; the cells of the window row are read with agent-scope loads (the
// adds into them are atomics).  The cleared cell is an ordinary store: nothing adds to a popped
// cell before the window after next is expanded, launches later on a stream that has waited for
// this one.
template <bool RECORD, int TPB>
__global__ __launch_bounds__(TPB) void k_step_chain(long long n, unsigned target, Dev d) {
  pin_args(d.win, d.V, d.row_ptr, d.nearcnt, d.tapeU, d.spk_count, d.spike_bits, d.tape_bits, d.synf, d.ctr,
           d.N, d.B, d.BN, d.W, d.wshift, d.d_max, d.R, d.words, d.dbits, d.dmask, d.alpha, d.theta,
           d.v_reset, d.ext_w, d.p_thresh, d.seed, d.res_spins, d.chain_sleep, n, target);
  const int g = blockIdx.x * TPB + threadIdx.x;
  const bool act = g < d.BN;
  const int phi = (int)(n & (long long)(d.W - 1));
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  int b = 0;
  bool s = false, xi = false;
  long long r0 = 0;
  unsigned ncnt = 0;
  int* __restrict__ win = win_of(d, n);
  const size_t idx = (size_t)phi * d.BN + g;
  if (act) {
    b = trial_of(d, g);
    const int i = g - b * d.N;
    r0 = d.row_ptr[i];
    if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
    if (d.p_thresh)
      xi = (unsigned long long)drive_bits(d.seed, (unsigned long long)g, (unsigned long long)n) < d.p_thresh;
  }
  chain_wait(d, target);
  if (act) {
    const int acc = ld_agent(&win[idx]);
    const float v = ld_agent(&d.V[g]);
    if (acc != 0) win[idx] = 0;
    float I = (float)acc * 0x1p-24f;
    if (d.p_thresh) I = I + (xi ? d.ext_w : 0.0f);
    const float U = __fmaf_rn(d.alpha, v, I);
    s = U >= d.theta;
    st_agent(&d.V[g], s ? d.v_reset : U);
    if (RECORD) {
      __builtin_nontemporal_store(U, &d.tapeU[(size_t)n * d.BN + g]);
      if (s) atomicAdd(&d.spk_count[g], 1);
    }
  }
  const unsigned long long bits = __ballot(s);
  const size_t word = (size_t)blockIdx.x * (TPB / 64) + (threadIdx.x >> 6);
  if ((threadIdx.x & 63) == 0 && word < (size_t)d.words) {
    d.spike_bits[(size_t)(n % d.R) * d.words + word] = bits;
    if (RECORD) d.tape_bits[(size_t)n * d.words + word] = bits;
  }
  unsigned long long m = __ballot(s && ncnt > 0);
  const int lane = threadIdx.x & 63;
  while (m) {
    long long pr[4]; unsigned cn[4]; int bs[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      pr[j] = 0; cn[j] = 0; bs[j] = 0;
      if (m) {
        const int L = __ffsll((long long)m) - 1;
        m &= m - 1;
        pr[j] = lane_get(r0, L); cn[j] = lane_get(ncnt, L); bs[j] = lane_get(b, L) * d.N;
      }
    }
    uint2 e[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      e[j] = make_uint2(0u, 0u);
      if ((unsigned)lane < cn[j]) e[j] = d.synf[pr[j] + lane];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if ((unsigned)lane < cn[j])
        atomicAdd(&win[(size_t)(phi + (int)(e[j].x & d.dmask)) * d.BN + (size_t)bs[j] + (e[j].x >> d.dbits)], (int)e[j].y);
      if (cn[j] > 64u) near_scatter(d, win, phi, pr[j] + 64, cn[j] - 64u, bs[j]);
    }
  }
  chain_arrive(d);
}

// near_gather of k_bwd_step_win for the entries beyond a row's first 64, read after the wait: the
// adjoints one step away come from the launch before, so every gather is an agent-scope load.
__device__ __forceinline__ float near_gather_agent(const Dev& d, const float* __restrict__ gwin, long long n,
                                                   long long T, int phi, long long pr0, unsigned cnt, int base) {
  const int lane = threadIdx.x & 63;
  float G = 0.0f;
  for (unsigned q = lane; q < cnt; q += 64) {
    const uint2 e = d.synb[pr0 + q];
    const int D = (int)(e.x & d.dmask);
    if (n + D < T) {
      const float gv = ld_agent(&gwin[(size_t)(phi + D) * d.BN + (size_t)base + (e.x >> d.dbits)]);
      unsafeAtomicAdd(&d.gsum[pr0 + q], gv);
      G += __uint_as_float(e.y) * gv;
    }
  }
  return wave_sum_f(G);
}

// One batch of up to four spikes of the wavefront in the reverse step: row bounds, the rows'
// first 64 entries, the adjoints they gather.
struct ChainBatch {
  long long pr[4]; unsigned cn[4]; int bs[4], Ls[4];
  uint2 e[4];
  float gv[4];
};

// Reverse step n as k_bwd_step_win runs it (delta synapse only), waiting for `target` arrivals
// before it reads what reverse step n + 1 wrote: its carry and row n + 1 of the adjoint window,
// i.e. the gathers of the entries with arrival offset 1.  Everything else -- the tape, the far queue
// term, the rows of the spikes and the gathers at offsets of two and more, whose rows were written
// by launches that the stream orders before this one -- is in flight or done before the wait.
template <int TPB>
__global__ __launch_bounds__(TPB) void k_bwd_step_chain(long long n, long long T, unsigned target,
                                                           const float* __restrict__ dL_dcount,
                                                           const float* __restrict__ dL_dU, Dev d) {
  pin_args(d.gwin, d.tapeU, d.bwd_carry, d.row_ptr, d.nearcnt, d.Gacc, d.synb, d.gsum, d.ctr,
           d.N, d.B, d.BN, d.W, d.wshift, d.d_max, d.R, d.dbits, d.dmask, d.surrogate, d.alpha,
           d.theta, d.v_reset, d.dt, d.tau, d.res_spins, d.chain_sleep, n, T, target, dL_dcount, dL_dU);
  const int g = blockIdx.x * TPB + threadIdx.x;
  const bool act = g < d.BN;
  const int phi = (int)(n & (long long)(d.W - 1));
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  float U = 0.0f, Uprev = 0.0f, inner = 0.0f, G = 0.0f, dU = 0.0f;
  bool s = false;
  int b = 0;
  long long r0 = 0;
  unsigned ncnt = 0;
  float* __restrict__ gwin = gwin_of(d, n);
  if (act) {
    b = trial_of(d, g);
    const int i = g - b * d.N;
    U = d.tapeU[(size_t)n * d.BN + g];
    if (d.surrogate == ADSEQ_GRAD_SPIKE_TIME && n > 0) Uprev = d.tapeU[(size_t)(n - 1) * d.BN + g];
    if (dL_dcount) inner = dL_dcount[g];
    if (dL_dU) dU = dL_dU[(size_t)n * d.BN + g];
    float* ga = &d.Gacc[(size_t)(n % d.R) * d.BN + g];
    r0 = d.row_ptr[i];
    if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
    G = *ga;
    s = U >= d.theta;
    if (G != 0.0f) *ga = 0.0f;
  }
  unsigned long long m = __ballot(s && ncnt > 0);
  const int lane = threadIdx.x & 63;
  // Up to four of the wavefront's spikes at a time: row bounds, the first 64 entries of each row, and the gathers two and
  // more steps away (rows of the adjoint window that the stream orders before this launch).
  ChainBatch cb;
  auto next_batch = [&]() {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      cb.pr[j] = 0; cb.cn[j] = 0; cb.bs[j] = 0; cb.Ls[j] = -1;
      if (m) {
        const int L = __ffsll((long long)m) - 1;
        m &= m - 1;
        cb.Ls[j] = L;
        cb.pr[j] = lane_get(r0, L); cb.cn[j] = lane_get(ncnt, L); cb.bs[j] = lane_get(b, L) * d.N;
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      cb.e[j] = make_uint2(0u, 0u);
      if ((unsigned)lane < cb.cn[j]) cb.e[j] = d.synb[cb.pr[j] + lane];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      cb.gv[j] = 0.0f;
      const int D = (int)(cb.e[j].x & d.dmask);
      if ((unsigned)lane < cb.cn[j] && D >= 2 && n + D < T)
        cb.gv[j] = gwin[(size_t)(phi + D) * d.BN + (size_t)cb.bs[j] + (cb.e[j].x >> d.dbits)];
    }
  };
  next_batch();   // the first batch is in flight before the wait
  chain_wait(d, target);
  float carry = 0.0f;
  if (act) carry = ld_agent(&d.bwd_carry[g]);
  for (;;) {
    // the gathers one step away: row n + 1, written by the launch this one has waited for
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int D = (int)(cb.e[j].x & d.dmask);
      if ((unsigned)lane < cb.cn[j] && D == 1 && n + D < T)
        cb.gv[j] = ld_agent(&gwin[(size_t)(phi + D) * d.BN + (size_t)cb.bs[j] + (cb.e[j].x >> d.dbits)]);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (cb.Ls[j] < 0) continue;    // uniform
      const int D = (int)(cb.e[j].x & d.dmask);
      float part = 0.0f;
      if ((unsigned)lane < cb.cn[j] && n + D < T) {
        part = __uint_as_float(cb.e[j].y) * cb.gv[j];
        unsafeAtomicAdd(&d.gsum[cb.pr[j] + lane], cb.gv[j]);
      }
      part = wave_sum_f(part);
      if (cb.cn[j] > 64u) part += near_gather_agent(d, gwin, n, T, phi, cb.pr[j] + 64, cb.cn[j] - 64u, cb.bs[j]);
      if (lane == cb.Ls[j]) G += part;
    }
    if (!m) break;
    next_batch();   // (more than four spikes among the wavefront's 64 neurons)
  }
  if (act) {
    float gu;
    st_agent(&d.bwd_carry[g], bwd_update(d, n, U, Uprev, s, carry, inner, G, dU, &gu));
    st_agent(&gwin[(size_t)phi * d.BN + g], gu);
  }
  chain_arrive(d);
}
