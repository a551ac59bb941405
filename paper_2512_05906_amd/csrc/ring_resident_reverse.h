// Ring queue, reverse sweep: the steps of one window in ONE launch, a grid barrier per step
// (delta synapse).  Included by adseq.hip after ring_window.h and ring_resident.h, whose layout
// (four consecutive neurons per thread, 16-byte buffer accesses), bounded waits (ERR_BARRIER) and
// agent-scope accesses it shares.
//
// The reverse step n (bwd_update; Section 3.2 eqs. 13 and 17 carried back through the steps) needs
// from step n + 1 the carry of its own neuron and, for the entries of its spikes' rows that arrive
// one step later, row n + 1 of the adjoint window -- nothing else.  And unlike the forward pass the
// reverse sweep KNOWS its spikes: they are on the tape.  So a block prepares a step ahead of time.
// In front of the barrier of step n, in this order: the list of its spikes of step n - 1 and the
// leading 64 entries of their rows requested; tape values of step n - 2, far queue terms and dL/dU of
// step n - 1 requested; every adjoint that step n's own entries (requested a step ago) gather two or
// more steps away (rows complete since the barrier before last); and the whole row n computed and
// stored with the near parts of the queue terms left out -- a neuron that does not spike at step n
// needs nothing of any other neuron.  Behind the barrier only the gathers one step away are left
// (row n + 1 was written through the L2s a moment ago), then the per-spike sums and the few spiking
// neurons again with their whole queue term (a spiking neuron's update does not use the carry: the
// reset cuts it); their cells are stored again and acknowledged before the block arrives.  The
// per-synapse gradient sums (atomic adds into gsum, read only when the sweep is over) are issued
// after the arrival.  The carry stays in registers for the whole launch.
//
// What the compiler must not be allowed to undo: a value requested steps ago is used in front of
// the barrier while newer requests are on their way, and the one counter of outstanding memory
// operations counts in order -- a wait for the old one that the compiler cannot bound becomes a wait
// for all.  So the waits are spelled with the compiler's own builtin (an inline-asm wait it does
// not see), the loop begins with nothing outstanding, no request is issued after the arrival, and
// no request stands behind a branch that depends on loaded data.
//
// The barrier: 128 blocks by default, spread over the chip's XCDs.  Arrivals at one counter
// queue up behind one another (11 ns each), so the blocks arrive on kArriveLines (16) counters, a
// line each; the last wavefront of a block owns no neurons, only passes the block's barriers,
// polls the counters side by side and adds the block's arrival.  Polls are loads of the very lines
// the arrivals add to (measured on 100,000 neurons: one counter, polls at once 4.5-6.8 us per
// step; eight counters, first poll delayed by half a microsecond 3.55 us; sixteen, no delay 3.5 us).
//
// The default reverse kernel is k_bwd_flow (ring_flow_reverse.h), which has no grid barrier; this
// one runs with ADSEQ_RING_REVERSE_FLOW = 0 and lends the other its lists, batches and helpers.
//
// Same arithmetic as k_bwd_step_win; the order in which a spike's terms are added differs (fp32
// rounding only).  Results do not depend on where the blocks run: what crosses blocks goes
// through agent-scope stores and loads and the barrier counters.
// Measured, reverse ms per run, this kernel / one launch per step: 100 neurons x 1,000 steps 2.4 / 3.6;
// 16 x 1,000 neurons x 2,000 steps 5.6 / 8.6; 10,000 neurons x 10,000 steps 39.7 / 46.5; 100,000 neurons
// x 1,000 steps 6.3 / 7.1 (3.55 against 4.45 us per step).

constexpr int kRevList = 1024;        // spikes of one step that a block lists in LDS (more: the owners' wavefronts take them one by one)
constexpr int kRevLocBits = 12;       // a block owns at most 2,048 neurons

// A listed spike: bounds of its sorted row, and place of its neuron in the block | trial << kRevLocBits.
struct RevSpike { long long r0; int len; int pk; };

// Up to four of a wavefront's listed spikes: per lane the leading 64 entries of their rows, the
// adjoints those gather, and which of the four hold an entry that arrives inside the window and the
// run (bit u of ok); the rows' bounds and the trials' first state index are the same in every lane.
struct RevBatch {
  uint2 e[4];
  float gv[4];
  unsigned ok;
  long long r0[4];
  int len[4], base[4], loc[4];
};

// The block's arrival at the step's barrier, as res_arrive, with the wait for the block's memory operations spelled
// as the compiler's own builtin: the compiler then knows that everything requested before is complete, and does not
// wait again (for the requests of the step after) where a value requested steps ago is first used.
__device__ __forceinline__ void rev_arrive(const Dev& d, bool arrive, int rank) {
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0); the other counters at their maximum
  __syncthreads();
  if (arrive && threadIdx.x == kResThreads) atomicAdd(&d.ctr->rev_arrivals[rank & (kArriveLines - 1)][0], 1u);
}

// The grid barrier's wait.  Arrivals at ONE counter queue up behind one another (11 ns each: 256 blocks, 2.8 us), so the
// blocks arrive on kArriveLines counters, a line each, and the synchronising wavefront polls them all side by side (one per
// lane) until their sum reaches the target.  The polls are loads of the very lines the arrivals add to, so the first
// poll waits for as long as the workers need at least for what they do in front of the barrier.
__device__ __forceinline__ void rev_wait(const Dev& d, unsigned target, int* dead) {
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

__device__ __forceinline__ long long uniform_of(long long v) {
  const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)v);
  const int hi = __builtin_amdgcn_readfirstlane((int)(v >> 32));
  return ((long long)hi << 32) | lo;
}

// Entries [q0, len) of a spike's sorted row, 64 at a time while they arrive inside the window (the
// rows ascend in the arrival offset): gathers the adjoints (agent scope: every row of the window was
// written by this launch), adds them to gsum, and returns the wavefront's sum of amplitude * adjoint.
__device__ __forceinline__ float rev_row_tail(const Dev& d, const float* __restrict__ gwin, int near_h, long long r0,
                                              int len, int base, int q0, bool more) {
  const int lane = threadIdx.x & 63;
  float part = 0.0f;
  for (; (__ballot(more) >> 63) && q0 < len; q0 += 64) {
    more = false;
    float t = 0.0f;
    if (q0 + lane < len) {
      const uint2 e = load_stream(&d.synb[r0 + q0 + lane]);
      const int D = (int)(e.x & d.dmask);
      if (D <= near_h) {
        const float gv = ld_agent(&gwin[(size_t)D * d.BN + (size_t)base + (e.x >> d.dbits)]);
        unsafeAtomicAdd(&d.gsum[r0 + q0 + lane], gv);
        t = __uint_as_float(e.y) * gv;
        more = true;
      }
    }
    part += wave_sum_f(t);
  }
  return part;
}

// What a worker thread carries through the launch.
struct RevState {
  float carry[4], dLc[4];        // its four neurons: carry of the adjoint, dL/dcount
  long long r0[4]; int rlen[4];  // bounds of their sorted rows
  unsigned actmask;              // bit c: neuron c exists
  res_v4f Ua, Ub, Uc;            // tape values of the step being run, of the one after it, of the one after that
  res_v4f Ga, Gb, dUa, dUb;      // far queue terms and dL/dU of the step being run and of the next
  unsigned ovf_cur;              // bit c: neuron c spiked in the step being run and did not fit the list
  int nspk_cur;                  // listed spikes of the step being run
  // the same in every lane
  long long n;                   // step being run
  int phi, tail, slot;           // n mod W, T - 1 - n, n mod R
  float* gwin;                   // row n of the adjoint window
  const float* tape2;            // tape row of step n - 2 (of step 0 below that)
  const float* du1;              // dL/dU row of step n - 1 (of step 0 below that)
  int g0, hi;
};

__device__ __forceinline__ int rev_near(const Dev& d, int phi, int tail) {
  int h = d.W - 1 - phi;
  if (h > d.d_max) h = d.d_max;
  if (h > tail) h = tail;   // arrivals n + D >= T were never delivered
  return h;
}

// One reverse step of a worker wavefront.  PAR: list buffer of the step being run (the other one takes the list of the
// step after it); cur: the batch of the step being run (rows requested a step ago), nxt: filled here for the next one.
// (One copy of this code in the kernel: two, for the two buffers, ran slower.)
template <bool HAS_DU>
__device__ __forceinline__ void rev_step(const Dev& d, RevState& S, const int PAR, RevBatch& cur, RevBatch& nxt, bool last, bool wait, unsigned wait_for,
                                         int* s_dead, int* s_nspk, RevSpike (*s_spk)[kRevList], float* s_G,
                                         const float* __restrict__ dL_dU) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int kWaves = kResThreads / 64;
  const long long n = S.n;
  const int near_h = rev_near(d, S.phi, S.tail);
  const int near1 = last ? 0 : rev_near(d, S.phi - 1, S.tail + 1);   // of the step after this one (same window: phi >= 1 there)
  float* __restrict__ gwin = S.gwin;
  const int g0 = S.g0, hi = S.hi;
  // ---- before the barrier: nothing here depends on the step before.  Every load of the step is requested here, the
  // ones that go furthest first, and none after the arrival: what was requested is complete when the gathers behind the
  // barrier are, so that no wait for an old request turns into a wait for a new one.
  float U[4], Gf[4], dU[4];
  unsigned smask = 0, s1 = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    U[c] = S.Ua[c]; Gf[c] = S.Ga[c]; dU[c] = HAS_DU ? S.dUa[c] : 0.0f;
    smask |= U[c] >= d.theta ? 1u << c : 0u;
    s1 |= S.Ub[c] >= d.theta ? 1u << c : 0u;
  }
  smask &= S.actmask; s1 &= S.actmask;
  // the step after this one: list of the block's spikes, the leading 64 entries of their rows requested
  int nspk_nxt = 0;
  unsigned ovf_nxt = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) { nxt.e[u] = make_uint2(0u, 0u); nxt.r0[u] = 0; nxt.len[u] = 0; nxt.base[u] = 0; nxt.loc[u] = 0; }
  if (near1 >= 1) {
    if (__ballot(s1 != 0u) != 0ull) {
      unsigned long long m[4];
      int total = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) { m[c] = __ballot(((s1 >> c) & 1u) && S.rlen[c] > 0); total += __popcll(m[c]); }   // (a spike with an empty row is not listed)
      int at = 0;
      if (lane == 0) at = atomicAdd(&s_nspk[PAR ^ 1], total);
      at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (m[c] == 0ull) continue;   // uniform
        if ((m[c] >> lane) & 1ull) {
          const int idx = at + __popcll(m[c] & ((1ull << lane) - 1ull));
          if (idx < kRevList) {
            RevSpike r;
            r.r0 = S.r0[c]; r.len = S.rlen[c];
            r.pk = (4 * (int)threadIdx.x + c) | (trial_of(d, g0 + c) << kRevLocBits);
            s_spk[PAR ^ 1][idx] = r;
          } else {
            ovf_nxt |= 1u << c;
          }
        }
        at += __popcll(m[c]);
      }
    }
    __syncthreads();
    nspk_nxt = s_nspk[PAR ^ 1] < kRevList ? s_nspk[PAR ^ 1] : kRevList;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int x = wave + u * kWaves;
      if (x < nspk_nxt) {   // (the same in every lane: a wavefront without a spike requests nothing)
        const RevSpike r = s_spk[PAR ^ 1][x];
        nxt.r0[u] = uniform_of(r.r0);
        nxt.len[u] = __builtin_amdgcn_readfirstlane(r.len);
        const int pk = __builtin_amdgcn_readfirstlane(r.pk);
        nxt.loc[u] = pk & ((1 << kRevLocBits) - 1);
        nxt.base[u] = (pk >> kRevLocBits) * d.N;
        // (a buffer load past the descriptor's length gives zero)
        const int shown = nxt.len[u] < 64 ? nxt.len[u] : 64;
        const __amdgpu_buffer_rsrc_t rs = res_rows(d.synb + nxt.r0[u], shown * 8);
        const unsigned long long ev = __builtin_bit_cast(unsigned long long, __builtin_amdgcn_raw_buffer_load_b64(rs, lane * 8, 0, 0));
        nxt.e[u] = make_uint2((unsigned)ev, (unsigned)(ev >> 32));
      }
    }
  }
  // (no branch that depends on the data around the requests of the rows: behind one the compiler can no longer tell
  // which requests are still on their way; below step 0 the rows are step 0's again and are never used)
  const int slot1 = n >= 1 ? (S.slot == 0 ? d.R - 1 : S.slot - 1) : 0;   // (n - 1) mod R
  {
    const __amdgpu_buffer_rsrc_t t2 = res_rows(S.tape2, hi * 4), f1 = res_rows(d.Gacc + (size_t)slot1 * d.BN, hi * 4);
    S.Uc = __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(t2, g0 * 4, 0, kBufNonTemporal));
    S.Gb = __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(f1, g0 * 4, 0, kBufNonTemporal));
    if (HAS_DU) {
      const __amdgpu_buffer_rsrc_t u1 = res_rows(S.du1, hi * 4);
      S.dUb = __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(u1, g0 * 4, 0, kBufNonTemporal));
    }
  }
  // this step's gathers two and more steps away: rows n + 2 and later, complete since the barrier before last
  // (every lane of a wavefront with a spike loads: one without such an entry reads a cell of this step's own row and drops it)
  cur.ok = 0u;
  float far_raw[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    far_raw[u] = 0.0f;
    if (cur.len[u] > 0) {   // (the same in every lane)
      const int D = (int)(cur.e[u].x & d.dmask);
      const bool ok = lane < cur.len[u] && D <= near_h;
      cur.ok |= ok ? 1u << u : 0u;
      const bool far = ok && D >= 2;
      far_raw[u] = ld_agent(&gwin[(size_t)(far ? D : 0) * d.BN + (size_t)cur.base[u] + (far ? cur.e[u].x >> d.dbits : 0u)]);
    }
  }
  if (__ballot(S.actmask != 0u) != 0ull) {   // (wavefronts without neurons skip the arithmetic)
    // the whole row without the near parts of the queue terms: final for every neuron that does not spike
    // (the membrane value the step started from matters to spiking neurons only: they are done again below)
    res_v4f gu4;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      float gu;
      S.carry[c] = bwd_update(d, n, U[c], 0.0f, (smask >> c) & 1u, S.carry[c], S.dLc[c], Gf[c], dU[c], &gu);
      gu4[c] = gu;
    }
    const __amdgpu_buffer_rsrc_t row = res_rows(gwin, hi * 4), far = res_rows(d.Gacc + (size_t)S.slot * d.BN, hi * 4);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(res_v4i, gu4), row, g0 * 4, 0, kBufAgent);
    // the far queue terms are used up: the slot is another step's R steps on (stored by every lane, set or not)
    const res_v4i z = {0, 0, 0, 0};
    __builtin_amdgcn_raw_buffer_store_b128(z, far, g0 * 4, 0, 0);
  }
  // ---- row n + 1 is in place once every block has arrived
  if (wait) rev_wait(d, wait_for, s_dead);
  float Gx[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // near parts that come back to the owner directly (spikes that did not fit the list)
  if (near_h >= 1) {
    float near_raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      near_raw[u] = 0.0f;
      if (cur.len[u] > 0) {   // (the same in every lane)
        const bool near = ((cur.ok >> u) & 1u) && (int)(cur.e[u].x & d.dmask) == 1;
        near_raw[u] = ld_agent(&gwin[(size_t)(near ? d.BN : 0) + (size_t)cur.base[u] + (near ? cur.e[u].x >> d.dbits : 0u)]);
      }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (cur.len[u] == 0) { cur.gv[u] = 0.0f; continue; }   // uniform: no spike in this place of the batch
      const bool ok = (cur.ok >> u) & 1u;
      cur.gv[u] = !ok ? 0.0f : ((int)(cur.e[u].x & d.dmask) == 1 ? near_raw[u] : far_raw[u]);
      float part = wave_sum_f(__uint_as_float(cur.e[u].y) * cur.gv[u]);
      part += rev_row_tail(d, gwin, near_h, cur.r0[u], cur.len[u], cur.base[u], 64, ok);
      if (lane == 0) s_G[cur.loc[u]] = part;
    }
    // more than 32 listed spikes in the block: the rest one at a time
    for (int x = wave + 4 * kWaves; x < S.nspk_cur; x += kWaves) {
      const RevSpike r = s_spk[PAR][x];
      const long long rr0 = uniform_of(r.r0);
      const int len = __builtin_amdgcn_readfirstlane(r.len), pk = __builtin_amdgcn_readfirstlane(r.pk);
      const float part = rev_row_tail(d, gwin, near_h, rr0, len, (pk >> kRevLocBits) * d.N, 0, true);
      if (lane == 0) s_G[pk & ((1 << kRevLocBits) - 1)] = part;
    }
    // more spikes than the list holds: the owner's wavefront takes them one by one
    if (__ballot(S.ovf_cur != 0u) != 0ull) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        unsigned long long m = __ballot((S.ovf_cur >> c) & 1u);
        while (m) {
          const int L = __ffsll((long long)m) - 1;
          m &= m - 1;
          const long long rr0 = lane_get(S.r0[c], L);
          const int len = lane_get(S.rlen[c], L);
          const int base = trial_of(d, lane_get(g0, L) + c) * d.N;
          const float part = rev_row_tail(d, gwin, near_h, rr0, len, base, 0, true);
          if (lane == L) Gx[c] = part;
        }
      }
    }
    __syncthreads();
  } else {
#pragma unroll
    for (int u = 0; u < 4; ++u) cur.gv[u] = 0.0f;
  }
  // the spiking neurons again, with their whole queue term and the membrane value the step started from
  if (smask) {
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      if (!((smask >> c) & 1u)) continue;
      float G = Gf[c] + Gx[c];
      if (near_h >= 1 && S.rlen[c] > 0 && !((S.ovf_cur >> c) & 1u)) G += s_G[4 * (int)threadIdx.x + c];
      float gu;
      S.carry[c] = bwd_update(d, n, U[c], S.Ub[c], true, 0.0f, S.dLc[c], G, dU[c], &gu);
      st_agent(&gwin[g0 + c], gu);
    }
  }
  if (threadIdx.x == 0) s_nspk[PAR] = 0;
  rev_arrive(d, !last, 0);   // (a worker adds no arrival)
  // ---- after the arrival, off the chain: per-synapse sums of this step's first batch (no load is issued here)
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (cur.len[u] > 0 && ((cur.ok >> u) & 1u)) unsafeAtomicAdd(&d.gsum[cur.r0[u] + lane], cur.gv[u]);
  // on to the next step
  S.nspk_cur = nspk_nxt; S.ovf_cur = ovf_nxt;
  S.Ua = S.Ub; S.Ub = S.Uc; S.Ga = S.Gb; S.dUa = S.dUb;
  S.slot = slot1;
  if (n >= 3) S.tape2 -= d.BN;
  if (HAS_DU && n >= 2) S.du1 -= d.BN;
  S.gwin -= d.BN;
  S.n = n - 1; S.phi -= 1; S.tail += 1;
}

// Reverse steps n_hi - 1, n_hi - 2, ..., n_hi - nsteps, all inside one window.  P taking-part blocks
// (every stride-th block of the grid), each owning `chunk` <= 2,048 neurons, four consecutive ones
// per thread (16-byte accesses); B N a multiple of 4.  bar_base: value of the barrier counter when
// the launch begins.  HAS_DU: a cotangent on the membrane values comes with the call.
// The block's last wavefront owns no neurons: it only passes the block's barriers, polls the
// grid barrier and adds the block's arrival (a poll never waits behind a worker's requests).
template <bool HAS_DU>
__global__ __launch_bounds__(kResLaunch) void k_bwd_xcd(long long n_hi, int nsteps, long long T, unsigned bar_base, int P,
                                                         int chunk, int stride, const float* __restrict__ dL_dcount,
                                                         const float* __restrict__ dL_dU, Dev d) {
  __shared__ int s_dead, s_nspk[2];
  __shared__ RevSpike s_spk[2][kRevList];     // the block's spikes of the step being run and of the step being prepared
  __shared__ float s_G[4 * kResThreads];      // near part of the queue term of every listed spike, by its neuron's place
  if (blockIdx.x % stride) return;
  const int rank = blockIdx.x / stride;
  if (rank >= P) return;
  if (threadIdx.x == 0) { s_dead = (ld_agent(&d.ctr->err) & ERR_BARRIER) ? 1 : 0; s_nspk[0] = 0; s_nspk[1] = 0; }
  const bool worker = threadIdx.x < kResThreads;   // uniform per wavefront
  const int phi0 = (int)((n_hi - 1) & (long long)(d.W - 1));
  const long long tail0 = T - n_hi < 0x3fffffffLL ? T - n_hi : 0x3fffffffLL;
  if (!worker) {
    // the block barriers of a step, in the workers' order: list of the next step complete, grid barrier, near parts
    // of the queue terms complete, arrival
    __syncthreads();
    for (int k = 0; k < nsteps; ++k) {
      const bool last = k + 1 == nsteps;
      const int near_h = rev_near(d, phi0 - k, (int)tail0 + k);
      const int near1 = last ? 0 : rev_near(d, phi0 - k - 1, (int)tail0 + k + 1);
      if (near1 >= 1) __syncthreads();
      if (k > 0) rev_wait(d, bar_base + (unsigned)k * (unsigned)P, &s_dead);
      if (near_h >= 1) __syncthreads();
      rev_arrive(d, !last, rank);   // (the launch's last step arrives nowhere)
    }
    return;
  }
  const int lo = rank * chunk;
  RevState S;
  S.hi = lo + chunk < d.BN ? lo + chunk : d.BN;
  S.g0 = lo + 4 * (int)threadIdx.x;
  S.actmask = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int g = S.g0 + c;
    S.rlen[c] = 0; S.r0[c] = 0; S.carry[c] = 0.0f; S.dLc[c] = 0.0f;
    if (g < S.hi) {
      S.actmask |= 1u << c;
      const int i = g - trial_of(d, g) * d.N;
      S.r0[c] = d.row_ptr[i];
      S.rlen[c] = (int)(d.row_ptr[i + 1] - S.r0[c]);
      S.carry[c] = d.bwd_carry[g];
      if (dL_dcount) S.dLc[c] = dL_dcount[g];
    }
  }
  auto load_row = [&](const float* p) {
    const __amdgpu_buffer_rsrc_t rs = res_rows(p, S.hi * 4);
    return __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, S.g0 * 4, 0, kBufNonTemporal));
  };
  const res_v4f zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
  S.n = n_hi - 1; S.phi = phi0; S.tail = (int)tail0;
  S.slot = (int)((n_hi - 1) % d.R);   // (one division per launch)
  S.gwin = gwin_of(d, n_hi - 1) + (size_t)phi0 * d.BN;
  S.tape2 = d.tapeU + (size_t)(n_hi >= 3 ? n_hi - 3 : 0) * d.BN;
  S.du1 = HAS_DU ? dL_dU + (size_t)(n_hi >= 2 ? n_hi - 2 : 0) * d.BN : nullptr;
  S.Ua = load_row(d.tapeU + (size_t)(n_hi - 1) * d.BN);
  S.Ub = n_hi >= 2 ? load_row(d.tapeU + (size_t)(n_hi - 2) * d.BN) : zero4;
  S.Uc = zero4;
  S.Ga = load_row(d.Gacc + (size_t)S.slot * d.BN); S.Gb = zero4;
  S.dUa = HAS_DU ? load_row(dL_dU + (size_t)(n_hi - 1) * d.BN) : zero4; S.dUb = zero4;
  S.nspk_cur = 0; S.ovf_cur = 0;   // (the launch's first step has no listed spike: nothing arrives after it inside the window)
  RevBatch A, B;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    A.e[u] = make_uint2(0u, 0u); A.gv[u] = 0.0f; A.r0[u] = 0; A.len[u] = 0; A.base[u] = 0; A.loc[u] = 0;
    B.e[u] = make_uint2(0u, 0u); B.gv[u] = 0.0f; B.r0[u] = 0; B.len[u] = 0; B.base[u] = 0; B.loc[u] = 0;
  }
  A.ok = 0u; B.ok = 0u;
  __builtin_amdgcn_s_waitcnt(0x0F70);   // (the loop starts with nothing on its way: see rev_arrive)
  __syncthreads();
  for (int k = 0; k < nsteps; ++k) {
    rev_step<HAS_DU>(d, S, k & 1, A, B, k + 1 == nsteps, k > 0, bar_base + (unsigned)k * (unsigned)P, &s_dead, s_nspk, s_spk, s_G, dL_dU);
    A = B;
  }
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if ((S.actmask >> c) & 1u) d.bwd_carry[S.g0 + c] = S.carry[c];
}
