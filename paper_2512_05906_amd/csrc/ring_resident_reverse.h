// Ring queue, reverse sweep: the steps of one window in ONE launch on the blocks of one XCD
// (delta synapse).  Included by adseq.hip after ring_window.h and ring_resident.h, whose layout
// (ResMap: four consecutive neurons per thread and group, 16-byte accesses), barrier (res_wait /
// res_arrive: bounded waits, ERR_BARRIER) and agent-scope accesses it shares.
//
// The reverse step n (bwd_update; Section 3.2 eqs. 13 and 17 carried back through the steps) needs
// from step n + 1 the carry of its own neuron and, for the entries of its spikes' rows that arrive
// one step later, row n + 1 of the adjoint window -- nothing else.  And unlike the forward pass the
// reverse sweep KNOWS its spikes: they are on the tape.  So a block prepares a step ahead of time:
// tape values two steps ahead, far queue terms and loss terms one step ahead; while it waits for the
// barrier of step n it lists its spikes of step n - 1 and requests the leading 64 entries of their
// rows; after its arrival at that barrier it gathers every adjoint those entries need two or more
// steps away (rows that are complete by then).  A neuron that does not spike at step n needs nothing
// of any other neuron, so the whole row n is computed and stored before the barrier as well, with
// the near parts of the queue terms left out.  Behind the barrier only the gathers one step away
// are left (row n + 1 was written through the L2s a moment ago), then the per-spike sums and the few
// spiking neurons again with their whole queue term (a spiking neuron's update does not use the
// carry: the reset cuts it); their cells are stored again and acknowledged before the block
// arrives.  The per-synapse gradient sums (atomic adds into gsum, read only when the sweep is over)
// are issued after the arrival.  The carry stays in registers for the whole launch.
//
// Same arithmetic as k_bwd_step_win; the order in which a spike's terms are added differs (fp32
// rounding only).  Results do not depend on where the blocks run: what crosses blocks goes
// through agent-scope stores and loads and the barrier counter.

#ifdef ADSEQ_PHASE_CLOCK
// builds with phase clocks: thread 0 of block 0 adds the 10 ns ticks since its last mark to Counters::phase[16 + i]
#define RPH_BEGIN unsigned long long rpc[8] = {0, 0, 0, 0, 0, 0, 0, 0}, rpt = wall_clock64();
#define RPH(i) { const unsigned long long t_ = wall_clock64(); rpc[i] += t_ - rpt; rpt = t_; }
#define RPH_SETTLE wait_all_memory();
#define RPH_END if (threadIdx.x == 0 && rank == 0) for (int i = 0; i < 8; ++i) atomicAdd(&d.ctr->phase[16 + i], rpc[i]);
#else
#define RPH_BEGIN
#define RPH(i)
#define RPH_SETTLE
#define RPH_END
#endif

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
__device__ __forceinline__ void rev_arrive(const Dev& d, bool arrive) {
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0); the other counters at their maximum
  __syncthreads();
  if (arrive && threadIdx.x == kResThreads) atomicAdd(&d.ctr->bar[0], 1u);
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
      const uint2 e = d.synb[r0 + q0 + lane];
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

// Reverse steps n_hi - 1, n_hi - 2, ..., n_hi - nsteps, all inside one window.  P taking-part blocks
// (every stride-th block of the grid), each owning `chunk` <= 2,048 neurons, four consecutive ones
// per thread (16-byte accesses); B N a multiple of 4.  bar_base: value of the barrier counter when
// the launch begins.  HAS_DU: a cotangent on the membrane values comes with the call.
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
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const bool worker = threadIdx.x < kResThreads;   // uniform per wavefront; the last wavefront only synchronises
  const int lo = rank * chunk;
  const int hi = worker ? (lo + chunk < d.BN ? lo + chunk : d.BN) : 0;
  constexpr int kWaves = kResThreads / 64;
  const int g0 = lo + 4 * (int)threadIdx.x;
  int rlen[4];
  long long r0[4];
  float carry[4], dLc[4];
  unsigned actmask = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const int g = g0 + c;
    rlen[c] = 0; r0[c] = 0; carry[c] = 0.0f; dLc[c] = 0.0f;
    if (g < hi) {
      actmask |= 1u << c;
      const int i = g - trial_of(d, g) * d.N;
      r0[c] = d.row_ptr[i];
      rlen[c] = (int)(d.row_ptr[i + 1] - r0[c]);
      carry[c] = d.bwd_carry[g];
      if (dL_dcount) dLc[c] = dL_dcount[g];
    }
  }
  auto near_of = [&](long long n) {
    int h = d.W - 1 - (int)(n & (long long)(d.W - 1));
    if (h > d.d_max) h = d.d_max;
    if ((long long)h > T - 1 - n) h = (int)(T - 1 - n);   // arrivals n + D >= T were never delivered
    return h;
  };
  auto load_row = [&](const float* p) {
    const __amdgpu_buffer_rsrc_t rs = res_rows(p, hi * 4);
    return __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, g0 * 4, 0, kBufNonTemporal));
  };
  const res_v4f zero4 = {0.0f, 0.0f, 0.0f, 0.0f};
  // tape values of the step being run, of the one after it and of the one after that; far queue terms and dL/dU of
  // the step being run and of the next
  res_v4f Ua = load_row(d.tapeU + (size_t)(n_hi - 1) * d.BN);
  res_v4f Ub = n_hi >= 2 ? load_row(d.tapeU + (size_t)(n_hi - 2) * d.BN) : zero4, Uc = zero4;
  res_v4f Ga = load_row(d.Gacc + (size_t)((n_hi - 1) % d.R) * d.BN), Gb = zero4;
  res_v4f dUa = HAS_DU ? load_row(dL_dU + (size_t)(n_hi - 1) * d.BN) : zero4, dUb = zero4;
  RevBatch cur, nxt;
#pragma unroll
  for (int u = 0; u < 4; ++u) { cur.e[u] = make_uint2(0u, 0u); cur.gv[u] = 0.0f; cur.r0[u] = 0; cur.len[u] = 0; cur.base[u] = 0; cur.loc[u] = 0; }
  cur.ok = 0u;
  int nspk_cur = 0;          // listed spikes of the step being run (its first step has none: nothing arrives after it inside the window)
  unsigned ovf_cur = 0;      // bit c: neuron c of this thread spiked and did not fit the list
  int par = 0;               // list buffer of the step being run
  int slot = (int)((n_hi - 1) % d.R);   // row of the far queue terms of the step being run (one division per launch)
  __builtin_amdgcn_s_waitcnt(0x0F70);   // (the loop starts with nothing on its way: see rev_arrive)
  __syncthreads();
  RPH_BEGIN
  for (int k = 0; k < nsteps; ++k) {
    const long long n = n_hi - 1 - k;
    const int phi = (int)(n & (long long)(d.W - 1));
    const int near_h = near_of(n);
    float* __restrict__ gwin = gwin_of(d, n) + (size_t)phi * d.BN;   // row of this step; an arrival offset D lies D rows on
    const __amdgpu_buffer_rsrc_t row = res_rows(gwin, hi * 4);
    // ---- before the barrier: nothing here depends on the step before.  Every load of the step is requested here, the
    // ones that go furthest first, and none after the arrival: what was requested is complete when the gathers behind the
    // barrier are, so that no wait for an old request turns into a wait for a new one.
    float U[4], Gf[4], dU[4];
    unsigned smask = 0, s1 = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      U[c] = Ua[c]; Gf[c] = Ga[c]; dU[c] = HAS_DU ? dUa[c] : 0.0f;
      smask |= U[c] >= d.theta ? 1u << c : 0u;
      s1 |= Ub[c] >= d.theta ? 1u << c : 0u;
    }
    smask &= actmask; s1 &= actmask;
    RPH(0)   // this step's own values
    // the step after this one: list of the block's spikes, the leading 64 entries of their rows requested
    const int near1 = k + 1 < nsteps ? near_of(n - 1) : 0;   // uniform over the launch
    int nspk_nxt = 0;
    unsigned ovf_nxt = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) { nxt.e[u] = make_uint2(0u, 0u); nxt.gv[u] = 0.0f; nxt.r0[u] = 0; nxt.len[u] = 0; nxt.base[u] = 0; nxt.loc[u] = 0; }
    nxt.ok = 0u;
    if (near1 >= 1) {
      if (__ballot(s1 != 0u) != 0ull) {
        unsigned long long m[4];
        int total = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) { m[c] = __ballot((s1 >> c) & 1u); total += __popcll(m[c]); }
        int at = 0;
        if (lane == 0) at = atomicAdd(&s_nspk[par ^ 1], total);
        at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          if (m[c] == 0ull) continue;   // uniform
          if ((m[c] >> lane) & 1ull) {
            const int idx = at + __popcll(m[c] & ((1ull << lane) - 1ull));
            if (idx < kRevList) {
              RevSpike r;
              r.r0 = r0[c]; r.len = rlen[c];
              r.pk = (4 * (int)threadIdx.x + c) | (trial_of(d, g0 + c) << kRevLocBits);
              s_spk[par ^ 1][idx] = r;
            } else {
              ovf_nxt |= 1u << c;
            }
          }
          at += __popcll(m[c]);
        }
      }
      __syncthreads();
      nspk_nxt = s_nspk[par ^ 1] < kRevList ? s_nspk[par ^ 1] : kRevList;
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int x = wave + u * kWaves;
        const bool have = worker && x < nspk_nxt;   // uniform
        const RevSpike r = s_spk[par ^ 1][have ? x : 0];
        nxt.r0[u] = have ? uniform_of(r.r0) : 0;
        nxt.len[u] = have ? __builtin_amdgcn_readfirstlane(r.len) : 0;
        const int pk = have ? __builtin_amdgcn_readfirstlane(r.pk) : 0;
        nxt.loc[u] = pk & ((1 << kRevLocBits) - 1);
        nxt.base[u] = (pk >> kRevLocBits) * d.N;
        // (a buffer load past the descriptor's length gives zero: no branch, and so no wait, between the four requests)
        if (nxt.len[u] > 0) {   // (the same in every lane: a wavefront without a spike requests nothing)
          const int shown = nxt.len[u] < 64 ? nxt.len[u] : 64;
          const __amdgpu_buffer_rsrc_t rs = res_rows(d.synb + nxt.r0[u], shown * 8);
          const unsigned long long ev = __builtin_bit_cast(unsigned long long, __builtin_amdgcn_raw_buffer_load_b64(rs, lane * 8, 0, 0));
          nxt.e[u] = make_uint2((unsigned)ev, (unsigned)(ev >> 32));
        }
      }
    }
    RPH(1)   // list of the next step's spikes, their rows requested
    // (no branch around a request, here or below: behind a branch the compiler can no longer tell which requests
    // are still on their way, and waits for all of them at the next use of any; below step 0 the rows are
    // step 0's again and are never used)
    Uc = load_row(d.tapeU + (size_t)(n >= 2 ? n - 2 : 0) * d.BN);
    const int slot1 = n >= 1 ? (slot == 0 ? d.R - 1 : slot - 1) : 0;   // (n - 1) mod R
    Gb = load_row(d.Gacc + (size_t)slot1 * d.BN);
    if (HAS_DU) dUb = load_row(dL_dU + (size_t)(n >= 1 ? n - 1 : 0) * d.BN);
    // this step's gathers two and more steps away: rows n + 2 and later, complete since the barrier before last
    // (every lane loads: one without such an entry reads the first cell of this step's own row and drops it)
    cur.ok = 0u;
    float far_raw[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int D = (int)(cur.e[u].x & d.dmask);
      const bool ok = lane < cur.len[u] && D <= near_h;
      cur.ok |= ok ? 1u << u : 0u;
      const bool far = ok && D >= 2;
      far_raw[u] = 0.0f;
      if (cur.len[u] > 0)   // (the same in every lane)
        far_raw[u] = ld_agent(&gwin[(size_t)(far ? D : 0) * d.BN + (size_t)cur.base[u] + (far ? cur.e[u].x >> d.dbits : 0u)]);
    }
    RPH(2)   // requests of the next steps' values, this step's far gathers
    if (__ballot(actmask != 0u) != 0ull) {   // (wavefronts without neurons skip the arithmetic)
      // the whole row without the near parts of the queue terms: final for every neuron that does not spike
      res_v4f gu4;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        float gu;
        carry[c] = bwd_update(d, n, U[c], 0.0f, (smask >> c) & 1u, carry[c], dLc[c], Gf[c], dU[c], &gu);
        gu4[c] = gu;
      }
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(res_v4i, gu4), row, g0 * 4, 0, kBufAgent);
    }
    {
      // the far queue terms are used up: the slot is another step's R steps on (stored by every lane, set or not)
      const __amdgpu_buffer_rsrc_t far = res_rows(d.Gacc + (size_t)slot * d.BN, hi * 4);
      const res_v4i z = {0, 0, 0, 0};
      __builtin_amdgcn_raw_buffer_store_b128(z, far, g0 * 4, 0, 0);
    }
    RPH(3)   // the row without near parts
    // ---- row n + 1 is in place once every block has arrived
    if (k > 0) res_wait(d, bar_base + (unsigned)k * (unsigned)P, &s_dead);
    RPH(4)   // barrier
    float Gx[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // near parts that come back to the owner directly (spikes that did not fit the list)
    {
      float near_raw[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const bool near = ((cur.ok >> u) & 1u) && (int)(cur.e[u].x & d.dmask) == 1;
        near_raw[u] = 0.0f;
        if (cur.len[u] > 0)   // (the same in every lane)
          near_raw[u] = ld_agent(&gwin[(size_t)(near ? d.BN : 0) + (size_t)cur.base[u] + (near ? cur.e[u].x >> d.dbits : 0u)]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int D = (int)(cur.e[u].x & d.dmask);
        cur.gv[u] = !((cur.ok >> u) & 1u) ? 0.0f : (D == 1 ? near_raw[u] : far_raw[u]);
      }
    }
    if (near_h >= 1) {
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int x = wave + u * kWaves;
        if (!(worker && x < nspk_cur)) continue;   // uniform
        const bool ok = (cur.ok >> u) & 1u;
        float part = wave_sum_f(ok ? __uint_as_float(cur.e[u].y) * cur.gv[u] : 0.0f);
        part += rev_row_tail(d, gwin, near_h, cur.r0[u], cur.len[u], cur.base[u], 64, ok);
        if (lane == 0) s_G[cur.loc[u]] = part;
      }
      // more than 32 listed spikes in the block: the rest one at a time
      for (int x = wave + 4 * kWaves; worker && x < nspk_cur; x += kWaves) {
        const RevSpike r = s_spk[par][x];
        const long long rr0 = uniform_of(r.r0);
        const int len = __builtin_amdgcn_readfirstlane(r.len), pk = __builtin_amdgcn_readfirstlane(r.pk);
        const float part = rev_row_tail(d, gwin, near_h, rr0, len, (pk >> kRevLocBits) * d.N, 0, true);
        if (lane == 0) s_G[pk & ((1 << kRevLocBits) - 1)] = part;
      }
      // more spikes than the list holds: the owner's wavefront takes them one by one
      if (__ballot(ovf_cur != 0u) != 0ull) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          unsigned long long m = __ballot((ovf_cur >> c) & 1u);
          while (m) {
            const int L = __ffsll((long long)m) - 1;
            m &= m - 1;
            const long long rr0 = lane_get(r0[c], L);
            const int len = lane_get(rlen[c], L);
            const int base = trial_of(d, lane_get(g0, L) + c) * d.N;
            const float part = rev_row_tail(d, gwin, near_h, rr0, len, base, 0, true);
            if (lane == L) Gx[c] = part;
          }
        }
      }
      __syncthreads();
    }
    RPH(5)   // gathers one step away, sums
    // the spiking neurons again, with their whole queue term and the membrane value the step started from
    if (smask) {
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (!((smask >> c) & 1u)) continue;
        float G = Gf[c] + Gx[c];
        if (near_h >= 1 && !((ovf_cur >> c) & 1u)) G += s_G[4 * (int)threadIdx.x + c];
        float gu;
        carry[c] = bwd_update(d, n, U[c], Ub[c], true, 0.0f, dLc[c], G, dU[c], &gu);
        st_agent(&gwin[g0 + c], gu);
      }
    }
    if (threadIdx.x == 0) s_nspk[par] = 0;
    rev_arrive(d, k + 1 < nsteps);   // (the launch's last step arrives nowhere)
    RPH(6)   // spiking neurons again, stores acknowledged, arrival
    // ---- after the arrival, off the chain: per-synapse sums of this step's first batch (no load is issued here)
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if ((cur.ok >> u) & 1u) unsafeAtomicAdd(&d.gsum[cur.r0[u] + lane], cur.gv[u]);
    RPH(7)   // per-synapse sums issued
    cur = nxt; nspk_cur = nspk_nxt; ovf_cur = ovf_nxt; par ^= 1;
    Ua = Ub; Ub = Uc; Ga = Gb; dUa = dUb;
    slot = slot1;
  }
  RPH_END
#pragma unroll
  for (int c = 0; c < 4; ++c)
    if ((actmask >> c) & 1u) d.bwd_carry[g0 + c] = carry[c];
}
