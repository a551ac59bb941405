// Ring queue, reverse sweep one WINDOW at a time (delta synapse).  Included by adseq.hip after
// ring_window.h.
//
// The reverse recursion (Section 3.2 eqs. 13 and 17 carried back through the steps; see
// bwd_update) is linear in the adjoint, and neurons are coupled only through the queue terms of
// the spikes: a few hundred neurons per step out of 100,000.  Per neuron,
//   gU[n] = (1 - s[n]) c[n+1] + sigma'(U[n] - theta) (dL/dcount + s[n] G[n]) + dL/dU[n],  c[n] = alpha gU[n] + E[n],
// and G[n] = far part (arrivals in later windows: already in Gacc) + near part (arrivals inside
// the window of n).  So a window of W steps is swept in three passes instead of W launches:
//   1. k_bwd_dense_win   every neuron runs its own W steps with the near parts left out (one
//                        thread per neuron, no coupling at all: a stream over the tape);
//   2. k_bwd_near_stage  the near events of the window's spikes (the front of each sorted row) are
//                        staged per emission step: target cell, amplitude, the spike's number within
//                        its step (whole chip, once per window);
//      k_bwd_near_seq    one workgroup goes through the steps from the last to the first: the staged
//                        events of a step gather their adjoints (final by then), sum a * adjoint per
//                        spike in LDS, and each spike's correction sigma' G_near is added to its own
//                        cell and carried down its neuron's column, alpha per step, until the
//                        neuron's previous spike (a reset cuts the carry) or into the carry of the
//                        next window.  Between two steps: a workgroup barrier, not a launch.
//   3. k_bwd_win         as before gathers, for all earlier spikes, the far queue terms that arrive
//                        in the window (into Gacc) and the per-synapse sums; it now also takes the
//                        window's own spikes for the per-synapse sums of their near events.
// Each adjoint cell is corrected by at most one spike (its neuron's next spike later in the
// window), so the corrections are single-writer.  The host checks, from counts taken over the tape
// before the sweep, that a window's spikes and near events fit the staging arrays, and sweeps a
// window that does not with the launches per step (k_bwd_step_win).

constexpr int kNearSpikeCap = 8192;    // spikes of one step whose near sums the sequential pass keeps in LDS
constexpr int kNearOrdBits = 26;       // staged record: spike number in the low bits, window row above them

// Spikes of every step n < T and (an upper bound of) their near events: entries with arrival offset
// <= W - 1 - (n mod W).  One block per step; counts[n] and counts[T + n].
__global__ __launch_bounds__(kBlock) void k_bwd_near_counts(Dev d, long long T, int* __restrict__ counts) {
  __shared__ int red[2][kBlock / 64];
  for (long long n = blockIdx.x; n < T; n += gridDim.x) {
    int near_h = d.W - 1 - (int)(n & (long long)(d.W - 1));
    if (near_h > d.d_max) near_h = d.d_max;
    long long c0 = 0, c1 = 0;
    for (int w = threadIdx.x; w < d.words; w += kBlock) {
      unsigned long long bits = d.tape_bits[(size_t)n * d.words + w];
      while (bits) {
        const int bit = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        const long long g = (long long)w * 64 + bit;
        if (g >= d.BN) break;
        const int i = (int)g - trial_of(d, (int)g) * d.N;
        c0 += 1;
        if (near_h >= 1) c1 += d.nearcnt[(size_t)near_h * d.N + i];
      }
    }
    c0 = wave_sum(c0); c1 = wave_sum(c1);
    if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = (int)(c0 > 0x7fffffff ? 0x7fffffff : c0); red[1][threadIdx.x >> 6] = (int)(c1 > 0x3fffffff ? 0x3fffffff : c1); }
    __syncthreads();
    if (threadIdx.x == 0) {
      long long a = 0, b = 0;
      for (int w = 0; w < kBlock / 64; ++w) { a += red[0][w]; b += red[1][w]; }
      counts[n] = (int)(a > 0x7fffffff ? 0x7fffffff : a);
      counts[T + n] = (int)(b > 0x7fffffff ? 0x7fffffff : b);
    }
    __syncthreads();
  }
}

// Pass 1: steps k0 + nsteps - 1 .. k0 (all inside one window) for every neuron on its own, near
// parts of the queue terms left out.  Writes the adjoint rows of the window, the carry into the
// step before k0, and the neuron's spikes of the window as a bit mask (bit = step - k0).
__global__ __launch_bounds__(kBlock) void k_bwd_dense_win(long long k0, int nsteps, const float* __restrict__ dL_dcount,
                                                          const float* __restrict__ dL_dU, Dev d) {
  const int g = blockIdx.x * kBlock + threadIdx.x;
  if (g >= d.BN) return;
  float* __restrict__ gwin = gwin_of(d, k0);
  float c = d.bwd_carry[g];
  const float inner = dL_dcount ? dL_dcount[g] : 0.0f;
  const bool spike_time = d.surrogate == ADSEQ_GRAD_SPIKE_TIME;
  unsigned long long mask = 0ull;
  long long n = k0 + nsteps - 1;
  int slot = (int)(n % d.R);
  // the tape values of eight steps are requested at once (a thread's steps depend on one another
  // only through the carry, so nothing but the loads' latency would pace the loop otherwise)
  for (int phi_hi = nsteps - 1; phi_hi >= 0; phi_hi -= 8) {
    float Ub[9], dUb[8];
#pragma unroll
    for (int t = 0; t < 9; ++t) {
      const long long m = k0 + phi_hi - t;        // step of Ub[t]; Ub[8] is only the "step before" of Ub[7]
      // (a step's own value, or -- spike-time rule only -- the value of the step before the last one wanted)
      Ub[t] = (m >= 0 && (phi_hi - t >= 0 || (spike_time && phi_hi - t >= -1))) ? d.tapeU[(size_t)m * d.BN + g] : 0.0f;
    }
#pragma unroll
    for (int t = 0; t < 8; ++t)
      dUb[t] = (dL_dU && phi_hi - t >= 0) ? dL_dU[(size_t)(k0 + phi_hi - t) * d.BN + g] : 0.0f;
#pragma unroll
    for (int t = 0; t < 8; ++t) {
      const int phi = phi_hi - t;
      if (phi < 0) break;
      const float U = Ub[t];
      const bool s = U >= d.theta;
      float G = 0.0f;
      if (s) {
        float* ga = &d.Gacc[(size_t)slot * d.BN + g];
        G = *ga;
        if (G != 0.0f) *ga = 0.0f;
        mask |= 1ull << phi;
      }
      float gu;
      c = bwd_update(d, n, U, Ub[t + 1], s, c, inner, G, dUb[t], &gu);
      gwin[(size_t)phi * d.BN + g] = gu;
      --n;
      if (--slot < 0) slot = d.R - 1;
    }
  }
  d.bwd_carry[g] = c;
  d.wspk[g] = mask;
}

// Pass 2a: stages the near events of the spikes of steps [k0, k1) (one window), per emission
// step: record {target state index, amplitude bits, spike number within its step | window row of
// the arrival << 26}; the spike table holds the neuron of every numbered spike.  Spikes without
// near events get no number.  As virtual block vb of nvb.
__global__ __launch_bounds__(kRingThreads) void k_bwd_near_stage(Dev d, long long k0, long long k1, long long T, int nvb) {
  __shared__ ExpandLds L;
  if (threadIdx.x == 0) { L.qn = 0; L.qhead = 0; }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  auto stage = [&](const Seg& o) {
    const int phi = -o.dlo;   // emission step - k0 (the walk hands down dlo = k0 - step)
    int ord = 0, at = 0;
    if (lane == 0) { ord = atomicAdd(&d.near_nspk[phi], 1); at = atomicAdd(&d.near_nev[phi], o.len); }
    ord = __builtin_amdgcn_readfirstlane(ord);
    at = __builtin_amdgcn_readfirstlane(at);
    // (the host has checked that the window fits; the bounds only keep a miscount from writing outside)
    if (ord >= kNearSpikeCap || at + o.len > d.near_ev_cap) { atomicOr(&d.ctr->err, ERR_TAPE_EVENTS); return; }
    if (lane == 0) d.near_spk[(size_t)phi * kNearSpikeCap + ord] = (int)o.g;
    for (int q = lane; q < o.len; q += 64) {
      const uint2 e = d.synb[o.p0 + q];
      const unsigned row = (unsigned)((int)(e.x & d.dmask) - o.dlo);
      d.near_ev[(size_t)phi * d.near_ev_cap + at + q] =
          make_uint4((unsigned)o.base + (e.x >> d.dbits), e.y, (unsigned)ord | (row << kNearOrdBits), 0u);
    }
  };
  long long cnt[3] = {0, 0, 0};
  walk_segments(d, L, d.tape_bits, false, k0, k0, k1, T, (int)blockIdx.x, nvb, k1, cnt, stage);
  const int qn = L.qn < kSegQueue ? L.qn : kSegQueue;
  for (int t = threadIdx.x >> 6; t < qn; t += kRingWaves) stage(L.q[t]);
}

// What the near part Gn of a spike's queue term adds to its adjoint (*dgu) and to the carry it
// hands to the step before (returned): the parts of bwd_update that are linear in G.
__device__ __forceinline__ float bwd_near_correction(const Dev& d, long long n, float U, float Uprev, float Gn, float* dgu) {
  float sg = 0.0f;
  if (d.surrogate == ADSEQ_SURR_SUPERSPIKE) {
    const float x = fabsf(U - d.theta) + 1.0f;
    sg = __builtin_amdgcn_rcpf(x * x);   // (as bwd_update)
  }
  *dgu = sg * Gn;
  float e = 0.0f;
  if (d.surrogate == ADSEQ_GRAD_SPIKE_TIME) {
    const float vprev = n > 0 ? (Uprev >= d.theta ? d.v_reset : Uprev) : 0.0f;
    float vdot = (U - vprev) / d.dt;
    if (vdot == 0.0f) vdot = 1.0f;
    e = -(1.0f / vdot) * (1.0f / d.tau) * Gn;
  }
  return __fmaf_rn(d.alpha, *dgu, e);
}

// Pass 2b: ONE workgroup; steps k0 + nsteps - 2 .. k0 in turn (the window's last step has no
// arrival inside the window).  See the header of this file.
__global__ __launch_bounds__(kRingThreads) void k_bwd_near_seq(Dev d, long long k0, int nsteps) {
  __shared__ float Gn[kNearSpikeCap];
  float* __restrict__ gw = gwin_of(d, k0);
  const bool spike_time = d.surrogate == ADSEQ_GRAD_SPIKE_TIME;
  for (int phi = nsteps - 2; phi >= 0; --phi) {
    const long long n = k0 + phi;
    int ns = d.near_nspk[phi], ne = d.near_nev[phi];
    ns = ns < kNearSpikeCap ? ns : kNearSpikeCap;
    ne = ne < d.near_ev_cap ? ne : d.near_ev_cap;
    if (ns == 0) continue;   // uniform over the workgroup
    for (int x = threadIdx.x; x < ns; x += kRingThreads) Gn[x] = 0.0f;
    __syncthreads();
    const uint4* __restrict__ ev = d.near_ev + (size_t)phi * d.near_ev_cap;
    for (int x = threadIdx.x; x < ne; x += kRingThreads) {
      const uint4 r = ev[x];
      const float gv = ld_agent(&gw[(size_t)(r.z >> kNearOrdBits) * d.BN + r.x]);
      atomicAdd(&Gn[r.z & ((1u << kNearOrdBits) - 1u)], __uint_as_float(r.y) * gv);
    }
    __syncthreads();
    for (int x = threadIdx.x; x < ns; x += kRingThreads) {
      const int g = d.near_spk[(size_t)phi * kNearSpikeCap + x];
      const float U = d.tapeU[(size_t)n * d.BN + g];
      const float Uprev = (spike_time && n > 0) ? d.tapeU[(size_t)(n - 1) * d.BN + g] : 0.0f;
      float dgu;
      float dc = bwd_near_correction(d, n, U, Uprev, Gn[x], &dgu);
      // cells [m_lo, phi) of the neuron's column take the carry, alpha per step down: from the
      // step after the neuron's previous spike in the window (its reset cuts the carry), or from
      // the window's first step, and then the carry goes on into the next window.  Every one of
      // these cells has this spike as its only writer, so all are loaded at once, eight at a time.
      const unsigned long long below = d.wspk[g] & ((1ull << phi) - 1ull);
      const int m_lo = below ? 64 - __clzll((long long)below) : 0;
      float* own = &gw[(size_t)phi * d.BN + g];
      const float own_v = ld_agent(own);
      for (int m_hi = phi - 1; m_hi >= m_lo; m_hi -= 8) {
        float v[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) v[t] = m_hi - t >= m_lo ? ld_agent(&gw[(size_t)(m_hi - t) * d.BN + g]) : 0.0f;
#pragma unroll
        for (int t = 0; t < 8; ++t)
          if (m_hi - t >= m_lo) { gw[(size_t)(m_hi - t) * d.BN + g] = v[t] + dc; dc *= d.alpha; }
      }
      *own = own_v + dgu;
      const int m = below ? 0 : -1;
      if (m < 0) d.bwd_carry[g] += dc;
    }
    // the corrected cells are gathered by the steps before: stores acknowledged, then the barrier
    wait_all_memory();
    __syncthreads();
  }
  // the staging counters are zero again when the next window is staged
  if ((int)threadIdx.x < d.W) { d.near_nspk[threadIdx.x] = 0; d.near_nev[threadIdx.x] = 0; }
}
