// Ring queue, forward: the steps of one window in ONE launch over the whole chip, with the rows of
// the neurons that are ABOUT to spike requested ahead (delta synapse).  Included by adseq.hip after
// ring_resident_reverse.h, whose barrier (rev_wait / rev_arrive: kArriveLines arrival counters, a
// wavefront per block that only synchronises, bounded waits) and list entries it shares.
//
// The chain a forward step cannot avoid is: cells of the row (final once every block has arrived
// from the step before) -> threshold -> the spikes' row entries -> their adds -> acknowledgement.
// k_run_xcd leaves all of it behind the barrier.  Here the trip for the row entries goes in front of it:
// while a block waits for the barrier it reads its cells once ahead of time -- everything is in them
// but the events emitted one step ago -- and lists as candidates the neurons that this early value
// takes to within `margin` of the threshold; the leading 64 entries of the candidates' rows are
// requested then.  Behind the barrier the cells are read again, the update is done for good, and the
// candidates that did spike have their entries in registers already: only the adds are left.  A
// neuron that spikes without having been a candidate (events of the last step lifted it by more
// than the margin), or beyond the 32 candidates a block prefetches, takes the slow way: row load
// behind the barrier, as in k_run_xcd.  The early read decides nothing: same arithmetic, in the
// same order, as k_step_win.
//
// Membrane state, row bounds and the step-independent half of the drive's hash stay in registers
// for the launch; the popped cells are cleared, and tape, spike words and spike counts stored, after
// the arrival.

constexpr int kFwdCand = 32;   // candidates per block and step whose rows are requested ahead (four per worker wavefront)

template <int NPT>
struct FwdState {
  float V[NPT];
  long long r0[NPT]; int rlen[NPT];
  unsigned long long zg[NPT];    // mix64(seed + G (g + 1)): the neuron's half of the drive's hash
  unsigned actmask;
  int g0, hi;
};

// Adds of the entries [q0, len) of a spike's sorted row that arrive inside the window, 64 at a time
// (the rows ascend in the arrival offset); `more`: the group before ended inside the window.
__device__ __forceinline__ void fwd_row_tail(const Dev& d, int* __restrict__ win, int near_h, long long r0, int len,
                                             int base, int q0, bool more) {
  const int lane = threadIdx.x & 63;
  for (; (__ballot(more) >> 63) && q0 < len; q0 += 64) {
    more = false;
    if (q0 + lane < len) {
      const uint2 e = load_stream(&d.synf[r0 + q0 + lane]);
      const int D = (int)(e.x & d.dmask);
      if (D <= near_h) {
        atomicAdd(&win[(size_t)D * d.BN + (size_t)base + (e.x >> d.dbits)], (int)e.y);
        more = true;
      }
    }
  }
}

// Steps n0 .. n0 + nsteps - 1, all inside one window.  P taking-part blocks (every stride-th block of
// the grid), each owning `chunk` <= NPT * 512 neurons, NPT consecutive ones per thread (four; eight for state arrays
// beyond 256 x 2,048 cells; one where a block owns no more neurons than it has threads: a step's instructions then
// spread over all its wavefronts); B N a multiple of 4.  bar_base: sum of the arrival counters when the launch begins.  margin: how far below the
// threshold the early value of a candidate may lie.
template <bool RECORD, int NPT>
__global__ __launch_bounds__(kResLaunch) void k_fwd_chip(long long n0, int nsteps, unsigned bar_base, int P, int chunk,
                                                          int stride, float margin, Dev d) {
  __shared__ int s_dead, s_ncand, s_nslow;
  __shared__ RevSpike s_cand[kFwdCand];            // candidates of the step: row bounds, place | trial << kRevLocBits
  __shared__ RevSpike s_slow[(NPT < 4 ? 4 : NPT) * kResThreads];     // spikes that were no candidates (one entry per neuron at most)
  __shared__ unsigned char s_fired[(NPT < 4 ? 4 : NPT) * kResThreads];   // by the neuron's place in the block: it spiked in this step
  if (blockIdx.x % stride) return;
  const int rank = blockIdx.x / stride;
  if (rank >= P) return;
  if (threadIdx.x == 0) { s_dead = (ld_agent(&d.ctr->err) & ERR_BARRIER) ? 1 : 0; s_ncand = 0; s_nslow = 0; }
  const bool worker = threadIdx.x < kResThreads;   // uniform per wavefront
  if (!worker) {
    // the block barriers of a step, in the workers' order: candidates listed, grid barrier, spikes known, arrival
    __syncthreads();
    for (int k = 0; k < nsteps; ++k) {
      __syncthreads();
      if (k > 0) rev_wait(d, bar_base + (unsigned)k * (unsigned)P, &s_dead);
      __syncthreads();
      rev_arrive(d, k + 1 < nsteps, rank);
    }
    return;
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int kWaves = kResThreads / 64;
  const int lo = rank * chunk;
  FwdState<NPT> S;
  S.hi = lo + chunk < d.BN ? lo + chunk : d.BN;
  S.g0 = lo + NPT * (int)threadIdx.x;
  S.actmask = 0;
  const unsigned long long G64 = 0x9E3779B97F4A7C15ull;
#pragma unroll
  for (int c = 0; c < NPT; ++c) {
    const int g = S.g0 + c;
    S.V[c] = 0.0f; S.r0[c] = 0; S.rlen[c] = 0; S.zg[c] = 0ull;
    if (g < S.hi) {
      S.actmask |= 1u << c;
      const int i = g - trial_of(d, g) * d.N;
      S.r0[c] = d.row_ptr[i];
      S.rlen[c] = (int)(d.row_ptr[i + 1] - S.r0[c]);
      S.V[c] = d.V[g];
      S.zg[c] = mix64(d.seed + G64 * ((unsigned long long)g + 1ull));
    }
  }
  const int g0 = S.g0, hi = S.hi;
  // the wavefront's NPT spike words: lane w < NPT stores word (first neuron of the wavefront) / 64 + w
  const int gw = __builtin_amdgcn_readfirstlane(g0);
  const int my_word = (lane < NPT && gw < lo + chunk && (gw >> 6) + lane < d.words) ? (gw >> 6) + lane : -1;
  int slot = (int)(n0 % d.R);   // row of the circular spike words that holds step n0 (one division per launch)
  int phi = (int)(n0 & (long long)(d.W - 1));
  int* __restrict__ win = win_of(d, n0) + (size_t)phi * d.BN;   // row of the step being run
  const float cand_theta = d.theta - margin;
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
  for (int k = 0; k < nsteps; ++k) {
    const long long n = n0 + k;
    int near_h = d.W - 1 - phi;
    if (near_h > d.d_max) near_h = d.d_max;
    const __amdgpu_buffer_rsrc_t cells = res_rows(win, hi * 4);
    // ---- in front of the barrier: drive bits, an early look at the cells, the candidates and their rows
    unsigned xi = 0;
    if (d.p_thresh) {
#pragma unroll
      for (int c = 0; c < NPT; ++c)
        xi |= (mix64(S.zg[c] + G64 * ((unsigned long long)n + 1ull)) >> 32) < d.p_thresh ? 1u << c : 0u;
    }
    unsigned cmask = 0;   // bit c: neuron c is a candidate
    {
      const FlowVec<NPT> early = flow_load<NPT, kBufAgent>(cells, g0 * 4);
#pragma unroll
      for (int c = 0; c < NPT; ++c) {
        float I = (float)__float_as_int(early.v[c]) * 0x1p-24f;
        if (d.p_thresh) I = I + (((xi >> c) & 1u) ? d.ext_w : 0.0f);
        cmask |= __fmaf_rn(d.alpha, S.V[c], I) >= cand_theta ? 1u << c : 0u;
      }
      cmask &= S.actmask;
      if (near_h < 1) cmask = 0;   // (nothing of this step's spikes arrives inside the window)
    }
    unsigned listed = 0;   // bit c: neuron c is among the block's first kFwdCand candidates
    if (__ballot(cmask != 0u) != 0ull) {
      unsigned long long m[NPT];
      int total = 0;
#pragma unroll
      for (int c = 0; c < NPT; ++c) { m[c] = __ballot(((cmask >> c) & 1u) && S.rlen[c] > 0); total += __popcll(m[c]); }
      int at = 0;
      if (lane == 0 && total) at = atomicAdd(&s_ncand, total);
      at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
      for (int c = 0; c < NPT; ++c) {
        if (m[c] == 0ull) continue;   // uniform
        if ((m[c] >> lane) & 1ull) {
          const int idx = at + __popcll(m[c] & ((1ull << lane) - 1ull));
          if (idx < kFwdCand) {
            RevSpike r;
            r.r0 = S.r0[c]; r.len = S.rlen[c];
            r.pk = (NPT * (int)threadIdx.x + c) | (trial_of(d, g0 + c) << kRevLocBits);
            s_cand[idx] = r;
            listed |= 1u << c;
          }
        }
        at += __popcll(m[c]);
      }
    }
    __syncthreads();
    const int ncand = s_ncand < kFwdCand ? s_ncand : kFwdCand;
    // this wavefront's candidates: wave, wave + 8, wave + 16, wave + 24 of the list
    // (the entries 64 .. 127 as well where a row may hold more than 64 inside the window: late in a window a spike
    // of the headline network has 60 of them on average, and a row's entries beyond those in registers are a trip to
    // memory between the threshold and the arrival)
    uint2 ce[4], ce2[4]; long long cr0[4]; int clen[4], cbase[4], cloc[4];
    const bool two = near_h >= 8;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int x = wave + u * kWaves;
      ce[u] = make_uint2(0u, 0u); ce2[u] = make_uint2(0u, 0u); cr0[u] = 0; clen[u] = 0; cbase[u] = 0; cloc[u] = 0;
      if (x < ncand) {   // (the same in every lane)
        const RevSpike r = s_cand[x];
        cr0[u] = uniform_of(r.r0);
        clen[u] = __builtin_amdgcn_readfirstlane(r.len);
        const int pk = __builtin_amdgcn_readfirstlane(r.pk);
        cloc[u] = pk & ((1 << kRevLocBits) - 1);
        cbase[u] = (pk >> kRevLocBits) * d.N;
        const int shown = clen[u] < 64 ? clen[u] : 64;
        const __amdgpu_buffer_rsrc_t rs = res_rows(d.synf + cr0[u], shown * 8);
        const unsigned long long ev = __builtin_bit_cast(unsigned long long, __builtin_amdgcn_raw_buffer_load_b64(rs, lane * 8, 0, 0));
        ce[u] = make_uint2((unsigned)ev, (unsigned)(ev >> 32));
        if (two && clen[u] > 64) {   // (uniform)
          const int shown2 = clen[u] < 128 ? clen[u] : 128;
          const __amdgpu_buffer_rsrc_t rs2 = res_rows(d.synf + cr0[u], shown2 * 8);
          const unsigned long long ev2 = __builtin_bit_cast(unsigned long long, __builtin_amdgcn_raw_buffer_load_b64(rs2, 512 + lane * 8, 0, 0));
          ce2[u] = make_uint2((unsigned)ev2, (unsigned)(ev2 >> 32));
        }
      }
    }
    // ---- the adds of step n - 1 are in place once every block has arrived
    if (k > 0) rev_wait(d, bar_base + (unsigned)k * (unsigned)P, &s_dead);
    float U[NPT];
    unsigned smask = 0;
    {
      const FlowVec<NPT> acc = flow_load<NPT, kBufAgent>(cells, g0 * 4);
#pragma unroll
      for (int c = 0; c < NPT; ++c) {
        float I = (float)__float_as_int(acc.v[c]) * 0x1p-24f;
        if (d.p_thresh) I = I + (((xi >> c) & 1u) ? d.ext_w : 0.0f);
        U[c] = __fmaf_rn(d.alpha, S.V[c], I);
        const bool s = U[c] >= d.theta;
        S.V[c] = s ? d.v_reset : U[c];
        smask |= s ? 1u << c : 0u;
      }
      smask &= S.actmask;
    }
    // which candidates spiked; the spikes that were no (listed) candidates go to the slow list
    if (__ballot(listed != 0u) != 0ull) {
#pragma unroll
      for (int c = 0; c < NPT; ++c)
        if ((listed >> c) & 1u) s_fired[NPT * (int)threadIdx.x + c] = (unsigned char)((smask >> c) & 1u);
    }
    const unsigned slowmask = near_h >= 1 ? (smask & ~listed) : 0u;
    if (__ballot(slowmask != 0u) != 0ull) {
      unsigned long long m[NPT];
      int total = 0;
#pragma unroll
      for (int c = 0; c < NPT; ++c) { m[c] = __ballot(((slowmask >> c) & 1u) && S.rlen[c] > 0); total += __popcll(m[c]); }
      int at = 0;
      if (lane == 0 && total) at = atomicAdd(&s_nslow, total);
      at = __builtin_amdgcn_readfirstlane(at);
#pragma unroll
      for (int c = 0; c < NPT; ++c) {
        if (m[c] == 0ull) continue;   // uniform
        if ((m[c] >> lane) & 1ull) {
          RevSpike r;
          r.r0 = S.r0[c]; r.len = S.rlen[c];
          r.pk = (NPT * (int)threadIdx.x + c) | (trial_of(d, g0 + c) << kRevLocBits);
          s_slow[at + __popcll(m[c] & ((1ull << lane) - 1ull))] = r;
        }
        at += __popcll(m[c]);
      }
    }
    __syncthreads();
    if (threadIdx.x == 0) s_ncand = 0;   // (every wavefront has read it; the next step's candidates are counted before the next block barrier)
    // the adds of the candidates that spiked: their leading entries are in registers
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (clen[u] == 0) continue;            // uniform
      if (!s_fired[cloc[u]]) continue;       // uniform (one address for the wavefront)
      const int D = (int)(ce[u].x & d.dmask);
      const bool ok = lane < clen[u] && D <= near_h;
      if (ok) atomicAdd(&win[(size_t)D * d.BN + (size_t)cbase[u] + (ce[u].x >> d.dbits)], (int)ce[u].y);
      if (two && clen[u] > 64) {   // (uniform)
        const int D2 = (int)(ce2[u].x & d.dmask);
        const bool ok2 = (__ballot(ok) >> 63) != 0ull && 64 + lane < clen[u] && D2 <= near_h;   // (the rows ascend: nothing behind an entry that arrives too late)
        if (ok2) atomicAdd(&win[(size_t)D2 * d.BN + (size_t)cbase[u] + (ce2[u].x >> d.dbits)], (int)ce2[u].y);
        fwd_row_tail(d, win, near_h, cr0[u], clen[u], cbase[u], 128, ok2);
      } else {
        fwd_row_tail(d, win, near_h, cr0[u], clen[u], cbase[u], 64, ok);
      }
    }
    // the others: row entries loaded now
    const int nslow = s_nslow;
    for (int x = wave; x < nslow; x += kWaves) {
      const RevSpike r = s_slow[x];
      const int pk = __builtin_amdgcn_readfirstlane(r.pk);
      fwd_row_tail(d, win, near_h, uniform_of(r.r0), __builtin_amdgcn_readfirstlane(r.len), (pk >> kRevLocBits) * d.N, 0, true);
    }
    rev_arrive(d, k + 1 < nsteps, rank);   // (adds acknowledged; every wavefront has read the lists)
    if (threadIdx.x == 0) s_nslow = 0;   // (the next step's slow spikes are counted behind its first block barrier)
    // ---- after the arrival, off the chain: the popped cells cleared (nothing adds to them before the window after next
    // is expanded, launches later), tape, spike words and counts of this step
    flow_store<NPT, 0>(flow_splat<NPT>(0.0f), cells, g0 * 4);   // (the bits of 0.0f are those of the integer 0)
    if (RECORD) {
      const __amdgpu_buffer_rsrc_t tape = res_rows(d.tapeU + (size_t)n * d.BN, hi * 4);
      FlowVec<NPT> u4;
#pragma unroll
      for (int c = 0; c < NPT; ++c) u4.v[c] = U[c];
      flow_store<NPT, kBufNonTemporal>(u4, tape, g0 * 4);
    }
    unsigned long long wbits = 0ull;
    if (__ballot(smask != 0u) != 0ull) {
      if (RECORD) {
#pragma unroll
        for (int c = 0; c < NPT; ++c)
          if ((smask >> c) & 1u) atomicAdd(&d.spk_count[g0 + c], 1);
      }
      if constexpr (NPT == 8) {
        // lane 8 w + x holds neurons 8 x .. 8 x + 7 of word w
#pragma unroll
        for (int w = 0; w < 8; ++w) {
          const int v = __shfl((int)smask, 8 * w + (lane >> 3), 64);
          const unsigned long long b = __ballot((v >> (lane & 7)) & 1);
          if (lane == w) wbits = b;
        }
      } else if constexpr (NPT == 4) {
        // lane 16 w + x holds neurons 4 x .. 4 x + 3 of word w; lane l of a ballot must stand for neuron l of the word
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int v = __shfl((int)smask, 16 * w + (lane >> 2), 64);
          const unsigned long long b = __ballot((v >> (lane & 3)) & 1);
          if (lane == w) wbits = b;
        }
      } else {
        wbits = __ballot(smask & 1u);   // lane l holds neuron l of the wavefront's one word
      }
    }
    if (my_word >= 0) {
      d.spike_bits[(size_t)slot * d.words + my_word] = wbits;
      if (RECORD) d.tape_bits[(size_t)n * d.words + my_word] = wbits;
    }
    if (++slot == d.R) slot = 0;
    phi += 1;
    win += d.BN;
  }
#pragma unroll
  for (int c = 0; c < NPT; ++c)
    if ((S.actmask >> c) & 1u) d.V[g0 + c] = S.V[c];
}
