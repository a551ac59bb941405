// Ring queue, reverse sweep: the steps of one window in ONE launch with NO grid barrier -- the blocks
// wait for the very cells they gather (delta synapse).  Included by adseq.hip after
// ring_resident_reverse.h, whose layout (P taking-part blocks, consecutive neurons per thread -- here
// one, four or eight --, spikes listed a step ahead, the leading 64 entries of their rows requested
// ahead) it shares.
//
// What a reverse step n needs from other blocks is only the adjoints its spikes' in-window entries
// gather: cells of the rows n + 1 .. of the adjoint window (Section 3.2 eqs. 13 and 17 carried back
// through the steps).  A cell is written exactly once with its final value, by one 4-byte store --
// so the cell itself can say whether it is there yet.  The host fills the window's buffer with a
// sentinel (a NaN that the arithmetic here never produces) before the launch; a block stores the
// row of a step as soon as it has it, final for every neuron that does not spike, the sentinel
// once more for those that do, and their final values when their queue terms are gathered.  A
// gather that reads the sentinel is repeated until it reads something else.  That is the whole
// synchronisation: no counters, no arrivals, no acknowledgement of stores before anything, and a
// block that needs nothing from a late block does not wait for it.  The waits follow the data:
// step n of one block waits only for steps > n of others, which need nothing of step n or below,
// so the blocks that are waited for can always go on -- provided they are running: like the
// kernels with a grid barrier this one needs all its blocks on the chip at the same time, and
// every wait is a bounded spin (Dev::res_spins polls, then ERR_BARRIER and no more waiting in the
// block: the kernels run to their end, the gradients are void, the host reports it).
//
// Against the barrier per step of k_bwd_xcd (same arithmetic, same order of a spike's terms):
// there a step was gathers behind the barrier, the stores of the spiking neurons, their
// acknowledgement, the arrival, the poll -- three and a half trips over the fabric; here it is the
// gathers, and a second round of them where the first came too early.  What a step costs then is
// mostly the instructions a wavefront issues: hence the kernel per gradient mode, the one neuron per
// thread where the blocks are small enough, the two block barriers per step instead of three.

constexpr unsigned kFlowSentinel = 0x7fa5c3e1u;   // "not written yet" (a NaN with this payload)

// Repeats the lanes' gathers (p: the lane's cell; want: the lane gathers at all; v: what its first
// load returned) until none of them holds the sentinel.  The whole wavefront takes the same way.
__device__ __forceinline__ float flow_settle(const Dev& d, const float* p, bool want, float v, int* s_dead) {
  int spins = 0;
  while (__ballot(want && __float_as_uint(v) == kFlowSentinel) != 0ull) {
    if (*(volatile int*)s_dead) break;
    if (++spins > d.res_spins) {
      if ((threadIdx.x & 63) == 0) { atomicOr(&d.ctr->err, ERR_BARRIER); *(volatile int*)s_dead = 1; }
      break;
    }
    if (want && __float_as_uint(v) == kFlowSentinel) v = ld_agent(p);
  }
  return v;
}

// Entries [q0, len) of a spike's sorted row, 64 at a time while they arrive inside the window (the
// rows ascend in the arrival offset): gathers the adjoints, waiting for those that are not there
// yet, adds them to gsum, and returns the wavefront's sum of amplitude * adjoint.
__device__ __forceinline__ float flow_row_tail(const Dev& d, const float* __restrict__ gwin, int near_h, long long r0,
                                               int len, int base, int q0, bool more, int* s_dead) {
  const int lane = threadIdx.x & 63;
  float part = 0.0f;
  for (; (__ballot(more) >> 63) && q0 < len; q0 += 64) {
    more = false;
    bool want = false;
    const float* p = gwin;
    unsigned amp = 0u;
    if (q0 + lane < len) {
      const uint2 e = load_stream(&d.synb[r0 + q0 + lane]);
      const int D = (int)(e.x & d.dmask);
      if (D <= near_h) {
        want = true;
        amp = e.y;
        p = &gwin[(size_t)D * d.BN + (size_t)base + (e.x >> d.dbits)];
      }
    }
    float gv = 0.0f;
    if (want) gv = ld_agent(p);
    gv = flow_settle(d, p, want, gv, s_dead);
    float t = 0.0f;
    if (want) {
      unsafeAtomicAdd(&d.gsum[r0 + q0 + lane], gv);
      t = __uint_as_float(amp) * gv;
      more = true;
    }
    part += wave_sum_f(t);
  }
  return part;
}

// One reverse step of a wavefront.  PAR: list buffer of the step being run (the other one takes the
// list of the step after it); cur: the batch of the step being run (rows requested a step ago),
// nxt: filled here for the next one.
// NPT consecutive neurons of a thread, loaded and stored with one access of 4 NPT bytes.
template <int NPT> struct FlowVec { float v[NPT]; };
template <int NPT, int AUX>
__device__ __forceinline__ FlowVec<NPT> flow_load(__amdgpu_buffer_rsrc_t rs, int off) {
  FlowVec<NPT> r;
  if constexpr (NPT == 8) {
    const res_v4f x = __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, AUX));
    const res_v4f y = __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, off + 16, 0, AUX));
    r.v[0] = x[0]; r.v[1] = x[1]; r.v[2] = x[2]; r.v[3] = x[3];
    r.v[4] = y[0]; r.v[5] = y[1]; r.v[6] = y[2]; r.v[7] = y[3];
  } else if constexpr (NPT == 4) {
    const res_v4f x = __builtin_bit_cast(res_v4f, __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, AUX));
    r.v[0] = x[0]; r.v[1] = x[1]; r.v[2] = x[2]; r.v[3] = x[3];
  } else {
    static_assert(NPT == 1, "one, four or eight neurons per thread");
    r.v[0] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs, off, 0, AUX));
  }
  return r;
}
template <int NPT, int AUX>
__device__ __forceinline__ void flow_store(const FlowVec<NPT>& x, __amdgpu_buffer_rsrc_t rs, int off) {
  if constexpr (NPT == 8) {
    const res_v4f y = {x.v[0], x.v[1], x.v[2], x.v[3]}, z = {x.v[4], x.v[5], x.v[6], x.v[7]};
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(res_v4i, y), rs, off, 0, AUX);
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(res_v4i, z), rs, off + 16, 0, AUX);
  } else if constexpr (NPT == 4) {
    const res_v4f y = {x.v[0], x.v[1], x.v[2], x.v[3]};
    __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(res_v4i, y), rs, off, 0, AUX);
  } else {
    __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(int, x.v[0]), rs, off, 0, AUX);
  }
}
template <int NPT>
__device__ __forceinline__ FlowVec<NPT> flow_splat(float a) {
  FlowVec<NPT> r;
#pragma unroll
  for (int c = 0; c < NPT; ++c) r.v[c] = a;
  return r;
}

// What a thread carries through the launch (as RevState, for NPT neurons per thread).
template <int NPT>
struct FlowState {
  float carry[NPT], dLc[NPT];        // its neurons: carry of the adjoint, dL/dcount
  long long r0[NPT]; int rlen[NPT];  // bounds of their sorted rows
  unsigned actmask;                  // bit c: neuron c exists
  FlowVec<NPT> Ua, Ub, Uc;           // tape values of the step being run, of the one after it, of the one after that
  FlowVec<NPT> Ga, Gb, dUa, dUb;     // far queue terms and dL/dU of the step being run and of the next
  unsigned ovf_cur;                  // bit c: neuron c spiked in the step being run and did not fit the list
  int nspk_cur;                      // listed spikes of the step being run
  // the same in every lane
  long long n;                       // step being run
  int phi, tail, slot;               // n mod W, T - 1 - n, n mod R
  float* gwin;                       // row n of the adjoint window
  const float* tape2;                // tape row of step n - 2 (of step 0 below that)
  const float* du1;                  // dL/dU row of step n - 1 (of step 0 below that)
  int g0, hi;
};

template <bool HAS_DU, int SURR, int NPT>
__device__ __forceinline__ void flow_step(const Dev& d, FlowState<NPT>& S, const int PAR, RevBatch& cur, RevBatch& nxt, bool last,
                                          int* s_dead, int* s_nspk, RevSpike (*s_spk)[kRevList], float (*s_G2)[(NPT < 4 ? 4 : NPT) * kResThreads],
                                          float* fill_row, int& cnt_base0, int& cnt_base1) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int kWaves = kResThreads / 64;
  const long long n = S.n;
  const int near_h = rev_near(d, S.phi, S.tail);
  const int near1 = last ? 0 : rev_near(d, S.phi - 1, S.tail + 1);   // of the step after this one (same window: phi >= 1 there)
  float* __restrict__ gwin = S.gwin;
  float* s_G = s_G2[PAR];
  const int g0 = S.g0, hi = S.hi;
  float U[NPT], Gf[NPT], dU[NPT];
  unsigned smask = 0, s1 = 0;
#pragma unroll
  for (int c = 0; c < NPT; ++c) {
    U[c] = S.Ua.v[c]; Gf[c] = S.Ga.v[c]; dU[c] = HAS_DU ? S.dUa.v[c] : 0.0f;
    smask |= U[c] >= d.theta ? 1u << c : 0u;
    s1 |= S.Ub.v[c] >= d.theta ? 1u << c : 0u;
  }
  smask &= S.actmask; s1 &= S.actmask;
  // ---- requested first, so that they are there when the step ends (the values move up a place then, and a move of a
  // register that a load has not filled yet waits for the load): tape values of step n - 2, far queue terms and dL/dU
  // of step n - 1 (below step 0 the rows are step 0's again and are never used)
  const int slot1 = n >= 1 ? (S.slot == 0 ? d.R - 1 : S.slot - 1) : 0;   // (n - 1) mod R
  {
    const __amdgpu_buffer_rsrc_t t2 = res_rows(S.tape2, hi * 4), f1 = res_rows(d.Gacc + (size_t)slot1 * d.BN, hi * 4);
    S.Uc = flow_load<NPT, kBufNonTemporal>(t2, g0 * 4);
    S.Gb = flow_load<NPT, kBufNonTemporal>(f1, g0 * 4);
    if (HAS_DU) S.dUb = flow_load<NPT, kBufNonTemporal>(res_rows(S.du1, hi * 4), g0 * 4);
  }
  // ---- the row of this step, as early as can be (others may be waiting for it): final for every neuron that does not
  // spike; a spiking neuron's cell says "not yet" until its queue term is gathered below
  if (__ballot(S.actmask != 0u) != 0ull) {   // (wavefronts without neurons skip the arithmetic)
    FlowVec<NPT> gu4;
#pragma unroll
    for (int c = 0; c < NPT; ++c) {
      float gu;
      S.carry[c] = bwd_update_as<SURR>(d, n, U[c], 0.0f, (smask >> c) & 1u, S.carry[c], S.dLc[c], Gf[c], dU[c], &gu);
      gu4.v[c] = ((smask >> c) & 1u) ? __uint_as_float(kFlowSentinel) : gu;
    }
    const __amdgpu_buffer_rsrc_t row = res_rows(gwin, hi * 4), far = res_rows(d.Gacc + (size_t)S.slot * d.BN, hi * 4);
    flow_store<NPT, kBufAgent>(gu4, row, g0 * 4);
    // the far queue terms are used up: the slot is another step's R steps on (stored by every lane, set or not)
    flow_store<NPT, 0>(flow_splat<NPT>(0.0f), far, g0 * 4);
    // the same row of the OTHER window buffer, which the next launch sweeps: "not written yet"
    if (fill_row) flow_store<NPT, 0>(flow_splat<NPT>(__uint_as_float(kFlowSentinel)), res_rows(fill_row, hi * 4), g0 * 4);
  }
  // ---- this step's gathers (rows requested a step ago): every entry of the leading 64 that arrives inside the window
  float gv[4];
  const float* gp[4];
  cur.ok = 0u;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    gv[u] = 0.0f; gp[u] = gwin;
    if (cur.len[u] > 0) {   // (the same in every lane)
      const int D = (int)(cur.e[u].x & d.dmask);
      const bool ok = lane < cur.len[u] && D <= near_h;
      cur.ok |= ok ? 1u << u : 0u;
      if (ok) {
        gp[u] = &gwin[(size_t)D * d.BN + (size_t)cur.base[u] + (cur.e[u].x >> d.dbits)];
        gv[u] = ld_agent(gp[u]);
      }
    }
  }
  // ---- the step after this one: list of the block's spikes, the leading 64 entries of their rows requested
  int nspk_nxt = 0;
  unsigned ovf_nxt = 0;
#pragma unroll
  for (int u = 0; u < 4; ++u) { nxt.e[u] = make_uint2(0u, 0u); nxt.r0[u] = 0; nxt.len[u] = 0; nxt.base[u] = 0; nxt.loc[u] = 0; }
  if (near1 >= 1) {
    if (__ballot(s1 != 0u) != 0ull) {
      unsigned long long m[NPT];
      int total = 0;
#pragma unroll
      for (int c = 0; c < NPT; ++c) { m[c] = __ballot(((s1 >> c) & 1u) && S.rlen[c] > 0); total += __popcll(m[c]); }   // (a spike with an empty row is not listed)
      // (the counters of the two lists only ever grow -- no reset to order against the other wavefronts: a list's
      // places count from what its counter held when the list before it was complete, cnt_base)
      int at = 0;
      if (lane == 0) at = atomicAdd(&s_nspk[PAR ^ 1], total);
      at = __builtin_amdgcn_readfirstlane(at) - (PAR ? cnt_base0 : cnt_base1);
#pragma unroll
      for (int c = 0; c < NPT; ++c) {
        if (m[c] == 0ull) continue;   // uniform
        if ((m[c] >> lane) & 1ull) {
          const int idx = at + __popcll(m[c] & ((1ull << lane) - 1ull));
          if (idx < kRevList) {
            RevSpike r;
            r.r0 = S.r0[c]; r.len = S.rlen[c];
            r.pk = (NPT * (int)threadIdx.x + c) | (trial_of(d, g0 + c) << kRevLocBits);
            s_spk[PAR ^ 1][idx] = r;
          } else {
            ovf_nxt |= 1u << c;
          }
        }
        at += __popcll(m[c]);
      }
    }
    __syncthreads();
    {
      const int tot = s_nspk[PAR ^ 1], had = PAR ? cnt_base0 : cnt_base1;
      nspk_nxt = tot - had < kRevList ? tot - had : kRevList;
      if (PAR) cnt_base0 = tot; else cnt_base1 = tot;
    }
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
  // ---- the gathered adjoints, once they are all there; per-spike sums; the spiking neurons' final values
  float Gx[NPT];   // near parts that come back to the owner directly (spikes that did not fit the list)
#pragma unroll
  for (int c = 0; c < NPT; ++c) Gx[c] = 0.0f;
  if (near_h >= 1) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (cur.len[u] == 0) { cur.gv[u] = 0.0f; continue; }   // uniform: no spike in this place of the batch
      const bool ok = (cur.ok >> u) & 1u;
      cur.gv[u] = flow_settle(d, gp[u], ok, gv[u], s_dead);
      float part = wave_sum_f(ok ? __uint_as_float(cur.e[u].y) * cur.gv[u] : 0.0f);
      part += flow_row_tail(d, gwin, near_h, cur.r0[u], cur.len[u], cur.base[u], 64, ok, s_dead);
      if (lane == 0) s_G[cur.loc[u]] = part;
    }
    // more than 32 listed spikes in the block: the rest one at a time
    for (int x = wave + 4 * kWaves; x < S.nspk_cur; x += kWaves) {
      const RevSpike r = s_spk[PAR][x];
      const long long rr0 = uniform_of(r.r0);
      const int len = __builtin_amdgcn_readfirstlane(r.len), pk = __builtin_amdgcn_readfirstlane(r.pk);
      const float part = flow_row_tail(d, gwin, near_h, rr0, len, (pk >> kRevLocBits) * d.N, 0, true, s_dead);
      if (lane == 0) s_G[pk & ((1 << kRevLocBits) - 1)] = part;
    }
    // more spikes than the list holds: the owner's wavefront takes them one by one
    if (__ballot(S.ovf_cur != 0u) != 0ull) {
#pragma unroll
      for (int c = 0; c < NPT; ++c) {
        unsigned long long m = __ballot((S.ovf_cur >> c) & 1u);
        while (m) {
          const int L = __ffsll((long long)m) - 1;
          m &= m - 1;
          const long long rr0 = lane_get(S.r0[c], L);
          const int len = lane_get(S.rlen[c], L);
          const int base = trial_of(d, lane_get(g0, L) + c) * d.N;
          const float part = flow_row_tail(d, gwin, near_h, rr0, len, base, 0, true, s_dead);
          if (lane == L) Gx[c] = part;
        }
      }
    }
    __syncthreads();
  } else {
#pragma unroll
    for (int u = 0; u < 4; ++u) cur.gv[u] = 0.0f;
  }
  // the spiking neurons, with their whole queue term and the membrane value the step started from (a spiking
  // neuron's update does not use the carry: the reset cuts it)
  if (smask) {
#pragma unroll
    for (int c = 0; c < NPT; ++c) {
      if (!((smask >> c) & 1u)) continue;
      float G = Gf[c] + Gx[c];
      if (near_h >= 1 && S.rlen[c] > 0 && !((S.ovf_cur >> c) & 1u)) G += s_G[NPT * (int)threadIdx.x + c];
      float gu;
      S.carry[c] = bwd_update_as<SURR>(d, n, U[c], S.Ub.v[c], true, 0.0f, S.dLc[c], G, dU[c], &gu);
      if (!d.flow_hold) st_agent(&gwin[g0 + c], gu);   // (withheld only by the test of the waits' failure path)
    }
  }
  // per-synapse sums of this step's first batch
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

// Reverse steps n_hi - 1, n_hi - 2, ..., n_hi - nsteps, all inside one window whose buffer the host
// has filled with the sentinel.  P taking-part blocks (every stride-th block of the grid), each
// owning `chunk` <= NPT * 512 neurons, NPT consecutive ones per thread (NPT = 4 or, for state arrays beyond
// 256 x 2,048 cells, 8: 16-byte accesses, B N a multiple of 4; NPT = 1 where the blocks own 512 neurons at most: the
// dense part of a step then spreads over all the block's wavefronts).  HAS_DU: a cotangent on the membrane values comes with the call; SURR: the gradient mode.
// fill_other: the launch also fills the OTHER window buffer (the one the next launch sweeps) with the sentinel, every
// block the cells of its own neurons, a row per step and what is left when the steps are done.
template <bool HAS_DU, int SURR, int NPT>
__global__ __launch_bounds__(kResThreads) void k_bwd_flow(long long n_hi, int nsteps, long long T, int P, int chunk, int stride,
                                                          int fill_other, const float* __restrict__ dL_dcount,
                                                          const float* __restrict__ dL_dU, Dev d) {
  __shared__ int s_dead, s_nspk[2];
  __shared__ RevSpike s_spk[2][kRevList];     // the block's spikes of the step being run and of the step being prepared
  __shared__ float s_G[2][(NPT < 4 ? 4 : NPT) * kResThreads];   // near part of the queue term of every listed spike, by its neuron's place (two steps' worth in turn)
  if (blockIdx.x % stride) return;
  const int rank = blockIdx.x / stride;
  if (rank >= P) return;
  if (threadIdx.x == 0) { s_dead = (ld_agent(&d.ctr->err) & ERR_BARRIER) ? 1 : 0; s_nspk[0] = 0; s_nspk[1] = 0; }
  const int phi0 = (int)((n_hi - 1) & (long long)(d.W - 1));
  const long long tail0 = T - n_hi < 0x3fffffffLL ? T - n_hi : 0x3fffffffLL;
  const int lo = rank * chunk;
  FlowState<NPT> S;
  S.hi = lo + chunk < d.BN ? lo + chunk : d.BN;
  S.g0 = lo + NPT * (int)threadIdx.x;
  S.actmask = 0;
#pragma unroll
  for (int c = 0; c < NPT; ++c) {
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
  auto load_row = [&](const float* p) { return flow_load<NPT, kBufNonTemporal>(res_rows(p, S.hi * 4), S.g0 * 4); };
  const FlowVec<NPT> zero4 = flow_splat<NPT>(0.0f);
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
  __syncthreads();
  float* const other = gwin_of(d, n_hi - 1 + d.W);   // (the buffers take turns window by window)
  int cnt_base0 = 0, cnt_base1 = 0;   // what the counters of list 0 and list 1 held when their last list was complete
  for (int k = 0; k < nsteps; ++k) {
    flow_step<HAS_DU, SURR, NPT>(d, S, k & 1, A, B, k + 1 == nsteps, &s_dead, s_nspk, s_spk, s_G,
                      fill_other ? other + (size_t)(phi0 - k) * d.BN : nullptr, cnt_base0, cnt_base1);
    A = B;
  }
  if (fill_other && (S.actmask != 0u)) {
    // rows of the other buffer that no step of this launch stood for (a window cut short by the end of the run)
    for (int r = 0; r < d.W; ++r)
      if (r > phi0 || r <= phi0 - nsteps)
        flow_store<NPT, 0>(flow_splat<NPT>(__uint_as_float(kFlowSentinel)), res_rows(other + (size_t)r * d.BN, S.hi * 4), S.g0 * 4);
  }
#pragma unroll
  for (int c = 0; c < NPT; ++c)
    if ((S.actmask >> c) & 1u) d.bwd_carry[S.g0 + c] = S.carry[c];
}
