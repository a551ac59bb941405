// Bounded per-target queues (ADSEQ_FIFO, ADSEQ_SORTED).  Included by adseq.hip inside its
// anonymous namespace, after Dev and the device helpers.
//
// Every target owns `capacity` slots, target-major (the slots of one target are contiguous).
// A step is two launches:
//   k_fanout_* one block per spike walks the CSR row; an event whose target is already full is
//              dropped at once (the occupancy only grows during a step's enqueue phase); every
//              other event registers as a contender of its target: ticket = atomic count,
//              tickets below kCont go to the target's contender slots (one 16-byte record),
//              later ones to an overflow list (linked list through a pool);
//   k_neurons  the thread that owns target j first admits j's contenders of the step before --
//              the min(K, free) with the smallest synapse index, the canonical order -- then pops
//              the events due now, integrates, and hands the spikes on as one ballot word per
//              wavefront plus the block's spike and event counts (no shared counter: atomics on
//              one address go through one at a time, and one that returns a value costs its
//              wavefront a round trip).
// So admission needs no atomics on the slots and no launch of its own; a contender's fate is known
// one launch later (entry points that read counters or admission flags admit what is pending first).
// An admitted event that is due in the very step it is admitted in (arrival offset 1) is
// delivered from registers and never stored.
// Admission flags (one byte per emitted event, kept for the reverse sweep): the fan-out writes the
// whole row at once, 0 for an event dropped at once and 1 for a contender; the owner thread only
// clears the flags of the contenders that lose.
//
// FIFO: an unordered bag.  Per target: a bit mask of the occupied slots (one 32-bit word per 32
// slots), the arrival steps as 16-bit keys (arrival mod 2^16: unambiguous because every stored
// arrival lies within d_max <= 1023 steps of now) and the Q8.24 amplitudes.  A pop moves nothing:
// the owner thread loads its 64 bytes of keys per mask word with full-width loads, compares them
// with the current step, clears the bits of the due slots and loads only their amplitudes; an
// admitted event goes to the first free bit.  With few targets (a step is then bound by the chain
// of dependent accesses) the keys are loaded beside the rest of the thread's state; with many (a
// step is then bound by bytes and instructions) only after the mask word has shown that the target
// holds something.
// SORTED: the slots {arrival step, amplitude} are a circular array ordered by arrival step; pop
// takes from the front (only targets whose front is due now load anything: the earliest stored
// arrival is kept per target), an admitted event is inserted at its place (binary search, then
// the tail moves up one slot).
//
// Event counters: the fan-out counts the offered events (row lengths and the per-row amplitude
// sums made at create: no reduction over the lanes), the owner threads count the admitted and the
// delivered ones; dropped = offered - admitted.  Per-thread values are summed over the wavefront
// with a DPP scan, added to LDS words (one atomic per wavefront and counter), and from there to
// the block's private 64-byte line in global memory.

constexpr int kCont = 8;   // contender slots per target and step before the overflow list is used

// The kinds with one queue per synapse.
__device__ __host__ constexpr bool per_synapse_kind(int kind) {
  return kind == ADSEQ_SYN_FIFO || kind == ADSEQ_SYN_LATEST || kind == ADSEQ_SYN_BINS;
}

// Contender record, 128 bits: synapse index (40 bits), index of the admission flag on the tape
// (40 bits, all ones = none), arrival step mod 2^16, Q8.24 amplitude.
constexpr long long kMask40 = (1LL << 40) - 1;
__device__ __forceinline__ uint4 cont_pack(long long p, long long t, unsigned k, int a) {
  const unsigned long long tt = (unsigned long long)t & (unsigned long long)kMask40;
  return make_uint4((unsigned)p, (unsigned)(((unsigned long long)p >> 32) & 0xffu) | ((unsigned)tt << 8),
                    (unsigned)(tt >> 24) | (k << 16), (unsigned)a);
}
__device__ __forceinline__ long long cont_syn(const uint4& c) {
  return (long long)(((unsigned long long)(c.y & 0xffu) << 32) | (unsigned long long)c.x);
}
__device__ __forceinline__ long long cont_flag(const uint4& c) {
  const long long t = (long long)(((unsigned long long)(c.z & 0xffffu) << 24) | (unsigned long long)(c.y >> 8));
  return t == kMask40 ? -1 : t;
}
// Arrival step of a record whose event was emitted in the step before kn: it lies in
// [kn, kn + d_max).
__device__ __forceinline__ unsigned cont_arrival(const uint4& c, unsigned kn) {
  return kn + (((c.z >> 16) - kn) & 0xffffu);
}

// Queue state of one target in registers: stored events, earliest stored arrival step
// (0xffffffff: none; SORTED only), index of the front (SORTED), first mask word (FIFO).
struct QState { int occ; unsigned mn; int hd; unsigned m0; };

// FIFO: stores an admitted event in the first free slot of target g.
__device__ __forceinline__ void fifo_insert(const Dev& d, int g, QState& q, unsigned k, int a) {
  const unsigned lim0 = d.C >= 32 ? 0xffffffffu : ((1u << d.C) - 1u);
  const unsigned free0 = ~q.m0 & lim0;
  int slot = -1;
  if (free0) {
    slot = __ffs((int)free0) - 1;
    q.m0 |= 1u << slot;
  } else {
    for (int w = 1; w < d.nw; ++w) {
      unsigned* mp = &d.vmask[(size_t)g * d.nw + w];
      const unsigned m = *mp;
      const int cw = d.C - 32 * w;
      const unsigned lim = cw >= 32 ? 0xffffffffu : ((1u << cw) - 1u);
      const unsigned fr = ~m & lim;
      if (fr) {
        const int j = __ffs((int)fr) - 1;
        *mp = m | (1u << j);
        slot = 32 * w + j;
        break;
      }
    }
  }
  if (slot < 0) return;   // not reached: the caller admits no more events than there are free slots
  d.fkey[(size_t)g * d.cpad + slot] = (unsigned short)k;
  d.famp[(size_t)g * d.C + slot] = a;
}

// SORTED: stores an admitted event at its place in the circular array ordered by arrival step
// (behind the stored events with the same step); the events behind it move up one slot, eight at
// a time so that the loads of a group are in flight together.
__device__ __forceinline__ void sorted_insert(const Dev& d, int g, QState& q, unsigned k, int a) {
  uint2* __restrict__ sl = d.slot + (size_t)g * d.C;
  const int occ = q.occ, hd = q.hd;
  int lo = 0, hi = occ;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    int ph = hd + mid; if (ph >= d.C) ph -= d.C;
    if (sl[ph].x <= k) lo = mid + 1; else hi = mid;
  }
  for (int top = occ; top > lo;) {
    const int nmove = top - lo < 8 ? top - lo : 8;     // move entries [top - nmove, top) up by one
    uint2 mv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < nmove) {
        int ph = hd + top - 1 - j; if (ph >= d.C) ph -= d.C;
        mv[j] = sl[ph];
      }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < nmove) {
        int pd = hd + top - j; if (pd >= d.C) pd -= d.C;
        sl[pd] = mv[j];
      }
    top -= nmove;
  }
  int pw = hd + lo; if (pw >= d.C) pw -= d.C;
  sl[pw] = make_uint2(k, (unsigned)a);
}

// Per-thread results of a step: popped current and event counts.
struct StepAcc { int acc; int popped, c_adm; long long s_adm; };

// An admitted event of target g.  One that is due in this very step (arrival = kn, possible only
// for arrival offset 1) is delivered at once; the others are stored.
template <int KIND, int MODE>
__device__ __forceinline__ void take_event(const Dev& d, int g, unsigned kn, QState& q, StepAcc& r,
                                           unsigned k, int a) {
  r.c_adm += 1; r.s_adm += a;
  if (MODE != 0 && k == kn) {
    r.acc = wrap_add(r.acc, a);
    r.popped += 1;
    return;
  }
  if (KIND == ADSEQ_FIFO) fifo_insert(d, g, q, k, a);
  else { sorted_insert(d, g, q, k, a); q.mn = k < q.mn ? k : q.mn; }
  q.occ += 1;
}

// The rare case: more than kCont contenders for one target in one step, the later ones in the
// overflow list.  Same rule, general selection.
template <int KIND, int MODE>
__device__ __forceinline__ void admit_overflowed(const Dev& d, int g, int K, int take, unsigned kn,
                                              QState& q, StepAcc& r, const uint4* cc) {
  const int nc = kCont;                // the contender slots are all taken
  const int ovf_head = d.c_head[g];    // the others: overflow list
  d.c_head[g] = -1;
  if (take == K) {
    // room for all: any order
#pragma unroll
    for (int x = 0; x < kCont; ++x)
      if (x < nc) take_event<KIND, MODE>(d, g, kn, q, r, cont_arrival(cc[x], kn), (int)cc[x].w);
    for (int y = ovf_head; y >= 0; y = d.pool_next[y])
      take_event<KIND, MODE>(d, g, kn, q, r, d.pool_k[y], d.pool_a[y]);
    return;
  }
  // oversubscribed: the `take` smallest synapse indices win, the others are dropped
  long long last = -1;
  for (int rnd = 0; rnd < take; ++rnd) {
    long long bp = 0x7fffffffffffffffLL; int bx = -1, by = -1;
#pragma unroll
    for (int x = 0; x < kCont; ++x)
      if (x < nc) { const long long p = cont_syn(cc[x]); if (p > last && p < bp) { bp = p; bx = x; } }
    for (int y = ovf_head; y >= 0; y = d.pool_next[y]) {
      const long long pp = d.pool_p[y];
      if (pp > last && pp < bp) { bp = pp; by = y; bx = -1; }
    }
    if (bx < 0 && by < 0) break;   // not reached: K counts exactly the registered contenders
    last = bp;
    unsigned k = 0; int a = 0;
    if (bx >= 0) {
#pragma unroll
      for (int x = 0; x < kCont; ++x) if (x == bx) { k = cont_arrival(cc[x], kn); a = (int)cc[x].w; }
    } else {
      k = d.pool_k[by]; a = d.pool_a[by];
    }
    take_event<KIND, MODE>(d, g, kn, q, r, k, a);
  }
#pragma unroll
  for (int x = 0; x < kCont; ++x)
    if (x < nc && cont_syn(cc[x]) > last) {
      const long long t = cont_flag(cc[x]);
      if (t >= 0) d.tape_adm[t] = 0;
    }
  for (int y = ovf_head; y >= 0; y = d.pool_next[y]) {
    if (d.pool_p[y] > last) {
      const long long t = d.pool_t[y];
      if (t >= 0) d.tape_adm[t] = 0;
    }
  }
}

// Admits the contenders registered for target g (owner thread): the min(K, free) with the
// smallest synapse index are admitted, the others dropped (their admission flags cleared).
// `free_slots` is the room the target had when the contenders were emitted (before this step's
// pop).  Common case: all K contenders sit in the record slots; a contender's rank among them
// (number of records with a smaller synapse index) decides, and is only computed when there are
// more contenders than free slots.
template <int KIND, int MODE>
__device__ __forceinline__ void admit_contenders(const Dev& d, int g, int K, int free_slots, unsigned kn,
                                                 QState& q, StepAcc& r, const uint4* cc) {
  d.cnt[g] = 0;
  const int take = K < free_slots ? K : free_slots;
  if (K <= kCont) {
    int rank[kCont];
#pragma unroll
    for (int x = 0; x < kCont; ++x) rank[x] = 0;
    if (take < K) {
      long long p[kCont];
#pragma unroll
      for (int x = 0; x < kCont; ++x) p[x] = x < K ? cont_syn(cc[x]) : 0x7fffffffffffffffLL;
#pragma unroll
      for (int x = 1; x < kCont; ++x) {
        if (!__ballot(x < K)) break;          // no lane of the wavefront has that many contenders
#pragma unroll
        for (int y = 0; y < x; ++y) {
          const bool lt = p[y] < p[x];         // each pair once
          rank[x] += lt ? 1 : 0; rank[y] += lt ? 0 : 1;
        }
      }
    }
#pragma unroll
    for (int x = 0; x < kCont; ++x) {
      if (!__ballot(x < K)) break;
      if (x < K) {
        if (rank[x] < take) {
          take_event<KIND, MODE>(d, g, kn, q, r, cont_arrival(cc[x], kn), (int)cc[x].w);
        } else {
          const long long t = cont_flag(cc[x]);
          if (t >= 0) d.tape_adm[t] = 0;
        }
      }
    }
    return;
  }
  admit_overflowed<KIND, MODE>(d, g, K, take, kn, q, r, cc);
}

// Block-level event counters in LDS: [0] offered, [1] admitted, [2] delivered, [3..5] the same as
// sums of Q8.24 amplitudes, [6] spikes, [7] events emitted by them.
struct BlockCounts { unsigned long long c[8]; };

__device__ __forceinline__ void counts_clear(BlockCounts& bc) {
  if (threadIdx.x < 8) bc.c[threadIdx.x] = 0ull;
  __syncthreads();
}
// Adds a wavefront's total to counter k (call it from one lane).
__device__ __forceinline__ void counts_add(BlockCounts& bc, int k, long long v) {
  if (v) atomicAdd(&bc.c[k], (unsigned long long)v);
}
// Adds the first six LDS counters to the block's private line.  Starts with a block barrier.
__device__ __forceinline__ void counts_flush(BlockCounts& bc, BlkCtr& out) {
  __syncthreads();
  if (threadIdx.x < 6) {
    const unsigned long long v = bc.c[threadIdx.x];
    unsigned long long* o = threadIdx.x == 0 ? &out.offered : threadIdx.x == 1 ? &out.admitted
                          : threadIdx.x == 2 ? &out.delivered
                          : threadIdx.x == 3 ? (unsigned long long*)&out.sum_offered
                          : threadIdx.x == 4 ? (unsigned long long*)&out.sum_admitted
                                             : (unsigned long long*)&out.sum_delivered;
    if (v) atomicAdd(o, v);   // private to this block; an atomic without return value, so that nobody waits for a load
  }
}

// One thread per (trial, neuron).  MODE 0: admission only (what is pending); 1: admission + pop,
// writes the popped current to I_out (open loop); 2: admission + pop + drive + LIF + spike words
// + tape (closed loop).
template <int KIND, int MODE>
__global__ __launch_bounds__(kBlock) void k_neurons(Dev d, long long n, int parity,
                                                    const float* __restrict__ i_ext,
                                                    unsigned char* __restrict__ spikes_out,
                                                    float* __restrict__ I_out) {
  __shared__ BlockCounts s_cnt;
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  const size_t BN = (size_t)d.BN;
  const unsigned kn = (unsigned)n;
  StepAcc r; r.acc = 0; r.popped = 0; r.c_adm = 0; r.s_adm = 0;
  if (!per_synapse_kind(KIND) && blockIdx.x == 0 && threadIdx.x == 0) d.ctr->pool_n[0] = 0;   // the overflow pool is consumed by this launch
  counts_clear(s_cnt);
  const bool dense = d.prefetch != 0;   // few targets: latency-bound, load everything in the first round
  float v = 0.0f, jsyn = 0.0f, jfast = 0.0f;
  int len = 0;
  if (per_synapse_kind(KIND)) {
    // per-synapse queues: k_synq_pop has summed the events due now into the target's cell
    if (act) {
      if (MODE != 0) { r.acc = d.I_acc[g]; if (r.acc != 0) d.I_acc[g] = 0; }
      if (MODE == 2) {
        v = d.V[g];
        if (d.alpha_s > 0.0f) jsyn = d.J[g];
        if (d.alpha_r > 0.0f) jfast = d.J[(size_t)d.BN + g];
        if (dense) len = d.rowlen[g - trial_of(d, g) * d.N];
      }
    }
  } else if (act) {
    // everything the thread needs first, loaded together
    const int K = d.cnt[g];
    QState q;
    q.mn = KIND == ADSEQ_SORTED ? d.min_k[g] : 0u;
    q.hd = KIND == ADSEQ_SORTED ? d.head[g] : 0;
    q.m0 = KIND == ADSEQ_FIFO ? d.vmask[(size_t)g * d.nw] : 0u;
    // FIFO with one mask word: the occupancy is the number of set bits
    q.occ = (KIND == ADSEQ_FIFO && d.nw == 1) ? __popc(q.m0) : d.occ[g];
    uint4 kq[4];   // FIFO: the keys of the first 32 slots
    const uint4* kp0 = reinterpret_cast<const uint4*>(d.fkey + (size_t)g * d.cpad);
#pragma unroll
    for (int c = 0; c < 4; ++c) kq[c] = make_uint4(0u, 0u, 0u, 0u);
    if (KIND == ADSEQ_FIFO && MODE != 0 && dense) {
#pragma unroll
      for (int c = 0; c < 4; ++c) if (8 * c < d.cpad) kq[c] = kp0[c];
    }
    if (MODE == 2) {
      v = d.V[g];
      if (d.alpha_s > 0.0f) jsyn = d.J[g];
      if (d.alpha_r > 0.0f) jfast = d.J[(size_t)d.BN + g];
      if (dense) len = d.rowlen[g - trial_of(d, g) * d.N];
    }
    const QState q0 = q;
    // second round of loads: the contender records (and, below, the amplitudes of the due events)
    uint4 cc[kCont];
#pragma unroll
    for (int x = 0; x < kCont; ++x) {
      cc[x] = make_uint4(0u, 0u, 0u, 0u);
      if (x < K) cc[x] = d.cont[(size_t)x * BN + g];
    }
    if (KIND == ADSEQ_FIFO) {
      // bounded bag: every stored event due now leaves, wherever it sits
      if (MODE != 0) {
        const unsigned kn16 = kn & 0xffffu;
        int ndue = 0;
        if (!dense && q.m0) {
#pragma unroll
          for (int c = 0; c < 4; ++c) if (8 * c < d.cpad) kq[c] = kp0[c];
        }
        for (int w = 0; w < d.nw; ++w) {
          unsigned m = q.m0;
          if (w > 0) {
            m = d.vmask[(size_t)g * d.nw + w];
            if (!m) continue;
            const uint4* kp = reinterpret_cast<const uint4*>(d.fkey + (size_t)g * d.cpad + 32 * w);
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              kq[c] = make_uint4(0u, 0u, 0u, 0u);
              if (32 * w + 8 * c < d.cpad) kq[c] = kp[c];
            }
          }
          unsigned due = 0u;
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const unsigned wd[4] = {kq[c].x, kq[c].y, kq[c].z, kq[c].w};
#pragma unroll
            for (int h = 0; h < 4; ++h) {
              if ((wd[h] & 0xffffu) == kn16) due |= 1u << (8 * c + 2 * h);
              if ((wd[h] >> 16) == kn16) due |= 1u << (8 * c + 2 * h + 1);
            }
          }
          due &= m;
          if (due) {
            m &= ~due;
            ndue += __popc(due);
            if (w == 0) q.m0 = m; else d.vmask[(size_t)g * d.nw + w] = m;
            const int* __restrict__ ap = d.famp + (size_t)g * d.C + 32 * w;
            while (due) {
              // up to four amplitude loads in flight
              int j[4], av[4];
#pragma unroll
              for (int x = 0; x < 4; ++x) { j[x] = due ? __ffs((int)due) - 1 : -1; due &= due - 1u; }
#pragma unroll
              for (int x = 0; x < 4; ++x) av[x] = j[x] >= 0 ? ap[j[x]] : 0;
#pragma unroll
              for (int x = 0; x < 4; ++x) r.acc = wrap_add(r.acc, av[x]);
            }
          }
        }
        r.popped += ndue;
        q.occ -= ndue;
      }
      if (K > 0) admit_contenders<KIND, MODE>(d, g, K, d.C - q0.occ, kn, q, r, cc);
    } else {
      // ordered by arrival: admission first (an insert may land at the front), then everything
      // due now is taken from the front of the circular array, four slots loaded at a time
      if (K > 0) admit_contenders<KIND, MODE>(d, g, K, d.C - q0.occ, kn, q, r, cc);
      if (MODE != 0) {
        const uint2* __restrict__ sl = d.slot + (size_t)g * d.C;
        int occ = q.occ, hd = q.hd;
        unsigned front = q.mn;
        while (occ > 0 && front == kn) {
          uint2 e[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            e[j] = make_uint2(0xffffffffu, 0u);
            if (j < occ) { int ph = hd + j; if (ph >= d.C) ph -= d.C; e[j] = sl[ph]; }
          }
          int took = 0;
          unsigned next = kn;     // four taken and more stored: the next trip looks at the new front
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (took == j && j < occ && e[j].x == kn) { r.acc = wrap_add(r.acc, (int)e[j].y); ++took; }
            else if (took == j) next = e[j].x;   // first slot not taken (0xffffffff past the end)
          }
          hd += took; if (hd >= d.C) hd -= d.C;
          occ -= took;
          r.popped += took;
          front = occ > 0 ? next : 0xffffffffu;
        }
        q.occ = occ; q.hd = hd; q.mn = occ > 0 ? front : 0xffffffffu;
      }
    }
    if (q.occ != q0.occ) d.occ[g] = q.occ;
    if (KIND == ADSEQ_SORTED && q.mn != q0.mn) d.min_k[g] = q.mn;
    if (KIND == ADSEQ_FIFO && q.m0 != q0.m0) d.vmask[(size_t)g * d.nw] = q.m0;
    if (KIND == ADSEQ_SORTED && q.hd != q0.hd) d.head[g] = q.hd;
  }
  bool s = false;
  if (act && MODE != 0) {
    float I = (float)r.acc * 0x1p-24f;
    if (MODE == 2) {
      if (d.alpha_s > 0.0f) {   // the jumps go into the synaptic current state(s)
        const float jump = I;
        I = __fmaf_rn(d.alpha_s, jsyn, jump);
        d.J[g] = I;
        if (d.alpha_r > 0.0f) {   // double-exponential synapse: current = slow state - fast state
          const float fast = __fmaf_rn(d.alpha_r, jfast, jump);
          d.J[(size_t)d.BN + g] = fast;
          I = I - fast;
        }
      }
      if (d.p_thresh) {
        const bool xi = (unsigned long long)drive_bits(d.seed, (unsigned long long)g,
                                                       (unsigned long long)n) < d.p_thresh;
        I = I + (xi ? d.ext_w : 0.0f);
      }
      if (i_ext) I = I + i_ext[g];
      const float U = __fmaf_rn(d.alpha, v, I);
      s = U >= d.theta;
      __builtin_nontemporal_store(s ? d.v_reset : U, &d.V[g]);   // (written once, not read again by this launch)
      if (s && !dense) len = d.rowlen[g - trial_of(d, g) * d.N];
      if (d.record && n < d.max_steps) {
        __builtin_nontemporal_store(U, &d.tapeU[(size_t)n * d.BN + g]);
        if (s) atomicAdd(&d.spk_count[g], 1);   // no return value: the wavefront does not wait for it
      }
      if (spikes_out) spikes_out[g] = s ? 1 : 0;
    } else {
      I_out[g] = I;
    }
  }
  {
    // wavefront totals (every lane is active here), one LDS atomic per wavefront and counter;
    // a wavefront that delivered and admitted nothing, or has no spike, skips the sums
    long long t_pop = 0, t_acc = 0, t_adm = 0, t_sadm = 0, t_ev = 0;
    if (!per_synapse_kind(KIND) && __ballot(r.popped != 0 || r.c_adm != 0)) {
      t_pop = wave_total(r.popped); t_acc = wave_total(r.acc);
      t_adm = wave_total(r.c_adm); t_sadm = wave_total64(r.s_adm);
    }
    const unsigned long long m = __ballot(s);
    if (MODE == 2 && m) t_ev = wave_total(s ? len : 0);
    if ((threadIdx.x & 63) == 0) {
      counts_add(s_cnt, 2, t_pop); counts_add(s_cnt, 5, t_acc);
      counts_add(s_cnt, 1, t_adm); counts_add(s_cnt, 4, t_sadm);
      if (MODE == 2) {
        // the spikes go to the fan-out launch as one ballot word per wavefront, plus the block's
        // spike and event counts (plain stores)
        d.spk_words[(size_t)parity * d.words + (size_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)] = m;
        counts_add(s_cnt, 6, __popcll(m)); counts_add(s_cnt, 7, t_ev);
      }
    }
  }
  counts_flush(s_cnt, d.blk[blockIdx.x]);
  if (MODE == 2 && threadIdx.x < 2)
    d.stepcnt[((size_t)parity * d.nblk + blockIdx.x) * 2 + threadIdx.x] = (long long)s_cnt.c[6 + threadIdx.x];
}

// A share of the row of a spike that is being offered: trial, row bounds, index of the row's first
// admission flag on the tape (-1: none), offset of the share's first entry in the row, and
// (ADSEQ_SYN_LATEST) index of the first admission flag of the source's previous spike (-1: none).
struct RowRef { int b; long long r0, r1, tbase, first, obase; };

// Per-synapse queues (synapse_queues.h): the push that takes the place of offer_rows.
__device__ __forceinline__ void push_rows(const Dev& d, long long n, const RowRef* rr, int nrows, long long stride,
                                          int& c_adm, long long& s_adm);
__device__ __forceinline__ void push_counts_flush(const Dev& d, int c_adm, long long s_adm, BlkCtr& bc);
__device__ __forceinline__ void push_rows_latest(const Dev& d, long long n, const RowRef* rr, int nrows,
                                                 long long stride, int& c_adm, long long& s_adm);
__device__ __forceinline__ void push_rows_bins(const Dev& d, long long n, const RowRef* rr, int nrows,
                                               long long stride, int& c_adm, long long& s_adm);

// Offers, for each of up to four row shares of step n, the entries r0 + first + threadIdx.x +
// t * stride (t = 0, 1, ...) to their targets.  An event whose target is already full
// is dropped here; the others register as contenders (see the header of this file).  Each stage is
// done for all four rows before the next, so that the loads, the occupancy gathers and the ticket
// atomics are in flight together.  The whole block must call it together.
__device__ __forceinline__ void offer_rows(const Dev& d, long long n, const RowRef* rr, int nrows,
                                           long long stride) {
  const int lane = threadIdx.x & 63;
  const size_t BN = (size_t)d.BN;
  long long longest = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (j < nrows && rr[j].r1 - rr[j].r0 - rr[j].first > longest) longest = rr[j].r1 - rr[j].r0 - rr[j].first;
  for (long long o = 0; o < longest; o += stride) {
    long long p[4]; bool valid[4]; unsigned pk[4]; int a[4], gt[4], tk[4]; bool contend[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p[j] = rr[j].r0 + rr[j].first + o + threadIdx.x;
      valid[j] = j < nrows && p[j] < rr[j].r1;
      pk[j] = 0; a[j] = 0;
      if (valid[j]) { pk[j] = d.packed[p[j]]; a[j] = d.a_q[p[j]]; }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      gt[j] = rr[j].b * d.N + (int)(pk[j] >> d.dbits);
      contend[j] = false;
      if (valid[j]) contend[j] = d.occ[gt[j]] < d.C;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      tk[j] = -1;
      if (contend[j]) tk[j] = atomicAdd(&d.cnt[gt[j]], 1);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int D = (int)(pk[j] & d.dmask);
      const long long tidx = (valid[j] && rr[j].tbase >= 0) ? rr[j].tbase + (p[j] - rr[j].r0) : -1;
      if (tidx >= 0) d.tape_adm[tidx] = contend[j] ? 1 : 0;
      if (contend[j] && tk[j] < kCont)
        d.cont[(size_t)tk[j] * BN + gt[j]] = cont_pack(p[j], tidx, (unsigned)(n + D) & 0xffffu, a[j]);
      // the others: wavefront-aggregated claim of pool entries, pushed on the target's list
      const bool over = contend[j] && tk[j] >= kCont;
      const unsigned long long cm = __ballot(over);
      if (cm) {
        int base = 0;
        if (lane == __ffsll((long long)cm) - 1) base = atomicAdd(&d.ctr->pool_n[0], __popcll(cm));
        base = lane_get(base, __ffsll((long long)cm) - 1);
        if (over) {
          const int x = base + __popcll(cm & ((1ull << lane) - 1ull));
          if (x >= d.pool_cap) {
            // no room to remember it: it can only be dropped, and the run is flagged as invalid
            atomicOr(&d.ctr->err, ERR_POOL);
            atomicSub(&d.cnt[gt[j]], 1);
            if (tidx >= 0) d.tape_adm[tidx] = 0;
          } else {
            d.pool_p[x] = p[j]; d.pool_t[x] = tidx;
            d.pool_k[x] = (unsigned)(n + D); d.pool_a[x] = a[j];
            d.pool_next[x] = atomicExch(&d.c_head[gt[j]], x);
          }
        }
      }
    }
  }
}

// Takes the next NROWS (<= 4) spikes of neuron block nb from its ballot words and requests their
// row bounds (and, for share 0, the row sums).  A macro, so that the ballot words stay in registers.
#define ADSEQ_LOAD_GROUP(NROWS)                                                                         \
  _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                       \
    rr[j].b = 0; rr[j].r0 = 0; rr[j].r1 = 0; rr[j].tbase = -1; rr[j].obase = -1; rr[j].first = (long long)c * kBlock; gs[j] = 0; \
    if (j < (NROWS)) {                                                                                  \
      while (!bits) { ++x; bits = x == 1 ? w[1] : x == 2 ? w[2] : w[3]; }                               \
      const int bit = __ffsll((long long)bits) - 1;                                                     \
      bits &= bits - 1;                                                                                 \
      gs[j] = (nb * (kBlock / 64) + x) * 64 + bit;                                                      \
    }                                                                                                   \
  }                                                                                                     \
  _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                                       \
    rs[j] = 0; kc[j] = 0;                                                                               \
    if (j < (NROWS)) {                                                                                  \
      rr[j].b = trial_of(d, gs[j]);                                                             \
      const int i = gs[j] - rr[j].b * d.N;                                                              \
      rr[j].r0 = d.row_ptr[i]; rr[j].r1 = d.row_ptr[i + 1];                                             \
      if (c == 0 && threadIdx.x == 0) rs[j] = d.rowsum[i];                                              \
      if (KIND == ADSEQ_SYN_LATEST && record) kc[j] = d.spk_count[gs[j]];                               \
    }                                                                                                   \
  }

// Closed-loop fan-out of step n: fsplit blocks per neuron block.  Block (nb, c) reads the four
// ballot words that neuron block nb of this step's k_neurons launch left (most find them zero
// and leave) and offers share c -- entries c * 256 .. c * 256 + 255 of every fsplit * 256 -- of
// the row of every spike in them, four spikes at a time.  A row is thus spread over fsplit compute
// units (one unit sustains well under 10^9 scattered accesses per
// second).  With `record`, the spikes and the index of each row's first admission flag go to the
// tape; the positions come from prefix sums over the per-block counts of the step launch.
constexpr int kFanSplitMax = 4;   // d.fsplit = blocks per neuron block: a row of average length needs 1 .. 4 shares of 256
template <int KIND>
__global__ __launch_bounds__(kBlock) void k_fanout_step(Dev d, long long n, int parity, int record) {
  __shared__ long long s_red[2][kBlock / 64];
  const int nb = blockIdx.x / d.fsplit, c = blockIdx.x - nb * d.fsplit;
  const unsigned long long* __restrict__ wp = d.spk_words + (size_t)parity * d.words + (size_t)nb * (kBlock / 64);
  unsigned long long w[kBlock / 64];
  int nspk = 0;
#pragma unroll
  for (int x = 0; x < kBlock / 64; ++x) { w[x] = wp[x]; nspk += __popcll(w[x]); }
  const bool closer = record && blockIdx.x == 0;      // also writes where the next step's spikes start
  if (nspk == 0 && !closer) return;
  pin_args(d.stepcnt, d.step_off, d.step_evoff, d.row_ptr, d.rowsum, d.packed, d.a_q, d.occ, d.cnt, d.cont,
           d.tape_adm, d.tape_spk, d.tape_evb, d.blk, d.ctr, d.N, d.B, d.BN, d.C, d.nblk, d.dbits, d.dmask,
           d.max_steps, d.spike_cap, d.event_cap, d.pool_cap, n);
  long long c_off = 0, s_off = 0;   // offered events and their amplitude sum (share 0, thread 0)
  int c_adm = 0;                    // per-synapse queues: events this thread admitted, and their sum
  long long s_adm = 0;
  {
    // the first group's row bounds are requested before the prefix sums, so that the two overlap
    int x = 0;
    unsigned long long bits = w[0];
    RowRef rr[4];
    int gs[4];
    long long rs[4];
    int kc[4];   // ADSEQ_SYN_LATEST with tape: spikes of the neuron so far, this one included
    { ADSEQ_LOAD_GROUP(nspk < 4 ? nspk : 4) }
    long long pre_s = 0, pre_e = 0;
    if (record) {
      // spikes and events of the neuron blocks before nb (the closing block: of all blocks)
      const long long off = d.step_off[n], evoff = d.step_evoff[n];
      const long long* __restrict__ sc = d.stepcnt + (size_t)parity * d.nblk * 2;
      long long ts = 0, te = 0, as = 0, ae = 0;
      for (int j = threadIdx.x; j < d.nblk; j += kBlock) {
        const long long cs = sc[2 * j], ce = sc[2 * j + 1];
        as += cs; ae += ce;
        if (j < nb) { ts += cs; te += ce; }
      }
      ts = wave_total64(ts); te = wave_total64(te);
      if ((threadIdx.x & 63) == 0) { s_red[0][threadIdx.x >> 6] = ts; s_red[1][threadIdx.x >> 6] = te; }
      __syncthreads();
      for (int x = 0; x < kBlock / 64; ++x) { pre_s += s_red[0][x]; pre_e += s_red[1][x]; }
      if (closer) {
        __syncthreads();
        as = wave_total64(as); ae = wave_total64(ae);
        if ((threadIdx.x & 63) == 0) { s_red[0][threadIdx.x >> 6] = as; s_red[1][threadIdx.x >> 6] = ae; }
        __syncthreads();
        if (threadIdx.x == 0) {
          long long all_s = 0, all_e = 0;
          for (int x = 0; x < kBlock / 64; ++x) { all_s += s_red[0][x]; all_e += s_red[1][x]; }
          if (n + 1 <= d.max_steps) { d.step_off[n + 1] = off + all_s; d.step_evoff[n + 1] = evoff + all_e; }
          d.ctr->tape_spikes = off + all_s;
          d.ctr->tape_events = evoff + all_e;
        }
        if (nspk == 0) return;
      }
      pre_s += off; pre_e += evoff;
    }
    for (int rank0 = 0; rank0 < nspk; rank0 += 4) {
      const int nrows = nspk - rank0 < 4 ? nspk - rank0 : 4;
      if (rank0 > 0) { ADSEQ_LOAD_GROUP(nrows) }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        if (j < nrows) {
          const long long len = rr[j].r1 - rr[j].r0;
          c_off += len; s_off += rs[j];
          if (record) {
            const bool fits = pre_s + rank0 + j < d.spike_cap;
            long long evb = pre_e;
            const bool ev_fits = evb + len <= d.event_cap;
            if (!ev_fits) evb = -1;
            if (c == 0 && threadIdx.x == 0) {
              if (fits) {
                d.tape_spk[pre_s + rank0 + j] = gs[j]; d.tape_evb[pre_s + rank0 + j] = evb;
                RowSpan rsn; rsn.r0 = rr[j].r0; rsn.r1 = rr[j].r1;
                d.tape_row[pre_s + rank0 + j] = rsn;
              }
              else atomicOr(&d.ctr->err, ERR_TAPE_SPIKES);
              if (!ev_fits) atomicOr(&d.ctr->err, ERR_TAPE_EVENTS);
            }
            rr[j].tbase = evb;
            if (KIND == ADSEQ_SYN_LATEST) {
              // where the flags of the neuron's previous spike start (two cells per neuron, used in
              // turn, so that the shares of this row read the old one while share 0 writes the new)
              if (kc[j] >= 2) rr[j].obase = d.last_evb[(size_t)((kc[j] - 1) & 1) * d.BN + gs[j]];
              if (c == 0 && threadIdx.x == 0) d.last_evb[(size_t)(kc[j] & 1) * d.BN + gs[j]] = evb;
            }
            pre_e += len;
          }
        }
      }
      if (KIND == ADSEQ_SYN_FIFO) push_rows(d, n, rr, nrows, (long long)d.fsplit * kBlock, c_adm, s_adm);
      else if (KIND == ADSEQ_SYN_LATEST) push_rows_latest(d, n, rr, nrows, (long long)d.fsplit * kBlock, c_adm, s_adm);
      else if (KIND == ADSEQ_SYN_BINS) push_rows_bins(d, n, rr, nrows, (long long)d.fsplit * kBlock, c_adm, s_adm);
      else offer_rows(d, n, rr, nrows, (long long)d.fsplit * kBlock);
    }
  }
  if (per_synapse_kind(KIND)) push_counts_flush(d, c_adm, s_adm, d.blk[d.nblk + blockIdx.x]);
  if (c == 0 && threadIdx.x == 0 && c_off) {
    BlkCtr& bc = d.blk[d.nblk + blockIdx.x];   // private to this block
    atomicAdd(&bc.offered, (unsigned long long)c_off);   // atomics without return value: nobody waits for a load
    atomicAdd((unsigned long long*)&bc.sum_offered, (unsigned long long)s_off);
  }
}

#undef ADSEQ_LOAD_GROUP

// Open-loop fan-out: the spikes come as the caller's list of flat neuron indices; one block per
// spike (grid-stride over the list).
template <int KIND>
__global__ __launch_bounds__(kBlock) void k_fanout_list(Dev d, long long n, const int* __restrict__ spk,
                                                        const int* __restrict__ n_spk_ptr) {
  int nspk = *n_spk_ptr;
  nspk = nspk < 0 ? 0 : (nspk > d.BN ? d.BN : nspk);
  long long c_off = 0, s_off = 0;
  int c_adm = 0;
  long long s_adm = 0;
  for (int e = blockIdx.x; e < nspk; e += gridDim.x) {
    const int g = spk[e];
    if ((unsigned)g >= (unsigned)d.BN) continue;  // uniform over the block
    const int b = trial_of(d, g), i = g - b * d.N;
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    RowRef rr[4];   // the one row as four interleaved shares: four entries per thread in flight
#pragma unroll
    for (int j = 0; j < 4; ++j) { rr[j].b = b; rr[j].r0 = r0; rr[j].r1 = r1; rr[j].tbase = -1; rr[j].obase = -1; rr[j].first = (long long)j * kBlock; }
    if (threadIdx.x == 0) { c_off += r1 - r0; s_off += d.rowsum[i]; }
    if (KIND == ADSEQ_SYN_FIFO) push_rows(d, n, rr, 4, 4LL * kBlock, c_adm, s_adm);
    else if (KIND == ADSEQ_SYN_LATEST) push_rows_latest(d, n, rr, 4, 4LL * kBlock, c_adm, s_adm);
    else if (KIND == ADSEQ_SYN_BINS) push_rows_bins(d, n, rr, 4, 4LL * kBlock, c_adm, s_adm);
    else offer_rows(d, n, rr, 4, 4LL * kBlock);
  }
  if (per_synapse_kind(KIND)) push_counts_flush(d, c_adm, s_adm, d.blk[d.nblk + blockIdx.x]);
  if (threadIdx.x == 0 && c_off) {
    BlkCtr& bc = d.blk[d.nblk + blockIdx.x];   // private to this block
    atomicAdd(&bc.offered, (unsigned long long)c_off);   // atomics without return value: nobody waits for a load
    atomicAdd((unsigned long long*)&bc.sum_offered, (unsigned long long)s_off);
  }
}

// Q8.24 amplitude sum (for the offered-event counters) and length of every row: one wavefront
// per row.
__global__ __launch_bounds__(kBlock) void k_row_sums(Dev d) {
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * kBlock + threadIdx.x) >> 6;
  const long long nwaves = ((long long)gridDim.x * kBlock) >> 6;
  for (long long i = wave; i < d.N; i += nwaves) {
    long long sum = 0;
    for (long long p = d.row_ptr[i] + lane; p < d.row_ptr[i + 1]; p += 64) sum += d.a_q[p];
    sum = wave_sum(sum);
    if (lane == 0) { d.rowsum[i] = sum; d.rowlen[i] = (int)(d.row_ptr[i + 1] - d.row_ptr[i]); }
  }
}
