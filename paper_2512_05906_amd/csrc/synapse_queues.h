// One bounded FIFO of arrival times per synapse and trial (ADSEQ_SYN_FIFO): the organisation
// of Section 4.1 (listing "Synapse implementation": one queue per synapse, popped at every
// step) with the "FIFORing(n)" of Section 4.3; capacity 1 is its "SingleSpike(Hold)".  Included by
// adseq.hip inside its anonymous namespace, after bounded_queues.h (whose step and fan-out
// kernels, tape and counters it shares).
//
// State of queue q = b * S + p (trial b, synapse p), C = capacity <= 8:
//   sq_next u16 [ceil(B S / 8) * 8]  arrival step of the head, mod 65535; 0xffff = empty
//   sq_hs   u16 [B S]                head << 8 | size
//   sq_key  u16 [B S][C]             arrival step mod 65535 of every slot, circular from head
// (arrival steps lie within d_max <= 1023 steps of now, so the residue is unambiguous).
// All events of a synapse have the same delay, so the head is always the earliest, and since a
// source spikes at most once per step at most one event per queue is due per step.
// A step is three launches:
//   k_synq_pop      looks at every queue: the heads' arrival steps, eight per thread in one
//                   16-byte load; only a queue whose head is due touches the rest of its state;
//                   a due event adds the synapse's amplitude to the target's cell of I_acc
//                   (Q8.24, integer atomic);
//   k_neurons       (bounded_queues.h, KIND = ADSEQ_SYN_FIFO) takes and clears the cell, then
//                   drive, LIF, spike words, tape -- no admission: that is settled at the push;
//   k_fanout_step   (bounded_queues.h) offers the rows of the step's spikes through push_rows
//                   below: every entry owns its queue, so the push is a plain read-modify-write of
//                   consecutive states: no atomics, no contenders, admission flags written once.
// The dense first launch is the cost the per-target kinds avoid: it streams 2 bytes per synapse
// and trial per step whether or not anything is in flight.
//
// ADSEQ_SYN_LATEST ("SingleSpike(Drop)": one slot per synapse, a new spike always replaces the one
// held) uses sq_next alone: the pop is the same launch without the rest of the state, the push
// overwrites (push_rows_latest at the end of this file).  ADSEQ_SYN_BINS ("LossyRingDelay(n)") keeps
// one such key array per time bin (push_rows_bins).

constexpr int kSynqCapMax = 8;
constexpr int kSynqBlocks = 2048;   // blocks of k_synq_pop (grid-stride), each with a private counter line
constexpr unsigned kSynqEmpty = 0xffffu;

__device__ __forceinline__ unsigned synq_key(long long k) { return (unsigned)(k % 65535); }

// Two phases per block, so that the scan stays a pure stream: the scan only notes the queues whose
// head is due in an LDS list; then every thread takes one listed queue (all their loads in flight
// together) -- delivers, moves the head on, and stores the new head key.
constexpr int kSynqList = 2048;   // due queues a block notes before it works them off

template <bool LATEST>
__device__ __forceinline__ void synq_deliver(const Dev& d, long long q, long long off, int& popped, long long& sum) {
  const long long b = q / d.S, p = q - b * d.S;
  const int a = d.a_q[p];
  const unsigned pk = d.packed[p];
  unsigned next = kSynqEmpty;
  if (!LATEST) {
    const unsigned hs = d.sq_hs[q];
    unsigned head = (hs >> 8) + 1u;
    if (head >= (unsigned)d.C) head = 0u;
    const unsigned size = (hs & 0xffu) - 1u;
    if (size) next = (unsigned)d.sq_key[(size_t)q * d.C + head];
    d.sq_hs[q] = (unsigned short)(size ? ((head << 8) | size) : 0u);
  }
  d.sq_next[off + q] = (unsigned short)next;
  atomicAdd(&d.I_acc[(size_t)b * d.N + (pk >> d.dbits)], a);
  popped += 1; sum += a;
}

// LATEST: the keys looked at are all there is (ADSEQ_SYN_LATEST: one slot per queue; ADSEQ_SYN_BINS:
// the bin of this step, whose keys start `off` elements into sq_next).
template <bool LATEST>
__global__ __launch_bounds__(kBlock) void k_synq_pop(Dev d, long long n, long long off) {
  __shared__ BlockCounts s_cnt;
  __shared__ long long s_list[kSynqList];
  __shared__ int s_n;
  counts_clear(s_cnt);
  if (threadIdx.x == 0) s_n = 0;
  __syncthreads();
  const unsigned nk = synq_key(n);
  const unsigned nk2 = nk | (nk << 16);
  const long long Q = (long long)d.B * d.S;
  const long long groups = (Q + 7) >> 3;
  int popped = 0;
  long long sum = 0;
  const long long stride = (long long)gridDim.x * kBlock;
  // the same number of trips for every thread of the block (block barriers inside)
  const long long first = (long long)blockIdx.x * kBlock;
  for (long long base = first; base < groups; base += 4 * stride) {
    const long long g0 = base + threadIdx.x;
    // four groups of eight queues per trip: their loads in flight together
    const long long gi[4] = {g0, g0 + stride, g0 + 2 * stride, g0 + 3 * stride};
    uint4 st[4];
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      st[h] = make_uint4(0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu);
      if (gi[h] < groups) st[h] = reinterpret_cast<const uint4*>(d.sq_next + off)[gi[h]];
    }
#pragma unroll
    for (int h = 0; h < 4; ++h) {
      const unsigned w[4] = {st[h].x, st[h].y, st[h].z, st[h].w};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const unsigned x = w[j >> 1] ^ nk2;                 // a zero half = a head that is due now
        if (((j & 1) ? (x >> 16) : (x & 0xffffu)) != 0u) continue;
        const long long q = gi[h] * 8 + j;
        const int pos = atomicAdd(&s_n, 1);
        if (pos < kSynqList) s_list[pos] = q;
        else synq_deliver<LATEST>(d, q, off, popped, sum);  // no room to note it: done at once
      }
    }
    __syncthreads();
    const int cnt = s_n < kSynqList ? s_n : kSynqList;
    if (cnt > kSynqList / 2 || base + 4 * stride >= groups) {   // list half full, or the last trip
      for (int x = threadIdx.x; x < cnt; x += kBlock) synq_deliver<LATEST>(d, s_list[x], off, popped, sum);
      __syncthreads();
      if (threadIdx.x == 0) s_n = 0;
      __syncthreads();
    }
  }
  const long long t_pop = wave_total(popped), t_sum = wave_total64(sum);
  if ((threadIdx.x & 63) == 0) { counts_add(s_cnt, 2, t_pop); counts_add(s_cnt, 5, t_sum); }
  counts_flush(s_cnt, d.blk[(size_t)d.blk_pop + blockIdx.x]);
}

// Pushes, for each of up to four row shares of step n, the entries r0 + first + threadIdx.x +
// t * stride (t = 0, 1, ...) into their own queues; counts the admitted events and their Q8.24 sum
// into c_adm / s_adm.  Each stage is done for all four rows before the next.
__device__ __forceinline__ void push_rows(const Dev& d, long long n, const RowRef* rr, int nrows, long long stride,
                                          int& c_adm, long long& s_adm) {
  long long longest = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (j < nrows && rr[j].r1 - rr[j].r0 - rr[j].first > longest) longest = rr[j].r1 - rr[j].r0 - rr[j].first;
  for (long long o = 0; o < longest; o += stride) {
    long long p[4]; bool valid[4]; unsigned pk[4], st[4]; int a[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p[j] = rr[j].r0 + rr[j].first + o + threadIdx.x;
      valid[j] = j < nrows && p[j] < rr[j].r1;
      pk[j] = 0; a[j] = 0; st[j] = 0;
      if (valid[j]) {
        pk[j] = d.packed[p[j]]; a[j] = d.a_q[p[j]];
        st[j] = d.sq_hs[(size_t)rr[j].b * d.S + p[j]];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!valid[j]) continue;
      const size_t q = (size_t)rr[j].b * d.S + p[j];
      const unsigned size = st[j] & 0xffu, head = st[j] >> 8;
      const bool admit = size < (unsigned)d.C;
      if (admit) {
        unsigned slot = head + size;
        if (slot >= (unsigned)d.C) slot -= (unsigned)d.C;
        const unsigned k16 = synq_key(n + (long long)(pk[j] & d.dmask));
        d.sq_key[q * d.C + slot] = (unsigned short)k16;
        d.sq_hs[q] = (unsigned short)(st[j] + 1u);
        if (size == 0u) d.sq_next[q] = (unsigned short)k16;   // the new event is the head
        c_adm += 1; s_adm += a[j];
      }
      if (rr[j].tbase >= 0) d.tape_adm[rr[j].tbase + (p[j] - rr[j].r0)] = admit ? 1 : 0;
    }
  }
}

// Adds a block's admitted-event counts to its private counter line.  The whole block must call it.
__device__ __forceinline__ void push_counts_flush(const Dev& d, int c_adm, long long s_adm, BlkCtr& bc) {
  const long long tc = wave_total(c_adm), ts = wave_total64(s_adm);
  if ((threadIdx.x & 63) == 0 && tc) {
    atomicAdd(&bc.admitted, (unsigned long long)tc);   // private to this block: no contention; without return value
    atomicAdd((unsigned long long*)&bc.sum_admitted, (unsigned long long)ts);
  }
}

// ADSEQ_SYN_LATEST: the push of a slot that always takes the newest spike.  The event it held, if
// any, is lost: it came from the source's previous spike, whose row of admission flags starts at
// rr.obase on the tape (-1: no tape), so its flag is cleared here.  c_adm / s_adm count the net
// change of the admitted events (a replacement changes neither: same synapse, same amplitude).
__device__ __forceinline__ void push_rows_latest(const Dev& d, long long n, const RowRef* rr, int nrows,
                                                 long long stride, int& c_adm, long long& s_adm) {
  long long longest = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (j < nrows && rr[j].r1 - rr[j].r0 - rr[j].first > longest) longest = rr[j].r1 - rr[j].r0 - rr[j].first;
  for (long long o = 0; o < longest; o += stride) {
    long long p[4]; bool valid[4]; unsigned pk[4], old[4]; int a[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p[j] = rr[j].r0 + rr[j].first + o + threadIdx.x;
      valid[j] = j < nrows && p[j] < rr[j].r1;
      pk[j] = 0; a[j] = 0; old[j] = kSynqEmpty;
      if (valid[j]) {
        pk[j] = d.packed[p[j]]; a[j] = d.a_q[p[j]];
        old[j] = d.sq_next[(size_t)rr[j].b * d.S + p[j]];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!valid[j]) continue;
      const size_t q = (size_t)rr[j].b * d.S + p[j];
      d.sq_next[q] = (unsigned short)synq_key(n + (long long)(pk[j] & d.dmask));
      const bool replaced = old[j] != kSynqEmpty;
      if (!replaced) { c_adm += 1; s_adm += a[j]; }
      if (rr[j].tbase >= 0) d.tape_adm[rr[j].tbase + (p[j] - rr[j].r0)] = 1;
      if (replaced && rr[j].obase >= 0) d.tape_adm[rr[j].obase + (p[j] - rr[j].r0)] = 0;
    }
  }
}

// ADSEQ_SYN_BINS: `capacity` time bins per queue, bin b of all queues contiguous (sq_next[b][.]),
// so that the pop of a step streams one bin.  An event with arrival step k is written to bin
// k mod capacity, over whatever is there; an undelivered event that is overwritten is lost, and
// its admission flag -- whose index on the tape is kept beside the key (sq_flag, with a tape
// only) -- is cleared.
__device__ __forceinline__ void push_rows_bins(const Dev& d, long long n, const RowRef* rr, int nrows,
                                               long long stride, int& c_adm, long long& s_adm) {
  const long long qpad = (((long long)d.B * d.S + 7) >> 3) << 3;
  long long longest = 0;
#pragma unroll
  for (int j = 0; j < 4; ++j)
    if (j < nrows && rr[j].r1 - rr[j].r0 - rr[j].first > longest) longest = rr[j].r1 - rr[j].r0 - rr[j].first;
  for (long long o = 0; o < longest; o += stride) {
    long long p[4], idx[4]; bool valid[4]; unsigned pk[4], old[4]; int a[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p[j] = rr[j].r0 + rr[j].first + o + threadIdx.x;
      valid[j] = j < nrows && p[j] < rr[j].r1;
      pk[j] = 0; a[j] = 0;
      if (valid[j]) { pk[j] = d.packed[p[j]]; a[j] = d.a_q[p[j]]; }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      old[j] = kSynqEmpty; idx[j] = 0;
      if (valid[j]) {
        const long long k = n + (long long)(pk[j] & d.dmask);
        idx[j] = (k % d.C) * qpad + (long long)rr[j].b * d.S + p[j];
        old[j] = d.sq_next[idx[j]];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (!valid[j]) continue;
      d.sq_next[idx[j]] = (unsigned short)synq_key(n + (long long)(pk[j] & d.dmask));
      const bool replaced = old[j] != kSynqEmpty;
      if (!replaced) { c_adm += 1; s_adm += a[j]; }
      if (rr[j].tbase >= 0) {
        const long long flag = rr[j].tbase + (p[j] - rr[j].r0);
        if (replaced) d.tape_adm[d.sq_flag[idx[j]]] = 0;
        d.sq_flag[idx[j]] = flag;
        d.tape_adm[flag] = 1;
      }
    }
  }
}
