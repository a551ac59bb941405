// MI355X (gfx950) kernels and C ABI for delayed spike-event delivery through
// autodifferentiable queues.  See include/adseq.h for the contract of every
// entry point; this file holds the device code and the host-side bookkeeping.
//
// Layout of the state in the caller's workspace (all arrays 256-byte aligned):
//   V            fp32  [BN]                 membrane state
//   win          i32   [W][BN]              RING: Q8.24 sums per arrival step of the current window
//   spike_bits   u64   [R][4 nblk]          RING: spike bit masks of the last R = d_max + 1 steps (one
//                                           word per wavefront): the events not yet in `win`
//   dstart, nearcnt, perm, rowsum           RING: index of the rows sorted by arrival offset
//   ebuf, ecnt                              RING: staging regions of the window expansion
//   slot_k/a     u32/i32 [C][BN]            FIFO/SORTED: arrival step and Q8.24 amplitude, slot-major
//                                           so that one slot of 64 consecutive targets is one line
//   occ, head    i32   [BN]                 FIFO/SORTED: stored events; SORTED: index of the front
//   c_head, pool_*                          per-step contender lists (one linked list per target)
//   packed, a_q  u32/i32 [S]                FIFO/SORTED synapses: (col << dbits | D) and Q8.24 amplitude
//   synf, synb   2 x u32 [S]                RING synapses, every row sorted by D: {packed, Q8.24 amplitude}
//                                           for the forward pass, {packed, fp32 amplitude} for the reverse
//   amp, fdec    fp32  [S]                  continuous delays: a = w f (FIFO/SORTED) and f
//   tape_*                                  membrane tape, spike list, admission flags
//   bwd_*                                   FIFO/SORTED: adjoint delay line [R][BN], carry, queue term
//   gwin, Gacc, gsum                        RING: adjoint rows of the window, far queue terms, per-synapse sums
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "adseq.h"

namespace {

constexpr int kBlock = 256;
constexpr int kFanoutBlocks = 1024;

enum : unsigned {
  ERR_DELAY = 1u, ERR_GRAPH = 2u, ERR_TAPE_SPIKES = 4u, ERR_TAPE_EVENTS = 8u, ERR_POOL = 16u
};

struct Counters {
  unsigned long long offered, dropped, delivered;
  long long sum_offered, sum_dropped, sum_delivered;
  long long tape_spikes, tape_events;
  unsigned err;
  int n_spk[2];
  int pool_n[2];
  unsigned long long in_flight[2];  // scratch of k_ring_in_flight: events, Q8.24 sum
  unsigned long long fold[3];       // scratch of k_count_spikes: spikes, events, Q8.24 sum
};

// FIFO / SORTED: private event counters of one block of k_neurons / k_fanout (one 64-byte line
// each, so that no two blocks add to the same address; summed on demand).
struct BlkCtr {
  unsigned long long offered, dropped, delivered;
  long long sum_offered, sum_dropped, sum_delivered;
  long long pad[2];
};

struct ExpCoef { double c[21]; };

struct Dev {
  int N, B, BN, R, C, kind, dbits, d_max;
  unsigned dmask;
  int continuous, record, surrogate, max_steps, pool_cap;
  float alpha, theta, v_reset, ext_w, dt, tau;
  unsigned long long p_thresh, seed;
  long long S, spike_cap, event_cap;
  const long long* row_ptr;
  const int* col;
  const float* weight;
  const unsigned char* delay_steps;
  const float* delay_ms;
  unsigned* packed;
  int* a_q;
  // RING (windowed delay line, see ring_window.h)
  int W, wshift;        // window length in steps (power of two) and its log2
  int tp_shift;         // log2 of the targets per part (W << tp_shift = cells of one LDS tile)
  int P, NB, cap;       // target parts, blocks of the staging pass, events per (part, block) region
  int wgroups;          // 8-word lines (64 bytes) per step in spike_bits
  int* win;             // [W][BN]
  uint2* synf;          // [S] sorted rows: {col << dbits | D, Q8.24 amplitude}
  uint2* synb;          // [S] sorted rows: {col << dbits | D, fp32 amplitude bits}
  unsigned* dstart;     // [N][d_max + 2]
  unsigned* nearcnt;    // [W + 1][N]
  unsigned* perm;       // [S]
  long long* rowsum;    // [N]
  uint2* ebuf;          // [min(P, kMaxParts)][NB][cap]
  int* ecnt;            // [min(P, kMaxParts)][NB]
  unsigned long long* tape_bits;  // [T][words]
  float* gwin;          // [W][BN]
  float* Gacc;          // [R][BN]
  float* gsum;          // [S]
  float* amp;
  float* fdec;
  float* V;
  unsigned long long* spike_bits;  // RING: [R][words] spikes of the last R steps
  unsigned* slot_k;
  int* slot_a;
  int* occ;
  int* head;
  unsigned* min_k;      // FIFO: earliest stored arrival step per target (0xffffffff: none)
  int* cnt;             // contenders registered per target since its last admission
  long long* cont_p;    // [kCont][BN] contender slots: synapse index,
  unsigned* cont_k;     //   arrival step,
  int* cont_a;          //   Q8.24 amplitude,
  long long* cont_t;    //   index of the admission flag on the tape (recording only)
  int* c_head;          // overflow list head per target (-1: empty)
  long long* pool_p;
  long long* pool_t;
  int* pool_next;
  unsigned* pool_k;
  int* pool_a;
  int* cur_spk;
  float* tapeU;
  int* spk_count;       // [BN] spikes per (trial, neuron) over the recorded steps
  long long* step_off;
  int* tape_spk;
  long long* tape_evb;
  unsigned char* tape_adm;
  float* bwd_ring;
  float* bwd_carry;
  float* bwd_G;
  Counters* ctr;
  BlkCtr* blk;   // FIFO / SORTED: [nblk + kFanoutBlocks]
  int nblk;      // neuron blocks of a step launch: ceil(BN / 256)
  int words;     // 64-neuron words per step in spike_bits (RING) = 4 * nblk
};

// ---------------------------------------------------------------- device helpers

// splitmix64 output function (Steele, Lea, Flood 2014)
__device__ __forceinline__ unsigned long long mix64(unsigned long long z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31; return z;
}
// 32 uniform bits for (seed, unit g, step n): the drive's counter-based generator
__device__ __forceinline__ unsigned drive_bits(unsigned long long seed, unsigned long long g,
                                               unsigned long long n) {
  const unsigned long long G = 0x9E3779B97F4A7C15ull;
  unsigned long long z = mix64(seed + G * (g + 1));
  z = mix64(z + G * (n + 1));
  return (unsigned)(z >> 32);
}

__device__ __forceinline__ int wrap_add(int a, int b) { return (int)((unsigned)a + (unsigned)b); }

__device__ __forceinline__ long long wave_sum(long long v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_sum_f(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  return v;
}

// Adds the block's totals of two per-thread values to two global 64-bit counters
// (one atomic each per block).  Every thread of the block must call it.
__device__ __forceinline__ void block_add2(unsigned long long* c0, long long v0, long long* c1,
                                           long long v1) {
  __shared__ long long red[2][kBlock / 64];
  v0 = wave_sum(v0); v1 = wave_sum(v1);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) { red[0][w] = v0; red[1][w] = v1; }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long a = 0, b = 0;
    for (int i = 0; i < kBlock / 64; ++i) { a += red[0][i]; b += red[1][i]; }
    if (a) atomicAdd(c0, (unsigned long long)a);
    if (b) atomicAdd((unsigned long long*)c1, (unsigned long long)b);
  }
  __syncthreads();
}

__global__ void k_fill_u32(unsigned* p, unsigned v, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    p[i] = v;
}

// ---------------------------------------------------------------- preparation

// Synapse p -> arrival offset D_p, Q8.24 amplitude, packed (col, D); validates delays and columns.
// Continuous delays: D = max(1, ceil(d/dt)), a = w exp(-(D dt - d)/tau); exp as the degree-20
// Taylor polynomial (Horner, fused multiply-add) so that the value is reproducible bit for bit.
__global__ __launch_bounds__(kBlock) void k_prepare(Dev d, ExpCoef ec) {
  const double dt = (double)d.dt, tau = (double)d.tau;
  for (long long p = (long long)blockIdx.x * kBlock + threadIdx.x; p < d.S;
       p += (long long)gridDim.x * kBlock) {
    unsigned err = 0;
    const double w = (double)d.weight[p];
    double f = 1.0;
    long long D;
    if (!d.continuous) {
      D = d.delay_steps[p];
      if (D < 1) { err |= ERR_DELAY; D = 1; }
    } else {
      const double dl = (double)d.delay_ms[p];
      if (!(dl > 0.0)) err |= ERR_DELAY;
      const double q = ceil(dl / dt);
      D = (q >= 1.0 && q < 1e9) ? (long long)q : 1;
      const double x = ((double)D * dt - dl) / tau;
      if (!(x >= 0.0 && x <= 1.0)) err |= ERR_DELAY;
      const double y = -x;
      double r = ec.c[20];
      for (int k = 19; k >= 0; --k) r = __fma_rn(r, y, ec.c[k]);
      f = r;
    }
    if (D > d.d_max) { err |= ERR_DELAY; D = d.d_max; }
    const int c = d.col[p];
    if (c < 0 || c >= d.N) err |= ERR_GRAPH;
    const double a = w * f;
    long long q = __double2ll_rn(a * 16777216.0);
    q = q > 2147483647LL ? 2147483647LL : (q < -2147483648LL ? -2147483648LL : q);
    d.a_q[p] = (int)q;
    d.packed[p] = ((unsigned)c << d.dbits) | (unsigned)D;
    if (d.continuous) { d.amp[p] = (float)a; d.fdec[p] = (float)f; }
    if (err) atomicOr(&d.ctr->err, err);
  }
  // row_ptr: starts at 0, ends at S, never decreases, rows shorter than 2^31
  for (long long i = (long long)blockIdx.x * kBlock + threadIdx.x; i < d.N;
       i += (long long)gridDim.x * kBlock) {
    const long long a = d.row_ptr[i], b = d.row_ptr[i + 1];
    bool bad = a > b || a < 0 || b > d.S || b - a > 0x7fffffffLL;
    if (i == 0 && a != 0) bad = true;
    if (i == d.N - 1 && b != d.S) bad = true;
    if (bad) atomicOr(&d.ctr->err, ERR_GRAPH);
  }
}

// ---------------------------------------------------------------- bounded queues (FIFO / SORTED)
//
// Every target owns `capacity` slots (arrival step, Q8.24 amplitude), slot-major so that one
// slot of 64 consecutive targets is one line.  A step is two launches:
//   k_fanout   one block per spike walks the CSR row; an event whose target is already full is
//              dropped at once (the occupancy only grows during a step's enqueue phase); every
//              other event registers as a contender of its target: ticket = atomic count,
//              tickets below kCont go to the target's contender slots, later ones to an overflow
//              list (linked list through a pool);
//   k_neurons  the thread that owns target j first admits j's contenders of the step before --
//              the min(K, free) with the smallest synapse index, the canonical order -- then pops
//              the events due now, integrates and compacts the spikes.
// So admission needs no atomics on the slots and no launch of its own; a contender's fate is known
// one launch later (entry points that read counters or admission flags admit what is pending first).
// FIFO keeps, per target, the earliest stored arrival step, so that only the targets with an event
// due now scan their slots; SORTED keeps the slots ordered and pops from the front.

constexpr int kCont = 8;   // contender slots per target and step before the overflow list is used

// Stores one admitted event for target g (owner thread).  FIFO: into the next free slot.
// SORTED: into its place in the circular array ordered by arrival step (behind the stored events
// with the same step); the events behind it move up one slot, eight at a time so that the loads
// of a group are in flight together.
template <int KIND>
__device__ __forceinline__ void store_event(const Dev& d, int g, int occ, int hd, unsigned k, int a) {
  const size_t BN = (size_t)d.BN;
  if (KIND == ADSEQ_FIFO) {
    const size_t si = (size_t)occ * BN + g;
    d.slot_k[si] = k; d.slot_a[si] = a;
    return;
  }
  // position: first index (from the front) whose arrival step exceeds k; binary search
  int lo = 0, hi = occ;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    int ph = hd + mid; if (ph >= d.C) ph -= d.C;
    if (d.slot_k[(size_t)ph * BN + g] <= k) lo = mid + 1; else hi = mid;
  }
  for (int top = occ; top > lo;) {
    const int nmove = top - lo < 8 ? top - lo : 8;     // move entries [top - nmove, top) up by one
    unsigned mk[8]; int ma[8];
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < nmove) {
        int ph = hd + top - 1 - j; if (ph >= d.C) ph -= d.C;
        mk[j] = d.slot_k[(size_t)ph * BN + g]; ma[j] = d.slot_a[(size_t)ph * BN + g];
      }
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (j < nmove) {
        int pd = hd + top - j; if (pd >= d.C) pd -= d.C;
        d.slot_k[(size_t)pd * BN + g] = mk[j]; d.slot_a[(size_t)pd * BN + g] = ma[j];
      }
    top -= nmove;
  }
  int pw = hd + lo; if (pw >= d.C) pw -= d.C;
  d.slot_k[(size_t)pw * BN + g] = k; d.slot_a[(size_t)pw * BN + g] = a;
}

// Admits the contenders registered for target g (owner thread): the min(K, free) with the
// smallest synapse index are stored, the others dropped (counted into c_drop / s_drop).
// Occupancy, earliest stored arrival (FIFO) and front index (SORTED) of a target: loaded once at
// the start of k_neurons, kept in registers through admission and pop, written back at the end.
struct QState { int occ; unsigned mn; int hd; };

template <int KIND>
__device__ __forceinline__ void admit_contenders(const Dev& d, int g, int K, QState& q, long long* c_drop,
                                                 long long* s_drop) {
  if (K <= 0) return;
  d.cnt[g] = 0;
  const size_t BN = (size_t)d.BN;
  int occ = q.occ;
  const int F = d.C - occ;
  const int nc = K < kCont ? K : kCont;              // in the contender slots
  const int ovf_head = K > kCont ? d.c_head[g] : -1; // the others: overflow list
  if (K > kCont) d.c_head[g] = -1;
  const int take = K < F ? K : F;
  const int hd = q.hd;
  unsigned mn = q.mn;
  // the contender slots, loaded together
  long long cp[kCont], ct[kCont]; unsigned ck[kCont]; int ca[kCont];
#pragma unroll
  for (int x = 0; x < kCont; ++x) {
    cp[x] = 0x7fffffffffffffffLL; ct[x] = -1; ck[x] = 0; ca[x] = 0;
    if (x < nc) {
      const size_t ci = (size_t)x * BN + g;
      cp[x] = d.cont_p[ci]; ck[x] = d.cont_k[ci]; ca[x] = d.cont_a[ci];
      if (d.record) ct[x] = d.cont_t[ci];
    }
  }
  if (take == K) {
    // room for all: any order
#pragma unroll
    for (int x = 0; x < kCont; ++x)
      if (x < nc) {
        store_event<KIND>(d, g, occ, hd, ck[x], ca[x]);
        ++occ; mn = ck[x] < mn ? ck[x] : mn;
        if (ct[x] >= 0) d.tape_adm[ct[x]] = 1;
      }
    for (int y = ovf_head; y >= 0; y = d.pool_next[y]) {
      const unsigned k = d.pool_k[y];
      store_event<KIND>(d, g, occ, hd, k, d.pool_a[y]);
      ++occ; mn = k < mn ? k : mn;
      const long long t = d.pool_t[y];
      if (t >= 0) d.tape_adm[t] = 1;
    }
  } else {
    // oversubscribed: the `take` smallest synapse indices win, the others are dropped
    long long last = -1;
    for (int r = 0; r < take; ++r) {
      long long bp = 0x7fffffffffffffffLL; int bx = -1, by = -1;
#pragma unroll
      for (int x = 0; x < kCont; ++x)
        if (cp[x] > last && cp[x] < bp) { bp = cp[x]; bx = x; }
      for (int y = ovf_head; y >= 0; y = d.pool_next[y]) {
        const long long pp = d.pool_p[y];
        if (pp > last && pp < bp) { bp = pp; by = y; bx = -1; }
      }
      if (bx < 0 && by < 0) break;   // not reached: K counts exactly the registered contenders
      last = bp;
      unsigned k = 0; int a = 0; long long t = -1;
      if (bx >= 0) {
#pragma unroll
        for (int x = 0; x < kCont; ++x) if (x == bx) { k = ck[x]; a = ca[x]; t = ct[x]; }
      } else {
        k = d.pool_k[by]; a = d.pool_a[by]; t = d.pool_t[by];
      }
      store_event<KIND>(d, g, occ, hd, k, a);
      ++occ; mn = k < mn ? k : mn;
      if (t >= 0) d.tape_adm[t] = 1;
    }
#pragma unroll
    for (int x = 0; x < kCont; ++x)
      if (x < nc && cp[x] > last) {
        *c_drop += 1; *s_drop += ca[x];
        if (ct[x] >= 0) d.tape_adm[ct[x]] = 0;
      }
    for (int y = ovf_head; y >= 0; y = d.pool_next[y]) {
      if (d.pool_p[y] > last) {
        *c_drop += 1; *s_drop += d.pool_a[y];
        const long long t = d.pool_t[y];
        if (t >= 0) d.tape_adm[t] = 0;
      }
    }
  }
  q.occ = occ; q.mn = mn;
}

// One thread per (trial, neuron).  MODE 0: admission only (what is pending); 1: admission + pop,
// writes the popped current to I_out (open loop); 2: admission + pop + drive + LIF + spike
// compaction + tape (closed loop).
template <int KIND, int MODE>
__global__ __launch_bounds__(kBlock) void k_neurons(Dev d, long long n, int parity,
                                                    const float* __restrict__ i_ext,
                                                    unsigned char* __restrict__ spikes_out,
                                                    float* __restrict__ I_out) {
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  int acc = 0;
  long long popped = 0, c_drop = 0, s_drop = 0;
  const unsigned kn = (unsigned)n;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    d.ctr->pool_n[0] = 0;                        // the overflow pool is consumed by this launch
    if (MODE == 2) d.ctr->n_spk[parity ^ 1] = 0;  // next step's spike counter; nobody reads it now
  }
  float v = 0.0f;
  if (act) {
    // everything the thread needs first, loaded together
    const int K = d.cnt[g];
    QState q, q0;
    q.occ = d.occ[g];
    q.mn = KIND == ADSEQ_FIFO ? d.min_k[g] : 0u;
    q.hd = KIND == ADSEQ_SORTED ? d.head[g] : 0;
    if (MODE == 2) v = d.V[g];
    q0 = q;
    admit_contenders<KIND>(d, g, K, q, &c_drop, &s_drop);
    if (MODE != 0) {
      const size_t BN = (size_t)d.BN;
      if (KIND == ADSEQ_FIFO) {
        // bounded bag: every stored event due now leaves.  Pass 1 only reads (all slot loads
        // in flight together): sum of the due events, their positions, earliest arrival among
        // the others.  Pass 2 fills each hole with the last stored event (the bag is unordered).
        if (q.mn == kn) {
          const int occ = q.occ;
          unsigned mn = 0xffffffffu;
          int ndue = 0;
          int due[8];                      // positions of the first 8 due events, ascending
          for (int s0 = 0; s0 < occ; s0 += 16) {
            unsigned kk[16];                // 16 slot loads in flight, then their tests
#pragma unroll
            for (int j = 0; j < 16; ++j) kk[j] = s0 + j < occ ? d.slot_k[(size_t)(s0 + j) * BN + g] : 0xffffffffu;
#pragma unroll
            for (int j = 0; j < 16; ++j) {
              if (s0 + j < occ) {
                if (kk[j] == kn) { if (ndue < 8) due[ndue] = s0 + j; ++ndue; }
                else mn = kk[j] < mn ? kk[j] : mn;
              }
            }
          }
          int top = occ;
          if (ndue <= 8) {
            for (int j = ndue - 1; j >= 0; --j) {   // from the back, so that the last event is a survivor or the hole itself
              const int s = due[j];
              acc = wrap_add(acc, d.slot_a[(size_t)s * BN + g]);
              --top;
              if (s != top) {
                d.slot_k[(size_t)s * BN + g] = d.slot_k[(size_t)top * BN + g];
                d.slot_a[(size_t)s * BN + g] = d.slot_a[(size_t)top * BN + g];
              }
            }
          } else {
            // many due at once: pack the survivors to the front
            int keep = 0;
            for (int s = 0; s < occ; ++s) {
              const size_t si = (size_t)s * BN + g;
              const unsigned k = d.slot_k[si];
              if (k == kn) {
                acc = wrap_add(acc, d.slot_a[si]);
              } else {
                if (keep != s) { d.slot_k[(size_t)keep * BN + g] = k; d.slot_a[(size_t)keep * BN + g] = d.slot_a[si]; }
                ++keep;
              }
            }
            top = keep;
          }
          popped += ndue;
          q.occ = top;
          q.mn = mn;
        }
      } else {
        // ordered by arrival: everything due now sits at the front of the circular array
        int occ = q.occ, hd = q.hd;
        while (occ > 0 && d.slot_k[(size_t)hd * BN + g] == kn) {
          acc = wrap_add(acc, d.slot_a[(size_t)hd * BN + g]);
          hd = hd + 1 == d.C ? 0 : hd + 1;
          --occ;
          ++popped;
        }
        q.occ = occ; q.hd = hd;
      }
    }
    if (q.occ != q0.occ) d.occ[g] = q.occ;
    if (KIND == ADSEQ_FIFO && q.mn != q0.mn) d.min_k[g] = q.mn;
    if (KIND == ADSEQ_SORTED && q.hd != q0.hd) d.head[g] = q.hd;
  }
  bool s = false;
  if (act && MODE != 0) {
    float I = (float)acc * 0x1p-24f;
    if (MODE == 2) {
      if (d.p_thresh) {
        const bool xi = (unsigned long long)drive_bits(d.seed, (unsigned long long)g,
                                                       (unsigned long long)n) < d.p_thresh;
        I = I + (xi ? d.ext_w : 0.0f);
      }
      if (i_ext) I = I + i_ext[g];
      const float U = __fmaf_rn(d.alpha, v, I);
      s = U >= d.theta;
      d.V[g] = s ? d.v_reset : U;
      if (d.record && n < d.max_steps) {
        d.tapeU[(size_t)n * d.BN + g] = U;
        if (s) d.spk_count[g] += 1;
      }
      if (spikes_out) spikes_out[g] = s ? 1 : 0;
    } else {
      I_out[g] = I;
    }
  }
  if (MODE == 2) {
    // wavefront ballot + prefix popcount; one atomic per wavefront that has spikes
    const unsigned long long m = __ballot(s);
    const int lane = threadIdx.x & 63;
    int base = 0;
    if (lane == 0 && m) base = atomicAdd(&d.ctr->n_spk[parity], __popcll(m));
    base = __shfl(base, 0, 64);
    if (s) d.cur_spk[base + __popcll(m & ((1ull << lane) - 1ull))] = g;
  }
  BlkCtr& bc = d.blk[blockIdx.x];
  block_add2(&bc.delivered, popped, &bc.sum_delivered, (long long)acc);
  block_add2(&bc.dropped, c_drop, &bc.sum_dropped, s_drop);
}

// One block per spike (grid-stride over the spike list); the block walks the CSR row with
// coalesced reads of (packed, a_q).  Events whose target is already full are dropped here; the
// others register as contenders of their target (see above).
template <int KIND>
__global__ __launch_bounds__(kBlock) void k_fanout(Dev d, long long n, const int* __restrict__ spk,
                                                   const int* __restrict__ n_spk_ptr, int record) {
  __shared__ long long s_evb;
  int nspk = *n_spk_ptr;
  nspk = nspk < 0 ? 0 : (nspk > d.BN ? d.BN : nspk);
  const long long off = record ? d.step_off[n] : 0;
  const int lane = threadIdx.x & 63;
  const size_t BN = (size_t)d.BN;
  long long c_off = 0, s_off = 0, c_drop = 0, s_drop = 0;
  for (int e = blockIdx.x; e < nspk; e += gridDim.x) {
    const int g = spk[e];
    if ((unsigned)g >= (unsigned)d.BN) continue;  // uniform over the block
    const int b = g / d.N, i = g - b * d.N;
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    long long tbase = -1;
    if (record) {
      const bool fits = off + e < d.spike_cap;
      if (threadIdx.x == 0) {
        if (fits) d.tape_spk[off + e] = g; else atomicOr(&d.ctr->err, ERR_TAPE_SPIKES);
        long long evb = (long long)atomicAdd((unsigned long long*)&d.ctr->tape_events,
                                             (unsigned long long)(r1 - r0));
        if (evb + (r1 - r0) > d.event_cap) { atomicOr(&d.ctr->err, ERR_TAPE_EVENTS); evb = -1; }
        if (fits) d.tape_evb[off + e] = evb;
        s_evb = evb;
      }
      __syncthreads();
      tbase = s_evb;
      __syncthreads();
    }
    // four row entries per thread and trip, each stage for all four before the next, so that
    // the loads, the occupancy gathers and the ticket atomics of a trip are in flight together
    for (long long p0 = r0; p0 < r1; p0 += 4 * kBlock) {
      long long p[4]; bool valid[4]; unsigned pk[4]; int a[4], gt[4], tk[4]; bool contend[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        p[j] = p0 + j * kBlock + threadIdx.x;
        valid[j] = p[j] < r1;
        pk[j] = 0; a[j] = 0;
        if (valid[j]) { pk[j] = d.packed[p[j]]; a[j] = d.a_q[p[j]]; }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        gt[j] = b * d.N + (int)(pk[j] >> d.dbits);
        contend[j] = false;
        if (valid[j]) { c_off += 1; s_off += a[j]; contend[j] = d.occ[gt[j]] < d.C; }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        tk[j] = -1;
        if (contend[j]) tk[j] = atomicAdd(&d.cnt[gt[j]], 1);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int D = (int)(pk[j] & d.dmask);
        const long long tidx = (valid[j] && tbase >= 0) ? tbase + (p[j] - r0) : -1;
        if (valid[j] && !contend[j]) { c_drop += 1; s_drop += a[j]; if (tidx >= 0) d.tape_adm[tidx] = 0; }
        if (contend[j] && tk[j] < kCont) {
          const size_t ci = (size_t)tk[j] * BN + gt[j];
          d.cont_p[ci] = p[j]; d.cont_k[ci] = (unsigned)(n + D); d.cont_a[ci] = a[j];
          if (d.record) d.cont_t[ci] = tidx;
        }
        // the others: wavefront-aggregated claim of pool entries, pushed on the target's list
        const bool over = contend[j] && tk[j] >= kCont;
        const unsigned long long cm = __ballot(over);
        if (cm) {
          int base = 0;
          if (lane == __ffsll((long long)cm) - 1) base = atomicAdd(&d.ctr->pool_n[0], __popcll(cm));
          base = __shfl(base, __ffsll((long long)cm) - 1, 64);
          if (over) {
            const int x = base + __popcll(cm & ((1ull << lane) - 1ull));
            if (x >= d.pool_cap) {
              // no room to remember it: it can only be dropped, and the run is flagged as invalid
              atomicOr(&d.ctr->err, ERR_POOL);
              atomicSub(&d.cnt[gt[j]], 1);
              c_drop += 1; s_drop += a[j]; if (tidx >= 0) d.tape_adm[tidx] = 0;
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
  if (record && blockIdx.x == 0 && threadIdx.x == 0) {
    if (n + 1 <= d.max_steps) d.step_off[n + 1] = off + nspk;
    d.ctr->tape_spikes = off + nspk;
  }
  BlkCtr& bc = d.blk[d.nblk + blockIdx.x];
  block_add2(&bc.offered, c_off, &bc.sum_offered, s_off);
  block_add2(&bc.dropped, c_drop, &bc.sum_dropped, s_drop);
}

__global__ __launch_bounds__(kBlock) void k_copy_i32(const int* __restrict__ src, int* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) dst[i] = src[i];
}

// ---------------------------------------------------------------- ring queue (windowed delay line)

#include "ring_window.h"

// ---------------------------------------------------------------- backward (FIFO / SORTED)

// Queue term of the reverse sweep at step n: one block per recorded spike (b, i, n).  Gathers the
// adjoint at each admitted event's arrival slot, reduces G_i, and accumulates the weight and
// delay gradients of the row.
template <bool ATOMIC>
__global__ __launch_bounds__(kBlock) void k_bwd_gather(Dev d, long long n, long long T, float dscale,
                                                       float* __restrict__ grad_w,
                                                       float* __restrict__ grad_d) {
  __shared__ float red[kBlock / 64];
  const long long off = d.step_off[n];
  const int cnt = (int)(d.step_off[n + 1] - off);
  const int m = (int)(n % d.R);
  for (int e = blockIdx.x; e < cnt; e += gridDim.x) {
    const int g = d.tape_spk[off + e];
    const int b = g / d.N, i = g - b * d.N;
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    const long long evb = d.tape_evb[off + e];
    float G = 0.0f;
    for (long long p = r0 + threadIdx.x; p < r1; p += kBlock) {
      const unsigned pk = d.packed[p];
      const int D = (int)(pk & d.dmask);
      const int col = (int)(pk >> d.dbits);
      if (n + D >= T) continue;                               // not delivered inside the run
      if (!d.tape_adm[evb + (p - r0)]) continue;              // refused by a full queue
      int slot = m + D; if (slot >= d.R) slot -= d.R;
      const float gv = d.bwd_ring[(size_t)slot * d.BN + (size_t)b * d.N + col];
      const float a = d.continuous ? d.amp[p] : d.weight[p];
      const float f = d.continuous ? d.fdec[p] : 1.0f;
      G += a * gv;
      const float gw = f * gv, gd = a * dscale * gv;
      if (ATOMIC) { unsafeAtomicAdd(&grad_w[p], gw); unsafeAtomicAdd(&grad_d[p], gd); }
      else { grad_w[p] += gw; grad_d[p] += gd; }
    }
    G = wave_sum_f(G);
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = G;
    __syncthreads();
    if (threadIdx.x == 0) {
      float t = 0.0f;
      for (int w = 0; w < kBlock / 64; ++w) t += red[w];
      d.bwd_G[g] = t;
    }
    __syncthreads();
  }
}

// Neuron part of the reverse sweep at step n:
//   gU[n] = (1 - s) alpha gU[n+1] + sigma'(U - theta) (dL/dcount + s G) + dL/dU[n]
__global__ __launch_bounds__(kBlock) void k_bwd_neurons(Dev d, long long n,
                                                        const float* __restrict__ dL_dcount,
                                                        const float* __restrict__ dL_dU) {
  const int g = blockIdx.x * kBlock + threadIdx.x;
  if (g >= d.BN) return;
  const float U = d.tapeU[(size_t)n * d.BN + g];
  const bool s = U >= d.theta;
  float sg = 0.0f;
  if (d.surrogate == ADSEQ_SURR_SUPERSPIKE) {
    const float x = fabsf(U - d.theta) + 1.0f;
    sg = 1.0f / (x * x);
  }
  float inner = dL_dcount ? dL_dcount[g] : 0.0f;
  if (s) inner += d.bwd_G[g];
  float gu = sg * inner;
  if (!s) gu = __fmaf_rn(d.alpha, d.bwd_carry[g], gu);
  if (dL_dU) gu += dL_dU[(size_t)n * d.BN + g];
  d.bwd_carry[g] = gu;
  d.bwd_ring[(size_t)(n % d.R) * d.BN + g] = gu;
}

}  // namespace

// ---------------------------------------------------------------- host side

struct adseq {
  adseq_config cfg;
  Dev dev;
  size_t ws_bytes;
  long long next_step;   // next step to deliver
  long long enq_calls;   // parity source for the pool / spike counters
  bool tape_ok;          // every step since reset went through adseq_step with recording
  char err[256];
  long long fold_upto = 0;  // RING: spikes of steps below this are in the device counters
  bool pending_admit = false;  // FIFO/SORTED: contenders registered, admission not yet launched
  hipStream_t last_stream = nullptr;  // stream of the last enqueue
  // optional kernel timing (adseq_profile): one event after each bracketed launch
  bool prof = false;
  std::vector<hipEvent_t> evs;
  std::vector<int> ev_kind;   // kernel class the event closes, -1 = start marker
  std::vector<int> ev_count;  // launches between the previous event and this one
  bool grp_open = false;      // RING: a group of consecutive step launches is being timed
  int grp_count = 0;
  size_t ev_used = 0;
};

namespace {

struct Layout {
  size_t V, win, spike_bits, slot_k, slot_a, occ, head, min_k, cnt, cont_p, cont_k, cont_a, cont_t, c_head, pool_p, pool_t, pool_next,
      pool_k, pool_a, cur_spk, packed, a_q, synf, synb, dstart, nearcnt, perm, rowsum, ebuf, ecnt, amp, fdec, tapeU,
      tape_bits, spk_count, step_off, tape_spk, tape_evb, tape_adm, bwd_ring, bwd_carry, bwd_G, gwin, Gacc, gsum, ctr, blk,
      total;
  long long spike_cap, event_cap, pool_cap;
  int R, dbits, nblk, words;
  int W, wshift, tp_shift, P, NB, cap, wgroups;  // RING
};

// A power of two in [lo, hi] from the environment, else the default (tuning knobs of the ring:
// results do not depend on them).
int env_pow2(const char* name, int dflt, int lo, int hi) {
  if (const char* e = getenv(name)) {
    const int v = atoi(e);
    if (v >= lo && v <= hi && (v & (v - 1)) == 0) return v;
  }
  return dflt;
}
// Window length of the ring in steps.
int ring_window_steps() { return env_pow2("ADSEQ_RING_WINDOW", 16, 2, 64); }
// Cells (target, step) of the LDS tile of one target part.
int ring_tile_cells() { return env_pow2("ADSEQ_RING_TILE", 4096, 1024, kMaxTileCells); }

int bit_width(unsigned v) { int b = 0; while (v) { ++b; v >>= 1; } return b; }

bool host_validate(const adseq_config* c) {
  if (!c) return false;
  if (c->n_neurons < 1 || c->batch < 1 || c->d_max_steps < 1 || c->d_max_steps > 1023) return false;
  if ((long long)c->n_neurons * c->batch > 0x7fffffffLL) return false;
  if (c->kind != ADSEQ_RING && c->kind != ADSEQ_FIFO && c->kind != ADSEQ_SORTED) return false;
  if (c->kind != ADSEQ_RING && (c->capacity < 1 || c->capacity > 32767)) return false;
  if (c->surrogate != ADSEQ_SURR_SUPERSPIKE && c->surrogate != ADSEQ_SURR_OFF) return false;
  if (!(c->dt_ms > 0.0f) || !(c->tau_m_ms > 0.0f) || c->dt_ms > c->tau_m_ms) return false;
  if (!(c->ext_rate_hz >= 0.0f)) return false;
  if (c->n_synapses < 0) return false;
  if (c->record_tape && c->max_steps < 1) return false;
  if (c->tape_spike_capacity < 0 || c->tape_event_capacity < 0 || c->step_event_capacity < 0)
    return false;
  if (bit_width((unsigned)(c->n_neurons - 1)) + bit_width((unsigned)c->d_max_steps) > 32) return false;
  return true;
}

bool make_layout(const adseq_config* c, Layout* L) {
  if (!host_validate(c)) return false;
  const size_t BN = (size_t)c->n_neurons * c->batch;
  const size_t S = (size_t)c->n_synapses;
  const bool bounded = c->kind != ADSEQ_RING;
  const bool cont = c->delay_ms != nullptr;
  L->R = c->d_max_steps + 1;
  L->dbits = bit_width((unsigned)c->d_max_steps);
  L->spike_cap = 0; L->event_cap = 0; L->pool_cap = 0;
  if (c->record_tape) {
    L->spike_cap = c->tape_spike_capacity ? c->tape_spike_capacity
                                          : (long long)((size_t)c->max_steps * BN / 16 + BN);
    if (bounded) {
      const long long fan = (long long)((S + c->n_neurons - 1) / c->n_neurons);
      L->event_cap = c->tape_event_capacity ? c->tape_event_capacity : L->spike_cap * (fan ? fan : 1);
    }
  }
  if (bounded) {
    long long cap = c->step_event_capacity;
    if (!cap) {
      const double bs = (double)c->batch * (double)S;
      cap = bs < 16777216.0 ? (long long)bs : 16777216LL;
      if (cap < 1) cap = 1;
    }
    if (cap > 0x7fffffffLL) cap = 0x7fffffffLL;
    L->pool_cap = cap;
  }
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o += (bytes + 255) & ~(size_t)255; return at; };
  L->nblk = (int)((BN + kBlock - 1) / kBlock);
  L->words = 0;
  L->W = L->wshift = L->tp_shift = L->P = L->NB = L->cap = L->wgroups = 0;
  size_t stage_parts = 0;
  if (!bounded) {
    L->words = L->nblk * (kBlock / 64);
    // the window is no longer than the largest delay (so that a window boundary comes before
    // any spike word is overwritten)
    L->W = ring_window_steps();
    while (L->W > c->d_max_steps) L->W >>= 1;
    L->wshift = bit_width((unsigned)L->W) - 1;
    int cells = ring_tile_cells();
    if (cells < L->W) cells = L->W;
    L->tp_shift = bit_width((unsigned)cells) - 1 - L->wshift;
    L->P = (int)((BN + ((size_t)1 << L->tp_shift) - 1) >> L->tp_shift);
    L->wgroups = (L->words + 7) / 8;
    // blocks of the staging pass: about four 8-word lines per wavefront when the history is
    // full, but no more than one block per compute unit (measured best on cfg3: 256 of 128..512)
    const long long lines = (long long)c->d_max_steps * L->wgroups;
    long long nb = (lines + 4 * kRingWaves - 1) / (4 * kRingWaves);
    L->NB = env_pow2("ADSEQ_RING_BINBLOCKS", (int)(nb < 1 ? 1 : (nb > 256 ? 256 : nb)), 1, kMaxBinBlocks);
    stage_parts = (size_t)(L->P < kMaxParts ? L->P : kMaxParts);
    // staging capacity in events: by default what a window holds when every neuron fires at
    // 1/32 per step, between 2^16 and 2^26 events
    double ev = c->step_event_capacity ? (double)c->step_event_capacity
                                       : (double)c->batch * (double)S * (double)L->W / 32.0;
    if (!c->step_event_capacity) ev = ev < 65536.0 ? 65536.0 : (ev > 67108864.0 ? 67108864.0 : ev);
    const double per = ev / ((double)stage_parts * (double)L->NB);
    L->cap = (int)(per > 65536.0 ? 65536.0 : per);
  }
  L->ctr = take(sizeof(Counters));
  L->blk = take(bounded ? ((size_t)L->nblk + kFanoutBlocks) * sizeof(BlkCtr) : 0);
  L->V = take(BN * 4);
  L->win = take(bounded ? 0 : 2 * (size_t)L->W * BN * 4);
  L->spike_bits = take(bounded ? 0 : (size_t)L->R * L->words * 8);
  L->slot_k = take(bounded ? (size_t)c->capacity * BN * 4 : 0);
  L->slot_a = take(bounded ? (size_t)c->capacity * BN * 4 : 0);
  L->occ = take(bounded ? BN * 4 : 0);
  L->head = take(bounded ? BN * 4 : 0);
  L->min_k = take(bounded ? BN * 4 : 0);
  L->cnt = take(bounded ? BN * 4 : 0);
  L->cont_p = take(bounded ? (size_t)kCont * BN * 8 : 0);
  L->cont_k = take(bounded ? (size_t)kCont * BN * 4 : 0);
  L->cont_a = take(bounded ? (size_t)kCont * BN * 4 : 0);
  L->cont_t = take(bounded && c->record_tape ? (size_t)kCont * BN * 8 : 0);
  L->c_head = take(bounded ? BN * 4 : 0);
  L->pool_p = take((size_t)L->pool_cap * 8);
  L->pool_t = take((size_t)L->pool_cap * 8);
  L->pool_next = take((size_t)L->pool_cap * 4);
  L->pool_k = take((size_t)L->pool_cap * 4);
  L->pool_a = take((size_t)L->pool_cap * 4);
  L->cur_spk = take(BN * 4);
  L->packed = take(bounded ? S * 4 : 0);
  L->a_q = take(bounded ? S * 4 : 0);
  L->synf = take(bounded ? 0 : S * 8);
  L->synb = take(bounded ? 0 : S * 8);
  L->dstart = take(bounded ? 0 : (size_t)c->n_neurons * (c->d_max_steps + 2) * 4);
  L->nearcnt = take(bounded ? 0 : (size_t)(L->W + 1) * c->n_neurons * 4);
  L->perm = take(bounded ? 0 : S * 4);
  L->rowsum = take(bounded ? 0 : (size_t)c->n_neurons * 8);
  L->ebuf = take(bounded ? 0 : stage_parts * L->NB * (size_t)L->cap * 8);
  L->ecnt = take(bounded ? 0 : stage_parts * L->NB * 4);
  L->amp = take(cont && bounded ? S * 4 : 0);
  L->fdec = take(cont ? S * 4 : 0);
  const size_t T = c->record_tape ? (size_t)c->max_steps : 0;
  L->tapeU = take(T * BN * 4);
  L->tape_bits = take(bounded ? 0 : T * L->words * 8);
  L->spk_count = take(c->record_tape ? BN * 4 : 0);
  L->step_off = take(c->record_tape ? (T + 1) * 8 : 0);
  L->tape_spk = take(bounded ? (size_t)L->spike_cap * 4 : 0);
  L->tape_evb = take(bounded ? (size_t)L->spike_cap * 8 : 0);
  L->tape_adm = take((size_t)L->event_cap);
  const bool tape = c->record_tape != 0;
  L->bwd_ring = take(tape && bounded ? (size_t)L->R * BN * 4 : 0);
  L->bwd_carry = take(tape ? BN * 4 : 0);
  L->bwd_G = take(tape && bounded ? BN * 4 : 0);
  L->gwin = take(tape && !bounded ? 2 * (size_t)L->W * BN * 4 : 0);
  L->Gacc = take(tape && !bounded ? (size_t)L->R * BN * 4 : 0);
  L->gsum = take(tape && !bounded ? S * 4 : 0);
  L->total = o;
  return true;
}

int fail(adseq* h, int code, const char* fmt, ...) {
  if (h) {
    va_list ap; va_start(ap, fmt);
    vsnprintf(h->err, sizeof(h->err), fmt, ap);
    va_end(ap);
  }
  return code;
}

#define HIP_TRY(h, call)                                                              \
  do {                                                                                \
    hipError_t e_ = (call);                                                           \
    if (e_ != hipSuccess)                                                             \
      return fail((h), ADSEQ_E_HIP, "%s failed: %s", #call, hipGetErrorString(e_));   \
  } while (0)

int grid_for(size_t n) {
  size_t g = (n + kBlock - 1) / kBlock;
  return (int)(g < 1 ? 1 : (g > 65535 * 16 ? 65535 * 16 : g));
}

void fill_u32(hipStream_t st, void* p, unsigned v, size_t count) {
  if (!count) return;
  size_t g = (count + kBlock - 1) / kBlock;
  if (g > 4096) g = 4096;
  hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)g), dim3(kBlock), 0, st, (unsigned*)p, v, count);
}

// Clears the dynamic state (not the prepared synapses).
void launch_reset(adseq* h, hipStream_t st) {
  const Dev& d = h->dev;
  h->fold_upto = 0;
  const size_t BN = (size_t)d.BN;
  fill_u32(st, d.ctr, 0u, sizeof(Counters) / 4);
  fill_u32(st, d.V, 0u, BN);
  if (d.kind == ADSEQ_RING) {
    fill_u32(st, d.win, 0u, 2 * (size_t)d.W * BN);
    fill_u32(st, d.spike_bits, 0u, (size_t)d.R * d.words * 2);
  } else {
    fill_u32(st, d.occ, 0u, BN);
    fill_u32(st, d.head, 0u, BN);
    fill_u32(st, d.c_head, 0xffffffffu, BN);
    fill_u32(st, d.min_k, 0xffffffffu, BN);
    fill_u32(st, d.cnt, 0u, BN);
    fill_u32(st, d.blk, 0u, ((size_t)d.nblk + kFanoutBlocks) * sizeof(BlkCtr) / 4);
    h->pending_admit = false;
  }
  if (d.record) {
    fill_u32(st, d.step_off, 0u, 2);  // step_off[0] = 0 (int64)
    fill_u32(st, d.spk_count, 0u, BN);
  }
  h->next_step = 0;
  h->enq_calls = 0;
  h->tape_ok = d.record != 0;
}

// FIFO / SORTED: admission of what is pending, then (MODE 1) pop or (MODE 2) the closed-loop step.
template <int MODE>
void launch_neurons(adseq* h, hipStream_t st, long long n, int parity, const float* i_ext,
                    unsigned char* spikes_out, float* I_out) {
  const Dev& d = h->dev;
  const dim3 grid(grid_for((size_t)d.BN)), block(kBlock);
  if (d.kind == ADSEQ_FIFO)
    hipLaunchKernelGGL((k_neurons<ADSEQ_FIFO, MODE>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
  else
    hipLaunchKernelGGL((k_neurons<ADSEQ_SORTED, MODE>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
  h->pending_admit = false;
}

void launch_fanout(adseq* h, hipStream_t st, long long n, const int* spk, const int* n_spk, int record) {
  const Dev& d = h->dev;
  const dim3 grid(kFanoutBlocks), block(kBlock);
  if (d.kind == ADSEQ_FIFO)
    hipLaunchKernelGGL((k_fanout<ADSEQ_FIFO>), grid, block, 0, st, d, n, spk, n_spk, record);
  else
    hipLaunchKernelGGL((k_fanout<ADSEQ_SORTED>), grid, block, 0, st, d, n, spk, n_spk, record);
  h->pending_admit = true;
  h->last_stream = st;
}

// FIFO / SORTED: admits the contenders that the last enqueue registered, if that has not
// happened yet (it normally rides on the next step's launch).
void flush_admit(adseq* h, hipStream_t st) {
  if (h->dev.kind != ADSEQ_RING && h->pending_admit) launch_neurons<0>(h, st, 0, 0, nullptr, nullptr, nullptr);
}

void mark(adseq* h, hipStream_t st, int kind, int count = 1);
void close_group(adseq* h, hipStream_t st, int kind);

// RING: called before step k0 is popped when k0 opens a window (k0 mod W = 0): expands the
// events of the spikes of the last d_max steps that arrive in the window (staging pass, then
// per-part accumulation; without staging room the first pass scatters with atomics and the
// second is skipped).  The staging pass also counts the spikes not counted yet, and their
// events, into the device counters.
void ring_open_window(adseq* h, hipStream_t st, long long k0) {
  const Dev& d = h->dev;
  if ((k0 & (long long)(d.W - 1)) != 0 || k0 <= 0) return;
  close_group(h, st, 1);
  mark(h, st, -1);
  const long long n_lo = k0 - d.d_max > 0 ? k0 - d.d_max : 0;
  hipLaunchKernelGGL(k_win_bin, dim3((unsigned)d.NB), dim3(kRingThreads), 0, st, d, k0, n_lo, k0, 0, d.NB,
                     d.cap > 0 ? 1 : 0, h->fold_upto);
  if (d.cap > 0) {
    const int parts = d.P < kMaxParts ? d.P : kMaxParts;
    hipLaunchKernelGGL(k_win_acc, dim3((unsigned)parts), dim3(kRingThreads), 0, st, d, k0, 0);
  }
  h->fold_upto = k0;
  mark(h, st, 0);
}

// Records an event that closes a launch of class `kind` (and opens the next one).
void mark(adseq* h, hipStream_t st, int kind, int count) {
  if (!h->prof) return;
  if (h->ev_used == h->evs.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    h->evs.push_back(e); h->ev_kind.push_back(kind); h->ev_count.push_back(count);
  }
  h->ev_kind[h->ev_used] = kind;
  h->ev_count[h->ev_used] = count;
  (void)hipEventRecord(h->evs[h->ev_used], st);
  h->ev_used += 1;
}

// RING: the step launches are timed in groups (all the steps between two window boundaries
// between one pair of events), since an event after every 5 us launch would add half as much.
void open_group(adseq* h, hipStream_t st) {
  if (!h->prof || h->grp_open) return;
  mark(h, st, -1);
  h->grp_open = true; h->grp_count = 0;
}
void close_group(adseq* h, hipStream_t st, int kind) {
  if (!h->prof || !h->grp_open) return;
  mark(h, st, kind, h->grp_count);
  h->grp_open = false;
}

int step_impl(adseq* h, long long step, const float* i_ext, unsigned char* spikes_out, hipStream_t st) {
  if (step != h->next_step)
    return fail(h, ADSEQ_E_ORDER, "adseq_step: got step %lld, expected %lld", step, h->next_step);
  const Dev& d = h->dev;
  const int parity = (int)(h->enq_calls & 1);
  const int record = (d.record && h->tape_ok && step < d.max_steps) ? 1 : 0;
  if (d.record && step >= d.max_steps) h->tape_ok = false;
  if (d.kind == ADSEQ_RING) {
    ring_open_window(h, st, step);
    open_group(h, st);
    const dim3 grid((unsigned)d.nblk), block(kBlock);
    if (record) hipLaunchKernelGGL((k_step_win<true>), grid, block, 0, st, d, step, i_ext, spikes_out);
    else hipLaunchKernelGGL((k_step_win<false>), grid, block, 0, st, d, step, i_ext, spikes_out);
    h->grp_count += 1;
  } else {
    mark(h, st, -1);
    launch_neurons<2>(h, st, step, parity, i_ext, spikes_out, nullptr);
    mark(h, st, 1);
    launch_fanout(h, st, step, d.cur_spk, &d.ctr->n_spk[parity], record);
    mark(h, st, 0);
  }
  h->enq_calls += 1;
  h->next_step = step + 1;
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

// RING: virtual blocks of one far gather over the spikes of steps [n_lo, n_hi): about four
// 8-word lines per wavefront.
int gather_blocks(const Dev& d, long long n_lo, long long n_hi) {
  const long long lines = (n_hi - n_lo) * d.wgroups;
  long long g = (lines + 4 * kRingWaves - 1) / (4 * kRingWaves);
  return env_pow2("ADSEQ_RING_GATHERBLOCKS", (int)(g < 1 ? 1 : (g > 256 ? 256 : g)), 1, 2048);
}

// RING: the whole reverse sweep on `st`.  One launch per reverse step; when a step closes a
// window (n mod W = 0) the far queue terms of all earlier spikes that arrive in that window are
// gathered in one pass.
void ring_backward_launch(adseq* h, hipStream_t st, long long T, float dscale, const float* dL_dcount,
                          const float* dL_dU, float* grad_w, float* grad_d) {
  const Dev& d = h->dev;
  const dim3 block(kBlock), gn((unsigned)d.nblk);
  fill_u32(st, d.bwd_carry, 0u, (size_t)d.BN);
  fill_u32(st, d.gsum, 0u, (size_t)d.S);
  fill_u32(st, d.gwin, 0u, 2 * (size_t)d.W * d.BN);
  fill_u32(st, d.Gacc, 0u, (size_t)d.R * d.BN);
  for (long long n = T - 1; n >= 0; --n) {
    open_group(h, st);
    hipLaunchKernelGGL(k_bwd_step_win, gn, block, 0, st, d, n, T, dL_dcount, dL_dU);
    h->grp_count += 1;
    if ((n & (long long)(d.W - 1)) == 0 && n > 0) {
      close_group(h, st, 3);
      mark(h, st, -1);
      const long long lo = n - d.d_max > 0 ? n - d.d_max : 0;
      const int nvb = gather_blocks(d, lo, n);
      hipLaunchKernelGGL(k_bwd_win, dim3((unsigned)nvb), dim3(kRingThreads), 0, st, d, n, lo, n, T, 0, nvb);
      mark(h, st, 2);
    }
  }
  close_group(h, st, 3);
  const unsigned gf = (unsigned)(d.N < 65536 ? d.N : 65536);
  hipLaunchKernelGGL(k_grad_finish, dim3(gf), block, 0, st, d, dscale, grad_w, grad_d);
}

}  // namespace

extern "C" {

size_t adseq_workspace_bytes(const adseq_config* cfg) {
  Layout L;
  if (!make_layout(cfg, &L)) return 0;
  return L.total;
}

int adseq_create(const adseq_config* cfg, adseq_t** out) {
  if (!cfg || !out) return ADSEQ_E_INVALID_ARG;
  Layout L;
  if (!make_layout(cfg, &L)) return ADSEQ_E_INVALID_ARG;
  if (!cfg->row_ptr || !cfg->weight || (!cfg->col && cfg->n_synapses > 0)) return ADSEQ_E_INVALID_ARG;
  if ((cfg->delay_steps == nullptr) == (cfg->delay_ms == nullptr)) return ADSEQ_E_INVALID_ARG;
  if (!cfg->workspace || ((uintptr_t)cfg->workspace & 255) || cfg->workspace_bytes < L.total)
    return ADSEQ_E_WORKSPACE;
  adseq* h = new (std::nothrow) adseq();
  if (!h) return ADSEQ_E_INVALID_ARG;
  h->cfg = *cfg;
  h->ws_bytes = L.total;
  h->err[0] = 0;
  Dev& d = h->dev;
  memset(&d, 0, sizeof(d));
  char* ws = (char*)cfg->workspace;
  d.N = cfg->n_neurons; d.B = cfg->batch; d.BN = cfg->n_neurons * cfg->batch;
  d.R = L.R; d.C = cfg->capacity; d.kind = cfg->kind; d.dbits = L.dbits; d.d_max = cfg->d_max_steps;
  d.dmask = (1u << L.dbits) - 1u;
  d.continuous = cfg->delay_ms ? 1 : 0;
  d.record = cfg->record_tape ? 1 : 0;
  d.surrogate = cfg->surrogate;
  d.max_steps = cfg->record_tape ? cfg->max_steps : 0;
  d.pool_cap = (int)L.pool_cap;
  d.alpha = (float)std::exp(-(double)cfg->dt_ms / (double)cfg->tau_m_ms);
  d.theta = cfg->v_thresh; d.v_reset = cfg->v_reset; d.ext_w = cfg->ext_weight;
  d.dt = cfg->dt_ms; d.tau = cfg->tau_m_ms;
  {
    double p = (double)cfg->ext_rate_hz * (double)cfg->dt_ms * 1e-3;
    if (p < 0.0) p = 0.0;
    if (p > 1.0) p = 1.0;
    d.p_thresh = (unsigned long long)std::floor(p * 4294967296.0);
  }
  d.seed = cfg->seed;
  d.S = cfg->n_synapses; d.spike_cap = L.spike_cap; d.event_cap = L.event_cap;
  d.row_ptr = (const long long*)cfg->row_ptr; d.col = cfg->col; d.weight = cfg->weight;
  d.delay_steps = cfg->delay_steps; d.delay_ms = cfg->delay_ms;
  d.ctr = (Counters*)(ws + L.ctr);
  d.nblk = L.nblk; d.words = L.words; d.blk = (BlkCtr*)(ws + L.blk);
  d.V = (float*)(ws + L.V); d.spike_bits = (unsigned long long*)(ws + L.spike_bits);
  d.W = L.W; d.wshift = L.wshift; d.tp_shift = L.tp_shift; d.P = L.P; d.NB = L.NB; d.cap = L.cap;
  d.wgroups = L.wgroups;
  d.win = (int*)(ws + L.win);
  d.dstart = (unsigned*)(ws + L.dstart); d.nearcnt = (unsigned*)(ws + L.nearcnt);
  d.perm = (unsigned*)(ws + L.perm); d.rowsum = (long long*)(ws + L.rowsum);
  d.ebuf = (uint2*)(ws + L.ebuf); d.ecnt = (int*)(ws + L.ecnt);
  d.tape_bits = (unsigned long long*)(ws + L.tape_bits);
  d.spk_count = (int*)(ws + L.spk_count);
  d.gwin = (float*)(ws + L.gwin); d.Gacc = (float*)(ws + L.Gacc); d.gsum = (float*)(ws + L.gsum);
  d.slot_k = (unsigned*)(ws + L.slot_k); d.slot_a = (int*)(ws + L.slot_a);
  d.occ = (int*)(ws + L.occ); d.head = (int*)(ws + L.head); d.c_head = (int*)(ws + L.c_head);
  d.pool_p = (long long*)(ws + L.pool_p); d.pool_t = (long long*)(ws + L.pool_t);
  d.pool_next = (int*)(ws + L.pool_next);
  d.min_k = (unsigned*)(ws + L.min_k); d.cnt = (int*)(ws + L.cnt);
  d.cont_p = (long long*)(ws + L.cont_p); d.cont_k = (unsigned*)(ws + L.cont_k);
  d.cont_a = (int*)(ws + L.cont_a); d.cont_t = (long long*)(ws + L.cont_t);
  d.pool_k = (unsigned*)(ws + L.pool_k); d.pool_a = (int*)(ws + L.pool_a);
  d.cur_spk = (int*)(ws + L.cur_spk);
  d.packed = (unsigned*)(ws + L.packed); d.a_q = (int*)(ws + L.a_q);
  d.amp = (d.continuous && d.kind != ADSEQ_RING) ? (float*)(ws + L.amp) : nullptr;
  d.synf = (uint2*)(ws + L.synf); d.synb = (uint2*)(ws + L.synb);
  d.fdec = d.continuous ? (float*)(ws + L.fdec) : nullptr;
  d.tapeU = (float*)(ws + L.tapeU); d.step_off = (long long*)(ws + L.step_off);
  d.tape_spk = (int*)(ws + L.tape_spk); d.tape_evb = (long long*)(ws + L.tape_evb);
  d.tape_adm = (unsigned char*)(ws + L.tape_adm);
  d.bwd_ring = (float*)(ws + L.bwd_ring); d.bwd_carry = (float*)(ws + L.bwd_carry);
  d.bwd_G = (float*)(ws + L.bwd_G);

  hipStream_t st = (hipStream_t)cfg->stream;
  launch_reset(h, st);
  ExpCoef ec;
  ec.c[0] = 1.0;
  for (int k = 1; k <= 20; ++k) ec.c[k] = ec.c[k - 1] / (double)k;
  unsigned err = 0;
  auto read_err = [&]() -> hipError_t {
    hipError_t e = hipGetLastError();
    if (e == hipSuccess) e = hipMemcpyAsync(&err, &d.ctr->err, sizeof(err), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    return e;
  };
  hipError_t e = hipSuccess;
  if (d.kind == ADSEQ_RING) {
    // the rows are walked by the sort, so row_ptr is checked (and the result read) first
    hipLaunchKernelGGL(k_check_rows, dim3((unsigned)grid_for((size_t)d.N)), dim3(kBlock), 0, st, d);
    e = read_err();
    if (e == hipSuccess && !err) {
      const unsigned g = (unsigned)(d.N < 262144 ? d.N : 262144);
      hipLaunchKernelGGL(k_sort_rows, dim3(g), dim3(kBlock), 0, st, d, ec);
      e = read_err();
    }
  } else {
    size_t work = (size_t)(d.S > d.N ? d.S : d.N);
    size_t g = (work + kBlock - 1) / kBlock;
    if (g > 8192) g = 8192;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(k_prepare, dim3((unsigned)g), dim3(kBlock), 0, st, d, ec);
    e = read_err();
  }
  if (e != hipSuccess) { delete h; return ADSEQ_E_HIP; }
  if (err & ERR_GRAPH) { delete h; return ADSEQ_E_GRAPH; }
  if (err & ERR_DELAY) { delete h; return ADSEQ_E_DELAY_RANGE; }
  *out = h;
  return ADSEQ_OK;
}

int adseq_destroy(adseq_t* h) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  for (hipEvent_t e : h->evs) (void)hipEventDestroy(e);
  delete h;
  return ADSEQ_OK;
}

int adseq_reset(adseq_t* h, void* stream) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  launch_reset(h, (hipStream_t)stream);
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

int adseq_deliver(adseq_t* h, int64_t step, float* I_out, void* stream) {
  if (!h || !I_out) return h ? fail(h, ADSEQ_E_INVALID_ARG, "adseq_deliver: null argument") : ADSEQ_E_INVALID_ARG;
  if (step != h->next_step)
    return fail(h, ADSEQ_E_ORDER, "adseq_deliver: got step %lld, expected %lld", (long long)step, h->next_step);
  const int parity = (int)(h->enq_calls & 1);
  if (h->dev.kind == ADSEQ_RING) {
    ring_open_window(h, (hipStream_t)stream, step);
    hipLaunchKernelGGL(k_deliver_win, dim3((unsigned)h->dev.nblk), dim3(kBlock), 0, (hipStream_t)stream,
                       h->dev, (long long)step, I_out);
  } else {
    launch_neurons<1>(h, (hipStream_t)stream, step, parity, nullptr, nullptr, I_out);
  }
  h->next_step = step + 1;
  h->tape_ok = false;
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

int adseq_enqueue(adseq_t* h, int64_t step, const int32_t* spike_ids, const int32_t* n_spikes,
                  void* stream) {
  if (!h || !spike_ids || !n_spikes)
    return h ? fail(h, ADSEQ_E_INVALID_ARG, "adseq_enqueue: null argument") : ADSEQ_E_INVALID_ARG;
  if (step != h->next_step - 1)
    return fail(h, ADSEQ_E_ORDER, "adseq_enqueue: got step %lld, expected %lld (the step last delivered)",
                (long long)step, h->next_step - 1);
  const int parity = (int)(h->enq_calls & 1);
  if (h->dev.kind == ADSEQ_RING)
    hipLaunchKernelGGL(k_enqueue_win, dim3(kFanoutBlocks), dim3(kBlock), 0, (hipStream_t)stream, h->dev,
                       (long long)step, spike_ids, n_spikes);
  else
    launch_fanout(h, (hipStream_t)stream, step, spike_ids, n_spikes, 0);
  h->enq_calls += 1;
  h->tape_ok = false;
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

int adseq_step(adseq_t* h, int64_t step, const float* i_ext, uint8_t* spikes_out, void* stream) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  return step_impl(h, step, i_ext, spikes_out, (hipStream_t)stream);
}

int adseq_run(adseq_t* h, int64_t step0, int64_t n_steps, void* stream) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  if (n_steps < 0) return fail(h, ADSEQ_E_INVALID_ARG, "adseq_run: negative step count");
  if (step0 != h->next_step)
    return fail(h, ADSEQ_E_ORDER, "adseq_run: got step %lld, expected %lld", (long long)step0, h->next_step);
  for (int64_t n = 0; n < n_steps; ++n) {
    const int rc = step_impl(h, step0 + n, nullptr, nullptr, (hipStream_t)stream);
    if (rc != ADSEQ_OK) return rc;
  }
  close_group(h, (hipStream_t)stream, 1);
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

int adseq_backward(adseq_t* h, const float* dL_dcount, const float* dL_dU, float* grad_w,
                   float* grad_d, void* stream) {
  if (!h || !grad_w || !grad_d)
    return h ? fail(h, ADSEQ_E_INVALID_ARG, "adseq_backward: null gradient buffer") : ADSEQ_E_INVALID_ARG;
  const Dev& d = h->dev;
  if (!d.record || !h->tape_ok)
    return fail(h, ADSEQ_E_NO_TAPE, "adseq_backward: no complete recorded forward run");
  hipStream_t st = (hipStream_t)stream;
  flush_admit(h, st);
  close_group(h, st, 1);
  unsigned err = 0;
  HIP_TRY(h, hipMemcpyAsync(&err, &d.ctr->err, sizeof(err), hipMemcpyDeviceToHost, st));
  HIP_TRY(h, hipStreamSynchronize(st));
  if (err & (ERR_TAPE_SPIKES | ERR_TAPE_EVENTS | ERR_POOL))
    return fail(h, ADSEQ_E_CAPACITY, "adseq_backward: tape or contender pool overflowed (bits %u)", err);
  const long long T = h->next_step;
  // gradient per unit the delay was given in: 1/tau per ms, dt/tau per step
  const float dscale = d.continuous ? (float)(1.0 / (double)d.tau) : (float)((double)d.dt / (double)d.tau);
  const dim3 block(kBlock), gn(grid_for((size_t)d.BN)), gg(kFanoutBlocks);
  const bool bounded = d.kind != ADSEQ_RING, atomic = d.B > 1;
  if (!bounded) {
    ring_backward_launch(h, st, T, dscale, dL_dcount, dL_dU, grad_w, grad_d);
    HIP_TRY(h, hipGetLastError());
    return ADSEQ_OK;
  }
  fill_u32(st, d.bwd_carry, 0u, (size_t)d.BN);
  fill_u32(st, grad_w, 0u, (size_t)d.S);
  fill_u32(st, grad_d, 0u, (size_t)d.S);
  fill_u32(st, d.bwd_ring, 0u, (size_t)d.R * d.BN);
  mark(h, st, -1);
  for (long long n = T - 1; n >= 0; --n) {
    if (atomic) hipLaunchKernelGGL((k_bwd_gather<true>), gg, block, 0, st, d, n, T, dscale, grad_w, grad_d);
    else hipLaunchKernelGGL((k_bwd_gather<false>), gg, block, 0, st, d, n, T, dscale, grad_w, grad_d);
    mark(h, st, 2);
    hipLaunchKernelGGL(k_bwd_neurons, gn, block, 0, st, d, n, dL_dcount, dL_dU);
    mark(h, st, 3);
  }
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

int adseq_counters(adseq_t* h, int64_t* out8, void* stream) {
  if (!h || !out8) return ADSEQ_E_INVALID_ARG;
  Counters c;
  hipStream_t st = (hipStream_t)stream;
  const Dev& d = h->dev;
  flush_admit(h, st);
  if (d.kind == ADSEQ_RING) {
    // The ring keeps no per-event counters.  Spikes and the events they emit are counted from
    // the spike words: up to the last window boundary by the boundary pass (device counters),
    // since then here; and delivered = offered - still in flight, the latter counted here from
    // the spike words of the last d_max + 1 steps.
    fill_u32(st, d.ctr->in_flight, 0u, 4 + 6);
    const long long items = (long long)d.R * d.words;
    hipLaunchKernelGGL(k_ring_in_flight, dim3((unsigned)items), dim3(kBlock), 0, st, d, h->next_step,
                       d.ctr->in_flight);
    if (h->fold_upto < h->next_step) {
      const long long it = (h->next_step - h->fold_upto) * d.words;
      hipLaunchKernelGGL(k_count_spikes, dim3((unsigned)grid_for((size_t)it)), dim3(kBlock), 0, st, d,
                         h->fold_upto, h->next_step, d.ctr->fold);
    }
  }
  HIP_TRY(h, hipMemcpyAsync(&c, d.ctr, sizeof(c), hipMemcpyDeviceToHost, st));
  HIP_TRY(h, hipStreamSynchronize(st));
  out8[0] = (int64_t)c.offered; out8[1] = (int64_t)c.dropped; out8[2] = (int64_t)c.delivered;
  out8[3] = c.sum_offered; out8[4] = c.sum_dropped; out8[5] = c.sum_delivered;
  out8[6] = c.tape_spikes; out8[7] = (int64_t)c.err;
  if (d.kind != ADSEQ_RING) {
    // the kernels keep private counters per block: add them up here
    const size_t nb = (size_t)d.nblk + kFanoutBlocks;
    std::vector<BlkCtr> hb(nb);
    HIP_TRY(h, hipMemcpyAsync(hb.data(), d.blk, sizeof(BlkCtr) * nb, hipMemcpyDeviceToHost, st));
    HIP_TRY(h, hipStreamSynchronize(st));
    for (const BlkCtr& b : hb) {
      out8[0] += (int64_t)b.offered; out8[1] += (int64_t)b.dropped; out8[2] += (int64_t)b.delivered;
      out8[3] += b.sum_offered; out8[4] += b.sum_dropped; out8[5] += b.sum_delivered;
    }
  }
  if (d.kind == ADSEQ_RING) {
    out8[6] += (int64_t)c.fold[0]; out8[0] += (int64_t)c.fold[1]; out8[3] += (int64_t)c.fold[2];
    out8[2] = out8[0] - (int64_t)c.in_flight[0];
    out8[5] = out8[3] - (int64_t)c.in_flight[1];
  }
  return ADSEQ_OK;
}

int adseq_drop_count(adseq_t* h, uint64_t* dropped, uint64_t* enqueued, uint64_t* delivered,
                     void* stream) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  int64_t c[8];
  const int rc = adseq_counters(h, c, stream);
  if (rc != ADSEQ_OK) return rc;
  if (dropped) *dropped = (uint64_t)c[1];
  if (enqueued) *enqueued = (uint64_t)c[0];
  if (delivered) *delivered = (uint64_t)c[2];
  if (c[7] & (ERR_TAPE_SPIKES | ERR_TAPE_EVENTS | ERR_POOL))
    return fail(h, ADSEQ_E_CAPACITY, "tape or contender pool overflowed (bits %lld)", (long long)c[7]);
  return ADSEQ_OK;
}

int adseq_tape(adseq_t* h, adseq_tape_view* out) {
  if (!h || !out) return ADSEQ_E_INVALID_ARG;
  const Dev& d = h->dev;
  if (!d.record) return ADSEQ_E_NO_TAPE;
  flush_admit(h, h->last_stream);   // the last step's admission flags
  out->membrane = d.tapeU;
  // the ring keeps no spike list: its spikes are exactly U >= v_thresh on the tape
  out->step_offset = d.kind != ADSEQ_RING ? (const int64_t*)d.step_off : nullptr;
  out->spike_id = d.kind != ADSEQ_RING ? d.tape_spk : nullptr;
  out->event_base = d.kind != ADSEQ_RING ? (const int64_t*)d.tape_evb : nullptr;
  out->admitted = d.kind != ADSEQ_RING ? d.tape_adm : nullptr;
  out->steps_recorded = h->tape_ok ? (h->next_step < d.max_steps ? h->next_step : d.max_steps) : 0;
  return ADSEQ_OK;
}

int adseq_spike_counts(adseq_t* h, int32_t* counts, void* stream) {
  if (!h || !counts) return h ? fail(h, ADSEQ_E_INVALID_ARG, "adseq_spike_counts: null argument") : ADSEQ_E_INVALID_ARG;
  const Dev& d = h->dev;
  if (!d.record || !h->tape_ok)
    return fail(h, ADSEQ_E_NO_TAPE, "adseq_spike_counts: no complete recorded forward run");
  hipStream_t st = (hipStream_t)stream;
  // the step kernels keep the counts (one owner thread per neuron and step)
  hipLaunchKernelGGL(k_copy_i32, dim3((unsigned)grid_for((size_t)d.BN)), dim3(kBlock), 0, st, d.spk_count, counts,
                     (size_t)d.BN);
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

int adseq_profile(adseq_t* h, int enable) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  h->prof = enable != 0;
  h->ev_used = 0;
  h->grp_open = false;
  return ADSEQ_OK;
}

int adseq_profile_read(adseq_t* h, double* ms4, int64_t* launches4, void* stream) {
  if (!h || !ms4 || !launches4) return ADSEQ_E_INVALID_ARG;
  close_group(h, (hipStream_t)stream, 1);
  HIP_TRY(h, hipStreamSynchronize((hipStream_t)stream));
  for (int k = 0; k < 4; ++k) { ms4[k] = 0.0; launches4[k] = 0; }
  for (size_t i = 1; i < h->ev_used; ++i) {
    const int k = h->ev_kind[i];
    if (k < 0 || k > 3) continue;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, h->evs[i - 1], h->evs[i]) != hipSuccess) continue;
    ms4[k] += (double)ms; launches4[k] += h->ev_count[i];
  }
  h->ev_used = 0;
  return ADSEQ_OK;
}

const char* adseq_last_error(const adseq_t* h) { return h ? h->err : "null handle"; }

}  // extern "C"
