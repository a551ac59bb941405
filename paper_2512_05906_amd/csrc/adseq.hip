// MI355X (gfx950) kernels and C ABI for delayed spike-event delivery through
// autodifferentiable queues.  See include/adseq.h for the contract of every
// entry point; this file holds the device code and the host-side bookkeeping.
//
// Layout of the state in the caller's workspace (all arrays 256-byte aligned):
//   V            fp32  [BN]                 membrane state
//   ring         i32   [R][BN]              RING: Q8.24 sums per arrival slot, R = d_max + 1
//   spike_bits   u64   [R][4 nblk]          RING: spike bit masks of the last R steps (one word per
//                                           wavefront), from which in-flight events are counted on demand
//   slot_k/a     u32/i32 [C][BN]            FIFO/SORTED: arrival step and Q8.24 amplitude, slot-major
//                                           so that one slot of 64 consecutive targets is one line
//   occ, head    i32   [BN]                 FIFO/SORTED: stored events; SORTED: index of the front
//   c_head, pool_*                          per-step contender lists (one linked list per target)
//   packed, a_q  u32/i32 [S]                synapses: (col << dbits | D) and Q8.24 amplitude
//   amp, fdec    fp32  [S]                  continuous delays only: a = w f and f
//   tape_*                                  membrane tape, spike list, admission flags
//   bwd_*                                   adjoint delay line [R][BN], carry, queue term
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "adseq.h"

namespace {

constexpr int kBlock = 256;
constexpr int kFanoutBlocks = 1024;
constexpr int kAdmitBlocks = 1024;

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
};

// Private counters of one block of the fused step kernel (no atomics; summed on demand).
struct BlkCtr {
  unsigned long long offered, delivered, spikes;
  long long sum_offered, sum_delivered;
  long long pad[3];
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
  long long* d1_ptr;   // RING: [N+1] per-row ranges into d1_off
  unsigned* d1_off;    // RING: positions (within the row) of the entries with arrival offset 1
  float* amp;
  float* fdec;
  float* V;
  int* ring;
  unsigned long long* spike_bits;  // RING: [R][words] spikes of the last R steps
  unsigned* slot_k;
  int* slot_a;
  int* occ;
  int* head;
  int* c_head;
  long long* pool_p;
  long long* pool_t;
  int* pool_g;
  int* pool_next;
  unsigned* pool_k;
  int* pool_a;
  int* cur_spk;
  float* tapeU;
  long long* step_off;
  int* tape_spk;
  long long* tape_evb;
  unsigned char* tape_adm;
  float* bwd_ring;
  float* bwd_carry;
  float* bwd_G;
  Counters* ctr;
  BlkCtr* blk;   // [nblk]
  int nblk;      // blocks of the fused step kernel = ceil(BN / 256)
  int words;     // 64-neuron words per step in spike_bits = 4 * nblk
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

// Per-row lists of the entries with arrival offset 1 (RING).  One wavefront per row.
// pass 0: d1_ptr[i + 1] = count; (then k_scan_rows turns counts into offsets;) pass 1: fill d1_off.
__global__ __launch_bounds__(kBlock) void k_d1_lists(Dev d, int pass) {
  const int lane = threadIdx.x & 63;
  const long long wave = ((long long)blockIdx.x * kBlock + threadIdx.x) >> 6;
  const long long nwaves = ((long long)gridDim.x * kBlock) >> 6;
  for (long long i = wave; i < d.N; i += nwaves) {
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    long long base = pass ? d.d1_ptr[i] : 0;
    int total = 0;
    for (long long q0 = r0; q0 < r1; q0 += 64) {
      const long long p = q0 + lane;
      const bool hit = p < r1 && (d.packed[p] & d.dmask) == 1u;
      const unsigned long long mk = __ballot(hit);
      if (pass && hit) d.d1_off[base + total + __popcll(mk & ((1ull << lane) - 1ull))] = (unsigned)(p - r0);
      total += __popcll(mk);
    }
    if (!pass && lane == 0) d.d1_ptr[i + 1] = total;
  }
  if (!pass && blockIdx.x == 0 && threadIdx.x == 0) d.d1_ptr[0] = 0;
}

// In-place inclusive scan of ptr[1..n] (single block; create-time only).
__global__ __launch_bounds__(1024) void k_scan_rows(long long* ptr, long long n) {
  __shared__ long long s_w[16];
  __shared__ long long s_carry;
  if (threadIdx.x == 0) s_carry = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  for (long long base = 1; base <= n; base += 1024) {
    const long long idx = base + threadIdx.x;
    long long v = idx <= n ? ptr[idx] : 0;
    for (int o = 1; o < 64; o <<= 1) { const long long t = __shfl_up(v, o, 64); if (lane >= o) v += t; }
    if (lane == 63) s_w[w] = v;
    __syncthreads();
    long long add = s_carry;
    for (int x = 0; x < w; ++x) add += s_w[x];
    if (idx <= n) ptr[idx] = v + add;
    __syncthreads();
    if (threadIdx.x == 1023) s_carry = v + add;
    __syncthreads();
  }
}

// ---------------------------------------------------------------- pop + drive + LIF + compaction

// One thread per (trial, neuron).  KIND selects how the due events are popped.
// LIF = true: closed-loop step (drive, membrane update, spike compaction, tape);
// LIF = false: open-loop delivery, writes the popped current to I_out.
template <int KIND, bool LIF>
__global__ __launch_bounds__(kBlock) void k_neurons(Dev d, long long n, int parity,
                                                    const float* __restrict__ i_ext,
                                                    unsigned char* __restrict__ spikes_out,
                                                    float* __restrict__ I_out) {
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  int acc = 0;
  long long popped = 0;
  const unsigned kn = (unsigned)n;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    d.ctr->n_spk[parity ^ 1] = 0;  // next step's spike counter; nobody reads it now
  }
  if (act) {
    if (KIND == ADSEQ_RING) {
      const size_t idx = (size_t)(n % d.R) * d.BN + g;
      acc = d.ring[idx];
      if (acc != 0) d.ring[idx] = 0;
    } else if (KIND == ADSEQ_FIFO) {
      // bounded bag: every stored event due now leaves; survivors are packed to the front
      const int occ = d.occ[g];
      int keep = 0;
      for (int s = 0; s < occ; ++s) {
        const size_t si = (size_t)s * d.BN + g;
        const unsigned k = d.slot_k[si];
        if (k == kn) {
          acc = wrap_add(acc, d.slot_a[si]);
          ++popped;
        } else {
          if (keep != s) {
            const size_t di = (size_t)keep * d.BN + g;
            d.slot_k[di] = k;
            d.slot_a[di] = d.slot_a[si];
          }
          ++keep;
        }
      }
      if (keep != occ) d.occ[g] = keep;
    } else {
      // ordered by arrival: everything due now sits at the front of the circular array
      int occ = d.occ[g];
      if (occ > 0) {
        int hd = d.head[g];
        while (occ > 0 && d.slot_k[(size_t)hd * d.BN + g] == kn) {
          acc = wrap_add(acc, d.slot_a[(size_t)hd * d.BN + g]);
          hd = hd + 1 == d.C ? 0 : hd + 1;
          --occ;
          ++popped;
        }
        if (popped) { d.occ[g] = occ; d.head[g] = hd; }
      }
    }
  }
  if (KIND == ADSEQ_RING && (threadIdx.x & 63) == 0) {
    // open-loop use: this step's spike bits start empty; adseq_enqueue sets them
    d.spike_bits[(size_t)(n % d.R) * d.words + (size_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)] = 0ull;
  }
  bool s = false;
  if (act) {
    float I = (float)acc * 0x1p-24f;
    if (LIF) {
      if (d.p_thresh) {
        const bool xi = (unsigned long long)drive_bits(d.seed, (unsigned long long)g,
                                                       (unsigned long long)n) < d.p_thresh;
        I = I + (xi ? d.ext_w : 0.0f);
      }
      if (i_ext) I = I + i_ext[g];
      const float U = __fmaf_rn(d.alpha, d.V[g], I);
      s = U >= d.theta;
      d.V[g] = s ? d.v_reset : U;
      if (d.record && n < d.max_steps) d.tapeU[(size_t)n * d.BN + g] = U;
      if (spikes_out) spikes_out[g] = s ? 1 : 0;
    } else {
      I_out[g] = I;
    }
  }
  if (LIF) {
    // wavefront ballot + prefix popcount; one atomic per wavefront that has spikes
    const unsigned long long m = __ballot(s);
    const int lane = threadIdx.x & 63;
    int base = 0;
    if (lane == 0 && m) base = atomicAdd(&d.ctr->n_spk[parity], __popcll(m));
    base = __shfl(base, 0, 64);
    if (s) d.cur_spk[base + __popcll(m & ((1ull << lane) - 1ull))] = g;
  }
  block_add2(&d.ctr->delivered, popped, &d.ctr->sum_delivered, (long long)acc);
}

// ---------------------------------------------------------------- fan-out + enqueue

// One block per spike (grid-stride over the spike list); the block walks the CSR row with
// coalesced reads of (packed, a_q).  RING: integer atomic add into the arrival slot.
// FIFO/SORTED: events whose target is already full are dropped here; the others become
// contenders, pushed on their target's linked list for k_admit.
template <int KIND>
__global__ __launch_bounds__(kBlock) void k_fanout(Dev d, long long n, const int* __restrict__ spk,
                                                   const int* __restrict__ n_spk_ptr, int parity,
                                                   int record) {
  __shared__ long long s_evb;
  int nspk = *n_spk_ptr;
  nspk = nspk < 0 ? 0 : (nspk > d.BN ? d.BN : nspk);
  if (KIND != ADSEQ_RING && blockIdx.x == 0 && threadIdx.x == 0) d.ctr->pool_n[parity ^ 1] = 0;
  const long long off = record ? d.step_off[n] : 0;
  const int m = (int)(n % d.R);
  const int lane = threadIdx.x & 63;
  long long c_off = 0, s_off = 0, c_drop = 0, s_drop = 0;
  for (int e = blockIdx.x; e < nspk; e += gridDim.x) {
    const int g = spk[e];
    if ((unsigned)g >= (unsigned)d.BN) continue;  // uniform over the block
    const int b = g / d.N, i = g - b * d.N;
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    long long tbase = -1;
    if (KIND == ADSEQ_RING && threadIdx.x == 0)
      atomicOr(&d.spike_bits[(size_t)m * d.words + (g >> 6)], 1ull << (g & 63));
    if (record) {
      const bool fits = off + e < d.spike_cap;
      if (threadIdx.x == 0) {
        if (fits) d.tape_spk[off + e] = g; else atomicOr(&d.ctr->err, ERR_TAPE_SPIKES);
      }
      if (KIND != ADSEQ_RING) {
        if (threadIdx.x == 0) {
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
    }
    for (long long p0 = r0; p0 < r1; p0 += kBlock) {
      const long long p = p0 + threadIdx.x;
      const bool valid = p < r1;
      unsigned pk = 0; int a = 0;
      if (valid) { pk = d.packed[p]; a = d.a_q[p]; c_off += 1; s_off += a; }
      const int D = (int)(pk & d.dmask);
      const int col = (int)(pk >> d.dbits);
      if (KIND == ADSEQ_RING) {
        if (valid) {
          int slot = m + D; if (slot >= d.R) slot -= d.R;
          atomicAdd(&d.ring[(size_t)slot * d.BN + (size_t)b * d.N + col], a);
        }
      } else {
        const int gt = b * d.N + col;
        const long long tidx = (valid && tbase >= 0) ? tbase + (p - r0) : -1;
        bool contend = false;
        if (valid) {
          contend = d.occ[gt] < d.C;
          if (!contend) { c_drop += 1; s_drop += a; if (tidx >= 0) d.tape_adm[tidx] = 0; }
        }
        // wavefront-aggregated claim of pool entries
        const unsigned long long cm = __ballot(contend);
        if (cm) {
          int base = 0;
          if (lane == __ffsll((long long)cm) - 1) base = atomicAdd(&d.ctr->pool_n[parity], __popcll(cm));
          base = __shfl(base, __ffsll((long long)cm) - 1, 64);
          if (contend) {
            const int x = base + __popcll(cm & ((1ull << lane) - 1ull));
            if (x >= d.pool_cap) {
              atomicOr(&d.ctr->err, ERR_POOL);
              c_drop += 1; s_drop += a; if (tidx >= 0) d.tape_adm[tidx] = 0;
            } else {
              d.pool_p[x] = p; d.pool_t[x] = tidx; d.pool_g[x] = gt;
              d.pool_k[x] = (unsigned)(n + D); d.pool_a[x] = a;
              d.pool_next[x] = atomicExch(&d.c_head[gt], x);
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
  block_add2(&d.ctr->offered, c_off, &d.ctr->sum_offered, s_off);
  if (KIND != ADSEQ_RING) block_add2(&d.ctr->dropped, c_drop, &d.ctr->sum_dropped, s_drop);
}

// Admission for the bounded kinds.  One thread per contender; the thread whose entry is the head
// of its target's list serves the whole list: the min(K, free) contenders with the smallest
// synapse index are stored (canonical order), the rest are dropped.
template <int KIND>
__global__ __launch_bounds__(kBlock) void k_admit(Dev d, int parity) {
  int np = d.ctr->pool_n[parity];
  np = np > d.pool_cap ? d.pool_cap : np;
  long long c_drop = 0, s_drop = 0;
  for (int x0 = blockIdx.x * kBlock; x0 < np; x0 += gridDim.x * kBlock) {
    const int x = x0 + threadIdx.x;
    if (x >= np) continue;
    const int gt = d.pool_g[x];
    if (d.c_head[gt] != x) continue;
    const int occ = d.occ[gt];
    const int F = d.C - occ;
    int K = 0;
    for (int y = x; y >= 0; y = d.pool_next[y]) ++K;
    const int take = K < F ? K : F;
    int hd = KIND == ADSEQ_SORTED ? d.head[gt] : 0;
    long long last = -1;
    for (int r = 0; r < take; ++r) {
      int best = -1; long long bp = 0x7fffffffffffffffLL;
      for (int y = x; y >= 0; y = d.pool_next[y]) {
        const long long pp = d.pool_p[y];
        if (pp > last && pp < bp) { bp = pp; best = y; }
      }
      last = bp;
      const unsigned k = d.pool_k[best];
      const int a = d.pool_a[best];
      if (KIND == ADSEQ_FIFO) {
        const size_t si = (size_t)(occ + r) * d.BN + gt;
        d.slot_k[si] = k; d.slot_a[si] = a;
      } else {
        // insertion from the back of the circular ordered array (stable for equal arrival steps)
        int pos = occ + r;
        while (pos > 0) {
          int ph = hd + pos - 1; if (ph >= d.C) ph -= d.C;
          const size_t si = (size_t)ph * d.BN + gt;
          const unsigned kk = d.slot_k[si];
          if (kk <= k) break;
          int pd = ph + 1; if (pd >= d.C) pd -= d.C;
          const size_t di = (size_t)pd * d.BN + gt;
          d.slot_k[di] = kk; d.slot_a[di] = d.slot_a[si];
          --pos;
        }
        int pw = hd + pos; if (pw >= d.C) pw -= d.C;
        const size_t wi = (size_t)pw * d.BN + gt;
        d.slot_k[wi] = k; d.slot_a[wi] = a;
      }
      const long long t = d.pool_t[best];
      if (t >= 0) d.tape_adm[t] = 1;
    }
    if (take < K) {
      for (int y = x; y >= 0; y = d.pool_next[y]) {
        if (d.pool_p[y] > last) {
          c_drop += 1; s_drop += d.pool_a[y];
          const long long t = d.pool_t[y];
          if (t >= 0) d.tape_adm[t] = 0;
        }
      }
    }
    d.occ[gt] = occ + take;
    d.c_head[gt] = -1;
  }
  block_add2(&d.ctr->dropped, c_drop, &d.ctr->sum_dropped, s_drop);
}

// Ascending in-block list of the flagged threads: ballot + popcount prefix per wavefront,
// wavefront totals through LDS.  Returns the number of entries and this thread's position.
__device__ __forceinline__ int block_compact(bool flag, int* s_list, int* s_wcnt, int* pos_out) {
  const unsigned long long m = __ballot(flag);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) s_wcnt[w] = __popcll(m);
  __syncthreads();
  int base = 0, total = 0;
  for (int x = 0; x < kBlock / 64; ++x) { const int c = s_wcnt[x]; if (x < w) base += c; total += c; }
  const int pos = base + __popcll(m & ((1ull << lane) - 1ull));
  if (flag) s_list[pos] = threadIdx.x;
  *pos_out = pos;
  return total;
}

// ---------------------------------------------------------------- closed-loop step (RING)
//
// One launch per time step, without an atomic on any shared counter, made of two kinds of blocks:
//   ring_lif   block b owns neurons [256 b, 256 b + 256): pops their ring slots, integrates,
//              records the membrane value, publishes the spike bits of its four wavefronts;
//   ring_fan   kSplit blocks per neuron block: block (b, c) re-derives b's spikes from the spike
//              bits and scatters chunk c (256 entries out of every kSplit * 256) of each spike's CSR
//              row, so that one neuron block's spikes are spread over kSplit compute units and the
//              row reads of all its spikes are in flight together.
// The ring is d_max + 1 deep, hence the row popped at step n is never a target of the events
// emitted at step n (arrival offsets are 1..d_max).

#ifndef ADSEQ_KSPLIT
#define ADSEQ_KSPLIT 4
#endif
constexpr int kSplit = ADSEQ_KSPLIT;  // fan-out blocks per neuron block
constexpr int kBatch = 8;  // spikes whose row entries a thread keeps in flight together

// Neuron part of a ring step for neuron block `nb`: pop, drive, LIF, tape, spike words; plus the
// scatter of the block's own events with arrival offset 1 (taken from the per-row lists built at
// create), which are the only ones the next step's pop depends on.
template <bool RECORD>
__device__ __forceinline__ void ring_lif(const Dev& d, long long n, int nb,
                                         const float* __restrict__ i_ext,
                                         unsigned char* __restrict__ spikes_out) {
  __shared__ long long s_red[3][kBlock / 64];
  const int g = nb * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  const int m = (int)(n % d.R);
  int acc = 0;
  bool s = false;
  if (act) {
    const size_t idx = (size_t)m * d.BN + g;
    acc = d.ring[idx];
    if (acc != 0) d.ring[idx] = 0;
    float I = (float)acc * 0x1p-24f;
    if (d.p_thresh) {
      const bool xi = (unsigned long long)drive_bits(d.seed, (unsigned long long)g,
                                                     (unsigned long long)n) < d.p_thresh;
      I = I + (xi ? d.ext_w : 0.0f);
    }
    if (i_ext) I = I + i_ext[g];
    const float U = __fmaf_rn(d.alpha, d.V[g], I);
    s = U >= d.theta;
    d.V[g] = s ? d.v_reset : U;
    if (RECORD) d.tapeU[(size_t)n * d.BN + g] = U;
    if (spikes_out) spikes_out[g] = s ? 1 : 0;
  }
  // spike bits of this step: read by the fan-out blocks of the next launch, and kept for
  // d_max + 1 steps so that the events still in flight can be counted on demand
  const unsigned long long bits = __ballot(s);
  if ((threadIdx.x & 63) == 0)
    d.spike_bits[(size_t)m * d.words + (size_t)nb * (kBlock / 64) + (threadIdx.x >> 6)] = bits;
  long long c1 = 0, s1 = 0;
  if (s) {
    const int b = g / d.N, i = g - b * d.N;
    const long long q0 = d.d1_ptr[i], q1 = d.d1_ptr[i + 1];
    if (q1 > q0) {
      const long long r0 = d.row_ptr[i];
      int slot = m + 1; if (slot >= d.R) slot -= d.R;
      int* __restrict__ dst = d.ring + (size_t)slot * d.BN + (size_t)b * d.N;
      for (long long q = q0; q < q1; ++q) {
        const long long p = r0 + d.d1_off[q];
        const int a = d.a_q[p];
        atomicAdd(&dst[d.packed[p] >> d.dbits], a);
        c1 += 1; s1 += a;
      }
    }
  }
  const long long sp = wave_sum((long long)acc);
  const long long ns = wave_sum((long long)(s ? 1 : 0));
  c1 = wave_sum(c1); s1 = wave_sum(s1);
  __shared__ long long s_c1[kBlock / 64];
  if ((threadIdx.x & 63) == 0) {
    const int w = threadIdx.x >> 6;
    s_red[0][w] = sp; s_red[1][w] = ns; s_red[2][w] = s1; s_c1[w] = c1;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long a = 0, c = 0, so = 0, co = 0;
    for (int w = 0; w < kBlock / 64; ++w) { a += s_red[0][w]; c += s_red[1][w]; so += s_red[2][w]; co += s_c1[w]; }
    // private counters of this block; atomics only so that nothing waits for a read
    BlkCtr& bc = d.blk[nb];
    if (a) atomicAdd((unsigned long long*)&bc.sum_delivered, (unsigned long long)a);
    if (c) atomicAdd(&bc.spikes, (unsigned long long)c);
    if (co) { atomicAdd(&bc.offered, (unsigned long long)co); atomicAdd((unsigned long long*)&bc.sum_offered, (unsigned long long)so); }
  }
}

// Spikes of neuron block `nb` at ring slot m, from the spike bits: fills s_r0 / s_len / s_base in
// ascending neuron order and returns their number (0: nothing to do; uniform over the block).
__device__ __forceinline__ int block_spikes_from_bits(const Dev& d, int m, int nb, long long* s_r0,
                                                      int* s_len, int* s_base) {
  const unsigned long long* w = d.spike_bits + (size_t)m * d.words + (size_t)nb * (kBlock / 64);
  const unsigned long long w0 = w[0], w1 = w[1], w2 = w[2], w3 = w[3];
  if ((w0 | w1 | w2 | w3) == 0ull) return 0;
  const int wi = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const unsigned long long mine = wi == 0 ? w0 : (wi == 1 ? w1 : (wi == 2 ? w2 : w3));
  if ((mine >> lane) & 1ull) {
    int pos = __popcll(mine & ((1ull << lane) - 1ull));
    if (wi > 0) pos += __popcll(w0);
    if (wi > 1) pos += __popcll(w1);
    if (wi > 2) pos += __popcll(w2);
    const int g = nb * kBlock + threadIdx.x;
    const int b = g / d.N, i = g - b * d.N;
    const long long r0 = d.row_ptr[i];
    s_r0[pos] = r0; s_len[pos] = (int)(d.row_ptr[i + 1] - r0); s_base[pos] = b * d.N;
  }
  __syncthreads();
  return __popcll(w0) + __popcll(w1) + __popcll(w2) + __popcll(w3);
}

// Fan-out part of a ring step: fan block `fb` = (neuron block fb / kSplit, chunk fb % kSplit)
// scatters its chunk of the rows of that neuron block's spikes at step n, except the entries with
// arrival offset 1 (already scattered by ring_lif in the launch that detected the spikes).
__device__ __forceinline__ void ring_fan(const Dev& d, long long n, int fb) {
  __shared__ long long s_r0[kBlock];
  __shared__ int s_len[kBlock];
  __shared__ int s_base[kBlock];
  __shared__ long long s_red[2][kBlock / 64];
  const int nb = fb / kSplit, c = fb % kSplit;
  const int m = (int)(n % d.R);
  const int nspk = block_spikes_from_bits(d, m, nb, s_r0, s_len, s_base);
  if (nspk == 0) return;
  long long c_off = 0, s_off = 0;
  for (int e0 = 0; e0 < nspk; e0 += kBatch) {
    int maxlen = 0;
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (e0 + j < nspk) { const int l = s_len[e0 + j]; maxlen = l > maxlen ? l : maxlen; }
    for (int q = c * kBlock + threadIdx.x; q < maxlen; q += kSplit * kBlock) {
      unsigned pk[kBatch]; int aq[kBatch]; int bs[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        bs[j] = -1; pk[j] = 0; aq[j] = 0;
        if (e0 + j < nspk && q < s_len[e0 + j]) {
          const long long p = s_r0[e0 + j] + q;
          pk[j] = d.packed[p]; aq[j] = d.a_q[p]; bs[j] = s_base[e0 + j];
        }
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        const int D = (int)(pk[j] & d.dmask);
        if (bs[j] >= 0 && D != 1) {
          int slot = m + D; if (slot >= d.R) slot -= d.R;
          atomicAdd(&d.ring[(size_t)slot * d.BN + (size_t)bs[j] + (pk[j] >> d.dbits)], aq[j]);
          c_off += 1; s_off += aq[j];
        }
      }
    }
  }
  c_off = wave_sum(c_off); s_off = wave_sum(s_off);
  if ((threadIdx.x & 63) == 0) { s_red[0][threadIdx.x >> 6] = c_off; s_red[1][threadIdx.x >> 6] = s_off; }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long a = 0, b = 0;
    for (int w = 0; w < kBlock / 64; ++w) { a += s_red[0][w]; b += s_red[1][w]; }
    BlkCtr& bc = d.blk[d.nblk + fb];
    if (a) { atomicAdd(&bc.offered, (unsigned long long)a); atomicAdd((unsigned long long*)&bc.sum_offered, (unsigned long long)b); }
  }
}

// One launch per time step for the ring.  The first nblk blocks (when n_lif >= 0) integrate step
// n_lif; the other nblk * kSplit blocks (when n_fan >= 0) fan out the spikes of step n_fan =
// n_lif - 1 with arrival offsets >= 2.  The two halves are independent: the pop of step n only
// needs offset-1 events of step n - 1 (scattered by ring_lif itself, one launch earlier) and
// events of older steps (complete), and with a ring d_max + 1 deep no fan-out event of step n - 1
// with offset >= 2 lands in the row being popped.  So the neuron update hides behind the scatter.
template <bool RECORD>
__global__ __launch_bounds__(kBlock) void k_step_ring(Dev d, long long n_lif, long long n_fan,
                                                      const float* __restrict__ i_ext,
                                                      unsigned char* __restrict__ spikes_out) {
  const int lif_blocks = n_lif >= 0 ? d.nblk : 0;
  if ((int)blockIdx.x < lif_blocks) ring_lif<RECORD>(d, n_lif, (int)blockIdx.x, i_ext, spikes_out);
  else ring_fan(d, n_fan, (int)blockIdx.x - lif_blocks);
}

// Events of the ring that are still in flight at step n_end (arrival >= n_end): counted from the
// spike bits of the last d_max + 1 steps.  One block per (slot, 64-neuron word); on demand only.
__global__ __launch_bounds__(kBlock) void k_ring_in_flight(Dev d, long long n_end,
                                                           unsigned long long* out /*[2]*/) {
  const long long item = blockIdx.x;
  const int slot = (int)(item / d.words);
  const long long word = item % d.words;
  // the step this slot last held: the largest n' < n_end with n' % R == slot
  long long np = n_end - 1 - ((n_end - 1 - slot) % d.R + d.R) % d.R;
  if (n_end <= 0 || np < 0) return;
  unsigned long long bits = d.spike_bits[(size_t)slot * d.words + word];
  long long cnt = 0, sum = 0;
  while (bits) {
    const int bit = __ffsll((long long)bits) - 1;
    bits &= bits - 1;
    const long long g = word * 64 + bit;
    if (g >= d.BN) break;
    const int i = (int)(g % d.N);
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    for (long long p = r0 + threadIdx.x; p < r1; p += kBlock) {
      const int D = (int)(d.packed[p] & d.dmask);
      if (np + D >= n_end) { cnt += 1; sum += d.a_q[p]; }
    }
  }
  block_add2(&out[0], cnt, (long long*)&out[1], sum);
}

// Queue term of the reverse sweep for the ring, kSplit blocks per neuron block: gather block
// (b, c) re-derives b's spikes at step n from the membrane tape (s = U >= theta), gathers the
// adjoint at the arrival slot of chunk c of each spike's row (arrival offsets >= 2), accumulates the
// row's weight and delay gradients, and leaves its partial queue term in g_part[n & 1][c][neuron].
template <bool ATOMIC>
__device__ __forceinline__ void ring_bwd_gather(const Dev& d, long long n, long long T, float dscale, int fb,
                                                float* __restrict__ grad_w, float* __restrict__ grad_d) {
  __shared__ int s_spk[kBlock];
  __shared__ int s_wcnt[kBlock / 64];
  __shared__ long long s_r0[kBlock];
  __shared__ int s_len[kBlock];
  __shared__ int s_base[kBlock];
  __shared__ float s_G[kBlock];
  const int nb = fb / kSplit, c = fb % kSplit;
  const int g = nb * kBlock + threadIdx.x;
  const int m = (int)(n % d.R);
  bool s = false;
  if (g < d.BN) s = d.tapeU[(size_t)n * d.BN + g] >= d.theta;
  if (!__syncthreads_or(s ? 1 : 0)) return;
  int pos;
  const int nspk = block_compact(s, s_spk, s_wcnt, &pos);
  if (s) {
    const int b = g / d.N, i = g - b * d.N;
    const long long r0 = d.row_ptr[i];
    s_r0[pos] = r0; s_len[pos] = (int)(d.row_ptr[i + 1] - r0); s_base[pos] = b * d.N; s_G[pos] = 0.0f;
  }
  __syncthreads();
  for (int e0 = 0; e0 < nspk; e0 += kBatch) {
    int maxlen = 0;
#pragma unroll
    for (int j = 0; j < kBatch; ++j)
      if (e0 + j < nspk) { const int l = s_len[e0 + j]; maxlen = l > maxlen ? l : maxlen; }
    float Gacc[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) Gacc[j] = 0.0f;
    for (int q = c * kBlock + threadIdx.x; q < maxlen; q += kSplit * kBlock) {
      unsigned pk[kBatch]; float am[kBatch]; float fd[kBatch]; int bs[kBatch]; long long pp[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        bs[j] = -1; pk[j] = 0; am[j] = 0.0f; fd[j] = 1.0f; pp[j] = 0;
        if (e0 + j < nspk && q < s_len[e0 + j]) {
          const long long p = s_r0[e0 + j] + q;
          pk[j] = d.packed[p];
          if (d.continuous) { am[j] = d.amp[p]; fd[j] = d.fdec[p]; } else { am[j] = d.weight[p]; }
          bs[j] = s_base[e0 + j]; pp[j] = p;
        }
      }
      float gv[kBatch];
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        gv[j] = 0.0f;
        const int D = (int)(pk[j] & d.dmask);
        if (bs[j] >= 0 && D != 1 && n + D < T) {  // offset 1: ring_bwd_neurons; n + D >= T: never delivered
          int slot = m + D; if (slot >= d.R) slot -= d.R;
          gv[j] = d.bwd_ring[(size_t)slot * d.BN + (size_t)bs[j] + (pk[j] >> d.dbits)];
        } else {
          bs[j] = -1;
        }
      }
#pragma unroll
      for (int j = 0; j < kBatch; ++j) {
        if (bs[j] >= 0) {
          Gacc[j] += am[j] * gv[j];
          const float gw = fd[j] * gv[j], gd = am[j] * dscale * gv[j];
          if (ATOMIC) { unsafeAtomicAdd(&grad_w[pp[j]], gw); unsafeAtomicAdd(&grad_d[pp[j]], gd); }
          else { grad_w[pp[j]] += gw; grad_d[pp[j]] += gd; }
        }
      }
    }
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      if (e0 + j < nspk) {  // uniform over the block
        const float t = wave_sum_f(Gacc[j]);
        if ((threadIdx.x & 63) == 0 && t != 0.0f) atomicAdd(&s_G[e0 + j], t);
      }
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < nspk)
    d.bwd_G[((size_t)(n & 1) * kSplit + c) * d.BN + (size_t)nb * kBlock + s_spk[threadIdx.x]] = s_G[threadIdx.x];
}

// Neuron part of the reverse sweep for the ring at step n: adds the offset-1 events of its own
// spikes (they need gU[n + 1], written one launch earlier) to the kSplit partial queue terms, then
//   gU[n] = (1 - s) alpha gU[n+1] + sigma'(U - theta) (dL/dcount + s G) + dL/dU[n]
template <bool ATOMIC>
__device__ __forceinline__ void ring_bwd_neurons(const Dev& d, long long n, long long T, float dscale, int nb,
                                                 const float* __restrict__ dL_dcount,
                                                 const float* __restrict__ dL_dU,
                                                 float* __restrict__ grad_w, float* __restrict__ grad_d) {
  const int g = nb * kBlock + threadIdx.x;
  if (g >= d.BN) return;
  const int m = (int)(n % d.R);
  const float U = d.tapeU[(size_t)n * d.BN + g];
  const bool s = U >= d.theta;
  float sg = 0.0f;
  if (d.surrogate == ADSEQ_SURR_SUPERSPIKE) {
    const float x = fabsf(U - d.theta) + 1.0f;
    sg = 1.0f / (x * x);
  }
  float inner = dL_dcount ? dL_dcount[g] : 0.0f;
  if (s) {
    float G = 0.0f;
    for (int c = 0; c < kSplit; ++c) G += d.bwd_G[((size_t)(n & 1) * kSplit + c) * d.BN + g];
    if (n + 1 < T) {
      const int b = g / d.N, i = g - b * d.N;
      const long long q0 = d.d1_ptr[i], q1 = d.d1_ptr[i + 1];
      if (q1 > q0) {
        const long long r0 = d.row_ptr[i];
        int slot = m + 1; if (slot >= d.R) slot -= d.R;
        const float* __restrict__ src = d.bwd_ring + (size_t)slot * d.BN + (size_t)b * d.N;
        for (long long q = q0; q < q1; ++q) {
          const long long p = r0 + d.d1_off[q];
          const float gv = src[d.packed[p] >> d.dbits];
          const float a = d.continuous ? d.amp[p] : d.weight[p];
          const float f = d.continuous ? d.fdec[p] : 1.0f;
          G += a * gv;
          const float gw = f * gv, gd = a * dscale * gv;
          if (ATOMIC) { unsafeAtomicAdd(&grad_w[p], gw); unsafeAtomicAdd(&grad_d[p], gd); }
          else { grad_w[p] += gw; grad_d[p] += gd; }
        }
      }
    }
    inner += G;
  }
  float gu = sg * inner;
  if (!s) gu = __fmaf_rn(d.alpha, d.bwd_carry[g], gu);
  if (dL_dU) gu += dL_dU[(size_t)n * d.BN + g];
  d.bwd_carry[g] = gu;
  d.bwd_ring[(size_t)m * d.BN + g] = gu;
}

// One launch per reverse step for the ring: the first nblk blocks (when n_neu >= 0) update the
// adjoint of step n_neu; the other nblk * kSplit blocks (when n_gat >= 0) gather the queue terms
// of step n_gat = n_neu - 1 (offsets >= 2, which only read adjoint rows written by earlier launches).
template <bool ATOMIC>
__global__ __launch_bounds__(kBlock) void k_bwd_step_ring(Dev d, long long n_neu, long long n_gat,
                                                          long long T, float dscale,
                                                          const float* __restrict__ dL_dcount,
                                                          const float* __restrict__ dL_dU,
                                                          float* __restrict__ grad_w,
                                                          float* __restrict__ grad_d) {
  const int neu_blocks = n_neu >= 0 ? d.nblk : 0;
  if ((int)blockIdx.x < neu_blocks)
    ring_bwd_neurons<ATOMIC>(d, n_neu, T, dscale, (int)blockIdx.x, dL_dcount, dL_dU, grad_w, grad_d);
  else
    ring_bwd_gather<ATOMIC>(d, n_gat, T, dscale, (int)blockIdx.x - neu_blocks, grad_w, grad_d);
}

// ---------------------------------------------------------------- backward

// Queue term of the reverse sweep at step n: one block per recorded spike (b, i, n).  Gathers the
// adjoint at each admitted event's arrival slot, reduces G_i, and accumulates the weight and
// delay gradients of the row.
template <bool BOUNDED, bool ATOMIC>
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
    const long long evb = BOUNDED ? d.tape_evb[off + e] : 0;
    float G = 0.0f;
    for (long long p = r0 + threadIdx.x; p < r1; p += kBlock) {
      const unsigned pk = d.packed[p];
      const int D = (int)(pk & d.dmask);
      const int col = (int)(pk >> d.dbits);
      if (n + D >= T) continue;                               // not delivered inside the run
      if (BOUNDED && !d.tape_adm[evb + (p - r0)]) continue;   // refused by a full queue
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
  long long pending_fan; // RING: step whose fan-out (offsets >= 2) rides with the next launch, or -1
  char err[256];
  // optional kernel timing (adseq_profile): one event after each bracketed launch
  bool prof = false;
  std::vector<hipEvent_t> evs;
  std::vector<int> ev_kind;   // kernel class the event closes, -1 = start marker
  size_t ev_used = 0;
};

namespace {

struct Layout {
  size_t V, ring, spike_bits, slot_k, slot_a, occ, head, c_head, pool_p, pool_t, pool_g, pool_next,
      pool_k, pool_a, cur_spk, packed, a_q, d1_ptr, d1_off, amp, fdec, tapeU, step_off, tape_spk, tape_evb, tape_adm,
      bwd_ring, bwd_carry, bwd_G, ctr, blk, total;
  long long spike_cap, event_cap, pool_cap;
  int R, dbits, nblk, words;
};

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
  L->words = L->nblk * (kBlock / 64);
  L->ctr = take(sizeof(Counters));
  L->blk = take((size_t)L->nblk * (kSplit + 1) * sizeof(BlkCtr));  // neuron blocks + kSplit fan-out blocks each
  L->V = take(BN * 4);
  L->ring = take(bounded ? 0 : (size_t)L->R * BN * 4);
  L->spike_bits = take(bounded ? 0 : (size_t)L->R * L->words * 8);
  L->slot_k = take(bounded ? (size_t)c->capacity * BN * 4 : 0);
  L->slot_a = take(bounded ? (size_t)c->capacity * BN * 4 : 0);
  L->occ = take(bounded ? BN * 4 : 0);
  L->head = take(bounded ? BN * 4 : 0);
  L->c_head = take(bounded ? BN * 4 : 0);
  L->pool_p = take((size_t)L->pool_cap * 8);
  L->pool_t = take((size_t)L->pool_cap * 8);
  L->pool_g = take((size_t)L->pool_cap * 4);
  L->pool_next = take((size_t)L->pool_cap * 4);
  L->pool_k = take((size_t)L->pool_cap * 4);
  L->pool_a = take((size_t)L->pool_cap * 4);
  L->cur_spk = take(BN * 4);
  L->packed = take(S * 4);
  L->a_q = take(S * 4);
  L->d1_ptr = take(bounded ? 0 : ((size_t)c->n_neurons + 1) * 8);
  L->d1_off = take(bounded ? 0 : S * 4);  // worst case: every entry has offset 1
  L->amp = take(cont ? S * 4 : 0);
  L->fdec = take(cont ? S * 4 : 0);
  const size_t T = c->record_tape ? (size_t)c->max_steps : 0;
  L->tapeU = take(T * BN * 4);
  L->step_off = take(c->record_tape ? (T + 1) * 8 : 0);
  L->tape_spk = take(bounded ? (size_t)L->spike_cap * 4 : 0);
  L->tape_evb = take(bounded ? (size_t)L->spike_cap * 8 : 0);
  L->tape_adm = take((size_t)L->event_cap);
  L->bwd_ring = take(c->record_tape ? (size_t)L->R * BN * 4 : 0);
  L->bwd_carry = take(c->record_tape ? BN * 4 : 0);
  L->bwd_G = take(c->record_tape ? BN * 4 * kSplit * 2 : 0);  // kSplit partial queue terms per neuron, two step parities
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
  const size_t BN = (size_t)d.BN;
  fill_u32(st, d.ctr, 0u, sizeof(Counters) / 4);
  fill_u32(st, d.blk, 0u, (size_t)d.nblk * (kSplit + 1) * sizeof(BlkCtr) / 4);
  fill_u32(st, d.V, 0u, BN);
  if (d.kind == ADSEQ_RING) {
    fill_u32(st, d.ring, 0u, (size_t)d.R * BN);
    fill_u32(st, d.spike_bits, 0u, (size_t)d.R * d.words * 2);
  } else {
    fill_u32(st, d.occ, 0u, BN);
    fill_u32(st, d.head, 0u, BN);
    fill_u32(st, d.c_head, 0xffffffffu, BN);
  }
  if (d.record) fill_u32(st, d.step_off, 0u, 2);  // step_off[0] = 0 (int64)
  h->next_step = 0;
  h->enq_calls = 0;
  h->pending_fan = -1;
  h->tape_ok = d.record != 0;
}

template <bool LIF>
void launch_neurons(adseq* h, hipStream_t st, long long n, int parity, const float* i_ext,
                    unsigned char* spikes_out, float* I_out) {
  const Dev& d = h->dev;
  const dim3 grid(grid_for((size_t)d.BN)), block(kBlock);
  switch (d.kind) {
    case ADSEQ_RING:
      hipLaunchKernelGGL((k_neurons<ADSEQ_RING, LIF>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
      break;
    case ADSEQ_FIFO:
      hipLaunchKernelGGL((k_neurons<ADSEQ_FIFO, LIF>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
      break;
    default:
      hipLaunchKernelGGL((k_neurons<ADSEQ_SORTED, LIF>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
      break;
  }
}

void launch_fanout(adseq* h, hipStream_t st, long long n, const int* spk, const int* n_spk,
                   int parity, int record) {
  const Dev& d = h->dev;
  const dim3 grid(kFanoutBlocks), block(kBlock);
  switch (d.kind) {
    case ADSEQ_RING:
      hipLaunchKernelGGL((k_fanout<ADSEQ_RING>), grid, block, 0, st, d, n, spk, n_spk, parity, record);
      break;
    case ADSEQ_FIFO:
      hipLaunchKernelGGL((k_fanout<ADSEQ_FIFO>), grid, block, 0, st, d, n, spk, n_spk, parity, record);
      hipLaunchKernelGGL((k_admit<ADSEQ_FIFO>), dim3(kAdmitBlocks), block, 0, st, d, parity);
      break;
    default:
      hipLaunchKernelGGL((k_fanout<ADSEQ_SORTED>), grid, block, 0, st, d, n, spk, n_spk, parity, record);
      hipLaunchKernelGGL((k_admit<ADSEQ_SORTED>), dim3(kAdmitBlocks), block, 0, st, d, parity);
      break;
  }
}

void mark(adseq* h, hipStream_t st, int kind);

// RING: one launch = neuron update of step n_lif (if >= 0) + fan-out of step n_fan (if >= 0).
void launch_ring_step(adseq* h, hipStream_t st, long long n_lif, long long n_fan, int record,
                      const float* i_ext, unsigned char* spikes_out) {
  const Dev& d = h->dev;
  const unsigned grid = (unsigned)((n_lif >= 0 ? d.nblk : 0) + (n_fan >= 0 ? d.nblk * kSplit : 0));
  if (!grid) return;
  mark(h, st, -1);
  if (record) hipLaunchKernelGGL((k_step_ring<true>), dim3(grid), dim3(kBlock), 0, st, d, n_lif, n_fan, i_ext, spikes_out);
  else hipLaunchKernelGGL((k_step_ring<false>), dim3(grid), dim3(kBlock), 0, st, d, n_lif, n_fan, i_ext, spikes_out);
  mark(h, st, 0);
}

// RING: launches the fan-out that is still riding, so that the queue state is complete.
void flush_ring(adseq* h, hipStream_t st) {
  if (h->dev.kind == ADSEQ_RING && h->pending_fan >= 0) {
    launch_ring_step(h, st, -1, h->pending_fan, 0, nullptr, nullptr);
    h->pending_fan = -1;
  }
}

// Records an event that closes a launch of class `kind` (and opens the next one).
void mark(adseq* h, hipStream_t st, int kind) {
  if (!h->prof) return;
  if (h->ev_used == h->evs.size()) {
    hipEvent_t e;
    if (hipEventCreate(&e) != hipSuccess) return;
    h->evs.push_back(e); h->ev_kind.push_back(kind);
  }
  h->ev_kind[h->ev_used] = kind;
  (void)hipEventRecord(h->evs[h->ev_used], st);
  h->ev_used += 1;
}

int step_impl(adseq* h, long long step, const float* i_ext, unsigned char* spikes_out, hipStream_t st) {
  if (step != h->next_step)
    return fail(h, ADSEQ_E_ORDER, "adseq_step: got step %lld, expected %lld", step, h->next_step);
  const Dev& d = h->dev;
  const int parity = (int)(h->enq_calls & 1);
  const int record = (d.record && h->tape_ok && step < d.max_steps) ? 1 : 0;
  if (d.record && step >= d.max_steps) h->tape_ok = false;
  if (d.kind == ADSEQ_RING) {
    launch_ring_step(h, st, step, h->pending_fan, record, i_ext, spikes_out);
    h->pending_fan = step;
  } else {
    mark(h, st, -1);
    launch_neurons<true>(h, st, step, parity, i_ext, spikes_out, nullptr);
    mark(h, st, 1);
    launch_fanout(h, st, step, d.cur_spk, &d.ctr->n_spk[parity], parity, record);
    mark(h, st, 0);
  }
  h->enq_calls += 1;
  h->next_step = step + 1;
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
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
  d.blk = (BlkCtr*)(ws + L.blk); d.nblk = L.nblk; d.words = L.words;
  d.V = (float*)(ws + L.V); d.ring = (int*)(ws + L.ring); d.spike_bits = (unsigned long long*)(ws + L.spike_bits);
  d.slot_k = (unsigned*)(ws + L.slot_k); d.slot_a = (int*)(ws + L.slot_a);
  d.occ = (int*)(ws + L.occ); d.head = (int*)(ws + L.head); d.c_head = (int*)(ws + L.c_head);
  d.pool_p = (long long*)(ws + L.pool_p); d.pool_t = (long long*)(ws + L.pool_t);
  d.pool_g = (int*)(ws + L.pool_g); d.pool_next = (int*)(ws + L.pool_next);
  d.pool_k = (unsigned*)(ws + L.pool_k); d.pool_a = (int*)(ws + L.pool_a);
  d.cur_spk = (int*)(ws + L.cur_spk);
  d.packed = (unsigned*)(ws + L.packed); d.a_q = (int*)(ws + L.a_q);
  d.d1_ptr = (long long*)(ws + L.d1_ptr); d.d1_off = (unsigned*)(ws + L.d1_off);
  d.amp = d.continuous ? (float*)(ws + L.amp) : nullptr;
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
  {
    size_t work = (size_t)(d.S > d.N ? d.S : d.N);
    size_t g = (work + kBlock - 1) / kBlock;
    if (g > 8192) g = 8192;
    if (g < 1) g = 1;
    hipLaunchKernelGGL(k_prepare, dim3((unsigned)g), dim3(kBlock), 0, st, d, ec);
    if (d.kind == ADSEQ_RING) {
      size_t gw = ((size_t)d.N * 64 + kBlock - 1) / kBlock;
      if (gw > 16384) gw = 16384;
      hipLaunchKernelGGL(k_d1_lists, dim3((unsigned)gw), dim3(kBlock), 0, st, d, 0);
      hipLaunchKernelGGL(k_scan_rows, dim3(1), dim3(1024), 0, st, d.d1_ptr, (long long)d.N);
      hipLaunchKernelGGL(k_d1_lists, dim3((unsigned)gw), dim3(kBlock), 0, st, d, 1);
    }
  }
  unsigned err = 0;
  hipError_t e = hipGetLastError();
  if (e == hipSuccess) e = hipMemcpyAsync(&err, &d.ctr->err, sizeof(err), hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
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
  flush_ring(h, (hipStream_t)stream);
  launch_neurons<false>(h, (hipStream_t)stream, step, parity, nullptr, nullptr, I_out);
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
  flush_ring(h, (hipStream_t)stream);
  launch_fanout(h, (hipStream_t)stream, step, spike_ids, n_spikes, parity, 0);
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
  for (int64_t n = 0; n < n_steps; ++n) {
    const int rc = step_impl(h, step0 + n, nullptr, nullptr, (hipStream_t)stream);
    if (rc != ADSEQ_OK) return rc;
  }
  flush_ring(h, (hipStream_t)stream);
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
  flush_ring(h, st);
  unsigned err = 0;
  HIP_TRY(h, hipMemcpyAsync(&err, &d.ctr->err, sizeof(err), hipMemcpyDeviceToHost, st));
  HIP_TRY(h, hipStreamSynchronize(st));
  if (err & (ERR_TAPE_SPIKES | ERR_TAPE_EVENTS | ERR_POOL))
    return fail(h, ADSEQ_E_CAPACITY, "adseq_backward: tape or contender pool overflowed (bits %u)", err);
  const long long T = h->next_step;
  fill_u32(st, grad_w, 0u, (size_t)d.S);
  fill_u32(st, grad_d, 0u, (size_t)d.S);
  fill_u32(st, d.bwd_ring, 0u, (size_t)d.R * d.BN);
  fill_u32(st, d.bwd_carry, 0u, (size_t)d.BN);
  // gradient per unit the delay was given in: 1/tau per ms, dt/tau per step
  const float dscale = d.continuous ? (float)(1.0 / (double)d.tau) : (float)((double)d.dt / (double)d.tau);
  const dim3 block(kBlock), gn(grid_for((size_t)d.BN)), gg(kFanoutBlocks);
  const bool bounded = d.kind != ADSEQ_RING, atomic = d.B > 1;
  if (!bounded) {
    // launch k: neuron update of step n (if any) + gather of step n - 1 (if any); T + 1 launches
    for (long long n = T; n >= 0; --n) {
      const long long n_neu = n < T ? n : -1, n_gat = n - 1;
      const unsigned grid = (unsigned)((n_neu >= 0 ? d.nblk : 0) + (n_gat >= 0 ? d.nblk * kSplit : 0));
      if (!grid) continue;
      mark(h, st, -1);
      if (atomic) hipLaunchKernelGGL((k_bwd_step_ring<true>), dim3(grid), block, 0, st, d, n_neu, n_gat, T, dscale, dL_dcount, dL_dU, grad_w, grad_d);
      else hipLaunchKernelGGL((k_bwd_step_ring<false>), dim3(grid), block, 0, st, d, n_neu, n_gat, T, dscale, dL_dcount, dL_dU, grad_w, grad_d);
      mark(h, st, 2);
    }
    HIP_TRY(h, hipGetLastError());
    return ADSEQ_OK;
  }
  mark(h, st, -1);
  for (long long n = T - 1; n >= 0; --n) {
    if (bounded) {
      if (atomic) hipLaunchKernelGGL((k_bwd_gather<true, true>), gg, block, 0, st, d, n, T, dscale, grad_w, grad_d);
      else hipLaunchKernelGGL((k_bwd_gather<true, false>), gg, block, 0, st, d, n, T, dscale, grad_w, grad_d);
    } else {
      if (atomic) hipLaunchKernelGGL((k_bwd_gather<false, true>), gg, block, 0, st, d, n, T, dscale, grad_w, grad_d);
      else hipLaunchKernelGGL((k_bwd_gather<false, false>), gg, block, 0, st, d, n, T, dscale, grad_w, grad_d);
    }
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
  flush_ring(h, st);
  if (d.kind == ADSEQ_RING) {
    // the ring sums amplitudes, so delivered = offered - still in flight; the latter is counted
    // here, on demand, from the spike bits of the last d_max + 1 steps
    fill_u32(st, d.ctr->in_flight, 0u, 4);
    const long long items = (long long)d.R * d.words;
    hipLaunchKernelGGL(k_ring_in_flight, dim3((unsigned)items), dim3(kBlock), 0, st, d, h->next_step,
                       d.ctr->in_flight);
  }
  HIP_TRY(h, hipMemcpyAsync(&c, d.ctr, sizeof(c), hipMemcpyDeviceToHost, st));
  HIP_TRY(h, hipStreamSynchronize(st));
  out8[0] = (int64_t)c.offered; out8[1] = (int64_t)c.dropped; out8[2] = (int64_t)c.delivered;
  out8[3] = c.sum_offered; out8[4] = c.sum_dropped; out8[5] = c.sum_delivered;
  out8[6] = c.tape_spikes; out8[7] = (int64_t)c.err;
  if (d.kind == ADSEQ_RING) {
    // the fused step kernel keeps private counters per block: add them up here
    const int nb = d.nblk * (kSplit + 1);
    BlkCtr* hb = new (std::nothrow) BlkCtr[nb];
    if (!hb) return fail(h, ADSEQ_E_INVALID_ARG, "adseq_counters: out of host memory");
    hipError_t e = hipMemcpyAsync(hb, d.blk, sizeof(BlkCtr) * nb, hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) { delete[] hb; return fail(h, ADSEQ_E_HIP, "copy of block counters failed: %s", hipGetErrorString(e)); }
    for (int i = 0; i < nb; ++i) {
      out8[0] += (int64_t)hb[i].offered; out8[3] += hb[i].sum_offered;
      out8[5] += hb[i].sum_delivered; out8[6] += (int64_t)hb[i].spikes;
    }
    delete[] hb;
    out8[2] = out8[0] - (int64_t)c.in_flight[0];
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

int adseq_tape(const adseq_t* h, adseq_tape_view* out) {
  if (!h || !out) return ADSEQ_E_INVALID_ARG;
  const Dev& d = h->dev;
  if (!d.record) return ADSEQ_E_NO_TAPE;
  out->membrane = d.tapeU;
  // the ring's fused step keeps no spike list: its spikes are exactly U >= v_thresh on the tape
  out->step_offset = d.kind != ADSEQ_RING ? (const int64_t*)d.step_off : nullptr;
  out->spike_id = d.kind != ADSEQ_RING ? d.tape_spk : nullptr;
  out->event_base = d.kind != ADSEQ_RING ? (const int64_t*)d.tape_evb : nullptr;
  out->admitted = d.kind != ADSEQ_RING ? d.tape_adm : nullptr;
  out->steps_recorded = h->tape_ok ? (h->next_step < d.max_steps ? h->next_step : d.max_steps) : 0;
  return ADSEQ_OK;
}

int adseq_profile(adseq_t* h, int enable) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  h->prof = enable != 0;
  h->ev_used = 0;
  return ADSEQ_OK;
}

int adseq_profile_read(adseq_t* h, double* ms4, int64_t* launches4, void* stream) {
  if (!h || !ms4 || !launches4) return ADSEQ_E_INVALID_ARG;
  HIP_TRY(h, hipStreamSynchronize((hipStream_t)stream));
  for (int k = 0; k < 4; ++k) { ms4[k] = 0.0; launches4[k] = 0; }
  for (size_t i = 1; i < h->ev_used; ++i) {
    const int k = h->ev_kind[i];
    if (k < 0 || k > 3) continue;
    float ms = 0.0f;
    if (hipEventElapsedTime(&ms, h->evs[i - 1], h->evs[i]) != hipSuccess) continue;
    ms4[k] += (double)ms; launches4[k] += 1;
  }
  h->ev_used = 0;
  return ADSEQ_OK;
}

const char* adseq_last_error(const adseq_t* h) { return h ? h->err : "null handle"; }

}  // extern "C"
