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
//   fkey, famp, vmask                       FIFO: per target, 16-bit arrival keys, Q8.24 amplitudes, occupied-slot bits
//   slot, head, min_k                       SORTED: per target, circular ordered array {arrival step, amplitude},
//                                           index of its front, earliest stored arrival step
//   occ          i32   [BN]                 FIFO/SORTED: stored events
//   cnt, cont, c_head, pool_*               contenders of the current step per target (slots, then a list)
//   spk_words, stepcnt                      FIFO/SORTED: ballot words and per-block spike / event counts of the current step
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
constexpr int kArriveLines = 16;   // arrival counters of a grid barrier, a 128-byte line each (ring_resident_reverse.h)
constexpr int kFanoutBlocks = 1024;

enum : unsigned {
  ERR_DELAY = 1u, ERR_GRAPH = 2u, ERR_TAPE_SPIKES = 4u, ERR_TAPE_EVENTS = 8u, ERR_POOL = 16u,
  ERR_BARRIER = 32u,  // a bounded wait of a resident kernel ran out
  ERR_RANGE = 64u     // some target's incoming amplitudes add up to 128 or more in magnitude: a Q8.24 sum could wrap
};

struct Counters {
  unsigned long long offered, dropped, delivered;
  long long sum_offered, sum_dropped, sum_delivered;
  long long tape_spikes, tape_events;
  unsigned err;
  int pool_n[2];
  unsigned long long in_flight[2];  // scratch of k_ring_in_flight: events, Q8.24 sum
  unsigned long long fold[3];       // scratch of k_count_spikes: spikes, events, Q8.24 sum
  alignas(128) unsigned bar[32];    // bar[0]: arrivals at the barriers of the resident step kernels (a line of its own)
  alignas(128) unsigned arrive[8][32];  // arrive[x][0]: blocks with index x mod 8 of the chained step launches that have arrived (ring_chain.h)
  alignas(128) unsigned rev_arrivals[kArriveLines][32];  // rev_arrivals[x][0]: arrivals of the blocks with rank x mod kArriveLines at the grid barriers of the resident reverse kernel and of the forward kernel over the whole chip
#ifdef ADSEQ_PHASE_CLOCK
  unsigned long long phase[24];     // builds with phase clocks: 10 ns ticks block 0 spent in each phase; [0, 8) resident steps or
                                    // staging pass of the window expansion, [8, 11) accumulation pass, [15] expansions counted, [16, 19) far gather of the reverse sweep (walk, pieces, waiting for the block's other wavefronts), [19] gathers counted
  unsigned long long span[3][512][2]; // the same builds: wall clock at begin and end of every block of the last staging [0], accumulation [1] and far gather [2] launch
#endif
};

// Private event counters of one block of k_neurons / k_fanout (FIFO / SORTED) or of one virtual
// block of the ring's staging pass (pad[0] = spikes): one 64-byte line each, so that no two blocks
// add to the same address; summed on demand.
struct BlkCtr {
  unsigned long long offered, admitted, delivered;
  long long sum_offered, sum_admitted, sum_delivered;
  long long pad[2];
};

struct ExpCoef { double c[21]; };
struct RowSpan { long long r0, r1; };

struct Dev {
  int N, B, BN, R, C, kind, dbits, d_max;
  unsigned dmask;
  unsigned n_magic;     // floor(2^32 / N) (2^32 - 1 for N = 1): see trial_of
  int continuous, record, surrogate, max_steps, pool_cap;
  float alpha, theta, v_reset, ext_w, dt;
  float tau;            // time constant of the state that takes the jump: tau_syn if there is a synaptic state, else tau_m
  float alpha_s;        // exp(-dt / tau_syn), 0 = no synaptic current state
  float alpha_r;        // exp(-dt / tau_rise), 0 = no second (fast) state: double-exponential synapse if > 0
  float alpha_diff;     // alpha_s - alpha_r
  float inv_tau_b, inv_tau_diff;   // 1 / tau_rise, 1 / tau_rise - 1 / tau_syn
  // what the ring's step kernels read, side by side: a launch fetches a few lines of its argument
  // block instead of a dozen
  int W, wshift;        // window length in steps (power of two) and its log2
  int nblk;      // neuron blocks of a step launch: ceil(BN / 256)
  int words;     // 64-neuron words per step in spike_bits (RING) = 4 * nblk
  int* win;             // [W][BN]
  float* V;
  const long long* row_ptr;
  unsigned* nearcnt;    // [W + 1][N]
  float* tapeU;
  int* spk_count;       // [BN] spikes per (trial, neuron) over the recorded steps
  unsigned long long* spike_bits;  // RING: [R][words] spikes of the last R steps
  unsigned long long* tape_bits;  // [T][words]
  uint2* synf;          // [S] sorted rows: {col << dbits | D, Q8.24 amplitude}
  float* J;             // [BN] synaptic current state (alpha_s > 0); [2][BN] with the fast state behind it (alpha_r > 0)
  unsigned long long p_thresh, seed;
  float* gwin;          // [W][BN]
  float* bwd_carry;
  float* bwd_carryJ;    // [BN] its adjoint dL/dJ[n+1] ([2][BN] if alpha_r > 0: the slow state's adjoint, the sum of both states')
  float* Gacc;          // [R][BN]
  uint2* synb;          // [S] sorted rows: {col << dbits | D, fp32 amplitude bits}
  float* gsum;          // [S]
  // the rest
  long long S, spike_cap, event_cap;
  const int* col;
  const float* weight;
  const unsigned char* delay_steps;
  const float* delay_ms;
  unsigned* packed;
  int* a_q;
  // RING (windowed delay line, see ring_window.h)
  int tp_shift;         // log2 of the targets per part (W << tp_shift = cells of one LDS tile)
  int P, NB, cap;       // target parts, blocks of the staging pass, events per (part, block) region
  int wgroups;          // 8-word lines (64 bytes) per step in spike_bits
  unsigned* dstart;     // [N][d_max + 2]
  unsigned* perm;       // [S]
  long long* rowsum;    // [N] Q8.24 amplitude sum of every row (all kinds)
  int* rowlen;          // FIFO/SORTED: [N] row lengths
  uint2* ebuf;          // [min(P, kMaxParts)][NB][cap]
  int* ecnt;            // [min(P, kMaxParts)][NB]
  float* amp;
  float* fdec;
  uint2* slot;          // SORTED: [BN][C] {arrival step, Q8.24 amplitude}, circular, ordered by arrival
  unsigned short* fkey; // FIFO: [BN][cpad] arrival step mod 2^16 of every slot
  int* famp;            // FIFO: [BN][C] Q8.24 amplitude of every slot
  unsigned* vmask;      // FIFO: [BN][nw] bit j of word w set = slot 32 w + j holds an event
  int prefetch;         // FIFO/SORTED: 1 = few targets (B N <= 2^18): the step kernel loads keys and row lengths up front
  int fsplit;           // FIFO/SORTED: blocks per neuron block of the closed-loop fan-out (1 .. kFanSplitMax)
  int nw, cpad;         // FIFO: mask words per target = ceil(C / 32); C rounded up to a multiple of 8
  int* occ;
  int* head;
  unsigned* min_k;      // FIFO/SORTED: earliest stored arrival step per target (0xffffffff: none)
  int* cnt;             // contenders registered per target since its last admission
  uint4* cont;          // [kCont][BN] contender records (see bounded_queues.h)
  int* c_head;          // overflow list head per target (-1: empty)
  long long* pool_p;
  long long* pool_t;
  int* pool_next;
  unsigned* pool_k;
  int* pool_a;
  unsigned short* sq_next; // SYN_FIFO: [ceil(B S / 8) * 8] arrival step of the head of every per-synapse queue (0xffff: empty)
  unsigned short* sq_hs;   // SYN_FIFO: [B S] head << 8 | size
  unsigned short* sq_key;  // SYN_FIFO: [B S][C] arrival step mod 2^16 of every slot
  long long* sq_flag;      // SYN_BINS with tape: [C][ceil(B S / 8) * 8] index on the tape of the admission flag of the event every bin holds
  long long* last_evb;     // SYN_LATEST with tape: [2][BN] index of the first admission flag of the neuron's last spike and of the one before, in turn
  int* I_acc;              // SYN_FIFO / SYN_LATEST: [BN] Q8.24 sum of the events popped for the step being run
  int blk_pop;             // SYN_FIFO: index of the first counter line of k_synq_pop's blocks in blk
  unsigned long long* spk_words;  // FIFO/SORTED: [2][words] ballot words of the step launch, by step parity
  long long* stepcnt;   // FIFO/SORTED: [2][nblk][2] spikes and emitted events of every neuron block, by step parity
  long long* step_off;
  long long* step_evoff;  // FIFO/SORTED: events emitted before step n (index of its first admission flag)
  int* tape_spk;
  long long* tape_evb;
  RowSpan* tape_row;    // FIFO/SORTED: row bounds of every recorded spike
  unsigned char* tape_adm;
  float* bwd_ring;
  float* bwd_G;         // FIFO/SORTED: [fsplit][BN] partial queue terms of the spikes of the step being swept
  Counters* ctr;
  BlkCtr* blk;   // FIFO / SORTED: [nblk + kFanoutBlocks]
  // (what was added later stays behind what the per-step kernels read, whose place in the argument block is tuned)
  long long* insum;     // [N] create only: sum of |Q8.24 amplitude| over every target's incoming synapses
  int flow_hold;        // RING, reverse kernel without a grid barrier: 1 = spiking neurons never store their final adjoints (ADSEQ_RING_FLOW_WITHHOLD: drives the waits' failure path from the host)
  int res_spins;        // RING, resident kernels: polls of one wait before it gives up (kResMaxSpins; ADSEQ_RING_RESIDENT_SPINS lowers it to test the failure path)
  int lazy_rows;        // RING: the step kernels fetch row start, in-window count and far queue term for spiking lanes only (experiment)
  int count_pop;        // RING: the step kernels add up the Q8.24 sums they pop (checking aid, off by default)
  int chain_sleep;      // RING, chained step launches: pauses of 128 cycles between two polls of a wait
  int rev_delay;        // RING, resident reverse kernel: pauses of 1,024 cycles before the first poll of a barrier
  int res_wide;         // RING, resident forward kernel: arrivals on eight counters instead of one (experiment)
#if defined(ADSEQ_PHASE_CLOCK) || defined(ADSEQ_ABLATE)
  int dbg;              // debugging builds: parts of the resident step to leave out (timing only)
#endif
  unsigned long long* drive_words;  // RING, resident kernels: drive bits of a stretch of steps, 16 per (step, block, thread)
  // RING, reverse sweep by windows (ring_reverse.h)
  unsigned long long* wspk;   // [BN] spikes of the window being swept, one bit per step
  int* near_nspk;       // [64] numbered spikes per step of the window
  int* near_nev;        // [64] staged near events per step of the window
  uint4* near_ev;       // [W][near_ev_cap] staged near events
  int* near_spk;        // [W][kNearSpikeCap] neuron of every numbered spike
  int* near_counts;     // [2][max_steps] spikes and near events of every recorded step
  int near_ev_cap;
};

// Trial b = g / N of the state index g = b * N + i (0 <= g < 2^31) without an integer division:
// with M = floor(2^32 / N), floor(g M / 2^32) is g / N or one less (g M / 2^32 > g / N - g / 2^32
// > g / N - 1/2), so one correction step makes it exact.
__device__ __forceinline__ int trial_of(const Dev& d, int g) {
  if (d.B == 1) return 0;
  unsigned q = __umulhi((unsigned)g, d.n_magic);
  if ((unsigned)g - q * (unsigned)d.N >= (unsigned)d.N) ++q;
  return (int)q;
}

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

// Makes a kernel fetch fields of its argument block where this is called: an empty asm statement
// that takes the values in scalar registers.  Without it the compiler fetches each field in the
// block that first uses it, and a step kernel starts with a chain of four to six dependent scalar
// loads (each a trip to memory: the argument block of a fresh dispatch is in no cache) before its
// first vector load.  pin_args(a, b, ...) at the top turns the chain into one batch.  (Measured per
// kernel: it pays in the short step kernels, not in the ones with many arguments and early exits.)
template <class T> __device__ __forceinline__ void pin_arg(T v) { asm volatile("" ::"s"(v)); }
template <class... Ts> __device__ __forceinline__ void pin_args(Ts... vs) { (pin_arg(vs), ...); }

__device__ __forceinline__ int wrap_add(int a, int b) { return (int)((unsigned)a + (unsigned)b); }

// Inclusive scan (sum) over the 64 lanes of a wavefront with DPP row shifts and row broadcasts;
// lane 63 ends up with the total.  Every lane of the wavefront must be active.
__device__ __forceinline__ int dpp_scan_add(int v) {
  v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
  v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
  v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
  v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
  v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 into rows 1 and 3
  v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 into rows 2 and 3
  return v;
}
// Sum of v over the wavefront, the same value in every lane.  |v| < 2^31 per lane.
__device__ __forceinline__ long long wave_total(int v) {
  const int lo = __builtin_amdgcn_readlane(dpp_scan_add(v & 0xffff), 63);
  const int hi = __builtin_amdgcn_readlane(dpp_scan_add(v >> 16), 63);
  return ((long long)hi << 16) + lo;
}
// The same for 64-bit values, |v| < 2^62 per lane: three slices of 21 bits.
__device__ __forceinline__ long long wave_total64(long long v) {
  const int s0 = __builtin_amdgcn_readlane(dpp_scan_add((int)(v & 0x1fffff)), 63);
  const int s1 = __builtin_amdgcn_readlane(dpp_scan_add((int)((v >> 21) & 0x1fffff)), 63);
  const int s2 = __builtin_amdgcn_readlane(dpp_scan_add((int)(v >> 42)), 63);
  return ((long long)s2 << 42) + ((long long)s1 << 21) + s0;
}

// Sum over the wavefront, the same value in every lane; every lane must be active.  (DPP row
// operations run at register speed; a butterfly of cross-lane shuffles goes through the LDS
// crossbar six times in a row, which shows in the short kernels.)
__device__ __forceinline__ long long wave_sum(long long v) { return wave_total64(v); }
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_add_f(float v) {
  return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, false));
}
__device__ __forceinline__ float wave_sum_f(float v) {
  v = dpp_add_f<0x111, 0xf>(v); v = dpp_add_f<0x112, 0xf>(v);
  v = dpp_add_f<0x114, 0xf>(v); v = dpp_add_f<0x118, 0xf>(v);
  v = dpp_add_f<0x142, 0xa>(v); v = dpp_add_f<0x143, 0xc>(v);
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
// Value of lane src (src the same in every lane) in every lane, through scalar registers.
__device__ __forceinline__ int lane_get(int v, int src) { return __builtin_amdgcn_readlane(v, src); }
__device__ __forceinline__ unsigned lane_get(unsigned v, int src) {
  return (unsigned)__builtin_amdgcn_readlane((int)v, src);
}
__device__ __forceinline__ long long lane_get(long long v, int src) {
  const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, src);
  const int hi = __builtin_amdgcn_readlane((int)(v >> 32), src);
  return ((long long)hi << 32) | lo;
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

#include "bounded_queues.h"
#include "synapse_queues.h"

__global__ __launch_bounds__(kBlock) void k_copy_i32(const int* __restrict__ src, int* __restrict__ dst, size_t n) {
  for (size_t i = (size_t)blockIdx.x * kBlock + threadIdx.x; i < n; i += (size_t)gridDim.x * kBlock) dst[i] = src[i];
}

// Create: worst case of every target's Q8.24 sum.  The delivered amplitudes of one step are summed
// as wrapping 32-bit integers (range +-128); if all synapses onto one target delivered at once the
// magnitude could reach the sum of their |amplitude|.  Where that sum is 2^31 or more, ERR_RANGE is
// set: a warning, reported with the counters (the oracle wraps the same way, so the two still agree).
__global__ __launch_bounds__(kBlock) void k_in_sums(Dev d) {
  for (long long p = (long long)blockIdx.x * kBlock + threadIdx.x; p < d.S; p += (long long)gridDim.x * kBlock) {
    unsigned pk; int a;
    if (d.kind == ADSEQ_RING) { const uint2 e = d.synf[p]; pk = e.x; a = (int)e.y; }
    else { pk = d.packed[p]; a = d.a_q[p]; }
    const long long mag = a < 0 ? -(long long)a : (long long)a;
    if (mag) atomicAdd((unsigned long long*)&d.insum[pk >> d.dbits], (unsigned long long)mag);
  }
}
__global__ __launch_bounds__(kBlock) void k_in_check(Dev d) {
  bool bad = false;
  for (long long j = (long long)blockIdx.x * kBlock + threadIdx.x; j < d.N; j += (long long)gridDim.x * kBlock)
    bad = bad || d.insum[j] > 0x7fffffffLL;
  if (__ballot(bad) && (threadIdx.x & 63) == 0) atomicOr(&d.ctr->err, ERR_RANGE);
}

// ---------------------------------------------------------------- ring queue (windowed delay line)

#include "ring_window.h"
#include "ring_resident.h"
#include "ring_reverse.h"
#include "ring_resident_reverse.h"
#include "ring_flow_reverse.h"
#include "ring_resident_forward.h"
#include "ring_chain.h"

// ---------------------------------------------------------------- backward (FIFO / SORTED)

// Queue term of the reverse sweep at step n for the bounded kinds: fsplit blocks per recorded
// spike (b, i, n), the spikes being tape entries [off, off + gridDim.x / fsplit).  Block (e, c)
// takes share c of the row (entries c * 256 .. + 255 of every fsplit * 256), four entries per
// thread in flight: row entry + admission flag, then the adjoint at the event's arrival slot of
// the adjoint delay line, then the gradient sums (atomics that return nothing: for one trial a
// synapse gets at most one term per launch, so the result is still deterministic) and the
// block's partial queue term.
__global__ __launch_bounds__(kBlock) void k_bwd_rows(Dev d, long long n, long long T, float dscale,
                                                     float* __restrict__ grad_w, float* __restrict__ grad_d,
                                                     long long off) {
  __shared__ float red[kBlock / 64];
  const int e = blockIdx.x / d.fsplit, c = blockIdx.x - e * d.fsplit;
  const int g = d.tape_spk[off + e];
  const long long evb = d.tape_evb[off + e];
  const RowSpan row = d.tape_row[off + e];
  const int b = trial_of(d, g);
  const int m = (int)(n % d.R);
  const long long stride = (long long)d.fsplit * kBlock;
  const bool dexp = d.alpha_r > 0.0f;              // double-exponential synapse: two adjoint delay lines,
  const size_t second = (size_t)d.R * d.BN;        // Y behind X (see bwd_receiver)
  float G = 0.0f;
  for (long long p0 = row.r0 + (long long)c * kBlock + threadIdx.x; p0 < row.r1; p0 += 4 * stride) {
    long long p[4]; bool use[4]; unsigned pk[4]; unsigned char adm[4]; float a[4], f[4], gv[4], gy[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      p[j] = p0 + j * stride;
      use[j] = p[j] < row.r1;
      pk[j] = 0; adm[j] = 0; a[j] = 0.0f; f[j] = 1.0f;
      if (use[j]) {
        pk[j] = d.packed[p[j]];
        adm[j] = d.tape_adm[evb + (p[j] - row.r0)];
        a[j] = d.continuous ? d.amp[p[j]] : d.weight[p[j]];
        if (d.continuous) f[j] = d.fdec[p[j]];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int D = (int)(pk[j] & d.dmask);
      use[j] = use[j] && adm[j] != 0 && n + D < T;   // admitted, and delivered inside the run
      gv[j] = 0.0f; gy[j] = 0.0f;
      if (use[j]) {
        int slot = m + D; if (slot >= d.R) slot -= d.R;
        const size_t cell = (size_t)slot * d.BN + (size_t)b * d.N + (pk[j] >> d.dbits);
        gv[j] = d.bwd_ring[cell];
        if (dexp) gy[j] = d.bwd_ring[second + cell];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (use[j]) {
        if (dexp) {   // X for the weight, Y (with the 1 / tau factors in it) for the delay
          G += a[j] * queue_term_of(d, gv[j], gy[j]);
          unsafeAtomicAdd(&grad_w[p[j]], f[j] * gv[j]);
          unsafeAtomicAdd(&grad_d[p[j]], a[j] * dscale * gy[j]);
        } else {
          G += a[j] * gv[j];
          unsafeAtomicAdd(&grad_w[p[j]], f[j] * gv[j]);
          unsafeAtomicAdd(&grad_d[p[j]], a[j] * dscale * gv[j]);
        }
      }
  }
  G = wave_sum_f(G);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = G;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.0f;
    for (int w = 0; w < kBlock / 64; ++w) t += red[w];
    d.bwd_G[(size_t)c * d.BN + g] = t;
  }
}

// Neuron part of the reverse sweep at step n for the bounded kinds (see bwd_update).
__global__ __launch_bounds__(kBlock) void k_bwd_neurons(Dev d, long long n,
                                                        const float* __restrict__ dL_dcount,
                                                        const float* __restrict__ dL_dU) {
  pin_args(d.tapeU, d.bwd_carry, d.bwd_carryJ, d.bwd_G, d.bwd_ring, d.BN, d.R, d.fsplit, d.surrogate, d.alpha, d.alpha_s,
           d.alpha_r, d.alpha_diff, d.inv_tau_b, d.inv_tau_diff, d.theta, d.v_reset, d.dt, d.tau, n, dL_dcount, dL_dU);
  const int g = blockIdx.x * kBlock + threadIdx.x;
  if (g >= d.BN) return;
  const float U = d.tapeU[(size_t)n * d.BN + g];
  const float Uprev = (d.surrogate == ADSEQ_GRAD_SPIKE_TIME && n > 0) ? d.tapeU[(size_t)(n - 1) * d.BN + g] : 0.0f;
  const bool s = U >= d.theta;
  float gu;
  float G = 0.0f;
  if (s)
    for (int c = 0; c < d.fsplit; ++c) G += d.bwd_G[(size_t)c * d.BN + g];   // the shares of the spike's row
  d.bwd_carry[g] = bwd_update(d, n, U, Uprev, s, d.bwd_carry[g], dL_dcount ? dL_dcount[g] : 0.0f,
                              G, dL_dU ? dL_dU[(size_t)n * d.BN + g] : 0.0f, &gu);
  float y = 0.0f;
  d.bwd_ring[(size_t)(n % d.R) * d.BN + g] = bwd_receiver(d, g, gu, &y);
  if (d.alpha_r > 0.0f) d.bwd_ring[(size_t)d.R * d.BN + (size_t)(n % d.R) * d.BN + g] = y;
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
  long long bits_clear_for;  // RING, open loop: the spike words of this step's slot have been cleared ahead (-1: of none)
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
  long long drive_from = 0, drive_upto = 0;   // RING, resident kernels: steps whose drive words are in place
  unsigned bar_base = 0;      // RING, resident kernels: value of the barrier counter after the launches so far
  unsigned rev_base = 0;      // RING, resident reverse kernel: sum of its arrival counters after the launches so far
  int res_P = 0, res_chunk = 0, res_npt = 0;   // RING: taking-part blocks, neurons per block, per thread (0: one launch per step)
  int rev_P = 0, rev_chunk = 0, rev_npt = 0;   // RING, reverse sweep: the same for the resident reverse kernel (0: one launch per step)
  bool rev_flow = false;                      // RING: the resident reverse kernel without a grid barrier (ring_flow_reverse.h)
  int fwd_P = 0, fwd_chunk = 0;                // RING: the same for the forward kernel over the whole chip (ring_resident_forward.h; 0: not used)
  float fwd_margin = 0.005f;                   // how far below the threshold the early value of a candidate may lie
  // RING, experimental (ADSEQ_RING_OVERLAP = 1): the far part of the next window expanded ahead on a stream of the library's own
  hipStream_t aux = nullptr;
  hipEvent_t ev_boundary = nullptr, ev_ahead = nullptr;
  long long ahead_for = -1;   // window start whose far part (spikes before the previous boundary) is being expanded ahead, or -1
  // RING, chained step launches (ring_chain.h): dealt out over the caller's stream and one of the library's own
  bool chain = false;         // the handle's runs and reverse sweeps use them
  hipStream_t chain_st = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  unsigned chain_arrivals = 0;   // arrivals of all chained launches so far (what the next one waits for)
  unsigned chain_turn = 0;       // chained launches so far: the parity picks the stream
  int chain_tpb = 256;           // threads per block of the chained launches (256 or 1024)
  bool range_warn = false;    // some target's incoming |amplitudes| add up to 128 or more (ERR_RANGE, reported with the counters)
  bool in_static = false;     // the handle is the device's static one (adseq_create_static): never deleted
};

namespace {

struct Layout {
  size_t V, J, bwd_carryJ, win, spike_bits, drive_words, sq_next, sq_hs, sq_key, sq_flag, I_acc, last_evb, slot, fkey, famp, vmask, occ, head, min_k, cnt, cont, c_head, pool_p, pool_t, pool_next,
      pool_k, pool_a, spk_words, stepcnt, packed, a_q, synf, synb, dstart, nearcnt, perm, rowsum, rowlen, ebuf, ecnt, amp, fdec, tapeU,
      tape_bits, spk_count, step_off, step_evoff, tape_spk, tape_evb, tape_row, tape_adm, bwd_ring, bwd_carry, bwd_G, gwin, Gacc, gsum, insum, wspk, near_cnt, near_ev, near_spk, near_counts, ctr, blk,
      total;
  long long spike_cap, event_cap, pool_cap;
  int R, dbits, nblk, words;
  int W, wshift, tp_shift, P, NB, cap, wgroups;  // RING
  int near_ev_cap;
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

// Resident step kernels (ring_resident.h): up to 32 blocks of 512 threads (up to 128 over several
// XCDs by ADSEQ_RING_RESIDENT_BLOCKS), one or two groups of four neurons per thread, B N a
// multiple of 4 (16-byte aligned rows).  Measured on the configs: 2.1 against 4.7 us per step at
// 100 state cells, 3.6 against 4.7 at 16,000, 4.9 against 5.3 at 10,000 with a long history, 4.4
// against 4.1 at 100,000 -- a launch per step uses all 256 compute units for the spikes' row
// loads and atomic adds, the resident kernel 32 -- so by default they run up to 32,768 state
// cells.  ADSEQ_RING_RESIDENT = 0: never, 1: whenever the layout allows (up to 131,072 cells).
struct ResidentPlan { int P = 0, chunk = 0, npt = 0; };   // taking-part blocks (0: a launch per step), cells per block, groups per thread
ResidentPlan resident_plan(long long BN) {
  ResidentPlan r;
  const int resident = env_pow2("ADSEQ_RING_RESIDENT", 2, 0, 2);
  const int res_blocks = env_pow2("ADSEQ_RING_RESIDENT_BLOCKS", kResBlocks, 8, 128);
  long long chunk = (BN + res_blocks - 1) / res_blocks;
  chunk = (chunk + 255) / 256 * 256;
  if (resident && chunk <= 8 * kResThreads && BN % 4 == 0 && (resident == 1 || BN <= 32768)) {
    r.chunk = (int)chunk;
    r.P = (int)((BN + chunk - 1) / chunk);
    r.npt = chunk <= 4 * kResThreads ? 1 : 2;
  }
  return r;
}
// Resident reverse and forward kernels (ring_flow_reverse.h, ring_resident_reverse.h, ring_resident_forward.h): up
// to 256 blocks of 512 worker threads with one, four or -- not the reverse kernel with a grid barrier -- eight
// consecutive neurons each (at most 4,096 neurons per block), B N a multiple of 4; delta synapse only.
// ADSEQ_RING_RESIDENT_REVERSE = 0: never, 1 (default): whenever the layout allows; ADSEQ_RING_REVERSE_BLOCKS:
// taking-part blocks (8 .. 256, default 128).
ResidentPlan reverse_plan(long long BN, bool forward = false) {
  ResidentPlan r;
  // (forward: 0 never, 1 wherever the layout fits, default from 2,048 state cells on: below that one XCD's blocks, whose
  // barrier is shorter, are faster -- 100 cells 2.4 against 2.9 us per step)
  const int fwd = env_pow2("ADSEQ_RING_FORWARD_CHIP", 2, 0, 2);
  const int on = forward ? ((fwd == 1 || (fwd == 2 && BN >= 2048)) ? 1 : 0) : env_pow2("ADSEQ_RING_RESIDENT_REVERSE", 1, 0, 1);
  // (reverse: 256 blocks for the kernel without a grid barrier, 128 for the one with: its barrier costs more with more blocks)
  const int blocks = forward ? env_pow2("ADSEQ_RING_FORWARD_BLOCKS", 256, 8, 256)
                             : env_pow2("ADSEQ_RING_REVERSE_BLOCKS", env_pow2("ADSEQ_RING_REVERSE_FLOW", 1, 0, 1) ? 256 : 128, 8, 256);
  long long chunk = (BN + blocks - 1) / blocks;
  chunk = (chunk + 255) / 256 * 256;
  // (the forward kernel and the reverse kernel without a grid barrier also take eight neurons per thread: a million state cells)
  const int per_thread = (forward || env_pow2("ADSEQ_RING_REVERSE_FLOW", 1, 0, 1)) ? 8 : 4;
  if (on && chunk <= per_thread * kResThreads && BN % 4 == 0) {
    r.chunk = (int)chunk;
    r.P = (int)((BN + chunk - 1) / chunk);
    r.npt = 1;
  }
  return r;
}
// The grid barrier of the resident kernels ends only when every block of the launch (kResLaunch threads each, 256
// blocks at most: one per compute unit of the MI355X) is on the chip at the same time.  True when the device can hold
// 256 blocks of kernel f at once; where it cannot (fewer compute units, or a kernel too large for one), the time steps
// go by one launch each.  ADSEQ_RING_ASSUME_CUS replaces the device's compute-unit count in this check (tests of the
// decision; it changes nothing else).
bool resident_fits(const void* f, int threads = kResLaunch) {
  int dev = 0, cus = 0, per = 0;
  if (hipGetDevice(&dev) != hipSuccess) return false;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) return false;
  if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per, f, threads, 0) != hipSuccess) { (void)hipGetLastError(); return false; }
  if (const char* e = getenv("ADSEQ_RING_ASSUME_CUS")) { const int v = atoi(e); if (v >= 1 && v <= 4096) cus = v; }
  return (long long)cus * per >= 256;
}
template <bool RECORD>
const void* run_xcd_kernel_of(int syn, int npt) {
  if (npt == 1) return syn == 0 ? (const void*)k_run_xcd<RECORD, 0, 1> : (syn == 1 ? (const void*)k_run_xcd<RECORD, 1, 1> : (const void*)k_run_xcd<RECORD, 2, 1>);
  return syn == 0 ? (const void*)k_run_xcd<RECORD, 0, 2> : (syn == 1 ? (const void*)k_run_xcd<RECORD, 1, 2> : (const void*)k_run_xcd<RECORD, 2, 2>);
}
template <bool DU, int NPT>
const void* flow_kernel_of(int surrogate) {
  if (surrogate == ADSEQ_SURR_SUPERSPIKE) return (const void*)k_bwd_flow<DU, ADSEQ_SURR_SUPERSPIKE, NPT>;
  if (surrogate == ADSEQ_GRAD_SPIKE_TIME) return (const void*)k_bwd_flow<DU, ADSEQ_GRAD_SPIKE_TIME, NPT>;
  return (const void*)k_bwd_flow<DU, ADSEQ_SURR_OFF, NPT>;
}
const void* flow_kernel(bool du, int surrogate, int chunk) {
  if (chunk <= kResThreads) return du ? flow_kernel_of<true, 1>(surrogate) : flow_kernel_of<false, 1>(surrogate);
  if (chunk <= 4 * kResThreads) return du ? flow_kernel_of<true, 4>(surrogate) : flow_kernel_of<false, 4>(surrogate);
  return du ? flow_kernel_of<true, 8>(surrogate) : flow_kernel_of<false, 8>(surrogate);
}
const void* run_xcd_kernel(bool record, int syn, int npt) {
  return record ? run_xcd_kernel_of<true>(syn, npt) : run_xcd_kernel_of<false>(syn, npt);
}
// Cells (target, step) of the LDS tile of one target part.
int ring_tile_cells() { return env_pow2("ADSEQ_RING_TILE", 4096, 1024, kMaxTileCells); }

// Private counter slots of the fan-out kernels (closed loop: up to kFanSplitMax blocks per neuron block).
size_t fan_slots(int nblk) {
  const size_t a = (size_t)nblk * kFanSplitMax;
  return a > (size_t)kFanoutBlocks ? a : (size_t)kFanoutBlocks;
}

int bit_width(unsigned v) { int b = 0; while (v) { ++b; v >>= 1; } return b; }

bool host_validate(const adseq_config* c) {
  if (!c) return false;
  if (c->n_neurons < 1 || c->batch < 1 || c->d_max_steps < 1 || c->d_max_steps > 1023) return false;
  if ((long long)c->n_neurons * c->batch > 0x7fffffffLL) return false;
  if (c->kind != ADSEQ_RING && c->kind != ADSEQ_FIFO && c->kind != ADSEQ_SORTED && c->kind != ADSEQ_SYN_FIFO &&
      c->kind != ADSEQ_SYN_LATEST && c->kind != ADSEQ_SYN_BINS) return false;
  if (c->kind != ADSEQ_RING && (c->capacity < 1 || c->capacity > 32767)) return false;
  if ((c->kind == ADSEQ_SYN_FIFO || c->kind == ADSEQ_SYN_BINS) && c->capacity > kSynqCapMax) return false;
  if (c->kind == ADSEQ_SYN_LATEST && c->capacity != 1) return false;
  if (c->surrogate != ADSEQ_SURR_SUPERSPIKE && c->surrogate != ADSEQ_SURR_OFF &&
      c->surrogate != ADSEQ_GRAD_SPIKE_TIME) return false;
  if (!(c->dt_ms > 0.0f) || !(c->tau_m_ms > 0.0f) || c->dt_ms > c->tau_m_ms) return false;
  if (!(c->tau_syn_ms >= 0.0f) || (c->tau_syn_ms > 0.0f && c->dt_ms > c->tau_syn_ms)) return false;
  if (!(c->tau_rise_ms >= 0.0f) || (c->tau_rise_ms > 0.0f && (c->dt_ms > c->tau_rise_ms || !(c->tau_syn_ms > c->tau_rise_ms) || c->delay_ms)))
    return false;
  if (!(c->ext_rate_hz >= 0.0f)) return false;
  if (c->n_synapses < 0 || c->n_synapses >= (1LL << 40)) return false;   // synapse indices are packed into 40 bits
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
  const bool ptq = c->kind == ADSEQ_FIFO || c->kind == ADSEQ_SORTED;   // bounded queues per target
  const bool synq = per_synapse_kind(c->kind);                         // one queue per synapse
  const bool synfifo = c->kind == ADSEQ_SYN_FIFO;
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
      if (L->event_cap >= (1LL << 40) - 1) return false;   // admission-flag indices are packed into 40 bits
    }
  }
  if (ptq) {
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
  L->W = L->wshift = L->tp_shift = L->P = L->NB = L->cap = L->wgroups = 0;
  size_t stage_parts = 0;
  if (!bounded) {
    // the window is no longer than the largest delay (so that a window boundary comes before
    // any spike word is overwritten)
    L->W = ring_window_steps();
    while (L->W > c->d_max_steps) L->W >>= 1;
    L->wshift = bit_width((unsigned)L->W) - 1;
    // LDS tile of the accumulation pass: by default 4,096 cells, fewer (down to 1,024) where the state array would
    // otherwise give fewer than 256 target parts, one workgroup each (cfg2, 10,000 targets: 40 parts of 256 targets
    // left five compute units in six idle; expansion 30.8 -> 22.2 us per window with 157 parts of 64)
    int cells = ring_tile_cells();
    if (!getenv("ADSEQ_RING_TILE"))
      while (cells > 1024 && cells > 2 * L->W && (long long)BN * L->W / cells < 256) cells >>= 1;
    if (cells < L->W) cells = L->W;
    L->tp_shift = bit_width((unsigned)cells) - 1 - L->wshift;
    L->P = (int)((BN + ((size_t)1 << L->tp_shift) - 1) >> L->tp_shift);
    L->wgroups = (L->words + 7) / 8;
    // blocks of the staging pass: one 8-word line per wavefront when the history is full, but no
    // more than one block per compute unit (measured best on cfg3: 256 of 128..512; cfg2, 4,000 lines:
    // 22.2 us per window with 63 blocks, 19.6 with 128 or 256; cfg1, 1,600 lines: 14.6 with 25, 12.0 with 128)
    const long long lines = (long long)c->d_max_steps * L->wgroups;
    long long nb = (lines + kRingWaves - 1) / kRingWaves;
    L->NB = env_pow2("ADSEQ_RING_BINBLOCKS", (int)(nb < 1 ? 1 : (nb > 256 ? 256 : nb)), 1, kMaxBinBlocks);
    stage_parts = (size_t)(L->P < kMaxParts ? L->P : kMaxParts);
    // staging capacity in events: by default what a window holds when every neuron fires at
    // 1/32 per step, between 2^16 and 2^26 events
    double ev = c->step_event_capacity ? (double)c->step_event_capacity
                                       : (double)c->batch * (double)S * (double)L->W / 32.0;
    if (!c->step_event_capacity) ev = ev < 65536.0 ? 65536.0 : (ev > 67108864.0 ? 67108864.0 : ev);
    const double per = ev / ((double)stage_parts * (double)L->NB);
    L->cap = (int)(per > 65536.0 ? 65536.0 : per);
    if (L->cap >= 16) L->cap &= ~15;   // regions begin on 128-byte lines: a run's first 16 events are one line
  }
  L->ctr = take(sizeof(Counters));
  L->blk = take(bounded ? ((size_t)L->nblk + fan_slots(L->nblk) + (synq ? kSynqBlocks : 0)) * sizeof(BlkCtr)
                        : kMaxBinBlocks * sizeof(BlkCtr));
  L->V = take(BN * 4);
  const size_t nstates = c->tau_rise_ms > 0.0f ? 2 : 1;   // double-exponential synapse: every adjoint twice
  L->J = take(c->tau_syn_ms > 0.0f ? nstates * BN * 4 : 0);
  L->win = take(bounded ? 0 : 2 * (size_t)L->W * BN * 4);
  L->spike_bits = take(bounded ? 0 : (size_t)L->R * L->words * 8);
  L->drive_words = take(bounded ? 0 : (size_t)kDriveSteps * resident_plan((long long)BN).P * kResThreads * 2);   // [kDriveSteps][taking-part blocks][kResThreads] u16
  const bool fifo = c->kind == ADSEQ_FIFO;
  L->slot = take(c->kind == ADSEQ_SORTED ? (size_t)c->capacity * BN * 8 : 0);
  L->fkey = take(fifo ? (size_t)((c->capacity + 7) / 8 * 8) * BN * 2 : 0);
  L->famp = take(fifo ? (size_t)c->capacity * BN * 4 : 0);
  L->vmask = take(fifo ? (size_t)((c->capacity + 31) / 32) * BN * 4 : 0);
  L->occ = take(ptq ? BN * 4 : 0);
  L->head = take(ptq ? BN * 4 : 0);
  L->min_k = take(ptq ? BN * 4 : 0);
  L->cnt = take(ptq ? BN * 4 : 0);
  L->cont = take(ptq ? (size_t)kCont * BN * 16 : 0);
  L->c_head = take(ptq ? BN * 4 : 0);
  L->pool_p = take((size_t)L->pool_cap * 8);
  L->pool_t = take((size_t)L->pool_cap * 8);
  L->pool_next = take((size_t)L->pool_cap * 4);
  L->pool_k = take((size_t)L->pool_cap * 4);
  L->pool_a = take((size_t)L->pool_cap * 4);
  {
    const size_t Q = (size_t)c->batch * S;
    const size_t nbins = c->kind == ADSEQ_SYN_BINS ? (size_t)c->capacity : 1;
    L->sq_next = take(synq ? nbins * ((Q + 7) / 8 * 16) : 0);
    L->sq_flag = take(c->kind == ADSEQ_SYN_BINS && c->record_tape ? nbins * ((Q + 7) / 8 * 8) * 8 : 0);
    L->sq_hs = take(synfifo ? Q * 2 : 0);
    L->sq_key = take(synfifo ? Q * (size_t)c->capacity * 2 : 0);
    L->I_acc = take(synq ? BN * 4 : 0);
    L->last_evb = take(c->kind == ADSEQ_SYN_LATEST && c->record_tape ? 2 * BN * 8 : 0);
  }
  L->spk_words = take(bounded ? 2 * (size_t)L->words * 8 : 0);
  L->stepcnt = take(bounded ? 2 * (size_t)L->nblk * 16 : 0);
  L->packed = take(bounded ? S * 4 : 0);
  L->a_q = take(bounded ? S * 4 : 0);
  L->synf = take(bounded ? 0 : S * 8);
  L->synb = take(bounded ? 0 : S * 8);
  L->dstart = take(bounded ? 0 : (size_t)c->n_neurons * (c->d_max_steps + 2) * 4);
  L->nearcnt = take(bounded ? 0 : (size_t)(L->W + 1) * c->n_neurons * 4);
  L->perm = take(bounded ? 0 : S * 4);
  L->rowsum = take((size_t)c->n_neurons * 8);
  L->insum = take((size_t)c->n_neurons * 8);
  L->rowlen = take(bounded ? (size_t)c->n_neurons * 4 : 0);
  L->ebuf = take(bounded ? 0 : stage_parts * L->NB * (size_t)L->cap * 8);
  L->ecnt = take(bounded ? 0 : stage_parts * L->NB * 4);
  L->amp = take(cont && bounded ? S * 4 : 0);
  L->fdec = take(cont ? S * 4 : 0);
  const size_t T = c->record_tape ? (size_t)c->max_steps : 0;
  L->tapeU = take(T * BN * 4);
  L->tape_bits = take(bounded ? 0 : T * L->words * 8);
  L->spk_count = take(c->record_tape ? BN * 4 : 0);
  L->step_off = take(c->record_tape ? (T + 1) * 8 : 0);
  L->step_evoff = take(c->record_tape && bounded ? (T + 1) * 8 : 0);
  L->tape_spk = take(bounded ? (size_t)L->spike_cap * 4 : 0);
  L->tape_evb = take(bounded ? (size_t)L->spike_cap * 8 : 0);
  L->tape_row = take(bounded ? (size_t)L->spike_cap * sizeof(RowSpan) : 0);
  L->tape_adm = take((size_t)L->event_cap);
  const bool tape = c->record_tape != 0;
  L->bwd_ring = take(tape && bounded ? nstates * (size_t)L->R * BN * 4 : 0);
  L->bwd_carry = take(tape ? BN * 4 : 0);
  L->bwd_carryJ = take(tape && c->tau_syn_ms > 0.0f ? nstates * BN * 4 : 0);
  L->bwd_G = take(tape && bounded ? (size_t)kFanSplitMax * BN * 4 : 0);
  L->gwin = take(tape && !bounded ? nstates * 2 * (size_t)L->W * BN * 4 : 0);
  L->Gacc = take(tape && !bounded ? (size_t)L->R * BN * 4 : 0);
  L->gsum = take(tape && !bounded ? nstates * S * 4 : 0);
  {
    // reverse sweep by windows (delta synapse only): staging of a window's near events, 4 per state
    // cell and step, between 4,096 and 262,144
    const bool byw = tape && !bounded && !(c->tau_syn_ms > 0.0f);
    size_t cap = 4 * BN;
    cap = cap < 4096 ? 4096 : (cap > 262144 ? 262144 : cap);
    L->near_ev_cap = byw ? (int)cap : 0;
    L->wspk = take(byw ? BN * 8 : 0);
    L->near_cnt = take(byw ? 2 * 64 * 4 : 0);
    L->near_ev = take(byw ? (size_t)L->W * cap * 16 : 0);
    L->near_spk = take(byw ? (size_t)L->W * kNearSpikeCap * 4 : 0);
    L->near_counts = take(byw ? 2 * T * 4 : 0);
  }
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

void join_ahead(adseq* h, hipStream_t st);

// Clears the dynamic state (not the prepared synapses).
void launch_reset(adseq* h, hipStream_t st) {
  const Dev& d = h->dev;
  join_ahead(h, st);
  h->ahead_for = -1;
  h->fold_upto = 0;
  h->bar_base = 0;   // (the counter itself is cleared with the other counters)
  h->rev_base = 0;   // (likewise)
  h->chain_arrivals = 0;   // (likewise)
  h->drive_from = h->drive_upto = 0;
  const size_t BN = (size_t)d.BN;
  fill_u32(st, d.ctr, 0u, sizeof(Counters) / 4);
  fill_u32(st, d.V, 0u, BN);
  if (d.alpha_s > 0.0f) fill_u32(st, d.J, 0u, (d.alpha_r > 0.0f ? 2 : 1) * BN);
  if (d.kind == ADSEQ_RING) {
    fill_u32(st, d.win, 0u, 2 * (size_t)d.W * BN);
    fill_u32(st, d.spike_bits, 0u, (size_t)d.R * d.words * 2);
    fill_u32(st, d.blk, 0u, kMaxBinBlocks * sizeof(BlkCtr) / 4);
    // staging counters: zero except between the two passes of a window's expansion
    if (d.cap > 0) fill_u32(st, d.ecnt, 0u, (size_t)(d.P < kMaxParts ? d.P : kMaxParts) * d.NB);
  } else if (per_synapse_kind(d.kind)) {
    fill_u32(st, d.sq_next, 0xffffffffu,
             (size_t)(d.kind == ADSEQ_SYN_BINS ? d.C : 1) * (((size_t)d.B * d.S + 7) / 8 * 4));   // every queue empty
    if (d.kind == ADSEQ_SYN_FIFO) fill_u32(st, d.sq_hs, 0u, ((size_t)d.B * d.S + 1) / 2);   // (the keys need no clearing)
    fill_u32(st, d.I_acc, 0u, BN);
    fill_u32(st, d.blk, 0u, ((size_t)d.blk_pop + kSynqBlocks) * sizeof(BlkCtr) / 4);
    h->pending_admit = false;
  } else {
    fill_u32(st, d.occ, 0u, BN);
    fill_u32(st, d.head, 0u, BN);
    fill_u32(st, d.c_head, 0xffffffffu, BN);
    fill_u32(st, d.min_k, 0xffffffffu, BN);
    if (d.kind == ADSEQ_FIFO) fill_u32(st, d.vmask, 0u, (size_t)d.nw * BN);
    fill_u32(st, d.cnt, 0u, BN);
    fill_u32(st, d.blk, 0u, ((size_t)d.nblk + fan_slots(d.nblk)) * sizeof(BlkCtr) / 4);
    h->pending_admit = false;
  }
  if (d.record) {
    fill_u32(st, d.step_off, 0u, 2);  // step_off[0] = 0 (int64)
    if (d.kind != ADSEQ_RING) fill_u32(st, d.step_evoff, 0u, 2);
    fill_u32(st, d.spk_count, 0u, BN);
  }
  h->next_step = 0;
  h->enq_calls = 0;
  h->tape_ok = d.record != 0;
  h->bits_clear_for = -1;
}

// FIFO / SORTED: admission of what is pending, then (MODE 1) pop or (MODE 2) the closed-loop step.
template <int MODE>
void launch_neurons(adseq* h, hipStream_t st, long long n, int parity, const float* i_ext,
                    unsigned char* spikes_out, float* I_out) {
  const Dev& d = h->dev;
  const dim3 grid(grid_for((size_t)d.BN)), block(kBlock);
  if (per_synapse_kind(d.kind)) {
    // per-synapse queues: every queue is looked at first (nothing is pending for MODE 0)
    if (MODE == 0) return;
    if (d.kind == ADSEQ_SYN_FIFO) {
      hipLaunchKernelGGL(k_synq_pop<false>, dim3(kSynqBlocks), block, 0, st, d, n, 0LL);
      hipLaunchKernelGGL((k_neurons<ADSEQ_SYN_FIFO, MODE>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
    } else if (d.kind == ADSEQ_SYN_LATEST) {
      hipLaunchKernelGGL(k_synq_pop<true>, dim3(kSynqBlocks), block, 0, st, d, n, 0LL);
      hipLaunchKernelGGL((k_neurons<ADSEQ_SYN_LATEST, MODE>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
    } else {
      // the bin of this step: its keys are contiguous
      const long long qpad = (((long long)d.B * d.S + 7) >> 3) << 3;
      hipLaunchKernelGGL(k_synq_pop<true>, dim3(kSynqBlocks), block, 0, st, d, n, (n % d.C) * qpad);
      hipLaunchKernelGGL((k_neurons<ADSEQ_SYN_BINS, MODE>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
    }
  } else if (d.kind == ADSEQ_FIFO)
    hipLaunchKernelGGL((k_neurons<ADSEQ_FIFO, MODE>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
  else
    hipLaunchKernelGGL((k_neurons<ADSEQ_SORTED, MODE>), grid, block, 0, st, d, n, parity, i_ext, spikes_out, I_out);
  h->pending_admit = false;
}

// FIFO / SORTED fan-out of step n: the spikes of this step's k_neurons launch (spk = nullptr,
// closed loop) or the caller's list of neuron indices (open loop).
void launch_fanout(adseq* h, hipStream_t st, long long n, const int* spk, const int* n_spk, int parity, int record) {
  const Dev& d = h->dev;
  const dim3 block(kBlock);
  if (!spk) {
    const dim3 grid((unsigned)d.nblk * d.fsplit);
    if (d.kind == ADSEQ_FIFO) hipLaunchKernelGGL((k_fanout_step<ADSEQ_FIFO>), grid, block, 0, st, d, n, parity, record);
    else if (d.kind == ADSEQ_SYN_FIFO) hipLaunchKernelGGL((k_fanout_step<ADSEQ_SYN_FIFO>), grid, block, 0, st, d, n, parity, record);
    else if (d.kind == ADSEQ_SYN_LATEST) hipLaunchKernelGGL((k_fanout_step<ADSEQ_SYN_LATEST>), grid, block, 0, st, d, n, parity, record);
    else if (d.kind == ADSEQ_SYN_BINS) hipLaunchKernelGGL((k_fanout_step<ADSEQ_SYN_BINS>), grid, block, 0, st, d, n, parity, record);
    else hipLaunchKernelGGL((k_fanout_step<ADSEQ_SORTED>), grid, block, 0, st, d, n, parity, record);
  } else {
    const dim3 grid(kFanoutBlocks);
    if (d.kind == ADSEQ_FIFO) hipLaunchKernelGGL((k_fanout_list<ADSEQ_FIFO>), grid, block, 0, st, d, n, spk, n_spk);
    else if (d.kind == ADSEQ_SYN_FIFO) hipLaunchKernelGGL((k_fanout_list<ADSEQ_SYN_FIFO>), grid, block, 0, st, d, n, spk, n_spk);
    else if (d.kind == ADSEQ_SYN_LATEST) hipLaunchKernelGGL((k_fanout_list<ADSEQ_SYN_LATEST>), grid, block, 0, st, d, n, spk, n_spk);
    else if (d.kind == ADSEQ_SYN_BINS) hipLaunchKernelGGL((k_fanout_list<ADSEQ_SYN_BINS>), grid, block, 0, st, d, n, spk, n_spk);
    else hipLaunchKernelGGL((k_fanout_list<ADSEQ_SORTED>), grid, block, 0, st, d, n, spk, n_spk);
  }
  h->pending_admit = !per_synapse_kind(d.kind);   // a per-synapse push is final
  h->last_stream = st;
}

// FIFO / SORTED: admits the contenders that the last enqueue registered, if that has not
// happened yet (it normally rides on the next step's launch).
void flush_admit(adseq* h, hipStream_t st) {
  if (h->dev.kind != ADSEQ_RING && h->pending_admit)
    launch_neurons<0>(h, st, h->next_step, 0, nullptr, nullptr, nullptr);
}

void mark(adseq* h, hipStream_t st, int kind, int count = 1);
void close_group(adseq* h, hipStream_t st, int kind);

// RING: called before step k0 is popped when k0 opens a window (k0 mod W = 0): expands the
// events of the spikes of the last d_max steps that arrive in the window (staging pass, then
// per-part accumulation; without staging room the first pass scatters with atomics and the
// second is skipped).  The staging pass also counts the spikes not counted yet, and their
// events, into the device counters.
// Expansion of the events of the spikes of steps [n_lo, n_hi) that arrive in window [k0, k0 + W) on `st`.
void launch_expansion(adseq* h, hipStream_t st, long long k0, long long n_lo, long long n_hi, long long count_from) {
  const Dev& d = h->dev;
  // staging mode: 0 none (atomics), 1 one store per event, 2 ordered by part in LDS first
  static const int sort_stage = env_pow2("ADSEQ_RING_SORTSTAGE", 1, 0, 1);
  const int stage = d.cap > 0 ? ((sort_stage && d.P <= kSortParts) ? 2 : 1) : 0;
  hipLaunchKernelGGL(k_win_bin, dim3((unsigned)d.NB), dim3(kRingThreads), 0, st, d, k0, n_lo, n_hi, 0, d.NB,
                     stage, count_from, h->res_P > 0 ? 1 : 0);
  if (d.cap > 0) {
    const int parts = d.P < kMaxParts ? d.P : kMaxParts;
    hipLaunchKernelGGL(k_win_acc, dim3((unsigned)parts), dim3(kRingThreads), 0, st, d, k0, 0);
  }
}

// The main stream waits for what was expanded ahead on the library's own stream (experimental overlap).
void join_ahead(adseq* h, hipStream_t st) {
  if (h->ahead_for >= 0 && h->ev_ahead) (void)hipStreamWaitEvent(st, h->ev_ahead, 0);
}

void ring_open_window(adseq* h, hipStream_t st, long long k0) {
  const Dev& d = h->dev;
  if ((k0 & (long long)(d.W - 1)) != 0 || k0 <= 0) return;
  close_group(h, st, 1);
  mark(h, st, -1);
#ifdef ADSEQ_PHASE_CLOCK
  // the phase clocks cover the windows from step 512 on (the spike history is full by then)
  if (k0 == 512) fill_u32(st, reinterpret_cast<unsigned*>(d.ctr->phase), 0u, 48);
#endif
  long long n_lo = k0 - d.d_max > 0 ? k0 - d.d_max : 0;
  static const int overlap = env_pow2("ADSEQ_RING_OVERLAP", 0, 0, 1);
  const bool ahead = overlap && h->res_P == 0;
  if (ahead) {
    if (!h->aux) {
      (void)hipStreamCreateWithFlags(&h->aux, hipStreamNonBlocking);
      (void)hipEventCreateWithFlags(&h->ev_boundary, hipEventDisableTiming);
      (void)hipEventCreateWithFlags(&h->ev_ahead, hipEventDisableTiming);
    }
    // what was expanded ahead covers the spikes before the previous boundary: only the last window's are left
    if (h->ahead_for == k0) { join_ahead(h, st); n_lo = k0 - d.W; }
    else join_ahead(h, st);
    h->ahead_for = -1;
  }
  launch_expansion(h, st, k0, n_lo, k0, h->fold_upto);
  h->fold_upto = k0;
  if (ahead && h->aux) {
    // the next window's events from the spikes before this boundary: on the other stream, beside the steps of this window
    const long long k1 = k0 + d.W;
    const long long lo2 = k1 - d.d_max > 0 ? k1 - d.d_max : 0;
    if (lo2 < k0) {
      (void)hipEventRecord(h->ev_boundary, st);
      (void)hipStreamWaitEvent(h->aux, h->ev_boundary, 0);
      launch_expansion(h, h->aux, k1, lo2, k0, k0 /* nothing is counted here */);
      (void)hipEventRecord(h->ev_ahead, h->aux);
      h->ahead_for = k1;
    }
  }
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
    const int syn = d.alpha_r > 0.0f ? 2 : (d.alpha_s > 0.0f ? 1 : 0);   // synaptic current states
#define ADSEQ_STEP_WIN(MODE)                                                                                   \
  do {                                                                                                         \
    if (record && syn == 0) hipLaunchKernelGGL((k_step_win<true, 0, MODE>), grid, block, 0, st, step, i_ext, spikes_out, d);       \
    else if (record && syn == 1) hipLaunchKernelGGL((k_step_win<true, 1, MODE>), grid, block, 0, st, step, i_ext, spikes_out, d);  \
    else if (record) hipLaunchKernelGGL((k_step_win<true, 2, MODE>), grid, block, 0, st, step, i_ext, spikes_out, d);              \
    else if (syn == 0) hipLaunchKernelGGL((k_step_win<false, 0, MODE>), grid, block, 0, st, step, i_ext, spikes_out, d);           \
    else if (syn == 1) hipLaunchKernelGGL((k_step_win<false, 1, MODE>), grid, block, 0, st, step, i_ext, spikes_out, d);           \
    else hipLaunchKernelGGL((k_step_win<false, 2, MODE>), grid, block, 0, st, step, i_ext, spikes_out, d);                         \
  } while (0)
    if (d.count_pop) ADSEQ_STEP_WIN(1);
    else if (d.lazy_rows) ADSEQ_STEP_WIN(2);
    else ADSEQ_STEP_WIN(0);
#undef ADSEQ_STEP_WIN
    h->grp_count += 1;
  } else {
    mark(h, st, -1);
    launch_neurons<2>(h, st, step, parity, i_ext, spikes_out, nullptr);
    mark(h, st, 1);
    launch_fanout(h, st, step, nullptr, nullptr, parity, record);
    mark(h, st, 0);
  }
  h->enq_calls += 1;
  h->next_step = step + 1;
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

// RING: steps step0 .. step0 + n_steps - 1 with one resident launch per window (ring_resident.h).
template <bool RECORD, int NG>
void launch_run_xcd(const Dev& d, hipStream_t st, int syn, long long n0, int cnt, unsigned bar_base, int P, int chunk) {
  // block b runs on XCD b mod 8: with stride 8 the taking-part blocks share one XCD
  // (at most 32 taking-part blocks per XCD, one per compute unit: what the barrier measurements cover)
  int stride = env_pow2("ADSEQ_RING_RESIDENT_STRIDE", kResStride, 1, 8);
  while (stride > 1 && (long long)P * stride > 32 * 8) stride >>= 1;
  const dim3 grid((unsigned)(P * stride)), block(kResLaunch);
  if (syn == 0) hipLaunchKernelGGL((k_run_xcd<RECORD, 0, NG>), grid, block, 0, st, n0, cnt, bar_base, P, chunk, stride, d);
  else if (syn == 1) hipLaunchKernelGGL((k_run_xcd<RECORD, 1, NG>), grid, block, 0, st, n0, cnt, bar_base, P, chunk, stride, d);
  else hipLaunchKernelGGL((k_run_xcd<RECORD, 2, NG>), grid, block, 0, st, n0, cnt, bar_base, P, chunk, stride, d);
}
void ring_run_resident(adseq* h, hipStream_t st, long long step0, long long n_steps) {
  const Dev& d = h->dev;
  const int syn = d.alpha_r > 0.0f ? 2 : (d.alpha_s > 0.0f ? 1 : 0);
  long long n = step0;
  const long long end = step0 + n_steps;
  while (n < end) {
    ring_open_window(h, st, n);
    open_group(h, st);
    const long long in_win = (long long)d.W - (n & (long long)(d.W - 1));
    int cnt = (int)(end - n < in_win ? end - n : in_win);
    // a launch either records all its steps or none: it ends where the tape ends
    const bool record = d.record && h->tape_ok && n < d.max_steps;
    if (record && n + cnt > d.max_steps) cnt = (int)(d.max_steps - n);
    if (d.record && n >= d.max_steps) h->tape_ok = false;
    if (d.p_thresh && (n < h->drive_from || n + cnt > h->drive_upto)) {
      // drive words for as much of this call as the buffer holds
      const long long upto = end - n < kDriveSteps ? end : n + kDriveSteps;
      const long long items = (upto - n) * h->res_P * kResThreads;
      const long long blocks = (items + kBlock - 1) / kBlock;
      hipLaunchKernelGGL(k_drive_words, dim3((unsigned)(blocks < 8192 ? blocks : 8192)), dim3(kBlock), 0, st, d, n, upto,
                         h->res_P, h->res_chunk, h->res_npt);
      h->drive_from = n; h->drive_upto = upto;
    }
    const unsigned base = d.res_wide ? h->rev_base : h->bar_base;
    if (record) {
      if (h->res_npt == 1) launch_run_xcd<true, 1>(d, st, syn, n, cnt, base, h->res_P, h->res_chunk);
      else launch_run_xcd<true, 2>(d, st, syn, n, cnt, base, h->res_P, h->res_chunk);
    } else {
      if (h->res_npt == 1) launch_run_xcd<false, 1>(d, st, syn, n, cnt, base, h->res_P, h->res_chunk);
      else launch_run_xcd<false, 2>(d, st, syn, n, cnt, base, h->res_P, h->res_chunk);
    }
    (d.res_wide ? h->rev_base : h->bar_base) += (unsigned)(cnt - 1) * (unsigned)h->res_P;
    h->grp_count += cnt;
    h->enq_calls += cnt;
    n += cnt;
    h->next_step = n;
  }
}

// RING: steps step0 .. step0 + n_steps - 1 with one launch per window over the whole chip (ring_resident_forward.h).
void ring_run_chip(adseq* h, hipStream_t st, long long step0, long long n_steps) {
  const Dev& d = h->dev;
  long long n = step0;
  const long long end = step0 + n_steps;
  int stride = env_pow2("ADSEQ_RING_RESIDENT_STRIDE", kResStride, 1, 8);
  while (stride > 1 && (long long)h->fwd_P * stride > 32 * 8) stride >>= 1;
  const dim3 grid((unsigned)(h->fwd_P * stride)), block(kResLaunch);
  while (n < end) {
    ring_open_window(h, st, n);
    open_group(h, st);
    const long long in_win = (long long)d.W - (n & (long long)(d.W - 1));
    int cnt = (int)(end - n < in_win ? end - n : in_win);
    // a launch either records all its steps or none: it ends where the tape ends
    const bool record = d.record && h->tape_ok && n < d.max_steps;
    if (record && n + cnt > d.max_steps) cnt = (int)(d.max_steps - n);
    if (d.record && n >= d.max_steps) h->tape_ok = false;
    // (one neuron per thread where a block owns no more neurons than it has worker threads, else four)
#define ADSEQ_FWD(REC, NPT) hipLaunchKernelGGL((k_fwd_chip<REC, NPT>), grid, block, 0, st, n, cnt, h->rev_base, h->fwd_P, h->fwd_chunk, stride, h->fwd_margin, d)
    if (h->fwd_chunk <= kResThreads) { if (record) ADSEQ_FWD(true, 1); else ADSEQ_FWD(false, 1); }
    else if (h->fwd_chunk <= 4 * kResThreads) { if (record) ADSEQ_FWD(true, 4); else ADSEQ_FWD(false, 4); }
    else { if (record) ADSEQ_FWD(true, 8); else ADSEQ_FWD(false, 8); }
#undef ADSEQ_FWD
    h->rev_base += (unsigned)(cnt - 1) * (unsigned)h->fwd_P;
    h->grp_count += 1;   // (launches of the group)
    h->enq_calls += cnt;
    n += cnt;
    h->next_step = n;
  }
}

// RING, chained step launches (ring_chain.h): the step launches go to the caller's stream and to a
// stream of the library's own in turn and wait for one another themselves.  The stream and the two
// events are made at the first use.
bool chain_ready(adseq* h) {
  if (h->chain_st) return true;
  hipStream_t s = nullptr;
  hipEvent_t a = nullptr, b = nullptr;
  if (hipStreamCreateWithFlags(&s, hipStreamNonBlocking) != hipSuccess) return false;
  if (hipEventCreateWithFlags(&a, hipEventDisableTiming) != hipSuccess) { (void)hipStreamDestroy(s); return false; }
  if (hipEventCreateWithFlags(&b, hipEventDisableTiming) != hipSuccess) { (void)hipEventDestroy(a); (void)hipStreamDestroy(s); return false; }
  h->chain_st = s; h->ev_fork = a; h->ev_join = b;
  return true;
}
// The library's stream goes on from where `st` is now / `st` goes on when the library's stream is done.
void chain_fork(adseq* h, hipStream_t st) {
  (void)hipEventRecord(h->ev_fork, st);
  (void)hipStreamWaitEvent(h->chain_st, h->ev_fork, 0);
}
void chain_join(adseq* h, hipStream_t st) {
  (void)hipEventRecord(h->ev_join, h->chain_st);
  (void)hipStreamWaitEvent(st, h->ev_join, 0);
}
hipStream_t chain_next_stream(adseq* h, hipStream_t st) { return (h->chain_turn++ & 1u) ? h->chain_st : st; }

// RING: steps step0 .. step0 + n_steps - 1 as chained launches.  At a window boundary both streams
// meet: the expansion runs on `st` after everything before it and before everything after it.
void ring_run_chain(adseq* h, hipStream_t st, long long step0, long long n_steps) {
  const Dev& d = h->dev;
  const dim3 grid((unsigned)d.nblk), block(kBlock);
  bool forked = false;
  for (long long n = step0; n < step0 + n_steps; ++n) {
    if ((n & (long long)(d.W - 1)) == 0 && n > 0 && forked) { chain_join(h, st); forked = false; }
    ring_open_window(h, st, n);
    open_group(h, st);
    if (!forked) { chain_fork(h, st); forked = true; }
    const bool record = d.record && h->tape_ok && n < d.max_steps;
    if (d.record && n >= d.max_steps) h->tape_ok = false;
    hipStream_t s = chain_next_stream(h, st);
    if (h->chain_tpb == 1024) {
      const dim3 g4((unsigned)((d.BN + 1023) / 1024)), b4(1024);
      if (record) hipLaunchKernelGGL((k_step_chain<true, 1024>), g4, b4, 0, s, n, h->chain_arrivals, d);
      else hipLaunchKernelGGL((k_step_chain<false, 1024>), g4, b4, 0, s, n, h->chain_arrivals, d);
      h->chain_arrivals += g4.x - (unsigned)d.nblk;
    } else if (record) hipLaunchKernelGGL((k_step_chain<true, 256>), grid, block, 0, s, n, h->chain_arrivals, d);
    else hipLaunchKernelGGL((k_step_chain<false, 256>), grid, block, 0, s, n, h->chain_arrivals, d);
    h->chain_arrivals += (unsigned)d.nblk;
    h->grp_count += 1;
    h->enq_calls += 1;
    h->next_step = n + 1;
  }
  if (forked) chain_join(h, st);
}

// RING: virtual blocks of one far gather over the spikes of steps [n_lo, n_hi): one 8-word line per
// wavefront, one block per compute unit at most (cfg2, 4,000 lines: 19.0 us per window with 63 blocks, 14.0 with 128,
// 12.2 with 256, 14.0 with 512; cfg3: 256 of 128..1,024).
int gather_blocks(const Dev& d, long long n_lo, long long n_hi) {
  const long long lines = (n_hi - n_lo) * d.wgroups;
  long long g = (lines + kRingWaves - 1) / kRingWaves;
  return env_pow2("ADSEQ_RING_GATHERBLOCKS", (int)(g < 1 ? 1 : (g > 256 ? 256 : g)), 1, 2048);
}

// RING: the whole reverse sweep on `st`.  A window is swept as a whole (ring_reverse.h: one dense
// pass, the near corrections step by step inside one workgroup, then the far gather) when
// `counts` (spikes and near events of every step, from k_bwd_near_counts; null: never) says that
// its staging fits; otherwise with one launch per reverse step (k_bwd_step_win).  Either way, when
// a window is complete the far queue terms of all earlier spikes that arrive in it are gathered in
// one pass.
void ring_backward_launch(adseq* h, hipStream_t st, long long T, float dscale, const float* dL_dcount,
                          const float* dL_dU, float* grad_w, float* grad_d, const int* counts) {
  const Dev& d = h->dev;
  const dim3 block(kBlock), gn((unsigned)d.nblk);
  const size_t nst = d.alpha_r > 0.0f ? 2 : 1;
  fill_u32(st, d.bwd_carry, 0u, (size_t)d.BN);
  if (d.alpha_s > 0.0f) fill_u32(st, d.bwd_carryJ, 0u, nst * (size_t)d.BN);
  fill_u32(st, d.gsum, 0u, nst * (size_t)d.S);
  fill_u32(st, d.gwin, 0u, nst * 2 * (size_t)d.W * d.BN);
  fill_u32(st, d.Gacc, 0u, (size_t)d.R * d.BN);
  if (counts) fill_u32(st, d.near_nspk, 0u, 128);
  int flow_filled = -1;   // window buffer that the resident reverse kernel before has filled with its sentinel (-1: none)
  for (long long k0 = (T - 1) & ~(long long)(d.W - 1); k0 >= 0; k0 -= d.W) {
    const long long k1 = k0 + d.W < T ? k0 + d.W : T;
    const int nsteps = (int)(k1 - k0);
    bool whole = counts != nullptr;
    for (long long n = k0; whole && n < k1; ++n)
      whole = counts[n] <= kNearSpikeCap && counts[T + n] <= d.near_ev_cap;
    open_group(h, st);
    if (whole) {
      hipLaunchKernelGGL(k_bwd_dense_win, gn, block, 0, st, k0, nsteps, dL_dcount, dL_dU, d);
      if (nsteps >= 2) {
        long long spikes = 0;
        for (long long n = k0; n < k1; ++n) spikes += counts[n];
        if (spikes > 0) {
          // about four 8-word lines of the window's spike words per wavefront
          const long long lines = (long long)nsteps * d.wgroups;
          long long nvb = (lines + 4 * kRingWaves - 1) / (4 * kRingWaves);
          nvb = nvb < 1 ? 1 : (nvb > 64 ? 64 : nvb);
          hipLaunchKernelGGL(k_bwd_near_stage, dim3((unsigned)nvb), dim3(kRingThreads), 0, st, d, k0, k1, T, (int)nvb);
          hipLaunchKernelGGL(k_bwd_near_seq, dim3(1), dim3(kRingThreads), 0, st, d, k0, nsteps);
        }
      }
    } else {
      if (h->rev_P > 0) {
        // the steps of the window in one launch on the blocks of one XCD (ring_resident_reverse.h)
        int stride = env_pow2("ADSEQ_RING_RESIDENT_STRIDE", kResStride, 1, 8);
        while (stride > 1 && (long long)h->rev_P * stride > 32 * 8) stride >>= 1;
        const dim3 rg((unsigned)(h->rev_P * stride)), rb(kResLaunch);
        if (h->rev_flow) {
          // no grid barrier: every cell of the window's buffer says "not written yet" until its owner stores it.
          // The launch before this one has filled the buffer in passing, unless this is the sweep's first launch or
          // the window after this one was swept another way
          const int buf = (int)((k0 >> d.wshift) & 1);
          if (flow_filled != buf) fill_u32(st, d.gwin + (size_t)buf * d.W * d.BN, kFlowSentinel, (size_t)d.W * d.BN);
          const int fill_other = (counts == nullptr && k0 > 0) ? 1 : 0;
          // (one neuron per thread where a block owns no more than it has threads, else four)
#define ADSEQ_FLOW3(DU, SURR, NPT) hipLaunchKernelGGL((k_bwd_flow<DU, SURR, NPT>), rg, dim3(kResThreads), 0, st, k1, nsteps, T, h->rev_P, h->rev_chunk, stride, fill_other, dL_dcount, dL_dU, d)
#define ADSEQ_FLOW(DU, SURR) do { if (h->rev_chunk <= kResThreads) ADSEQ_FLOW3(DU, SURR, 1); else if (h->rev_chunk <= 4 * kResThreads) ADSEQ_FLOW3(DU, SURR, 4); else ADSEQ_FLOW3(DU, SURR, 8); } while (0)
          if (d.surrogate == ADSEQ_SURR_SUPERSPIKE) { if (dL_dU) ADSEQ_FLOW(true, ADSEQ_SURR_SUPERSPIKE); else ADSEQ_FLOW(false, ADSEQ_SURR_SUPERSPIKE); }
          else if (d.surrogate == ADSEQ_GRAD_SPIKE_TIME) { if (dL_dU) ADSEQ_FLOW(true, ADSEQ_GRAD_SPIKE_TIME); else ADSEQ_FLOW(false, ADSEQ_GRAD_SPIKE_TIME); }
          else { if (dL_dU) ADSEQ_FLOW(true, ADSEQ_SURR_OFF); else ADSEQ_FLOW(false, ADSEQ_SURR_OFF); }
#undef ADSEQ_FLOW
#undef ADSEQ_FLOW3
          flow_filled = fill_other ? 1 - buf : -1;
        } else {
        if (dL_dU) hipLaunchKernelGGL((k_bwd_xcd<true>), rg, rb, 0, st, k1, nsteps, T, h->rev_base, h->rev_P, h->rev_chunk, stride, dL_dcount, dL_dU, d);
        else hipLaunchKernelGGL((k_bwd_xcd<false>), rg, rb, 0, st, k1, nsteps, T, h->rev_base, h->rev_P, h->rev_chunk, stride, dL_dcount, dL_dU, d);
        h->rev_base += (unsigned)(nsteps - 1) * (unsigned)h->rev_P;
        }
      } else if (h->chain && chain_ready(h)) {
        chain_fork(h, st);
        for (long long n = k1 - 1; n >= k0; --n) {
          if (h->chain_tpb == 1024) {
            const dim3 g4((unsigned)((d.BN + 1023) / 1024));
            hipLaunchKernelGGL((k_bwd_step_chain<1024>), g4, dim3(1024), 0, chain_next_stream(h, st), n, T, h->chain_arrivals, dL_dcount, dL_dU, d);
            h->chain_arrivals += g4.x;
          } else {
            hipLaunchKernelGGL((k_bwd_step_chain<256>), gn, block, 0, chain_next_stream(h, st), n, T, h->chain_arrivals, dL_dcount, dL_dU, d);
            h->chain_arrivals += (unsigned)d.nblk;
          }
        }
        chain_join(h, st);
      } else
      for (long long n = k1 - 1; n >= k0; --n) {
        if (d.alpha_r > 0.0f) hipLaunchKernelGGL((k_bwd_step_win<2, false>), gn, block, 0, st, n, T, dL_dcount, dL_dU, d);
        else if (d.alpha_s > 0.0f) hipLaunchKernelGGL((k_bwd_step_win<1, false>), gn, block, 0, st, n, T, dL_dcount, dL_dU, d);
        else if (d.lazy_rows) hipLaunchKernelGGL((k_bwd_step_win<0, true>), gn, block, 0, st, n, T, dL_dcount, dL_dU, d);
        else hipLaunchKernelGGL((k_bwd_step_win<0, false>), gn, block, 0, st, n, T, dL_dcount, dL_dU, d);
      }
    }
    h->grp_count += (!whole && h->rev_P > 0) ? 1 : nsteps;   // launches of the group: the resident reverse kernel takes the window in one
    // far gather into the window (and, after a sweep of the whole window, the per-synapse sums of
    // its own near events): spikes of steps [lo, hi)
    const long long lo = k0 - d.d_max > 0 ? k0 - d.d_max : 0;
    const long long hi = whole ? k1 : k0;
    if (hi > lo) {
      close_group(h, st, 3);
      mark(h, st, -1);
      const int nvb = gather_blocks(d, lo, hi);
      if (d.alpha_r > 0.0f) hipLaunchKernelGGL((k_bwd_win<true>), dim3((unsigned)nvb), dim3(kRingThreads), 0, st, d, k0, lo, hi, T, 0, nvb);
      else hipLaunchKernelGGL((k_bwd_win<false>), dim3((unsigned)nvb), dim3(kRingThreads), 0, st, d, k0, lo, hi, T, 0, nvb);
      mark(h, st, 2);
    }
  }
  close_group(h, st, 3);
  const unsigned gf = (unsigned)(d.N < 65536 ? d.N : 65536);
  hipLaunchKernelGGL(k_grad_finish, dim3(gf), block, 0, st, d, dscale, grad_w, grad_d);
}

}  // namespace

// Workspace of adseq_create_static: one array per GPU the library runs on, held until the
// process ends.  In host code the name stands for the symbol, not for device memory: its device
// address is looked up once per device (static_workspace) and only that pointer is handed on.
static __device__ __align__(256) unsigned char scratch[ADSEQ_STATIC_WORKSPACE_BYTES];

namespace {

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];      // device address of `scratch` on every device, once looked up
adseq g_static_handle[kMaxDevices];    // the one handle per device that lives in the static workspace
bool g_static_busy[kMaxDevices];

// Device address of this device's copy of `scratch` (nullptr, with *dev_out = -1, on failure).
void* static_workspace(int* dev_out) {
  int dev = -1;
  *dev_out = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    g_scratch_ptr[dev] = p;
  }
  *dev_out = dev;
  return g_scratch_ptr[dev];
}

int create_in(const adseq_config* cfg, void* workspace, size_t workspace_bytes, adseq* storage, adseq_t** out);

}  // namespace

extern "C" {

size_t adseq_workspace_bytes(const adseq_config* cfg) {
  Layout L;
  if (!make_layout(cfg, &L)) return 0;
  return L.total;
}

int adseq_create(const adseq_config* cfg, adseq_t** out) {
  if (!cfg || !out) return ADSEQ_E_INVALID_ARG;
  return create_in(cfg, cfg->workspace, cfg->workspace_bytes, nullptr, out);
}

int adseq_create_static(const adseq_config* cfg, adseq_t** out) {
  if (!cfg || !out) return ADSEQ_E_INVALID_ARG;
  Layout L;
  if (!make_layout(cfg, &L)) return ADSEQ_E_INVALID_ARG;
  if (L.total > (size_t)ADSEQ_STATIC_WORKSPACE_BYTES) return ADSEQ_E_WORKSPACE;   // does not fit the static workspace
  int dev = -1;
  void* ws = static_workspace(&dev);
  if (!ws) return ADSEQ_E_HIP;
  if (g_static_busy[dev]) return ADSEQ_E_WORKSPACE;   // this device's static workspace already holds a live handle
  const int rc = create_in(cfg, ws, (size_t)ADSEQ_STATIC_WORKSPACE_BYTES, &g_static_handle[dev], out);
  if (rc == ADSEQ_OK) g_static_busy[dev] = true;
  return rc;
}

}  // extern "C"

namespace {

// Body of adseq_create / adseq_create_static: the handle lives in `storage` if given (nothing is
// allocated then), else on the heap.
int create_in(const adseq_config* cfg, void* workspace, size_t workspace_bytes, adseq* storage, adseq_t** out) {
  Layout L;
  if (!make_layout(cfg, &L)) return ADSEQ_E_INVALID_ARG;
  if (!cfg->row_ptr) return ADSEQ_E_INVALID_ARG;
  if (cfg->n_synapses > 0) {   // a network without synapses needs none of the per-synapse arrays
    if (!cfg->weight || !cfg->col) return ADSEQ_E_INVALID_ARG;
    if ((cfg->delay_steps == nullptr) == (cfg->delay_ms == nullptr)) return ADSEQ_E_INVALID_ARG;
  } else if (cfg->delay_steps && cfg->delay_ms) {
    return ADSEQ_E_INVALID_ARG;
  }
  if (!workspace || ((uintptr_t)workspace & 255) || workspace_bytes < L.total)
    return ADSEQ_E_WORKSPACE;
  adseq* h = storage;
  if (h) {
    for (hipEvent_t e : h->evs) (void)hipEventDestroy(e);
    *h = adseq();
    h->in_static = true;
  } else {
    h = new (std::nothrow) adseq();
    if (!h) return ADSEQ_E_HOST_MEMORY;
  }
  auto drop = [&]() { if (!storage) delete h; };
  h->cfg = *cfg;
  h->cfg.workspace = workspace;
  h->cfg.workspace_bytes = workspace_bytes;
  h->ws_bytes = L.total;
  h->err[0] = 0;
  Dev& d = h->dev;
  memset(&d, 0, sizeof(d));
  char* ws = (char*)workspace;
  d.N = cfg->n_neurons; d.B = cfg->batch; d.BN = cfg->n_neurons * cfg->batch;
  d.n_magic = cfg->n_neurons == 1 ? 0xffffffffu : (unsigned)(0x100000000ull / (unsigned long long)cfg->n_neurons);
  d.R = L.R; d.C = cfg->capacity; d.kind = cfg->kind; d.dbits = L.dbits; d.d_max = cfg->d_max_steps;
  d.dmask = (1u << L.dbits) - 1u;
  d.continuous = cfg->delay_ms ? 1 : 0;
  d.record = cfg->record_tape ? 1 : 0;
  d.surrogate = cfg->surrogate;
  d.max_steps = cfg->record_tape ? cfg->max_steps : 0;
  d.pool_cap = (int)L.pool_cap;
  d.alpha = (float)std::exp(-(double)cfg->dt_ms / (double)cfg->tau_m_ms);
  d.theta = cfg->v_thresh; d.v_reset = cfg->v_reset; d.ext_w = cfg->ext_weight;
  d.dt = cfg->dt_ms;
  d.tau = cfg->tau_syn_ms > 0.0f ? cfg->tau_syn_ms : cfg->tau_m_ms;
  d.alpha_s = cfg->tau_syn_ms > 0.0f ? (float)std::exp(-(double)cfg->dt_ms / (double)cfg->tau_syn_ms) : 0.0f;
  d.alpha_r = cfg->tau_rise_ms > 0.0f ? (float)std::exp(-(double)cfg->dt_ms / (double)cfg->tau_rise_ms) : 0.0f;
  d.alpha_diff = (float)((double)d.alpha_s - (double)d.alpha_r);
  d.inv_tau_b = cfg->tau_rise_ms > 0.0f ? (float)(1.0 / (double)cfg->tau_rise_ms) : 0.0f;
  d.inv_tau_diff = cfg->tau_rise_ms > 0.0f ? (float)(1.0 / (double)cfg->tau_rise_ms - 1.0 / (double)cfg->tau_syn_ms) : 0.0f;
  d.J = (float*)(ws + L.J); d.bwd_carryJ = (float*)(ws + L.bwd_carryJ);
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
  d.drive_words = (unsigned long long*)(ws + L.drive_words);
#if defined(ADSEQ_PHASE_CLOCK) || defined(ADSEQ_ABLATE)
  d.dbg = getenv("ADSEQ_DBG") ? atoi(getenv("ADSEQ_DBG")) : 0;
#endif
  d.count_pop = env_pow2("ADSEQ_RING_COUNT_POPPED", 0, 0, 1);
  d.lazy_rows = env_pow2("ADSEQ_RING_LAZY_ROWS", 0, 0, 1);
  d.res_spins = env_pow2("ADSEQ_RING_RESIDENT_SPINS", kResMaxSpins, 1, kResMaxSpins);
  d.flow_hold = env_pow2("ADSEQ_RING_FLOW_WITHHOLD", 0, 0, 1);
  d.W = L.W; d.wshift = L.wshift; d.tp_shift = L.tp_shift; d.P = L.P; d.NB = L.NB; d.cap = L.cap;
  d.wgroups = L.wgroups;
  d.win = (int*)(ws + L.win);
  d.dstart = (unsigned*)(ws + L.dstart); d.nearcnt = (unsigned*)(ws + L.nearcnt);
  d.perm = (unsigned*)(ws + L.perm); d.rowsum = (long long*)(ws + L.rowsum); d.rowlen = (int*)(ws + L.rowlen);
  d.insum = (long long*)(ws + L.insum);
  d.ebuf = (uint2*)(ws + L.ebuf); d.ecnt = (int*)(ws + L.ecnt);
  d.tape_bits = (unsigned long long*)(ws + L.tape_bits);
  d.spk_count = (int*)(ws + L.spk_count);
  d.gwin = (float*)(ws + L.gwin); d.Gacc = (float*)(ws + L.Gacc); d.gsum = (float*)(ws + L.gsum);
  d.wspk = (unsigned long long*)(ws + L.wspk); d.near_nspk = (int*)(ws + L.near_cnt); d.near_nev = d.near_nspk + 64;
  d.near_ev = (uint4*)(ws + L.near_ev); d.near_spk = (int*)(ws + L.near_spk); d.near_counts = (int*)(ws + L.near_counts);
  d.near_ev_cap = L.near_ev_cap;
  d.slot = (uint2*)(ws + L.slot); d.vmask = (unsigned*)(ws + L.vmask);
  d.fkey = (unsigned short*)(ws + L.fkey); d.famp = (int*)(ws + L.famp);
  d.nw = (cfg->capacity + 31) / 32; d.cpad = (cfg->capacity + 7) / 8 * 8;
  {
    // shares of 256 entries that a row of average length needs
    const long long avg = cfg->n_synapses / cfg->n_neurons;
    const long long f = (avg + kBlock - 1) / kBlock;
    d.fsplit = (int)(f < 1 ? 1 : (f > kFanSplitMax ? kFanSplitMax : f));
    d.prefetch = (long long)cfg->n_neurons * cfg->batch <= (1LL << 18) ? 1 : 0;
  }
  d.occ = (int*)(ws + L.occ); d.head = (int*)(ws + L.head); d.c_head = (int*)(ws + L.c_head);
  d.pool_p = (long long*)(ws + L.pool_p); d.pool_t = (long long*)(ws + L.pool_t);
  d.pool_next = (int*)(ws + L.pool_next);
  d.min_k = (unsigned*)(ws + L.min_k); d.cnt = (int*)(ws + L.cnt);
  d.cont = (uint4*)(ws + L.cont);
  d.pool_k = (unsigned*)(ws + L.pool_k); d.pool_a = (int*)(ws + L.pool_a);
  d.spk_words = (unsigned long long*)(ws + L.spk_words); d.stepcnt = (long long*)(ws + L.stepcnt);
  d.sq_next = (unsigned short*)(ws + L.sq_next); d.sq_hs = (unsigned short*)(ws + L.sq_hs); d.sq_key = (unsigned short*)(ws + L.sq_key);
  d.sq_flag = (long long*)(ws + L.sq_flag);
  d.I_acc = (int*)(ws + L.I_acc); d.last_evb = (long long*)(ws + L.last_evb); d.blk_pop = L.nblk + (int)fan_slots(L.nblk);
  d.packed = (unsigned*)(ws + L.packed); d.a_q = (int*)(ws + L.a_q);
  d.amp = (d.continuous && d.kind != ADSEQ_RING) ? (float*)(ws + L.amp) : nullptr;
  d.synf = (uint2*)(ws + L.synf); d.synb = (uint2*)(ws + L.synb);
  d.fdec = d.continuous ? (float*)(ws + L.fdec) : nullptr;
  d.tapeU = (float*)(ws + L.tapeU); d.step_off = (long long*)(ws + L.step_off);
  d.step_evoff = (long long*)(ws + L.step_evoff);
  d.tape_spk = (int*)(ws + L.tape_spk); d.tape_evb = (long long*)(ws + L.tape_evb);
  d.tape_row = (RowSpan*)(ws + L.tape_row);
  d.tape_adm = (unsigned char*)(ws + L.tape_adm);
  d.bwd_ring = (float*)(ws + L.bwd_ring); d.bwd_carry = (float*)(ws + L.bwd_carry);
  d.bwd_G = (float*)(ws + L.bwd_G);

  if (d.kind == ADSEQ_RING) {
    const int syn = d.alpha_r > 0.0f ? 2 : (d.alpha_s > 0.0f ? 1 : 0);
    ResidentPlan rp = resident_plan((long long)d.BN);
    if (rp.P > 0 && !(resident_fits(run_xcd_kernel(true, syn, rp.npt)) && resident_fits(run_xcd_kernel(false, syn, rp.npt)))) rp = ResidentPlan();
    h->res_chunk = rp.chunk; h->res_P = rp.P; h->res_npt = rp.npt;
    if (!(d.alpha_s > 0.0f)) {
      ResidentPlan vp = reverse_plan((long long)d.BN);
      if (vp.P > 0 && vp.chunk <= 4 * kResThreads && !(resident_fits((const void*)k_bwd_xcd<true>) && resident_fits((const void*)k_bwd_xcd<false>))) vp = ResidentPlan();
      h->rev_chunk = vp.chunk; h->rev_P = vp.P; h->rev_npt = vp.npt;
      // the same layout without a grid barrier: the blocks wait for the cells they gather (ring_flow_reverse.h);
      // ADSEQ_RING_REVERSE_FLOW = 0: the kernel with a barrier per step
      h->rev_flow = vp.P > 0 && env_pow2("ADSEQ_RING_REVERSE_FLOW", 1, 0, 1) &&
                    resident_fits(flow_kernel(true, d.surrogate, vp.chunk), kResThreads) && resident_fits(flow_kernel(false, d.surrogate, vp.chunk), kResThreads);
      if (!h->rev_flow && vp.chunk > 4 * kResThreads) { h->rev_chunk = 0; h->rev_P = 0; h->rev_npt = 0; }   // (the kernel with a barrier holds four neurons per thread)
      // forward kernel over the whole chip with the candidates' rows requested ahead (ring_resident_forward.h): the
      // reverse kernel's layout (ADSEQ_RING_FORWARD_BLOCKS taking-part blocks, default 256).  ADSEQ_RING_FORWARD_CHIP:
      // see reverse_plan; ADSEQ_RING_FORWARD_MARGIN: candidate margin in thousandths of the membrane unit (default 5).
      ResidentPlan fp = reverse_plan((long long)d.BN, true);
      if (fp.P > 0 && !(fp.chunk <= kResThreads
                            ? resident_fits((const void*)k_fwd_chip<true, 1>) && resident_fits((const void*)k_fwd_chip<false, 1>)
                            : fp.chunk <= 4 * kResThreads
                            ? resident_fits((const void*)k_fwd_chip<true, 4>) && resident_fits((const void*)k_fwd_chip<false, 4>)
                            : resident_fits((const void*)k_fwd_chip<true, 8>) && resident_fits((const void*)k_fwd_chip<false, 8>)))
        fp = ResidentPlan();
      if (fp.P > 0 && !d.count_pop) {
        h->fwd_P = fp.P; h->fwd_chunk = fp.chunk; h->res_P = 0;
        if (const char* e = getenv("ADSEQ_RING_FORWARD_MARGIN")) { const int v = atoi(e); if (v >= 0 && v <= 100000) h->fwd_margin = (float)v * 1e-3f; }
      }
    }
    // chained step launches (ring_chain.h; experimental, off by default: measured slower than a launch per step on
    // one stream): delta synapse, and two launches' blocks must fit the chip side by side (512 blocks each at
    // most).  ADSEQ_RING_CHAIN = 1: wherever that holds (instead of the resident kernels too).  The static handle
    // makes no stream of its own.
    const int chain = env_pow2("ADSEQ_RING_CHAIN", 0, 0, 1);
    h->chain = chain && !h->in_static && !(d.alpha_s > 0.0f) && !d.count_pop && !d.lazy_rows && d.nblk <= 512;
    if (h->chain) h->res_P = 0;
    h->chain_tpb = env_pow2("ADSEQ_RING_CHAIN_THREADS", 256, 256, 1024) == 1024 ? 1024 : 256;
    d.chain_sleep = env_pow2("ADSEQ_RING_CHAIN_SLEEP", 1, 0, 64);
    d.rev_delay = env_pow2("ADSEQ_RING_REVERSE_DELAY", 0, 0, 16);
    d.res_wide = env_pow2("ADSEQ_RING_RESIDENT_WIDE", 0, 0, 1);
  }
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
    if (e == hipSuccess && !err) {
      const unsigned gr = (unsigned)((d.N + 3) / 4 < 8192 ? (d.N + 3) / 4 : 8192);
      hipLaunchKernelGGL(k_row_sums, dim3(gr), dim3(kBlock), 0, st, d);
    }
  }
  if (e == hipSuccess && !(err & (ERR_GRAPH | ERR_DELAY)) && d.S > 0) {
    fill_u32(st, d.insum, 0u, (size_t)d.N * 2);
    size_t g = ((size_t)d.S + kBlock - 1) / kBlock;
    hipLaunchKernelGGL(k_in_sums, dim3((unsigned)(g > 16384 ? 16384 : g)), dim3(kBlock), 0, st, d);
    hipLaunchKernelGGL(k_in_check, dim3((unsigned)grid_for((size_t)d.N)), dim3(kBlock), 0, st, d);
    e = read_err();
  }
  if (e != hipSuccess) { drop(); return ADSEQ_E_HIP; }
  if (err & ERR_GRAPH) { drop(); return ADSEQ_E_GRAPH; }
  if (err & ERR_DELAY) { drop(); return ADSEQ_E_DELAY_RANGE; }
  h->range_warn = (err & ERR_RANGE) != 0;
  if (h->range_warn) {   // the warning is kept on the host (a reset clears the device word)
    unsigned zero = 0;
    (void)hipMemcpyAsync(&d.ctr->err, &zero, sizeof(zero), hipMemcpyHostToDevice, st);
    (void)hipStreamSynchronize(st);
  }
  *out = h;
  return ADSEQ_OK;
}

}  // namespace

extern "C" {

int adseq_destroy(adseq_t* h) {
  if (!h) return ADSEQ_E_INVALID_ARG;
  if (h->chain_st) {
    (void)hipStreamSynchronize(h->chain_st);
    (void)hipStreamDestroy(h->chain_st); (void)hipEventDestroy(h->ev_fork); (void)hipEventDestroy(h->ev_join);
    h->chain_st = nullptr;
  }
  if (h->aux) {
    (void)hipStreamSynchronize(h->aux);
    (void)hipStreamDestroy(h->aux); (void)hipEventDestroy(h->ev_boundary); (void)hipEventDestroy(h->ev_ahead);
    h->aux = nullptr;
  }
  for (hipEvent_t e : h->evs) (void)hipEventDestroy(e);
  if (h->in_static) {
    h->evs.clear();
    g_static_busy[h - g_static_handle] = false;
    return ADSEQ_OK;
  }
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
    launch_fanout(h, (hipStream_t)stream, step, spike_ids, n_spikes, parity, 0);
  h->enq_calls += 1;
  h->tape_ok = false;
  HIP_TRY(h, hipGetLastError());
  return ADSEQ_OK;
}

int adseq_run_open(adseq_t* h, int64_t step0, int64_t n_steps, const int32_t* spike_ids,
                   const int64_t* spike_offsets, const int32_t* n_spikes, float* I_out, int64_t I_stride,
                   void* stream) {
  if (!h || !spike_ids || !spike_offsets || !n_spikes || !I_out || n_steps < 0 || I_stride < 0)
    return h ? fail(h, ADSEQ_E_INVALID_ARG, "adseq_run_open: null or negative argument") : ADSEQ_E_INVALID_ARG;
  if (h->dev.kind == ADSEQ_RING) {
    // pop and enqueue of a step in one launch (k_open_step_win)
    const Dev& d = h->dev;
    hipStream_t st = (hipStream_t)stream;
    for (int64_t k = 0; k < n_steps; ++k) {
      const long long step = step0 + k;
      if (step != h->next_step)
        return fail(h, ADSEQ_E_ORDER, "adseq_run_open: got step %lld, expected %lld", step, h->next_step);
      ring_open_window(h, st, step);
      if (h->bits_clear_for != step)
        fill_u32(st, d.spike_bits + (size_t)(step % d.R) * d.words, 0u, (size_t)d.words * 2);
      hipLaunchKernelGGL(k_open_step_win, dim3((unsigned)d.nblk), dim3(kBlock), 0, st, d, step,
                         spike_ids + spike_offsets[k], n_spikes + k, I_out + k * I_stride);
      h->bits_clear_for = step + 1;
      h->next_step = step + 1;
      h->enq_calls += 1;
      h->tape_ok = false;
    }
    HIP_TRY(h, hipGetLastError());
    return ADSEQ_OK;
  }
  for (int64_t k = 0; k < n_steps; ++k) {
    int rc = adseq_deliver(h, step0 + k, I_out + k * I_stride, stream);
    if (rc == ADSEQ_OK) rc = adseq_enqueue(h, step0 + k, spike_ids + spike_offsets[k], n_spikes + k, stream);
    if (rc != ADSEQ_OK) return rc;
  }
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
  if (h->dev.kind == ADSEQ_RING && h->fwd_P > 0) {
    ring_run_chip(h, (hipStream_t)stream, step0, n_steps);
  } else if (h->dev.kind == ADSEQ_RING && h->res_P > 0) {
    ring_run_resident(h, (hipStream_t)stream, step0, n_steps);
  } else if (h->dev.kind == ADSEQ_RING && h->chain && n_steps >= 2 && chain_ready(h)) {
    ring_run_chain(h, (hipStream_t)stream, step0, n_steps);
  } else {
    for (int64_t n = 0; n < n_steps; ++n) {
      const int rc = step_impl(h, step0 + n, nullptr, nullptr, (hipStream_t)stream);
      if (rc != ADSEQ_OK) return rc;
    }
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
  join_ahead(h, st);
  close_group(h, st, 1);
  unsigned err = 0;
  const long long T = h->next_step;
  // RING, delta synapse: the reverse sweep goes window by window where a window's spikes and near
  // events fit the staging arrays; their counts per step come back with the error word
  std::vector<int> near_counts;
  // (measured, backward ms per run with / without: cfg0, 100 state cells, 1.6 / 3.6; cfg1, 16,000,
  // 9.1 / 7.9; cfg2, 10,000 over 10,000 steps, 71 / 47; cfg3, 100,000, 21.6 / 7.1 -- the one
  // workgroup that carries the near corrections from step to step pays a chain of trips to memory
  // per step unless the whole window sits in the caches -- so by default only up to 1,024 state
  // cells; ADSEQ_RING_REVERSE_WINDOWS = 1: always, 0: never)
  const int rw = env_pow2("ADSEQ_RING_REVERSE_WINDOWS", 2, 0, 2);
  const bool by_windows = d.kind == ADSEQ_RING && d.near_ev_cap > 0 && T > 0 && (rw == 1 || (rw == 2 && d.BN <= 1024));
  if (by_windows) {
    near_counts.resize(2 * (size_t)T);
    hipLaunchKernelGGL(k_bwd_near_counts, dim3((unsigned)(T < 4096 ? T : 4096)), dim3(kBlock), 0, st, d, T, d.near_counts);
    HIP_TRY(h, hipMemcpyAsync(near_counts.data(), d.near_counts, sizeof(int) * 2 * (size_t)T, hipMemcpyDeviceToHost, st));
  }
  HIP_TRY(h, hipMemcpyAsync(&err, &d.ctr->err, sizeof(err), hipMemcpyDeviceToHost, st));
  HIP_TRY(h, hipStreamSynchronize(st));
  if (err & ERR_BARRIER)
    return fail(h, ADSEQ_E_HIP, "adseq_backward: a wait inside a resident kernel ran out (the blocks of a launch were not running together); the run is void, reset and run again");
  if (err & (ERR_TAPE_SPIKES | ERR_TAPE_EVENTS | ERR_POOL))
    return fail(h, ADSEQ_E_CAPACITY, "adseq_backward: tape or contender pool overflowed (bits %u)", err);
  // gradient per unit the delay was given in: 1/tau per ms, dt/tau per step
  // (double-exponential synapse: the 1/tau factors are in the gathered adjoint, one per state)
  const float dscale = d.alpha_r > 0.0f ? d.dt
                       : d.continuous ? (float)(1.0 / (double)d.tau) : (float)((double)d.dt / (double)d.tau);
  const dim3 block(kBlock), gn(grid_for((size_t)d.BN));
  const bool bounded = d.kind != ADSEQ_RING;
  const size_t nst = d.alpha_r > 0.0f ? 2 : 1;
  if (!bounded) {
    ring_backward_launch(h, st, T, dscale, dL_dcount, dL_dU, grad_w, grad_d, by_windows ? near_counts.data() : nullptr);
    HIP_TRY(h, hipGetLastError());
    return ADSEQ_OK;
  }
  fill_u32(st, d.bwd_carry, 0u, (size_t)d.BN);
  if (d.alpha_s > 0.0f) fill_u32(st, d.bwd_carryJ, 0u, nst * (size_t)d.BN);
  fill_u32(st, grad_w, 0u, (size_t)d.S);
  fill_u32(st, grad_d, 0u, (size_t)d.S);
  fill_u32(st, d.bwd_ring, 0u, nst * (size_t)d.R * d.BN);
  // where the spikes of every step sit on the tape (the launch grids are sized by it)
  std::vector<long long> offs((size_t)T + 1);
  HIP_TRY(h, hipMemcpyAsync(offs.data(), d.step_off, sizeof(long long) * ((size_t)T + 1), hipMemcpyDeviceToHost, st));
  HIP_TRY(h, hipStreamSynchronize(st));
  mark(h, st, -1);
  for (long long n = T - 1; n >= 0; --n) {
    const long long cnt = offs[n + 1] - offs[n];
    if (cnt > 0)
      hipLaunchKernelGGL(k_bwd_rows, dim3((unsigned)(cnt * d.fsplit)), block, 0, st, d, n, T, dscale, grad_w, grad_d,
                         offs[n]);
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
  join_ahead(h, st);
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
  out8[6] = c.tape_spikes; out8[7] = (int64_t)c.err | (h->range_warn ? (int64_t)ERR_RANGE : 0);
  if (d.kind != ADSEQ_RING) {
    // the kernels keep private counters per block: add them up here
    const size_t nb = (size_t)d.nblk + fan_slots(d.nblk) + (per_synapse_kind(d.kind) ? kSynqBlocks : 0);
    std::vector<BlkCtr> hb(nb);
    HIP_TRY(h, hipMemcpyAsync(hb.data(), d.blk, sizeof(BlkCtr) * nb, hipMemcpyDeviceToHost, st));
    HIP_TRY(h, hipStreamSynchronize(st));
    int64_t admitted = 0, sum_admitted = 0;
    for (const BlkCtr& b : hb) {
      out8[0] += (int64_t)b.offered; admitted += (int64_t)b.admitted; out8[2] += (int64_t)b.delivered;
      out8[3] += b.sum_offered; sum_admitted += b.sum_admitted; out8[5] += b.sum_delivered;
    }
    // every offered event has been admitted or refused by now (what was pending was admitted above)
    out8[1] = out8[0] - admitted;
    out8[4] = out8[3] - sum_admitted;
  }
  if (d.kind == ADSEQ_RING) {
    // spikes and offered events up to the last window boundary: private counters of the staging
    // pass's blocks; since then: c.fold
    std::vector<BlkCtr> hb(kMaxBinBlocks);
    HIP_TRY(h, hipMemcpyAsync(hb.data(), d.blk, sizeof(BlkCtr) * kMaxBinBlocks, hipMemcpyDeviceToHost, st));
    HIP_TRY(h, hipStreamSynchronize(st));
    for (const BlkCtr& b : hb) { out8[6] += b.pad[0]; out8[0] += (int64_t)b.offered; out8[3] += b.sum_offered; }
    out8[6] += (int64_t)c.fold[0]; out8[0] += (int64_t)c.fold[1]; out8[3] += (int64_t)c.fold[2];
    out8[2] = out8[0] - (int64_t)c.in_flight[0];
    out8[5] = out8[3] - (int64_t)c.in_flight[1];
    if (d.count_pop) {
      // counted instead of derived: what the step kernels popped, cell by cell
      int64_t popped = 0;
      for (const BlkCtr& b : hb) popped += b.sum_delivered;
      out8[5] = popped;
    }
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
  if (c[7] & ERR_BARRIER)
    return fail(h, ADSEQ_E_HIP, "a wait inside a resident kernel ran out; the run is void");
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

#ifdef ADSEQ_PHASE_CLOCK
// Builds with phase clocks only (python -m paper_2512_05906_amd.build --phase-clocks; not part of
// the C ABI): the 24 tick counters (10 ns each) of the phases, see Counters.
int adseq_debug_phase_clocks(adseq_t* h, uint64_t* out24, void* stream) {
  if (!h || !out24) return ADSEQ_E_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (hipMemcpyAsync(out24, h->dev.ctr->phase, sizeof(unsigned long long) * 24, hipMemcpyDeviceToHost, st) != hipSuccess) return ADSEQ_E_HIP;
  return hipStreamSynchronize(st) == hipSuccess ? ADSEQ_OK : ADSEQ_E_HIP;
}
// The block spans of the last staging, accumulation and far gather launch: out[3][512][2] ticks.
int adseq_debug_block_spans(adseq_t* h, uint64_t* out, void* stream) {
  if (!h || !out) return ADSEQ_E_INVALID_ARG;
  hipStream_t st = (hipStream_t)stream;
  if (hipMemcpyAsync(out, h->dev.ctr->span, sizeof(unsigned long long) * 3 * 512 * 2, hipMemcpyDeviceToHost, st) != hipSuccess) return ADSEQ_E_HIP;
  return hipStreamSynchronize(st) == hipSuccess ? ADSEQ_OK : ADSEQ_E_HIP;
}
#endif

}  // extern "C"
