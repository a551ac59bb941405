// Ring queue (ADSEQ_RING) as a windowed delay line.  Included by adseq.hip inside its
// anonymous namespace, after Dev and the device helpers.
//
// Time is cut into windows of W steps (W a power of two).  The queue state is
//   win        i32 [2][W][BN] Q8.24 sums of the events that arrive inside the current window
//                            (buffer (n / W) & 1) and, being prepared, inside the next one,
//   spike_bits u64 [R][words] the spikes of the last R = d_max + 1 steps,
// and the synapse rows, re-ordered at create so that every row is ascending in its arrival
// offset D, with dstart[i][D] = position in row i of the first entry with offset >= D.
// An event emitted at step n with offset D arrives at n + D:
//   * if that is still inside n's window, the step kernel adds it to win at once (a few
//     per cent of the events: offsets 1 .. W - 1 - (n mod W), the front of the sorted row);
//   * otherwise it stays implicit -- (spike bit, sorted row) -- until the window that holds
//     n + D begins.  Then one expansion pass walks the spikes of the last d_max steps; for a
//     spike at step n the entries that land in window [k0, k0 + W) are the contiguous piece
//     D in [k0 - n, k0 - n + W) of its row, read with full-width loads.
// The expansion does not scatter with one memory-side atomic per event.  It stages the events
// by target range ("part") into per-(part, block) regions of a buffer (LDS cursors, no global
// atomics; a block first orders a chunk of its events by part in LDS, so that a region receives
// runs of consecutive events instead of one scattered store per event); then every part is given
// to one workgroup, which sums the part's events into an LDS
// tile [W][targets of the part] with LDS atomics and adds the tile to win with coalesced
// accesses.  Events that do not fit their region fall back to a global atomic on win, so the
// result never depends on the staging capacity.
// Both passes run once per window, at its first step, on all spikes of the last d_max steps.
// The first pass also counts the spikes of the window just finished, and the events they emit,
// into the device counters (the step kernel itself counts nothing).  Two window buffers, used
// alternately, so that the cells a window's steps clear are not the ones being filled for the
// next.  (Measured and dropped: expanding the next window's old spikes on a second stream, or
// in slices riding as extra blocks on the step launches -- the loaded memory system slows the
// latency-bound step kernels by as much as is gained.)
//
// The reverse sweep mirrors it: gwin f32 [2][W][BN] holds the adjoint rows of the current
// window.  A spike's queue term is the sum of a near part (gathered by the step kernel) and one
// far part per later window, gathered by k_bwd_win from the window (6.4 MB: the L2 holds it) into
// Gacc[n mod R][g].  The per-synapse sum of gathered adjoints goes to gsum in sorted order and is
// scaled and un-permuted into grad_w / grad_d by k_grad_finish.

constexpr int kRingThreads = 1024;  // threads per block of the ring's step and expansion kernels
constexpr int kRingWaves = kRingThreads / 64;
constexpr int kMaxTileCells = 16384; // cells (target, row) of the largest LDS tile = 64 KB
constexpr int kMaxParts = 4096;     // LDS cursors of k_win_bin; targets beyond them use atomics
constexpr int kMaxBinBlocks = 512;

// ---------------------------------------------------------------- create: sorted rows

// Arrival offset, Q8.24 amplitude, fp32 amplitude and decay factor of synapse p.
struct Syn { int D; int a_q; float amp; float f; unsigned err; };

__device__ __forceinline__ Syn syn_prepare(const Dev& d, const ExpCoef& ec, long long p) {
  Syn s; s.err = 0;
  const double w = (double)d.weight[p];
  double f = 1.0;
  long long D;
  if (!d.continuous) {
    D = d.delay_steps[p];
    if (D < 1) { s.err |= ERR_DELAY; D = 1; }
  } else {
    const double dt = (double)d.dt, tau = (double)d.tau;
    const double dl = (double)d.delay_ms[p];
    if (!(dl > 0.0)) s.err |= ERR_DELAY;
    const double q = ceil(dl / dt);
    D = (q >= 1.0 && q < 1e9) ? (long long)q : 1;
    const double x = ((double)D * dt - dl) / tau;
    if (!(x >= 0.0 && x <= 1.0)) s.err |= ERR_DELAY;
    const double y = -x;
    double r = ec.c[20];
    for (int k = 19; k >= 0; --k) r = __fma_rn(r, y, ec.c[k]);
    f = r;
  }
  if (D > d.d_max) { s.err |= ERR_DELAY; D = d.d_max; }
  const double a = w * f;
  long long q = __double2ll_rn(a * 16777216.0);
  q = q > 2147483647LL ? 2147483647LL : (q < -2147483648LL ? -2147483648LL : q);
  s.D = (int)D; s.a_q = (int)q; s.amp = (float)a; s.f = (float)f;
  return s;
}

// row_ptr: starts at 0, ends at S, never decreases, rows shorter than 2^31.  Runs before any
// kernel that walks the rows.
__global__ __launch_bounds__(kBlock) void k_check_rows(Dev d) {
  for (long long i = (long long)blockIdx.x * kBlock + threadIdx.x; i < d.N;
       i += (long long)gridDim.x * kBlock) {
    const long long a = d.row_ptr[i], b = d.row_ptr[i + 1];
    bool bad = a > b || a < 0 || b > d.S || b - a > 0x7fffffffLL;
    if (i == 0 && a != 0) bad = true;
    if (i == d.N - 1 && b != d.S) bad = true;
    if (bad) atomicOr(&d.ctr->err, ERR_GRAPH);
  }
}

// One block per row: counting sort of the row by arrival offset.  Writes the sorted synapse
// arrays (synf = {packed, Q8.24 amplitude} for the forward pass, synb = {packed, fp32 amplitude}
// for the reverse sweep, fdec), perm (sorted position -> position in the caller's row),
// dstart, nearcnt and the row's Q8.24 amplitude sum.
__global__ __launch_bounds__(kBlock) void k_sort_rows(Dev d, ExpCoef ec) {
  __shared__ unsigned s_hist[1026];
  __shared__ unsigned s_part[kBlock];
  __shared__ long long s_sum[kBlock / 64];
  const int nb = d.d_max + 2;  // offsets 0 .. d_max + 1
  for (long long i = blockIdx.x; i < d.N; i += gridDim.x) {
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    for (int k = threadIdx.x; k < nb; k += kBlock) s_hist[k] = 0;
    __syncthreads();
    unsigned err = 0;
    for (long long p = r0 + threadIdx.x; p < r1; p += kBlock) {
      const Syn s = syn_prepare(d, ec, p);
      err |= s.err;
      const int c = d.col[p];
      if (c < 0 || c >= d.N) err |= ERR_GRAPH;
      atomicAdd(&s_hist[s.D], 1u);
    }
    if (err) atomicOr(&d.ctr->err, err);
    __syncthreads();
    // exclusive scan of s_hist[0 .. nb): thread t owns the K consecutive bins from t * K
    const int K = (nb + kBlock - 1) / kBlock;
    unsigned loc = 0;
    for (int k = 0; k < K; ++k) { const int x = threadIdx.x * K + k; if (x < nb) loc += s_hist[x]; }
    s_part[threadIdx.x] = loc;
    __syncthreads();
    if (threadIdx.x < 64) {
      // 256 partial sums, 4 per lane of the first wavefront
      unsigned v[4], t = 0;
      for (int k = 0; k < 4; ++k) { v[k] = s_part[threadIdx.x * 4 + k]; t += v[k]; }
      unsigned inc = t;
      for (int o = 1; o < 64; o <<= 1) { const unsigned u = __shfl_up(inc, o, 64); if ((int)threadIdx.x >= o) inc += u; }
      unsigned run = inc - t;
      for (int k = 0; k < 4; ++k) { s_part[threadIdx.x * 4 + k] = run; run += v[k]; }
    }
    __syncthreads();
    unsigned run = s_part[threadIdx.x];
    for (int k = 0; k < K; ++k) {
      const int x = threadIdx.x * K + k;
      if (x < nb) { const unsigned c = s_hist[x]; s_hist[x] = run; run += c; }
    }
    __syncthreads();
    for (int k = threadIdx.x; k < nb; k += kBlock) d.dstart[(size_t)i * nb + k] = s_hist[k];
    for (int h = threadIdx.x; h <= d.W; h += kBlock) {
      const int x = h + 1 < nb - 1 ? h + 1 : nb - 1;       // entries with offset <= h
      d.nearcnt[(size_t)h * d.N + i] = s_hist[x];
    }
    __syncthreads();
    long long sum = 0;
    for (long long p = r0 + threadIdx.x; p < r1; p += kBlock) {
      const Syn s = syn_prepare(d, ec, p);
      int c = d.col[p];
      if (c < 0 || c >= d.N) c = 0;
      const long long q = r0 + atomicAdd(&s_hist[s.D], 1u);
      const unsigned pk = ((unsigned)c << d.dbits) | (unsigned)s.D;
      d.synf[q] = make_uint2(pk, (unsigned)s.a_q);
      d.synb[q] = make_uint2(pk, __float_as_uint(s.amp));
      if (d.continuous) d.fdec[q] = s.f;
      d.perm[q] = (unsigned)(p - r0);
      sum += s.a_q;
    }
    sum = wave_sum(sum);
    if ((threadIdx.x & 63) == 0) s_sum[threadIdx.x >> 6] = sum;
    __syncthreads();
    if (threadIdx.x == 0) {
      long long t = 0;
      for (int w = 0; w < kBlock / 64; ++w) t += s_sum[w];
      d.rowsum[i] = t;
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------- forward: one launch per step

// Window buffer that holds arrival step k.
__device__ __forceinline__ int* win_of(const Dev& d, long long k) {
  return d.win + (size_t)((k >> d.wshift) & 1) * d.W * d.BN;
}
__device__ __forceinline__ float* gwin_of(const Dev& d, long long k) {
  return d.gwin + (size_t)((k >> d.wshift) & 1) * d.W * d.BN;
}

// Adds the entries [0, cnt) of the sorted row at pr0 (arrival offsets 1 .. W - 1 - phi) of a
// spike of trial base / N to the rows phi + D of the window.  Whole wavefront.
__device__ __forceinline__ void near_scatter(const Dev& d, int* __restrict__ win, int phi, long long pr0,
                                             unsigned cnt, int base) {
  const int lane = threadIdx.x & 63;
  for (unsigned q = lane; q < cnt; q += 64) {
    const uint2 e = d.synf[pr0 + q];
    const int D = (int)(e.x & d.dmask);
    atomicAdd(&win[(size_t)(phi + D) * d.BN + (size_t)base + (e.x >> d.dbits)], (int)e.y);
  }
}

// Checking aid (count_pop): adds the wavefront's sum of the Q8.24 values it has popped to a
// private counter line of the block.  The ring's delivered counters are otherwise derived from the
// spikes (offered minus still in flight); this one is counted cell by cell, so a lost add shows.
// Every lane of the wavefront must call it.
__device__ __forceinline__ void count_popped(const Dev& d, long long v) {
  const long long t = wave_sum(v);
  if ((threadIdx.x & 63) == 0 && t) atomicAdd((unsigned long long*)&d.blk[blockIdx.x & (kMaxBinBlocks - 1)].sum_delivered, (unsigned long long)t);
}

// One launch per time step.  Block b owns neurons [256 b, 256 b + 256): pops their cells of
// row phi = n mod W, adds the drive, integrates, records the membrane value and the spike bits,
// and scatters the in-window events of its own spikes.  No block-level synchronisation and no
// counter: spikes and offered events are counted from the spike bits when a window closes.
// SYN: synaptic current states (0: the jumps go into the membrane, 1: first-order synapse, 2: double-
// exponential synapse, the slow and the fast state both take the jump and the current is their difference)
// MODE 1: the checking aid count_popped (a template parameter, so that the kernel that is timed reads
// nothing more of its argument block than it did).  MODE 2: row start and in-window count are
// fetched by the spiking lanes only (12 bytes per neuron less HBM traffic, one more memory round
// trip between the spike and its fan-out).
template <bool RECORD, int SYN, int MODE>
__global__ __launch_bounds__(kBlock) void k_step_win(long long n, const float* __restrict__ i_ext,
                                                     unsigned char* __restrict__ spikes_out, Dev d) {
  pin_args(d.win, d.V, d.row_ptr, d.nearcnt, d.tapeU, d.spk_count, d.spike_bits, d.tape_bits, d.synf, d.J,
           d.N, d.B, d.BN, d.W, d.wshift, d.d_max, d.R, d.words, d.dbits, d.dmask, d.alpha, d.theta,
           d.v_reset, d.ext_w, d.alpha_s, d.alpha_r, d.p_thresh, d.seed, n, i_ext, spikes_out);
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  const int phi = (int)(n & (long long)(d.W - 1));
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  int b = 0;
  bool s = false;
  long long r0 = 0;
  unsigned ncnt = 0;
  int popped = 0;
  int* __restrict__ win = win_of(d, n);
  if (act) {
    b = trial_of(d, g);
    const int i = g - b * d.N;
    const size_t idx = (size_t)phi * d.BN + g;
    const int acc = win[idx];
    popped = acc;
    // row start and in-window entry count of every neuron, loaded beside the pop so that a
    // spiking neuron's fan-out does not wait for them (both arrays stay in the L2)
    if (MODE != 2) {
      r0 = d.row_ptr[i];
      if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
    }
    const float v = d.V[g];
    const float jsyn = SYN ? d.J[g] : 0.0f;
    const float jfast = SYN == 2 ? d.J[(size_t)d.BN + g] : 0.0f;
    if (acc != 0) win[idx] = 0;
    float I = (float)acc * 0x1p-24f;
    if (SYN) {   // the jumps go into the synaptic current state(s)
      const float jump = I;
      I = __fmaf_rn(d.alpha_s, jsyn, jump);
      d.J[g] = I;
      if (SYN == 2) {
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
    if (MODE == 2 && s) {
      r0 = d.row_ptr[i];
      if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
    }
    // state and tape are written once per launch and not read again by it: non-temporal stores
    // leave no dirty lines behind for the end of the kernel to write back (2^20 cells: 8.8 -> 7.6 us)
    __builtin_nontemporal_store(s ? d.v_reset : U, &d.V[g]);
    if (RECORD) {
      __builtin_nontemporal_store(U, &d.tapeU[(size_t)n * d.BN + g]);
      if (s) atomicAdd(&d.spk_count[g], 1);   // no return value: the wavefront does not wait for it
    }
    if (spikes_out) spikes_out[g] = s ? 1 : 0;
  }
  const unsigned long long bits = __ballot(s);
  if ((threadIdx.x & 63) == 0) {
    const size_t word = (size_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    d.spike_bits[(size_t)(n % d.R) * d.words + word] = bits;
    if (RECORD) d.tape_bits[(size_t)n * d.words + word] = bits;
  }
  if (MODE == 1) count_popped(d, popped);
  // in-window events of the wavefront's spikes, up to four spikes at a time: the row loads of all
  // four are in flight before the first atomic, so that a wavefront with several spikes does not
  // pay one memory round trip per spike
  unsigned long long m = __ballot(s && ncnt > 0);
  const int lane = threadIdx.x & 63;
  while (m) {
    long long pr[4]; unsigned cn[4]; int bs[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      pr[j] = 0; cn[j] = 0; bs[j] = 0;
      if (m) {
        const int L = __ffsll((long long)m) - 1;
        m &= m - 1;
        pr[j] = lane_get(r0, L); cn[j] = lane_get(ncnt, L); bs[j] = lane_get(b, L) * d.N;
      }
    }
    uint2 e[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      e[j] = make_uint2(0u, 0u);
      if ((unsigned)lane < cn[j]) e[j] = d.synf[pr[j] + lane];
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if ((unsigned)lane < cn[j])
        atomicAdd(&win[(size_t)(phi + (int)(e[j].x & d.dmask)) * d.BN + (size_t)bs[j] + (e[j].x >> d.dbits)], (int)e[j].y);
      if (cn[j] > 64u) near_scatter(d, win, phi, pr[j] + 64, cn[j] - 64u, bs[j]);   // rows with many in-window entries
    }
  }
}

// Open-loop pop of row phi: writes the delivered current, clears the cells and this step's
// spike bits (adseq_enqueue sets them).
__global__ __launch_bounds__(kBlock) void k_deliver_win(Dev d, long long n, float* __restrict__ I_out) {
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const int phi = (int)(n & (long long)(d.W - 1));
  int* __restrict__ win = win_of(d, n);
  int popped = 0;
  if (g < d.BN) {
    const size_t idx = (size_t)phi * d.BN + g;
    const int acc = win[idx];
    popped = acc;
    if (acc != 0) win[idx] = 0;
    I_out[g] = (float)acc * 0x1p-24f;
  }
  if (d.count_pop) count_popped(d, popped);
  if ((threadIdx.x & 63) == 0)
    d.spike_bits[(size_t)(n % d.R) * d.words + (size_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)] = 0ull;
}

// Open-loop enqueue of the listed spikes at step n: one wavefront per spike sets its bit and
// scatters its in-window events; everything else stays implicit until its window begins.
__global__ __launch_bounds__(kBlock) void k_enqueue_win(Dev d, long long n, const int* __restrict__ spk,
                                                        const int* __restrict__ n_spk_ptr) {
  int nspk = *n_spk_ptr;
  nspk = nspk < 0 ? 0 : (nspk > d.BN ? d.BN : nspk);
  const int phi = (int)(n & (long long)(d.W - 1));
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6, nwaves = (gridDim.x * kBlock) >> 6;
  for (int e = wave; e < nspk; e += nwaves) {
    const int g = spk[e];
    if ((unsigned)g >= (unsigned)d.BN) continue;  // uniform over the wavefront
    const int b = trial_of(d, g), i = g - b * d.N;
    if (lane == 0) atomicOr(&d.spike_bits[(size_t)(n % d.R) * d.words + (g >> 6)], 1ull << (g & 63));
    if (near_h >= 1)
      near_scatter(d, win_of(d, n), phi, d.row_ptr[i], d.nearcnt[(size_t)near_h * d.N + i], b * d.N);
  }
}

// Open loop, pop and enqueue of one step in ONE launch (adseq_run_open knows both): block b pops
// its 256 cells of row phi as k_deliver_win does, then the wavefronts share out the listed spikes
// as in k_enqueue_win (their events go to later rows of the window, so the two parts never touch
// the same cell).  The spike words being set are those of slot n mod R; nobody may clear them in
// the same launch, so every launch clears the words of the NEXT step's slot instead (the host
// clears this step's slot itself when the launch before was not one of these).
__global__ __launch_bounds__(kBlock) void k_open_step_win(Dev d, long long n, const int* __restrict__ spk,
                                                          const int* __restrict__ n_spk_ptr,
                                                          float* __restrict__ I_out) {
  int nspk = *n_spk_ptr;
  nspk = nspk < 0 ? 0 : (nspk > d.BN ? d.BN : nspk);
  const int g0 = blockIdx.x * kBlock + threadIdx.x;
  const int phi = (int)(n & (long long)(d.W - 1));
  int* __restrict__ win = win_of(d, n);
  int popped = 0;
  if (g0 < d.BN) {
    const size_t idx = (size_t)phi * d.BN + g0;
    const int acc = win[idx];
    popped = acc;
    if (acc != 0) win[idx] = 0;
    I_out[g0] = (float)acc * 0x1p-24f;
  }
  if (d.count_pop) count_popped(d, popped);
  if ((threadIdx.x & 63) == 0 && blockIdx.x < d.nblk)
    d.spike_bits[(size_t)((n + 1) % d.R) * d.words + (size_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)] = 0ull;
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  const int lane = threadIdx.x & 63;
  const int wave = (blockIdx.x * kBlock + threadIdx.x) >> 6, nwaves = (gridDim.x * kBlock) >> 6;
  for (int e = wave; e < nspk; e += nwaves) {
    const int g = spk[e];
    if ((unsigned)g >= (unsigned)d.BN) continue;  // uniform over the wavefront
    const int b = trial_of(d, g), i = g - b * d.N;
    if (lane == 0) atomicOr(&d.spike_bits[(size_t)(n % d.R) * d.words + (g >> 6)], 1ull << (g & 63));
    if (near_h >= 1)
      near_scatter(d, win, phi, d.row_ptr[i], d.nearcnt[(size_t)near_h * d.N + i], b * d.N);
  }
}

// ---------------------------------------------------------------- forward: window expansion

// Phase clocks of the expansion (builds with ADSEQ_PHASE_CLOCK only): thread 0 of block 0 adds the
// 10 ns ticks since the last mark to Counters::phase[i].
#ifdef ADSEQ_PHASE_CLOCK
#define XPH_BEGIN unsigned long long xpt = wall_clock64();
#define XPH_ARG , unsigned long long& xpt
#define XPH_PASS , xpt
#define XPH(i) { if (blockIdx.x == 0 && threadIdx.x == 0) { const unsigned long long t_ = wall_clock64(); d.ctr->phase[i] += t_ - xpt; xpt = t_; } }
#define XPH_COUNT(i) { if (blockIdx.x == 0 && threadIdx.x == 0) d.ctr->phase[i] += 1; }
#define XPH_SPAN(k, e) { if (threadIdx.x == 0 && blockIdx.x < 512) d.ctr->span[k][blockIdx.x][e] = wall_clock64(); }
#else
#define XPH_BEGIN
#define XPH_ARG
#define XPH_PASS
#define XPH(i) {}          // (empty blocks, so that a mark after an `if` never leaves the next statement under it)
#define XPH_COUNT(i) {}
#define XPH_SPAN(k, e) {}
#endif

// Streaming loads of the expansion and gather passes (row pieces and staged events are read
// once per pass): non-temporal, so that they do not push the window out of the L2.  (The staging
// stores stay ordinary: as non-temporal 8-byte stores they reach memory one by one, 2.6x slower.)
// Also what the resident kernels read a row's later entries with: ONE 8-byte load (written as
// `const uint2 e = row[i]` with e.y used only under a test of e.x, the compiler loads the two halves
// one after the other, the second behind the test: two trips to memory for one).
__device__ __forceinline__ uint2 load_stream(const uint2* p) {
  const unsigned long long v = __builtin_nontemporal_load(reinterpret_cast<const unsigned long long*>(p));
  return make_uint2((unsigned)v, (unsigned)(v >> 32));
}

// The piece of one spike's sorted row that lands in the window being expanded.
struct Seg { long long p0; int len; int base; int dlo; int slot; long long g; };
constexpr int kSegQueue = 768;   // queue entries per block (32 B each)

// LDS of a block of an expansion / gather role.
struct ExpandLds {
  int cur[kMaxParts];        // staging cursors of k_win_bin's parts
  Seg q[kSegQueue];          // segments found by the walk, shared out among the wavefronts
  int qn, qhead, qlen;       // queued pieces, next to hand out, events in the queued pieces
  long long red[3][kRingWaves];
};
static_assert(sizeof(ExpandLds) <= kMaxTileCells * 4, "roles share one LDS buffer");

// One far event of the window: staged in region (part, vb) if there is room, else added to
// win with a global atomic.
__device__ __forceinline__ void stage_event(const Dev& d, int* __restrict__ win, int* s_cur, int nparts,
                                            int vb, unsigned pk, int a, int dlo, int base) {
  const int r = (int)(pk & d.dmask) - dlo;             // row of the window, 0 .. W - 1
  const int gt = base + (int)(pk >> d.dbits);
  const int part = gt >> d.tp_shift;
  if (part < nparts) {
    const int pos = atomicAdd(&s_cur[part], 1);
    if (pos < d.cap) {
      d.ebuf[((size_t)part * d.NB + vb) * d.cap + pos] =
          make_uint2((unsigned)((r << d.tp_shift) | (gt & ((1 << d.tp_shift) - 1))), (unsigned)a);
      return;
    }
  }
  atomicAdd(&win[(size_t)r * d.BN + gt], a);
}

// A wavefront's share of a walk over the spike words of steps [n_lo, n_hi): the words of a step
// are cut into lines of 8 (64 bytes); the line numbered c = gw + nwaves * (8 t + group) belongs
// to the 8-lane group `group` of wavefront gw in trip t, so that lines are dealt round-robin over
// all wavefronts and one wavefront sees up to 8 lines of different steps at once.  A lane keeps
// its line as (step index si, line of the step rem) and moves on by a fixed stride per trip, so
// the walk divides once per lane and not once per trip.
struct WalkPos {
  long long si;   // step n_lo + si
  int rem;        // line of that step, 0 .. lps - 1
};
__device__ __forceinline__ void walk_advance(WalkPos& p, long long dq, int dr, int lps) {
  p.si += dq;
  p.rem += dr;
  if (p.rem >= lps) { p.rem -= lps; p.si += 1; }
}

// Walks the spike words of steps [n_lo, n_hi) as virtual block vb of nvb (16 wavefronts each)
// and, for every spike, looks up the piece of its sorted row with arrival offsets
// [k0 - n, k0 - n + W) (cut at arrival T when T >= 0; from offset 1 for a spike at a step n >= k0,
// whose piece is the front of its row) and appends it to the block's LDS queue;
// handle(seg) is called instead when the queue is full.  Spikes of steps >= count_from are
// counted into cnt[3] (spikes, their events, Q8.24 sum of those).  Ends with a block barrier.
template <class Direct>
__device__ __forceinline__ void walk_segments(const Dev& d, ExpandLds& L, const unsigned long long* __restrict__ words,
                                              bool circular, long long k0, long long n_lo, long long n_hi,
                                              long long T, int vb, int nvb, long long count_from,
                                              long long* cnt, Direct handle) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const long long gw = vb + (long long)nvb * wv;   // blocks interleaved: every block sees every step
  const long long nwaves = (long long)nvb * kRingWaves;
  const int lps = (d.words + 7) >> 3;                   // lines per step
  const long long nsteps = n_hi - n_lo;                  // at most d_max + 1 <= R
  const long long nlines = nsteps * lps;
  const int nb = d.d_max + 2;
  // this lane's first line, the stride of a trip (the same for every lane), and the row of the
  // circular spike words that holds step n_lo
  WalkPos pos;
  {
    const long long c = gw + nwaves * (lane >> 3);
    pos.si = c / lps;
    pos.rem = (int)(c - pos.si * lps);
  }
  const long long stride = nwaves * 8;
  const long long dq = stride / lps;
  const int dr = (int)(stride - dq * lps);
  const int slot_lo = (int)(n_lo % d.R);
  // four trips' words are requested before the first is looked at
  for (long long c00 = gw; c00 < nlines; c00 += stride * 4) {
    unsigned long long bw[4]; long long nn[4]; int ww[4], sl[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      bw[j] = 0ull; nn[j] = n_lo; ww[j] = 0; sl[j] = slot_lo;
      if (pos.si < nsteps) {   // (a trip past the end gives no word)
        nn[j] = n_lo + pos.si;
        ww[j] = pos.rem * 8 + (lane & 7);
        int slot = slot_lo + (int)pos.si;
        while (slot >= d.R) slot -= d.R;   // (a walk may span up to d_max + W steps)
        sl[j] = slot;
        if (ww[j] < d.words) bw[j] = words[(size_t)(circular ? (long long)slot : nn[j]) * d.words + ww[j]];
      }
      walk_advance(pos, dq, dr, lps);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      unsigned long long bits = bw[j];
      const long long n = nn[j];
      const int word = ww[j];
      const int dlo = (int)(k0 - n);                      // 1 .. d_max; <= 0 for a spike inside the window itself
      int dhi = dlo + d.W < nb - 1 ? dlo + d.W : nb - 1;
      if (T >= 0) {
        if ((long long)dhi > T - n) dhi = (int)(T - n);   // arrivals n + D >= T are never delivered
        if (dhi < dlo) dhi = dlo;
      }
      const bool counted = n >= count_from;
      while (__ballot(bits != 0ull)) {
        // every lane that still has a spike takes its lowest one
        Seg sg; sg.p0 = 0; sg.len = 0; sg.base = 0; sg.dlo = dlo; sg.slot = sl[j]; sg.g = 0;
        if (bits) {
          const int bit = __ffsll((long long)bits) - 1;
          bits &= bits - 1;
          const long long g = (long long)word * 64 + bit;
          if (g < d.BN) {
            const int b = trial_of(d, (int)g), i = (int)g - b * d.N;
            const unsigned* ds = d.dstart + (size_t)i * nb;
            // all loads of the spike are requested before the first is used
            const unsigned q0 = ds[dlo > 0 ? dlo : 0], q1 = ds[dhi];
            const long long r0 = d.row_ptr[i];
            // (the row's length and sum are loaded for every spike, counted or not: under a branch
            // of their own they would be a second round trip to memory)
            const long long r1 = d.row_ptr[i + 1], rs = d.rowsum[i];
            sg.p0 = r0 + q0; sg.len = (int)(q1 - q0); sg.base = b * d.N; sg.g = g;
            cnt[0] += counted ? 1 : 0; cnt[1] += counted ? r1 - r0 : 0; cnt[2] += counted ? rs : 0;
          }
        }
        const bool has = sg.len > 0;
        const unsigned long long mask = __ballot(has);
        if (mask) {
          int pos = 0;
          if (lane == 0) pos = atomicAdd(&L.qn, __popcll(mask));
          pos = __builtin_amdgcn_readfirstlane(pos) + __popcll(mask & ((1ull << lane) - 1ull));
          if (has && pos < kSegQueue) L.q[pos] = sg;
          unsigned long long ovf = __ballot(has && pos >= kSegQueue);
          while (ovf) {
            const int src = __ffsll((long long)ovf) - 1;
            ovf &= ovf - 1;
            Seg o;
            o.p0 = __shfl(sg.p0, src, 64); o.len = __shfl(sg.len, src, 64); o.base = __shfl(sg.base, src, 64);
            o.dlo = __shfl(sg.dlo, src, 64); o.slot = __shfl(sg.slot, src, 64); o.g = __shfl(sg.g, src, 64);
            handle(o);
          }
        }
      }
    }
  }
  __syncthreads();
}

// Adds the block's totals of cnt[0..3) (spikes, their events, Q8.24 sum of those) to the private
// counters of virtual block vb: 256 blocks adding to three shared addresses would queue up behind
// one another at the end of the pass.
__device__ __forceinline__ void fold_counts(const Dev& d, ExpandLds& L, long long* cnt, int vb) {
  for (int k = 0; k < 3; ++k) {
    const long long v = wave_total64(cnt[k]);
    if ((threadIdx.x & 63) == 0) L.red[k][threadIdx.x >> 6] = v;
  }
  __syncthreads();
  if (threadIdx.x < 3) {
    const int k = threadIdx.x;
    long long t = 0;
    for (int w = 0; w < kRingWaves; ++w) t += L.red[k][w];
    BlkCtr& bc = d.blk[vb & (kMaxBinBlocks - 1)];
    unsigned long long* dst = k == 0 ? (unsigned long long*)&bc.pad[0]
                            : k == 1 ? &bc.offered : (unsigned long long*)&bc.sum_offered;
    if (t) atomicAdd(dst, (unsigned long long)t);
  }
}

// LDS of the ordered staging (role_bin with stage = 2): the block's events are taken in chunks
// of kSortChunk, ordered by target part in LDS (counting sort) and written to the staging regions
// as runs of consecutive events, instead of one scattered 8-byte store per event.
constexpr int kSortParts = 512;     // parts the ordered staging handles
constexpr int kSortChunk = 8192;    // events per chunk = 8 per thread
struct SortLds {
  int cnt[kSortParts];              // events of the chunk per part (zero between chunks)
  int base[kSortParts + 1];         // exclusive prefix of cnt: the part's first position in ev
  int g0[kSortParts];               // the part's first free position of its staging region
  int off[kSegQueue + 1];           // exclusive prefix of the queued pieces' lengths
  int map[kSortChunk / 64];         // piece that holds the first event of each 64-event group of the chunk
  int scan[kRingWaves];
  uint2 ev[kSortChunk];
};

// Exclusive prefix of v over the block's threads (total in *total).  Two block barriers.
__device__ __forceinline__ int block_scan_excl(int v, int* s_w, int* total) {
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int x = dpp_scan_add(v);
  if (lane == 63) s_w[wv] = x;
  __syncthreads();
  int add = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < kRingWaves; ++w) {
    const int c = s_w[w];
    if (w < wv) add += c;
    tot += c;
  }
  __syncthreads();
  *total = tot;
  return add + x - v;
}

// Ordered staging of the pieces L.q[0, qn): see SortLds.  L.cur[part] stays the cursor of the
// part's staging region (the pieces that overflowed the queue during the walk used it too).
__device__ __forceinline__ void stage_sorted(const Dev& d, ExpandLds& L, SortLds& S, int* __restrict__ win,
                                             int nparts, int vb, int qn XPH_ARG) {
  const int t = threadIdx.x;
  int total = 0;
  {
    const int len = t < qn ? L.q[t].len : 0;
    const int ex = block_scan_excl(len, S.scan, &total);
    if (t < qn) S.off[t] = ex;
    if (t == 0) S.off[qn] = total;
    if (t < kSortParts) S.cnt[t] = 0;
  }
  __syncthreads();
  XPH(2)
  const unsigned lmask = (1u << d.tp_shift) - 1u;
  constexpr int kPer = kSortChunk / kRingThreads;
  for (int c0 = 0; c0 < total; c0 += kSortChunk) {
    const int cend = c0 + kSortChunk < total ? c0 + kSortChunk : total;
    // every piece enters itself for the 64-event groups of the chunk that start inside it
    if (t < qn) {
      const int p_lo = S.off[t], p_hi = S.off[t + 1] < cend ? S.off[t + 1] : cend;
      int b = ((p_lo > c0 ? p_lo : c0) + 63) >> 6;
      for (; (b << 6) < p_hi; ++b) S.map[b - (c0 >> 6)] = t;
    }
    __syncthreads();
    XPH(2)
    // A: this thread's events of the chunk (all row entries requested before the first is used):
    // piece, row entry, part, rank within (chunk, part)
    uint2 e[kPer]; int dlo[kPer], tb[kPer];
#pragma unroll
    for (int m = 0; m < kPer; ++m) {
      const int x = c0 + m * kRingThreads + t;
      e[m] = make_uint2(0u, 0u); dlo[m] = 0; tb[m] = -1;
      if (x < cend) {
        int lo = S.map[(x - c0) >> 6];
        while (x >= S.off[lo + 1]) ++lo;
        const Seg& o = L.q[lo];
        dlo[m] = o.dlo; tb[m] = o.base;
        e[m] = load_stream(&d.synf[o.p0 + (x - S.off[lo])]);
      }
    }
    unsigned w0[kPer]; int pr[kPer];   // staged word | part << 16, rank
#pragma unroll
    for (int m = 0; m < kPer; ++m) {
      w0[m] = 0u; pr[m] = -1;
      if (tb[m] >= 0) {
        const int r = (int)(e[m].x & d.dmask) - dlo[m];
        const int gt = tb[m] + (int)(e[m].x >> d.dbits);
        const int part = gt >> d.tp_shift;
        if (part < nparts) {
          w0[m] = ((unsigned)part << 16) | ((unsigned)r << d.tp_shift) | ((unsigned)gt & lmask);
          pr[m] = atomicAdd(&S.cnt[part], 1);
        } else {
          atomicAdd(&win[(size_t)r * d.BN + gt], (int)e[m].y);
        }
      }
    }
    __syncthreads();
    XPH(3)
    // B: positions of the parts in the chunk and in their staging regions
    {
      const int c = t < nparts ? S.cnt[t] : 0;
      int tot;
      const int ex = block_scan_excl(c, S.scan, &tot);
      if (t < nparts) {
        S.base[t] = ex;
        S.g0[t] = L.cur[t];
        L.cur[t] += c;
        S.cnt[t] = 0;
      }
      if (t == 0) S.base[nparts] = tot;
    }
    __syncthreads();
    XPH(4)
    // C: order the chunk by part
#pragma unroll
    for (int m = 0; m < kPer; ++m)
      if (pr[m] >= 0) S.ev[S.base[w0[m] >> 16] + pr[m]] = make_uint2(w0[m], e[m].y);
    __syncthreads();
    XPH(5)
    // D: write the runs
    const int staged = S.base[nparts];
    for (int x = t; x < staged; x += kRingThreads) {
      const uint2 e = S.ev[x];
      const int part = (int)(e.x >> 16);
      const unsigned word = e.x & 0xffffu;
      const int pos = S.g0[part] + (x - S.base[part]);
      if (pos < d.cap) {
        d.ebuf[((size_t)part * d.NB + vb) * d.cap + pos] = make_uint2(word, e.y);
      } else {
        const int r = (int)(word >> d.tp_shift);
        const long long gt = ((long long)part << d.tp_shift) | (word & lmask);
        atomicAdd(&win[(size_t)r * d.BN + gt], (int)e.y);
      }
    }
    __syncthreads();
    XPH(6)
  }
}

// Staging role (pass 1 of the expansion of window [k0, k0 + W)) for the spikes of steps
// [n_lo, n_hi), k0 - d_max <= n_lo, n_hi <= k0, as virtual block vb of nvb.  The walk fills the
// block's queue of row pieces; then the wavefronts take pieces four at a time (8 full-width loads
// in flight) and stage the events by target part.  stage = 0: every event is added to the window
// with a global atomic instead.  With stage != 0, nvb must be d.NB (one staging region per part
// and virtual block).
__device__ __forceinline__ void role_bin(const Dev& d, ExpandLds& L, SortLds& S, long long k0, long long n_lo,
                                         long long n_hi, int vb, int nvb, int stage, long long count_from) {
  int nparts = (stage && d.cap > 0) ? (d.P < kMaxParts ? d.P : kMaxParts) : 0;
  int* __restrict__ win = win_of(d, k0);
  for (int x = threadIdx.x; x < nparts; x += kRingThreads) L.cur[x] = 0;
  if (threadIdx.x == 0) { L.qn = 0; L.qhead = 0; L.qlen = 0; }
  __syncthreads();
  XPH_BEGIN
  const int lane = threadIdx.x & 63;
  auto one = [&](const Seg& o) {
    for (int q = lane; q < o.len; q += 64) {
      const uint2 e = d.synf[o.p0 + q];
      stage_event(d, win, L.cur, nparts, vb, e.x, (int)e.y, o.dlo, o.base);
    }
  };
  long long cnt[3] = {0, 0, 0};
  walk_segments(d, L, d.spike_bits, true, k0, n_lo, n_hi, -1, vb, nvb, count_from, cnt, one);
  XPH(0)
  // counters first: their atomics complete while the events are staged
  if (count_from < n_hi) fold_counts(d, L, cnt, vb);
  const int qn = L.qn < kSegQueue ? L.qn : kSegQueue;
  // Few events for many parts (fewer queued events than parts: large B x N, low rates): a staging
  // region would hold one event at most, and the pass would cost its cursors (one counter per
  // part and block, written here and read again by the accumulation pass) rather than its
  // events.  Such a block adds its events to the window with global atomics and leaves its
  // counters as they are: zero.  (Pieces that did not fit the queue were staged during the walk:
  // then the block stays with staging.)
  if (nparts > 0) {
    int mine = 0;
    for (int x = threadIdx.x; x < qn; x += kRingThreads) mine += L.q[x].len;
    mine = (int)wave_total64((long long)mine);
    if (lane == 0 && mine) atomicAdd(&L.qlen, mine);
    __syncthreads();
    if (L.qn <= kSegQueue && L.qlen < nparts) nparts = 0;   // uniform over the block
  }
  XPH(1)
  const bool staged = nparts > 0;
  if (stage == 2 && nparts > 0 && nparts <= kSortParts) {
    stage_sorted(d, L, S, win, nparts, vb, qn XPH_PASS);
  } else {
    for (;;) {
      int t = 0;
      if (lane == 0) t = atomicAdd(&L.qhead, 4);
      t = __builtin_amdgcn_readfirstlane(t);
      if (t >= qn) break;
      Seg o[4];
      uint2 ev[4][2];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        o[j].len = 0;
        if (t + j < qn) o[j] = L.q[t + j];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          ev[j][h] = make_uint2(0u, 0u);
          if (lane + 64 * h < o[j].len) ev[j][h] = load_stream(&d.synf[o[j].p0 + lane + 64 * h]);
        }
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
          if (lane + 64 * h < o[j].len)
            stage_event(d, win, L.cur, nparts, vb, ev[j][h].x, (int)ev[j][h].y, o[j].dlo, o[j].base);
        for (int q = 128 + lane; q < o[j].len; q += 64) {
          const uint2 e = d.synf[o[j].p0 + q];
          stage_event(d, win, L.cur, nparts, vb, e.x, (int)e.y, o[j].dlo, o[j].base);
        }
      }
    }
  }
  __syncthreads();
  XPH(7)
  XPH_COUNT(15)
  // (the counters are zero when the pass begins: the accumulation pass clears what it has read)
  if (staged)
    for (int x = threadIdx.x; x < nparts; x += kRingThreads) {
      const int c = L.cur[x];
      if (c) d.ecnt[(size_t)x * d.NB + vb] = c < d.cap ? c : d.cap;
    }
}

// Accumulation role (pass 2): sums the staged events of target part `part` into an LDS tile
// [W][targets per part] and adds the tile to the buffer of window k0.  A run (the events one
// virtual block of pass 1 staged for this part) is read by a 16-lane group, 4 runs per load
// instruction, 4 instructions in flight.
__device__ __forceinline__ void role_acc(const Dev& d, int* tile, long long k0, int part) {
  const int cells = d.W << d.tp_shift;
  const int nb_runs = d.NB;
  int* __restrict__ cnts = d.ecnt + (size_t)part * nb_runs;
  XPH_BEGIN
  // nothing staged for this part (its blocks of pass 1 chose atomics, or had no event for it):
  // leave before the tile is touched
  int any = 0;
  for (int x = threadIdx.x; x < nb_runs; x += kRingThreads) any |= cnts[x];
  for (int x = threadIdx.x; x < cells; x += kRingThreads) tile[x] = 0;
  if (!__syncthreads_or(any)) return;
  XPH(8)
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  for (int r0 = (wv * 4 + grp) * 4; r0 < nb_runs; r0 += kRingWaves * 16) {
    int cn[4]; uint2 ev[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) cn[j] = r0 + j < nb_runs ? cnts[r0 + j] : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (sub == 0 && cn[j]) cnts[r0 + j] = 0;   // consumed: zero again for the next window
      ev[j] = make_uint2(0u, 0u);
      if (sub < cn[j]) ev[j] = load_stream(&d.ebuf[((size_t)part * nb_runs + r0 + j) * d.cap + sub]);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (sub < cn[j]) atomicAdd(&tile[ev[j].x], (int)ev[j].y);
      for (int q = 16 + sub; q < cn[j]; q += 16) {
        const uint2 e = d.ebuf[((size_t)part * nb_runs + r0 + j) * d.cap + q];
        atomicAdd(&tile[e.x], (int)e.y);
      }
    }
  }
  __syncthreads();
  XPH(9)
  const int tp = 1 << d.tp_shift;
  int* __restrict__ win = win_of(d, k0);
  for (int x = threadIdx.x; x < cells; x += kRingThreads) {
    const int v = tile[x];
    const int r = x >> d.tp_shift;
    const long long t = (long long)part * tp + (x & (tp - 1));
    // the part's cells have no other writer during this pass; an atomic without return value, so
    // that nobody waits for a load
    if (v != 0 && t < d.BN) atomicAdd(&win[(size_t)r * d.BN + t], v);
  }
#ifdef ADSEQ_PHASE_CLOCK
  __syncthreads();
  XPH(10)
#endif
}

// The two passes of the expansion as kernels.
// The same roles as launches of their own (window boundaries, catching up, open loop).
__global__ __launch_bounds__(kRingThreads) void k_win_bin(Dev d, long long k0, long long n_lo, long long n_hi,
                                                          int vb0, int nvb, int stage, long long count_from, int clear_other) {
  __shared__ ExpandLds L;
  __shared__ SortLds S;
  XPH_SPAN(0, 0)
  role_bin(d, L, S, k0, n_lo, n_hi, vb0 + (int)blockIdx.x, nvb, stage, count_from);
  XPH_SPAN(0, 1)
  // The other window buffer -- the one the steps before k0 have just used up -- is zeroed here, a
  // slice per block, for the expansion that fills it next: the resident step kernels do not clear
  // the cells they pop (their one XCD would spend a fifth of a step on those stores), and the
  // per-step kernels, which do, lose nothing (clear_other is set when the handle runs resident kernels).
  if (clear_other) {
    int* other = d.win + (size_t)((((k0 >> d.wshift) & 1) ^ 1)) * d.W * d.BN;
    const size_t cells = (size_t)d.W * d.BN;
    const size_t per = ((cells + nvb - 1) / nvb + 3) & ~(size_t)3;
    const size_t lo = per * (size_t)(vb0 + (int)blockIdx.x);
    const size_t hi = lo + per < cells ? lo + per : cells;
    // (lo is a multiple of 4: whole 16-byte stores where the buffer is 16-byte aligned, then the tail)
    const bool aligned = (reinterpret_cast<size_t>(other) & 15) == 0;   // (W = 2 with odd B N: the second buffer is not)
    const size_t hi4 = aligned ? lo + ((hi > lo ? hi - lo : 0) & ~(size_t)3) : lo;
    for (size_t x = lo + 4 * (size_t)threadIdx.x; x < hi4; x += 4 * (size_t)kRingThreads)
      *reinterpret_cast<int4*>(other + x) = make_int4(0, 0, 0, 0);
    for (size_t x = (hi4 < hi ? hi4 : hi) + threadIdx.x; x < hi; x += kRingThreads) other[x] = 0;
  }
}
__global__ __launch_bounds__(kRingThreads) void k_win_acc(Dev d, long long k0, int p0) {
  __shared__ int tile[kMaxTileCells];
  XPH_SPAN(1, 0)
  role_acc(d, tile, k0, p0 + (int)blockIdx.x);
  XPH_SPAN(1, 1)
}

// Spikes of steps [n_lo, n_hi) (still in the circular spike words), their events and the Q8.24
// sum of those, added to out[0..3).  On demand only (counters of the steps since the last window
// boundary).
__global__ __launch_bounds__(kBlock) void k_count_spikes(Dev d, long long n_lo, long long n_hi,
                                                         unsigned long long* out /*[3]*/) {
  const long long items = (n_hi - n_lo) * d.words;
  long long c0 = 0, c1 = 0, c2 = 0;
  for (long long it = (long long)blockIdx.x * kBlock + threadIdx.x; it < items; it += (long long)gridDim.x * kBlock) {
    const long long n = n_lo + it / d.words;
    const long long word = it % d.words;
    unsigned long long bits = d.spike_bits[(size_t)(n % d.R) * d.words + word];
    while (bits) {
      const int bit = __ffsll((long long)bits) - 1;
      bits &= bits - 1;
      const long long g = word * 64 + bit;
      if (g >= d.BN) break;
      const int i = (int)(g % d.N);
      c0 += 1; c1 += d.row_ptr[i + 1] - d.row_ptr[i]; c2 += d.rowsum[i];
    }
  }
  c0 = wave_sum(c0); c1 = wave_sum(c1); c2 = wave_sum(c2);
  if ((threadIdx.x & 63) == 0) {
    if (c0) atomicAdd(&out[0], (unsigned long long)c0);
    if (c1) atomicAdd(&out[1], (unsigned long long)c1);
    if (c2) atomicAdd(&out[2], (unsigned long long)c2);
  }
}

// Events of the ring still in flight at step n_end (arrival >= n_end), counted from the spike
// bits of the last d_max + 1 steps.  One block per (slot, 64-neuron word); on demand only.
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
      const uint2 e = d.synf[p];
      if (np + (int)(e.x & d.dmask) >= n_end) { cnt += 1; sum += (int)e.y; }
    }
  }
  block_add2(&out[0], cnt, (long long*)&out[1], sum);
}

// ---------------------------------------------------------------- reverse sweep

// Neuron part of a reverse step (all queue kinds).  U: recorded membrane value of step n, Uprev:
// that of step n - 1 (spike-time mode only), s: spike at n, carry: what step n + 1 handed back to
// the membrane state (alpha gU[n+1] + E[n+1]), dcount: dL/dcount, G: queue term, dU: dL/dU[n].
// Writes gU[n] to *gu_out and returns the new carry.
//   gU[n] = (1 - s) carry + sigma'(U - theta) (dL/dcount + s G) + dL/dU[n]       (Section 2.2 eq. 7)
// Spike-time mode (no surrogate; Section 3.1 eq. 8, Section 4.1 spike detection): a spike's
// emission time depends on the membrane value v the step started from, dt_spk/dv = -1 / vdot with
// vdot = (U - v) / dt (1 where that is 0), and hands (1 / tau) G to its receivers (eq. 17), so
// E = -(1 / vdot)(1 / tau) G goes back to the state before the step.
// (SURR: the gradient mode, d.surrogate, as a constant of the caller where it has one: a reverse step of a resident
// kernel is bound by the instructions it issues)
template <int SURR>
__device__ __forceinline__ float bwd_update_as(const Dev& d, long long n, float U, float Uprev, bool s, float carry,
                                               float dcount, float G, float dU, float* gu_out) {
  float sg = 0.0f;
  if (SURR == ADSEQ_SURR_SUPERSPIKE) {
    const float x = fabsf(U - d.theta) + 1.0f;
    sg = __builtin_amdgcn_rcpf(x * x);   // (one instruction, 1 ulp: the division's dozen were a third of a dense reverse step)
  }
  float inner = dcount;
  if (s) inner += G;
  float gu = sg * inner;
  if (!s) gu += carry;
  gu += dU;
  *gu_out = gu;
  float e = 0.0f;
  if (SURR == ADSEQ_GRAD_SPIKE_TIME && s) {
    const float vprev = n > 0 ? (Uprev >= d.theta ? d.v_reset : Uprev) : 0.0f;
    float vdot = (U - vprev) / d.dt;
    if (vdot == 0.0f) vdot = 1.0f;
    // (double-exponential synapse: G was gathered with the 1 / tau factors of the two states in it)
    e = d.alpha_r > 0.0f ? -(1.0f / vdot) * G : -(1.0f / vdot) * (1.0f / d.tau) * G;
  }
  return __fmaf_rn(d.alpha, gu, e);
}
__device__ __forceinline__ float bwd_update(const Dev& d, long long n, float U, float Uprev, bool s, float carry,
                                            float dcount, float G, float dU, float* gu_out) {
  if (d.surrogate == ADSEQ_SURR_SUPERSPIKE) return bwd_update_as<ADSEQ_SURR_SUPERSPIKE>(d, n, U, Uprev, s, carry, dcount, G, dU, gu_out);
  if (d.surrogate == ADSEQ_GRAD_SPIKE_TIME) return bwd_update_as<ADSEQ_GRAD_SPIKE_TIME>(d, n, U, Uprev, s, carry, dcount, G, dU, gu_out);
  return bwd_update_as<ADSEQ_SURR_OFF>(d, n, U, Uprev, s, carry, dcount, G, dU, gu_out);
}

// What an event delivered to neuron g at this step gathers: the adjoint of the state that took its
// jump.  Without a synaptic current state that is gU itself; with one, dL/dJ[n] = gU[n] + alpha_s
// dL/dJ[n+1] (kept in bwd_carryJ).
// Double-exponential synapse (states A, B; current A - B): gA[n] = dL/dA[n] = gU[n] + alpha_s gA[n+1],
// gB[n] = dL/dB[n] = -gU[n] + alpha_r gB[n+1]; the weight gathers X = gA + gB (returned), the
// delay and the emission time gather Y = gA / tau_syn + gB / tau_rise (*y_out).  Kept are gA and X
// rather than gA and gB: gU cancels in the sum, X[n] = alpha_r X[n+1] + (alpha_s - alpha_r) gA[n+1],
// which fp32 follows without the loss of digits that adding two nearly opposite numbers has.
__device__ __forceinline__ float bwd_receiver(const Dev& d, int g, float gu, float* y_out) {
  if (!(d.alpha_s > 0.0f)) return gu;
  const float ga_next = d.bwd_carryJ[g];
  const float gj = __fmaf_rn(d.alpha_s, ga_next, gu);
  d.bwd_carryJ[g] = gj;
  if (!(d.alpha_r > 0.0f)) return gj;
  const float x = __fmaf_rn(d.alpha_r, d.bwd_carryJ[(size_t)d.BN + g], d.alpha_diff * ga_next);
  d.bwd_carryJ[(size_t)d.BN + g] = x;
  *y_out = x * d.inv_tau_b - gj * d.inv_tau_diff;   // = gA / tau_syn + (X - gA) / tau_rise
  return x;
}

// Double-exponential synapse: which of the two gathered adjoints the queue term of the emitting
// spike is made of (its value in the surrogate modes, its time in the spike-time mode).
__device__ __forceinline__ float queue_term_of(const Dev& d, float x, float y) {
  return d.surrogate == ADSEQ_GRAD_SPIKE_TIME ? y : x;
}

// Gathers the adjoint at the arrival cell of the entries [0, cnt) of the sorted row at pr0
// (a spike at step n, window phase phi; arrivals inside the same window), adds it to gsum and
// returns the wavefront's sum of amplitude * adjoint in every lane.
template <bool DEXP>
__device__ __forceinline__ float near_gather(const Dev& d, const float* __restrict__ gwin, long long n,
                                             long long T, int phi, long long pr0, unsigned cnt, int base) {
  const int lane = threadIdx.x & 63;
  const size_t second = 2 * (size_t)d.W * d.BN;   // the Y rows lie behind the two window buffers of X
  float G = 0.0f;
  for (unsigned q = lane; q < cnt; q += 64) {
    const uint2 e = d.synb[pr0 + q];
    const int D = (int)(e.x & d.dmask);
    if (n + D < T) {
      const size_t cell = (size_t)(phi + D) * d.BN + (size_t)base + (e.x >> d.dbits);
      const float gv = gwin[cell];
      unsafeAtomicAdd(&d.gsum[pr0 + q], gv);
      if (DEXP) {
        const float gy = gwin[second + cell];
        unsafeAtomicAdd(&d.gsum[(size_t)d.S + pr0 + q], gy);
        G += __uint_as_float(e.y) * queue_term_of(d, gv, gy);
      } else {
        G += __uint_as_float(e.y) * gv;
      }
    }
  }
  return wave_sum_f(G);
}

// Reverse step n: queue term of the block's spikes = far part (left in Gacc by the windows
// already swept) + near part (gathered here from the rows of this window written by the earlier
// launches), then
//   gU[n] = (1 - s) carry + sigma'(U - theta) (dL/dcount + s G) + dL/dU[n]
//   carry <- alpha gU[n] + E,  E = -(1 / vdot)(1 / tau) G for a spike in the spike-time mode
// (see bwd_update)
// SYN: synaptic current states, as in k_step_win; 2 = double-exponential synapse: every gather
// takes two adjoints, X for the weight and Y for the delay (see bwd_receiver)
// LAZY: row start, in-window count and far queue term are fetched by the spiking lanes only (16
// bytes per neuron less HBM traffic, one more memory round trip before the gathers)
template <int SYN, bool LAZY>
__global__ __launch_bounds__(kBlock) void k_bwd_step_win(long long n, long long T,
                                                         const float* __restrict__ dL_dcount,
                                                         const float* __restrict__ dL_dU, Dev d) {
  pin_args(d.gwin, d.tapeU, d.bwd_carry, d.bwd_carryJ, d.row_ptr, d.nearcnt, d.Gacc, d.synb, d.gsum,
           d.N, d.B, d.BN, d.W, d.wshift, d.d_max, d.R, d.dbits, d.dmask, d.surrogate, d.alpha, d.alpha_s,
           d.theta, d.v_reset, d.dt, d.tau, n, T, dL_dcount, dL_dU);
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  const int phi = (int)(n & (long long)(d.W - 1));
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  float U = 0.0f, Uprev = 0.0f, carry = 0.0f, inner = 0.0f, G = 0.0f, dU = 0.0f;
  bool s = false;
  int b = 0;
  long long r0 = 0;
  unsigned ncnt = 0;
  float* __restrict__ gwin = gwin_of(d, n);
  constexpr bool DEXP = SYN == 2;
  const size_t second = 2 * (size_t)d.W * d.BN;   // the Y rows lie behind the two window buffers of X
  if (act) {
    b = trial_of(d, g);
    const int i = g - b * d.N;
    U = d.tapeU[(size_t)n * d.BN + g];
    if (d.surrogate == ADSEQ_GRAD_SPIKE_TIME && n > 0) Uprev = d.tapeU[(size_t)(n - 1) * d.BN + g];
    carry = d.bwd_carry[g];
    if (dL_dcount) inner = dL_dcount[g];
    if (dL_dU) dU = dL_dU[(size_t)n * d.BN + g];
    // far queue term: only spiking neurons have one, but (unless LAZY) it is loaded for all so
    // that it does not wait for the membrane value; the same for the row start and count
    float* ga = &d.Gacc[(size_t)(n % d.R) * d.BN + g];
    if (!LAZY) {
      r0 = d.row_ptr[i];
      if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
      G = *ga;
    }
    s = U >= d.theta;
    if (LAZY && s) {
      r0 = d.row_ptr[i];
      if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
      G = *ga;
    }
    if (G != 0.0f) *ga = 0.0f;
  }
  // in-window part of the queue term of the wavefront's spikes, up to four spikes at a time (row
  // loads, then adjoint gathers, each for all four before the next stage)
  unsigned long long m = __ballot(s && ncnt > 0);
  const int lane = threadIdx.x & 63;
  while (m) {
    long long pr[4]; unsigned cn[4]; int bs[4], Ls[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      pr[j] = 0; cn[j] = 0; bs[j] = 0; Ls[j] = -1;
      if (m) {
        const int L = __ffsll((long long)m) - 1;
        m &= m - 1;
        Ls[j] = L;
        pr[j] = lane_get(r0, L); cn[j] = lane_get(ncnt, L); bs[j] = lane_get(b, L) * d.N;
      }
    }
    uint2 e[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      e[j] = make_uint2(0u, 0u);
      if ((unsigned)lane < cn[j]) e[j] = d.synb[pr[j] + lane];
    }
    float gv[4], gy[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      gv[j] = 0.0f; gy[j] = 0.0f;
      const int D = (int)(e[j].x & d.dmask);
      if ((unsigned)lane < cn[j] && n + D < T) {
        const size_t cell = (size_t)(phi + D) * d.BN + (size_t)bs[j] + (e[j].x >> d.dbits);
        gv[j] = gwin[cell];
        if (DEXP) gy[j] = gwin[second + cell];
      }
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (Ls[j] < 0) continue;    // uniform
      const int D = (int)(e[j].x & d.dmask);
      float part = 0.0f;
      if ((unsigned)lane < cn[j] && n + D < T) {
        part = __uint_as_float(e[j].y) * (DEXP ? queue_term_of(d, gv[j], gy[j]) : gv[j]);
        unsafeAtomicAdd(&d.gsum[pr[j] + lane], gv[j]);
        if (DEXP) unsafeAtomicAdd(&d.gsum[(size_t)d.S + pr[j] + lane], gy[j]);
      }
      part = wave_sum_f(part);
      if (cn[j] > 64u) part += near_gather<DEXP>(d, gwin, n, T, phi, pr[j] + 64, cn[j] - 64u, bs[j]);
      if (lane == Ls[j]) G += part;
    }
  }
  if (act) {
    float gu;
    __builtin_nontemporal_store(bwd_update(d, n, U, Uprev, s, carry, inner, G, dU, &gu), &d.bwd_carry[g]);
    float y = 0.0f;
    gwin[(size_t)phi * d.BN + g] = SYN ? bwd_receiver(d, g, gu, &y) : gu;
    if (DEXP) gwin[second + (size_t)phi * d.BN + g] = y;
  }
}

// Gather role: far part of the queue terms for window [k0, k0 + W), whose adjoint rows are
// complete, for the recorded spikes of steps [n_lo, n_hi) (k0 - d_max <= n_lo; n_hi <= k0, or up to
// the end of the window when the window was swept as a whole (ring_reverse.h): then the window's own
// spikes take part for the per-synapse sums of their near events), as virtual block vb of nvb.  The piece of each spike's sorted row that arrives in the window
// gathers its adjoints from the window (6.4 MB: the L2 holds it), adds them to gsum, and the
// wavefront's sum of amplitude * adjoint is added to Gacc[n mod R][g] (one wavefront per piece,
// one piece per spike and window).
// DEXP (double-exponential synapse): two adjoints per arrival cell, X and Y (see bwd_receiver).
template <bool DEXP>
__device__ __forceinline__ void role_gather(const Dev& d, ExpandLds& L, long long k0, long long n_lo, long long n_hi,
                                            long long T, int vb, int nvb) {
  XPH_BEGIN
#ifdef ADSEQ_PHASE_CLOCK
  if (k0 == 512) XPH_SPAN(2, 0)   // (one window from the middle of the run)
#endif
  if (threadIdx.x == 0) { L.qn = 0; L.qhead = 0; }
  __syncthreads();
  const int lane = threadIdx.x & 63;
  const float* __restrict__ gwin = gwin_of(d, k0);
  const size_t second = 2 * (size_t)d.W * d.BN;   // the Y rows lie behind the two window buffers of X
  // one gathered entry: amplitude bits ab, arrival cell `cell`, sorted-row position q
  auto take = [&](unsigned ab, size_t cell, long long q, float x) -> float {
    unsafeAtomicAdd(&d.gsum[q], x);
    if (DEXP) {
      const float y = gwin[second + cell];
      unsafeAtomicAdd(&d.gsum[(size_t)d.S + q], y);
      return __uint_as_float(ab) * queue_term_of(d, x, y);
    }
    return __uint_as_float(ab) * x;
  };
  auto finish = [&](const Seg& o, float G) {
    if (o.dlo < 1) return;   // a spike inside the window: its near queue term has been taken already; only the per-synapse sums were wanted
    G = wave_sum_f(G);
    if (lane == 0) {
      // one wavefront per piece, one piece per spike and window: the add has no competitor; an
      // atomic without return value so that the wavefront does not wait for a load
      unsafeAtomicAdd(&d.Gacc[(size_t)o.slot * d.BN + o.g], G);
    }
  };
  auto one = [&](const Seg& o) {
    float G = 0.0f;
    for (int q = lane; q < o.len; q += 64) {
      const uint2 e = d.synb[o.p0 + q];
      const size_t cell = (size_t)((int)(e.x & d.dmask) - o.dlo) * d.BN + (size_t)o.base + (e.x >> d.dbits);
      G += take(e.y, cell, o.p0 + q, gwin[cell]);
    }
    finish(o, G);
  };
  long long cnt[3] = {0, 0, 0};
  walk_segments(d, L, d.tape_bits, false, k0, n_lo, n_hi, T, vb, nvb, n_hi, cnt, one);
  XPH(16)
  const int qn = L.qn < kSegQueue ? L.qn : kSegQueue;
  for (;;) {
    int t = 0;
    if (lane == 0) t = atomicAdd(&L.qhead, 4);
    t = __builtin_amdgcn_readfirstlane(t);
    if (t >= qn) break;
    Seg o[4];
    uint2 ev[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      o[j].len = 0;
      if (t + j < qn) o[j] = L.q[t + j];
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        ev[j][h] = make_uint2(0u, 0u);
        if (lane + 64 * h < o[j].len) ev[j][h] = load_stream(&d.synb[o[j].p0 + lane + 64 * h]);
      }
    }
    float gv[4][2];
    size_t cell[4][2];
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        gv[j][h] = 0.0f;
        cell[j][h] = (size_t)((int)(ev[j][h].x & d.dmask) - o[j].dlo) * d.BN + (size_t)o[j].base + (ev[j][h].x >> d.dbits);
        if (lane + 64 * h < o[j].len) gv[j][h] = gwin[cell[j][h]];
      }
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (t + j >= qn) continue;
      float G = 0.0f;
#pragma unroll
      for (int h = 0; h < 2; ++h)
        if (lane + 64 * h < o[j].len) G += take(ev[j][h].y, cell[j][h], o[j].p0 + lane + 64 * h, gv[j][h]);
      for (int q = 128 + lane; q < o[j].len; q += 64) {
        const uint2 e = d.synb[o[j].p0 + q];
        const size_t c = (size_t)((int)(e.x & d.dmask) - o[j].dlo) * d.BN + (size_t)o[j].base + (e.x >> d.dbits);
        G += take(e.y, c, o[j].p0 + q, gwin[c]);
      }
      finish(o[j], G);
    }
  }
#ifdef ADSEQ_PHASE_CLOCK
  __builtin_amdgcn_s_waitcnt(0x0F70);   // (the clock reads after the wavefront's own loads and adds)
  XPH(17)
  __syncthreads();
  XPH(18)
  XPH_COUNT(19)
  if (k0 == 512) XPH_SPAN(2, 1)
#endif
}

template <bool DEXP>
__global__ __launch_bounds__(kRingThreads) void k_bwd_win(Dev d, long long k0, long long n_lo, long long n_hi,
                                                          long long T, int vb0, int nvb) {
  __shared__ ExpandLds L;
  role_gather<DEXP>(d, L, k0, n_lo, n_hi, T, vb0 + (int)blockIdx.x, nvb);
}

// grad_w[p] = f_p * gsum, grad_d[p] = a_p * dscale * gsum, back in the caller's synapse order.
// One block per row: rows of up to kFinishRow entries are un-permuted through LDS so that both
// the reads (sorted order) and the writes (caller's order) are coalesced; longer rows write
// through perm directly.
constexpr int kFinishRow = 4096;
__global__ __launch_bounds__(kBlock) void k_grad_finish(Dev d, float dscale, float* __restrict__ grad_w,
                                                        float* __restrict__ grad_d) {
  __shared__ float s_w[kFinishRow];
  __shared__ float s_d[kFinishRow];
  for (long long i = blockIdx.x; i < d.N; i += gridDim.x) {
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    const bool small = r1 - r0 <= kFinishRow;   // uniform over the block
    for (long long q = r0 + threadIdx.x; q < r1; q += kBlock) {
      const float gs = d.gsum[q];
      const unsigned pp = d.perm[q];
      const float gw = (d.continuous ? d.fdec[q] : 1.0f) * gs;
      // (double-exponential synapse: the delay's own sum lies behind the weight's)
      const float gd = __uint_as_float(d.synb[q].y) * dscale * (d.alpha_r > 0.0f ? d.gsum[(size_t)d.S + q] : gs);
      if (small) { s_w[pp] = gw; s_d[pp] = gd; }
      else { grad_w[r0 + pp] = gw; grad_d[r0 + pp] = gd; }
    }
    if (small) {
      __syncthreads();
      for (long long p = r0 + threadIdx.x; p < r1; p += kBlock) { grad_w[p] = s_w[p - r0]; grad_d[p] = s_d[p - r0]; }
      __syncthreads();
    }
  }
}
