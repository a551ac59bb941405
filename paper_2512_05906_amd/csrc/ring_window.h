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
// The expansion pass does not scatter with one memory-side atomic per event.  It bins the
// events by target range into per-(part, block) regions of a staging buffer (LDS cursors, no
// global atomics); a second kernel gives each part to one workgroup, which sums the part's
// events into a 64 KB LDS tile with LDS atomics and adds the tile to win with coalesced
// accesses.  Events that do not fit their region fall back to a global atomic on win, so the
// result never depends on the staging capacity.
// The expansion of window q + 1 is split in two: the spikes older than window q ("old part", 15/16
// of the events for W = 16, d_max = 250) are expanded on a second stream while the steps of
// window q run; the spikes of window q itself ("recent part") follow at the boundary with plain
// atomics.  Hence the two window buffers.
//
// The reverse sweep mirrors it: gwin f32 [2][W][BN] holds the adjoint rows of the current window
// and of the one swept before it (still being read by the old part of its gather);
// a spike's queue term is the sum of a near part (gathered by the step kernel) and one far part
// per later window (gathered by k_bwd_win from the 6.4 MB window, which the L2 holds, into
// Gacc[n mod R][g]); the per-synapse sum of gathered adjoints goes to gsum in sorted order and is
// scaled and un-permuted into grad_w / grad_d by k_grad_finish.

constexpr int kBinThreads = 1024;   // threads per block of k_win_bin / k_win_acc
constexpr int kBinWaves = kBinThreads / 64;
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

// Block b owns neurons [256 b, 256 b + 256): pops their cells of row phi = n mod W, adds the
// drive, integrates, records the membrane value and the spike bits, and scatters the in-window
// events of its own spikes.  No atomic on any shared counter.
template <bool RECORD>
__global__ __launch_bounds__(kBlock) void k_step_win(Dev d, long long n, const float* __restrict__ i_ext,
                                                     unsigned char* __restrict__ spikes_out) {
  __shared__ long long s_red[4][kBlock / 64];
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  const int phi = (int)(n & (long long)(d.W - 1));
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  int acc = 0, b = 0, i = 0;
  bool s = false;
  long long r0 = 0;
  unsigned ncnt = 0;
  int* __restrict__ win = win_of(d, n);
  if (act) {
    b = g / d.N; i = g - b * d.N;
    const size_t idx = (size_t)phi * d.BN + g;
    acc = win[idx];
    // row start and in-window entry count of every neuron, loaded beside the pop so that a
    // spiking neuron's fan-out does not wait for them (both arrays stay in the L2)
    r0 = d.row_ptr[i];
    if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
    const float v = d.V[g];
    if (acc != 0) win[idx] = 0;
    float I = (float)acc * 0x1p-24f;
    if (d.p_thresh) {
      const bool xi = (unsigned long long)drive_bits(d.seed, (unsigned long long)g,
                                                     (unsigned long long)n) < d.p_thresh;
      I = I + (xi ? d.ext_w : 0.0f);
    }
    if (i_ext) I = I + i_ext[g];
    const float U = __fmaf_rn(d.alpha, v, I);
    s = U >= d.theta;
    d.V[g] = s ? d.v_reset : U;
    if (RECORD) d.tapeU[(size_t)n * d.BN + g] = U;
    if (spikes_out) spikes_out[g] = s ? 1 : 0;
  }
  const unsigned long long bits = __ballot(s);
  if ((threadIdx.x & 63) == 0) {
    const size_t word = (size_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6);
    d.spike_bits[(size_t)(n % d.R) * d.words + word] = bits;
    if (RECORD) d.tape_bits[(size_t)n * d.words + word] = bits;
  }
  long long c_off = 0, s_off = 0;
  if (s) { c_off = d.row_ptr[i + 1] - r0; s_off = d.rowsum[i]; }
  unsigned long long m = __ballot(s && ncnt > 0);
  while (m) {
    const int L = __ffsll((long long)m) - 1;
    m &= m - 1;
    near_scatter(d, win, phi, __shfl(r0, L, 64), __shfl(ncnt, L, 64), __shfl(b, L, 64) * d.N);
  }
  const long long sp = wave_sum((long long)acc);
  const long long ns = wave_sum((long long)(s ? 1 : 0));
  c_off = wave_sum(c_off); s_off = wave_sum(s_off);
  if ((threadIdx.x & 63) == 0) {
    const int w = threadIdx.x >> 6;
    s_red[0][w] = sp; s_red[1][w] = ns; s_red[2][w] = c_off; s_red[3][w] = s_off;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    long long a = 0, c = 0, co = 0, so = 0;
    for (int w = 0; w < kBlock / 64; ++w) { a += s_red[0][w]; c += s_red[1][w]; co += s_red[2][w]; so += s_red[3][w]; }
    // private counters of this block; atomics only so that nothing waits for a read
    BlkCtr& bc = d.blk[blockIdx.x];
    if (a) atomicAdd((unsigned long long*)&bc.sum_delivered, (unsigned long long)a);
    if (c) atomicAdd(&bc.spikes, (unsigned long long)c);
    if (co) atomicAdd(&bc.offered, (unsigned long long)co);
    if (so) atomicAdd((unsigned long long*)&bc.sum_offered, (unsigned long long)so);
  }
}

// Open-loop pop of row phi: writes the delivered current, clears the cells and this step's
// spike bits (adseq_enqueue sets them).
__global__ __launch_bounds__(kBlock) void k_deliver_win(Dev d, long long n, float* __restrict__ I_out) {
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const int phi = (int)(n & (long long)(d.W - 1));
  int acc = 0;
  int* __restrict__ win = win_of(d, n);
  if (g < d.BN) {
    const size_t idx = (size_t)phi * d.BN + g;
    acc = win[idx];
    if (acc != 0) win[idx] = 0;
    I_out[g] = (float)acc * 0x1p-24f;
  }
  if ((threadIdx.x & 63) == 0)
    d.spike_bits[(size_t)(n % d.R) * d.words + (size_t)blockIdx.x * (kBlock / 64) + (threadIdx.x >> 6)] = 0ull;
  block_add2(&d.ctr->delivered, 0, &d.ctr->sum_delivered, (long long)acc);
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
  long long c_off = 0, s_off = 0;
  for (int e = wave; e < nspk; e += nwaves) {
    const int g = spk[e];
    if ((unsigned)g >= (unsigned)d.BN) continue;  // uniform over the wavefront
    const int b = g / d.N, i = g - b * d.N;
    const long long r0 = d.row_ptr[i];
    if (lane == 0) {
      atomicOr(&d.spike_bits[(size_t)(n % d.R) * d.words + (g >> 6)], 1ull << (g & 63));
      c_off += d.row_ptr[i + 1] - r0; s_off += d.rowsum[i];
    }
    if (near_h >= 1) near_scatter(d, win_of(d, n), phi, r0, d.nearcnt[(size_t)near_h * d.N + i], b * d.N);
  }
  block_add2(&d.ctr->offered, c_off, &d.ctr->sum_offered, s_off);
}

// ---------------------------------------------------------------- forward: window expansion

// One far event of the window: staged in region (part, block) if there is room, else added to
// win with a global atomic.
__device__ __forceinline__ void stage_event(const Dev& d, int* __restrict__ win, int* s_cur, int nparts,
                                            unsigned pk, int a, int dlo, int base) {
  const int r = (int)(pk & d.dmask) - dlo;             // row of the window, 0 .. W - 1
  const int gt = base + (int)(pk >> d.dbits);
  const int part = gt >> d.tp_shift;
  if (part < nparts) {
    const int pos = atomicAdd(&s_cur[part], 1);
    if (pos < d.cap) {
      d.ebuf[((size_t)part * gridDim.x + blockIdx.x) * d.cap + pos] =
          make_uint2((unsigned)((r << d.tp_shift) | (gt & ((1 << d.tp_shift) - 1))), (unsigned)a);
      return;
    }
  }
  atomicAdd(&win[(size_t)r * d.BN + gt], a);
}

// A wavefront's share of a walk over the spike words of steps [n_lo, n_hi): the words of a step
// are cut into lines of 8 (64 bytes); the line numbered c = gw + nwaves * (8 t + group) belongs
// to the 8-lane group `group` of wavefront gw in trip t, so that lines are dealt round-robin over
// all wavefronts and one wavefront sees up to 8 lines of different steps at once.  Sets the step
// and the spike word of this lane (0 if it has none).
__device__ __forceinline__ unsigned long long walk_word(const Dev& d, const unsigned long long* __restrict__ words,
                                                        bool circular, long long n_lo, long long n_hi,
                                                        long long c0, long long nwaves, long long* n_out,
                                                        int* word_out) {
  const int lane = threadIdx.x & 63;
  const long long lps = (d.words + 7) >> 3;
  const long long c = c0 + nwaves * (lane >> 3);
  *n_out = n_lo; *word_out = 0;
  if (c >= (n_hi - n_lo) * lps) return 0ull;
  const long long si = c / lps;
  const long long n = n_lo + si;
  const int word = (int)(c - si * lps) * 8 + (lane & 7);
  *n_out = n; *word_out = word;
  if (word >= d.words) return 0ull;
  return words[(size_t)(circular ? n % d.R : n) * d.words + word];
}

// Pass 1 of the expansion of window [k0, k0 + W) for the spikes of steps [n_lo, n_hi), with
// k0 - d_max <= n_lo and n_hi <= k0.  Every lane that holds a spike looks up the piece of the
// spike's sorted row that lands in the window (dstart); the wavefront then reads the pieces four
// at a time (8 full-width loads in flight) and stages the events by target part.  stage = 0:
// every event is added to the window with a global atomic instead.  With stage != 0, gridDim.x
// must be d.NB (the staging regions are per block).
__global__ __launch_bounds__(kBinThreads) void k_win_bin(Dev d, long long k0, long long n_lo, long long n_hi,
                                                         int stage) {
  __shared__ int s_cur[kMaxParts];
  const int nparts = (stage && d.cap > 0) ? (d.P < kMaxParts ? d.P : kMaxParts) : 0;
  int* __restrict__ win = win_of(d, k0);
  for (int x = threadIdx.x; x < nparts; x += kBinThreads) s_cur[x] = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const long long gw = blockIdx.x + (long long)gridDim.x * wv;   // blocks interleaved: every block sees every step
  const long long nwaves = (long long)gridDim.x * kBinWaves;
  const long long nlines = (n_hi - n_lo) * ((d.words + 7) >> 3);
  const int nb = d.d_max + 2;
  for (long long c0 = gw; c0 < nlines; c0 += nwaves * 8) {
    long long n; int word;
    unsigned long long bits = walk_word(d, d.spike_bits, true, n_lo, n_hi, c0, nwaves, &n, &word);
    const int dlo = (int)(k0 - n);                      // 1 .. d_max
    const int dhi = dlo + d.W < nb - 1 ? dlo + d.W : nb - 1;
    while (__ballot(bits != 0ull)) {
      // every lane that still has a spike takes its lowest one: row piece [p0, p0 + len)
      long long p0 = 0; int len = 0, base = 0;
      if (bits) {
        const int bit = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        const long long g = (long long)word * 64 + bit;
        if (g < d.BN) {
          const int b = (int)(g / d.N), i = (int)(g - (long long)b * d.N);
          const unsigned* ds = d.dstart + (size_t)i * nb;
          const unsigned q0 = ds[dlo], q1 = ds[dhi];
          p0 = d.row_ptr[i] + q0; len = (int)(q1 - q0); base = b * d.N;
        }
      }
      unsigned long long todo = __ballot(len > 0);
      while (todo) {
        int L[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { L[j] = -1; if (todo) { L[j] = __ffsll((long long)todo) - 1; todo &= todo - 1; } }
        long long P0[4]; int LEN[4], BASE[4], DLO[4];
        uint2 ev[4][2];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          LEN[j] = 0; P0[j] = 0; BASE[j] = 0; DLO[j] = 0;
          if (L[j] >= 0) {
            P0[j] = __shfl(p0, L[j], 64); LEN[j] = __shfl(len, L[j], 64);
            BASE[j] = __shfl(base, L[j], 64); DLO[j] = __shfl(dlo, L[j], 64);
          }
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            ev[j][h] = make_uint2(0u, 0u);
            if (lane + 64 * h < LEN[j]) ev[j][h] = d.synf[P0[j] + lane + 64 * h];
          }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
#pragma unroll
          for (int h = 0; h < 2; ++h)
            if (lane + 64 * h < LEN[j]) stage_event(d, win, s_cur, nparts, ev[j][h].x, (int)ev[j][h].y, DLO[j], BASE[j]);
          for (int q = 128 + lane; q < LEN[j]; q += 64) {
            const uint2 e = d.synf[P0[j] + q];
            stage_event(d, win, s_cur, nparts, e.x, (int)e.y, DLO[j], BASE[j]);
          }
        }
      }
    }
  }
  __syncthreads();
  for (int x = threadIdx.x; x < nparts; x += kBinThreads) {
    const int c = s_cur[x];
    d.ecnt[(size_t)x * gridDim.x + blockIdx.x] = c < d.cap ? c : d.cap;
  }
}

// Pass 2: block `part` sums the staged events of its target range into an LDS tile
// [W][targets per part] and adds the tile to the buffer of window k0.  nb_runs = grid size of
// pass 1 (a multiple of 16 or below 16).  A run (the events one block of pass 1 staged for this
// part) is read by a 16-lane group, 4 runs per load instruction, 4 instructions in flight.
__global__ __launch_bounds__(kBinThreads) void k_win_acc(Dev d, long long k0, int nb_runs) {
  __shared__ int tile[kMaxTileCells];
  const int part = blockIdx.x;
  const int cells = d.W << d.tp_shift;
  for (int x = threadIdx.x; x < cells; x += kBinThreads) tile[x] = 0;
  __syncthreads();
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int sub = lane & 15, grp = lane >> 4;
  const int* __restrict__ cnts = d.ecnt + (size_t)part * nb_runs;
  for (int r0 = (wv * 4 + grp) * 4; r0 < nb_runs; r0 += kBinWaves * 16) {
    int cn[4]; uint2 ev[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) cn[j] = r0 + j < nb_runs ? cnts[r0 + j] : 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      ev[j] = make_uint2(0u, 0u);
      if (sub < cn[j]) ev[j] = d.ebuf[((size_t)part * nb_runs + r0 + j) * d.cap + sub];
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
  const int tp = 1 << d.tp_shift;
  int* __restrict__ win = win_of(d, k0);
  for (int x = threadIdx.x; x < cells; x += kBinThreads) {
    const int v = tile[x];
    const int r = x >> d.tp_shift;
    const long long t = (long long)part * tp + (x & (tp - 1));
    if (v != 0 && t < d.BN) {
      int* cell = &win[(size_t)r * d.BN + t];
      *cell = wrap_add(*cell, v);
    }
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

// Gathers the adjoint at the arrival cell of the entries [0, cnt) of the sorted row at pr0
// (a spike at step n, window phase phi; arrivals inside the same window), adds it to gsum and
// returns the wavefront's sum of amplitude * adjoint in every lane.
__device__ __forceinline__ float near_gather(const Dev& d, const float* __restrict__ gwin, long long n,
                                             long long T, int phi, long long pr0, unsigned cnt, int base) {
  const int lane = threadIdx.x & 63;
  float G = 0.0f;
  for (unsigned q = lane; q < cnt; q += 64) {
    const uint2 e = d.synb[pr0 + q];
    const unsigned pk = e.x;
    const int D = (int)(pk & d.dmask);
    if (n + D < T) {
      const float gv = gwin[(size_t)(phi + D) * d.BN + (size_t)base + (pk >> d.dbits)];
      G += __uint_as_float(e.y) * gv;
      unsafeAtomicAdd(&d.gsum[pr0 + q], gv);
    }
  }
  for (int o = 32; o > 0; o >>= 1) G += __shfl_xor(G, o, 64);
  return G;
}

// Reverse step n: queue term of the block's spikes = far part (left in Gacc by the windows
// already swept) + near part (gathered here from the rows of this window written by the
// earlier launches), then
//   gU[n] = (1 - s) alpha gU[n+1] + sigma'(U - theta) (dL/dcount + s G) + dL/dU[n]
__global__ __launch_bounds__(kBlock) void k_bwd_step_win(Dev d, long long n, long long T,
                                                         const float* __restrict__ dL_dcount,
                                                         const float* __restrict__ dL_dU) {
  const int g = blockIdx.x * kBlock + threadIdx.x;
  const bool act = g < d.BN;
  const int phi = (int)(n & (long long)(d.W - 1));
  int near_h = d.W - 1 - phi;
  if (near_h > d.d_max) near_h = d.d_max;
  float U = 0.0f, carry = 0.0f, inner = 0.0f, G = 0.0f, dU = 0.0f;
  bool s = false;
  int b = 0, i = 0;
  long long r0 = 0;
  unsigned ncnt = 0;
  float* __restrict__ gwin = gwin_of(d, n);
  if (act) {
    b = g / d.N; i = g - b * d.N;
    U = d.tapeU[(size_t)n * d.BN + g];
    carry = d.bwd_carry[g];
    r0 = d.row_ptr[i];
    if (near_h >= 1) ncnt = d.nearcnt[(size_t)near_h * d.N + i];
    if (dL_dcount) inner = dL_dcount[g];
    if (dL_dU) dU = dL_dU[(size_t)n * d.BN + g];
    s = U >= d.theta;
    if (s) {
      float* ga = &d.Gacc[(size_t)(n % d.R) * d.BN + g];
      G = *ga;
      if (G != 0.0f) *ga = 0.0f;
    }
  }
  unsigned long long m = __ballot(s && ncnt > 0);
  const int lane = threadIdx.x & 63;
  while (m) {
    const int L = __ffsll((long long)m) - 1;
    m &= m - 1;
    const float t = near_gather(d, gwin, n, T, phi, __shfl(r0, L, 64), __shfl(ncnt, L, 64), __shfl(b, L, 64) * d.N);
    if (lane == L) G += t;
  }
  if (act) {
    float sg = 0.0f;
    if (d.surrogate == ADSEQ_SURR_SUPERSPIKE) {
      const float x = fabsf(U - d.theta) + 1.0f;
      sg = 1.0f / (x * x);
    }
    if (s) inner += G;
    float gu = sg * inner;
    if (!s) gu = __fmaf_rn(d.alpha, carry, gu);
    gu += dU;
    d.bwd_carry[g] = gu;
    gwin[(size_t)phi * d.BN + g] = gu;
  }
}

// Far part of the queue terms for window [k0, k0 + W), whose adjoint rows are complete: for
// every recorded spike of steps [n_lo, n_hi) (k0 - d_max <= n_lo, n_hi <= k0) the piece of its
// sorted row that arrives in the window gathers its adjoints, adds them to gsum, and the
// wavefront's sum of amplitude * adjoint is added to Gacc[n mod R][g] (one wavefront per spike
// and launch: plain update).  Same walk over the spike words as k_win_bin.
__global__ __launch_bounds__(kBlock) void k_bwd_win(Dev d, long long k0, long long n_lo, long long n_hi,
                                                    long long T) {
  const int lane = threadIdx.x & 63;
  const long long gw = ((long long)blockIdx.x * kBlock + threadIdx.x) >> 6;
  const long long nwaves = ((long long)gridDim.x * kBlock) >> 6;
  const long long nlines = (n_hi - n_lo) * ((d.words + 7) >> 3);
  const int nb = d.d_max + 2;
  const float* __restrict__ gwin = gwin_of(d, k0);
  for (long long c0 = gw; c0 < nlines; c0 += nwaves * 8) {
    long long n; int word;
    unsigned long long bits = walk_word(d, d.tape_bits, false, n_lo, n_hi, c0, nwaves, &n, &word);
    const int dlo = (int)(k0 - n);
    int dhi = dlo + d.W < nb - 1 ? dlo + d.W : nb - 1;
    if ((long long)dhi > T - n) dhi = (int)(T - n);    // arrivals n + D >= T are never delivered
    if (dhi < dlo) dhi = dlo;
    const int slot = (int)(n % d.R);
    while (__ballot(bits != 0ull)) {
      long long p0 = 0, g = 0; int len = 0, base = 0;
      if (bits) {
        const int bit = __ffsll((long long)bits) - 1;
        bits &= bits - 1;
        g = (long long)word * 64 + bit;
        if (g < d.BN) {
          const int b = (int)(g / d.N), i = (int)(g - (long long)b * d.N);
          const unsigned* ds = d.dstart + (size_t)i * nb;
          const unsigned q0 = ds[dlo], q1 = ds[dhi];
          p0 = d.row_ptr[i] + q0; len = (int)(q1 - q0); base = b * d.N;
        }
      }
      unsigned long long todo = __ballot(len > 0);
      while (todo) {
        int L[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) { L[j] = -1; if (todo) { L[j] = __ffsll((long long)todo) - 1; todo &= todo - 1; } }
        long long P0[4]; int LEN[4], BASE[4], DLO[4];
        uint2 ev[4][2];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          LEN[j] = 0; P0[j] = 0; BASE[j] = 0; DLO[j] = 0;
          if (L[j] >= 0) {
            P0[j] = __shfl(p0, L[j], 64); LEN[j] = __shfl(len, L[j], 64);
            BASE[j] = __shfl(base, L[j], 64); DLO[j] = __shfl(dlo, L[j], 64);
          }
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            ev[j][h] = make_uint2(0u, 0u);
            if (lane + 64 * h < LEN[j]) ev[j][h] = d.synb[P0[j] + lane + 64 * h];
          }
        }
        float gv[4][2];
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
          for (int h = 0; h < 2; ++h) {
            gv[j][h] = 0.0f;
            if (lane + 64 * h < LEN[j])
              gv[j][h] = gwin[(size_t)((int)(ev[j][h].x & d.dmask) - DLO[j]) * d.BN + (size_t)BASE[j] + (ev[j][h].x >> d.dbits)];
          }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          if (L[j] < 0) continue;
          float G = 0.0f;
#pragma unroll
          for (int h = 0; h < 2; ++h)
            if (lane + 64 * h < LEN[j]) {
              G += __uint_as_float(ev[j][h].y) * gv[j][h];
              unsafeAtomicAdd(&d.gsum[P0[j] + lane + 64 * h], gv[j][h]);
            }
          for (int q = 128 + lane; q < LEN[j]; q += 64) {
            const uint2 e = d.synb[P0[j] + q];
            const float x = gwin[(size_t)((int)(e.x & d.dmask) - DLO[j]) * d.BN + (size_t)BASE[j] + (e.x >> d.dbits)];
            G += __uint_as_float(e.y) * x;
            unsafeAtomicAdd(&d.gsum[P0[j] + q], x);
          }
          G = wave_sum_f(G);
          const long long GG = __shfl(g, L[j], 64);
          const int SL = __shfl(slot, L[j], 64);
          if (lane == 0) {
            float* ga = &d.Gacc[(size_t)SL * d.BN + GG];
            *ga += G;
          }
        }
      }
    }
  }
}

// grad_w[p] = f_p * gsum, grad_d[p] = a_p * dscale * gsum, back in the caller's synapse order.
__global__ __launch_bounds__(kBlock) void k_grad_finish(Dev d, float dscale, float* __restrict__ grad_w,
                                                        float* __restrict__ grad_d) {
  for (long long i = blockIdx.x; i < d.N; i += gridDim.x) {
    const long long r0 = d.row_ptr[i], r1 = d.row_ptr[i + 1];
    for (long long q = r0 + threadIdx.x; q < r1; q += kBlock) {
      const float gs = d.gsum[q];
      const long long p = r0 + d.perm[q];
      grad_w[p] = (d.continuous ? d.fdec[q] : 1.0f) * gs;
      grad_d[p] = __uint_as_float(d.synb[q].y) * dscale * gs;
    }
  }
}
