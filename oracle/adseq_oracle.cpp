// CPU oracle for delayed spike-event delivery with autodifferentiable queues.
//
// TEST INFRASTRUCTURE ONLY.  Nothing on the product path may include, link or
// call this file; only tests/, the smoke check and the benchmark's CPU-baseline
// leg use it.  It shares no code with the HIP library.
//
// What it is: a plain, slow, single-thread-per-trial, time-stepped simulator
// that keeps every in-flight event in one exact priority queue
// (std::priority_queue keyed by (arrival step, synapse index)), written from
// the paper's statement of the problem:
//   * an event emitted at t_pre with delay d is delivered at t_post = t_pre + d
//     (Section 3.2, eqs. 10-11), as a unit jump scaled by the synaptic weight
//     (Section 2.1 eq. 1; weighted events add linearly under the LTI
//     assumption, Section 4.3 "Ring");
//   * lossy queues refuse an incoming event when they are full (Section 4.3
//     "FIFORing", "SingleSpike(Hold)");
//   * spikes are threshold crossings H(U - theta) with the SuperSpike surrogate
//     derivative 1/(|x|+1)^2 (Section 2.2.1, eqs. 5-7);
//   * the delay gradient enters through d t_post / d d = 1 (eq. 13) and the
//     receive rule  dx+/dtheta = dx-/dtheta + (1/tau) dt_post/dtheta (eq. 17),
//     here scaled by the jump amplitude a because the jump is a, not 1;
//   * spike-time mode (no surrogate): the emission time of a spike depends on
//     the membrane value the step started from, dt_spk/dv = -1/vdot (Section 3.1
//     eq. 8), vdot from the first forward difference, 1 where that is 0 (the
//     spike-detection rule of Section 4.1).
//
// Readings of points the paper leaves open (all restated in the design notes):
//   step order      pop(n) -> drive -> LIF -> enqueue(arrival n + D), D >= 1
//   jump target     the membrane state itself (delta-current synapse), so the
//                   tau of eq. 17 is tau_m
//   accumulation    amplitudes are summed as 32-bit fixed point (Q8.24, wrapping
//                   add) so the sum does not depend on order; converted to
//                   float once per neuron and step
//   bounded queues  a per-target bounded bag: pop removes every event due now;
//                   an incoming event is refused iff the target already holds
//                   `capacity` undelivered events at that point of the canonical
//                   order (step, source index, position in the row)
//   per-synapse     kind 3: the paper's own organisation (Section 4.1 listing 1:
//                   one queue per synapse; Section 4.3 "FIFORing(n)",
//                   "SingleSpike(Hold)" = capacity 1): an incoming event is
//                   refused iff its own synapse already holds `capacity`
//                   undelivered events; all events of a synapse share one delay,
//                   so arrival order is emission order and an ordered queue
//                   ("SortedArray") gives the same result
//   latest spike    kind 4: one slot per synapse in which a new spike always takes
//                   the place of the one held (Section 4.3 "SingleSpike(Drop)"): the
//                   event that was held is lost (counted as dropped, never delivered)
//   time bins       kind 5: `capacity` bins per synapse, an event with arrival step k
//                   goes to bin k mod capacity and takes the place of whatever
//                   undelivered event is there (Section 4.3 "LossyRingDelay(n)": a ring
//                   shorter than the delay, which loses events that fall into the same
//                   bin; the paper does not say which of the two is lost -- a plain ring
//                   write keeps the newer, and with one bin that is exactly
//                   "SingleSpike(Drop)", as "FIFORing(1)" is "SingleSpike(Hold)")
//   continuous d    arrival D = max(1, ceil(d/dt)) steps, amplitude
//                   a = w * exp(-(D*dt - d)/tau_m)
//   backward        event-sparse: the queue term exists only for emitted spikes
//
// Parity pins (tests/test_oracle_*.py): brute-force I_j(n) = sum a_ij s_i(n-D_ij),
// D==1 sparse mat-vec, exactly-once delivery and weight conservation, closed-form
// LIF charge curve, one-synapse closed-form delay gradient, central finite
// differences on a frozen raster, forward-mode tangent vs reverse-mode
// dot-product identity (surrogate and spike-time modes), closed-form spike-time
// gradient along a three-neuron chain, bounded-bag replay, FIFO(1) == hold-one-spike.
// Unpinned: nothing in the forward pass; the surrogate-through-spike-count
// gradient is pinned only by the dot-product identity (a surrogate is not the
// derivative of anything finite differences can see).
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <queue>
#include <string>
#include <thread>
#include <vector>

extern "C" {

struct oracle_config {
  int32_t n_neurons, batch, d_max_steps, capacity;
  int32_t kind;        // 0 ring (lossless), 1 fifo (bounded), 2 sorted (bounded), 3 one bounded FIFO per synapse,
                       // 4 one slot per synapse that holds the latest spike, 5 `capacity` time bins per synapse
  int32_t n_steps;
  int32_t surrogate;   // 0 SuperSpike, 1 off (sigma' == 0), 2 spike-time gradient (no surrogate)
  int32_t exact_f64;   // 0: fp32 state + Q8.24 sums (the method), 1: fp64, no quantisation
  float dt_ms, tau_m_ms, v_thresh, v_reset, ext_rate_hz, ext_weight;
  uint64_t seed;
  int64_t n_synapses;
  const int64_t* row_ptr;
  const int32_t* col;
  const float* weight;
  const uint8_t* delay_steps;  // exactly one of delay_steps / delay_ms
  const float* delay_ms;
  const float* i_ext;          // [T,B,N] or NULL: extra input current
  const uint8_t* forced_spikes;  // [T,B,N] or NULL: spikes imposed instead of U >= theta
  int32_t log_events;          // keep delivered / dropped event logs
  int32_t keep_currents;       // keep the popped fixed-point sums per step
  int32_t n_threads;           // trials are spread over this many threads
  float tau_syn_ms;            // > 0: first-order synapse, the jump goes into a synaptic current state
                               // with this time constant (Section 2.1 eq. 1); 0: straight into the membrane
  float tau_rise_ms;           // > 0 (needs tau_syn_ms > tau_rise_ms and integer delays): double-exponential
                               // synapse built from two such states (Section 3.2, closing remark): A with
                               // tau_syn_ms, B with tau_rise_ms, both take every jump, isyn = A - B
  const char* progress_file;   // NULL, or a file that long runs append progress lines to (copied at the call)
};

}  // extern "C"

namespace {

struct Event {
  int32_t k;       // arrival step
  int64_t syn;     // global synapse index
  int32_t n_emit;  // emission step
  int64_t idx;     // its admission flag (kind 4 looks at it again when the event comes up)
};
struct Later {     // std::priority_queue is a max-heap: "less" = arrives later
  bool operator()(const Event& a, const Event& b) const {
    if (a.k != b.k) return a.k > b.k;
    return a.syn > b.syn;
  }
};

struct EventLog {
  std::vector<int64_t> syn;
  std::vector<int32_t> n_emit, k, b;
  void add(int64_t s, int32_t n, int32_t kk, int32_t bb) {
    syn.push_back(s); n_emit.push_back(n); k.push_back(kk); b.push_back(bb);
  }
  void append(const EventLog& o) {
    syn.insert(syn.end(), o.syn.begin(), o.syn.end());
    n_emit.insert(n_emit.end(), o.n_emit.begin(), o.n_emit.end());
    k.insert(k.end(), o.k.begin(), o.k.end());
    b.insert(b.end(), o.b.begin(), o.b.end());
  }
};

struct SpikeRec { int32_t n, i; int64_t ev_base; };

struct Trial {
  std::vector<SpikeRec> spikes;        // in emission order
  std::vector<uint8_t> admitted;       // one flag per emitted event, emission order
  EventLog delivered, dropped;
  int64_t enqueued = 0, n_dropped = 0, n_delivered = 0, in_flight = 0;
  int64_t sum_enq = 0, sum_drop = 0, sum_deliv = 0, sum_flight = 0;
  int32_t max_occ = 0;
};

// splitmix64 output function (Steele, Lea, Flood 2014).
inline uint64_t mix64(uint64_t z) {
  z ^= z >> 30; z *= 0xBF58476D1CE4E5B9ull;
  z ^= z >> 27; z *= 0x94D049BB133111EBull;
  z ^= z >> 31; return z;
}
// Counter-based Bernoulli source: 32 uniform bits for (seed, unit g, step n).
inline uint32_t drive_bits(uint64_t seed, uint64_t g, uint64_t n) {
  const uint64_t G = 0x9E3779B97F4A7C15ull;
  uint64_t z = mix64(seed + G * (g + 1));
  z = mix64(z + G * (n + 1));
  return (uint32_t)(z >> 32);
}

// exp(-x) for 0 <= x <= 1 as the degree-20 Taylor polynomial in Horner form
// with fused multiply-adds; coefficients 1/k! by the recurrence c_k = c_{k-1}/k.
// Fixed operation order so that any IEEE-754 double implementation agrees bit
// for bit (truncation error < 2e-20).
double exp_neg_taylor(double x) {
  double c[21]; c[0] = 1.0;
  for (int k = 1; k <= 20; ++k) c[k] = c[k - 1] / (double)k;
  const double y = -x;
  double r = c[20];
  for (int k = 19; k >= 0; --k) r = std::fma(r, y, c[k]);
  return r;
}

inline int32_t sat_i32(long long v) {
  if (v > 2147483647LL) return 2147483647;
  if (v < -2147483648LL) return (int32_t)(-2147483647 - 1);
  return (int32_t)v;
}

}  // namespace

struct oracle_run {
  oracle_config cfg;
  int status = 0;  // 0 ok, -1 invalid argument, -2 delay out of range
  // per-synapse static data
  std::vector<int32_t> D;       // arrival offset in steps
  std::vector<int32_t> a_q;     // Q8.24 amplitude
  std::vector<float> a_f, f_f;  // fp32 amplitude w*f and decay factor f
  std::vector<double> a_d, f_d; // exact amplitude and decay factor (fp64 mode)
  double alpha_d = 0; float alpha_f = 0; uint64_t p_thresh = 0;
  double alpha_s_d = 0; float alpha_s_f = 0;   // leak of the synaptic current state (0: no such state)
  double alpha_r_d = 0; float alpha_r_f = 0;   // leak of the second (fast) state of the double-exponential synapse
  double tau_rcv = 0;                          // time constant of the state that receives the jump
  // tape [T,B,N]
  std::vector<float> U; std::vector<double> U64; std::vector<uint8_t> S;
  std::vector<int32_t> Iq; std::vector<float> I;
  std::vector<Trial> trials;
  EventLog delivered, dropped;  // all trials concatenated
  std::string progress_file;    // empty: no progress lines
};

namespace {

int prepare_synapses(oracle_run& r) {
  const oracle_config& c = r.cfg;
  const int64_t S = c.n_synapses;
  if ((c.delay_steps == nullptr) == (c.delay_ms == nullptr)) return -1;
  r.D.resize(S); r.a_q.resize(S); r.a_f.resize(S); r.f_f.resize(S); r.a_d.resize(S); r.f_d.resize(S);
  const double dt = (double)c.dt_ms, tau = r.tau_rcv;
  for (int64_t p = 0; p < S; ++p) {
    const double w = (double)c.weight[p];
    double f = 1.0; int64_t D;
    if (c.delay_steps) {
      D = c.delay_steps[p];
      if (D < 1) return -2;
    } else {
      const double d = (double)c.delay_ms[p];
      if (!(d > 0.0)) return -2;
      D = (int64_t)std::ceil(d / dt);
      if (D < 1) D = 1;
      const double x = ((double)D * dt - d) / tau;  // time from true arrival to the grid step
      f = exp_neg_taylor(x);
    }
    if (D > c.d_max_steps) return -2;
    const double a = w * f;
    r.D[p] = (int32_t)D;
    r.a_d[p] = a; r.f_d[p] = f;
    r.a_q[p] = sat_i32(std::llrint(a * 16777216.0));
    r.a_f[p] = (float)a;
    r.f_f[p] = (float)f;
  }
  return 0;
}

using EventQueue = std::priority_queue<Event, std::vector<Event>, Later>;

// Queue discipline of kinds 0-2: one queue per TARGET neuron.  Kind 0 (ring) is unbounded; kinds 1
// (FIFO) and 2 (sorted) hold at most `capacity` events per target and refuse a newcomer while
// full (Section 4.3, "FIFORing": incoming spikes are dropped when the queue is full).  Both deliver
// at the arrival step, so the exact priority queue serves them; only the occupancy count differs
// from the ring.
struct TargetQueues {
  const oracle_run& r; const bool bounded; const int b;
  std::vector<int32_t> occ;   // events held per target
  TargetQueues(const oracle_run& run, int trial)
      : r(run), bounded(run.cfg.kind != 0), b(trial), occ((size_t)run.cfg.n_neurons, 0) {}
  // an event comes up at its arrival step: true = it is delivered
  bool arrive(Trial&, const Event& e) { occ[r.cfg.col[e.syn]] -= 1; return true; }
  // synapse p offers an event emitted at step n that arrives at step k
  void offer(Trial& tr, EventQueue& pq, int64_t p, int32_t n, int32_t k) {
    const oracle_config& c = r.cfg;
    const size_t j = (size_t)c.col[p];
    if (bounded && occ[j] >= c.capacity) {
      tr.admitted.push_back(0);
      tr.n_dropped += 1; tr.sum_drop += r.a_q[p];
      if (c.log_events) tr.dropped.add(p, n, k, b);
      return;
    }
    tr.admitted.push_back(1);
    occ[j] += 1;
    tr.max_occ = std::max(tr.max_occ, occ[j]);
    pq.push(Event{k, p, n, (int64_t)tr.admitted.size() - 1});
  }
  bool counts_at_end(const Trial&, const Event&) const { return true; }
};

// Queue disciplines of kinds 3-5: one queue per SYNAPSE (Section 4.3, the per-synapse variants).
// Kind 3: a FIFO of `capacity` events per synapse, a full one refuses the newcomer.
// Kinds 4 and 5: the newest event replaces the one held in its slot, and the replaced one is
// lost: kind 4 has one slot per synapse, kind 5 `capacity` bins chosen by arrival step mod capacity.
// A replaced event stays in the priority queue with its admission flag cleared and is skipped
// when it comes up.
struct SynapseQueues {
  const oracle_run& r; const int b;
  const bool latest; const int nbins;
  std::vector<int32_t> occ;      // kind 3: events held per synapse
  std::vector<int64_t> held;     // kinds 4, 5: admission flag of the event held per (synapse, bin), -1 = none
  std::vector<int32_t> held_n;   // its emission step
  SynapseQueues(const oracle_run& run, int trial)
      : r(run), b(trial), latest(run.cfg.kind == 4 || run.cfg.kind == 5),
        nbins(run.cfg.kind == 5 ? run.cfg.capacity : 1),
        occ(latest ? (size_t)0 : (size_t)run.cfg.n_synapses, 0),
        held(latest ? (size_t)run.cfg.n_synapses * nbins : 0, -1),
        held_n(latest ? (size_t)run.cfg.n_synapses * nbins : 0, 0) {}
  bool arrive(Trial& tr, const Event& e) {
    if (latest) {
      if (!tr.admitted[e.idx]) return false;     // it was replaced while in transit
      held[(size_t)e.syn * nbins + e.k % nbins] = -1;
    } else {
      occ[(size_t)e.syn] -= 1;
    }
    return true;
  }
  void offer(Trial& tr, EventQueue& pq, int64_t p, int32_t n, int32_t k) {
    const oracle_config& c = r.cfg;
    if (latest) {
      const size_t hb = (size_t)p * nbins + k % nbins;
      if (held[hb] >= 0) {                 // the event held there so far is lost
        tr.admitted[held[hb]] = 0;
        tr.n_dropped += 1; tr.sum_drop += r.a_q[p];
        if (c.log_events) tr.dropped.add(p, held_n[hb], held_n[hb] + r.D[p], b);
      }
      held[hb] = (int64_t)tr.admitted.size(); held_n[hb] = n;
      tr.admitted.push_back(1);
      tr.max_occ = std::max(tr.max_occ, 1);
      pq.push(Event{k, p, n, held[hb]});
      return;
    }
    if (occ[(size_t)p] >= c.capacity) {
      tr.admitted.push_back(0);
      tr.n_dropped += 1; tr.sum_drop += r.a_q[p];
      if (c.log_events) tr.dropped.add(p, n, k, b);
      return;
    }
    tr.admitted.push_back(1);
    occ[(size_t)p] += 1;
    tr.max_occ = std::max(tr.max_occ, occ[(size_t)p]);
    pq.push(Event{k, p, n, (int64_t)tr.admitted.size() - 1});
  }
  bool counts_at_end(const Trial& tr, const Event& e) const { return !latest || tr.admitted[e.idx]; }
};

// State of one trial's neurons between steps: membrane value and the synaptic current state(s),
// in fp32 (the arithmetic the method is compared in) and in fp64 (exact_f64 runs).
struct NeuronState {
  std::vector<float> V, J, J2;
  std::vector<double> V64, J64, J264;
  explicit NeuronState(int N) : V(N, 0.0f), J(N, 0.0f), J2(N, 0.0f), V64(N, 0.0), J64(N, 0.0), J264(N, 0.0) {}
};

// Steps (2) and (3) of a time step for every neuron of trial b: drive, synapse model, leaky
// integration, threshold and reset (Section 2.1 eqs. 1-3 on the grid of Section 3.2 eqs. 10-11).
// acc / acc64: what step (1) popped for each neuron (Q8.24 sum / exact sum).  Records the tape
// row and appends the neurons that spiked to `fired` in ascending order.
void step_neurons(oracle_run& r, int b, int n, const std::vector<int32_t>& acc, const std::vector<double>& acc64,
                  NeuronState& st, std::vector<int32_t>& fired) {
  const oracle_config& c = r.cfg;
  const int N = c.n_neurons, B = c.batch;
  const bool exact = c.exact_f64 != 0;
  const bool dexp = c.tau_rise_ms > 0.0f;          // two states A = J, B = J2; isyn = A - B
  const bool syn_state = c.tau_syn_ms > 0.0f;
  const size_t base = ((size_t)n * B + b) * N;
  std::vector<float>& V = st.V; std::vector<float>& J = st.J; std::vector<float>& J2 = st.J2;
  std::vector<double>& V64 = st.V64; std::vector<double>& J64 = st.J64; std::vector<double>& J264 = st.J264;
  fired.clear();
  for (int j = 0; j < N; ++j) {
    const bool xi = (uint64_t)drive_bits(c.seed, (uint64_t)b * N + j, (uint64_t)n) < r.p_thresh;
    bool s;
    if (!exact) {
      float I = (float)acc[j] * 0x1p-24f;
      if (dexp) {
        const float jump = I;
        J[j] = std::fmaf(r.alpha_s_f, J[j], jump); J2[j] = std::fmaf(r.alpha_r_f, J2[j], jump);
        I = J[j] - J2[j];
      } else if (syn_state) { I = std::fmaf(r.alpha_s_f, J[j], I); J[j] = I; }   // isyn = alpha_s isyn + jumps
      I = I + (xi ? c.ext_weight : 0.0f);
      if (c.i_ext) I = I + c.i_ext[base + j];
      const float u = std::fmaf(r.alpha_f, V[j], I);
      s = c.forced_spikes ? (c.forced_spikes[base + j] != 0) : (u >= c.v_thresh);
      V[j] = s ? c.v_reset : u;
      r.U[base + j] = u; r.I[base + j] = I;
    } else {
      double I = acc64[j];
      if (dexp) {
        const double jump = I;
        J64[j] = r.alpha_s_d * J64[j] + jump; J264[j] = r.alpha_r_d * J264[j] + jump;
        I = J64[j] - J264[j];
      } else if (syn_state) { I = r.alpha_s_d * J64[j] + I; J64[j] = I; }
      I += xi ? (double)c.ext_weight : 0.0;
      if (c.i_ext) I += (double)c.i_ext[base + j];
      const double u = r.alpha_d * V64[j] + I;
      s = c.forced_spikes ? (c.forced_spikes[base + j] != 0) : (u >= (double)c.v_thresh);
      V64[j] = s ? (double)c.v_reset : u;
      r.U64[base + j] = u; r.U[base + j] = (float)u; r.I[base + j] = (float)I;
    }
    r.S[base + j] = s ? 1 : 0;
    if (c.keep_currents) r.Iq[base + j] = acc[j];
    if (s) fired.push_back(j);
  }
}

// One trial, forward: the event-driven simulation with one exact priority queue keyed by
// (arrival step, synapse).  Per time step: (1) pop every event whose arrival step is n, (2) drive
// and (3) LIF for every neuron, (4) fan the step's spikes out in ascending (source, row position)
// order, each synapse offering its event to the queue discipline Q.
template <class Q>
void run_trial(oracle_run& r, int b) {
  const oracle_config& c = r.cfg;
  const int N = c.n_neurons, T = c.n_steps, B = c.batch;
  Trial& tr = r.trials[b];
  EventQueue pq;
  Q queues(r, b);
  NeuronState state(N);
  std::vector<int32_t> acc(N);
  std::vector<double> acc64(N);
  std::vector<int32_t> fired;

  // Long runs say how far they are: a line per 50 steps of trial 0 appended to the progress file
  // of the call, if it names one (a run of the largest configuration takes minutes).  (The path
  // comes with the call and not from the environment: reading the environment here, in a thread,
  // while another thread of the process changes it is a crash waiting to happen.)
  FILE* progress = nullptr;
  if (b == 0 && !r.progress_file.empty()) progress = fopen(r.progress_file.c_str(), "a");

  for (int n = 0; n < T; ++n) {
    if (progress && n % 50 == 0) { fprintf(progress, "oracle run: kind %d, N %d, step %d of %d\n", c.kind, N, n, T); fflush(progress); }
    // (1) pop every event whose arrival step is n
    std::fill(acc.begin(), acc.end(), 0);
    std::fill(acc64.begin(), acc64.end(), 0.0);
    while (!pq.empty() && pq.top().k == n) {
      const Event e = pq.top(); pq.pop();
      if (!queues.arrive(tr, e)) continue;
      const int j = c.col[e.syn];
      acc[j] = (int32_t)((uint32_t)acc[j] + (uint32_t)r.a_q[e.syn]);  // wrapping add
      acc64[j] += r.a_d[e.syn];
      tr.n_delivered += 1; tr.sum_deliv += r.a_q[e.syn];
      if (c.log_events) tr.delivered.add(e.syn, e.n_emit, e.k, b);
    }
    // (2) drive and (3) LIF
    step_neurons(r, b, n, acc, acc64, state, fired);
    // (4) fan out the spikes of this step in ascending (source, row position) order
    for (int i : fired) {
      SpikeRec rec{n, i, (int64_t)tr.admitted.size()};
      tr.spikes.push_back(rec);
      for (int64_t p = c.row_ptr[i]; p < c.row_ptr[i + 1]; ++p) {
        tr.enqueued += 1; tr.sum_enq += r.a_q[p];
        queues.offer(tr, pq, p, n, n + r.D[p]);
      }
    }
  }
  if (progress) fclose(progress);
  if (b > 0 && !r.progress_file.empty())   // the other trials of a batch say when they are done
    if (FILE* f = fopen(r.progress_file.c_str(), "a")) { fprintf(f, "oracle run: kind %d, N %d, trial %d of %d done\n", c.kind, N, b, B); fclose(f); }
  tr.in_flight = 0;
  while (!pq.empty()) {
    if (queues.counts_at_end(tr, pq.top())) { tr.in_flight += 1; tr.sum_flight += r.a_q[pq.top().syn]; }
    pq.pop();
  }
}

void run_trial(oracle_run& r, int b) {
  if (r.cfg.kind <= 2) run_trial<TargetQueues>(r, b);
  else run_trial<SynapseQueues>(r, b);
}

// Reverse-time sweep for one trial; adds this trial's contribution to gw, gd.
void backward_trial(const oracle_run& r, int b, const float* dL_dcount, const float* dL_dU,
                    std::vector<double>& gw, std::vector<double>& gd, double* gU_out) {
  const oracle_config& c = r.cfg;
  const int N = c.n_neurons, T = c.n_steps, B = c.batch;
  const bool exact = c.exact_f64 != 0;
  const Trial& tr = r.trials[b];
  const double tau = r.tau_rcv, theta = (double)c.v_thresh;
  // gradient per unit the delay was given in: ms, or steps of dt ms
  const double d_unit = c.delay_ms ? 1.0 : (double)c.dt_ms;
  // dU[n+1]/dV[n]: the leak factor the forward pass actually multiplied by
  const double alpha = exact ? r.alpha_d : (double)r.alpha_f;
  // gU[n][i] = dL/dU_i[n], with gU[T] == 0.  carry[i] = dL/dV_i[n] = what reaches the membrane
  // state that step n left behind: alpha gU[n+1], plus, in the spike-time mode, the cotangent
  // that the emission time of a spike at n+1 hands to the state it started from.
  std::vector<double> gU((size_t)(T + 1) * N, 0.0);
  std::vector<double> carry(N, 0.0);
  // gR[n][j]: what an event delivered to j at step n gathers = dL/d(state that received the jump):
  // dL/dU_j[n] without a synaptic current state; with one, dL/dJ_j[n] = gU_j[n] + alpha_s dL/dJ_j[n+1]
  std::vector<double> gR((size_t)(T + 1) * N, 0.0);
  const double alpha_s = exact ? r.alpha_s_d : (double)r.alpha_s_f;
  // Double-exponential synapse: every event jumps into two states, A (tau_syn) and B (tau_rise),
  // and isyn = A - B.  dL/dA[n] = gU[n] + alpha_s dL/dA[n+1], dL/dB[n] = -gU[n] + alpha_r dL/dB[n+1].
  // An event delivered at k gathers gX = dL/dA[k] + dL/dB[k] for its amplitude, and, by the receive
  // rule applied to each state with its own time constant, gY = dL/dA[k]/tau_A + dL/dB[k]/tau_B for
  // its arrival time.
  const bool dexp = c.tau_rise_ms > 0.0f;
  const double alpha_r = exact ? r.alpha_r_d : (double)r.alpha_r_f;
  const double tau_a = (double)c.tau_syn_ms, tau_b = (double)c.tau_rise_ms;
  std::vector<double> gA(dexp ? N : 0, 0.0), gB(dexp ? N : 0, 0.0);
  std::vector<double> gY(dexp ? (size_t)(T + 1) * N : 0, 0.0);   // (gX is kept in gR)
  int64_t sp = (int64_t)tr.spikes.size() - 1;  // spikes are stored in emission order
  std::vector<double> G(N);
  const bool spike_time = c.surrogate == 2;
  for (int n = T - 1; n >= 0; --n) {
    const size_t base = ((size_t)n * B + b) * N;
    std::fill(G.begin(), G.end(), 0.0);
    // queue term: only neurons that emitted a spike at n have events to carry a cotangent
    while (sp >= 0 && tr.spikes[sp].n == n) {
      const SpikeRec& rec = tr.spikes[sp];
      const int i = rec.i;
      double g_sum = 0.0;
      for (int64_t p = c.row_ptr[i]; p < c.row_ptr[i + 1]; ++p) {
        if (!tr.admitted[rec.ev_base + (p - c.row_ptr[i])]) continue;
        const int k = n + r.D[p];
        if (k >= T) continue;  // never delivered inside the run
        const double g = gR[(size_t)k * N + c.col[p]];
        const double a = exact ? r.a_d[p] : (double)r.a_f[p];
        const double f = exact ? r.f_d[p] : (double)r.f_f[p];
        if (dexp) {
          const double gy = gY[(size_t)k * N + c.col[p]];
          g_sum += a * (spike_time ? gy : g);   // what the emitting spike's time (value) is worth
          gw[p] += f * g;
          gd[p] += a * d_unit * gy;
          continue;
        }
        g_sum += a * g;
        gw[p] += f * g;                   // dI/dw = f (amplitude a = w f)
        gd[p] += (a / tau) * d_unit * g;  // receive rule: (jump / tau) * dt_post/dd, dt_post/dd = 1
      }
      G[i] = g_sum;
      --sp;
    }
    for (int i = 0; i < N; ++i) {
      const double u = exact ? r.U64[base + i] : (double)r.U[base + i];
      const double s = r.S[base + i] ? 1.0 : 0.0;
      const double x = u - theta;
      const double sg = c.surrogate == 0 ? 1.0 / ((std::fabs(x) + 1.0) * (std::fabs(x) + 1.0)) : 0.0;
      const double direct = dL_dU ? (double)dL_dU[base + i] : 0.0;
      const double dc = dL_dcount ? (double)dL_dcount[(size_t)b * N + i] : 0.0;
      const double g_now = (1.0 - s) * carry[i] + sg * (dc + s * G[i]) + direct;
      gU[(size_t)n * N + i] = g_now;
      if (dexp) {
        gA[i] = g_now + alpha_s * gA[i];
        gB[i] = -g_now + alpha_r * gB[i];
        gR[(size_t)n * N + i] = gA[i] + gB[i];
        gY[(size_t)n * N + i] = gA[i] / tau_a + gB[i] / tau_b;
      } else {
        gR[(size_t)n * N + i] = g_now + alpha_s * gR[(size_t)(n + 1) * N + i];
      }
      // Spike-time mode: the spike's emission time depends on the membrane value v the step
      // started from, dt_spk/dv = -1 / vdot with vdot = (U - v) / dt from the first forward
      // difference (1 where that is 0), and every event of the spike hands (jump / tau) dt_post
      // to its receiver, dt_post/dt_spk = 1: the state before the step gets -(1/vdot)(1/tau) G.
      double e = 0.0;
      if (spike_time && s != 0.0) {
        double vprev = 0.0;   // V starts at 0
        if (n > 0) {
          const size_t pb = ((size_t)(n - 1) * B + b) * N + i;
          vprev = r.S[pb] ? (double)c.v_reset : (exact ? r.U64[pb] : (double)r.U[pb]);
        }
        double vdot = (u - vprev) / (double)c.dt_ms;
        if (vdot == 0.0) vdot = 1.0;
        e = dexp ? -(1.0 / vdot) * G[i] : -(1.0 / vdot) * (1.0 / tau) * G[i];   // (gY holds the 1/tau factors)
      }
      carry[i] = alpha * g_now + e;
    }
  }
  if (gU_out)
    for (int n = 0; n < T; ++n)
      std::memcpy(gU_out + ((size_t)n * B + b) * N, &gU[(size_t)n * N], sizeof(double) * N);
}

}  // namespace

extern "C" {

// Runs the forward simulation; the returned object owns the tape and logs.
oracle_run* oracle_forward(const oracle_config* cfg) {
  oracle_run* r = new oracle_run();
  r->cfg = *cfg;
  if (cfg->progress_file) r->progress_file = cfg->progress_file;
  r->cfg.progress_file = nullptr;   // (the caller's string need not outlive the call)
  const oracle_config& c = r->cfg;
  if (c.n_neurons < 1 || c.batch < 1 || c.n_steps < 0 || c.d_max_steps < 1 ||
      (c.kind != 0 && c.capacity < 1) || c.kind < 0 || c.kind > 5 ||
      !(c.dt_ms > 0.0f) || !(c.tau_m_ms > 0.0f) || c.dt_ms > c.tau_m_ms) {
    r->status = -1; return r;
  }
  if (c.tau_syn_ms < 0.0f || (c.tau_syn_ms > 0.0f && c.dt_ms > c.tau_syn_ms)) { r->status = -1; return r; }
  if (c.tau_rise_ms < 0.0f ||
      (c.tau_rise_ms > 0.0f && (c.dt_ms > c.tau_rise_ms || !(c.tau_syn_ms > c.tau_rise_ms) || c.delay_ms))) {
    r->status = -1; return r;   // the two states would decay a sub-step arrival differently: integer delays only
  }
  r->tau_rcv = c.tau_syn_ms > 0.0f ? (double)c.tau_syn_ms : (double)c.tau_m_ms;
  r->status = prepare_synapses(*r);
  if (r->status != 0) return r;
  r->alpha_d = std::exp(-(double)c.dt_ms / (double)c.tau_m_ms);
  r->alpha_f = (float)r->alpha_d;
  if (c.tau_syn_ms > 0.0f) {
    r->alpha_s_d = std::exp(-(double)c.dt_ms / (double)c.tau_syn_ms);
    r->alpha_s_f = (float)r->alpha_s_d;
  }
  if (c.tau_rise_ms > 0.0f) {
    r->alpha_r_d = std::exp(-(double)c.dt_ms / (double)c.tau_rise_ms);
    r->alpha_r_f = (float)r->alpha_r_d;
  }
  {
    // Bernoulli probability per step rate*dt, as a 32-bit threshold
    double p = (double)c.ext_rate_hz * (double)c.dt_ms * 1e-3;
    if (p < 0.0) p = 0.0;
    if (p > 1.0) p = 1.0;
    r->p_thresh = (uint64_t)std::floor(p * 4294967296.0);
  }
  const size_t tot = (size_t)c.n_steps * c.batch * c.n_neurons;
  r->U.assign(tot, 0.0f); r->S.assign(tot, 0); r->I.assign(tot, 0.0f);
  if (c.exact_f64) r->U64.assign(tot, 0.0);
  if (c.keep_currents) r->Iq.assign(tot, 0);
  r->trials.resize(c.batch);
  const int nt = std::max(1, std::min(c.n_threads, c.batch));
  if (nt == 1) {
    for (int b = 0; b < c.batch; ++b) run_trial(*r, b);
  } else {
    std::vector<std::thread> th;
    for (int t = 0; t < nt; ++t)
      th.emplace_back([r, t, nt]() {
        for (int b = t; b < r->cfg.batch; b += nt) run_trial(*r, b);
      });
    for (auto& x : th) x.join();
  }
  if (c.log_events)
    for (int b = 0; b < c.batch; ++b) {
      r->delivered.append(r->trials[b].delivered);
      r->dropped.append(r->trials[b].dropped);
    }
  return r;
}

int oracle_status(const oracle_run* r) { return r->status; }
const float* oracle_U(const oracle_run* r) { return r->U.data(); }
const double* oracle_U64(const oracle_run* r) { return r->U64.data(); }
const uint8_t* oracle_S(const oracle_run* r) { return r->S.data(); }
const float* oracle_I(const oracle_run* r) { return r->I.data(); }
const int32_t* oracle_Iq(const oracle_run* r) { return r->Iq.data(); }
const int32_t* oracle_D(const oracle_run* r) { return r->D.data(); }
const int32_t* oracle_aq(const oracle_run* r) { return r->a_q.data(); }
const float* oracle_af(const oracle_run* r) { return r->a_f.data(); }
const float* oracle_ff(const oracle_run* r) { return r->f_f.data(); }
const double* oracle_ad(const oracle_run* r) { return r->a_d.data(); }

// counters[0..8]: enqueued (attempted), dropped, delivered, in flight at the end,
// the same four as sums of Q8.24 amplitudes, and the largest occupancy any target reached.
void oracle_counters(const oracle_run* r, int64_t* out) {
  for (int k = 0; k < 9; ++k) out[k] = 0;
  for (const Trial& t : r->trials) {
    out[0] += t.enqueued; out[1] += t.n_dropped; out[2] += t.n_delivered; out[3] += t.in_flight;
    out[4] += t.sum_enq; out[5] += t.sum_drop; out[6] += t.sum_deliv; out[7] += t.sum_flight;
    out[8] = std::max<int64_t>(out[8], t.max_occ);
  }
}

// which = 0 delivered, 1 dropped.  Returns the number of events; pointers stay
// valid until oracle_free.
int64_t oracle_event_log(const oracle_run* r, int which, const int64_t** syn,
                         const int32_t** n_emit, const int32_t** k, const int32_t** b) {
  const EventLog& L = which == 0 ? r->delivered : r->dropped;
  *syn = L.syn.data(); *n_emit = L.n_emit.data(); *k = L.k.data(); *b = L.b.data();
  return (int64_t)L.syn.size();
}

// Reverse-mode gradients (fp64).  dL_dcount [B,N] or NULL, dL_dU [T,B,N] or NULL;
// grad_w, grad_d [S] are overwritten; gU_out [T,B,N] or NULL receives dL/dU.
int oracle_backward(const oracle_run* r, const float* dL_dcount, const float* dL_dU,
                    double* grad_w, double* grad_d, double* gU_out) {
  if (r->status != 0) return r->status;
  const int64_t S = r->cfg.n_synapses;
  std::vector<double> gw(S, 0.0), gd(S, 0.0);
  const bool say = r->cfg.batch > 1 && !r->progress_file.empty();
  for (int b = 0; b < r->cfg.batch; ++b) {
    backward_trial(*r, b, dL_dcount, dL_dU, gw, gd, gU_out);
    if (say)
      if (FILE* f = fopen(r->progress_file.c_str(), "a")) { fprintf(f, "oracle reverse sweep: trial %d of %d done\n", b, r->cfg.batch); fclose(f); }
  }
  std::memcpy(grad_w, gw.data(), sizeof(double) * S);
  std::memcpy(grad_d, gd.data(), sizeof(double) * S);
  return 0;
}

double oracle_exp_neg(double x) { return exp_neg_taylor(x); }
uint32_t oracle_drive_bits(uint64_t seed, uint64_t g, uint64_t n) { return drive_bits(seed, g, n); }
uint64_t oracle_mix64(uint64_t z) { return mix64(z); }

void oracle_free(oracle_run* r) { delete r; }

}  // extern "C"
