/* adseq.h -- C ABI of the MI355X (gfx950) delayed spike-event delivery library.
 *
 * The library runs, per time step, the hot path of autodifferentiable
 * spike-event queues: pop the events due now, add the external drive, update
 * the LIF state, compact the neurons that spiked, fan each spike out over its
 * CSR row and enqueue the events at (step + delay); and, afterwards, the
 * reverse-time sweep that yields weight and delay gradients.
 *
 * Conventions for every entry point
 *   - returns ADSEQ_OK (0) or a negative ADSEQ_E_* code; never throws or aborts;
 *     on error the outputs are left untouched and the handle stays usable;
 *   - every array argument is a DEVICE pointer owned by the caller unless the
 *     comment says "host"; the library never allocates device memory and never
 *     creates streams: all state lives in the caller's workspace and all work
 *     is launched on the `stream` argument (a hipStream_t passed as void*,
 *     NULL = the default stream) without synchronising, except where stated;
 *   - one handle = one network x `batch` independent trials; a handle is not
 *     thread safe; neuron (b, i) has flat index b * n_neurons + i;
 *   - steps are numbered 0, 1, 2, ... and must be issued in that order.
 *
 * Semantics of one step n (Section 3.2 eqs. 10-11: an event emitted at t_pre with
 * delay d is delivered at t_post = t_pre + d; Section 4.1 listing "Synapse
 * implementation": detect, enqueue, pop, integrate):
 *   1. pop     Iq_j = sum of the amplitudes of the stored events with arrival
 *              step n and target j (summed as 32-bit fixed point Q8.24, so the
 *              result does not depend on the order of arrival);
 *   2. drive   I_j = Iq_j * 2^-24 + (xi_j ? ext_weight : 0) (+ i_ext_j)   [with tau_syn_ms > 0:
 *              J_j = fma(alpha_s, J_j, Iq_j * 2^-24), alpha_s = (float)exp(-dt/tau_syn), takes the
 *              place of Iq_j * 2^-24; with tau_rise_ms > 0 as well, J_j - B_j does,
 *              B_j = fma(alpha_r, B_j, Iq_j * 2^-24), alpha_r = (float)exp(-dt/tau_rise)], xi_j a
 *              Bernoulli(ext_rate_hz * dt) draw from a counter-based hash of
 *              (seed, b * N + j, n);
 *   3. LIF     U_j = fma(alpha, V_j, I_j), alpha = (float)exp(-dt/tau_m);
 *              s_j = U_j >= v_thresh (Heaviside, eq. 6); V_j = s_j ? v_reset : U_j;
 *   4. enqueue for every spiking i and every synapse p of row i: an event with
 *              target col[p], arrival n + D_p and amplitude a_p.
 *   Integer delays: D_p = delay_steps[p], a_p = weight[p].  Continuous delays:
 *   D_p = max(1, ceil(delay_ms[p] / dt)), a_p = weight[p] * exp(-(D_p dt - delay_ms[p]) / tau),
 *   tau = the time constant of the state that takes the jump (tau_syn_ms if > 0, else tau_m_ms).
 *
 * Queue kinds (Section 4.3)
 *   ADSEQ_RING    dense delay line: one summed cell per (arrival step, target) for
 *                 the arrival steps of the current window of 16 steps, plus the
 *                 spikes of the last d_max_steps + 1 steps as bit masks, from
 *                 which the cells of the next window are filled when it opens;
 *                 lossless ("Ring").
 *   ADSEQ_FIFO    per target, `capacity` unordered slots; an incoming event is
 *                 dropped (and counted) when the target already holds `capacity`
 *                 undelivered events (the rule of the paper's "FIFORing": a full
 *                 queue refuses what comes in); every stored event is delivered
 *                 exactly at its arrival step.
 *   ADSEQ_SORTED  per target, `capacity` slots kept ordered by arrival step; pop
 *                 takes from the front ("SortedArray"); same admission rule.
 *   ADSEQ_SYN_FIFO one first-in-first-out queue of `capacity` (1..8) arrival times per
 *                 synapse and trial, the organisation of Section 4.1 (one queue per
 *                 synapse; "FIFORing(n)", capacity 1 = "SingleSpike(Hold)"): an incoming
 *                 event is dropped (and counted) when its own synapse already holds
 *                 `capacity` undelivered events.  All events of a synapse share one
 *                 delay, so arrival order is emission order and an ordered queue
 *                 ("SortedArray") behaves the same.  Every queue is looked at in every
 *                 step (the cost the per-target kinds avoid); state: 2 capacity + 4
 *                 bytes per synapse and trial.
 *   ADSEQ_SYN_LATEST one slot per synapse and trial in which a new spike always takes the place
 *                 of the one held ("SingleSpike(Drop)"): the event that was held is lost --
 *                 counted as dropped, never delivered, its admission flag on the tape
 *                 cleared.  capacity must be 1.  State: 2 bytes per synapse and trial.
 *   ADSEQ_SYN_BINS `capacity` (1..8) time bins per synapse and trial: an event with arrival step k
 *                 goes to bin k mod capacity and takes the place of whatever undelivered
 *                 event is there, which is lost ("LossyRingDelay(n)", a ring shorter than the
 *                 delay, read as a ring of arrival times in which a write keeps the newer
 *                 event; one bin is ADSEQ_SYN_LATEST).  State: 2 capacity bytes per synapse
 *                 and trial, with a tape 8 capacity more (where each held event's flag is).
 *   Admission order within a step is canonical: ascending global synapse index
 *   (= ascending source neuron, then position in the row), independently per trial.
 */
#ifndef ADSEQ_H
#define ADSEQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct adseq adseq_t; /* opaque; host memory owned by the library, freed by adseq_destroy */

enum { ADSEQ_RING = 0, ADSEQ_FIFO = 1, ADSEQ_SORTED = 2, ADSEQ_SYN_FIFO = 3, ADSEQ_SYN_LATEST = 4, ADSEQ_SYN_BINS = 5 };
/* How a spike passes gradients back (config field `surrogate`):
 *   ADSEQ_SURR_SUPERSPIKE  the spike function has the SuperSpike derivative 1/(|U - theta| + 1)^2 (eq. 7);
 *   ADSEQ_SURR_OFF         it has derivative 0 (only the direct dependence of amplitudes on weights
 *                          and delays remains);
 *   ADSEQ_GRAD_SPIKE_TIME  no surrogate: the emission time of a spike depends on the membrane value
 *                          v its step started from, dt_spk/dv = -1 / vdot (Section 3.1 eq. 8), vdot =
 *                          (U - v) / dt from the first forward difference, 1 where that is 0 (the
 *                          spike-detection rule of Section 4.1), and every event of the spike hands
 *                          (amplitude / tau_m) dt_post to its receiver (eq. 17), dt_post/dt_spk = 1
 *                          (eq. 13).  dL_dcount is ignored in this mode. */
enum { ADSEQ_SURR_SUPERSPIKE = 0, ADSEQ_SURR_OFF = 1, ADSEQ_GRAD_SPIKE_TIME = 2 };

enum {
  ADSEQ_OK = 0,
  ADSEQ_E_INVALID_ARG = -1, /* null pointer, non-positive size, unknown enum, dt > tau_m ...    */
  ADSEQ_E_DELAY_RANGE = -2, /* a delay below one step (or <= 0 ms) or above d_max_steps         */
  ADSEQ_E_WORKSPACE = -3,   /* workspace missing, misaligned (256 B) or smaller than required   */
  ADSEQ_E_ORDER = -4,       /* step issued out of order                                         */
  ADSEQ_E_NO_TAPE = -5,     /* backward without a complete recorded forward run                 */
  ADSEQ_E_HIP = -6,         /* a HIP call failed; adseq_last_error has the text                 */
  ADSEQ_E_CAPACITY = -7,    /* tape (steps, spikes, events) or per-step contender pool overflow */
  ADSEQ_E_GRAPH = -8,       /* CSR malformed: row_ptr not monotone from 0 to n_synapses, or a
                               column index outside [0, n_neurons)                             */
  ADSEQ_E_HOST_MEMORY = -9  /* the host-side handle could not be allocated                     */
};

typedef struct {
  int32_t n_neurons;    /* N >= 1                                                             */
  int32_t batch;        /* B >= 1 independent trials sharing the network                      */
  int32_t d_max_steps;  /* largest arrival offset in steps, 1..1023                           */
  int32_t capacity;     /* slots per target for FIFO / SORTED (1..32767), per synapse for
                           SYN_FIFO and SYN_BINS (1..8), 1 for SYN_LATEST; ignored for RING   */
  int32_t kind;         /* ADSEQ_RING / _FIFO / _SORTED / _SYN_FIFO / _SYN_LATEST / _SYN_BINS   */
  int32_t surrogate;    /* ADSEQ_SURR_SUPERSPIKE / ADSEQ_SURR_OFF / ADSEQ_GRAD_SPIKE_TIME      */
  int32_t record_tape;  /* 1 = adseq_step keeps what adseq_backward needs                     */
  int32_t max_steps;    /* tape length in steps (needed when record_tape = 1)                 */
  float dt_ms, tau_m_ms, v_thresh, v_reset; /* LIF; requires 0 < dt_ms <= tau_m_ms            */
  float ext_rate_hz, ext_weight;            /* Poisson drive, 0 rate = none                   */
  float tau_syn_ms;                         /* > 0: first-order synapse (Section 2.1 eq. 1): the events
                                               jump into a synaptic current state J with this time
                                               constant (dt_ms <= tau_syn_ms), J <- alpha_s J + Iq,
                                               and J is what the membrane integrates; 0: the events
                                               jump straight into the membrane state               */
  float tau_rise_ms;                        /* > 0: double-exponential synapse (Section 3.2, closing
                                               remark): a second, faster state B with this time
                                               constant takes every jump too, B <- alpha_r B + Iq,
                                               and the membrane integrates J - B; needs
                                               dt_ms <= tau_rise_ms < tau_syn_ms and whole-step
                                               delays (delay_steps); 0: none                       */
  uint64_t seed;                            /* of the drive's counter-based generator         */
  int64_t n_synapses;                       /* S = row_ptr[N], below 2^40                     */
  const int64_t *row_ptr;     /* [N+1] CSR by source neuron                                   */
  const int32_t *col;         /* [S] target neuron                                            */
  const float *weight;        /* [S] finite fp32; |amplitude| saturates at 128                */
  const uint8_t *delay_steps; /* [S] integer delays in steps, or NULL                         */
  const float *delay_ms;      /* [S] continuous delays in ms, or NULL (exactly one is given;
                                 with S = 0 the four per-synapse arrays may all be NULL)       */
  /* The four arrays above must stay valid and unchanged for the life of the handle. */
  int64_t tape_spike_capacity; /* FIFO/SORTED with tape: spikes the tape's spike list can hold
                                  in total; 0 = default (max_steps * B * N / 16 + B * N)      */
  int64_t tape_event_capacity; /* FIFO/SORTED with tape: emitted events it can hold (one
                                  admission flag each); 0 = default
                                  (tape_spike_capacity * ceil(S / N))                         */
  int64_t step_event_capacity; /* FIFO/SORTED: events per step that may wait in the overflow
                                  list of their target (more than 8 contenders for one target
                                  in one step); 0 = default min(B * S, 2^24).  RING: events
                                  the staging buffer of a window holds (the rest takes a slower
                                  route, same result); 0 = default                            */
  void *workspace;             /* device memory, 256-byte aligned                             */
  size_t workspace_bytes;      /* >= adseq_workspace_bytes(cfg)                               */
  void *stream;                /* stream for the preparation kernels of adseq_create          */
} adseq_config;

/* Bytes of device workspace `cfg` needs (pointer fields are not read). 0 if cfg is invalid. */
size_t adseq_workspace_bytes(const adseq_config *cfg);

/* The queues' "init" (Section 4.2: every queue structure offers init, enqueue and pop; the kinds
 * are those of Section 4.3), for the whole network at once.
 * Builds a handle: validates cfg (host), then on cfg->stream converts the synapses into the
 * packed internal form, validates delays and the CSR on the device, clears all state, and
 * synchronises that stream once.  *out is written only on success. */
int adseq_create(const adseq_config *cfg, adseq_t **out);

/* For callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  The same as adseq_create, except that the state lives in a workspace
 * of ADSEQ_STATIC_WORKSPACE_BYTES that is part of the library's device image (every GPU the
 * library runs on holds its own copy until the process ends) and the handle in static host
 * storage: no device or host allocation, no allocating library call.  cfg->workspace and
 * cfg->workspace_bytes are ignored.  The device current at the call is the one used.  Returns
 * ADSEQ_E_WORKSPACE if adseq_workspace_bytes(cfg) exceeds the limit, or if the device's static
 * workspace already holds a live handle (one at a time per device: two would share the memory
 * and race); adseq_destroy releases it.  The workspace keeps the last handle's contents;
 * everything a new handle needs to start from zero is cleared here. */
#define ADSEQ_STATIC_WORKSPACE_BYTES (32u << 20)
int adseq_create_static(const adseq_config *cfg, adseq_t **out);

/* Frees the host-side handle.  The workspace stays the caller's. */
int adseq_destroy(adseq_t *h);

/* Back to step 0: V = 0, queues empty, counters zero, tape empty.  Stream ordered. */
int adseq_reset(adseq_t *h, void *stream);

/* Open-loop delivery (the queue's pop, Section 4.2): writes the current delivered at `step`,
 * I_out[b*N + j] = (float)Iq * 2^-24, fp32 [B*N], and removes those events.  `step` must be
 * the next step not yet delivered.  LIF state and tape are not touched. */
int adseq_deliver(adseq_t *h, int64_t step, float *I_out, void *stream);

/* Open-loop enqueue (the queue's enqueue, Section 4.2): fans out the spikes listed in
 * spike_ids[0 .. *n_spikes) (flat ids b*N + i, each id at most once per step; both DEVICE
 * pointers) with emission step `step`, which must be the step last delivered.  May be called
 * several times for one step; for the bounded kinds the events of all these calls are then
 * admitted together, in canonical order. */
int adseq_enqueue(adseq_t *h, int64_t step, const int32_t *spike_ids, const int32_t *n_spikes,
                  void *stream);

/* n_steps open-loop steps from `step0`: for k = 0 .. n_steps-1, adseq_deliver(step0 + k) into
 * I_out + k * I_stride (fp32 [B*N] each; I_stride = 0 overwrites one buffer), then
 * adseq_enqueue(step0 + k) of the spikes spike_ids[spike_offsets[k] .. + n_spikes[k]).  spike_ids
 * and n_spikes [n_steps] are DEVICE pointers, spike_offsets [n_steps] is a HOST array.  The shape
 * of the paper's Poisson benchmark (Section 5.1: externally generated spike trains through the
 * queues).  Same results as those calls; the ring does the two of a step in one launch.  Stops at
 * the first error. */
int adseq_run_open(adseq_t *h, int64_t step0, int64_t n_steps, const int32_t *spike_ids,
                   const int64_t *spike_offsets /*host*/, const int32_t *n_spikes, float *I_out,
                   int64_t I_stride, void *stream);

/* One closed-loop step (pop, drive, LIF, compaction, fan-out, enqueue; see the header comment).
 * i_ext: optional extra input current fp32 [B*N] or NULL.  spikes_out: optional 0/1 bytes
 * [B*N] or NULL. */
int adseq_step(adseq_t *h, int64_t step, const float *i_ext, uint8_t *spikes_out, void *stream);

/* n_steps closed-loop steps starting at `step0` (same results as calling adseq_step in a loop with
 * i_ext = spikes_out = NULL).  ADSEQ_RING runs the steps between two window boundaries in ONE kernel
 * whose blocks (at most one per compute unit) wait for one another at a barrier per step; such a
 * launch needs the device free enough for all its blocks to run at the same time.  adseq_create
 * asks the runtime how many such blocks the device holds at once and, below 256, keeps to one
 * launch per step (same results).  Every wait is
 * bounded: if one runs out, the kernels still run to their end, the run is void, and the error
 * word carries bit 32 (adseq_counters; adseq_drop_count and adseq_backward then return
 * ADSEQ_E_HIP until adseq_reset). */
int adseq_run(adseq_t *h, int64_t step0, int64_t n_steps, void *stream);

/* Reverse-time sweep over the T steps recorded since the last reset (Section 3.2: the event
 * carries d t_post / d d = 1, eq. 13; on delivery the receiving state gets (jump / tau_m) times
 * that, eq. 17; the spike function's derivative is the surrogate of eq. 7, applied only where a
 * spike was emitted for the queue term).  With gU[T] = 0, for n = T-1 .. 0:
 *   G_i   = sum over admitted events p of row i emitted at n with n + D_p < T of a_p * gU[col_p][n + D_p]
 *   gU_i[n] = (1 - s_i[n]) * c_i[n+1] + sigma'(U_i[n] - theta) * (dL_dcount_i + s_i[n] * G_i) + dL_dU_i[n]
 *   c_i[n]  = alpha * gU_i[n] + E_i[n],  E_i[n] = -(1 / vdot_i[n]) (1 / tau_m) s_i[n] G_i in the spike-time
 *             mode (sigma' = 0 there), 0 otherwise
 *   grad_w[p] += f_p * gU[col_p][n + D_p],   grad_d[p] += (a_p / tau_m) * unit * gU[col_p][n + D_p]
 * (f_p = a_p / weight_p; unit = 1 per ms for delay_ms, dt per step for delay_steps; with a synaptic
 * current state, gJ_j[n] = gU_j[n] + alpha_s gJ_j[n+1] takes the place of gU in G_i, grad_w and
 * grad_d, and tau_syn that of tau_m in grad_d and E; with the double-exponential synapse,
 * gB_j[n] = -gU_j[n] + alpha_r gB_j[n+1] beside it, gJ + gB takes the place of gU in grad_w and in
 * G_i of the surrogate modes, and gJ / tau_syn + gB / tau_rise that of gU / tau_m in grad_d and in
 * the spike-time mode's E), summed over
 * trials.  dL_dcount: fp32 [B*N] or NULL; dL_dU: fp32 [T][B*N] or NULL; grad_w, grad_d: fp32 [S],
 * overwritten.  Synchronises the stream once at the start to read the device error word.
 * ADSEQ_RING runs the reverse steps of a window in one kernel whose blocks wait for one another's
 * results (for the adjoint cells they gather; every wait bounded); should such a wait run out --
 * the blocks of a launch were not running together, or a cotangent held the NaN that marks a cell
 * as not written yet (bits 0x7fa5c3e1) -- the kernels still run to their end, the gradients are void, and
 * the error word carries bit 32 afterwards: read it with adseq_counters once the stream is done
 * (adseq_drop_count and the next adseq_backward refuse the run with ADSEQ_E_HIP). */
int adseq_backward(adseq_t *h, const float *dL_dcount, const float *dL_dU, float *grad_w,
                   float *grad_d, void *stream);

/* Event counters since the last reset (host pointers, any may be NULL): events refused by a
 * full queue (Section 4.3 "FIFORing": a lossy queue drops what arrives while it is full; Section
 * 6.5 "Spike drop rates" reports these losses), events offered to the queues, events delivered.
 * ADSEQ_RING keeps no per-event counters: its `enqueued` is counted from the recorded spikes and
 * their row lengths, and its `delivered` is derived from that as enqueued minus the events still in
 * flight (rows of the spikes of the last d_max_steps steps whose arrival lies ahead); the Q8.24
 * sum of what each step actually popped is counted separately, see adseq_counters.
 * Synchronises `stream`.
 * Returns ADSEQ_E_CAPACITY if a tape or pool overflow happened since the last reset. */
int adseq_drop_count(adseq_t *h, uint64_t *dropped, uint64_t *enqueued, uint64_t *delivered,
                     void *stream);

/* Further counters (host pointer to 8 int64): [0] offered, [1] dropped, [2] delivered events;
 * [3..5] the same as sums of Q8.24 amplitudes; [6] spikes recorded on the tape; [7] error bits:
 * 4, 8, 16 tape or contender-pool overflow (ADSEQ_E_CAPACITY), 32 a bounded wait inside a resident
 * kernel ran out (ADSEQ_E_HIP; the run is void), 64 a warning from adseq_create: for some target the
 * |amplitudes| of its incoming synapses add up to 128 or more, so that a step in which enough of them
 * deliver together would wrap its 32-bit fixed-point sum (range +-128) without further notice.
 * Synchronises `stream`. */
int adseq_counters(adseq_t *h, int64_t *out8, void *stream);

/* Where the tape lives inside the workspace (device pointers; valid for the handle's life).
 * membrane: fp32 [max_steps][B*N] pre-reset membrane values U (a spike is exactly U >= v_thresh);
 * step_offset (NULL for ADSEQ_RING, whose fused step keeps no spike list): int64 [max_steps+1],
 * spikes of step n are spike_id[step_offset[n] .. step_offset[n+1]) (flat ids, unordered within
 * a step); event_base: int64 per recorded spike, index of its row's first admission flag;
 * admitted: one byte per emitted event (bounded kinds only, else NULL).  FIFO / SORTED decide the
 * admission of a step's events in the launch of the next step (or of adseq_counters,
 * adseq_drop_count, adseq_backward); adseq_tape launches what is pending on the stream of the
 * last enqueue, so the flags are final once that stream has been synchronised. */
typedef struct {
  const float *membrane;
  const int64_t *step_offset;
  const int32_t *spike_id;
  const int64_t *event_base;
  const uint8_t *admitted;
  int64_t steps_recorded;
} adseq_tape_view;
int adseq_tape(adseq_t *h, adseq_tape_view *out);

/* Spike count of every (trial, neuron) over the steps recorded since the last reset (what a
 * spike-count loss such as the mean squared error of this build's gradient configs needs; the
 * paper's recurrent-network benchmark, Section 5.1, names no loss): counts int32
 * [B*N], overwritten.  Needs record_tape = 1 and a complete recorded run.  Stream ordered. */
int adseq_spike_counts(adseq_t *h, int32_t *counts, void *stream);

/* Kernel timing for benchmarks (not a call of the method; for callers that want per-kernel
 * durations without an external profiler).  While enabled, adseq_step / adseq_run /
 * adseq_backward record HIP events on the caller's stream around the kernels they launch (events
 * are created by the library on first use and destroyed with the handle).  adseq_profile_read
 * synchronises `stream` and returns, per kernel class, the summed time in ms and the number of
 * launches since the last read, then forgets them.  Classes for FIFO / SORTED (an event after
 * every launch): [0] fan-out + contender registration, [1] admission + pop + drive + LIF,
 * [2] backward queue term + gradients, [3] backward neuron update.  Classes for RING: [0] the
 * expansion of one window (staging pass + accumulation pass, timed as a pair and counted as one
 * launch), [1] forward step kernel, [2] backward far gather of one window, [3] backward step
 * kernel (where the reverse steps of a window run in one launch, that launch); the step kernels are timed in groups (all the step launches between two window
 * boundaries between one pair of events), because an event after every 5 us launch would add
 * half as much again. */
int adseq_profile(adseq_t *h, int enable);
int adseq_profile_read(adseq_t *h, double *ms4 /*host*/, int64_t *launches4 /*host*/, void *stream);

/* Text of the last error on this handle (host string owned by the handle). */
const char *adseq_last_error(const adseq_t *h);

#ifdef __cplusplus
}
#endif
#endif /* ADSEQ_H */
