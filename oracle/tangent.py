"""Forward-mode tangent propagation through the delayed-delivery simulation.

TEST INFRASTRUCTURE ONLY.  Written in numpy from the paper's tangent rules,
independently of the reverse-mode sweep in the C++ oracle, so that the
identity <u, J v> = <J^T u, v> checks the reverse sweep's transposition (the
paper's own JVP -> VJP check, Section 4.4):

  * a delayed event carries the tangent of its delivery time,
    t_post' = t_pre' + d'  (Section 3.2, eq. 13);
  * on delivery the receiving state gets  x+' = x-' + (jump / tau) t_post'
    (eq. 17), zero when nothing is delivered (spike-receive rule, Section 4.1);
  * the tangent queue stores one float per event in transit (Section 4.2);
  * the spike function's tangent is the SuperSpike surrogate times the
    membrane tangent (eq. 7), and only an emitted spike has a queue entry to
    carry it (event-sparse reading);
  * spike-time mode (no surrogate): the emission time of a spike has the tangent
    t_spk' = -v' / vdot, with v the membrane value the step started from and vdot the
    first forward difference (U - v) / dt, 1 where that is 0 (Section 3.1 eq. 8 and the
    spike-detection rule of Section 4.1); the event then carries t_post' = t_spk' + d'.
"""
from __future__ import annotations

import numpy as np


def jvp(U, S, events, col, src, a, f, alpha, theta, tau, d_unit, w_t, d_t, surrogate=True,
        spike_time=False, dt=None, v_reset=0.0, alpha_s=0.0):
    """Tangents of (U [T,N], spike counts [N]) for one trial.

    U, S        recorded membrane values / spikes [T, N]
    events      iterable of (syn, n_emit, k) admitted events with k < T
    col, src    target / source neuron of each synapse
    a, f        amplitude a = w f and decay factor f per synapse (float64)
    w_t, d_t    tangent directions on weights and delays [S]
    d_unit      1 for delays in ms, dt for delays in steps
    tau         time constant of the state that receives the jump (synaptic current state if
                alpha_s > 0, eq. 1: isyn = alpha_s isyn + jumps, U = alpha V + isyn; else the membrane)
    """
    T, N = U.shape
    by_arrival = [[] for _ in range(T)]
    for p, n, k in events:
        if k < T:
            by_arrival[k].append((int(p), int(n)))
    x = U.astype(np.float64) - theta
    sg = 1.0 / (np.abs(x) + 1.0) ** 2 if surrogate else np.zeros_like(x)
    if spike_time:
        sg = np.zeros_like(x)
    U_t = np.zeros((T, N))
    s_t = np.zeros((T, N))
    tspk_t = np.zeros((T, N))      # tangent of the emission time (ms) of the spike at (n, i)
    V_t = np.zeros(N)
    V = np.zeros(N)                # membrane value each step starts from
    J_t = np.zeros(N)              # tangent of the synaptic current state
    for n in range(T):
        I_t = np.zeros(N)
        for p, n_emit in by_arrival[n]:
            # amplitude tangent (weight and delay) + amplitude * tangent of the emitting spike
            I_t[col[p]] += f[p] * w_t[p] + (a[p] / tau) * d_unit * d_t[p] + a[p] * s_t[n_emit, src[p]]
            if spike_time:
                I_t[col[p]] += (a[p] / tau) * tspk_t[n_emit, src[p]]
        if spike_time:
            vdot = (U[n].astype(np.float64) - V) / dt
            vdot = np.where(vdot == 0.0, 1.0, vdot)
            tspk_t[n] = np.where(S[n] != 0, -V_t / vdot, 0.0)
        if alpha_s > 0.0:
            J_t = alpha_s * J_t + I_t
            I_t = J_t
        U_t[n] = alpha * V_t + I_t
        s_t[n] = sg[n] * U_t[n]
        V_t = (1.0 - S[n]) * U_t[n]
        V = np.where(S[n] != 0, v_reset, U[n].astype(np.float64))
    return U_t, s_t.sum(axis=0)
