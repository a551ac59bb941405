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
        spike_time=False, dt=None, v_reset=0.0, alpha_s=0.0, alpha_r=0.0, tau_r=None):
    """Tangents of (U [T,N], spike counts [N]) for one trial.

    U, S        recorded membrane values / spikes [T, N]
    events      iterable of (syn, n_emit, k) admitted events with k < T
    col, src    target / source neuron of each synapse
    a, f        amplitude a = w f and decay factor f per synapse (float64)
    w_t, d_t    tangent directions on weights and delays [S]
    d_unit      1 for delays in ms, dt for delays in steps
    tau         time constant of the state that receives the jump (synaptic current state if
                alpha_s > 0, eq. 1: isyn = alpha_s isyn + jumps, U = alpha V + isyn; else the membrane)
    alpha_r, tau_r   > 0: double-exponential synapse (Section 3.2, closing remark): a second state
                with leak alpha_r and time constant tau_r takes every jump too, isyn = A - B; the
                receive rule applies to each state with its own time constant
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
    J_t = np.zeros(N)              # tangent of the synaptic current state (A)
    B_t = np.zeros(N)              # tangent of the second state of the double-exponential synapse
    for n in range(T):
        I_w = np.zeros(N)          # tangent of the delivered amplitude (weight, emitting spike's value)
        I_k = np.zeros(N)          # amplitude x tangent of the delivery time (delay, emission time)
        for p, n_emit in by_arrival[n]:
            I_w[col[p]] += f[p] * w_t[p] + a[p] * s_t[n_emit, src[p]]
            I_k[col[p]] += a[p] * d_unit * d_t[p]
            if spike_time:
                I_k[col[p]] += a[p] * tspk_t[n_emit, src[p]]
        I_t = I_w + I_k / tau      # receive rule: (jump / tau) x tangent of the delivery time
        if spike_time:
            vdot = (U[n].astype(np.float64) - V) / dt
            vdot = np.where(vdot == 0.0, 1.0, vdot)
            tspk_t[n] = np.where(S[n] != 0, -V_t / vdot, 0.0)
        if alpha_r > 0.0:
            J_t = alpha_s * J_t + I_w + I_k / tau
            B_t = alpha_r * B_t + I_w + I_k / tau_r
            I_t = J_t - B_t
        elif alpha_s > 0.0:
            J_t = alpha_s * J_t + I_t
            I_t = J_t
        U_t[n] = alpha * V_t + I_t
        s_t[n] = sg[n] * U_t[n]
        V_t = (1.0 - S[n]) * U_t[n]
        V = np.where(S[n] != 0, v_reset, U[n].astype(np.float64))
    return U_t, s_t.sum(axis=0)
