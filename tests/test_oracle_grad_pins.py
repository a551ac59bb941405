"""Pins of the oracle's reverse-mode sweep: closed form for one synapse,
central finite differences on a frozen raster (fp64, no quantisation), and the
forward-mode / reverse-mode dot-product identity."""
import copy
import math

import numpy as np
import pytest

from oracle import oracle, tangent
from paper_2512_05906_amd import synth


def _src(wl):
    return np.repeat(np.arange(wl.n_neurons), np.diff(wl.row_ptr))


def test_single_synapse_closed_form_delay_and_weight_gradient():
    """One synapse 0 -> 1, one spike at n0: for m >= k = n0 + D,
    dU_1[m]/dd = (a / tau) alpha^(m-k) (receive rule, eq. 17, carried on by the leak)
    and dU_1[m]/dw = f alpha^(m-k)."""
    T, n0, m = 60, 5, 40
    d_ms = np.float32(1.2345)
    w = np.float32(0.3)
    wl = synth.Workload("pair", 2, 1, T, 1, 20, ext_rate_hz=0.0,
                        row_ptr=np.array([0, 1, 1], np.int64), col=np.array([1], np.int32),
                        weight=np.array([w], np.float32), delay_ms=np.array([d_ms], np.float32))
    forced = np.zeros((T, 1, 2), np.uint8)
    forced[n0, 0, 0] = 1
    dL_dU = np.zeros((T, 1, 2), np.float32)
    dL_dU[m, 0, 1] = 1.0
    dt, tau = float(np.float32(0.1)), 20.0
    D = math.ceil(float(d_ms) / dt)
    k = n0 + D
    f = math.exp(-(D * dt - float(d_ms)) / tau)
    a = float(w) * f
    for exact in (False, True):
        r = oracle.Run(wl, oracle.RING, forced_spikes=forced, exact_f64=exact, surrogate=1)
        gw, gd = r.backward(None, dL_dU)
        alpha = math.exp(-dt / tau)
        np.testing.assert_allclose(gd[0], a / tau * alpha ** (m - k), rtol=1e-6)
        np.testing.assert_allclose(gw[0], f * alpha ** (m - k), rtol=1e-6)
        # and the value itself: U_1[m] = a alpha^(m-k)
        np.testing.assert_allclose(r.U[m, 0, 1], a * alpha ** (m - k), rtol=1e-5)
    # integer delays: gradient per step is dt times the gradient per ms
    wl2 = copy.copy(wl)
    wl2.delay_ms, wl2.delay_steps = None, np.array([D], np.uint8)
    r = oracle.Run(wl2, oracle.RING, forced_spikes=forced, surrogate=1)
    gw, gd = r.backward(None, dL_dU)
    np.testing.assert_allclose(gd[0], float(w) * dt / tau * alpha ** (m - k), rtol=1e-6)
    np.testing.assert_allclose(gw[0], alpha ** (m - k), rtol=1e-6)


@pytest.mark.parametrize("kind,cap,tau_syn", [(oracle.RING, 0, 0.0), (oracle.FIFO, 3, 0.0), (oracle.RING, 0, 2.0),
                                              (oracle.SYN_FIFO, 1, 0.0), (oracle.SYN_LATEST, 1, 0.0),
                                              (oracle.SYN_BINS, 2, 0.0)])
def test_central_finite_differences_frozen_raster(kind, cap, tau_syn):
    """Smooth loss L = sum c[n,j] U_j[n] on a 10-neuron net, raster frozen, fp64
    without quantisation, surrogate off: reverse-mode grad_w / grad_d must equal
    central differences.  (With the raster frozen the surrogate terms are not a
    derivative of anything, hence off.)"""
    wl = synth.ragged_network(10, 6, 12, seed=17, rate_hz=1500.0, t=150, continuous=True,
                              w_mean=0.2, w_std=0.1)
    wl.tau_syn_ms = tau_syn     # > 0: the jumps go into a synaptic current state (eq. 1)
    free = oracle.Run(wl, kind, cap)
    forced = free.spikes
    assert forced.sum() > 50
    c = synth.random_cotangent(wl)

    def loss(w):
        r = oracle.Run(w, kind, cap, forced_spikes=forced, exact_f64=True, surrogate=1)
        return float((c.astype(np.float64) * r.U64).sum()), r

    L0, r0 = loss(wl)
    gw, gd = r0.backward(None, c)
    if kind in (oracle.FIFO, oracle.SYN_FIFO, oracle.SYN_LATEST, oracle.SYN_BINS):
        assert r0.counters()["dropped"] > 0
    rng = np.random.default_rng(1)
    dt = float(np.float32(wl.dt_ms))
    checked = 0
    for p in rng.permutation(wl.n_synapses)[:25]:
        # weight
        h = 1e-3
        wp, wm = copy.copy(wl), copy.copy(wl)
        wp.weight, wm.weight = wl.weight.copy(), wl.weight.copy()
        wp.weight[p] += np.float32(h)
        wm.weight[p] -= np.float32(h)
        hh = (float(wp.weight[p]) - float(wm.weight[p])) / 2
        fd = (loss(wp)[0] - loss(wm)[0]) / (2 * hh)
        np.testing.assert_allclose(gw[p], fd, rtol=1e-6, atol=1e-9)
        # delay (keep the arrival step unchanged)
        d = float(wl.delay_ms[p])
        h = 2e-4
        if math.ceil((d + h) / dt) != math.ceil((d - h) / dt):
            continue
        wp, wm = copy.copy(wl), copy.copy(wl)
        wp.delay_ms, wm.delay_ms = wl.delay_ms.copy(), wl.delay_ms.copy()
        wp.delay_ms[p] = np.float32(d + h)
        wm.delay_ms[p] = np.float32(d - h)
        hh = (float(wp.delay_ms[p]) - float(wm.delay_ms[p])) / 2
        fd = (loss(wp)[0] - loss(wm)[0]) / (2 * hh)
        np.testing.assert_allclose(gd[p], fd, rtol=1e-5, atol=1e-9)
        checked += 1
    assert checked > 10
    assert np.abs(gd).max() > 0 and np.abs(gw).max() > 0


@pytest.mark.parametrize("kind,cap,continuous", [(oracle.RING, 0, False), (oracle.FIFO, 3, False),
                                                  (oracle.SORTED, 4, True), (oracle.SYN_FIFO, 1, True),
                                                  (oracle.SYN_LATEST, 1, False), (oracle.SYN_BINS, 2, True)])
def test_reverse_mode_is_transpose_of_forward_mode(kind, cap, continuous):
    """<u, J v> == <J^T u, v> with J propagated in forward mode by oracle/tangent.py
    (surrogate on, spike-count and membrane cotangents, several trials)."""
    B = 2
    wl = synth.ragged_network(12, 7, 10, seed=23, rate_hz=1500.0, t=120, b=B, continuous=continuous,
                              w_mean=0.2, w_std=0.15)
    r = oracle.Run(wl, kind, cap, log_events=True)
    assert r.spikes.sum() > 80
    u_U = synth.random_cotangent(wl)
    u_c = synth.spike_count_targets(wl) - 2.5
    gw, gd = r.backward(u_c, u_U)
    rng = np.random.default_rng(5)
    w_t = rng.standard_normal(wl.n_synapses)
    d_t = rng.standard_normal(wl.n_synapses)
    lhs = 0.0
    dl = r.event_log("delivered")
    U, S = r.U, r.spikes
    alpha = float(np.float32(math.exp(-float(np.float32(wl.dt_ms)) / float(np.float32(wl.tau_m_ms)))))
    d_unit = 1.0 if continuous else float(np.float32(wl.dt_ms))
    for b in range(B):
        sel = dl["b"] == b
        ev = list(zip(dl["syn"][sel], dl["n_emit"][sel], dl["k"][sel]))
        U_t, c_t = tangent.jvp(U[:, b], S[:, b], ev, wl.col, _src(wl), r.a_f.astype(np.float64),
                               r.f_f.astype(np.float64), alpha, float(wl.v_thresh),
                               float(np.float32(wl.tau_m_ms)), d_unit, w_t, d_t)
        lhs += float((u_U[:, b].astype(np.float64) * U_t).sum() + (u_c[b].astype(np.float64) * c_t).sum())
    rhs = float(gw @ w_t + gd @ d_t)
    assert abs(lhs) > 1e-3
    np.testing.assert_allclose(lhs, rhs, rtol=1e-9)


def test_surrogate_is_superspike():
    """One neuron, dL/dcount = 1, no synapses: dL/dU[n] follows
    g[n] = (1 - s) alpha g[n+1] + 1/(|U - theta| + 1)^2  (eq. 7)."""
    T = 50
    wl = synth.Workload("one", 1, 0, T, 1, 1, ext_rate_hz=2000.0,
                        row_ptr=np.zeros(2, np.int64), col=np.zeros(0, np.int32),
                        weight=np.zeros(0, np.float32), delay_steps=np.zeros(0, np.uint8))
    r = oracle.Run(wl, oracle.RING)
    U, S = r.U[:, 0, 0].astype(np.float64), r.spikes[:, 0, 0]
    assert S.sum() >= 2
    _, _, gU = r.backward(np.ones((1, 1), np.float32), None, want_gU=True)
    alpha = float(np.float32(math.exp(-float(np.float32(0.1)) / 20.0)))
    g = 0.0
    for n in range(T - 1, -1, -1):
        g = (1 - S[n]) * alpha * g + 1.0 / (abs(U[n] - 1.0) + 1.0) ** 2
        np.testing.assert_allclose(gU[n, 0, 0], g, rtol=1e-12)


# ---------------------------------------------------------------- spike-time gradient (no surrogate)

def test_spike_time_gradient_chain_closed_form():
    """Three neurons in a chain A -> B -> C.  A fires once (input pulse), its event reaches B
    ten steps later; B, charged by a constant input current, crosses the threshold some 80 steps
    after that; B's event reaches C, and the loss is C's membrane value 20 steps on.  The only
    way w1 and d1 (synapse A -> B) reach the loss is B's emission time, t_B' = -v_B' / vdot_B
    (Section 3.1 eq. 8), received by C with (w2 / tau) t_post' (eq. 17):
        dL/dw1 = (w2 / tau) alpha^(m - k2) * (-dt / (U_B[n_B] - U_B[n_B - 1])) * alpha^(n_B - 1 - k1)
        dL/dd1 = (w1 dt / tau) dL/dw1,   dL/dw2 = alpha^(m - k2),   dL/dd2 = (w2 dt / tau) alpha^(m - k2)."""
    T = 200
    wl = synth.Workload("chain", 3, 1, T, 1, 20, ext_rate_hz=0.0,
                        row_ptr=np.array([0, 1, 2, 2], np.int64), col=np.array([1, 2], np.int32),
                        weight=np.array([0.05, 0.3], np.float32), delay_steps=np.array([10, 7], np.uint8))
    i_ext = np.zeros((T, 1, 3), np.float32)
    i_ext[5, 0, 0] = 1.5          # A fires at step 5
    i_ext[:, 0, 1] = 0.012        # B charges towards 2.4 thresholds
    r = oracle.Run(wl, oracle.RING, i_ext=i_ext, surrogate=2)
    S, U = r.spikes[:, 0], r.U[:, 0].astype(np.float64)
    assert S[:, 0].sum() == 1 and S[5, 0] == 1
    n_B = int(np.nonzero(S[:, 1])[0][0])
    k1, k2 = 5 + 10, n_B + 7
    assert k1 + 20 < n_B < 150 and S[:, 2].sum() == 0
    m = k2 + 20
    dU = np.zeros((T, 1, 3), np.float32)
    dU[m, 0, 2] = 1.0
    gw, gd = r.backward(None, dU)
    alpha = float(np.float32(math.exp(-float(np.float32(wl.dt_ms)) / float(np.float32(wl.tau_m_ms)))))
    dt, tau = float(np.float32(wl.dt_ms)), float(np.float32(wl.tau_m_ms))
    w1, w2 = float(r.a_f[0]), float(r.a_f[1])
    direct = alpha ** (m - k2)
    via_tB = (w2 / tau) * direct * (-dt / (U[n_B, 1] - U[n_B - 1, 1])) * alpha ** (n_B - 1 - k1)
    np.testing.assert_allclose(gw, [via_tB, direct], rtol=1e-9)
    np.testing.assert_allclose(gd, [(w1 * dt / tau) * via_tB, (w2 * dt / tau) * direct], rtol=1e-9)
    assert via_tB < 0          # a larger w1 makes B fire earlier, C's jump has decayed more by step m
    # with the surrogate switched off and no spike-time rule, w1 cannot reach the loss at all
    r0 = oracle.Run(wl, oracle.RING, i_ext=i_ext, surrogate=1)
    gw0, gd0 = r0.backward(None, dU)
    np.testing.assert_allclose(gw0, [0.0, direct], rtol=1e-9)


@pytest.mark.parametrize("kind,cap,continuous", [(oracle.RING, 0, False), (oracle.FIFO, 3, True)])
def test_spike_time_reverse_mode_is_transpose_of_forward_mode(kind, cap, continuous):
    """<u, J v> == <J^T u, v> for the spike-time rules, J propagated in forward mode by
    oracle/tangent.py from the paper's tangent rules."""
    B = 2
    wl = synth.ragged_network(12, 7, 10, seed=29, rate_hz=1500.0, t=120, b=B, continuous=continuous,
                              w_mean=0.2, w_std=0.15)
    r = oracle.Run(wl, kind, cap, log_events=True, surrogate=2)
    assert r.spikes.sum() > 80
    u_U = synth.random_cotangent(wl)
    gw, gd = r.backward(None, u_U)
    rng = np.random.default_rng(6)
    w_t = rng.standard_normal(wl.n_synapses)
    d_t = rng.standard_normal(wl.n_synapses)
    dl = r.event_log("delivered")
    U, S = r.U, r.spikes
    alpha = float(np.float32(math.exp(-float(np.float32(wl.dt_ms)) / float(np.float32(wl.tau_m_ms)))))
    d_unit = 1.0 if continuous else float(np.float32(wl.dt_ms))
    lhs = 0.0
    for b in range(B):
        sel = dl["b"] == b
        ev = list(zip(dl["syn"][sel], dl["n_emit"][sel], dl["k"][sel]))
        U_t, _ = tangent.jvp(U[:, b], S[:, b], ev, wl.col, _src(wl), r.a_f.astype(np.float64),
                             r.f_f.astype(np.float64), alpha, float(wl.v_thresh),
                             float(np.float32(wl.tau_m_ms)), d_unit, w_t, d_t, spike_time=True,
                             dt=float(np.float32(wl.dt_ms)), v_reset=float(wl.v_reset))
        lhs += float((u_U[:, b].astype(np.float64) * U_t).sum())
    rhs = float(gw @ w_t + gd @ d_t)
    assert abs(lhs) > 1e-3
    np.testing.assert_allclose(lhs, rhs, rtol=1e-9)
    # the spike-time paths matter: without them the same product is different
    r1 = oracle.Run(wl, kind, cap, surrogate=1)
    gw1, gd1 = r1.backward(None, u_U)
    assert abs(float(gw1 @ w_t + gd1 @ d_t) - rhs) > 1e-6 * abs(rhs)


# ---------------------------------------------------------------- first-order synapse (synaptic current state)

def test_first_order_synapse_closed_form():
    """One synapse 0 -> 1 with a synaptic current state (Section 2.1 eq. 1, discretised as
    isyn = alpha_s isyn + jump, U = alpha V + isyn), one spike at n0, arrival k = n0 + D.  For
    m >= k:  U_1[m] = a sum_{r=k..m} alpha^(m-r) alpha_s^(r-k) = a (alpha^(L+1) - alpha_s^(L+1)) / (alpha - alpha_s),
    L = m - k;  dU_1[m]/dw = that / w,  dU_1[m]/dd = (a / tau_syn) dt times the same kernel
    (receive rule, eq. 17, with the time constant of the state that takes the jump)."""
    T, n0, m, D = 80, 5, 50, 7
    w, tau_syn, tau_m, dt = 0.3, 2.0, 20.0, float(np.float32(0.1))
    wl = synth.Workload("pair", 2, 1, T, 1, 20, ext_rate_hz=0.0, tau_syn_ms=tau_syn,
                        row_ptr=np.array([0, 1, 1], np.int64), col=np.array([1], np.int32),
                        weight=np.array([w], np.float32), delay_steps=np.array([D], np.uint8))
    forced = np.zeros((T, 1, 2), np.uint8)
    forced[n0, 0, 0] = 1
    dL_dU = np.zeros((T, 1, 2), np.float32)
    dL_dU[m, 0, 1] = 1.0
    k = n0 + D
    al, als = math.exp(-dt / tau_m), math.exp(-dt / tau_syn)
    kern = (al ** (m - k + 1) - als ** (m - k + 1)) / (al - als)
    a = float(np.float32(w))
    r = oracle.Run(wl, oracle.RING, forced_spikes=forced, exact_f64=True, surrogate=1)
    np.testing.assert_allclose(r.U64[m, 0, 1], a * kern, rtol=1e-12)
    assert r.U64[k - 1, 0, 1] == 0.0 and r.U64[k, 0, 1] == a
    gw, gd = r.backward(None, dL_dU)
    np.testing.assert_allclose(gw[0], kern, rtol=1e-12)
    np.testing.assert_allclose(gd[0], a / tau_syn * dt * kern, rtol=1e-12)
    # fp32 path (Q8.24 amplitude, fused multiply-adds): same values to rounding
    r32 = oracle.Run(wl, oracle.RING, forced_spikes=forced, surrogate=1)
    np.testing.assert_allclose(r32.U[m, 0, 1], a * kern, rtol=1e-5)
    # continuous delay: the decay between true arrival and grid step is that of the synaptic state
    d_ms = 0.6543
    wl2 = copy.copy(wl)
    wl2.delay_steps, wl2.delay_ms = None, np.array([d_ms], np.float32)
    r2 = oracle.Run(wl2, oracle.RING, forced_spikes=forced, exact_f64=True, surrogate=1)
    D2 = math.ceil(float(np.float32(d_ms)) / dt)
    f = math.exp(-(D2 * dt - float(np.float32(d_ms))) / tau_syn)
    np.testing.assert_allclose(r2.a_d[0], a * f, rtol=1e-12)


@pytest.mark.parametrize("mode", [0, 2])
def test_first_order_synapse_reverse_mode_is_transpose_of_forward_mode(mode):
    """<u, J v> == <J^T u, v> with a synaptic current state, surrogate and spike-time modes."""
    B = 2
    wl = synth.ragged_network(12, 7, 10, seed=31, rate_hz=1500.0, t=120, b=B, continuous=True,
                              w_mean=0.25, w_std=0.15)
    wl.tau_syn_ms = 1.5
    r = oracle.Run(wl, oracle.FIFO, 4, log_events=True, surrogate=mode)
    assert r.spikes.sum() > 60 and r.counters()["dropped"] > 0
    u_U = synth.random_cotangent(wl)
    u_c = synth.spike_count_targets(wl) - 2.5 if mode == 0 else None
    gw, gd = r.backward(u_c, u_U)
    rng = np.random.default_rng(8)
    w_t = rng.standard_normal(wl.n_synapses)
    d_t = rng.standard_normal(wl.n_synapses)
    dl = r.event_log("delivered")
    U, S = r.U, r.spikes
    dt = float(np.float32(wl.dt_ms))
    alpha = float(np.float32(math.exp(-dt / float(np.float32(wl.tau_m_ms)))))
    alpha_s = float(np.float32(math.exp(-dt / float(np.float32(wl.tau_syn_ms)))))
    lhs = 0.0
    for b in range(B):
        sel = dl["b"] == b
        ev = list(zip(dl["syn"][sel], dl["n_emit"][sel], dl["k"][sel]))
        U_t, c_t = tangent.jvp(U[:, b], S[:, b], ev, wl.col, _src(wl), r.a_f.astype(np.float64),
                               r.f_f.astype(np.float64), alpha, float(wl.v_thresh),
                               float(np.float32(wl.tau_syn_ms)), 1.0, w_t, d_t, surrogate=(mode == 0),
                               spike_time=(mode == 2), dt=dt, v_reset=float(wl.v_reset), alpha_s=alpha_s)
        lhs += float((u_U[:, b].astype(np.float64) * U_t).sum())
        if mode == 0:
            lhs += float((u_c[b].astype(np.float64) * c_t).sum())
    rhs = float(gw @ w_t + gd @ d_t)
    assert abs(lhs) > 1e-3
    np.testing.assert_allclose(lhs, rhs, rtol=1e-9)


def test_double_exponential_synapse_closed_form():
    """One synapse 0 -> 1 through a double-exponential synapse built from two first-order states
    (Section 3.2, closing remark): A (tau_syn) and B (tau_rise) both take the jump a at the arrival
    step k, isyn = A - B, U = alpha V + isyn.  For m >= k, with L = m - k and
    K(x) = (alpha^(L+1) - x^(L+1)) / (alpha - x):
      U_1[m] = a (K(alpha_A) - K(alpha_B)),  dU_1[m]/dw = U_1[m] / w,
      dU_1[m]/dd = a dt (K(alpha_A) / tau_A - K(alpha_B) / tau_B)   (receive rule, eq. 17, per state).
    There is no jump in the current itself: isyn[k] = 0."""
    T, n0, m, D = 90, 5, 60, 7
    w, tau_a, tau_b, tau_m, dt = 0.3, 3.0, 0.8, 20.0, float(np.float32(0.1))
    wl = synth.Workload("pair", 2, 1, T, 1, 20, ext_rate_hz=0.0, tau_syn_ms=tau_a, tau_rise_ms=tau_b,
                        row_ptr=np.array([0, 1, 1], np.int64), col=np.array([1], np.int32),
                        weight=np.array([w], np.float32), delay_steps=np.array([D], np.uint8))
    forced = np.zeros((T, 1, 2), np.uint8)
    forced[n0, 0, 0] = 1
    dL_dU = np.zeros((T, 1, 2), np.float32)
    dL_dU[m, 0, 1] = 1.0
    k = n0 + D
    al = math.exp(-dt / tau_m)
    ala, alb = math.exp(-dt / float(np.float32(tau_a))), math.exp(-dt / float(np.float32(tau_b)))
    L = m - k
    Ka = (al ** (L + 1) - ala ** (L + 1)) / (al - ala)
    Kb = (al ** (L + 1) - alb ** (L + 1)) / (al - alb)
    a = float(np.float32(w))
    r = oracle.Run(wl, oracle.RING, forced_spikes=forced, exact_f64=True, surrogate=1)
    np.testing.assert_allclose(r.U64[m, 0, 1], a * (Ka - Kb), rtol=1e-11)
    assert r.U64[k, 0, 1] == 0.0 and r.U64[k + 1, 0, 1] > 0.0       # the current rises from zero
    gw, gd = r.backward(None, dL_dU)
    np.testing.assert_allclose(gw[0], Ka - Kb, rtol=1e-11)
    np.testing.assert_allclose(gd[0], a * dt * (Ka / float(np.float32(tau_a)) - Kb / float(np.float32(tau_b))), rtol=1e-11)
    r32 = oracle.Run(wl, oracle.RING, forced_spikes=forced, surrogate=1)
    np.testing.assert_allclose(r32.U[m, 0, 1], a * (Ka - Kb), rtol=2e-5)
    # continuous delays are refused: the two states would decay a sub-step arrival differently
    wl2 = copy.copy(wl)
    wl2.delay_steps, wl2.delay_ms = None, np.array([0.65], np.float32)
    with pytest.raises(Exception):
        oracle.Run(wl2, oracle.RING, forced_spikes=forced)


def test_double_exponential_weight_gradient_finite_differences():
    """Central differences in the weights on a frozen raster (fp64, no quantisation): the part of the
    double-exponential reverse sweep that a finite difference can see (delays are whole steps here)."""
    wl = synth.ragged_network(10, 6, 12, seed=19, rate_hz=1500.0, t=150, w_mean=0.4, w_std=0.2)
    wl.tau_syn_ms, wl.tau_rise_ms = 2.5, 0.7
    forced = oracle.Run(wl, oracle.FIFO, 3).spikes
    assert forced.sum() > 40
    c = synth.random_cotangent(wl)

    def loss(w):
        r = oracle.Run(w, oracle.FIFO, 3, forced_spikes=forced, exact_f64=True, surrogate=1)
        return float((c.astype(np.float64) * r.U64).sum()), r

    _, r0 = loss(wl)
    gw, _ = r0.backward(None, c)
    rng = np.random.default_rng(2)
    for p in rng.permutation(wl.n_synapses)[:20]:
        h = 1e-3
        wp, wm = copy.copy(wl), copy.copy(wl)
        wp.weight, wm.weight = wl.weight.copy(), wl.weight.copy()
        wp.weight[p] += np.float32(h)
        wm.weight[p] -= np.float32(h)
        hh = (float(wp.weight[p]) - float(wm.weight[p])) / 2
        fd = (loss(wp)[0] - loss(wm)[0]) / (2 * hh)
        np.testing.assert_allclose(gw[p], fd, rtol=1e-6, atol=1e-9)
    assert np.abs(gw).max() > 0


@pytest.mark.parametrize("mode", [0, 2])
def test_double_exponential_reverse_mode_is_transpose_of_forward_mode(mode):
    """<u, J v> == <J^T u, v> with the double-exponential synapse (weights and delays, surrogate and
    spike-time modes, lossy queue)."""
    B = 2
    wl = synth.ragged_network(12, 7, 10, seed=37, rate_hz=1500.0, t=120, b=B, w_mean=0.5, w_std=0.3)
    wl.tau_syn_ms, wl.tau_rise_ms = 2.0, 0.6
    r = oracle.Run(wl, oracle.FIFO, 4, log_events=True, surrogate=mode)
    assert r.spikes.sum() > 60 and r.counters()["dropped"] > 0
    u_U = synth.random_cotangent(wl)
    u_c = synth.spike_count_targets(wl) - 2.5 if mode == 0 else None
    gw, gd = r.backward(u_c, u_U)
    rng = np.random.default_rng(9)
    w_t = rng.standard_normal(wl.n_synapses)
    d_t = rng.standard_normal(wl.n_synapses)
    dl = r.event_log("delivered")
    U, S = r.U, r.spikes
    dt = float(np.float32(wl.dt_ms))
    alpha = float(np.float32(math.exp(-dt / float(np.float32(wl.tau_m_ms)))))
    alpha_s = float(np.float32(math.exp(-dt / float(np.float32(wl.tau_syn_ms)))))
    alpha_r = float(np.float32(math.exp(-dt / float(np.float32(wl.tau_rise_ms)))))
    lhs = 0.0
    for b in range(B):
        sel = dl["b"] == b
        ev = list(zip(dl["syn"][sel], dl["n_emit"][sel], dl["k"][sel]))
        U_t, c_t = tangent.jvp(U[:, b], S[:, b], ev, wl.col, _src(wl), r.a_f.astype(np.float64),
                               r.f_f.astype(np.float64), alpha, float(wl.v_thresh),
                               float(np.float32(wl.tau_syn_ms)), dt, w_t, d_t, surrogate=(mode == 0),
                               spike_time=(mode == 2), dt=dt, v_reset=float(wl.v_reset), alpha_s=alpha_s,
                               alpha_r=alpha_r, tau_r=float(np.float32(wl.tau_rise_ms)))
        lhs += float((u_U[:, b].astype(np.float64) * U_t).sum())
        if mode == 0:
            lhs += float((u_c[b].astype(np.float64) * c_t).sum())
    rhs = float(gw @ w_t + gd @ d_t)
    assert abs(lhs) > 1e-3
    np.testing.assert_allclose(lhs, rhs, rtol=1e-9)
