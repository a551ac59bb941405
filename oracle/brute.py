"""Brute-force definitions the oracle is pinned against (numpy / pure Python).

TEST INFRASTRUCTURE ONLY.  Nothing here calls the C++ oracle or the HIP path;
each function restates a definition so a mistake in the oracle's queue logic
shows up as a disagreement.
"""
from __future__ import annotations

import numpy as np


def delivered_currents(spikes: np.ndarray, row_ptr, col, amp, D) -> np.ndarray:
    """I_j(n) = sum_i a_ij * s_i(n - D_ij)  (delivery at t_post = t_pre + d,
    Section 3.2 eqs. 10-11; weighted events add linearly, Section 4.3 "Ring").

    spikes [T, N] (0/1), amp [S] float64, D [S] int  ->  I [T, N] float64.
    """
    T, N = spikes.shape
    I = np.zeros((T, N), np.float64)
    src = np.repeat(np.arange(N), np.diff(row_ptr))
    s = spikes.astype(np.float64)
    for p in range(len(col)):
        d = int(D[p])
        if d < T:
            I[d:, col[p]] += amp[p] * s[:T - d, src[p]]
    return I


def replay_bounded(spikes: np.ndarray, row_ptr, col, D, capacity: int):
    """Replay of the bounded-bag rule on a given raster [T, N].

    At each step: events due now leave their target's bag; then the spikes of
    the step are taken in ascending source order, each row in storage order,
    and an event is admitted iff its target currently holds fewer than
    `capacity` undelivered events (an incoming event is dropped when the queue
    is full, Section 4.3 "FIFORing").  Returns (admitted, dropped) as lists of
    (syn, n_emit, k) tuples in canonical order.
    """
    T, N = spikes.shape
    occ = [0] * N
    due = {}           # arrival step -> list of targets
    admitted, dropped = [], []
    for n in range(T):
        for j in due.pop(n, []):
            occ[j] -= 1
        for i in np.nonzero(spikes[n])[0]:
            for p in range(int(row_ptr[i]), int(row_ptr[i + 1])):
                j = int(col[p])
                k = n + int(D[p])
                if occ[j] >= capacity:
                    dropped.append((p, n, k))
                else:
                    occ[j] += 1
                    admitted.append((p, n, k))
                    due.setdefault(k, []).append(j)
    return admitted, dropped


def hold_one_spike(spikes: np.ndarray, row_ptr, col, D):
    """A queue that stores one spike time and refuses newcomers while occupied
    (Section 4.3 "SingleSpike(Hold)", stated there to behave like a FIFO of
    capacity one).  One such queue per target.  Returns the set of delivered
    (syn, n_emit, k)."""
    T, N = spikes.shape
    EMPTY = None
    held = [EMPTY] * N
    out = set()
    for n in range(T):
        for j in range(N):
            if held[j] is not EMPTY and held[j][2] <= n:
                out.add(held[j])
                held[j] = EMPTY
        for i in np.nonzero(spikes[n])[0]:
            for p in range(int(row_ptr[i]), int(row_ptr[i + 1])):
                j = int(col[p])
                if held[j] is EMPTY:
                    held[j] = (p, n, n + int(D[p]))
    return out


def replay_per_synapse(spikes: np.ndarray, row_ptr, D, capacity: int):
    """One first-in-first-out queue of `capacity` spike times per synapse (the organisation of
    Section 4.1, listing 1, with the "FIFORing(n)" of Section 4.3; capacity 1 is its
    "SingleSpike(Hold)").  Written per synapse from the spike train of its source alone: a
    synapse's queue is a list of arrival times; at step n the head leaves if it is due, then a
    spike of the source at n enters unless the list is full.  Returns (admitted, dropped) as sets
    of (syn, n_emit, k)."""
    T, N = spikes.shape
    admitted, dropped = set(), set()
    for i in range(N):
        times = np.nonzero(spikes[:, i])[0]
        for p in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            d = int(D[p])
            queue = []                       # arrival times, oldest first
            for n in times:
                n = int(n)
                while queue and queue[0] <= n:
                    queue.pop(0)
                if len(queue) >= capacity:
                    dropped.add((p, n, n + d))
                else:
                    queue.append(n + d)
                    admitted.add((p, n, n + d))
    return admitted, dropped


def replay_latest(spikes: np.ndarray, row_ptr, D):
    """One slot per synapse in which a new spike always replaces the one held (Section 4.3
    "SingleSpike(Drop)").  Stated directly from the source's spike train: the event a spike at n
    sends through a synapse of delay d is delivered iff the source does not fire again before it
    arrives, i.e. at no step in (n, n + d); otherwise it is lost.  Returns (delivered-or-in-flight,
    lost) as sets of (syn, n_emit, k)."""
    T, N = spikes.shape
    kept, lost = set(), set()
    for i in range(N):
        times = [int(t) for t in np.nonzero(spikes[:, i])[0]]
        for p in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            d = int(D[p])
            for x, n in enumerate(times):
                nxt = times[x + 1] if x + 1 < len(times) else None
                (lost if nxt is not None and nxt < n + d else kept).add((p, n, n + d))
    return kept, lost


def replay_time_bins(spikes: np.ndarray, row_ptr, D, bins: int):
    """`bins` time bins per synapse (Section 4.3 "LossyRingDelay(n)", read as a ring of spike times
    shorter than the delay): an event with arrival step k is written to bin k mod bins, over
    whatever is there; at step t bin t mod bins is looked at and delivers if its event is due.
    Replayed per synapse step by step.  Returns (delivered-or-in-flight, lost) as sets of
    (syn, n_emit, k)."""
    T, N = spikes.shape
    kept, lost = set(), set()
    for i in range(N):
        fired = spikes[:, i] != 0
        for p in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            d = int(D[p])
            ring = [None] * bins                     # (n_emit, k) or None
            for t in range(T):
                held = ring[t % bins]
                if held is not None and held[1] == t:
                    kept.add((p, held[0], held[1]))
                    ring[t % bins] = None
                if fired[t]:
                    k = t + d
                    if ring[k % bins] is not None:
                        lost.add((p,) + ring[k % bins])
                    ring[k % bins] = (t, k)
            for held in ring:                        # still in flight when the run ends
                if held is not None:
                    kept.add((p,) + held)
    return kept, lost


def currents_from_events(events, col, amp, T: int, N: int) -> np.ndarray:
    """Sum the amplitudes of a list of (syn, n_emit, k) at their arrival step."""
    I = np.zeros((T, N), np.float64)
    for p, _, k in events:
        if k < T:
            I[k, col[p]] += amp[p]
    return I


def erlang_b(c: int, a: float) -> float:
    """Blocking probability of an M/G/c/c loss system with offered load a
    (recurrence B(0)=1, B(k) = a B(k-1) / (k + a B(k-1)))."""
    b = 1.0
    for k in range(1, c + 1):
        b = a * b / (k + a * b)
    return b
