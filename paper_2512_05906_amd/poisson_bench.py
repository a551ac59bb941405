#!/usr/bin/env python3
"""Open-loop Poisson benchmark and drop-rate sweep on one MI355X.

The workload has the shape of the paper's Poisson benchmark (Section 5.1): many independent
queues, each fed by its own Poisson source (mean interval lambda = 400 steps) through one
homogeneous delay (80 steps, dt = 0.025 ms); per time step the queue is popped
(adseq_deliver) and the step's spikes are enqueued (adseq_enqueue).  The spike lists are
drawn beforehand (seeded) and are resident on the GPU when the timed region starts.

Prints one JSON line per (queue kind, capacity, pressure): time per time step, delivered
events/s, drop rate, and the Erlang-B blocking probability of a loss system with `capacity`
servers and offered load a = delay / lambda (a bounded bag with on-time delivery is one: the
holding time of a slot is the delay, and the loss formula does not depend on the holding-time
distribution).  The paper's own rule of thumb (Section 6.5 "Spike drop rates": pressure delay / lambda around 0.5
needs only a very small queue) is the a << capacity corner of this table.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def erlang_b(servers: int, load: float) -> float:
    """Blocking probability B(c, a) by the standard recurrence B(0) = 1, B(k) = a B(k-1) / (k + a B(k-1))."""
    b = 1.0
    for k in range(1, servers + 1):
        b = load * b / (k + load * b)
    return b


def run_case(torch, adseq, synth, kind_name, cap, n_queues, delay, interval, T, repeats=3, network=None):
    """One open-loop run.  network = None: n_queues independent queues with one source each and one
    delay; else a Workload whose neurons all fire as Poisson sources with mean interval `interval`
    steps (the network's own delays and fan-out)."""
    import numpy as np
    kind = {"ring": adseq.RING, "fifo": adseq.FIFO, "sorted": adseq.SORTED, "syn": adseq.SYN_FIFO, "latest": adseq.SYN_LATEST, "bins": adseq.SYN_BINS}[kind_name]
    wl = network if network is not None else synth.poisson_queues(n_queues, delay, n_steps=T)
    if network is not None:
        n_queues = wl.n_neurons
    if interval > 0:
        rate_hz = 1.0 / (interval * wl.dt_ms * 1e-3)
        lists = synth.poisson_spike_lists(n_queues, 1, T, rate_hz, wl.dt_ms, seed=11)
    else:   # control: no source ever fires
        lists = [np.zeros(0, np.int32) for _ in range(T)]
    counts = np.array([len(x) for x in lists], np.int32)
    offs = np.concatenate([[0], np.cumsum(counts)]).astype(np.int64)
    sim = adseq.Adseq(wl, kind, cap if kind != adseq.RING else 0)
    dev = sim.dev
    ids = torch.from_numpy(np.concatenate(lists + [np.zeros(1, np.int32)])).to(dev)
    cnt = torch.from_numpy(counts).to(dev)
    I = torch.empty(n_queues, dtype=torch.float32, device=dev)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    times = []
    for _ in range(repeats + 1):
        sim.reset()
        ev[0].record()
        sim.run_open(0, T, ids, offs[:T], cnt, I, 0)
        ev[1].record()
        torch.cuda.synchronize()
        times.append(ev[0].elapsed_time(ev[1]))
    ms = float(np.median(times[1:]))
    c = sim.counters()
    sim.close()
    a = delay / interval if interval > 0 else 0.0
    if network is not None and interval > 0:
        # offered load of one target's queue: fan-in x rate x mean delay (all in steps)
        fan_in = wl.n_synapses / wl.n_neurons
        a = fan_in * (1.0 + wl.d_max_steps) / 2.0 / interval
    return {"queue": kind_name if interval > 0 else kind_name + " (control: no events)", "capacity": cap if kind != adseq.RING else None, "n_queues": n_queues,
            "delay_steps": delay, "mean_interval_steps": interval, "pressure": a, "time_steps": T,
            "us_per_time_step": ms * 1e3 / T, "ns_per_time_step_per_queue": ms * 1e6 / T / n_queues,
            "delivered_events_per_s": c["delivered"] / (ms * 1e-3),
            "offered": c["enqueued"], "dropped": c["dropped"],
            "drop_rate": c["dropped"] / max(1, c["enqueued"]),
            "erlang_b": None if kind in (adseq.RING, adseq.SYN_LATEST, adseq.SYN_BINS) else erlang_b(cap, a)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--queues", type=int, default=10000)
    ap.add_argument("--time-steps", type=int, default=4000)
    ap.add_argument("--delay", type=int, default=80)
    ap.add_argument("--sweep", action="store_true", help="capacity x pressure sweep of the drop rate")
    ap.add_argument("--capacities", default="1,2,4,8", help="FIFO capacities of the sweep")
    ap.add_argument("--pressures", default="0.2,0.5,1,2,4",
                    help="pressures a = delay / mean interval of the sweep (keep the interval well above one step: "
                         "a source fires at most once per step, so short intervals are not Poisson any more)")
    ap.add_argument("--cfg2-rates", action="store_true",
                    help="the 10,000-neuron x 1,000-fan-out network driven open loop at exactly 5, 20 and 80 Hz: "
                         "ring against per-target FIFOs of capacity 8 and 32")
    args = ap.parse_args()
    import torch
    from paper_2512_05906_amd import adseq, synth
    if not torch.cuda.is_available():
        print("poisson_bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    # the last case is the control the paper's "DoNothing" queue gives (Section 4.3): the same
    # calls with no event ever inserted, i.e. the cost that does not depend on the queue's content
    cases = [("ring", 0, 400), ("fifo", 4, 400), ("sorted", 4, 400), ("syn", 4, 400), ("latest", 1, 400), ("bins", 4, 400), ("ring", 0, 0)]
    if args.sweep:
        caps = [int(x) for x in args.capacities.split(",")]
        kinds = [("fifo", c) for c in caps] + [(k, c) for k, c in (("sorted", 4), ("syn", 4)) if c in caps]
        cases = [(k, c, args.delay / float(a)) for a in args.pressures.split(",") for k, c in kinds]
    if args.cfg2_rates:
        net = synth.cfg2(n_steps=min(args.time_steps, 2000))
        for hz in (5.0, 20.0, 80.0):
            interval = 1.0 / (hz * net.dt_ms * 1e-3)
            for kind, cap in (("ring", 0), ("fifo", 8), ("fifo", 32)):
                r = run_case(torch, adseq, synth, kind, cap, 0, 0, interval, net.n_steps, network=net)
                r["rate_hz"] = hz
                print(json.dumps(r), flush=True)
        return
    for kind, cap, lam in cases:
        print(json.dumps(run_case(torch, adseq, synth, kind, cap, args.queues, args.delay, lam,
                                  args.time_steps)), flush=True)


if __name__ == "__main__":
    main()
