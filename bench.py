#!/usr/bin/env python3
"""Benchmark of the delayed spike-event delivery hot path on one MI355X.

One "step" is one pass of the whole hot path over the workload: reset, T time
steps forward (pop, drive, LIF, compaction, fan-out, enqueue) and the reverse
sweep with weight and delay gradients.  Default workload: the 100,000-neuron x
1,000-fan-out network (1e8 synapses, delays 1..250 steps, 1,000 time steps,
ring queue), synthetic and seeded.

Prints ONE JSON line: metric "synaptic events delivered/s (fwd)" plus the
forward+backward time per time step, the HBM roofline of the dominant kernel,
the drop rate (of the selected queue, and of FIFO[32] on the same network in a
short leg of its own when the default workload runs), and the CPU oracle timed
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
# algorithmic bytes per event and per neuron-step: forward 8 B row entry + 1 B delay share + 8 B
# cell read-modify-write (ring) or 9 + 8 B slot write + 8 B occupancy (bounded); backward 9 + 4 B
# adjoint gather + 16 B of gradient read-modify-writes; per-synapse queues: 9 + 2 B key write + 4 B
# state read-modify-write per event, and 2 B of queue state per synapse, trial and time step (every
# queue is looked at in every step: that is what the organisation costs)
FWD_B_EVENT = {"ring": 17, "fifo": 25, "sorted": 25, "syn": 15, "latest": 13, "bins": 21}
SYN_B_QUEUE_STEP = 2
FWD_B_NEURON = 20          # queue row read + clear, V read + write, U tape write
BWD_B_EVENT = 29
BWD_B_NEURON = 16


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg3", choices=["cfg0", "cfg1", "cfg2", "cfg3", "cfg4"])
    ap.add_argument("--queue", default="ring", choices=["ring", "fifo", "sorted", "syn", "latest", "bins"])
    ap.add_argument("--capacity", type=int, default=32)
    ap.add_argument("--time-steps", type=int, default=0, help="override the workload's T")
    ap.add_argument("--drive-hz", type=float, default=0.0, help="override the rate of the Poisson drive")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-fifo-leg", action="store_true", help="skip the FIFO[32] comparison leg of the default workload")
    ap.add_argument("--graph-forward", action="store_true",
                    help="also time the forward run replayed from a captured HIP graph (reported as graph_forward_ms)")
    ap.add_argument("--phase-clocks", action="store_true",
                    help="run on the library built with phase clocks (python -m paper_2512_05906_amd.build --phase-clocks) "
                         "and add the phases of the ring's window expansion to the line; a diagnostic, not a bench line")
    ap.add_argument("--cpu-sample-events", type=float, default=4e7)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2512_05906_amd import build

    if args.phase_clocks:
        if not os.path.exists(build.LIB_PHASE):
            build.build_library(phase_clocks=True)
        os.environ["ADSEQ_LIB"] = build.LIB_PHASE
    from paper_2512_05906_amd import adseq, synth

    if not os.path.exists(build.LIB):   # load what is built; build only if nothing is
        build.build_library()
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    wl = getattr(synth, args.workload)()
    if args.drive_hz > 0.0:
        wl.ext_rate_hz = args.drive_hz
    T = args.time_steps or wl.n_steps
    B, N = wl.batch, wl.n_neurons
    BN = B * N
    kind = {"ring": adseq.RING, "fifo": adseq.FIFO, "sorted": adseq.SORTED, "syn": adseq.SYN_FIFO, "latest": adseq.SYN_LATEST, "bins": adseq.SYN_BINS}[args.queue]
    cap = 0 if kind == adseq.RING else (1 if kind == adseq.SYN_LATEST else args.capacity)
    fan = wl.n_synapses // N
    # room on the tape of the bounded kinds: ten times the spikes of a run at 20 Hz
    spike_cap = max(int(10 * BN * T * 20.0 * wl.dt_ms * 1e-3), 4 * BN)
    sim = adseq.Adseq(wl, kind, cap, record_tape=True, max_steps=T, tape_spike_capacity=spike_cap,
                      tape_event_capacity=(spike_cap * fan if kind != adseq.RING else 0))
    y = torch.from_numpy(synth.spike_count_targets(wl)).to(dev).reshape(-1)
    g_w = torch.empty(wl.n_synapses, dtype=torch.float32, device=dev)
    g_d = torch.empty(wl.n_synapses, dtype=torch.float32, device=dev)
    counts_i = torch.empty(BN, dtype=torch.int32, device=dev)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]

    def one_step(evs=None):
        sim.reset()
        if evs:
            evs[0].record()
        sim.run(0, T)
        if evs:
            evs[1].record()
        # loss glue (plumbing, not the path): dL/dcount of the MSE spike-count loss
        sim.spike_counts(counts_i)
        dc = (2.0 / BN) * (counts_i.to(torch.float32) - y)
        sim.backward(dc, None, g_w, g_d)
        if evs:
            evs[2].record()

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        one_step(ev[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    fwd_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    bwd_ms = float(np.mean([e[1].elapsed_time(e[2]) for e in ev]))
    phase_clocks = None
    if args.phase_clocks and kind == adseq.RING:
        import ctypes
        ticks = (ctypes.c_uint64 * 24)()
        rc = sim.lib.adseq_debug_phase_clocks(sim.h, ticks, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
        assert rc == 0, rc
        names = ["staging: walk over the spike words", "staging: counters", "staging: piece offsets", "staging: row loads + counting in LDS",
                 "staging: scan", "staging: ordering in LDS", "staging: run stores", "staging: cursors", "accumulation: counters + clearing the tile",
                 "accumulation: run loads + adds in LDS", "accumulation: tile to window"]
        nwin = max(1, int(ticks[15]))
        # (block 0 of each launch; the expansions of the last forward run from step 512 on, where the spike history is full)
        phase_clocks = {"windows": nwin, "us_per_window": {nm: round(ticks[i] * 0.01 / nwin, 3) for i, nm in enumerate(names)}}
        ngat = max(1, int(ticks[19]))
        phase_clocks["gathers"] = ngat   # (far gathers of the last reverse sweep, block 0 of each launch)
        phase_clocks["us_per_gather"] = {nm: round(ticks[16 + i] * 0.01 / ngat, 3) for i, nm in enumerate(
            ["gather: walk over the spike words", "gather: row pieces, adjoints, sums", "gather: the block's other wavefronts"])}
        spans = (ctypes.c_uint64 * 3072)()
        assert sim.lib.adseq_debug_block_spans(sim.h, spans, ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)) == 0
        sp = np.array(spans[:], dtype=np.float64).reshape(3, 512, 2)
        for k, nm in enumerate(("staging", "accumulation", "gather")):   # blocks of the last launch of each pass: when they began and ended
            on = sp[k][:, 1] > 0
            if on.any():
                t0 = sp[k][on, 0].min()
                phase_clocks[nm + "_blocks_last_launch_us"] = {
                    "blocks": int(on.sum()), "last_begin": round((sp[k][on, 0].max() - t0) * 0.01, 2),
                    "first_end": round((sp[k][on, 1].min() - t0) * 0.01, 2), "median_end": round((np.median(sp[k][on, 1]) - t0) * 0.01, 2),
                    "last_end": round((sp[k][on, 1].max() - t0) * 0.01, 2)}
    c = sim.counters()
    assert c["error_bits"] == 0, c
    delivered, offered, dropped = c["delivered"], c["enqueued"], c["dropped"]
    spikes = c["tape_spikes"]
    mean_rate_hz = spikes / BN / (T * wl.dt_ms * 1e-3)
    value = delivered / (fwd_ms * 1e-3)
    # Events the passes actually handle.  The ring materialises an event only when the window that
    # holds its arrival step opens, so its forward pass handles the events delivered inside the run
    # (not the ones still implicit at its end); the bounded kinds read every offered row entry.  The
    # reverse sweep of every kind gathers for the events delivered inside the run.
    fwd_events = delivered if args.queue == "ring" else offered
    fwd_bytes = FWD_B_EVENT[args.queue] * fwd_events + FWD_B_NEURON * BN * T
    if args.queue in ("syn", "latest", "bins"):
        fwd_bytes += SYN_B_QUEUE_STEP * B * wl.n_synapses * T
    bwd_bytes = BWD_B_EVENT * delivered + BWD_B_NEURON * BN * T
    achieved_run = (fwd_bytes + bwd_bytes) / ((fwd_ms + bwd_ms) * 1e-3) / 1e9

    # Per-kernel durations, measured live with HIP events on the launch stream in one extra
    # pass after the timed steps (an event after every launch would perturb the timed ones).
    sim.profile(True)
    one_step()
    prof = sim.profile_read()
    sim.profile(False)
    in_run = delivered  # admitted events that arrive inside the run: the ones backward touches
    alg = {  # algorithmic bytes per run of each kernel class
        "fan_out": (FWD_B_EVENT[args.queue]) * fwd_events,
        "lif": FWD_B_NEURON * BN * T + (SYN_B_QUEUE_STEP * B * wl.n_synapses * T if args.queue in ("syn", "latest", "bins") else 0),
        "bwd_gather": BWD_B_EVENT * in_run,
        "bwd_neurons": BWD_B_NEURON * BN * T,
    }
    if args.queue == "ring":
        # events that arrive inside the window they were emitted in are scattered by the step
        # kernel itself; the others by the window expansion.  Share of the former for a spike at
        # a uniformly distributed window phase: sum_D P(D) max(0, W - D) / W.
        W = int(os.environ.get("ADSEQ_RING_WINDOW", "16"))
        if wl.delay_steps is not None:
            D = np.bincount(wl.delay_steps, minlength=W + 1).astype(np.float64)
        else:
            D = np.bincount(np.maximum(1, np.ceil(wl.delay_ms.astype(np.float64) / wl.dt_ms)).astype(np.int64),
                            minlength=W + 1).astype(np.float64)
        near = float((D[:W] * (W - np.arange(W))).sum() / (W * D.sum()))
        alg["lif"] += FWD_B_EVENT["ring"] * fwd_events * near
        alg["fan_out"] = FWD_B_EVENT["ring"] * fwd_events * (1.0 - near)
        alg["bwd_neurons"] += BWD_B_EVENT * in_run * near
        alg["bwd_gather"] = BWD_B_EVENT * in_run * (1.0 - near)
        label = {"fan_out": "k_win_bin + k_win_acc (expansion of one window: stage by target part, sum in LDS)",
                 "lif": "k_step_win (pop + drive + LIF + spike bits + in-window scatter)",
                 "bwd_gather": "k_bwd_win (far queue terms and gradient sums of one window)",
                 "bwd_neurons": "k_bwd_step_win (adjoint update + in-window gather)"}
    else:
        label = {"fan_out": "k_fanout_step (CSR fan-out, full-target drops, contender registration)",
                 "lif": ("k_synq_pop + k_neurons (look at every queue, then drive + LIF + spike words)"
                         if args.queue in ("syn", "latest", "bins") else "k_neurons (admission + pop + drive + LIF + spike words)"),
                 "bwd_gather": "k_bwd_rows (adjoint gathers and gradient sums of the step's recorded spikes)",
                 "bwd_neurons": "k_bwd_neurons (adjoint update)"}
    if args.queue == "ring" and prof.get("bwd_neurons", {}).get("launches", T) < T:
        # fewer launches than steps: the reverse steps of a window ran in one launch each (resident reverse kernel)
        label["bwd_neurons"] = ("k_bwd_xcd (the reverse steps of one window in one launch: adjoint update + in-window gather, a grid barrier per step)"
                                if os.environ.get("ADSEQ_RING_REVERSE_FLOW", "1") == "0" else
                                "k_bwd_flow (the reverse steps of one window in one launch: adjoint update + in-window gather, no grid barrier: a gather waits for the cell it reads)")
    if args.queue == "ring" and prof.get("lif", {}).get("launches", T) < T:
        # likewise forward: the steps of a window in one launch over the whole chip
        label["lif"] = "k_fwd_chip (the steps of one window in one launch: pop + drive + LIF + spike bits + in-window scatter, a grid barrier per step)"
    kernels = {}
    for k, v in prof.items():
        if v["launches"]:
            kernels[k] = {"kernel": label[k], "ms_per_run": v["ms"], "launches": v["launches"],
                          "avg_us": v["ms"] * 1e3 / v["launches"],
                          "algorithmic_bytes_per_launch": alg[k] / v["launches"],
                          "achieved_GBs": alg[k] / (v["ms"] * 1e-3) / 1e9}
    dom = max(kernels, key=lambda k: kernels[k]["ms_per_run"])
    # HBM bytes per launch of the dominant kernel from the committed rocprofv3 --pmc runs (not
    # measured in this run: counters need the profiler), with the commit they were taken at
    traffic = None
    traffic_at = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        tj = json.load(open(tpath))
        traffic = tj.get(f"{args.workload}/{args.queue}", {}).get(dom)
        traffic_at = tj.get("_taken_at")

    # what a plain device-to-device copy of 1 GiB reaches on this machine (read + write bytes per second):
    # the practical ceiling next to the datasheet peak
    ca = torch.empty(1 << 28, dtype=torch.float32, device=dev)
    cb = torch.empty_like(ca)
    ce = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
    copy_gbs = 0.0
    for _ in range(3):
        ce[0].record(); cb.copy_(ca); ce[1].record(); torch.cuda.synchronize()
        copy_gbs = max(copy_gbs, 2.0 * ca.numel() * 4 / (ce[0].elapsed_time(ce[1]) * 1e-3) / 1e9)
    del ca, cb

    out = {
        "metric": "synaptic events delivered/s (fwd)",
        "value": value,
        "unit": "events/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall * 1e3 / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={N} fan_out={fan} synapses={wl.n_synapses} "
                               f"d_max={wl.d_max_steps} T={T} B={B} queue={args.queue}"
                               + (f"[{cap}]" if cap else "") + f" drive={wl.ext_rate_hz}Hz",
                   "mean_rate_hz": mean_rate_hz, "events_per_run": offered,
                   "delivered_per_run": delivered},
        "fwd_ms_per_run": fwd_ms,
        "bwd_ms_per_run": bwd_ms,
        "fwd_us_per_timestep": fwd_ms * 1e3 / T,
        "fwdbwd_us_per_timestep": (fwd_ms + bwd_ms) * 1e3 / T,
        "drop_rate": dropped / max(1, offered),
        "roofline": {"bound": "hbm", "achieved": kernels[dom]["achieved_GBs"], "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": kernels[dom]["achieved_GBs"] / HBM_PEAK_GBS,
                     "traffic": traffic, "traffic_taken_at_commit": traffic_at, "kernel": label[dom],
                     "avg_launch_us": kernels[dom]["avg_us"],
                     "algorithmic_bytes_per_launch": kernels[dom]["algorithmic_bytes_per_launch"],
                     "whole_run_achieved_GBs": achieved_run,
                     "whole_run_frac": achieved_run / HBM_PEAK_GBS,
                     "measured_copy_GBs": copy_gbs,
                     "frac_of_measured_copy": kernels[dom]["achieved_GBs"] / copy_gbs if copy_gbs else None},
        "kernels": kernels,
    }
    if phase_clocks:
        out["phase_clocks"] = phase_clocks

    if args.graph_forward:
        # The forward run (reset + T steps) captured once into a HIP graph and replayed: what graph
        # launch would buy over the launches issued one by one (it does not shorten the gaps between
        # dependent kernels).  The reset's clearing is done by fill kernels, never by memset nodes.
        gstream = torch.cuda.Stream()
        gstream.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(gstream):
            sim.reset()
            sim.run(0, T)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=gstream):
            sim.reset()
            sim.run(0, T)
        ge = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        times = []
        for _ in range(3):
            torch.cuda.synchronize()
            ge[0].record(); graph.replay(); ge[1].record()
            torch.cuda.synchronize()
            times.append(ge[0].elapsed_time(ge[1]))
        U_graph = sim.membrane_tape(T).clone()
        sim.reset(); sim.run(0, T); torch.cuda.synchronize()
        out["graph_forward_ms"] = min(times)
        out["graph_forward_matches_eager"] = bool(torch.equal(U_graph.view(torch.int32), sim.membrane_tape(T).view(torch.int32)))

    # The comparison the headline config asks for (ring against FIFO[32], Section 6.5 "Spike drop
    # rates"): a short leg with the bounded FIFO on the same network and drive.  The lost recurrent
    # input lowers the firing rate, so its events per second are not comparable one to one; the
    # drop rate is the figure.
    if args.queue == "ring" and args.workload == "cfg3" and not args.no_fifo_leg:
        fsim = adseq.Adseq(wl, adseq.FIFO, 32, record_tape=True, max_steps=T, tape_spike_capacity=spike_cap,
                           tape_event_capacity=spike_cap * fan)
        fev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]

        def fifo_step(evs=None):
            fsim.reset()
            if evs:
                evs[0].record()
            fsim.run(0, T)
            if evs:
                evs[1].record()
            fsim.spike_counts(counts_i)
            dc = (2.0 / BN) * (counts_i.to(torch.float32) - y)
            fsim.backward(dc, None, g_w, g_d)
            if evs:
                evs[2].record()

        fifo_step()
        fifo_step(fev)
        torch.cuda.synchronize()
        fc = fsim.counters()
        assert fc["error_bits"] == 0, fc
        f_fwd, f_bwd = fev[0].elapsed_time(fev[1]), fev[1].elapsed_time(fev[2])
        out["fifo32"] = {"fwd_ms": f_fwd, "bwd_ms": f_bwd, "events_per_s": fc["delivered"] / (f_fwd * 1e-3),
                         "drop_rate": fc["dropped"] / max(1, fc["enqueued"]),
                         "mean_rate_hz": fc["tape_spikes"] / BN / (T * wl.dt_ms * 1e-3),
                         "offered": fc["enqueued"], "dropped": fc["dropped"], "delivered": fc["delivered"]}
        fsim.close()

    if not args.no_cpu_baseline:
        from oracle import oracle
        per_step = (sim.membrane_tape(T) >= wl.v_thresh).sum(dim=(1, 2)).cpu().numpy()
        ev_cum = np.concatenate([[0], np.cumsum(per_step)]) * fan
        Ts = int(np.searchsorted(ev_cum, args.cpu_sample_events))
        Ts = max(10, min(T, Ts))
        t1 = time.perf_counter()
        ref = oracle.Run(wl, kind, cap, n_steps=Ts, n_threads=min(B, os.cpu_count() or 1))
        t_or = time.perf_counter() - t1
        rc = ref.counters()
        U = sim.tape()["U"][:Ts].cpu().numpy()
        parity = bool(np.array_equal(U.view(np.uint32), ref.U.view(np.uint32)))
        out["cpu_baseline"] = {"value": rc["delivered"] / t_or, "unit": "events/s",
                               "cores": min(B, os.cpu_count() or 1), "cores_available": os.cpu_count(),
                               "kind": "oracle",
                               "sample": f"first {Ts} of {T} time steps of the same network "
                                         f"({rc['enqueued']} events offered, {rc['delivered']} delivered), "
                                         f"forward only, {t_or:.1f} s",
                               "membrane_bit_exact_vs_gpu_on_sample": parity}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
