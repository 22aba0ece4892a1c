#!/usr/bin/env python3
"""Benchmark of the SERE batch-decode MoE layer on one MI355X.

A "step" is one pass of the whole hot path (router, top-K, re-routing,
compaction, grouped expert FFN, combine) over one decode batch whose inputs
and weights are already resident in HBM.  Consecutive steps use different
copies of the layer's weights so that the 256 MB last-level cache cannot serve
them (a real model runs a different layer next).  Prints ONE JSON line.

The headline is the largest Qwen3-30B-A3B-shaped configuration (batch 128, S = 2, rho = 0);
the same JSON line carries, under "configs", every layer shape of the task (and the
Qwen1.5-MoE-shaped one) with its (S, rho) grid from the paper's main tables.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--only-headline]
                    [--S s] [--rho r] [--sweep] [--rho-sweep] [--layers L] [--no-graph]
"""
from __future__ import annotations

import argparse
from dataclasses import replace
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X HBM3E, published peak
TARGET_FRAC = 0.70        # the task's target: whole SERE step at >= 70 % of that peak on the expert bytes read
GRAPH_STEPS = 32          # decode steps captured in one HIP graph (fewer if fewer are timed; see Runner.time)
STAT_REPLAYS = 8          # graph replays behind median / p10 / p90 (extra, untimed for `value`, if fewer were timed)
HEADLINE = "qwen3_b128"
ALL_WORKLOADS = ("qwen3_b128", "qwen3_b32", "dsv2lite_b64", "mixtral_b64", "qwen15_b32", "tiny")
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def recorded_traffic(workload, S, rho):
    """HBM bytes per launch (read + write) of the two FFN kernels as recorded from rocprofv3
    --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/hbm_traffic.json; commands and scale factors in
    profiles/sere_step_<workload>.md).  The record names the library sources it was taken on;
    if they have changed since, nothing is reported (null)."""
    from paper_2602_07616_amd import build as lib_build
    try:
        rec = json.load(open(TRAFFIC_FILE))
    except (OSError, ValueError):
        return {}, "no record"
    if rec.get("source_hash") != lib_build.source_hash():
        return {}, "library sources changed since the counters were read (commit %s)" % rec.get("commit")
    entry = rec.get("entries", {}).get(f"{workload}|{S}|{float(rho)}")
    if entry is None:
        return {}, "this configuration was not counted"
    return entry, "rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE at commit %s" % rec.get("commit")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=384)
    ap.add_argument("--warmup", type=int, default=40)
    ap.add_argument("--workload", default=None,
                    help=f"headline workload (default {HEADLINE}); naming one implies --only-headline")
    ap.add_argument("--only-headline", action="store_true",
                    help="skip the other layer shapes of the \"configs\" object")
    ap.add_argument("--tokens", type=int, default=0,
                    help="with --workload: batch size T in place of the workload's own (same layer, same seeds)")
    ap.add_argument("--S", type=int, default=0, help="select_top_k of the headline SERE step (0: the workload's first grid setting)")
    ap.add_argument("--rho", type=float, default=0.0, help="threshold of the headline SERE step")
    ap.add_argument("--copies", type=int, default=0, help="weight copies to rotate over (0: auto)")
    ap.add_argument("--grid", action="store_true", help="(kept for compatibility: the grid is always timed)")
    ap.add_argument("--sweep", action="store_true", help="also time the batch-size sweep")
    ap.add_argument("--prefill", action="store_true",
                    help="also time prefill-sized batches (512, 1024, 2048 tokens) of the Qwen3-shaped layer")
    ap.add_argument("--batches", default="",
                    help="with --prefill: comma-separated batch sizes in place of 512,1024,2048")
    ap.add_argument("--rho-sweep", action="store_true",
                    help="also time thresholds 0.0 .. 1.0 at select_top_k = 1 (active experts and us)")
    ap.add_argument("--layers", type=int, default=0,
                    help="also time a chained stack of this many layers (x <- x + MoE(x), one HIP graph)")
    ap.add_argument("--no-graph", action="store_true", help="plain stream launches, no HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-sere", action="store_true",
                    help="time only the headline SERE step (for per-kernel profiles)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="with --only-sere: also run a plain 256 MiB device copy 4 times, so that a "
                         "counter run holds a kernel of known traffic to scale FETCH_SIZE/WRITE_SIZE by")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    return ap.parse_args()


class Runner:
    """One workload resident in HBM `copies` times; times steps of one entry point."""

    def __init__(self, wl, sim, copies, use_graph):
        import numpy as np
        import torch
        from paper_2602_07616_amd import device
        self.torch = torch
        self.wl = wl
        self.use_graph = use_graph
        weights = device.DeviceLayer.from_workload(wl, np.zeros((1, 1), np.float32), 1, 0.0).weights() \
            if sim is None else None
        if sim is None:
            # the similarity matrix is part of the product path too: estimated on the GPU from the
            # layer's own weights and seeded calibration tokens (untimed set-up, as in the paper)
            sim = device.similarity_on_device(wl, weights)
        first = device.DeviceLayer.from_workload(wl, sim, 1, 0.0, weights=weights)
        self.sim = sim
        self.layers = [first]
        for _ in range(copies - 1):
            w = tuple(None if t is None else t.clone() for t in first.weights())
            self.layers.append(device.DeviceLayer.from_workload(wl, sim, 1, 0.0, weights=w))
        self.stream = torch.cuda.Stream()

    def _call(self, layer, mode):
        if mode == "sere":
            layer.run_decode(self.stream, with_outputs=False)
        elif mode == "baseline":
            layer.run_baseline(self.stream, with_outputs=False)
        elif mode == "reroute":
            layer.run_reroute(self.stream, with_outputs=False)
        else:
            layer.run_route(self.stream, with_outputs=False)

    def set_knobs(self, S, rho):
        for l in self.layers:
            l.set_knobs(S, rho)

    def time(self, mode, steps, warmup, hot=False):
        """-> (mean us/step over exactly `steps` steps, per-replay us/step list, host wall us/step,
        launch label).  hot: every step on the same copy of the weights (the last-level cache may
        serve them).  One HIP graph holds min(steps, GRAPH_STEPS) consecutive steps, each on the
        next copy of the weights, as a decoder's graph holds all its layers (a graph launch costs
        about 12 us on this machine, which a graph of four steps would add as 3 us to every step).
        Exactly `steps` steps are timed: whole replays of that graph plus, if `steps` is not a
        multiple, one replay of a second graph holding the remainder.  The per-replay list (for
        median / p10 / p90) has at least STAT_REPLAYS entries: replays beyond the timed ones are
        made after the timed region and do not enter the mean."""
        torch = self.torch
        layers = self.layers[:1] * len(self.layers) if hot else self.layers
        n = len(layers)
        per_graph = min(steps, GRAPH_STEPS) if self.use_graph else min(steps, n)
        rounds, rem = divmod(steps, per_graph)

        def capture(count, first):
            if not self.use_graph or count == 0:
                return None
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g, stream=self.stream):
                for i in range(count):
                    self._call(layers[(first + i) % n], mode)
            for _ in range(3):      # settle: the first replays of a new graph run slower
                g.replay()
            return g

        def run(graph, count, first):
            if graph is not None:
                graph.replay()
            else:
                for i in range(count):
                    self._call(layers[(first + i) % n], mode)

        with torch.cuda.stream(self.stream):
            for i in range(warmup):
                self._call(layers[i % n], mode)
            self.stream.synchronize()
            main = capture(per_graph, 0)
            tail = capture(rem, rounds * per_graph)
            self.stream.synchronize()
            extra = max(0, STAT_REPLAYS - rounds)
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(rounds + 2 + extra)]
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            ev[0].record(self.stream)
            for r in range(rounds):
                run(main, per_graph, r * per_graph)
                ev[r + 1].record(self.stream)
            run(tail, rem, rounds * per_graph)
            ev[rounds + 1].record(self.stream)
            torch.cuda.synchronize()
            wall = time.perf_counter() - t0
            for r in range(extra):
                run(main, per_graph, 0)
                ev[rounds + 2 + r].record(self.stream)
            torch.cuda.synchronize()
        total_ms = ev[0].elapsed_time(ev[rounds + 1])
        per_round = [ev[r].elapsed_time(ev[r + 1]) * 1e3 / per_graph for r in range(rounds)]
        per_round += [ev[rounds + 1 + r].elapsed_time(ev[rounds + 2 + r]) * 1e3 / per_graph for r in range(extra)]
        label = (f"hip-graph of {per_graph} steps x {rounds} replays" + (f" + one graph of {rem} steps" if rem else "")
                 if self.use_graph else "stream")
        return total_ms * 1e3 / steps, per_round, wall * 1e6 / steps, label

    def stage_times(self, mode, steps):
        """Average duration of each kernel stage (HIP events attached to each dispatch on the launch stream)."""
        from paper_2602_07616_amd import binding as B
        n = len(self.layers)
        with self.torch.cuda.stream(self.stream):
            for i in range(n):
                self._call(self.layers[i], mode)
            self.stream.synchronize()
            B.sere_stage_timing(True)
            for i in range(steps):
                self._call(self.layers[i % n], mode)
            ms, cnt = B.sere_stage_timing_read()
            B.sere_stage_timing(False)
        return {s: (ms[s] * 1e3 / cnt[s] if cnt[s] else 0.0) for s in ms}

    def similarity_timing(self):
        """The set-up step (sere_similarity, Frobenius metric) once more with per-kernel events: us per
        calibration batch of the experts' forward pass and of the pair stage (Gram matrix of the
        experts' outputs on the fp64 matrix cores, distances, accumulation), and the pair stage's
        share of the fp64 MFMA peak: 2 * (upper-triangular 64 x 64 blocks) * n * d_h flop per batch."""
        from paper_2602_07616_amd import binding as B, device
        sp = self.wl.spec
        batches, n = self.wl.calib.shape[0], self.wl.calib.shape[1]
        B.sere_stage_timing(True)
        device.similarity_on_device(self.wl, self.layers[0].weights())
        ms, cnt = B.sere_stage_timing_read()
        B.sere_stage_timing(False)
        nb = (sp.experts + 63) // 64
        flop = 2.0 * (nb * (nb + 1) // 2) * 64 * 64 * n * sp.hidden
        pair_us = ms["sim_pairs"] * 1e3 / batches
        return {"calibration_batches": batches, "tokens_per_batch": n,
                "forward_us_per_batch": round((ms["gate_up"] + ms["down"]) * 1e3 / batches, 2),
                "pair_stage_us_per_batch": round(pair_us, 2),
                "pair_stage_roofline": {"bound": "mfma", "dtype": "f64", "achieved": round(flop / pair_us * 1e-6, 2),
                                        "peak": 78.6, "unit": "TFLOP/s", "frac": round(flop / pair_us * 1e-6 / 78.6, 4),
                                        "flop_per_batch": flop}}

    def plain_read(self, nbytes, launches=64):
        """What the memory system delivers for a plain read of `nbytes` of this workload's own weight
        bytes (library helper sere_stream_read): us per launch over back-to-back launches that each
        read a different region of the resident copies, so that no cache can serve them."""
        from paper_2602_07616_amd import binding as B
        torch = self.torch
        tensors = [l.w_gate_up for l in self.layers]
        cap = tensors[0].numel() * tensors[0].element_size()
        nbytes = min(int(nbytes) // 16 * 16, cap)
        per = max(1, cap // nbytes)
        regions = [(t, r * nbytes) for t in tensors for r in range(per)]
        sink = torch.zeros(4, dtype=torch.int32, device=tensors[0].device)
        flat = {id(t): t.view(torch.uint8).reshape(-1) for t in tensors}
        start, stop = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        with torch.cuda.stream(self.stream):
            for i in range(8):
                t, off = regions[i % len(regions)]
                B.sere_stream_read(flat[id(t)][off:], nbytes, sink, self.stream)
            start.record(self.stream)
            for i in range(launches):
                t, off = regions[i % len(regions)]
                B.sere_stream_read(flat[id(t)][off:], nbytes, sink, self.stream)
            stop.record(self.stream)
            stop.synchronize()
        return start.elapsed_time(stop) * 1e3 / launches, nbytes

    def active(self, mode):
        """(n_active_before, n_active_after) of the current knobs."""
        l = self.layers[0]
        if mode == "baseline":
            l.run_baseline(self.stream)
        else:
            l.run_decode(self.stream)
        self.stream.synchronize()
        na = l.route.num_active.cpu().tolist()
        return na[0], na[1]


def cpu_baseline(wl, sim, S, rho, budget_s):
    """The oracle as it stands, timed on the host cores on the same workload."""
    import oracle
    sp = wl.spec
    threads = oracle.max_threads()

    def step():
        oracle.layer(wl.hidden, wl.router_w, wl.w_gate_up, wl.w_down, wl.shared_gate_up,
                     wl.shared_down, sp.dtype, sp.top_k, sim, S, rho, want_base=False)
    t0 = time.perf_counter()
    step()
    first = time.perf_counter() - t0
    reps = max(1, min(300, int(budget_s / max(first, 1e-3)) - 1))
    times = [first]
    for _ in range(reps):
        t0 = time.perf_counter()
        step()
        times.append(time.perf_counter() - t0)
    return {"value": round(min(times) * 1e6, 1), "unit": "us/step", "cores": threads, "kind": "oracle",
            "sample": f"{len(times)} full SERE steps (S={S}, rho={rho}) of {sp.name} on all host threads; value = fastest step, mean_us = their mean",
            "mean_us": round(statistics.mean(times) * 1e6, 1)}


def measure_config(args, name, S, rho, steps, warmup, headline):
    """Everything reported for one layer shape: the SERE step at (S, rho), the step without
    re-routing, the (S, rho) grid of the paper's main tables, the routing-only entry points, the
    per-kernel durations and the roofline of the dominant kernel."""
    import numpy as np
    from paper_2602_07616_amd import workloads as wk
    spec = wk.SPECS[name]
    if headline and args.tokens > 0 and args.workload:
        spec = replace(spec, name=f"{spec.name}@T{args.tokens}", tokens=args.tokens)
    wl = wk.make_workload(spec)
    eb = spec.elem_bytes
    expert_bytes = spec.expert_bytes
    copies = args.copies or max(2, min(16, int(np.ceil(4.0e9 / (spec.experts * expert_bytes)))))
    run = Runner(wl, None, copies, not args.no_graph)
    if S <= 0:
        S, rho = spec.grid[0]
    quick = min(steps, 200)

    def measure(mode, S_, rho_, steps_, warmup_):
        run.set_knobs(S_, rho_)
        nb, na = run.active(mode)
        us, per_round, wall_us, label = run.time(mode, steps_, warmup_)
        n_exp = (nb if mode == "baseline" else na) + spec.shared
        gbs = n_exp * expert_bytes / us * 1e-3
        pr = sorted(per_round)
        pct = lambda q: round(pr[min(len(pr) - 1, int(q * len(pr)))], 2) if pr else None
        at_target = n_exp * expert_bytes / (TARGET_FRAC * HBM_PEAK_GBS) * 1e-3
        return {"us_per_step": round(us, 2), "median_round_us": round(statistics.median(per_round), 2) if per_round else None,
                "p10_round_us": pct(0.10), "p90_round_us": pct(0.90), "replays": len(per_round),
                "host_wall_us": round(wall_us, 2), "active_before": nb, "active_after": na,
                "experts_read": n_exp, "expert_gb_per_s": round(gbs, 1),
                "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                "target": {"frac_of_hbm_peak": TARGET_FRAC, "us_per_step_at_target": round(at_target, 2),
                           "met": bool(gbs / HBM_PEAK_GBS >= TARGET_FRAC), "us_above_target": round(max(0.0, us - at_target), 2)},
                "launch": label}

    sere = measure("sere", S, rho, steps, warmup)
    if args.only_sere:
        return {"sere": sere}, run, wl, S, rho
    base = measure("baseline", spec.top_k, 0.0, steps, warmup)
    out = {"tokens": spec.tokens, "hidden": spec.hidden, "experts": spec.experts, "top_k": spec.top_k,
           "inter": spec.inter, "shared": spec.shared, "dtype": "bf16" if spec.dtype == wk.BF16 else "f32",
           "select_top_k": S, "threshold": rho, "weight_copies": copies,
           "sere": sere, "no_reroute": base,
           "speedup_vs_no_reroute": round(base["us_per_step"] / sere["us_per_step"], 3)}
    grid = {}
    for gS, grho in spec.grid:
        if (gS, grho) == (S, rho):
            g = sere
        else:
            g = measure("sere", gS, grho, quick, min(warmup, 10))
        grid[f"S={gS},rho={grho}"] = {k: g[k] for k in ("us_per_step", "active_before", "active_after", "experts_read",
                                                         "expert_gb_per_s", "frac_of_hbm_peak")}
        grid[f"S={gS},rho={grho}"]["speedup_vs_no_reroute"] = round(base["us_per_step"] / g["us_per_step"], 3)
    out["grid"] = grid
    run.set_knobs(S, rho)
    route_us, _, _, _ = run.time("route", quick, 10)
    out["route_only_us"] = round(route_us, 2)
    if headline:
        hot_us, _, _, _ = run.time("sere", quick, 10, hot=True)
        for l in run.layers:      # top-K ids for the re-routing-only entry point
            l.run_route(run.stream)
        reroute_us, _, _, _ = run.time("reroute", quick, 10)
        out["reroute_only_us"] = round(reroute_us, 2)
        out["sere_hot_weights_us"] = round(hot_us, 2)
        out["similarity_setup"] = run.similarity_timing()

    # roofline of the dominant kernel: the gate/up projection streams 2/3 of the
    # surviving experts' bytes
    run.set_knobs(S, rho)
    stages = run.stage_times("sere", quick)
    gateup_bytes = sere["experts_read"] * 2 * spec.hidden * spec.inter * eb
    down_bytes = sere["experts_read"] * spec.hidden * spec.inter * eb
    achieved = gateup_bytes / stages["gate_up"] * 1e-3 if stages["gate_up"] else 0.0
    traffic, traffic_source = recorded_traffic(spec.name, S, rho)
    roofline = {"bound": "hbm", "kernel": "gate_up", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": traffic.get("gate_up"),
                "traffic_source": traffic_source,
                "algorithmic_bytes_per_launch": gateup_bytes,
                "avg_launch_us": round(stages["gate_up"], 2),
                "down": {"achieved": round(down_bytes / stages["down"] * 1e-3, 1) if stages["down"] else 0.0,
                         "frac": round(down_bytes / stages["down"] * 1e-3 / HBM_PEAK_GBS, 4) if stages["down"] else 0.0,
                         "avg_launch_us": round(stages["down"], 2), "algorithmic_bytes_per_launch": down_bytes,
                         "traffic": traffic.get("down")},
                "stage_us": {k: round(v, 2) for k, v in stages.items()}}
    if headline:
        # what a plain read of as many bytes of the same weights takes on this machine (context for
        # `frac`: the published peak is not attainable by any kernel), and a long read
        read_us, read_bytes = run.plain_read(gateup_bytes)
        long_us, long_bytes = run.plain_read(spec.experts * 2 * spec.hidden * spec.inter * eb, launches=16)
        roofline["plain_read"] = {"bytes": read_bytes, "us": round(read_us, 2),
                                  "gb_per_s": round(read_bytes / read_us * 1e-3, 1),
                                  "long_read_bytes": long_bytes, "long_read_gb_per_s": round(long_bytes / long_us * 1e-3, 1)}
    out["roofline"] = roofline
    return out, run, wl, S, rho


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py measures ONE GPU: the decode MoE layer runs whole on a single MI355X "
              "(no sharding, no collectives); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_07616_amd import binding as B, workloads as wk
    if not torch.cuda.is_available():
        print("bench.py needs the MI355X (no CPU fallback exists)", file=sys.stderr)
        sys.exit(2)
    B.load()

    name = args.workload or HEADLINE
    only_headline = args.only_headline or args.workload is not None or args.only_sere
    head, run, wl, S, rho = measure_config(args, name, args.S, args.rho, args.steps, args.warmup, True)
    if args.only_sere:
        if args.copy_calibration:
            src = torch.ones(128 << 20, dtype=torch.bfloat16, device="cuda")   # 256 MiB
            dst = torch.empty_like(src)
            for _ in range(4):
                dst.copy_(src)
            torch.cuda.synchronize()
        print(json.dumps(head))
        return
    spec = wl.spec
    sere, base = head["sere"], head["no_reroute"]
    sim_host = run.sim.cpu().numpy()
    result = {
        "metric": "us per MoE-layer decode step (SERE) + achieved HBM GB/s, SERE vs no-reroute",
        "value": sere["us_per_step"], "unit": "us/step", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(sere["us_per_step"] * 1e-3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic",
        "config": {"workload": spec.name, "tokens": spec.tokens, "hidden": spec.hidden,
                   "experts": spec.experts, "top_k": spec.top_k, "inter": spec.inter,
                   "shared": spec.shared, "select_top_k": S, "threshold": rho,
                   "weight_copies": head["weight_copies"], "launch": sere["launch"],
                   "similarity": "Frobenius estimate on the GPU (sere_similarity) from seeded calibration tokens"},
        "sere": sere, "no_reroute": base,
        "speedup_vs_no_reroute": head["speedup_vs_no_reroute"],
        "expert_gb_per_s": sere["expert_gb_per_s"], "frac_of_hbm_peak": sere["frac_of_hbm_peak"],
        "target": sere["target"],
        "grid": head["grid"],
        "route_only_us": head["route_only_us"],
        "reroute_only_us": head["reroute_only_us"],
        "sere_hot_weights_us": head["sere_hot_weights_us"],
        "similarity_setup": head["similarity_setup"],
        "roofline": head["roofline"],
        "paper_context": "paper: up to 2.0x whole-model decode speedup on NVIDIA H20 under vLLM; "
                         "MoE MLP 227 us and re-routing kernel 6 us per layer-step at batch 32 on H20 "
                         "(not this machine, not the target)",
    }
    if args.rho_sweep:
        def quick(rho_):
            run.set_knobs(1, rho_)
            nb, na = run.active("sere")
            us, _, _, _ = run.time("sere", 100, 10)
            return {"us_per_step": round(us, 2), "active_before": nb, "active_after": na}
        result["rho_sweep"] = {f"{r:.1f}": quick(r) for r in [i / 10 for i in range(11)]}
    if args.layers > 0:
        result["stack"] = stack(args, run, S, rho)
    del run
    torch.cuda.empty_cache()

    if not only_headline:
        configs = {}
        for other in ALL_WORKLOADS:
            if other == name:
                configs[other] = {k: v for k, v in head.items()}
                continue
            cfg, r2, _, _, _ = measure_config(args, other, 0, 0.0, args.steps, args.warmup, False)
            configs[other] = cfg
            del r2
            torch.cuda.empty_cache()
        result["configs"] = configs
    if args.sweep:
        result["sweep"] = sweep(args)
    if args.prefill:
        batches = tuple(int(b) for b in args.batches.split(",")) if args.batches else (512, 1024, 2048)
        result["prefill_sized"] = sweep(args, batches)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(wl, sim_host, S, rho, args.cpu_seconds)
    print(json.dumps(result))


def stack(args, run, S, rho):
    """L chained layers (layer l reads what layer l-1 wrote; the residual is added by the combine
    step), one HIP graph per pass.  Every layer has its own weights (independent seeds) and its own
    similarity matrix, estimated on the GPU from that layer's weights (Sec. 3.1.1 defines one
    matrix per layer).  Per-layer active counts."""
    import torch
    from paper_2602_07616_amd import device, workloads as wk
    specs = wk.stack_specs(run.wl.spec, args.layers)
    wls = [wk.make_workload(sp) for sp in specs]
    sims = [device.similarity_on_device(w) for w in wls]
    stk = device.DecodeStack(wls, sims, S, rho)
    del wls
    out = {}
    stream = run.stream
    for label, reroute in (("sere", True), ("no_reroute", False)):
        with torch.cuda.stream(stream):
            stk.run(stream, reroute, True)
            stream.synchronize()
            counts = stk.active_counts()
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                stk.run(stream, reroute, False)
            for _ in range(3):
                graph.replay()
            reps = max(4, args.steps // args.layers)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record(stream)
            for _ in range(reps):
                graph.replay()
            e1.record(stream)
            torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        out[label] = {"us_per_pass": round(us, 2), "us_per_layer": round(us / args.layers, 2),
                      "active_before": [c[0] for c in counts], "active_after": [c[1] for c in counts]}
    out["layers"] = args.layers
    out["weights"] = "independent per layer; one similarity matrix per layer (sere_similarity on that layer's weights)"
    out["speedup_vs_no_reroute"] = round(out["no_reroute"]["us_per_pass"] / out["sere"]["us_per_pass"], 3)
    return out


def sweep(args, batches=None):
    """Batch-size sweep on the Qwen3-shaped layer: active experts and latency."""
    from paper_2602_07616_amd import workloads as wk
    out = {}
    sim = None
    for T in (batches or wk.BATCH_SWEEP):
        wl = wk.make_workload("qwen3_b128", tokens=T)
        run = Runner(wl, sim, 4, not args.no_graph)
        sim = run.sim
        row = {}
        for label, mode, S in (("no_reroute", "baseline", 8), ("S=2", "sere", 2), ("S=1", "sere", 1)):
            run.set_knobs(S, 0.0)
            nb, na = run.active(mode)
            us, _, _, _ = run.time(mode, 200 if T <= 256 else 40, 20 if T <= 256 else 4)
            row[label] = {"us_per_step": round(us, 2), "active": nb if mode == "baseline" else na}
            if T >= 512 and label == "S=2":
                # prefill-sized: the expert FFN against both of its bounds, the matrix cores
                # (6 d_h d_m flop per slot) and the weight stream (every active expert once)
                sp = wl.spec
                st = run.stage_times(mode, 20)
                ffn_us = st["gate_up"] + st["down"]
                flop = 6.0 * sp.hidden * sp.inter * T * sp.top_k
                wbytes = na * sp.expert_bytes
                row["ffn_roofline"] = {
                    "stage_us": {k: round(v, 2) for k, v in st.items() if v},
                    "mfma": {"bound": "mfma", "achieved": round(flop / ffn_us * 1e-6, 1), "peak": 2500.0, "unit": "TFLOP/s",
                             "frac": round(flop / ffn_us * 1e-6 / 2500.0, 4)},
                    "hbm": {"bound": "hbm", "achieved": round(wbytes / ffn_us * 1e-3, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": round(wbytes / ffn_us * 1e-3 / HBM_PEAK_GBS, 4)},
                    "binding": "hbm" if wbytes / HBM_PEAK_GBS * 1e-3 > flop / 2500.0 * 1e-6 else "mfma"}
        out[str(T)] = row
        del run
    return out


if __name__ == "__main__":
    main()
