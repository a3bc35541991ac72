#!/usr/bin/env python3
"""Benchmark of the LASER routing step on one MI355X.

A "step" is one pass of the whole routing path (gate projection, per-token
analysis, load-ordered selection, dispatch) over every MoE layer of the workload:
`layers` calls of laser_route on T tokens each, every layer with its own hidden
states and gate matrix resident in HBM (distinct buffers, so that no layer is
served from a cache warmed by the previous step) and its load counters zeroed
at the start of the step.  Prints one JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, vendor figure

# HBM bytes per launch of the gate kernel from rocprofv3 counters (two --pmc runs,
# FETCH_SIZE then WRITE_SIZE, KiB per dispatch, each scaled by what the same counter
# read for a plain 256 MiB device copy in the same run; summary under profiles/).
# A constant taken from those runs, not measured by this program; valid only for the
# kernel sources it was taken on: the record carries their hash and `traffic` is
# reported as null once the sources differ.
PMC_TRAFFIC = {
    "sources_sha256_16": "fe2af7228f7149c9",
    "workload": "deepseek",
    "fetch_kib": 33902.35, "fetch_scale": 1.9997,
    "write_kib": 1024.23, "write_scale": 1.0,
}
GATE_SOURCES = ("paper_2510_03293_amd/csrc/gate.hip", "paper_2510_03293_amd/csrc/gate_tile.h",
                "paper_2510_03293_amd/csrc/analyse.h")


def measured_traffic_bytes(workload):
    import hashlib
    h = hashlib.sha256()
    for rel in GATE_SOURCES:
        with open(os.path.join(ROOT, rel), "rb") as f:
            h.update(f.read())
    if h.hexdigest()[:16] != PMC_TRAFFIC["sources_sha256_16"] or workload != PMC_TRAFFIC["workload"]:
        return None
    return (PMC_TRAFFIC["fetch_kib"] * PMC_TRAFFIC["fetch_scale"] +
            PMC_TRAFFIC["write_kib"] * PMC_TRAFFIC["write_scale"]) * 1024.0


def algorithmic_bytes(T, H, E, k, sz):
    """Bytes the method must move per layer: read hidden and the gate matrix once,
    write ids, weights and permutation, read and write the counters, write offsets."""
    whole = T * H * sz + E * H * sz + T * k * 12 + (E + 1) * 4 + 2 * E * 4
    # the fused gate + per-token analysis kernel: reads both operands once, writes the
    # expert ids and weights of every token whose choice does not depend on loads
    gate = T * H * sz + E * H * sz + T * k * 8
    return whole, gate


def max_over_mean(loads_2d) -> float:
    lo = loads_2d.cpu().numpy().astype(np.float64)
    return float(np.mean(lo.max(1) / lo.mean(1)))


class Workload:
    """One benchmark configuration resident on the GPU: `layers` layers of inputs."""

    def __init__(self, name, preset, layers=0, pipeline_tiles=0):
        import torch
        from paper_2510_03293_amd import binding as B
        from synth import workloads as wl
        self.name, self.preset = name, preset
        s = wl.SHAPES[name]
        self.s = s
        self.layers = layers or s.layers
        self.sz = 2 if s.dtype == wl.DTYPE_BF16 else 4
        self.hidden, self.wgate, self.params, self.host = [], [], [], []
        for layer in range(self.layers):
            inp = wl.layer_inputs(name, layer)
            if layer == 0:
                self.host.append(inp)          # kept for the oracle check of layer 0
            self.hidden.append(torch.from_numpy(inp["hidden"].view(np.int16)).view(torch.bfloat16).cuda())
            self.wgate.append(torch.from_numpy(inp["w_gate"].view(np.int16)).view(torch.bfloat16).cuda())
            eps, tfix = wl.thresholds(name, layer, preset)
            self.params.append(B.make_params(s.k, s.c, eps, tfix, dtype=s.dtype, pipeline_tiles=pipeline_tiles))
        self.loads = torch.zeros((self.layers, s.E), dtype=torch.int32, device="cuda")
        self.loads_of = [self.loads[layer] for layer in range(self.layers)]
        self.buf = B.RouteBuffers(s.T, s.H, s.E, self.params[0])
        self.stream = torch.cuda.current_stream()

    def step(self, params=None, route=None, nlayers=None):
        from paper_2510_03293_amd import binding as B
        s, buf = self.s, self.buf
        route = route or B.laser_route
        self.loads.zero_()
        for layer in range(nlayers or self.layers):
            p = self.params[layer] if params is None else (params[layer] if isinstance(params, list) else params)
            route(self.hidden[layer], self.wgate[layer], s.T, s.H, s.E, p, self.loads_of[layer],
                  buf.expert_ids, buf.weights, buf.permutation, buf.expert_offsets, None,
                  buf.workspace, self.stream)

    def measure(self, steps, warmup, event_overhead_s):
        """Wall clock over `steps` steps (the headline), then the same steps with every
        call's launches bracketed by HIP events: how the time divides between the fused
        projection/analysis kernel and the tail kernel."""
        import torch
        from paper_2510_03293_amd import binding as B
        s = self.s
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        imbalance = max_over_mean(self.loads)
        us_per_layer = wall * 1e6 / (steps * self.layers)

        timer = B.BenchTimer(self.layers * steps)
        for _ in range(steps):
            self.step(route=timer.route)
        torch.cuda.synchronize()
        first_ms, tail_ms = timer.read()
        timer.close()
        ov_us = event_overhead_s * 1e6
        first_us = np.array(first_ms) * 1e3 - ov_us     # an event pair adds a fixed cost to what it brackets
        tail_us = np.array(tail_ms) * 1e3 - ov_us
        # The events give the split; the wall clock gives the total.  The kernel's
        # duration is its share of the wall time per layer, so that the two kernels
        # add up to the path exactly and every gap between launches is charged.
        share = float(first_us.mean() / (first_us.mean() + tail_us.mean()))
        whole_bytes, gate_bytes = algorithmic_bytes(s.T, s.H, s.E, s.k, self.sz)
        return {
            "wall_s": wall, "us_per_layer": us_per_layer, "max_over_mean_load": imbalance,
            "gate_us": us_per_layer * share, "tail_us": us_per_layer * (1.0 - share),
            "gate_us_events": float(first_us.mean()), "tail_us_events": float(tail_us.mean()),
            "median_us_per_layer_events": float(np.median(first_us + tail_us)),
            "timed_calls": int(first_us.size),
            "whole_bytes": whole_bytes, "gate_bytes": gate_bytes,
            "hbm_frac": whole_bytes / (us_per_layer * 1e-6) / 1e9 / HBM_PEAK_GBS,
            "gate_hbm_frac": gate_bytes / (us_per_layer * share * 1e-6) / 1e9 / HBM_PEAK_GBS,
        }

    def topk_imbalance(self):
        """Plain top-k on the same inputs (c = k: every token keeps its k best)."""
        import torch
        from paper_2510_03293_amd import binding as B
        s = self.s
        self.step(params=B.make_params(s.k, s.k, 0.5, 0.5, dtype=s.dtype))
        torch.cuda.synchronize()
        return max_over_mean(self.loads)

    def load_only_imbalance(self, nlayers):
        """The load-only baseline (scores ignored: every token takes the load-aware branch
        with all E experts as candidates), a few layers: the floor of the metric."""
        import torch
        from paper_2510_03293_amd import binding as B
        s = self.s
        p = B.make_params(s.k, s.E, 2.0, 1e-30, dtype=s.dtype)
        wide = B.RouteBuffers(s.T, s.H, s.E, p)
        keep, self.buf = self.buf, wide
        try:
            self.step(params=p, nlayers=nlayers)
            torch.cuda.synchronize()
            assert B.laser_status(wide.workspace) == B.STATUS_COMPLETE
            return max_over_mean(self.loads[:nlayers])
        finally:
            self.buf = keep

    def check_layer0(self):
        """The timed call (no logits buffer) on layer 0 against the same call with a logits
        buffer, bit for bit, and that one against the CPU oracle fed with the GPU's
        logits.  Raises if anything differs."""
        import torch
        import oracle
        from paper_2510_03293_amd import binding as B
        s, inp = self.s, self.host[0]
        outs = []
        for want_logits in (False, True):
            loads = torch.zeros(s.E, dtype=torch.int32, device="cuda")
            buf = B.route(self.hidden[0], self.wgate[0], self.params[0], loads, want_logits=want_logits)
            torch.cuda.synchronize()
            assert B.laser_status(buf.workspace) == B.STATUS_COMPLETE
            outs.append((buf, loads))
        (b0, l0), (b1, l1) = outs
        for name in ("expert_ids", "permutation", "expert_offsets"):
            assert torch.equal(getattr(b0, name), getattr(b1, name)), f"no-logits call differs: {name}"
        assert torch.equal(b0.weights.view(torch.int32), b1.weights.view(torch.int32)), "no-logits call differs: weights"
        assert torch.equal(l0, l1), "no-logits call differs: loads"
        z = b1.logits.cpu().numpy()
        p = self.params[0]
        ref = oracle.route(z, s.k, s.c, p.eps_high, p.t_fix, inp["loads_in"])
        assert np.array_equal(b1.expert_ids.cpu().numpy(), ref["expert_ids"]), "expert_ids differ from the oracle"
        assert np.array_equal(b1.permutation.cpu().numpy(), ref["permutation"]), "permutation differs from the oracle"
        assert np.array_equal(b1.expert_offsets.cpu().numpy(), ref["expert_offsets"]), "offsets differ from the oracle"
        assert np.array_equal(l1.cpu().numpy(), ref["loads"]), "loads differ from the oracle"
        assert np.abs(b1.weights.cpu().numpy() - ref["weights"]).max() <= 2e-3, "weights off"
        rows = np.arange(0, s.T, max(1, s.T // 256))
        zz = oracle.gate(inp["hidden"][rows], inp["w_gate"], s.dtype)
        assert np.abs(z[rows] - zz).max() <= 2e-3, "logits off"
        return {"expanded_fraction": float(ref["expanded"].mean()),
                "load_dependent_fraction": float((ref["cstar"] > s.k).mean())}


def cpu_baseline(name, preset, budget_s):
    """The oracle as it stands, single thread, on a bounded sample of the workload:
    whole layers (gate + routing + dispatch) until about `budget_s` seconds are spent."""
    import oracle
    from synth import workloads as wl
    s = wl.SHAPES[name]
    spent, spent_route, tokens, layers_done = 0.0, 0.0, 0, 0
    expanded, flexible = [], []
    for layer in range(s.layers):
        inp = wl.layer_inputs(name, layer)
        eps, tfix = wl.thresholds(name, layer, preset)
        t0 = time.perf_counter()
        z = oracle.gate(inp["hidden"], inp["w_gate"], s.dtype).astype(np.float32)
        t1 = time.perf_counter()
        out = oracle.route(z, s.k, s.c, eps, tfix, inp["loads_in"])
        t2 = time.perf_counter()
        spent += t2 - t0
        spent_route += t2 - t1
        tokens += s.T
        layers_done += 1
        expanded.append(float(out["expanded"].mean()))
        flexible.append(float((out["cstar"] > s.k).mean()))
        if spent >= budget_s:
            break
    cpu_model = ""
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    cpu_model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return {
        "value": tokens / spent, "unit": "tokens/s", "cores": 1, "kind": "oracle",
        "sample": f"layers 0..{layers_done - 1} of the {name} workload ({tokens} tokens), gate + "
                  f"routing + dispatch, {spent:.1f} s on one host core",
        "routing_and_dispatch_only_tokens_per_s": tokens / spent_route,
        "host": {"cpu": cpu_model, "logical_cpus": os.cpu_count()},
    }, float(np.mean(expanded)), float(np.mean(flexible))


def side_workload(name, preset, layers, steps, event_overhead_s, check):
    """A second configuration, fewer layers and steps: where the time goes when a
    material share of the tokens is load-dependent."""
    import torch
    w = Workload(name, preset, layers)
    m = w.measure(steps, 2, event_overhead_s)
    out = {
        "workload": f"{name}-shaped gate: T={w.s.T} H={w.s.H} E={w.s.E} k={w.s.k} c={w.s.c}, {w.layers} layers, "
                    f"preset '{preset}'",
        "us_per_layer": m["us_per_layer"], "gate_us": m["gate_us"], "tail_us": m["tail_us"],
        "hbm_frac": m["hbm_frac"], "gate_hbm_frac": m["gate_hbm_frac"],
        "tokens_per_s": w.s.T / (m["us_per_layer"] * 1e-6),
        "max_over_mean_load": m["max_over_mean_load"],
        "max_over_mean_load_topk": w.topk_imbalance(),
        "max_over_mean_load_loadonly": w.load_only_imbalance(min(w.layers, 1)),
    }
    # Batches of 96 K tokens and more are pipelined (the walk over a segment's
    # load-dependent tokens runs inside the projection kernel while later segments
    # stream): the same call with the pipeline switched off, for comparison.
    from paper_2510_03293_amd import binding as B
    from synth import workloads as wl
    out["pipelined"] = bool(w.s.T >= 97920)   # (six rounds of 255 tiles of 64 tokens)
    if out["pipelined"]:
        off = [B.make_params(w.s.k, w.s.c, *wl.thresholds(name, layer, preset), dtype=w.s.dtype,
                             pipeline_tiles=1) for layer in range(w.layers)]
        w.step(params=off)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            w.step(params=off)
        torch.cuda.synchronize()
        out["us_per_layer_not_pipelined"] = (time.perf_counter() - t0) * 1e6 / (steps * w.layers)
        # (the buffers hold the last layer's outputs: the same from both kinds of call)
        one_piece = [t.clone() for t in (w.buf.expert_ids, w.buf.permutation, w.buf.expert_offsets, w.loads,
                                         w.buf.weights.view(torch.int32))]
        w.step()
        torch.cuda.synchronize()
        pipelined = (w.buf.expert_ids, w.buf.permutation, w.buf.expert_offsets, w.loads,
                     w.buf.weights.view(torch.int32))
        if not all(torch.equal(x, y) for x, y in zip(one_piece, pipelined)):
            raise SystemExit(f"{name}: the pipelined call differs from the call in one piece")
        out["pipelined_equals_not_pipelined"] = True
    if check:
        out.update(w.check_layer0())
        out["parity_checked"] = True
    del w
    torch.cuda.empty_cache()
    return out


def decode_figures(preset, extras):
    """Decode-shaped calls (64 tokens per call, loads carried over 512 steps): eager
    calls, the same 512 steps replayed from one HIP graph, and 16 problems per call."""
    import torch
    from paper_2510_03293_amd import binding as B
    from synth import workloads as wl
    sd = wl.SHAPES["decode"]
    stream = torch.cuda.current_stream()
    wdec = wl.decode_gate_weight()
    wdec_d = torch.from_numpy(wdec.view(np.int16)).view(torch.bfloat16).cuda()
    hdec = [torch.from_numpy(wl.layer_inputs("decode", i, w=wdec)["hidden"].view(np.int16))
            .view(torch.bfloat16).cuda() for i in range(16)]
    eps_d, tfix_d = wl.thresholds("decode", 0, preset)
    p_dec = B.make_params(sd.k, sd.c, eps_d, tfix_d, dtype=sd.dtype)
    bufd = B.RouteBuffers(sd.T, sd.H, sd.E, p_dec)
    ld = torch.zeros(sd.E, dtype=torch.int32, device="cuda")

    def decode_steps(n, s=None):
        for i in range(n):
            B.laser_route(hdec[i % len(hdec)], wdec_d, sd.T, sd.H, sd.E, p_dec, ld, bufd.expert_ids,
                          bufd.weights, bufd.permutation, bufd.expert_offsets, None,
                          bufd.workspace, s)
    decode_steps(32, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    decode_steps(sd.layers, stream)
    torch.cuda.synchronize()
    extras["decode_us_per_call"] = (time.perf_counter() - t0) * 1e6 / sd.layers
    extras["decode_tokens_per_call"] = sd.T

    # the 512 steps as one HIP graph (a call only enqueues kernels, so it can be captured)
    ld.zero_()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        decode_steps(sd.layers)          # (on the capture stream: torch's current stream)
    ld.zero_()
    g.replay()
    torch.cuda.synchronize()
    after_one = ld.clone()
    reps = 5
    t0 = time.perf_counter()
    for _ in range(reps):
        g.replay()
    torch.cuda.synchronize()
    extras["decode_us_per_step_graph"] = (time.perf_counter() - t0) * 1e6 / (reps * sd.layers)
    ld.zero_()
    decode_steps(sd.layers, stream)
    torch.cuda.synchronize()
    extras["decode_graph_equals_eager"] = bool(torch.equal(ld, after_one))
    del g

    nbd = len(hdec)
    hb = torch.stack(hdec)
    wb = wdec_d.unsqueeze(0).repeat(nbd, 1, 1).contiguous()
    lb = torch.zeros((nbd, sd.E), dtype=torch.int32, device="cuda")
    one = B.laser_workspace_bytes(sd.T, sd.H, sd.E, p_dec)
    wsb = torch.empty(nbd * one, dtype=torch.uint8, device="cuda")
    idb = torch.empty((nbd, sd.T, sd.k), dtype=torch.int32, device="cuda")
    wtb = torch.empty((nbd, sd.T, sd.k), dtype=torch.float32, device="cuda")
    pmb = torch.empty((nbd, sd.T * sd.k), dtype=torch.int32, device="cuda")
    ofb = torch.empty((nbd, sd.E + 1), dtype=torch.int32, device="cuda")

    def decode_batched(n):
        for _ in range(n):
            B.laser_route_batched(hb, wb, nbd, sd.T, sd.H, sd.E, p_dec, lb, idb, wtb, pmb, ofb, None,
                                  wsb, stream)
    decode_batched(8)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    decode_batched(64)
    torch.cuda.synchronize()
    extras["batched_decode_us_per_problem"] = (time.perf_counter() - t0) * 1e6 / (64 * nbd)
    extras["batched_decode_problems_per_call"] = nbd


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="deepseek", choices=["deepseek", "mixtral", "prefill"])
    ap.add_argument("--preset", default="paper", choices=["paper", "gsm8k", "stress", "topk"])
    ap.add_argument("--layers", type=int, default=0, help="override the layer count (0 = workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--no-chain-stress", action="store_true",
                    help="skip the extra full-duty chain measurement (keeps kernel traces to the timed workload)")
    ap.add_argument("--no-context", action="store_true",
                    help="skip the context figures (plain read, top-k, rerun, decode calls)")
    ap.add_argument("--no-side-workloads", action="store_true",
                    help="skip the Mixtral- and prefill-shaped side measurements")
    ap.add_argument("--no-pipeline", action="store_true",
                    help="route large batches in one piece (laser_params_t.pipeline_tiles = 1)")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one plain 256 MiB device copy (reference for HBM byte counters)")
    args = ap.parse_args()

    if args.gpus != 1:
        print("bench.py: the library runs on one GPU; --gpus above 1 is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_03293_amd import binding as B
    from synth import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    # ---- inputs, resident in HBM before anything is timed --------------------
    w = Workload(args.workload, args.preset, args.layers, pipeline_tiles=1 if args.no_pipeline else 0)
    s, layers = w.s, w.layers
    T, H, E, k, c = s.T, s.H, s.E, s.k, s.c
    event_overhead_s = B.laser_bench_event_overhead(stream) * 1e-3
    m = w.measure(args.steps, args.warmup, event_overhead_s)
    ms_per_step = m["wall_s"] * 1e3 / args.steps
    tokens_per_s = T * layers * args.steps / m["wall_s"]

    # the timed call's outputs, checked (a mismatch fails the run)
    parity = w.check_layer0()

    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    # ---- the load-ordered chain at full duty: every token takes the load-aware
    # branch with c candidates (preset "stress"), a few layers, reported separately
    # because it is bound by the dependency through the counters, not by any roofline
    eps_s, tfix_s = wl.thresholds(args.workload, 0, "stress")
    p_stress = B.make_params(k, c, eps_s, tfix_s, dtype=s.dtype)
    n_stress = min(layers, 3)
    stress = None
    if not args.no_chain_stress:
        w.step(params=p_stress, nlayers=n_stress)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        w.step(params=p_stress, nlayers=n_stress)
        torch.cuda.synchronize()
        stress_us = (time.perf_counter() - t0) * 1e6 / n_stress
        stress = {"us_per_layer": stress_us, "ns_per_load_dependent_token": stress_us * 1e3 / T,
                  "max_over_mean_load": max_over_mean(w.loads[:n_stress]),
                  "note": "every token load-dependent (eps_high=2, t_fix=1e-30): chain-bound"}

    # ---- context figures (none of them enters `value`) --------------------------
    extras = {}
    if not args.no_context:
        # the box's own ceiling: a plain kernel reads the same number of bytes per launch
        # as the gate kernel reads activations, from one buffer far beyond the cache
        flat = torch.cat([h.view(torch.uint8).reshape(-1) for h in w.hidden])
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.laser_bench_plain_read(flat, T * H * w.sz, sink, stream)
        read_ms, read_n = B.laser_bench_plain_read(flat, T * H * w.sz, sink, stream)
        read_s = (read_ms * 1e-3 - event_overhead_s) / max(read_n, 1)
        extras["plain_read"] = {"bytes_per_launch": T * H * w.sz, "us_per_launch": read_s * 1e6,
                                "GBps": T * H * w.sz / read_s / 1e9, "launches": read_n,
                                "frac_of_peak": T * H * w.sz / read_s / 1e9 / HBM_PEAK_GBS}
        del flat

        extras["max_over_mean_load_topk"] = w.topk_imbalance()
        extras["max_over_mean_load_loadonly"] = w.load_only_imbalance(min(layers, 2))

        # the statistics pass (laser_route_stats): cost beside the plain call, and what
        # the synthetic gate scores look like (layer means of per-token values)
        st_mass = torch.empty(T, dtype=torch.float32, device="cuda")
        st_ent = torch.empty(T, dtype=torch.float32, device="cuda")
        st_pool = torch.empty(T, dtype=torch.int32, device="cuda")

        def stats_route(hidden, wgate, T_, H_, E_, p, loads, ids, wts, perm, offs, logits, ws, stream_):
            B.laser_route_stats(hidden, wgate, T_, H_, E_, p, loads, ids, wts, perm, offs, logits,
                                st_mass, st_ent, st_pool, ws, stream_)
        w.step(route=stats_route)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        w.step(route=stats_route)
        torch.cuda.synchronize()
        us_stats = (time.perf_counter() - t0) * 1e6 / layers
        # the layer summaries the thresholds are chosen from, by the library's own kernel
        m_mean, m_q = B.laser_summary_f32(st_mass, [5, 50, 95])
        e_mean, e_q = B.laser_summary_f32(st_ent, [50])
        p_mean, p_q = B.laser_summary_f32(st_pool.float(), [50, 95])
        extras["route_stats"] = {
            "us_per_layer": us_stats,
            "last_layer_mean_topk_mass": float(m_mean),
            "last_layer_topk_mass_p5_p50_p95": [float(v) for v in m_q.cpu()],
            "last_layer_mean_entropy_nats": float(e_mean),
            "last_layer_median_entropy_nats": float(e_q[0]),
            "last_layer_mean_pool_size": float(p_mean),
            "last_layer_pool_size_p50_p95": [float(v) for v in p_q.cpu()],
        }

        # trimming mode RANDOM on the same inputs (the deterministic analysis with pool
        # sizes, then the tokens whose pool exceeds c are drawn again)
        n_rand = min(layers, 3)
        p_rand = []
        for layer in range(n_rand):
            eps_r, tfix_r = wl.thresholds(args.workload, layer, args.preset)
            p_rand.append(B.make_params(k, c, eps_r, tfix_r, dtype=s.dtype, trim_mode=B.TRIM_RANDOM,
                                        seed=20251003, stream=layer))

        def random_pass():
            w.loads.zero_()
            for layer in range(n_rand):
                B.laser_route(w.hidden[layer], w.wgate[layer], T, H, E, p_rand[layer], w.loads_of[layer],
                              w.buf.expert_ids, w.buf.weights, w.buf.permutation, w.buf.expert_offsets, None,
                              w.buf.workspace, stream)
        random_pass()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            random_pass()
        torch.cuda.synchronize()
        extras["random_trim_us_per_layer"] = (time.perf_counter() - t0) * 1e6 / (5 * n_rand)

        # the same figure from the device-side metrics (counts = loads after a step
        # that started from zero loads)
        w.step()
        im = B.laser_imbalance(w.loads)
        torch.cuda.synchronize()
        extras["device_I_agg"] = float(im["agg"][0])
        extras["device_max_violation_mean"] = float(im["MV"].mean())
        loads_seq = w.loads.clone()

        # run-to-run determinism: one layer twice into separate buffers, every output bit
        buf2 = B.RouteBuffers(T, H, E, w.params[0])
        l1 = torch.zeros(E, dtype=torch.int32, device="cuda")
        l2 = torch.zeros_like(l1)
        for bb, ll in ((w.buf, l1), (buf2, l2)):
            B.laser_route(w.hidden[0], w.wgate[0], T, H, E, p_stress, ll, bb.expert_ids, bb.weights,
                          bb.permutation, bb.expert_offsets, None, bb.workspace, stream)
        torch.cuda.synchronize()
        extras["bit_identical_rerun"] = bool(
            torch.equal(w.buf.expert_ids, buf2.expert_ids) and torch.equal(w.buf.permutation, buf2.permutation)
            and torch.equal(w.buf.weights.view(torch.int32), buf2.weights.view(torch.int32))
            and torch.equal(w.buf.expert_offsets, buf2.expert_offsets) and torch.equal(l1, l2))
        del buf2

        decode_figures(args.preset, extras)

        # what a call costs as the batch shrinks: the first rows of the same layers
        # (a prefix of a row-major [T, H] buffer is itself one), each with its own gate
        by_tokens = {}
        lsm = torch.zeros(E, dtype=torch.int32, device="cuda")
        for Ts in (64, 256, 1024, 4096, 8192):
            if Ts >= T:
                continue
            bs = B.RouteBuffers(Ts, H, E, w.params[0])   # (a workspace of the call's own size)

            def small_calls(n):
                for i in range(n):
                    layer = i % layers
                    B.laser_route(w.hidden[layer], w.wgate[layer], Ts, H, E, w.params[layer], lsm,
                                  bs.expert_ids, bs.weights, bs.permutation, bs.expert_offsets,
                                  None, bs.workspace, stream)
            lsm.zero_()
            small_calls(20)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            small_calls(200)
            torch.cuda.synchronize()
            by_tokens[str(Ts)] = (time.perf_counter() - t0) * 1e6 / 200
        extras["us_per_call_by_tokens"] = by_tokens

        # all layers of the timed workload in one batched call -- possible only where
        # their inputs exist together (micro-batches in flight at different layers), so
        # it is context, never the headline
        same = all(p_.eps_high == w.params[0].eps_high and p_.t_fix == w.params[0].t_fix for p_ in w.params)
        free_b, _ = torch.cuda.mem_get_info()
        need = layers * (T * H * w.sz + B.laser_workspace_bytes(T, H, E, w.params[0]) + T * k * 12)
        if same and need < free_b // 2:
            hall = torch.stack(w.hidden)
            wall_ = torch.stack(w.wgate)
            one = B.laser_workspace_bytes(T, H, E, w.params[0])
            wsa = torch.empty(layers * one, dtype=torch.uint8, device="cuda")
            ida = torch.empty((layers, T, k), dtype=torch.int32, device="cuda")
            wta = torch.empty((layers, T, k), dtype=torch.float32, device="cuda")
            pma = torch.empty((layers, T * k), dtype=torch.int32, device="cuda")
            ofa = torch.empty((layers, E + 1), dtype=torch.int32, device="cuda")
            la = torch.zeros((layers, E), dtype=torch.int32, device="cuda")

            def all_layers(n):
                for _ in range(n):
                    la.zero_()
                    B.laser_route_batched(hall, wall_, layers, T, H, E, w.params[0], la, ida, wta, pma, ofa,
                                          None, wsa, stream)
            all_layers(2)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            all_layers(10)
            torch.cuda.synchronize()
            extras["batched_all_layers_us_per_layer"] = (time.perf_counter() - t0) * 1e6 / (10 * layers)
            extras["batched_all_layers_equal_sequential"] = bool(torch.equal(la, loads_seq))
            del hall, wall_, wsa

    gate_bytes, whole_bytes = m["gate_bytes"], m["whole_bytes"]
    traffic = measured_traffic_bytes(args.workload)
    out = {
        "metric": "routed tokens/sec + % HBM roofline (fused gate+route+dispatch); max/mean load",
        "value": tokens_per_s, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {
            "workload": f"{args.workload}-shaped gate: T={T} H={H} E={E} k={k} c={c}, "
                        f"{layers} layers per step, thresholds preset '{args.preset}'",
            "tokens_per_layer": T, "layers": layers, "preset": args.preset,
        },
        # the dominant kernel (fused projection + per-token analysis)
        "roofline": {
            "bound": "hbm", "achieved": gate_bytes / (m["gate_us"] * 1e-6) / 1e9, "peak": HBM_PEAK_GBS,
            "unit": "GB/s", "frac": m["gate_hbm_frac"], "traffic": traffic,
            "traffic_source": ("constant from the rocprofv3 --pmc summary under profiles/ (not measured by "
                               "this run); null when the kernel sources have changed since"),
            "kernel": "gate_analyse_bf16_kernel", "avg_launch_us": m["gate_us"],
            "avg_launch_us_how": "share of the wall time per layer, split by HIP events around the launches",
            "avg_launch_us_events": m["gate_us_events"],
            "algorithmic_bytes_per_launch": gate_bytes,
            "event_pair_overhead_us": event_overhead_s * 1e6,
            "tail_kernel_us": m["tail_us"],
            "whole_path_frac": m["hbm_frac"],
            "target_frac": 0.60,
        },
        "whole_path": {
            "us_per_layer": m["us_per_layer"],
            "median_us_per_layer_events": m["median_us_per_layer_events"],
            "timed_calls_for_median": m["timed_calls"],
            "algorithmic_bytes_per_layer": whole_bytes,
            "hbm_frac": m["hbm_frac"],
        },
        "parity_checked": True,
        "expanded_fraction_layer0": parity["expanded_fraction"],
        "load_dependent_fraction_layer0": parity["load_dependent_fraction"],
        "max_over_mean_load": m["max_over_mean_load"],
        "chain_stress": stress,
        "context": extras,
    }
    if "plain_read" in extras:
        pr = extras["plain_read"]["us_per_launch"]
        out["roofline"]["frac_of_plain_read"] = pr / m["gate_us"]
        out["whole_path"]["frac_of_plain_read"] = pr / m["us_per_layer"]

    # ---- other configurations, where tokens are load-dependent -------------------
    if not args.no_side_workloads:
        del w
        torch.cuda.empty_cache()
        side = {}
        for name, nl, st in (("mixtral", 4, 10), ("prefill", 1, 10)):
            if name != args.workload:
                side[name] = side_workload(name, "paper", nl, st, event_overhead_s, check=True)
        out["workloads"] = side

    if not args.no_cpu_baseline:
        base, expanded, flexible = cpu_baseline(args.workload, args.preset, args.cpu_seconds)
        out["cpu_baseline"] = base
        out["expanded_fraction_sample"] = expanded
        out["load_dependent_fraction_sample"] = flexible
    print(json.dumps(out))


if __name__ == "__main__":
    main()
