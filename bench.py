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
# Valid only for the kernel sources they were taken on: the record carries their hash
# and `traffic` is reported as null once the sources differ.
PMC_TRAFFIC = {
    "sources_sha256_16": "3587a7c9a1f4825a",
    "workload": "deepseek",
    "fetch_kib": 33904.92, "fetch_scale": 1.9997,
    "write_kib": 994.33, "write_scale": 1.0,
}
GATE_SOURCES = ("paper_2510_03293_amd/csrc/gate.hip", "paper_2510_03293_amd/csrc/analyse.h")


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
    s = wl.SHAPES[args.workload]
    layers = args.layers or s.layers
    T, H, E, k, c = s.T, s.H, s.E, s.k, s.c
    sz = 2 if s.dtype == wl.DTYPE_BF16 else 4

    # ---- inputs, resident in HBM before anything is timed --------------------
    hidden, wgate, params = [], [], []
    for layer in range(layers):
        inp = wl.layer_inputs(args.workload, layer)
        hidden.append(torch.from_numpy(inp["hidden"].view(np.int16)).view(torch.bfloat16).cuda())
        wgate.append(torch.from_numpy(inp["w_gate"].view(np.int16)).view(torch.bfloat16).cuda())
        eps, tfix = wl.thresholds(args.workload, layer, args.preset)
        params.append(B.make_params(k, c, eps, tfix, dtype=s.dtype))
    loads = torch.zeros((layers, E), dtype=torch.int32, device="cuda")
    buf = B.RouteBuffers(T, H, E, params[0])
    stream = torch.cuda.current_stream()
    loads_of = [loads[layer] for layer in range(layers)]

    def step():
        loads.zero_()
        for layer in range(layers):
            B.laser_route(hidden[layer], wgate[layer], T, H, E, params[layer], loads_of[layer],
                          buf.expert_ids, buf.weights, buf.permutation, buf.expert_offsets, None,
                          buf.workspace, stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    tokens_per_s = T * layers * args.steps / wall

    # ---- the gate kernel alone, HIP events on the launch stream ---------------
    B.laser_profile_enable(layers * args.steps)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    gate_ms, gate_launches = B.laser_profile_read()
    B.laser_profile_enable(0)
    # an event pair adds a fixed cost to whatever it brackets; it is measured on the
    # spot with a kernel of known duration and taken off the per-launch average
    event_overhead_s = B.laser_profile_event_overhead(stream) * 1e-3
    whole_bytes, gate_bytes = algorithmic_bytes(T, H, E, k, sz)
    gate_avg_s = gate_ms * 1e-3 / max(gate_launches, 1) - event_overhead_s
    achieved = gate_bytes / gate_avg_s / 1e9

    if args.copy_probe:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    lo = loads.cpu().numpy().astype(np.float64)
    imbalance = float(np.mean(lo.max(1) / lo.mean(1)))

    # ---- the load-ordered chain at full duty: every token takes the load-aware
    # branch with c candidates (preset "stress"), a few layers, reported separately
    # because it is bound by the dependency through the counters, not by any roofline
    eps_s, tfix_s = wl.thresholds(args.workload, 0, "stress")
    p_stress = B.make_params(k, c, eps_s, tfix_s, dtype=s.dtype)
    n_stress = min(layers, 3)

    def stress_pass():
        loads.zero_()
        for layer in range(n_stress):
            B.laser_route(hidden[layer], wgate[layer], T, H, E, p_stress, loads_of[layer],
                          buf.expert_ids, buf.weights, buf.permutation, buf.expert_offsets, None,
                          buf.workspace, stream)
    stress = None
    if not args.no_chain_stress:
        stress_pass()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        stress_pass()
        torch.cuda.synchronize()
        stress_us = (time.perf_counter() - t0) * 1e6 / n_stress
        lo_s = loads[:n_stress].cpu().numpy().astype(np.float64)
        stress = {"us_per_layer": stress_us, "ns_per_load_dependent_token": stress_us * 1e3 / T,
                  "max_over_mean_load": float(np.mean(lo_s.max(1) / lo_s.mean(1))),
                  "note": "every token load-dependent (eps_high=2, t_fix=1e-30): chain-bound"}

    # ---- context figures (none of them enters `value`) --------------------------
    extras = {}
    if not args.no_context:
        # the box's own ceiling: a plain kernel reads the same number of bytes per launch
        # as the gate kernel reads activations, from one buffer far beyond the cache
        flat = torch.cat([h.view(torch.uint8).reshape(-1) for h in hidden])
        sink = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.laser_profile_plain_read(flat, T * H * sz, sink, stream)
        read_ms, read_n = B.laser_profile_plain_read(flat, T * H * sz, sink, stream)
        read_s = (read_ms * 1e-3 - event_overhead_s) / max(read_n, 1)
        extras["plain_read"] = {"bytes_per_launch": T * H * sz, "us_per_launch": read_s * 1e6,
                                "GBps": T * H * sz / read_s / 1e9, "launches": read_n}
        del flat

        # plain top-k on the same inputs (c = k: every token keeps its k best)
        p_topk = B.make_params(k, k, 0.5, 0.5, dtype=s.dtype)
        loads.zero_()
        for layer in range(layers):
            B.laser_route(hidden[layer], wgate[layer], T, H, E, p_topk, loads_of[layer],
                          buf.expert_ids, buf.weights, buf.permutation, buf.expert_offsets, None,
                          buf.workspace, stream)
        lo_k = loads.cpu().numpy().astype(np.float64)
        extras["max_over_mean_load_topk"] = float(np.mean(lo_k.max(1) / lo_k.mean(1)))
        # the load-only baseline (scores ignored: every token takes the load-aware branch
        # with all experts as candidates) needs c = E, which the kernels carry up to 16
        if E <= 16:
            p_lo = B.make_params(k, E, 2.0, 1e-30, dtype=s.dtype)
            loads.zero_()
            for layer in range(layers):
                B.laser_route(hidden[layer], wgate[layer], T, H, E, p_lo, loads_of[layer],
                              buf.expert_ids, buf.weights, buf.permutation, buf.expert_offsets, None,
                              buf.workspace, stream)
            lo_l = loads.cpu().numpy().astype(np.float64)
            extras["max_over_mean_load_loadonly"] = float(np.mean(lo_l.max(1) / lo_l.mean(1)))

        # the statistics pass (laser_route_stats): cost beside the plain call, and what
        # the synthetic gate scores look like (layer means of per-token values)
        st_mass = torch.empty(T, dtype=torch.float32, device="cuda")
        st_ent = torch.empty(T, dtype=torch.float32, device="cuda")
        st_pool = torch.empty(T, dtype=torch.int32, device="cuda")

        def stats_pass():
            loads.zero_()
            for layer in range(layers):
                B.laser_route_stats(hidden[layer], wgate[layer], T, H, E, params[layer],
                                    loads_of[layer], buf.expert_ids, buf.weights, buf.permutation,
                                    buf.expert_offsets, None, st_mass, st_ent, st_pool,
                                    buf.workspace, stream)
        stats_pass()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        stats_pass()
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
            loads.zero_()
            for layer in range(n_rand):
                B.laser_route(hidden[layer], wgate[layer], T, H, E, p_rand[layer], loads_of[layer],
                              buf.expert_ids, buf.weights, buf.permutation, buf.expert_offsets, None,
                              buf.workspace, stream)
        random_pass()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            random_pass()
        torch.cuda.synchronize()
        extras["random_trim_us_per_layer"] = (time.perf_counter() - t0) * 1e6 / (5 * n_rand)

        # the same figure from the device-side metrics (counts = loads after a step
        # that started from zero loads)
        step()
        im = B.laser_imbalance(loads)
        torch.cuda.synchronize()
        extras["device_I_agg"] = float(im["agg"][0])
        extras["device_max_violation_mean"] = float(im["MV"].mean())

        # run-to-run determinism: one layer twice into separate buffers, every output bit
        buf2 = B.RouteBuffers(T, H, E, params[0])
        l1 = torch.zeros(E, dtype=torch.int32, device="cuda")
        l2 = torch.zeros_like(l1)
        for bb, ll in ((buf, l1), (buf2, l2)):
            B.laser_route(hidden[0], wgate[0], T, H, E, p_stress, ll, bb.expert_ids, bb.weights,
                          bb.permutation, bb.expert_offsets, None, bb.workspace, stream)
        torch.cuda.synchronize()
        extras["bit_identical_rerun"] = bool(
            torch.equal(buf.expert_ids, buf2.expert_ids) and torch.equal(buf.permutation, buf2.permutation)
            and torch.equal(buf.weights.view(torch.int32), buf2.weights.view(torch.int32))
            and torch.equal(buf.expert_offsets, buf2.expert_offsets) and torch.equal(l1, l2))
        del buf2

        # decode-shaped calls (64 tokens per call, loads carried): launch-latency-bound
        sd = wl.SHAPES["decode"]
        wdec = wl.decode_gate_weight()
        wdec_d = torch.from_numpy(wdec.view(np.int16)).view(torch.bfloat16).cuda()
        hdec = [torch.from_numpy(wl.layer_inputs("decode", i, w=wdec)["hidden"].view(np.int16))
                .view(torch.bfloat16).cuda() for i in range(16)]
        eps_d, tfix_d = wl.thresholds("decode", 0, args.preset)
        p_dec = B.make_params(sd.k, sd.c, eps_d, tfix_d, dtype=sd.dtype)
        bufd = B.RouteBuffers(sd.T, sd.H, sd.E, p_dec)
        ld = torch.zeros(sd.E, dtype=torch.int32, device="cuda")

        def decode_steps(n):
            for i in range(n):
                B.laser_route(hdec[i % len(hdec)], wdec_d, sd.T, sd.H, sd.E, p_dec, ld, bufd.expert_ids,
                              bufd.weights, bufd.permutation, bufd.expert_offsets, None,
                              bufd.workspace, stream)
        decode_steps(32)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        decode_steps(512)
        torch.cuda.synchronize()
        extras["decode_us_per_call"] = (time.perf_counter() - t0) * 1e6 / 512
        extras["decode_tokens_per_call"] = sd.T

        # the batched entry point: independent problems in one call.  (a) 16 decode-sized
        # problems; (b) all layers of the timed workload at once -- possible only where
        # their inputs exist together (micro-batches in flight at different layers), so
        # it is context, never the headline
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
        del hb, wb, wsb

        same = all(p_.eps_high == params[0].eps_high and p_.t_fix == params[0].t_fix for p_ in params)
        free_b, _ = torch.cuda.mem_get_info()
        need = layers * (T * H * sz + B.laser_workspace_bytes(T, H, E, params[0]) + T * k * 12)
        if same and need < free_b // 2:
            hall = torch.stack(hidden)
            wall_ = torch.stack(wgate)
            one = B.laser_workspace_bytes(T, H, E, params[0])
            wsa = torch.empty(layers * one, dtype=torch.uint8, device="cuda")
            ida = torch.empty((layers, T, k), dtype=torch.int32, device="cuda")
            wta = torch.empty((layers, T, k), dtype=torch.float32, device="cuda")
            pma = torch.empty((layers, T * k), dtype=torch.int32, device="cuda")
            ofa = torch.empty((layers, E + 1), dtype=torch.int32, device="cuda")
            la = torch.zeros((layers, E), dtype=torch.int32, device="cuda")

            def all_layers(n):
                for _ in range(n):
                    la.zero_()
                    B.laser_route_batched(hall, wall_, layers, T, H, E, params[0], la, ida, wta, pma, ofa,
                                          None, wsa, stream)
            all_layers(2)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            all_layers(10)
            torch.cuda.synchronize()
            extras["batched_all_layers_us_per_layer"] = (time.perf_counter() - t0) * 1e6 / (10 * layers)
            extras["batched_all_layers_equal_sequential"] = bool(torch.equal(la, loads))
            del hall, wall_, wsa

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
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": measured_traffic_bytes(args.workload),
            "kernel": "gate_analyse_bf16_kernel", "avg_launch_us": gate_avg_s * 1e6,
            "algorithmic_bytes_per_launch": gate_bytes,
            "event_pair_overhead_us": event_overhead_s * 1e6,
            "other_kernels_us_per_layer": ms_per_step * 1e3 / layers - gate_avg_s * 1e6,
        },
        "whole_path": {
            "us_per_layer": ms_per_step * 1e3 / layers,
            "algorithmic_bytes_per_layer": whole_bytes,
            "hbm_frac": whole_bytes / (ms_per_step * 1e-3 / layers) / 1e9 / HBM_PEAK_GBS,
        },
        "max_over_mean_load": imbalance,
        "chain_stress": stress,
        "context": extras,
    }
    if not args.no_cpu_baseline:
        base, expanded, flexible = cpu_baseline(args.workload, args.preset, args.cpu_seconds)
        out["cpu_baseline"] = base
        out["expanded_fraction_sample"] = expanded
        out["load_dependent_fraction_sample"] = flexible
    print(json.dumps(out))


if __name__ == "__main__":
    main()
