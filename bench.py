#!/usr/bin/env python3
"""Benchmark of the decentralized-averaging hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--no-extra]

Headline workload: the largest of the five benchmark configurations, the fifth -- decentralized
momentum SGD in adapt-then-combine form on the static exponential graph, n = 32 agents,
d = 25,557,032 (a ResNet-50's parameter count), X and G stored as bf16, momentum fp32, all resident
in HBM (11.4 GB moved per step, far beyond the 256 MB memory-side cache).  One step = one fused
bf_atc_step: m <- beta m + g, x_i <- sum_j w_ij (x_j - alpha m_j), updating X and M in place.  The
matrices live in the library's column-block layout (include/bf.h, BF_LD_BLOCKED; blocks of
bf_recommended_block columns); the same step on agent-major rows is timed too and reported under
per_config.config5_agent_major_rows.  The
metric is the effective HBM bandwidth: compulsory bytes (every operand element read once, every
result element written once: 2 + 2 + 4 read and 2 + 4 written = 14 bytes per element) divided by
time.  The other four configurations are timed in the same run and reported under "per_config",
each with its own roofline object; rows beyond the five configurations under "next_rows"; the CPU
oracle on a bounded sample of the headline workload under "cpu_baseline" (one thread) and
"cpu_baseline_whole_host" (column chunks over all host cores).  Prints ONE JSON line.
"""

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
MFMA_F32_PEAK_TFLOPS = 157.3


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline legs")
    ap.add_argument("--no-extra", action="store_true", help="time the headline workload only")
    return ap.parse_args()


def load_traffic():
    """HBM bytes per launch from the committed rocprofv3 counter summary (FETCH_SIZE + WRITE_SIZE,
    scaled by the plain-copy calibration), keyed by workload, with the commit they were measured at."""
    out = {}
    path = os.path.join(ROOT, "profiles", "traffic_per_launch.txt")
    if os.path.exists(path):
        for line in open(path):
            if ":" in line and not line.startswith("#"):
                k, v = line.split(":", 1)
                out[k.strip()] = v.strip()
    return out


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.stderr.write("bench.py: this build runs on ONE GPU (all n agents are rows of one matrix in one "
                         "GPU's HBM); there is no multi-GPU path, so --gpus must be 1.\n")
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2111_04287_amd as bf
    import workloads

    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    traffic = load_traffic()

    def timed(step_fn, steps, warmup):
        """Spin-up + W untimed + K timed calls of step_fn(k).  Returns (wall seconds, mean ms per
        launch by HIP events recorded on the launch stream around every call).  The spin-up (about
        a quarter second of the same step, untimed) lets the device leave its idle clocks; without
        it the first milliseconds after an idle period run 3-7 % slower."""
        t_spin = time.perf_counter()
        j = 0
        while time.perf_counter() - t_spin < 0.25:
            for _ in range(10):
                step_fn(j)
                j += 1
            torch.cuda.synchronize()
        for k in range(warmup):
            step_fn(k)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        t0 = time.perf_counter()
        for k in range(steps):
            ev[k].record()
            step_fn(warmup + k)
        ev[steps].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        per_step = sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(steps))
        timed.last = {"launch_ms_median": round(per_step[len(per_step) // 2], 5), "launch_ms_min": round(per_step[0], 5)}
        return wall, sum(per_step) / steps

    def roofline(kernel, bytes_per_launch, ev_ms, key, note=None):
        ach = bytes_per_launch / (ev_ms * 1e-3) / 1e9
        r = {"bound": "hbm", "kernel": kernel, "achieved": round(ach, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
             "frac": round(ach / HBM_PEAK_GBPS, 4),
             "traffic": float(traffic[key]) if key in traffic else None,
             "traffic_measured_at_commit": traffic.get("commit") if key in traffic else None,
             "algorithmic_bytes_per_launch": bytes_per_launch, "launch_ms": round(ev_ms, 5)}
        r.update(timed.last)
        if note:
            r["note"] = note
        return r

    # ------------------------------------------------------------------ headline: configuration 5
    # in the library's column-block layout (blocks of bf_recommended_block columns); the same step on
    # agent-major rows is timed right after it and reported under per_config
    n5, d5 = 32, workloads.RESNET50_PARAMS
    c5 = workloads.CONFIG5
    t5 = bf.bf_topology_create(bf.BF_EXP_STATIC, n5)
    ld5 = bf.bf_recommended_ld(d5, bf.BF_BF16)
    B5 = bf.bf_recommended_block(t5, d5, bf.BF_BF16)
    bytes5 = n5 * d5 * 14

    def blocked(n, d, B, dtype, src=None):
        data = torch.zeros(((d + B - 1) // B, n, B), dtype=dtype, device=dev)
        m = bf.Blocked(data, d)
        if src is not None:
            bf.bf_blocked_pack(src, m)
        return m

    X5 = workloads.alloc_rows(n5, d5, torch.bfloat16, dev, ld=ld5, fill=0)
    C5 = workloads.config5_centres(dev, n=n5, d=d5, ld=ld5)
    E5 = workloads.config5_noise(dev, 0, n=n5, d=d5, ld=ld5)
    G5 = workloads.alloc_rows(n5, d5, torch.bfloat16, dev, ld=ld5)
    M5 = workloads.alloc_rows(n5, d5, torch.float32, dev, ld=ld5, fill=0)
    bf.bf_grad_quadratic(X5, C5, E5, c5["lam"], c5["sigma"], G5)         # gradient generator: outside the timed region
    del C5, E5
    X5b = blocked(n5, d5, B5, torch.bfloat16, X5)                        # same state, converted once
    G5b = blocked(n5, d5, B5, torch.bfloat16, G5)
    M5b = blocked(n5, d5, B5, torch.float32, M5)

    def step5(k):
        bf.bf_atc_step(t5, k, X5b, X5b, G5b, M5b, c5["alpha"], c5["beta"], bf.BF_ATC)

    wall, ev_ms = timed(step5, args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    value = bytes5 * args.steps / wall / 1e9
    out = {
        "metric": "mixing effective HBM GB/s",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16 storage (X, G), fp32 momentum and accumulation",
        "data": "synthetic",
        "config": {"workload": "configs[4] (the largest single-GPU configuration): momentum SGD, adapt-then-combine, static "
                               "exponential graph n=32 (10 nonzeros per row, weights 1/10), d=25,557,032, X and G bf16, "
                               "M fp32, one fused in-place bf_atc_step per step, 14 bytes per element; matrices resident "
                               "in HBM in the library's column-block layout (blocks of %d columns); the same step on "
                               "agent-major rows: per_config.config5_agent_major_rows" % B5,
                   "n": n5, "d": d5, "layout": "column blocks", "block": B5, "topology": "static_exp",
                   "step": "bf_atc_step(momentum, ATC)"},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "agent_row_updates_per_s": round(n5 * args.steps / wall, 1),
        "roofline": roofline("bf_pipe_kernel<bf16, momentum ATC>", bytes5, ev_ms, "config5_momentum_atc_column_blocks"),
    }
    rows5 = None
    mixed5 = None
    mom5 = None
    if not args.no_extra:
        bf.bf_blocked_pack(G5, G5b)        # (unchanged data: a marker between the legs in a kernel trace)
        # state in column blocks, each agent's gradient as it arrives from a per-agent producer: one
        # contiguous vector (agent-major rows)
        w5m, e5m = timed(lambda k: bf.bf_atc_step_layouts(t5, k, X5b, X5b, G5, M5b, c5["alpha"], c5["beta"], bf.BF_ATC),
                         min(args.steps, 100), args.warmup)
        mixed5 = {"ms_per_step": round(w5m * 1e3 / min(args.steps, 100), 5), "steps": min(args.steps, 100), "block": B5, "ld_g": ld5,
                  "effective_GBps": round(bytes5 * min(args.steps, 100) / w5m / 1e9, 1),
                  "pct_of_hbm_peak": round(100 * bytes5 * min(args.steps, 100) / w5m / 1e9 / HBM_PEAK_GBPS, 2),
                  "roofline": roofline("bf_pipe_kernel<bf16, momentum ATC>", bytes5, e5m, "config5_momentum_atc_state_blocks_gradient_rows",
                                       note="bf_atc_step_layouts: X and M in column blocks, G on agent-major rows")}
        bf.bf_blocked_pack(G5, G5b)
        # parameters and gradients as per-agent vectors (agent-major rows), only the momentum, which no
        # one but the library reads, in column blocks
        w5o, e5o = timed(lambda k: bf.bf_atc_step_layouts(t5, k, X5, X5, G5, M5b, c5["alpha"], c5["beta"], bf.BF_ATC),
                         min(args.steps, 100), args.warmup)
        mom5 = {"ms_per_step": round(w5o * 1e3 / min(args.steps, 100), 5), "steps": min(args.steps, 100), "block": B5, "ld": ld5,
                "effective_GBps": round(bytes5 * min(args.steps, 100) / w5o / 1e9, 1),
                "pct_of_hbm_peak": round(100 * bytes5 * min(args.steps, 100) / w5o / 1e9 / HBM_PEAK_GBPS, 2),
                "roofline": roofline("bf_pipe_kernel<bf16, momentum ATC>", bytes5, e5o, "config5_momentum_atc_momentum_blocks",
                                     note="bf_atc_step_layouts: X and G on agent-major rows, M in column blocks")}
        # the agent-major leg goes on from the state the column-block leg reached
        bf.bf_blocked_unpack(X5b, X5)
        bf.bf_blocked_unpack(M5b, M5)
        def step5_rows(k):
            bf.bf_atc_step(t5, k, X5, X5, G5, M5, c5["alpha"], c5["beta"], bf.BF_ATC)

        wall5r, ev5r = timed(step5_rows, min(args.steps, 100), args.warmup)
        rows5 = {"ms_per_step": round(wall5r * 1e3 / min(args.steps, 100), 5), "steps": min(args.steps, 100), "ld": ld5,
                 "effective_GBps": round(bytes5 * min(args.steps, 100) / wall5r / 1e9, 1),
                 "pct_of_hbm_peak": round(100 * bytes5 * min(args.steps, 100) / wall5r / 1e9 / HBM_PEAK_GBPS, 2),
                 "roofline": roofline("bf_pipe_kernel<bf16, momentum ATC>", bytes5, ev5r, "config5_momentum_atc",
                                      note="agent-major rows (row i at i * ld): a column tile is 32 row segments in 32 distant "
                                           "places of each of X, G and M")}
    del X5, G5, M5, X5b, G5b, M5b

    if not args.no_extra:
        per = {"config5_agent_major_rows": rows5, "config5_state_in_column_blocks_gradient_on_agent_major_rows": mixed5,
               "config5_parameters_and_gradient_on_agent_major_rows_momentum_in_column_blocks": mom5}

        def entry(name, kernel, bytes_per_step, n_agents, steps, wall, ev_ms, key, extra=None, note=None):
            e = {"ms_per_step": round(wall * 1e3 / steps, 5), "steps": steps,
                 "effective_GBps": round(bytes_per_step * steps / wall / 1e9, 1),
                 "pct_of_hbm_peak": round(100 * bytes_per_step * steps / wall / 1e9 / HBM_PEAK_GBPS, 2),
                 "agent_row_updates_per_s": round(n_agents * steps / wall, 1),
                 "roofline": roofline(kernel, bytes_per_step, ev_ms, key, note)}
            if extra:
                e.update(extra)
            per[name] = e

        # configuration 2: pure averaging on the static exponential graph, n=64, d=2^20
        n, d = 64, 1 << 20
        topo = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
        ld = bf.bf_recommended_ld(d, bf.BF_F32)
        X = workloads.config2_state(dev, n=n, d=d, ld=ld)
        bytes2 = 2 * n * d * 4
        w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce(topo, k, X, X), args.steps, args.warmup)
        entry("config2_static_exp_n64_d1048576_f32_in_place", "bf_tile_kernel<f32, mix>", bytes2, n, args.steps, w_, e_,
              "config2_in_place",
              note="CACHE ASSISTED: the state (256 MiB) is the size of the 256 MB memory-side cache, and this in-place "
                   "round is left cacheable on purpose; not an HBM figure")
        X2 = [X, workloads.alloc_rows(n, d, torch.float32, dev, ld=ld)]
        w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce(topo, k, X2[k & 1], X2[1 - (k & 1)]), args.steps, args.warmup)
        entry("config2_static_exp_n64_d1048576_f32_out_of_place", "bf_pipe_kernel<f32, mix>", bytes2, n, args.steps, w_, e_,
              "config2_out_of_place", note="separate input and output buffers (512 MiB working set), streaming loads and stores")
        del X2
        B2 = bf.bf_recommended_block(topo, d, bf.BF_F32)
        X2b = [blocked(n, d, B2, torch.float32, X), blocked(n, d, B2, torch.float32)]
        w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce(topo, k, X2b[k & 1], X2b[1 - (k & 1)]), args.steps, args.warmup)
        entry("config2_static_exp_n64_d1048576_f32_out_of_place_column_blocks", "bf_pipe_kernel<f32, mix>", bytes2, n, args.steps,
              w_, e_, "config2_out_of_place_column_blocks", extra={"block": B2},
              note="as above with the matrices in column blocks of %d" % B2)
        del X2b, X

        # practical ceilings: a plain device-to-device copy of 1 GiB, and the library's own 128-bit
        # streaming kernels (best persistent-grid size of a small sweep)
        a = torch.empty(1 << 28, device=dev)
        b = torch.empty_like(a)
        w_, e_ = timed(lambda k: b.copy_(a), 20, 3)
        out["copy_ceiling_GBps"] = round(2 * a.numel() * 4 * 20 / w_ / 1e9, 1)
        ceil = {}
        for mode, name, nbytes in ((0, "copy", 2 * a.numel() * 4), (1, "read_only", a.numel() * 4), (2, "write_only", a.numel() * 4)):
            best = 0.0
            for wgs in (1, 2, 4, 8, 16):
                w_, e_ = timed(lambda k: bf.bf_stream_probe(mode, None if mode == 2 else a, b, wgs), 10, 2)
                best = max(best, nbytes * 10 / w_ / 1e9)
            ceil[name + "_GBps"] = round(best, 1)
        out["stream_ceilings_128bit"] = ceil
        del a, b

        # configuration 3: dynamic one-peer exponential-2, n=256, d=2^22, 8 rounds per sweep
        n3, d3 = 256, 1 << 22
        t3 = bf.bf_topology_create(bf.BF_EXP2_ONE_PEER, n3)
        ld3 = bf.bf_recommended_ld(d3, bf.BF_F32)
        X3 = workloads.config3_state(dev, n=n3, d=d3, ld=ld3)
        w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce(t3, k, X3, X3), 24, 8)
        entry("config3_one_peer_exp2_n256_d4194304_f32", "bf_chain_kernel<f32, mix>", 2 * n3 * d3 * 4, n3, 24, w_, e_, "config3")
        B3 = bf.bf_recommended_block(t3, d3, bf.BF_F32)
        X3b = blocked(n3, d3, B3, torch.float32, X3)
        w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce(t3, k, X3b, X3b), 24, 8)
        entry("config3_one_peer_exp2_n256_d4194304_f32_column_blocks", "bf_chain_kernel<f32, mix>", 2 * n3 * d3 * 4, n3, 24, w_, e_,
              "config3_column_blocks", extra={"block": B3}, note="as above with X in column blocks of %d" % B3)
        del X3b

        # rows beyond the five configurations, part 1 (needs X3): several rounds per pass.  Reported
        # apart from the per-round figures: a fused pass moves each element through HBM once for
        # several rounds, so its GB/s is per PASS (one read + one write of X).
        nxt = {}
        for cnt in (2, 4, 8):
            w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce_multi(t3, (k * cnt) % 8, cnt, X3, X3), 16, 4)
            nxt["fused_rounds_one_peer_n256_d4194304_x%d" % cnt] = {
                "rounds_per_pass": cnt, "ms_per_pass": round(w_ * 1e3 / 16, 4),
                "ms_per_round_equivalent": round(w_ * 1e3 / 16 / cnt, 4),
                "separate_rounds_ms": round(cnt * per["config3_one_peer_exp2_n256_d4194304_f32"]["ms_per_step"], 4),
                "pass_GBps": round(2 * n3 * d3 * 4 * 16 / w_ / 1e9, 1),
                "pass_pct_of_hbm_peak": round(100 * 2 * n3 * d3 * 4 * 16 / w_ / 1e9 / HBM_PEAK_GBPS, 2)}
        X3s = blocked(n3, d3, 64, torch.float32, X3)
        w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce_multi(t3, 0, 8, X3s, X3s), 16, 4)
        nxt["fused_rounds_one_peer_n256_d4194304_x8_column_blocks"] = {
            "rounds_per_pass": 8, "ms_per_pass": round(w_ * 1e3 / 16, 4), "block": 64,
            "pass_GBps": round(2 * n3 * d3 * 4 * 16 / w_ / 1e9, 1),
            "pass_pct_of_hbm_peak": round(100 * 2 * n3 * d3 * 4 * 16 / w_ / 1e9 / HBM_PEAK_GBPS, 2),
            "note": "X in column blocks of 64 (the register-round kernel's tile)"}
        del X3, X3s

        # configuration 4: push-sum on the random directed graph, n=128, d=2^21
        n4, d4 = 128, 1 << 21
        t4 = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n4, out_degree=4, seed=workloads.CONFIG4_GRAPH_SEED)
        ld4 = bf.bf_recommended_ld(d4, bf.BF_F32)
        X4 = workloads.config4_state(dev, n=n4, d=d4, ld=ld4)
        w4 = torch.ones(n4, device=dev)
        w_, e_ = timed(lambda k: bf.bf_pushsum_step(t4, k, X4, X4, w4, w4, None), 50, 5)
        entry("config4_pushsum_random_directed_n128_d2097152_f32", "bf_pushsum_w_kernel + bf_pipe_kernel<f32, mix>",
              2 * n4 * d4 * 4, n4, 50, w_, e_, "config4", note="launch_ms covers both kernels of a step (the n-scalar update and the mix)")
        B4 = bf.bf_recommended_block(t4, d4, bf.BF_F32)
        X4b = blocked(n4, d4, B4, torch.float32, X4)
        w4.fill_(1.0)
        w_, e_ = timed(lambda k: bf.bf_pushsum_step(t4, k, X4b, X4b, w4, w4, None), 50, 5)
        entry("config4_pushsum_random_directed_n128_d2097152_f32_column_blocks", "bf_pushsum_w_kernel + bf_pipe_kernel<f32, mix>",
              2 * n4 * d4 * 4, n4, 50, w_, e_, "config4_column_blocks", extra={"block": B4},
              note="as above with X in column blocks of %d" % B4)
        del X4, X4b

        # configuration 1: decentralized gradient descent on least squares (latency bound)
        d1 = workloads.config1_least_squares(dev)
        A1, b1 = d1["A"], d1["b"]
        n1, m1, dd1 = A1.shape
        t1 = bf.bf_topology_create(bf.BF_RING, n1)
        X1 = [torch.zeros((n1, dd1), device=dev), torch.zeros((n1, dd1), device=dev)]
        G1 = torch.empty((n1, dd1), device=dev)

        def dgd(k):
            bf.bf_grad_least_squares(A1, b1, X1[k & 1], G1)
            bf.bf_atc_step(t1, k, X1[k & 1], X1[1 - (k & 1)], G1, None, d1["alpha"], 0.0, bf.BF_ATC)

        w_, e_ = timed(dgd, 200, 20)
        wg_, eg_ = timed(lambda k: bf.bf_grad_least_squares(A1, b1, X1[0], G1), 200, 20)      # a7 alone
        # the same 200 iterations as 10 replays of a HIP graph holding 20 of them (40 kernel nodes)
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            dgd(0)
            dgd(1)
        torch.cuda.current_stream().wait_stream(side)
        with torch.cuda.graph(graph):
            for k in range(20):
                dgd(k)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(10):
            graph.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter() - tg
        # the same 200 iterations in one launch: A_i resident in LDS, one workgroup per agent, a grid
        # barrier per iteration
        Xp = torch.zeros((n1, dd1), device=dev)
        workp = torch.empty(2 * n1 * dd1, device=dev)
        for _ in range(3):
            bf.bf_dgd_least_squares_run(t1, 0, 200, A1, b1, Xp, workp, d1["alpha"])
        torch.cuda.synchronize()
        tp = time.perf_counter()
        for _ in range(10):
            bf.bf_dgd_least_squares_run(t1, 0, 200, A1, b1, Xp, workp, d1["alpha"])
        gave_up = bf.bf_dgd_status(t1)                  # waits for the stream
        tp = time.perf_counter() - tp
        bytes1 = A1.numel() * 4 + b1.numel() * 4 + 2 * n1 * dd1 * 4
        per["config1_dgd_least_squares_ring_n16_d1024_f32"] = {
            "ms_per_step": round(w_ * 1e3 / 200, 5), "steps": 200,
            "iterations_per_s": round(200 / w_, 1),
            "iterations_per_s_hip_graph": round(200 / tg, 1),
            "iterations_per_s_one_launch": None if gave_up else round(2000 / tp, 1),
            "event_ms_per_iteration": round(e_, 5),
            "ls_gradient_us_per_call": round(eg_ * 1e3, 3),
            "ls_gradient_GBps_of_A": round(A1.numel() * 4 / (eg_ * 1e-3) / 1e9, 1),
            "roofline": {"bound": "latency", "kernel": "bf_ls_grad_kernel + bf_tile_kernel<f32, ATC>", "achieved": round(bytes1 / (e_ * 1e-3) / 1e9, 1),
                         "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(bytes1 / (e_ * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                         "traffic": None, "algorithmic_bytes_per_launch": bytes1, "launch_ms": round(e_, 5),
                         "note": "2.2 MB per iteration, all cache resident: neither HBM nor the matrix cores bound this "
                                 "configuration, launch and synchronisation latency does; the figure of merit is iterations/s"},
            "note": "two launches per iteration on a 64 KiB state; the second figure replays a HIP graph of 20 iterations; "
                    "the third runs 200 iterations per launch with A_i resident in LDS and a grid barrier per iteration "
                    "(bf_dgd_least_squares_run)"}
        del graph

        # dense W on the fp32 matrix cores (a8): fully connected W = 11^T/n
        dn = {}
        for nd in (64, 256):
            dd = 1 << 20
            J = np.full((nd, nd), 1.0 / nd, dtype=np.float32)
            td = bf.bf_topology_create(bf.BF_DENSE_USER, nd, dense_w=J, require_class=bf.BF_W_STANDARD)
            ldd = bf.bf_recommended_ld(dd, bf.BF_F32)
            Xd = [workloads.normal_rows(nd, dd, 701, dev, ld=ldd), workloads.alloc_rows(nd, dd, torch.float32, dev, ld=ldd)]
            w_, e_ = timed(lambda k: bf.bf_dense_mix(td, 0, Xd[k & 1], Xd[1 - (k & 1)]), 40, 5)
            flops = 2.0 * nd * nd * dd
            tf = flops / (e_ * 1e-3) / 1e12
            gb = 2 * nd * dd * 4 / (e_ * 1e-3) / 1e9
            compute_bound = nd >= 128
            dn["dense_w_n%d_d1048576_f32" % nd] = {
                "ms_per_step": round(w_ * 1e3 / 40, 5), "TFLOPs": round(tf, 2), "effective_GBps": round(gb, 1),
                "roofline": ({"bound": "mfma", "kernel": "bf_dense_kernel (v_mfma_f32_32x32x2_f32)", "achieved": round(tf, 2),
                              "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(tf / MFMA_F32_PEAK_TFLOPS, 4),
                              "traffic": None, "launch_ms": round(e_, 5), "flops_per_launch": flops}
                             if compute_bound else
                             {"bound": "hbm", "kernel": "bf_dense_kernel (v_mfma_f32_32x32x2_f32)", "achieved": round(gb, 1),
                              "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gb / HBM_PEAK_GBPS, 4), "traffic": None,
                              "launch_ms": round(e_, 5), "algorithmic_bytes_per_launch": 2 * nd * dd * 4,
                              "note": "n/4 = 16 flop per byte: below the fp32 matrix-core ridge (about 20), HBM bound"})}
            del Xd
        per.update(dn)
        out["per_config"] = per

        # -------------------------------------------------------------- rows beyond the five configurations, part 2
        nh, Lh, dh = 8, 8, 1 << 22
        th = bf.bf_topology_create(bf.BF_EXP_STATIC, nh)
        ldh = bf.bf_recommended_ld(dh, bf.BF_F32)
        Xh2 = workloads.normal_rows(nh * Lh, dh, 601, dev, ld=ldh)
        w_, e_ = timed(lambda k: bf.bf_hierarchical_neighbor_allreduce(th, k, Lh, Xh2, Xh2), 30, 5)
        nxt["hierarchical_8_machines_x_8_agents_d4194304"] = {
            "ms_per_step": round(w_ * 1e3 / 30, 4), "effective_GBps": round(2 * nh * Lh * dh * 4 * 30 / w_ / 1e9, 1),
            "pct_of_hbm_peak": round(100 * 2 * nh * Lh * dh * 4 * 30 / w_ / 1e9 / HBM_PEAK_GBPS, 2),
            "note": "local average, machine-level round, copy back: three fused rounds, one pass over X"}
        Bh = 16384
        Xhb = blocked(nh * Lh, dh, Bh, torch.float32, Xh2)
        w_, e_ = timed(lambda k: bf.bf_hierarchical_neighbor_allreduce(th, k, Lh, Xhb, Xhb), 30, 5)
        nxt["hierarchical_8_machines_x_8_agents_d4194304_column_blocks"] = {
            "ms_per_step": round(w_ * 1e3 / 30, 4), "effective_GBps": round(2 * nh * Lh * dh * 4 * 30 / w_ / 1e9, 1),
            "pct_of_hbm_peak": round(100 * 2 * nh * Lh * dh * 4 * 30 / w_ / 1e9 / HBM_PEAK_GBPS, 2), "block": Bh,
            "note": "the same pass with X in column blocks of %d" % Bh}
        del Xh2, Xhb
        Ew = bf.bf_topology_window_slots(t4, 0)
        Xw = workloads.config4_state(dev, n=n4, d=d4, ld=ld4)
        Ww = workloads.alloc_rows(Ew, d4, torch.float32, dev, ld=ld4, fill=0)
        pw, wpw = torch.ones(n4, device=dev), torch.zeros(Ew, device=dev)

        def async_round(k):
            bf.bf_win_accumulate(t4, 0, Xw, pw, Ww, wpw)
            bf.bf_win_update_then_collect(t4, 0, Xw, pw, Ww, wpw)

        w_, e_ = timed(async_round, 10, 2)
        wbytes = 2 * (2 * n4 + 2 * Ew) * d4 * 4
        nxt["window_pushsum_round_n128_slots%d_d2097152" % Ew] = {
            "ms_per_step": round(w_ * 1e3 / 10, 4), "effective_GBps": round(wbytes * 10 / w_ / 1e9, 1),
            "pct_of_hbm_peak": round(100 * wbytes * 10 / w_ / 1e9 / HBM_PEAK_GBPS, 2),
            "note": "win_accumulate + win_update_then_collect, everybody active; bytes = x read and written "
                    "and every slot read and written, in each of the two calls"}
        del Xw, Ww
        # the fused steps without a state matrix, and a graph with many entries per row: the cases the
        # pipelined kernel runs at the rate of its issued instructions rather than at the HBM rate
        # (column blocks, out of place; bytes = every operand read once, every result written once)
        for tag, nn, dd, dtype, bdt in (("bf16_n32_d25557032", 32, workloads.RESNET50_PARAMS, torch.bfloat16, bf.BF_BF16),
                                         ("f32_n128_d4194304", 128, 1 << 22, torch.float32, bf.BF_F32)):
            tt = bf.bf_topology_create(bf.BF_EXP_STATIC, nn)
            Bt = bf.bf_recommended_block(tt, dd, bdt)
            eb = 2 if dtype == torch.bfloat16 else 4
            Xs, Ys, Gs = (blocked(nn, dd, Bt, dtype) for _ in range(3))
            Xs.data.normal_()
            Gs.data.normal_()
            for what, fn, nb in (("mix", lambda k: bf.bf_neighbor_allreduce(tt, 0, Xs, Ys), 2 * nn * dd * eb),
                                 ("atc", lambda k: bf.bf_atc_step(tt, 0, Xs, Ys, Gs, None, 0.01, 0.0, bf.BF_ATC), 3 * nn * dd * eb),
                                 ("awc", lambda k: bf.bf_atc_step(tt, 0, Xs, Ys, Gs, None, 0.01, 0.0, bf.BF_AWC), 3 * nn * dd * eb)):
                w_, e_ = timed(fn, 30, 5)
                nxt["static_exp_%s_%s_column_blocks" % (tag, what)] = {
                    "ms_per_step": round(e_, 4), "effective_GBps": round(nb / (e_ * 1e-3) / 1e9, 1),
                    "pct_of_hbm_peak": round(100 * nb / (e_ * 1e-3) / 1e9 / HBM_PEAK_GBPS, 2), "block": Bt,
                    "note": "bound by issued vector and scalar instructions, not by HBM"}
            del Xs, Ys, Gs
        out["next_rows"] = nxt

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    if not args.no_cpu:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import iterations as O
        from oracle import topology as OT
        rowptr, col, wgt, _ = bf.bf_topology_export_csr(t5, 0)
        W = OT.from_csr(rowptr, col, wgt)
        a64, b64 = float(np.float32(c5["alpha"])), float(np.float32(c5["beta"]))
        dc = 1 << 19                                   # sample: the first 2^19 columns of every agent
        rng = np.random.default_rng(501)
        Xh = np.zeros((n5, dc))
        Mh = np.zeros((n5, dc))
        Gh = rng.standard_normal((n5, dc))
        steps = 0
        t0 = time.perf_counter()
        while True:
            Xh, Mh = O.dmsgd_atc_step(Xh, Mh, Gh, W, a64, b64)
            steps += 1
            el = time.perf_counter() - t0
            if el > 8.0 or steps >= 50:
                break
        out["cpu_baseline"] = {"value": round(n5 * dc * 14 * steps / el / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                               "sample": "%d fused momentum steps of the headline workload restricted to its first 2^19 columns "
                                         "(n=32; the step is column separable) by the fp64 numpy oracle, %.1f s, one thread; "
                                         "bytes counted as for the GPU (14 per element)" % (steps, el)}
        # the same oracle over disjoint column chunks on all host cores (the path is column separable
        # and numpy releases the GIL inside its array operations)
        threads = max(1, min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)))
        chunk = dc // 4
        nchunks = 4 * threads
        Xs = [np.zeros((n5, chunk)) for _ in range(nchunks)]
        Ms = [np.zeros((n5, chunk)) for _ in range(nchunks)]
        Gs = [rng.standard_normal((n5, chunk)) for _ in range(nchunks)]

        def work(c):
            Xs[c], Ms[c] = O.dmsgd_atc_step(Xs[c], Ms[c], Gs[c], W, a64, b64)

        steps = 0
        with ThreadPoolExecutor(max_workers=threads) as pool:
            t0 = time.perf_counter()
            while True:
                list(pool.map(work, range(nchunks)))
                steps += 1
                el = time.perf_counter() - t0
                if el > 8.0 or steps >= 50:
                    break
        out["cpu_baseline_whole_host"] = {
            "value": round(n5 * chunk * nchunks * 14 * steps / el / 1e9, 3), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "host_logical_cores": os.cpu_count(),
            "sample": "%d steps over %d disjoint column chunks of 2^17 columns (n=32), a pool of %d threads, %.1f s"
                      % (steps, nchunks, threads, el)}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
