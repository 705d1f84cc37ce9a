#!/usr/bin/env python3
"""Benchmark of the decentralized-averaging hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-cpu] [--no-extra]

Headline workload (the second benchmark configuration): pure averaging on the static exponential
graph, n = 64 agents, X 64 x 2^20 fp32 ~ U(-1,1) (seed 201).  One step = one mixing round
X <- W X (bf_neighbor_allreduce, updating the agents' states in place, inputs resident in HBM;
the same round with separate input and output buffers is reported under "per_config").  The metric is the
effective HBM bandwidth: compulsory bytes (every element read once and written once,
2*n*d*4 per round) divided by time.  The other four configurations are timed in the same run and
reported under "per_config"; the CPU oracle is timed on a bounded sample under "cpu_baseline".
Prints ONE JSON line.
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


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-extra", action="store_true", help="time the headline workload only")
    return ap.parse_args()


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

    def mat(n, d, dtype, fill=None):
        ld = bf.bf_recommended_ld(d, bf.BF_F32 if dtype == torch.float32 else bf.BF_BF16)
        return workloads.alloc_rows(n, d, dtype, dev, ld=ld, fill=fill), ld

    def timed(step_fn, steps, warmup, per_launch_events=True):
        """Spin-up + W untimed + K timed calls of step_fn(k).  Returns (wall seconds, mean ms per
        launch by HIP events recorded on the launch stream around every call).  The spin-up (about
        a quarter second of the same step, untimed) lets the device leave its idle clocks; without
        it the first milliseconds after an idle period run 3-7 % slower."""
        t_spin = time.perf_counter()
        j = 0
        while time.perf_counter() - t_spin < 0.25:
            for _ in range(20):
                step_fn(j)
                j += 1
            torch.cuda.synchronize()
        j += j & 1                      # keep the round parity of the timed steps independent of the spin-up
        for k in range(warmup):
            step_fn(k)
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)] if per_launch_events else None
        t0 = time.perf_counter()
        for k in range(steps):
            if ev:
                ev[k].record()
            step_fn(warmup + k)
        if ev:
            ev[steps].record()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        if not ev:
            return wall, None
        per_step = sorted(ev[k].elapsed_time(ev[k + 1]) for k in range(steps))
        timed.last = {"event_ms_median": round(per_step[len(per_step) // 2], 5), "event_ms_min": round(per_step[0], 5)}
        return wall, sum(per_step) / steps

    # ------------------------------------------------------------------ headline: configuration 2
    n, d = 64, 1 << 20
    topo = bf.bf_topology_create(bf.BF_EXP_STATIC, n)
    ld = bf.bf_recommended_ld(d, bf.BF_F32)
    X = workloads.config2_state(dev, n=n, d=d, ld=ld)
    bytes_per_round = 2 * n * d * 4

    def mix_step(k):
        bf.bf_neighbor_allreduce(topo, k, X, X)

    wall, ev_ms = timed(mix_step, args.steps, args.warmup)
    ms_per_step = wall * 1e3 / args.steps
    value = bytes_per_round * args.steps / wall / 1e9
    achieved = bytes_per_round / (ev_ms * 1e-3) / 1e9
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "traffic_mix_static_exp_n64_d1048576.txt")
    if os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = float(line.split(":")[1])
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
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "configs[1]: static exponential graph n=64 (12 nonzeros per row, weights 1/12), "
                               "X 64 x 2^20 fp32 ~U(-1,1) seed 201, one in-place mixing round per step",
                   "n": n, "d": d, "ld": ld, "topology": "static_exp", "step": "bf_neighbor_allreduce"},
        "pct_of_hbm_peak": round(100 * value / HBM_PEAK_GBPS, 2),
        "agent_row_updates_per_s": round(n * args.steps / wall, 1),
        "roofline": {"bound": "hbm", "kernel": "bf_tile_kernel<f32, mix>", "achieved": round(achieved, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "traffic": traffic, "algorithmic_bytes_per_launch": bytes_per_round,
                     "launch_ms": round(ev_ms, 5), "launch_ms_median": timed.last["event_ms_median"],
                     "launch_ms_min": timed.last["event_ms_min"],
                     "note": "X (256 MiB) is the size of the 256 MB memory-side Infinity Cache, which an in-place "
                             "round can partly reuse; configs 3-5 under per_config are 1-4.6 GB and are the "
                             "HBM-only figures"},
    }

    # ------------------------------------------------------------------ the other configurations
    if not args.no_extra:
        per = {}

        def entry(name, bytes_per_step, n_agents, steps, wall, ev_ms, extra=None):
            e = {"ms_per_step": round(wall * 1e3 / steps, 5), "steps": steps,
                 "effective_GBps": round(bytes_per_step * steps / wall / 1e9, 1),
                 "pct_of_hbm_peak": round(100 * bytes_per_step * steps / wall / 1e9 / HBM_PEAK_GBPS, 2),
                 "agent_row_updates_per_s": round(n_agents * steps / wall, 1),
                 "event_ms_per_step": round(ev_ms, 5)}
            e.update(timed.last)
            if extra:
                e.update(extra)
            per[name] = e

        # the headline round with separate input and output buffers (512 MiB working set)
        X2 = [X, workloads.alloc_rows(n, d, torch.float32, dev, ld=ld)]
        w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce(topo, k, X2[k & 1], X2[1 - (k & 1)]), args.steps, args.warmup)
        entry("config2_static_exp_n64_d1048576_f32_out_of_place", bytes_per_round, n, args.steps, w_, e_)
        del X2

        # practical ceiling: a plain device-to-device copy of 1 GiB
        a = torch.empty(1 << 28, device=dev)
        b = torch.empty_like(a)
        w_, e_ = timed(lambda k: b.copy_(a), 20, 3)
        out["copy_ceiling_GBps"] = round(2 * a.numel() * 4 * 20 / w_ / 1e9, 1)
        # the library's own plain 128-bit streaming kernels, best persistent-grid size of a small sweep
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
        entry("config3_one_peer_exp2_n256_d4194304_f32", 2 * n3 * d3 * 4, n3, 24, w_, e_)
        del X3

        # configuration 4: push-sum on the random directed graph, n=128, d=2^21
        n4, d4 = 128, 1 << 21
        t4 = bf.bf_topology_create(bf.BF_RANDOM_DIRECTED, n4, out_degree=4, seed=workloads.CONFIG4_GRAPH_SEED)
        ld4 = bf.bf_recommended_ld(d4, bf.BF_F32)
        X4 = workloads.config4_state(dev, n=n4, d=d4, ld=ld4)
        w4 = torch.ones(n4, device=dev)
        w_, e_ = timed(lambda k: bf.bf_pushsum_step(t4, k, X4, X4, w4, w4, None), 50, 5)
        entry("config4_pushsum_random_directed_n128_d2097152_f32", 2 * n4 * d4 * 4, n4, 50, w_, e_)
        del X4

        # configuration 5: momentum ATC, bf16 X/G, fp32 M, n=32, d=25,557,032 (14 bytes per element)
        n5, d5 = 32, workloads.RESNET50_PARAMS
        c5 = workloads.CONFIG5
        t5 = bf.bf_topology_create(bf.BF_EXP_STATIC, n5)
        ld5 = bf.bf_recommended_ld(d5, bf.BF_BF16)
        X5 = workloads.alloc_rows(n5, d5, torch.bfloat16, dev, ld=ld5, fill=0)
        C5 = workloads.config5_centres(dev, n=n5, d=d5, ld=ld5)
        E5 = workloads.config5_noise(dev, 0, n=n5, d=d5, ld=ld5)
        G5 = workloads.alloc_rows(n5, d5, torch.bfloat16, dev, ld=ld5)
        M5 = workloads.alloc_rows(n5, d5, torch.float32, dev, ld=ld5, fill=0)
        bf.bf_grad_quadratic(X5, C5, E5, c5["lam"], c5["sigma"], G5)         # generator: outside the timed region
        w_, e_ = timed(lambda k: bf.bf_atc_step(t5, k, X5, X5, G5, M5, c5["alpha"], c5["beta"], bf.BF_ATC), 20, 3)
        entry("config5_dmsgd_atc_n32_d25557032_bf16", n5 * d5 * 14, n5, 20, w_, e_,
              {"bytes_per_element": 14, "note": "bf16 X and G, fp32 momentum"})
        del X5, C5, E5, G5, M5

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
        entry("config1_dgd_least_squares_ring_n16_d1024_f32", A1.numel() * 4 + b1.numel() * 4 + 2 * n1 * dd1 * 4,
              n1, 200, w_, e_, {"iterations_per_s": round(200 / w_, 1),
                                "iterations_per_s_hip_graph": round(200 / tg, 1),
                                "iterations_per_s_one_launch": None if gave_up else round(2000 / tp, 1),
                                "note": "latency bound: two launches per iteration on a 64 KiB state; the second "
                                        "figure replays a HIP graph of 20 iterations; the third runs 200 iterations "
                                        "per launch with A_i resident in LDS and a grid barrier per iteration "
                                        "(bf_dgd_least_squares_run)"})
        del graph
        out["per_config"] = per

        # -------------------------------------------------------------- rows beyond the five configurations
        # Reported apart from the per-round figures above: the fused passes move each element through
        # HBM once for several rounds, so their "effective GB/s" is per PASS (one read + one write of X).
        nxt = {}
        X3 = workloads.config3_state(dev, n=n3, d=d3, ld=ld3)
        for cnt in (2, 4, 8):
            w_, e_ = timed(lambda k: bf.bf_neighbor_allreduce_multi(t3, (k * cnt) % 8, cnt, X3, X3), 16, 4)
            nxt["fused_rounds_one_peer_n256_d4194304_x%d" % cnt] = {
                "rounds_per_pass": cnt, "ms_per_pass": round(w_ * 1e3 / 16, 4),
                "ms_per_round_equivalent": round(w_ * 1e3 / 16 / cnt, 4),
                "separate_rounds_ms": round(cnt * per["config3_one_peer_exp2_n256_d4194304_f32"]["ms_per_step"], 4),
                "pass_GBps": round(2 * n3 * d3 * 4 * 16 / w_ / 1e9, 1)}
        del X3
        nh, Lh, dh = 8, 8, 1 << 22
        th = bf.bf_topology_create(bf.BF_EXP_STATIC, nh)
        ldh = bf.bf_recommended_ld(dh, bf.BF_F32)
        Xh2 = workloads.normal_rows(nh * Lh, dh, 601, dev, ld=ldh)
        w_, e_ = timed(lambda k: bf.bf_hierarchical_neighbor_allreduce(th, k, Lh, Xh2, Xh2), 30, 5)
        nxt["hierarchical_8_machines_x_8_agents_d4194304"] = {
            "ms_per_step": round(w_ * 1e3 / 30, 4), "effective_GBps": round(2 * nh * Lh * dh * 4 * 30 / w_ / 1e9, 1),
            "pct_of_hbm_peak": round(100 * 2 * nh * Lh * dh * 4 * 30 / w_ / 1e9 / HBM_PEAK_GBPS, 2),
            "note": "local average, machine-level round, copy back: three fused rounds, one pass over X"}
        del Xh2
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
        out["next_rows"] = nxt
    del X

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    if not args.no_cpu:
        from oracle import iterations as O
        from oracle import topology as OT
        rowptr, col, wgt, _ = bf.bf_topology_export_csr(topo, 0)
        W = OT.from_csr(rowptr, col, wgt)
        rng = np.random.default_rng(201)
        Xh = rng.uniform(-1.0, 1.0, size=(n, d))
        rounds = 0
        t0 = time.perf_counter()
        while True:
            Xh = O.mix(Xh, W)
            rounds += 1
            el = time.perf_counter() - t0
            if el > 10.0 or rounds >= 50:
                break
        out["cpu_baseline"] = {"value": round(bytes_per_round * rounds / el / 1e9, 3), "unit": "GB/s",
                               "cores": 1, "kind": "oracle",
                               "sample": "%d mixing rounds of the full headline workload (n=64, d=2^20) by the fp64 "
                                         "numpy oracle, %.1f s, single thread; host has %d logical cores"
                                         % (rounds, el, os.cpu_count())}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
