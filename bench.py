#!/usr/bin/env python3
"""Benchmark of the replay hot path on one MI355X.

Workload (N=1): the decode-step chain at batch 1 -- 24 layers x 5 sub-blocks of RMSNorm(2048) ->
bf16 GEMV 2048x2048 -> GELU -> residual add, plus 31 input-inject adds: 511 kernels per iteration,
32 fresh bf16[2048] activation inputs per iteration, 1.0066 GB of bf16 weights ~N(0, 0.02^2).

A "step" is one pass of the whole hot path over one batch of inputs: one eager iteration, one
graph-copy replay, one graph-indirect replay and one replay in the selected mode.  Each mode is
timed on its own: W untimed warm-up iterations, then exactly K iterations back to back on one
stream, bracketed by a device synchronisation on both sides (host clock, inputs resident in HBM,
rotating through three input sets at distinct addresses).  `value` is the graph-indirect figure.

One JSON line on stdout; progress on stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-copy-bench", action="store_true", help="skip the copy-kernel bandwidth leg (config 3 sizes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-refresh-baselines", action="store_true",
                    help="skip the legs added beside the three modes (host-side node updates, per-tensor memcpy, the two alternating table "
                         "mechanisms, the dispatch-floor chain, the event-timed medians); the rocprofv3 runs use this: counter-collection runs that included them "
                         "did not complete (one went silent, one ended in a segmentation fault inside a profiler thread)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle timing leg")
    ap.add_argument("--profile-iters", type=int, default=20, help="samples per (segment, mode) of the slow-path profiler")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); run it with --gpus 1", file=sys.stderr)
        return 2

    import torch
    import paper_2503_19779_amd as pg
    from paper_2503_19779_amd.binding import to_device
    from pg_workloads import decode_chain, refresh_stress_chain, make_weights, make_inputs

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)
    K, W = args.steps, args.warmup
    HBM_PEAK = 8000.0   # GB/s, MI355X

    # ------------------------------------------------------------------ workload: decode chain, batch 1
    spec = decode_chain()
    log(f"[bench] {spec.name}: {len(spec.kernels)} kernels; generating {sum(w.nbytes for w in spec.weights) / 1e9:.3f} GB of weights")
    t0 = time.time()
    w_np = make_weights(spec)
    w_dev = [to_device(w, dev) for w in w_np]
    log(f"[bench] weights resident after {time.time() - t0:.1f} s")
    chain = pg.Chain(spec, w_dev, dev)
    stream = torch.cuda.Stream(device=dev)
    n_sets = 3
    x_np = [make_inputs(spec, t) for t in range(n_sets)]
    x_dev = [[to_device(x, dev) for x in xs] for xs in x_np]
    t0 = time.time()
    chain.capture(stream)
    capture_s = time.time() - t0
    cost = chain.profile(x_dev[0], stream, iters=args.profile_iters, inner=3)
    sel = pg.select(cost)
    log(f"[bench] captured in {capture_s * 1e3:.1f} ms; cost table (us) {cost.tolist()} -> selected mode {sel.tolist()}")

    def timed(mode, modes=None):
        chain.time_loop(mode, x_dev, max(W, 1), stream, modes)      # warm-up, untimed
        torch.cuda.synchronize()
        us = chain.time_loop(mode, x_dev, K, stream, modes)         # synchronises before and after
        torch.cuda.synchronize()
        return us

    us, us_median, us_p90 = {}, {}, {}
    for name, mode, modes in (("eager", pg.EAGER, None), ("graph_copy", pg.GRAPH_COPY, None),
                              ("graph_indirect", pg.GRAPH_INDIRECT, None), ("selected", pg.SELECTED, sel)):
        us[name] = timed(mode, modes)
        log(f"[bench] {name}: {us[name]:.1f} us/iteration")
        if not args.no_refresh_baselines:
            each = chain.time_loop_each(mode, x_dev, min(K, 100), stream, modes)     # per-iteration times, from events on the stream
            us_median[name], us_p90[name] = float(np.median(each)), float(np.quantile(each, 0.9))
            log(f"[bench] {name}: median {us_median[name]:.1f}, p90 {us_p90[name]:.1f} us over {len(each)} event-timed iterations")
    chain.set_table_refresh(pg.TABLE_MEMCPY)
    us_ind_memcpy = timed(pg.GRAPH_INDIRECT)
    chain.set_table_refresh(pg.TABLE_KERNARG)
    log(f"[bench] graph_indirect with a pinned-memcpy table refresh: {us_ind_memcpy:.1f} us/iteration")
    # the baselines the two refresh designs stand against: the host rewrites the external-reading
    # kernel nodes' arguments before each launch; the copy refresh as one memcpy per tensor
    us_update = us_copy_memcpy = us_ind_graph_memcpy = us_ind_host_table = None
    if not args.no_refresh_baselines:
        # the other two ways of getting the pointers to the kernels: a copy node inside the graph, a host-resident table
        chain.set_table_refresh(pg.TABLE_GRAPH_MEMCPY)
        us_ind_graph_memcpy = timed(pg.GRAPH_INDIRECT)
        chain.set_table_refresh(pg.TABLE_HOST)
        us_ind_host_table = timed(pg.GRAPH_INDIRECT)
        chain.set_table_refresh(pg.TABLE_KERNARG)
        log(f"[bench] graph_indirect, pointers by a copy node inside the graph: {us_ind_graph_memcpy:.1f}; from a host-resident table: {us_ind_host_table:.1f} us/iteration")
        us_update = timed(pg.GRAPH_UPDATE)
        log(f"[bench] graph with host-side node updates: {us_update:.1f} us/iteration")
        chain.set_copy_refresh(pg.COPY_MEMCPY)
        us_copy_memcpy = timed(pg.GRAPH_COPY)
        chain.set_copy_refresh(pg.COPY_KERNEL)
        log(f"[bench] graph_copy with per-tensor memcpy: {us_copy_memcpy:.1f} us/iteration")

    # ------------------------------------------------------------------ the dominant kernel alone: GEMV 2048x2048, HIP events on the launch stream
    # A graph of the chain's 120 GEMV launches and nothing else (same kernel, same launch shape, the
    # chain's own 120 weight matrices, input vector fixed): events around R replays give the time per
    # launch.  It includes the dispatch gap between two dependent launches, so it is an upper bound of
    # the kernel's own duration (the rocprofv3 kernel trace gives the latter).
    from pg_workloads import ChainSpec, KernelSpec, TensorSpec, Ref, INT, WEIGHT
    n_k = len(spec.kernels)
    n_gemv = sum(1 for k in spec.kernels if k.op == "gemv")
    H = spec.meta["hidden"]
    gspec = ChainSpec("gemv_only", [KernelSpec("gemv", "bf16", 0, (Ref(WEIGHT, s), Ref(WEIGHT, n_gemv)), H, rows=1, cols=H) for s in range(n_gemv)],
                      [], [TensorSpec("bf16", H)], list(spec.weights[:n_gemv]) + [TensorSpec("bf16", H)], [0])
    gchain = pg.Chain(gspec, w_dev[:n_gemv] + [x_dev[0][0]], dev)
    gchain.capture(stream)
    reps = 50
    for _ in range(5):
        gchain.replay_copy([], stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(reps):
        gchain.replay_copy([], stream)        # no external input: this is the graph launch alone
    e1.record(stream)
    e1.synchronize()
    gemv_us = e0.elapsed_time(e1) * 1e3 / (reps * n_gemv)
    gchain.close()
    gemv_bytes = H * H * 2 + H * 2 + H * 2       # bf16 weight matrix + input vector + output vector
    log(f"[bench] GEMV alone: {gemv_us:.2f} us per launch = {gemv_bytes / gemv_us / 1e3:.0f} GB/s")
    roofline = {"kernel": "k_gemv_shared<bf16> 2048x2048, batch 1", "bound": "hbm", "achieved": gemv_bytes / gemv_us / 1e3,
                "peak": HBM_PEAK, "unit": "GB/s", "frac": gemv_bytes / gemv_us / 1e3 / HBM_PEAK,
                "bytes_per_launch": gemv_bytes, "avg_launch_us": gemv_us, "launches_timed": reps * n_gemv,
                "how": "HIP events on the launch stream around 50 replays of a graph of the chain's 120 GEMV launches; per-launch time includes the inter-kernel dispatch gap",
                # HBM bytes per launch from the hardware-counter runs (FETCH_SIZE x 1.9996 + WRITE_SIZE x 1.0000,
                # factors from a plain 256 MiB copy in the same run); the summary sits beside the other profiles
                "traffic": 8.471e6, "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/gemv_and_copy_kernel_hbm_traffic.md"}
    # The dispatch floor of this machine: the time per node of a graph of 512 dependent kernels that do next
    # to nothing (64 elements each).  What the GEMV adds to it is its own memory time.
    # (Left out of the profiler runs together with the refresh baselines: see the flag's help text.)
    if not args.no_refresh_baselines:
        from pg_workloads import elementwise_chain
        fspec = elementwise_chain(n_kernels=512, numel=64, dtype="bf16")
        fchain = pg.Chain(fspec, [], dev)
        fchain.capture(stream)
        fx = [[to_device(x, dev) for x in make_inputs(fspec, t)] for t in range(2)]
        fchain.time_loop(pg.GRAPH_INDIRECT, fx, 10, stream)
        floor_us = fchain.time_loop(pg.GRAPH_INDIRECT, fx, 50, stream) / len(fspec.kernels)
        fchain.close()
        roofline["dispatch_floor_us_per_node"] = floor_us
        roofline["achieved_above_floor"] = gemv_bytes / max(gemv_us - floor_us, 1e-3) / 1e3
        roofline["frac_above_floor"] = roofline["achieved_above_floor"] / HBM_PEAK
        log(f"[bench] dispatch floor {floor_us:.2f} us per node; the GEMV's bytes over the time it adds to the floor: {roofline['achieved_above_floor']:.0f} GB/s")
    chain_bytes = sum(t.nbytes for t in spec.weights)     # every weight is read once per iteration
    chain_level = {m: chain_bytes / us[m] / 1e3 for m in us}

    # ------------------------------------------------------------------ copy kernel on the config-3 size mix
    copy = None
    if not args.no_copy_bench:
        spec3 = refresh_stress_chain()
        log(f"[bench] copy kernel: {len(spec3.ext)} tensors, {spec3.ext_bytes() / 1e6:.1f} MB payload; generating inputs")
        w3 = [to_device(w, dev) for w in make_weights(spec3)]
        chain3 = pg.Chain(spec3, w3, dev)
        chain3.capture(stream)
        g = torch.Generator(device=dev)
        g.manual_seed(spec3.seed)
        # bandwidth does not depend on the values: draw them on the device (parity of this kernel is tested with the seeded host recipe)
        sets3 = [[torch.randn(t.numel, device=dev, generator=g, dtype=torch.float32).to(torch.bfloat16) for t in spec3.ext] for _ in range(2)]
        for r in range(3):
            chain3.time_refresh_copy(sets3[r % 2], stream)
        cu = np.array([chain3.time_refresh_copy(sets3[r % 2], stream) for r in range(20)])
        payload = spec3.ext_bytes()
        copy = {"kernel": "k_copy (batched multi-tensor)", "bound": "hbm", "achieved": 2 * payload / float(cu.mean()) / 1e3,
                "peak": HBM_PEAK, "unit": "GB/s", "frac": 2 * payload / float(cu.mean()) / 1e3 / HBM_PEAK,
                "payload_bytes": payload, "bytes_per_launch": 2 * payload, "avg_launch_us": float(cu.mean()),
                "min_launch_us": float(cu.min()), "launches_timed": 20,
                "traffic": 892.4e6, "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/gemv_and_copy_kernel_hbm_traffic.md"}
        log(f"[bench] copy kernel: {cu.mean():.1f} us for {2 * payload / 1e6:.1f} MB of traffic = {copy['achieved']:.0f} GB/s")
        us3 = {}
        for name, mode in (("eager", pg.EAGER), ("graph_copy", pg.GRAPH_COPY), ("graph_indirect", pg.GRAPH_INDIRECT)):
            chain3.time_loop(mode, sets3, 3, stream)
            us3[name] = chain3.time_loop(mode, sets3, 20, stream)
        if not args.no_refresh_baselines:
            chain3.time_loop(pg.GRAPH_UPDATE, sets3, 3, stream)
            us3["graph_update"] = chain3.time_loop(pg.GRAPH_UPDATE, sets3, 20, stream)
            log(f"[bench] refresh-stress chain, host-side node updates: {us3['graph_update']:.1f} us/iteration")
            chain3.set_copy_refresh(pg.COPY_MEMCPY)
            chain3.time_loop(pg.GRAPH_COPY, sets3, 3, stream)
            us3["graph_copy_per_tensor_memcpy"] = chain3.time_loop(pg.GRAPH_COPY, sets3, 20, stream)
            chain3.set_copy_refresh(pg.COPY_KERNEL)
        # a plain device-to-device copy of known size (256 MiB read + 256 MiB written): the yardstick the
        # hardware-counter byte counts of a profiled run are scaled by
        cal_src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        cal_dst = torch.empty_like(cal_src)
        with torch.cuda.stream(stream):
            for _ in range(3):
                cal_dst.copy_(cal_src)
        stream.synchronize()
        del cal_src, cal_dst
        copy["refresh_stress_chain_us_per_iter"] = us3
        log(f"[bench] refresh-stress chain (256 kernels): {us3}")
        chain3.close()
        del sets3, chain3

    # ------------------------------------------------------------------ the CPU oracle on the same workload, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        oracle.run_chain(spec, w_np, x_np[0])
        n_done, t0 = 0, time.time()
        while True:
            out = oracle.run_chain(spec, w_np, x_np[n_done % n_sets])
            n_done += 1
            if time.time() - t0 > args.cpu_seconds or n_done >= 100:
                break
        cpu_us = (time.time() - t0) / n_done * 1e6
        cpu = {"value": cpu_us, "unit": "us/iteration", "cores": oracle.max_threads(), "kind": "oracle",
               "sample": f"{n_done} whole iterations of the same 511-kernel chain and inputs ({time.time() - t0:.1f} s of wall time)"}
        # the same oracle on one thread (two iterations): how much of the figure above is the core count
        n_all = oracle.max_threads()
        try:
            oracle.set_threads(1)
            t1 = time.time()
            for i in range(2):
                oracle.run_chain(spec, w_np, x_np[i % n_sets])
            cpu["value_on_1_thread"] = (time.time() - t1) / 2 * 1e6
        finally:
            oracle.set_threads(n_all)
        # the sample doubles as a live parity check of the timed configuration
        chain.replay_indirect(x_dev[(n_done - 1) % n_sets], stream)
        stream.synchronize()
        g, o = chain.output(0), out[0]
        from pg_workloads import bf16_bits_to_f32
        gf, of = bf16_bits_to_f32(g).astype(np.float64), bf16_bits_to_f32(o).astype(np.float64)
        cpu["rel_l2_gpu_vs_oracle"] = float(np.sqrt(((gf - of) ** 2).sum() / (of ** 2).sum()))
        # elements whose bf16 patterns differ, and the largest |g - o| / max(|o|, rms(o)) (the bf16 bound is 2e-2)
        rms = float(np.sqrt(np.mean(of * of)))
        cpu["elements_differing"] = int((g != o).sum())
        cpu["max_err_over_scale"] = float((np.abs(gf - of) / np.maximum(np.abs(of), rms)).max())
        log(f"[bench] oracle: {cpu_us / 1e3:.1f} ms/iteration on {cpu['cores']} threads; GPU vs oracle rel L2 {cpu['rel_l2_gpu_vs_oracle']:.2e}")

    step_us = sum(us.values())
    result = {
        "metric": "us/iteration of the 511-kernel decode chain: graph-indirect replay (eager, graph-copy, selected alongside); copy-kernel HBM GB/s",
        "value": us["graph_indirect"], "unit": "us/iteration", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": step_us / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "decode-step chain, batch 1: 24 layers x 5 x (RMSNorm 2048 + bf16 GEMV 2048x2048 + GELU + residual add) + 31 input adds = 511 kernels/iteration, 32 fresh bf16[2048] inputs/iteration, weights ~N(0,0.02^2)",
                   "kernels_per_iteration": n_k, "external_inputs": len(spec.ext), "input_sets": n_sets,
                   "step": "one iteration in each of: eager, graph-copy, graph-indirect, selected"},
        "us_per_iteration": us, "us_per_iteration_median": us_median, "us_per_iteration_p90": us_p90,
        "launches_per_s": {m: n_k / us[m] * 1e6 for m in us},
        "speedup_vs_eager": {m: us["eager"] / us[m] for m in us},
        "graph_indirect_memcpy_table_us": us_ind_memcpy,
        "graph_indirect_copy_node_in_graph_us": us_ind_graph_memcpy, "graph_indirect_host_table_us": us_ind_host_table,
        "graph_host_node_update_us": us_update, "graph_copy_per_tensor_memcpy_us": us_copy_memcpy,
        "selection": {"cost_table_us": [[None if not np.isfinite(v) else float(v) for v in row] for row in cost.tolist()], "mode": sel.tolist()},
        "idle_gap_fraction": None,   # needs per-kernel durations: taken from the rocprofv3 kernel trace, reported with the profile summaries
        "chain_level_GBps": chain_level, "chain_level_hbm_frac": {m: chain_level[m] / HBM_PEAK for m in us},
        "bytes_refreshed_per_replay": {"graph_copy": chain.stats()["copy_bytes_per_replay"], "graph_indirect": chain.stats()["table_bytes_per_replay"]},
        "capture_ms": capture_s * 1e3,
        "roofline": roofline, "copy_kernel": copy, "cpu_baseline": cpu,
    }
    chain.close()
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
