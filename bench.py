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

Beside it, in the same JSON line: the same graphs captured with one node per kernel (dispatch
merging off), the dispatch floor of this machine (`graph_node_us`, `eager_launch_us`), the dominant
kernel against the HBM roofline, the copy kernel, the other benchmark chains (`configs`: 1, 3, 4
and the eight batch-size buckets of 5 with the 1000-iteration bucket sequence), and the CPU oracle
timed on the host.  One JSON line on stdout; progress on stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
HBM_PEAK = 8000.0   # GB/s, MI355X


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def profiler_attached() -> bool:
    """True under rocprofv3 (it preloads its tool library and announces it in the environment)."""
    keys = ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "HSA_TOOLS_LIB", "ROCPROFILER_LIBRARY_CTOR")
    return any("rocprof" in os.environ.get(k, "").lower() for k in keys) or "ROCPROF_OUTPUT_PATH" in os.environ


def profile_figures(name: str) -> dict:
    """`key: number` lines of the 'Figures read by bench.py' section of a committed rocprofv3 summary."""
    path = os.path.join(ROOT, "profiles", name)
    out = {}
    try:
        text = open(path).read()
    except OSError:
        return out
    if "## Figures read by bench.py" not in text:
        return out
    for line in text.split("## Figures read by bench.py", 1)[1].splitlines():
        m = re.match(r"\s*([a-z0-9_]+):\s*([-+0-9.eE]+)\s*$", line)
        if m:
            out[m.group(1)] = float(m.group(2))
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--no-copy-bench", action="store_true", help="skip the copy-kernel bandwidth leg (config 3 sizes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="skip the other benchmark chains (configs 1, 4, 5)")
    ap.add_argument("--no-refresh-baselines", action="store_true",
                    help="skip the legs added beside the three modes (host-side node updates, per-tensor memcpy, the two alternating table "
                         "mechanisms, the event-timed medians).  They are skipped by themselves when a profiler is attached: two counter-collection "
                         "runs that included them did not complete (one went silent, one ended in a segmentation fault inside a profiler thread)")
    ap.add_argument("--no-gemv-graphs", action="store_true",
                    help="skip the graphs of the dominant kernel alone (they build, capture and destroy two more chains).  For counter-collection "
                         "runs, which only need the kernels of the main chain: one such run went silent inside these legs")
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="budget of the oracle timing leg")
    ap.add_argument("--profile-iters", type=int, default=20, help="samples per (segment, mode) of the slow-path profiler")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); run it with --gpus 1", file=sys.stderr)
        return 2
    under_profiler = profiler_attached()
    if under_profiler and not args.no_refresh_baselines:
        log("[bench] a profiler is attached: the refresh-baseline legs are skipped")
        args.no_refresh_baselines = True

    import torch
    import paper_2503_19779_amd as pg
    from paper_2503_19779_amd.binding import to_device
    from pg_workloads import (ChainSpec, KernelSpec, TensorSpec, Ref, WEIGHT, decode_chain, decode_buckets, bucket_sequence,
                              elementwise_chain, large_tensor_chain, refresh_stress_chain, make_weights, make_inputs, bf16_bits_to_f32)

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = "cuda:0"
    torch.cuda.set_device(0)
    K, W = args.steps, args.warmup
    stream = torch.cuda.Stream(device=dev)
    MODES = (("eager", pg.EAGER), ("graph_copy", pg.GRAPH_COPY), ("graph_indirect", pg.GRAPH_INDIRECT))
    DT = {"f32": torch.float32, "bf16": torch.bfloat16}

    def device_sets(spec, n, seed_offset=0):
        """n sets of external inputs drawn on the device (timing legs whose values do not matter)."""
        g = torch.Generator(device=dev)
        g.manual_seed(spec.seed + seed_offset)
        return [[torch.randn(t.numel, device=dev, generator=g, dtype=torch.float32).to(DT[t.dtype]) for t in spec.ext] for _ in range(n)]

    def timed(chain, sets, mode, iters, warm, modes=None):
        chain.time_loop(mode, sets, max(warm, 1), stream, modes)      # warm-up, untimed
        torch.cuda.synchronize()
        us = chain.time_loop(mode, sets, iters, stream, modes)        # synchronises before and after
        torch.cuda.synchronize()
        return us

    def clean(cost):
        return [[None if not np.isfinite(v) else float(v) for v in row] for row in np.asarray(cost).tolist()]

    # ------------------------------------------------------------------ workload: decode chain, batch 1
    spec = decode_chain()
    log(f"[bench] {spec.name}: {len(spec.kernels)} kernels; generating {sum(w.nbytes for w in spec.weights) / 1e9:.3f} GB of weights")
    t0 = time.time()
    w_np = make_weights(spec)
    w_dev = [to_device(w, dev) for w in w_np]
    log(f"[bench] weights resident after {time.time() - t0:.1f} s")
    chain = pg.Chain(spec, w_dev, dev)
    n_sets = 3
    x_np = [make_inputs(spec, t) for t in range(n_sets)]
    x_dev = [[to_device(x, dev) for x in xs] for xs in x_np]
    n_k = len(spec.kernels)
    dispatches_merged, dispatches_unmerged = chain.graph_dispatches()

    # graphs with one node per kernel first (the plain form of a captured graph), then with dispatch merging
    us_plain = {}
    if not under_profiler:          # a re-capture destroys graphs: kept out of profiled runs (see --no-refresh-baselines)
        chain.set_dispatch_merge(False)
        chain.capture(stream)
        us_plain = {name: timed(chain, x_dev, mode, K, W) for name, mode in MODES[1:]}
        log(f"[bench] graphs with one node per kernel ({dispatches_unmerged} nodes): {us_plain}")
    chain.set_dispatch_merge(True)
    t0 = time.time()
    chain.capture(stream)
    capture_s = time.time() - t0
    cost = chain.profile(x_dev[0], stream, iters=args.profile_iters, inner=3)
    sel = pg.select(cost)
    log(f"[bench] captured in {capture_s * 1e3:.1f} ms ({dispatches_merged} nodes); cost table (us) {cost.tolist()} -> selected mode {sel.tolist()}")

    us, us_median, us_p90 = {}, {}, {}
    for name, mode, modes in (("eager", pg.EAGER, None), ("graph_copy", pg.GRAPH_COPY, None),
                              ("graph_indirect", pg.GRAPH_INDIRECT, None), ("selected", pg.SELECTED, sel)):
        us[name] = timed(chain, x_dev, mode, K, W, modes)
        log(f"[bench] {name}: {us[name]:.1f} us/iteration")
        if not args.no_refresh_baselines:
            each = chain.time_loop_each(mode, x_dev, min(K, 100), stream, modes)     # per-iteration times, from events on the stream
            us_median[name], us_p90[name] = float(np.median(each)), float(np.quantile(each, 0.9))
            log(f"[bench] {name}: median {us_median[name]:.1f}, p90 {us_p90[name]:.1f} us over {len(each)} event-timed iterations")
    chain.set_table_refresh(pg.TABLE_MEMCPY)
    us_ind_memcpy = timed(chain, x_dev, pg.GRAPH_INDIRECT, K, W)
    chain.set_table_refresh(pg.TABLE_KERNARG)
    log(f"[bench] graph_indirect with a pinned-memcpy table refresh: {us_ind_memcpy:.1f} us/iteration")
    # the baselines the two refresh designs stand against: the host rewrites the external-reading
    # kernel nodes' arguments before each launch; the copy refresh as one memcpy per tensor
    us_update = us_copy_memcpy = us_ind_graph_memcpy = us_ind_host_table = None
    if not args.no_refresh_baselines:
        chain.set_table_refresh(pg.TABLE_GRAPH_MEMCPY)
        us_ind_graph_memcpy = timed(chain, x_dev, pg.GRAPH_INDIRECT, K, W)
        chain.set_table_refresh(pg.TABLE_HOST)
        us_ind_host_table = timed(chain, x_dev, pg.GRAPH_INDIRECT, K, W)
        chain.set_table_refresh(pg.TABLE_KERNARG)
        log(f"[bench] graph_indirect, pointers by a copy node inside the graph: {us_ind_graph_memcpy:.1f}; from a host-resident table: {us_ind_host_table:.1f} us/iteration")
        us_update = timed(chain, x_dev, pg.GRAPH_UPDATE, K, W)
        log(f"[bench] graph with host-side node updates (one node per kernel): {us_update:.1f} us/iteration")
        chain.set_copy_refresh(pg.COPY_MEMCPY)
        us_copy_memcpy = timed(chain, x_dev, pg.GRAPH_COPY, K, W)
        chain.set_copy_refresh(pg.COPY_KERNEL)
        log(f"[bench] graph_copy with per-tensor memcpy: {us_copy_memcpy:.1f} us/iteration")

    # ------------------------------------------------------------------ the dispatch floor of this machine
    # 512 dependent kernels that do next to nothing (64 elements each), one graph node per kernel: the
    # time per node of a replay and the time per launch of the eager loop are what a kernel costs here
    # before it does any work; their ratio is the ceiling of graph over eager for launch-bound chains.
    # (Not under a profiler: it belongs to the legs whose profiled runs did not complete.)
    graph_node_us = eager_launch_us = None
    if not under_profiler:
        fspec = elementwise_chain(n_kernels=512, numel=64, dtype="bf16")
        fchain = pg.Chain(fspec, [], dev)
        fchain.set_dispatch_merge(False)
        fchain.capture(stream)
        fx = [[to_device(x, dev) for x in make_inputs(fspec, t)] for t in range(3)]
        graph_node_us = timed(fchain, fx, pg.GRAPH_INDIRECT, 50, 10) / len(fspec.kernels)
        eager_launch_us = timed(fchain, fx, pg.EAGER, 50, 10) / len(fspec.kernels)
        fchain.close()
        log(f"[bench] dispatch floor: {graph_node_us:.2f} us per graph node, {eager_launch_us:.2f} us per eager launch")

    # ------------------------------------------------------------------ the dominant kernel alone, HIP events on the launch stream
    # In graph replay the dominant kernel is the decode sub-block's one dispatch: the GEMV 2048x2048 with the
    # RMSNorm in front of it as its prologue and the GELU and the residual add behind it as its epilogue; in
    # eager launches it is the plain GEMV.  Each is timed in a graph of the chain's 120 such launches (same
    # kernels, same launch shapes, the chain's own 120 weight matrices, the stream initialised by one small
    # add): events around R replays give the time per launch.  It includes the dispatch gap between two
    # dependent launches, so it is an upper bound of the kernel's own duration (the rocprofv3 kernel trace
    # gives the latter).
    from pg_workloads import INT
    n_gemv = sum(1 for k in spec.kernels if k.op == "gemv")
    H = spec.meta["hidden"]
    reps = 50

    def gemv_graph_us(sub_block: bool):
        """(us per launch, launches per replay) of a graph of the chain's GEMVs alone, or of its whole sub-blocks."""
        X, T1, T2 = 0, 1, 2
        gain = n_gemv + 1
        ks = []
        if sub_block:
            ks.append(KernelSpec("add", "bf16", X, (Ref(WEIGHT, n_gemv), Ref(WEIGHT, n_gemv)), H, m=H))       # the stream, before the first sub-block
        for s_ in range(n_gemv):
            if sub_block:
                ks.append(KernelSpec("rmsnorm", "bf16", T1, (Ref(INT, X), Ref(WEIGHT, gain)), H, rows=1, cols=H, eps=1e-6))
                ks.append(KernelSpec("gemv", "bf16", T2, (Ref(WEIGHT, s_), Ref(INT, T1)), H, rows=1, cols=H))
                ks.append(KernelSpec("gelu", "bf16", T2, (Ref(INT, T2),), H))
                ks.append(KernelSpec("add", "bf16", X, (Ref(INT, X), Ref(INT, T2)), H, m=H))
            else:
                ks.append(KernelSpec("gemv", "bf16", 0, (Ref(WEIGHT, s_), Ref(WEIGHT, n_gemv)), H, rows=1, cols=H))
        gspec = ChainSpec("gemv_only", ks, [], [TensorSpec("bf16", H)] * 3,
                          list(spec.weights[:n_gemv]) + [TensorSpec("bf16", H), TensorSpec("bf16", H)], [0])
        gchain = pg.Chain(gspec, w_dev[:n_gemv] + [x_dev[0][0], w_dev[n_gemv]], dev)
        nodes = gchain.graph_dispatches()[0]
        assert nodes == n_gemv + (1 if sub_block else 0), nodes      # an even number of renaming sub-blocks: none is split back into RMSNorm + GEMV dispatch
        gchain.capture(stream)
        for _ in range(5):
            gchain.replay_copy([], stream)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(reps):
            gchain.replay_copy([], stream)        # no external input: this is the graph launch alone
        e1.record(stream)
        e1.synchronize()
        gchain.close()
        return e0.elapsed_time(e1) * 1e3 / (reps * nodes), nodes

    if args.no_gemv_graphs:       # the figures that need them are then reported as NaN
        gemv_us = epi_us = float("nan")
        epi_nodes = n_gemv + 1
    else:
        gemv_us, _ = gemv_graph_us(False)
        epi_us, epi_nodes = gemv_graph_us(True)
    gemv_bytes = H * H * 2 + H * 2 + H * 2       # bf16 weight matrix + input vector + output vector
    # weight matrix; read: the stream and the gain; written: the normalised vector, the GELU result, the new stream
    epi_bytes = H * H * 2 + 2 * H * 2 + 3 * H * 2
    log(f"[bench] GEMV alone: {gemv_us:.2f} us per launch = {gemv_bytes / gemv_us / 1e3:.0f} GB/s; the whole sub-block (RMSNorm, GEMV, GELU, residual add) in one dispatch: {epi_us:.2f} us = {epi_bytes / epi_us / 1e3:.0f} GB/s")
    tr = profile_figures("decode_chain_b1_kernel_trace.md")
    hb = profile_figures("gemv_and_copy_kernel_hbm_traffic.md")
    how = ("HIP events on the launch stream around 50 replays of a graph of the chain's 120 launches of this kernel (and one small add that "
           "initialises the stream, counted as a launch); the time per launch includes the dispatch gap between two dependent launches")
    roofline = {"kernel": "k_gemv_epilogue<1, prologue>: bf16 GEMV 2048x2048, batch 1, with the RMSNorm as its prologue and GELU and the residual add as its epilogue (a decode sub-block in one graph node; the dominant kernel of graph replay)",
                "bound": "hbm", "achieved": epi_bytes / epi_us / 1e3, "peak": HBM_PEAK, "unit": "GB/s", "frac": epi_bytes / epi_us / 1e3 / HBM_PEAK,
                "frac_denominator": "avg_launch_us: " + how,
                "bytes_per_launch": epi_bytes, "avg_launch_us": epi_us, "launches_timed": reps * epi_nodes,
                # the same bytes over the kernel's own duration in the committed rocprofv3 kernel trace (dispatch start to end, mean over all its dispatches)
                "profile_kernel_mean_us": tr.get("gemv_epilogue_kernel_mean_us"),
                "frac_from_profile": (epi_bytes / tr["gemv_epilogue_kernel_mean_us"] / 1e3 / HBM_PEAK) if tr.get("gemv_epilogue_kernel_mean_us") else None,
                "frac_from_profile_source": "profiles/decode_chain_b1_kernel_trace.md (rocprofv3 --kernel-trace --stats)",
                # HBM bytes per launch from the committed hardware-counter runs (FETCH_SIZE, WRITE_SIZE, each scaled by what the same counter reads for a plain 256 MiB copy)
                "traffic": hb.get("gemv_epilogue_traffic_bytes_per_launch"),
                "traffic_source": "profiles/gemv_and_copy_kernel_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)",
                "dispatch_floor_us_per_node": graph_node_us,
                # the plain GEMV (what an eager launch and a graph with one node per kernel run), measured the same way
                "gemv_alone": {"kernel": "k_gemv_shared<bf16> 2048x2048, batch 1", "achieved": gemv_bytes / gemv_us / 1e3, "frac": gemv_bytes / gemv_us / 1e3 / HBM_PEAK,
                               "bytes_per_launch": gemv_bytes, "avg_launch_us": gemv_us, "launches_timed": reps * n_gemv,
                               "profile_kernel_mean_us": tr.get("gemv_kernel_mean_us"),
                               "frac_from_profile": (gemv_bytes / tr["gemv_kernel_mean_us"] / 1e3 / HBM_PEAK) if tr.get("gemv_kernel_mean_us") else None,
                               "traffic": hb.get("gemv_traffic_bytes_per_launch")}}
    chain_bytes = sum(t.nbytes for t in spec.weights)     # every weight is read once per iteration
    chain_level = {m: chain_bytes / us[m] / 1e3 for m in us}

    # idle-gap fraction: 1 - (sum of the kernels' own durations in one iteration, from the committed kernel trace) / (this run's time per iteration)
    idle = None
    if tr.get("busy_us_per_iteration_eager") and tr.get("busy_us_per_iteration_graph"):
        idle = {"eager": max(0.0, 1 - tr["busy_us_per_iteration_eager"] / us["eager"]),
                "graph_copy": max(0.0, 1 - tr["busy_us_per_iteration_graph"] / us["graph_copy"]),
                "graph_indirect": max(0.0, 1 - tr["busy_us_per_iteration_graph"] / us["graph_indirect"]),
                "busy_us_per_iteration": {"eager": tr["busy_us_per_iteration_eager"], "graph": tr["busy_us_per_iteration_graph"]},
                "source": "busy time: profiles/decode_chain_b1_kernel_trace.md (sum over one iteration's dispatches of their start-to-end durations); "
                          "time per iteration: this run"}

    # ------------------------------------------------------------------ copy kernel on the config-3 size mix, and config 3's chain
    copy = None
    configs = {}
    if not args.no_copy_bench:
        spec3 = refresh_stress_chain()
        log(f"[bench] copy kernel: {len(spec3.ext)} tensors, {spec3.ext_bytes() / 1e6:.1f} MB payload; generating inputs")
        w3 = [to_device(w, dev) for w in make_weights(spec3)]
        chain3 = pg.Chain(spec3, w3, dev)
        chain3.capture(stream)
        # bandwidth does not depend on the values: draw them on the device (parity of this kernel is tested with the seeded host recipe)
        sets3 = device_sets(spec3, 2)
        for r in range(3):
            chain3.time_refresh_copy(sets3[r % 2], stream)
        cu = np.array([chain3.time_refresh_copy(sets3[r % 2], stream) for r in range(20)])
        payload = spec3.ext_bytes()
        copy = {"kernel": "k_copy (batched multi-tensor)", "bound": "hbm", "achieved": 2 * payload / float(cu.mean()) / 1e3,
                "peak": HBM_PEAK, "unit": "GB/s", "frac": 2 * payload / float(cu.mean()) / 1e3 / HBM_PEAK,
                "payload_bytes": payload, "bytes_per_launch": 2 * payload, "avg_launch_us": float(cu.mean()),
                "min_launch_us": float(cu.min()), "launches_timed": 20,
                "traffic": hb.get("copy_traffic_bytes_per_launch"),
                "traffic_source": "profiles/gemv_and_copy_kernel_hbm_traffic.md (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE)"}
        log(f"[bench] copy kernel: {cu.mean():.1f} us for {2 * payload / 1e6:.1f} MB of traffic = {copy['achieved']:.0f} GB/s")
        cost3 = chain3.profile(sets3[0], stream, iters=5, inner=2)
        sel3 = pg.select(cost3)
        us3 = {name: timed(chain3, sets3, mode, 20, 3) for name, mode in MODES}
        us3["selected"] = timed(chain3, sets3, pg.SELECTED, 20, 3, sel3)
        if not args.no_refresh_baselines:
            us3["graph_update"] = timed(chain3, sets3, pg.GRAPH_UPDATE, 20, 3)
            chain3.set_copy_refresh(pg.COPY_MEMCPY)
            us3["graph_copy_per_tensor_memcpy"] = timed(chain3, sets3, pg.GRAPH_COPY, 20, 3)
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
        st3 = chain3.stats()
        configs["3"] = {"workload": "256 bf16 tensors, 1 KB .. 16 MB log-uniform, refreshed per iteration, then 256 elementwise kernels reading them",
                        "kernels": st3["n_kernels"], "us_per_iteration": us3, "launches_per_s": {m: st3["n_kernels"] / v * 1e6 for m, v in us3.items()},
                        "selection": {"cost_table_us": clean(cost3), "mode": sel3.tolist()},
                        "bytes_refreshed_per_replay": {"graph_copy": st3["copy_bytes_per_replay"], "graph_indirect": st3["table_bytes_per_replay"]}}
        copy["refresh_stress_chain_us_per_iter"] = us3
        log(f"[bench] config 3 (256 kernels): {us3} selected {sel3.tolist()}")
        chain3.close()
        del sets3, chain3, w3

    # ------------------------------------------------------------------ the other benchmark chains
    if not args.no_configs:
        # config 1: 64 fp32 elementwise kernels on 4096 elements, 4 external inputs, seeded host inputs
        spec1 = elementwise_chain()
        c1 = pg.Chain(spec1, [], dev)
        c1.capture(stream)
        x1 = [[to_device(x, dev) for x in make_inputs(spec1, t)] for t in range(3)]
        cost1 = c1.profile(x1[0], stream, iters=10, inner=3)
        sel1 = pg.select(cost1)
        us1 = {name: timed(c1, x1, mode, 100, 10) for name, mode in MODES}
        us1["selected"] = timed(c1, x1, pg.SELECTED, 100, 10, sel1)
        configs["1"] = {"workload": "64 fp32 elementwise kernels (add, mul, GELU) on 4096 elements, 4 external inputs",
                        "kernels": len(spec1.kernels), "graph_nodes": c1.graph_dispatches()[0], "us_per_iteration": us1,
                        "launches_per_s": {m: len(spec1.kernels) / v * 1e6 for m, v in us1.items()},
                        "selection": {"cost_table_us": clean(cost1), "mode": sel1.tolist()}}
        log(f"[bench] config 1: {us1} selected {sel1.tolist()}")
        c1.close()

        # config 4: 40 fp32 scale+bias+ReLU kernels on [32,64,112,112] in 4 segments; one 103 MB external input
        spec4 = large_tensor_chain()
        w4 = [to_device(w, dev) for w in make_weights(spec4)]
        c4 = pg.Chain(spec4, w4, dev)
        c4.capture(stream)
        x4 = device_sets(spec4, 3)
        cost4 = c4.profile(x4[0], stream, iters=5, inner=2)
        sel4 = pg.select(cost4)
        us4 = {name: timed(c4, x4, mode, 20, 3) for name, mode in MODES}
        us4["selected"] = timed(c4, x4, pg.SELECTED, 20, 3, sel4)
        bytes4 = 2 * spec4.ext[0].nbytes * len(spec4.kernels)
        configs["4"] = {"workload": "40 fp32 scale+bias+ReLU kernels on [32,64,112,112] in 4 segments, one 102.8 MB external input",
                        "kernels": len(spec4.kernels), "segments": 4, "us_per_iteration": us4,
                        "launches_per_s": {m: len(spec4.kernels) / v * 1e6 for m, v in us4.items()},
                        "selection": {"cost_table_us": clean(cost4), "mode": sel4.tolist()},
                        "algorithmic_GBps": {m: bytes4 / v / 1e3 for m, v in us4.items()},
                        "hbm_frac": {m: bytes4 / v / 1e3 / HBM_PEAK for m, v in us4.items()}}
        log(f"[bench] config 4: {us4} selected {sel4.tolist()}")
        c4.close()
        del x4, c4, w4

        # config 5: the decode chain at 8 batch sizes, one chain (one set of graphs) per bucket over one set of
        # weights, then a random bucket sequence of 1000 iterations.  The weights are the batch-1 chain's (same
        # shapes; timing does not depend on the values, parity of these shapes is tested with the seeded recipe).
        specs5 = decode_buckets()
        chains5, sets5, per_bucket = [], [], []
        for s5 in specs5:
            c5 = pg.Chain(s5, w_dev, dev)
            c5.capture(stream)
            chains5.append(c5)
            sets5.append(device_sets(s5, 2))
        for i, (s5, c5) in enumerate(zip(specs5, chains5)):
            # cost table measured where the bucket will run: between iterations of another bucket's chain
            j = (i + 1) % len(chains5)
            cost5 = c5.profile_in_context(sets5[i][0], chains5[j], sets5[j][0], pg.GRAPH_INDIRECT, stream, iters=5, inner=3)
            alone5 = c5.profile(sets5[i][0], stream, iters=5, inner=2)
            sel5 = pg.select(cost5)
            us5 = {name: timed(c5, sets5[i], mode, 20, 3) for name, mode in MODES}
            per_bucket.append({"batch": s5.meta["batch"], "us_per_iteration": us5, "graph_nodes": c5.graph_dispatches()[0],
                               "launches_per_s": {m: len(s5.kernels) / v * 1e6 for m, v in us5.items()},
                               "selection": {"cost_table_us_in_context": clean(cost5), "cost_table_us_alone": clean(alone5), "mode": sel5.tolist(),
                                             "context": f"between graph-indirect replays of the batch-{specs5[j].meta['batch']} chain"}})
            log(f"[bench] config 5 bucket B={s5.meta['batch']}: {us5} selected {sel5.tolist()}")
        seq = bucket_sequence(len(specs5), 1000).tolist()
        seq_us = {}
        for name, mode in MODES + (("selected", pg.SELECTED),):
            for warm in (True, False):
                order = seq[:16] if warm else seq
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for it, b in enumerate(order):
                    ch, x = chains5[b], sets5[b][it % 2]
                    if mode == pg.EAGER:
                        ch.eager(x, stream)
                    elif mode == pg.GRAPH_COPY:
                        ch.replay_copy(x, stream)
                    elif mode == pg.GRAPH_INDIRECT:
                        ch.replay_indirect(x, stream)
                    else:
                        ch.run_selected(per_bucket[b]["selection"]["mode"], x, stream)
                torch.cuda.synchronize()
                seq_us[name] = (time.perf_counter() - t0) / len(order) * 1e6
        configs["5"] = {"workload": "decode chain at batch 1, 2, 4, ..., 128 (one chain and one set of graphs per bucket, shared weights); "
                                    "i.i.d. uniform bucket sequence of 1000 iterations, each bucket in the mode its cost table selects",
                        "kernels": len(specs5[0].kernels), "per_bucket": per_bucket, "us_per_iteration_over_sequence": seq_us,
                        "selected_not_slower_than_best_single_mode": bool(seq_us["selected"] <= 1.02 * min(seq_us[m] for m, _ in MODES))}
        log(f"[bench] config 5 sequence of 1000: {seq_us}")
        for c5 in chains5:
            c5.close()
        del sets5, chains5

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
                   "graph_nodes_per_iteration": dispatches_merged,
                   "step": "one iteration in each of: eager, graph-copy, graph-indirect, selected"},
        "us_per_iteration": us, "us_per_iteration_median": us_median, "us_per_iteration_p90": us_p90,
        "us_per_iteration_one_node_per_kernel": us_plain,
        "launches_per_s": {m: n_k / us[m] * 1e6 for m in us},
        "speedup_vs_eager": {m: us["eager"] / us[m] for m in us},
        "speedup_vs_eager_one_node_per_kernel": {m: us["eager"] / v for m, v in us_plain.items()},
        "graph_node_us": graph_node_us, "eager_launch_us": eager_launch_us,
        "graph_indirect_memcpy_table_us": us_ind_memcpy,
        "graph_indirect_copy_node_in_graph_us": us_ind_graph_memcpy, "graph_indirect_host_table_us": us_ind_host_table,
        "graph_host_node_update_us": us_update, "graph_copy_per_tensor_memcpy_us": us_copy_memcpy,
        "selection": {"cost_table_us": clean(cost), "mode": sel.tolist()},
        "idle_gap_fraction": idle,
        "chain_level_GBps": chain_level, "chain_level_hbm_frac": {m: chain_level[m] / HBM_PEAK for m in us},
        "bytes_refreshed_per_replay": {"graph_copy": chain.stats()["copy_bytes_per_replay"], "graph_indirect": chain.stats()["table_bytes_per_replay"]},
        "capture_ms": capture_s * 1e3,
        "roofline": roofline, "copy_kernel": copy, "configs": configs, "cpu_baseline": cpu,
    }
    chain.close()
    print(json.dumps(result), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
