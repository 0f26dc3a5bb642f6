"""Timing report for the benchmark chains other than the one bench.py times:

    python configs_report.py --config 0 1 3 4 5

(config 0 is the launch floor: 512 dependent kernels on 64 elements each; 6 sweeps the batch-1
GEMV over matrix sizes; 7 is the decode chain read literally; 8 the GEMV at every batch size;
9 compares cost tables predicted from a few measured constants with the profiled ones.)

Per chain: capture, slow-path profile -> cost table -> selection, then microseconds per iteration
for eager, graph-copy, graph-indirect and the selected mixture (back-to-back iterations on one
stream, one synchronisation at the end, inputs rotating over distinct allocations), launches per
second, bytes per iteration against the 8 TB/s HBM figure.  One JSON line per config on stdout.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def log(*a):
    print(*a, file=sys.stderr, flush=True)


HBM_PEAK = 8000.0  # GB/s


def chain_bytes(spec) -> int:
    """Algorithmic bytes one iteration moves: every operand read once, every output written once."""
    eb = {"f32": 4, "bf16": 2}
    total = 0
    for k in spec.kernels:
        e = eb[k.dtype]
        if k.op in ("add", "mul"):
            total += (2 * k.n + min(k.m or k.n, k.n)) * e
        elif k.op == "gelu":
            total += 2 * k.n * e
        elif k.op == "rmsnorm":
            total += (2 * k.rows * k.cols + k.cols) * e
        elif k.op == "gemv":
            total += (k.n * k.cols + k.rows * k.cols + k.rows * k.n) * e
        else:
            total += (2 * k.n + 2 * k.channels) * e
    return total


def kernel_bytes(k) -> int:
    e = {"f32": 4, "bf16": 2}[k.dtype]
    if k.op in ("add", "mul"):
        return (2 * k.n + min(k.m or k.n, k.n)) * e
    if k.op == "gelu":
        return 2 * k.n * e
    if k.op == "rmsnorm":
        return (2 * k.rows * k.cols + k.cols) * e
    if k.op == "gemv":
        return (k.n * k.cols + k.rows * k.cols + k.rows * k.n) * e
    return (2 * k.n + 2 * k.channels) * e


def model_cost(spec, c) -> np.ndarray:
    """The cost table predicted from a handful of measured constants instead of profiled per chain:
    launch cost saved against copy cost added (Sec. 3 "Selective CUDA Graphs" argues with exactly
    these terms).  Per kernel the GPU needs a dispatch slot plus its memory time; eager costs the slower of the host's launches and the GPU's slots; a graph
    costs one graph launch plus its nodes, plus either the copy kernel (a node and 2 x the bytes) or
    the table writer (a node) and one dereference per external-reading kernel."""
    n_seg = spec.kernels[-1].segment + 1
    out = np.full((n_seg, 3), np.nan)
    for s in range(n_seg):
        ks = [k for k in spec.kernels if k.segment == s]
        # memory time of a kernel on top of its slot; one that streams from HBM also waits for its first byte
        extra = [kernel_bytes(k) / c["kernel_GBps"] / 1e3 + (c["first_byte_us"] if kernel_bytes(k) >= (1 << 20) else 0.0) for k in ks]
        ext = sorted({r.index for k in ks for r in k.ins if r.kind == "ext"})
        readers = sum(1 for k in ks if any(r.kind == "ext" for r in k.ins))
        copy_bytes = sum(spec.ext[i].nbytes for i in ext)
        out[s, 0] = max(len(ks) * c["eager_launch_us"], len(ks) * c["stream_node_us"] + sum(extra))
        graph = c["graph_launch_us"] + len(ks) * c["graph_node_us"] + sum(extra)
        out[s, 1] = graph + ((c["graph_node_us"] + 2 * copy_bytes / c["copy_GBps"] / 1e3) if ext else 0.0)
        if ext:
            out[s, 2] = graph + c["graph_node_us"] + readers * c["deref_us"]
    return out


def profiler_attached() -> bool:
    """True under rocprofv3 (it preloads its tool library and announces it in the environment)."""
    import os
    keys = ("LD_PRELOAD", "ROCP_TOOL_LIBRARIES", "HSA_TOOLS_LIB", "ROCPROFILER_LIBRARY_CTOR")
    return any("rocprof" in os.environ.get(k, "").lower() for k in keys) or "ROCPROF_OUTPUT_PATH" in os.environ


def time_chain(pg, torch, spec, w_dev, make_sets, iters, warmup, stream, profile_iters=10, merge=True):
    chain = pg.Chain(spec, w_dev)
    chain.set_dispatch_merge(merge)       # off: one graph node per kernel
    t0 = time.time()
    chain.capture(stream)
    cap_ms = (time.time() - t0) * 1e3
    sets = make_sets()
    cost = chain.profile(sets[0], stream, iters=profile_iters, inner=2)
    sel = pg.select(cost)
    us = {}
    for name, mode, modes in (("eager", pg.EAGER, None), ("graph_copy", pg.GRAPH_COPY, None),
                              ("graph_indirect", pg.GRAPH_INDIRECT, None), ("selected", pg.SELECTED, sel)):
        chain.time_loop(mode, sets, warmup, stream, modes)
        us[name] = chain.time_loop(mode, sets, iters, stream, modes)
    st = chain.stats()
    if profiler_attached():
        # the legs below build and destroy further graphs; two counter-collection runs that included them did not complete
        return chain, {"us_per_iteration": us, "capture_ms": cap_ms,
                       "cost_table_us": [[None if not np.isfinite(v) else float(v) for v in row] for row in cost.tolist()],
                       "selected_mode": sel.tolist(), "kernels": st["n_kernels"], "segments": st["n_segments"],
                       "launches_per_s": {m: st["n_kernels"] / v * 1e6 for m, v in us.items()}}
    # the two baselines the refresh designs are measured against: host-side rewrite of the kernel
    # nodes' arguments, and the copy refresh as one device-to-device memcpy per tensor
    chain.time_loop(pg.GRAPH_UPDATE, sets, warmup, stream)
    us["graph_update"] = chain.time_loop(pg.GRAPH_UPDATE, sets, iters, stream)
    chain.set_copy_refresh(pg.COPY_MEMCPY)
    chain.time_loop(pg.GRAPH_COPY, sets, warmup, stream)
    us["graph_copy_per_tensor_memcpy"] = chain.time_loop(pg.GRAPH_COPY, sets, iters, stream)
    chain.set_copy_refresh(pg.COPY_KERNEL)
    # the other ways of getting the pointers to the kernels (the default is a writer kernel)
    if chain.n_ext:
        for name, how in (("graph_indirect_pinned_memcpy", pg.TABLE_MEMCPY), ("graph_indirect_copy_node_in_graph", pg.TABLE_GRAPH_MEMCPY),
                          ("graph_indirect_host_table", pg.TABLE_HOST)):
            chain.set_table_refresh(how)
            chain.time_loop(pg.GRAPH_INDIRECT, sets, warmup, stream)
            us[name] = chain.time_loop(pg.GRAPH_INDIRECT, sets, iters, stream)
        chain.set_table_refresh(pg.TABLE_KERNARG)
    st = chain.stats()
    return chain, {"us_per_iteration": us, "capture_ms": cap_ms,
                   "cost_table_us": [[None if not np.isfinite(v) else float(v) for v in row] for row in cost.tolist()],
                   "selected_mode": sel.tolist(), "kernels": st["n_kernels"], "segments": st["n_segments"],
                   "graph_nodes": chain.graph_dispatches()[0] if merge else st["n_kernels"],
                   "bytes_refreshed_per_replay": {"graph_copy": st["copy_bytes_per_replay"], "graph_indirect": st["table_bytes_per_replay"]},
                   "launches_per_s": {m: st["n_kernels"] / v * 1e6 for m, v in us.items()}}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, nargs="+", default=[1, 3, 4, 5])
    ap.add_argument("--iters", type=int, default=100)
    args = ap.parse_args()
    import torch
    import paper_2503_19779_amd as pg
    from paper_2503_19779_amd.binding import to_device
    from pg_workloads import (elementwise_chain, refresh_stress_chain, large_tensor_chain, decode_buckets, bucket_sequence,
                              make_weights, make_inputs)
    stream = torch.cuda.Stream()

    def host_sets(spec, n):
        return lambda: [[to_device(x) for x in make_inputs(spec, t)] for t in range(n)]

    def device_sets(spec, n):
        def make():
            g = torch.Generator(device="cuda")
            g.manual_seed(spec.seed)
            dt = {"f32": torch.float32, "bf16": torch.bfloat16}
            return [[torch.randn(t.numel, device="cuda", generator=g, dtype=torch.float32).to(dt[t.dtype]) for t in spec.ext] for _ in range(n)]
        return make

    for cfg in args.config:
        if cfg == 6:
            # The batch-1 GEMV kernel away from the launch-bound size: graphs of 24 launches over
            # matrices that together exceed the 256 MB memory-side cache, per-launch time and bandwidth.
            # Shows what part of the 2048 x 2048 figure is the fixed cost of a dispatch slot.
            from pg_workloads import ChainSpec, KernelSpec, TensorSpec, Ref, WEIGHT
            rows_out = []
            for H in (1024, 2048, 4096, 8192, 16384):
                n_mat = max(2, min(24, (640 << 20) // (H * H * 2) + 1))
                mats = [torch.randn(H * H, device="cuda", dtype=torch.float32).mul_(0.02).to(torch.bfloat16) for _ in range(n_mat)]
                vec = torch.randn(H, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                ks = [KernelSpec("gemv", "bf16", 0, (Ref(WEIGHT, s % n_mat), Ref(WEIGHT, n_mat)), H, rows=1, cols=H) for s in range(24)]
                spec = ChainSpec(f"gemv_{H}", ks, [], [TensorSpec("bf16", H)], [TensorSpec("bf16", H * H)] * n_mat + [TensorSpec("bf16", H)], [0])
                chain = pg.Chain(spec, mats + [vec])
                chain.capture(stream)
                chain.time_loop(pg.GRAPH_COPY, [[]], 5, stream)
                us = chain.time_loop(pg.GRAPH_COPY, [[]], 20, stream) / 24
                chain.close()
                b = H * H * 2 + 4 * H
                rows_out.append({"n": H, "cols": H, "matrices": n_mat, "us_per_launch": us, "GBps": b / us / 1e3, "hbm_frac": b / us / 1e3 / HBM_PEAK})
                log(f"[configs] GEMV {H} x {H}: {us:.2f} us per launch, {b / us / 1e3:.0f} GB/s")
                del mats, vec
            print(json.dumps({"config": 6, "workload": "batch-1 bf16 GEMV size sweep, 24 launches per graph", "gemv": rows_out}), flush=True)
            continue
        if cfg == 9:
            # Predicted against profiled cost tables.  The constants come from three small measurements
            # (a do-nothing chain, a one-kernel chain, the large-tensor chain), not from the chains judged.
            from pg_workloads import decode_chain
            floor = elementwise_chain(n_kernels=512, numel=64, dtype="bf16")
            ch = pg.Chain(floor, [])
            ch.capture(stream)
            fx = host_sets(floor, 3)()
            t = {}
            for name, mode in (("eager", pg.EAGER), ("graph", pg.GRAPH_INDIRECT)):
                ch.time_loop(mode, fx, 10, stream)
                t[name] = ch.time_loop(mode, fx, 100, stream)
            ch.close()
            one = elementwise_chain(n_kernels=1, numel=64, dtype="bf16")
            ch = pg.Chain(one, [])
            ch.capture(stream)
            ox = host_sets(one, 3)()
            one_cost = ch.profile(ox[0], stream, iters=21, inner=1)     # launch + run + synchronise, once
            ch.close()
            big = large_tensor_chain()
            wb = [to_device(a) for a in make_weights(big)]
            ch = pg.Chain(big, wb)
            bx = device_sets(big, 1)()[0]
            d = ch.time_kernels(bx, stream)
            d = ch.time_kernels(bx, stream)
            ch.close()
            stress = refresh_stress_chain()
            ws = [to_device(a) for a in make_weights(stress)]
            ch = pg.Chain(stress, ws)
            ch.capture(stream)
            sx = device_sets(stress, 2)()
            cu = np.array([ch.time_refresh_copy(sx[i % 2], stream) for i in range(13)][3:])
            ch.close()
            del sx, ws
            node = t["graph"] / 512
            consts = {"eager_launch_us": t["eager"] / 512, "graph_node_us": node, "stream_node_us": node,
                      "graph_launch_us": max(0.0, float(one_cost[0, 2] - one_cost[0, 0])),
                      "first_byte_us": 0.4, "kernel_GBps": 2 * big.ext[0].nbytes / float(np.median(d)) / 1e3,
                      "copy_GBps": 2 * stress.ext_bytes() / float(cu.mean()) / 1e3, "deref_us": 0.08}
            log(f"[configs] model constants: {consts}")
            rows_out = []
            for name, spec, mk in (("config 1", elementwise_chain(), "host"), ("config 2", decode_chain(), "dev"),
                                   ("config 3", stress, "dev"), ("config 4", big, "dev"), ("config 5, B=128", decode_chain(batch=128), "dev")):
                w = [to_device(a) for a in make_weights(spec)]
                ch = pg.Chain(spec, w)
                ch.capture(stream)
                x = (host_sets(spec, 1) if mk == "host" else device_sets(spec, 1))()[0]
                prof = ch.profile(x, stream, iters=9, inner=2)
                ch.close()
                pred = model_cost(spec, consts)
                sel_p, sel_m = pg.select(prof), pg.select(pred)
                rows_out.append({"chain": name, "profiled_us": [[None if not np.isfinite(v) else round(float(v), 1) for v in r] for r in prof.tolist()],
                                 "model_us": [[None if not np.isfinite(v) else round(float(v), 1) for v in r] for r in pred.tolist()],
                                 "selected_from_profile": sel_p.tolist(), "selected_from_model": sel_m.tolist()})
                log(f"[configs] {name}: profiled {rows_out[-1]['profiled_us']} -> {sel_p.tolist()}; model {rows_out[-1]['model_us']} -> {sel_m.tolist()}")
                del w, x
            print(json.dumps({"config": 9, "workload": "cost tables predicted from measured constants against profiled ones", "constants": consts, "chains": rows_out}), flush=True)
            continue
        if cfg == 8:
            # The batched GEMV alone at every bucket size: graphs of the decode chain's 120 launches over
            # its 120 weight matrices (1 GB, so every launch streams its weights from HBM).
            from pg_workloads import ChainSpec, KernelSpec, TensorSpec, Ref, WEIGHT
            H = 2048
            mats = [torch.randn(H * H, device="cuda", dtype=torch.float32).mul_(0.02).to(torch.bfloat16) for _ in range(120)]
            rows_out = []
            for B in (1, 2, 4, 8, 16, 32, 64, 128):
                act = torch.randn(B * H, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                ks = [KernelSpec("gemv", "bf16", 0, (Ref(WEIGHT, s), Ref(WEIGHT, 120)), H, rows=B, cols=H) for s in range(120)]
                spec = ChainSpec(f"gemv_b{B}", ks, [], [TensorSpec("bf16", B * H)], [TensorSpec("bf16", H * H)] * 120 + [TensorSpec("bf16", B * H)], [0])
                chain = pg.Chain(spec, mats + [act])
                chain.capture(stream)
                chain.time_loop(pg.GRAPH_COPY, [[]], 5, stream)
                us = chain.time_loop(pg.GRAPH_COPY, [[]], 20, stream) / 120
                chain.close()
                b = H * H * 2 + 2 * B * H * 2
                rows_out.append({"batch": B, "us_per_launch": us, "GBps": b / us / 1e3, "TFLOPs": 2.0 * B * H * H / us / 1e6})
                log(f"[configs] GEMV 2048 x 2048, batch {B}: {us:.2f} us per launch, {b / us / 1e3:.0f} GB/s, {2.0 * B * H * H / us / 1e6:.1f} TFLOP/s")
            print(json.dumps({"config": 8, "workload": "bf16 GEMV 2048 x 2048 at batch 1..128, 120 launches per graph over 120 matrices", "gemv": rows_out}), flush=True)
            continue
        if cfg == 7:
            # the decode chain read literally: 24 layers x one (RMSNorm, GEMV, GELU, add) = 96 kernels,
            # with 24 external inputs (23 input adds): 119 kernels per iteration
            from pg_workloads import decode_chain
            spec = decode_chain(blocks_per_layer=1, n_ext=24)
            w = [to_device(a) for a in make_weights(spec)]
            chain, r = time_chain(pg, torch, spec, w, device_sets(spec, 3), args.iters, 10, stream)
        elif cfg == 0:
            # launch floor: 512 dependent kernels on 64 elements each, so the time per kernel is the
            # cost of dispatching one dependent kernel (host launch for eager, graph node for replay)
            spec = elementwise_chain(n_kernels=512, numel=64, dtype="bf16")
            chain, r = time_chain(pg, torch, spec, [], host_sets(spec, 3), args.iters, 10, stream, merge=False)
            r["us_per_kernel"] = {m: v / len(spec.kernels) for m, v in r["us_per_iteration"].items()}
        elif cfg == 1:
            spec = elementwise_chain()
            chain, r = time_chain(pg, torch, spec, [], host_sets(spec, 3), args.iters, 10, stream)
        elif cfg == 3:
            spec = refresh_stress_chain()
            w = [to_device(a) for a in make_weights(spec)]
            chain, r = time_chain(pg, torch, spec, w, device_sets(spec, 2), min(args.iters, 30), 3, stream)
            sets = device_sets(spec, 2)()
            cu = np.array([chain.time_refresh_copy(sets[i % 2], stream) for i in range(23)][3:])
            r["copy_kernel"] = {"us": float(cu.mean()), "GBps": 2 * spec.ext_bytes() / float(cu.mean()) / 1e3,
                                "hbm_frac": 2 * spec.ext_bytes() / float(cu.mean()) / 1e3 / HBM_PEAK}
        elif cfg == 4:
            spec = large_tensor_chain()
            w = [to_device(a) for a in make_weights(spec)]
            chain, r = time_chain(pg, torch, spec, w, device_sets(spec, 3), min(args.iters, 30), 3, stream)
            x = device_sets(spec, 1)()[0]
            d = chain.time_kernels(x, stream)
            d = chain.time_kernels(x, stream)
            r["kernel_us"] = float(np.median(d))
            r["kernel_GBps"] = 2 * spec.ext[0].nbytes / float(np.median(d)) / 1e3
        elif cfg == 5:
            specs = decode_buckets()
            w = [to_device(a) for a in make_weights(specs[0])]
            per_bucket, chains, sets = [], [], []
            for spec in specs:
                chain, r = time_chain(pg, torch, spec, w, device_sets(spec, 2), 20, 3, stream, profile_iters=5)
                per_bucket.append({"batch": spec.meta["batch"], **r,
                                   "algorithmic_GBps": {m: chain_bytes(spec) / v / 1e3 for m, v in r["us_per_iteration"].items()}})
                chains.append(chain)
                sets.append(device_sets(spec, 2)())
                log(f"[configs] bucket B={spec.meta['batch']}: {r['us_per_iteration']} selected {r['selected_mode']}")
            seq = bucket_sequence(len(specs), 1000)
            out = {}
            for name, mode in (("eager", pg.EAGER), ("graph_copy", pg.GRAPH_COPY), ("graph_indirect", pg.GRAPH_INDIRECT), ("selected", pg.SELECTED)):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for it, b in enumerate(seq.tolist()):
                    ch, x = chains[b], sets[b][it % 2]
                    if mode == pg.EAGER:
                        ch.eager(x, stream)
                    elif mode == pg.GRAPH_COPY:
                        ch.replay_copy(x, stream)
                    elif mode == pg.GRAPH_INDIRECT:
                        ch.replay_indirect(x, stream)
                    else:
                        ch.run_selected(per_bucket[b]["selected_mode"], x, stream)
                torch.cuda.synchronize()
                out[name] = (time.perf_counter() - t0) / len(seq) * 1e6
            print(json.dumps({"config": 5, "workload": "decode chain, 8 batch-size buckets 1..128, random bucket sequence of 1000 iterations",
                              "us_per_iteration_over_sequence": out, "per_bucket": per_bucket}), flush=True)
            for ch in chains:
                ch.close()
            continue
        else:
            log(f"config {cfg}: use bench.py for the decode chain")
            continue
        b = chain_bytes(spec)
        r.update({"config": cfg, "workload": spec.name, "algorithmic_bytes_per_iteration": b,
                  "algorithmic_GBps": {m: b / v / 1e3 for m, v in r["us_per_iteration"].items()},
                  "hbm_floor_us": b / HBM_PEAK / 1e3})
        log(f"[configs] config {cfg}: {r['us_per_iteration']} selected {r['selected_mode']}")
        print(json.dumps(r), flush=True)
        chain.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
