#!/usr/bin/env python3
"""Benchmark of the CodedReduce hot path on one MI355X.

One "step" is one pass of the whole path over one batch of synthetic input already resident in HBM:
host-drawn straggler mask -> cr_partial_grads -> cr_encode_tree -> cr_decode_root -> cr_gd_update
(issued through cr_gd_run, which enqueues these steps for every mask; the gradient step rides in the decode launch).
Prints ONE JSON line: iterations/s, the roofline of the dominant kernel (measured live with HIP events on the
library's stream, over the timed steps) and the CPU oracle timed on a bounded sample of the same workload.  The other
kernels' averages come from a few more steps after the timed region ("timed_region": false in the "kernels" table).

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0           # MI355X published HBM3E bandwidth
FP32_VECTOR_PEAK_TFLOPS = 157.3   # MI355X, published (packed fp32); 78.6 without packed instructions
KERNEL_NAMES = ["partial_grads", "reduce_pieces", "encode", "decode", "update"]
DESCRIPTIONS = {
    "cfg1": "CR tree L=2 n=3 s=1, linear regression fp32, m=1200 d=100",
    "cfg2": "CR tree L=2 n=4 s=1 (20 workers), linear regression fp32, m=100000 d=10000, GD lr=1e-6, random mask per step",
    "cfg3": "CR tree L=3 n=4 s=1 (84 workers), logistic regression fp32, m=252000 d=4096, random mask per step",
    "cfg4": "aggregation only: CR tree L=2 n=8 s=2 (72 workers), 248 fp32 partition-gradient vectors of length 2^24, encode+decode",
    "cfg5": "CR tree L=3 n=6 s=2 (258 workers), linear regression, X bf16 / fp32 accumulate, m=2064000 d=1024, random mask per step",
    "gc20": "one-layer gradient coding, n=20 s=4 (same data and resiliency as cfg2), linear regression fp32, m=100000 d=10000",
    "umw20": "uncoded master-worker, n=20 s=0 (same data as cfg2), linear regression fp32, m=100000 d=10000",
    "paper84": "the paper's linear-regression experiment: CR tree L=3 n=4 s=1 (84 workers), fp32, m=7644 d=6500, noise N(0,1)",
    "nn12": "aggregation only: CR tree L=2 n=12 s=3 (156 workers), fp32 partition-gradient vectors of length 117706 (network sized), encode+decode",
}


def log(msg: str) -> None:
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def load_traffic(workload: str):
    """HBM bytes per launch of the dominant kernel, from the committed rocprofv3 --pmc summary (None if not measured)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if not os.path.exists(path):
        return None
    with open(path) as f:
        table = json.load(f)
    entry = table.get(workload)
    return None if entry is None else entry.get("bytes_per_launch")


def cpu_baseline(cfg, data, plan_B, w_host, mask, g_gpu, budget_s: float):
    """The oracle as it stands: the CR tree literally (every holder visits its own rows) in fp64 on the host cores."""
    from oracle import cr_tree, gc_code, native

    L, n, s = cfg["L"], cfg["n"], cfg["s"]
    B = gc_code.design_code(n, s, L, 190201981)[0]
    own, _ = cr_tree.cr_allocate(L, n, s, cfg["m"], B)
    slabs = cr_tree.slabs_of(own)
    visits = sum(e - b for _, b, e, _ in slabs)
    native.num_threads()
    t0 = time.perf_counter()
    done_rows = 0
    node_grads = [np.zeros(cfg["d"]) for _ in own]
    complete = True
    for k, (node, b, e, c) in enumerate(slabs):
        node_grads[node] += float(c) * native.segment_gradient(data["X"], data["y"], w_host, b, e, cfg["model"])
        done_rows += e - b
        if time.perf_counter() - t0 > budget_s and k + 1 < len(slabs):
            complete = False
            break
    parity = None
    if complete:
        rows = {}
        _, g = cr_tree.cr_execute(L, n, s, node_grads, mask, lambda T: rows.setdefault(T, gc_code.decoding_row(B, T)))
        parity = float(np.linalg.norm(g_gpu - g) / np.linalg.norm(g))
    elapsed = time.perf_counter() - t0
    its = (done_rows / visits) / elapsed
    sample = (f"one whole CR iteration ({visits} row visits, all {len(slabs)} slabs, tree execute included)" if complete else
              f"first {k + 1} of {len(slabs)} slabs ({done_rows} of {visits} row visits), scaled to one iteration")
    return {"value": its, "unit": "iterations/s", "cores": native.num_threads(), "kind": "oracle", "sample": sample,
            "seconds": elapsed}, parity


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2", choices=sorted(DESCRIPTIONS))
    ap.add_argument("--cpu-budget", type=float, default=20.0, help="seconds of oracle work for the CPU baseline (0 = skip)")
    ap.add_argument("--teams", type=int, default=0, help="stage-1 split: this many equal contiguous ranges")
    ap.add_argument("--cell-rows", type=int, default=0, help="stage-1 split: row cells of this many rows")
    ap.add_argument("--shared-rows", type=int, default=0, help="stage-1 split: cells of at most this many rows shared through LDS")
    ap.add_argument("--calibrate", action="store_true",
                    help="run only a plain 1 GiB elementwise copy kernel a few times (reference for rocprofv3 byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        return 2

    import torch

    import paper_1902_01981_amd as cr
    from cr_inputs import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    if args.calibrate:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)                 # reads 2^30 bytes, writes 2^30 bytes per launch
        torch.cuda.synchronize()
        print(json.dumps({"calibrate": "torch.mul(src, 1.0, out=dst)", "bytes_read": 1 << 30, "bytes_written": 1 << 30, "launches": 5}))
        return 0
    cr.load_library()
    cfg = wl.config(args.workload)
    L, n, s, m, d = cfg["L"], cfg["n"], cfg["s"], cfg["m"], cfg["d"]
    aggregate = cfg["model"] == wl.AGGREGATE_ONLY
    t0 = time.perf_counter()
    plan = cr.cr_plan_ex(L, n, s, m, d, model=cfg["model"], x_dtype=cfg["x_dtype"])
    if args.teams and not aggregate:
        cr.cr_plan_set_split(plan, cr.CR_SPLIT_EQUAL_RANGES, args.teams)
    elif args.cell_rows and not aggregate:
        cr.cr_plan_set_split(plan, cr.CR_SPLIT_ROW_CELLS, args.cell_rows)
    elif args.shared_rows and not aggregate:
        cr.cr_plan_set_split(plan, cr.CR_SPLIT_SHARED_CELLS, args.shared_rows)

    # ---- inputs, generated on the host from the seed and moved to HBM before any timing
    data = None
    if aggregate:
        rb, re_, coef, node = cr.cr_plan_get_segments(plan)
        cuts, member = wl.atoms_of(rb, re_)
        atoms_dev = torch.empty((len(cuts) - 1, d), dtype=torch.float32, device="cuda")
        step_cols = 1 << 22
        for lo in range(0, d, step_cols):
            hi = min(d, lo + step_cols)
            atoms_dev[:, lo:hi] = torch.from_numpy(wl.atom_vectors(cfg["seed"], len(cuts) - 1, lo, hi)).cuda()
        G_dev = torch.empty((len(member), d), dtype=torch.float32, device="cuda")
        for q, idx in enumerate(member):                 # input preparation: redundant copies of a row range must agree
            G_dev[q] = atoms_dev[idx].sum(dim=0)
        del atoms_dev
        w_dev = torch.zeros(d, dtype=torch.float32, device="cuda")
    else:
        data = wl.make_dataset(cfg, threads=min(16, os.cpu_count() or 8))
        X = data["X"]
        X_dev = torch.from_numpy(X.view(np.int16) if X.dtype == np.uint16 else X).cuda()
        y_dev = torch.from_numpy(data["y"]).cuda()
        w_dev = torch.from_numpy(data["w0"]).cuda()
    log(f"inputs ready in {time.perf_counter() - t0:.1f}s")
    ws = cr.Workspace(plan)
    info = ws.info
    g_dev = torch.empty(d, dtype=torch.float32, device="cuda")
    rng = wl.mask_stream(cfg)
    lr = float(cfg["lr"])

    def run(steps):
        # host-drawn straggler masks, then the whole path; for regression workloads the gradient-descent loop is a library call
        # that enqueues its steps without waiting for the device, so the masks of the next batch are drawn while this one runs
        done = 0
        while done < steps:
            batch = min(8, steps - done)
            masks = np.stack([wl.draw_mask(rng, L, n, s) for _ in range(batch)])
            if aggregate:
                for mask in masks:
                    cr.cr_load_partial_grads(plan, G_dev)
                    cr.cr_encode_tree(plan, mask)
                    cr.cr_decode_root(plan, g_dev)
            else:
                cr.cr_gd_run(plan, X_dev, y_dev, w_dev, g_dev, masks, lr)
            done += batch

    dominant = "encode" if aggregate else "partial_grads"

    def read_kernels(into):
        for kid, name in enumerate(KERNEL_NAMES):
            ms, launches, nbytes = cr.cr_profile_read(plan, kid)
            if launches:
                into[name] = {"avg_ms": ms / launches, "launches": launches, "algorithmic_bytes_per_launch": nbytes // launches,
                              "algorithmic_GBps": nbytes / (ms * 1e-3) / 1e9 if ms > 0 else None}

    run(args.warmup)
    torch.cuda.synchronize()
    # timed region: only the dominant kernel is bracketed by events (every bracket costs a few microseconds of device time)
    cr.cr_profile_enable(plan, 1 << KERNEL_NAMES.index(dominant))
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    run(args.steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    kernels = {}
    read_kernels(kernels)
    # the other kernels, from a few more steps outside the timed region with every launch bracketed
    cr.cr_profile_enable(plan, True)
    run(min(args.steps, 10))
    others = {}
    read_kernels(others)
    for name, entry in others.items():
        kernels.setdefault(name, dict(entry, timed_region=False))
    cr.cr_profile_enable(plan, False)
    dk = kernels[dominant]
    roofline = {"bound": "hbm", "kernel": dominant, "achieved": dk["algorithmic_GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": dk["algorithmic_GBps"] / HBM_PEAK_GBPS, "traffic": load_traffic(args.workload),
                "avg_kernel_ms": dk["avg_ms"], "algorithmic_bytes_per_launch": dk["algorithmic_bytes_per_launch"]}
    # yardstick: what a plain streaming read of the same buffer reaches on this device right now
    big = G_dev if aggregate else X_dev
    sink = torch.empty(16384, dtype=torch.float32, device="cuda")
    nbytes = min(big.numel() * big.element_size(), 4 << 30) // 16 * 16
    roofline["stream_read_GBps"] = cr.cr_probe_read_bandwidth(big, nbytes, sink, 10, torch.cuda.current_stream().cuda_stream)
    if roofline["traffic"]:
        # what HBM really moved (rocprofv3 counters of an earlier run of this workload), as a rate over this run's kernel time
        roofline["traffic_GBps"] = roofline["traffic"] / (dk["avg_ms"] * 1e-3) / 1e9
        roofline["traffic_frac_of_stream_read"] = roofline["traffic_GBps"] / roofline["stream_read_GBps"]
    if not aggregate and cfg["x_dtype"] == wl.BF16:
        # bf16 rows: stage 1 is bound by vector-ALU issue (a widening operation and two multiply-adds per element), not by memory;
        # 4 flop per element of X visited against the chip's fp32 vector peak (256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz x 2 flop,
        # x 2 with packed instructions, which this build does not use)
        flops = 4.0 * info.row_visits * d
        achieved = flops / (dk["avg_ms"] * 1e-3) / 1e12
        roofline = dict(roofline, bound="alu", achieved=achieved, peak=FP32_VECTOR_PEAK_TFLOPS, unit="TFLOP/s",
                        frac=achieved / FP32_VECTOR_PEAK_TFLOPS, flops_per_launch=flops,
                        hbm_view={"achieved_GBps": dk["algorithmic_GBps"], "frac": dk["algorithmic_GBps"] / HBM_PEAK_GBPS})

    # ---- CPU baseline: the oracle on the host cores, same inputs, bounded; also a parity check of one more GPU iteration
    baseline, parity = None, None
    if args.cpu_budget > 0 and not aggregate:
        # at the starting model: after many steps w sits at the optimum, where the gradient is the difference of large
        # cancelling terms and a relative error says nothing
        mask = wl.draw_mask(rng, L, n, s)
        w_host = data["w0"]
        w_dev.copy_(torch.from_numpy(w_host))
        cr.cr_partial_grads(plan, X_dev, y_dev, w_dev)
        cr.cr_encode_tree(plan, mask)
        cr.cr_decode_root(plan, g_dev)
        cr.cr_synchronize(plan)
        baseline, parity = cpu_baseline(cfg, data, None, w_host, mask, g_dev.cpu().numpy().astype(np.float64), args.cpu_budget)
        log(f"cpu baseline: {baseline}")

    total_bytes = sum(k["algorithmic_bytes_per_launch"] for k in kernels.values())
    out = {
        "metric": "CR gradient iterations/sec",
        "value": args.steps / elapsed,
        "unit": "iterations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16" if cfg["x_dtype"] == wl.BF16 else "f32",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: {DESCRIPTIONS[args.workload]}", "L": L, "n": n, "s": s, "m": m, "d": d,
                   "workers": info.num_workers, "slabs": info.num_slabs, "row_visits": info.row_visits,
                   "stage1_teams": info.num_teams, "stage1_pieces": info.num_pieces, "code_gamma": info.gamma,
                   "stage1_split": ["equal_ranges", "row_cells", "shared_cells"][info.split_kind] if info.split_kind >= 0 else None,
                   "stage1_split_value": info.split_value, "stage1_team_size": info.stage1_team_size,
                   "stage1_holders_per_workgroup": info.stage1_teams_per_group if info.stage1_staged else 1},
        "algorithmic_GBps_whole_step": total_bytes / (elapsed / args.steps) / 1e9,
        "hbm_frac_whole_step": total_bytes / (elapsed / args.steps) / 1e9 / HBM_PEAK_GBPS,
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": baseline,
        "parity_rel_l2_vs_oracle": parity,
    }
    print(json.dumps(out), flush=True)
    cr.cr_plan_destroy(plan)
    return 0


if __name__ == "__main__":
    sys.exit(main())
