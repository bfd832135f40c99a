#!/usr/bin/env python3
"""Benchmark of the property-aware matrix-chain evaluator on one MI355X.

A step is one whole chain evaluation (every kernel of the plan) on seeded synthetic factors
that already sit in HBM.  The default workload is the single lowerTri * general product with
n = 4096, whose useful work is counted as n^3 FLOP; the other workloads are reachable with
--workload.  Prints ONE JSON line.

The metric follows the paper's protocol for its only experiment (Sec. 4: f32 operands, the
minimum over single runs is logged as min_ms next to the mean that `value` is computed from).
"""
import argparse
import json
import os
import sys
import time

import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import synthetic_chains as sc  # noqa: E402

F32_MFMA_PEAK_TFLOPS = 157.3        # 256 CUs x 256 FLOP/clk x 2.4 GHz
HBM_PEAK_GBS = 8000.0

# HBM-side bytes per launch of the dominant kernel, from two counter passes of this very
# program (rocprofv3 --pmc FETCH_SIZE, then WRITE_SIZE; KiB per dispatch), each scaled by what
# the same counter reads for the copy8192 workload, whose traffic is known.  The figures hold
# for the kernel sources they were taken with: `sources` is the digest kernel_sources_digest()
# gave then, and any other digest turns the field into null.
# (scale factors of that calibration: FETCH_SIZE x 1.9997, WRITE_SIZE x 1.0000; all launches of one step summed)
MEASURED_TRAFFIC = {
    "trmm4096": {"fetch_bytes": 449996754, "write_bytes": 67108884, "sources": "96752c54a085d577"},
    "general5": {"fetch_bytes": 123315758, "write_bytes": 87158912, "sources": "96752c54a085d577"},
    "general5_left_to_right": {"fetch_bytes": 1876441223, "write_bytes": 527158985, "sources": "96752c54a085d577"},
    "mixed5": {"fetch_bytes": 3701566704, "write_bytes": 100968522, "sources": "96752c54a085d577"},
    "mixed5_tri_intermediate": {"fetch_bytes": 7936007970, "write_bytes": 201653276, "sources": "96752c54a085d577"},
    "mixed5_left_to_right": {"fetch_bytes": 15400234152, "write_bytes": 436568715, "sources": "96752c54a085d577"},
    "batched32": {"fetch_bytes": 50368472, "write_bytes": 16777216, "sources": "96752c54a085d577"},
    "copy8192": {"fetch_bytes": 268435456, "write_bytes": 268435456, "sources": "96752c54a085d577"},
}

# forced parenthesisations of the mixed-property chain (the planner's own tree never forms
# L1*L2, so two trees that do are timed as well)
WORKLOADS = {
    "trmm4096": ("trmm4096", None),
    "general5": ("general5", None),
    "general5_left_to_right": ("general5", [3, 2, 1, 0]),
    "mixed5": ("mixed5", None),
    "mixed5_tri_intermediate": ("mixed5", [2, 0, 3]),
    "mixed5_left_to_right": ("mixed5", [3, 2, 0]),
    "batched32": ("batched32", None),
    # plain copy of a general 8192x8192 matrix (a chain with one factor): the known-size kernel
    # that HBM counters are calibrated against
    "copy8192": ("copy8192", None),
}

sc.CONFIGS["copy8192"] = sc.ChainConfig("copy8192", 9, (8192, 8192), (sc.GENERAL,))


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    # what decides the kernels and their launch geometry; the planner's host code is left out
    names = ("batched_kernel.h", "eval.hip", "product_kernel.h", "schedule.h")
    for path in (os.path.join(ROOT, "paper_2208_10391_amd", "csrc", n) for n in names):
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload):
    """(bytes per step, {fetch, write}) or (None, None) when the kernels have changed since."""
    m = MEASURED_TRAFFIC.get(workload)
    if not m or m["sources"] != kernel_sources_digest():
        return None, None
    return m["fetch_bytes"] + m["write_bytes"], {"fetch_bytes": m["fetch_bytes"], "write_bytes": m["write_bytes"]}


def useful_flop(name, plan, cfg):
    if name == "trmm4096":
        return float(cfg.dims[0]) ** 3            # the non-zero half of 2*n^3
    return 2.0 * plan.cost_mults * max(cfg.batch, 1)


def algorithmic_bytes(cfg):
    """Bytes that must cross HBM once: the structural part of every factor plus the result."""
    total = 0
    for t, p in enumerate(cfg.props):
        r, c = cfg.dims[t], cfg.dims[t + 1]
        if p == sc.IDENTITY:
            continue
        total += (r * (r + 1) // 2 if p in (sc.LOWER_TRI, sc.UPPER_TRI) else r * c) * 4
    total += cfg.dims[0] * cfg.dims[-1] * 4
    return total * max(cfg.batch, 1)


def cpu_baseline(cfg, host, splits, flop):
    """The oracle as it stands, timed on the host cores along the same tree (f64, loops
    restricted by the properties).  For the batched workload a bounded number of chains."""
    import numpy as np
    import oracle
    np_f = [None if f is None else f.numpy() for f in host]
    if cfg.batch:
        chains = min(cfg.batch, 512)
        t0 = time.perf_counter()
        for b in range(chains):
            oracle.eval_plan(cfg.dims, cfg.props, [None if f is None else f[b] for f in np_f], splits)
        dt = time.perf_counter() - t0
        done = flop * chains / cfg.batch
        sample = "%d of %d chains, same tree" % (chains, cfg.batch)
    else:
        # bound the work to roughly 70 GFLOP by narrowing the last factor to a column panel
        full_cols = cfg.dims[-1]
        cols = full_cols
        while flop * cols / full_cols > 7.5e10 and cols > 64 and cfg.props[-1] == sc.GENERAL:
            cols //= 2
        dims = list(cfg.dims[:-1]) + [cols]
        if cols != full_cols:
            np_f = np_f[:-1] + [np.ascontiguousarray(np_f[-1][:, :cols])]
            mults, _ = oracle.tree_cost(dims, cfg.props, splits)
            done = 2.0 * mults
            sample = "same tree, last factor narrowed to its first %d of %d columns" % (cols, full_cols)
        else:
            done = flop
            sample = "the whole workload, same tree, one run"
        t0 = time.perf_counter()
        oracle.eval_plan(dims, cfg.props, np_f, splits)
        dt = time.perf_counter() - t0
    return {"value": done / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": sample, "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=100)
    ap.add_argument("--workload", default="trmm4096", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this evaluator runs on one GPU; --gpus %d is not supported "
                 "(no sharding or collectives are part of it)" % args.gpus)
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    import paper_2208_10391_amd as mom   # fails loudly when libmom.so is missing

    cfg_name, splits = WORKLOADS[args.workload]
    cfg = sc.CONFIGS[cfg_name]
    host = sc.make_config(cfg_name)
    plan = mom.mom_chain_plan(cfg.dims, cfg.props) if splits is None else \
        mom.mom_plan_from_splits(cfg.dims, cfg.props, splits)
    dev = [None if f is None else f.cuda() for f in host]
    rows, cols, _ = plan.result
    # arguments are marshalled once; a step is one call of the C entry point
    if cfg.batch:
        out = torch.empty((cfg.batch, rows, cols), dtype=torch.float32, device="cuda")
        step = mom.bind_chain_eval_batched(plan, dev, out=out)
    else:
        out = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
        step = mom.bind_chain_eval(plan, dev, out=out, workspace=ws)

    flop = useful_flop(args.workload, plan, cfg)

    # The clocks take some tens of launches to settle, hence the long default warm-up.  The
    # event pair sits on the launch stream (the library enqueues on torch's current stream) and
    # brackets the timed region: device time per step, which feeds the roofline.
    for _ in range(args.warmup):
        step()
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    first.record()
    for _ in range(args.steps):
        step()
    last.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    avg_ms = first.elapsed_time(last) / args.steps

    # one evaluation at a time: minimum and median (the paper logs the minimum of its runs)
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(min(args.steps, 50))]
    for s, e in events:
        s.record()
        step()
        e.record()
    torch.cuda.synchronize()
    per = sorted(s.elapsed_time(e) for s, e in events)

    value = flop / (ms_per_step * 1e-3) / 1e9
    traffic, traffic_detail = measured_traffic(args.workload)

    # what the matrix pipes of this very GPU sustain with no memory traffic (register-only MFMA
    # loop of the library), best of five launches: reported beside the nominal peak
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    probe_tflops = 0.0
    for _ in range(8):
        ps, pe = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ps.record()
        probe_flop = mom.mom_probe_mfma_peak(2000, sink)
        pe.record()
        torch.cuda.synchronize()
        probe_tflops = max(probe_tflops, probe_flop / (ps.elapsed_time(pe) * 1e-3) / 1e12)
    if cfg.batch or args.workload == "copy8192":   # HBM-bound: factors in and result out, once
        byts = algorithmic_bytes(cfg)
        ach = byts / (avg_ms * 1e-3) / 1e9
        roofline = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                    "frac": ach / HBM_PEAK_GBS, "traffic": traffic, "traffic_detail": traffic_detail,
                    "kernel": "batched_chain3_right_kernel" if cfg.batch else "copy_structure_kernel",
                    "algorithmic_bytes_per_launch": byts}
    else:
        ach = flop / (avg_ms * 1e-3) / 1e12
        roofline = {"bound": "mfma", "achieved": ach, "peak": F32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / F32_MFMA_PEAK_TFLOPS, "traffic": traffic, "traffic_detail": traffic_detail,
                    "kernel": "product_kernel", "launches_per_step": mom.mom_plan_num_products(plan),
                    "algorithmic_flop_per_step": flop, "measured_peak": probe_tflops,
                    "frac_of_measured_peak": ach / probe_tflops}
    line = {
        "metric": "useful GFLOP/s per chain eval (f32)",
        "value": value,
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "dims": list(cfg.dims), "props": list(cfg.props),
                   "batch": cfg.batch, "plan": plan.string, "mults": plan.cost_mults,
                   "useful_flop": flop},
        "pct_of_f32_mfma_peak": 100.0 * value / 1e3 / F32_MFMA_PEAK_TFLOPS,
        "device_ms_per_step": avg_ms,
        "min_ms": per[0],
        "median_ms": per[len(per) // 2],
        "roofline": roofline,
    }
    if not args.no_cpu_baseline and args.workload != "copy8192":
        line["cpu_baseline"] = cpu_baseline(cfg, host, plan.splits, flop)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
