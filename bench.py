#!/usr/bin/env python3
"""Benchmark of the property-aware matrix-chain evaluator on one MI355X.

A step is one whole chain evaluation (every kernel of the plan) on seeded synthetic factors
that already sit in HBM.  The headline workload is the mixed-property chain L1*I*L2*U*G with
n = 8192 evaluated along the planner's tree; the other workloads are timed in the same run and
reported under "configs" of the one JSON line that is printed (--workload picks another
headline, --no-configs leaves the others out).

Protocol: the paper's only experiment (Sec. 4) uses f32 operands and logs the minimum over
single runs; here `value` comes from the mean over the timed steps, and min_ms / median_ms of
single evaluations are reported next to it.  Before any timing the workload's own launches run
until the shader clock has settled (settle_ms), whatever --warmup says.
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
COUNTERS_FILE = os.path.join(ROOT, "bench_counters.json")   # written by bench_counters.py

# workload -> (input configuration, forced preorder splits or None for the planner's tree)
WORKLOADS = {
    "mixed5": ("mixed5", None),
    "mixed5_tri_intermediate": ("mixed5", [2, 0, 3]),       # forms L1*L2 as a lowerTri temporary
    "mixed5_left_to_right": ("mixed5", [3, 2, 0]),
    "trmm4096": ("trmm4096", None),
    "trmm4096_transposed": ("trmm4096_transposed", None),   # both operands read from transposed buffers
    "general5": ("general5", None),
    "general5_left_to_right": ("general5", [3, 2, 1, 0]),   # the tree Sec. 4 would start from
    "batched32": ("batched32", None),
    # a chain on which the two planning objectives part: the multiplication-optimal tree, and the
    # tree of the time objective (timed with its own, larger, multiplication count as tree_flop)
    "gggl256_min_mults": ("gggl256", None),
    "gggl256_min_time": ("gggl256", "min_time"),
    # element-wise passes, bound by HBM: a diagonal times a general matrix (one scaling launch)
    # and the sum of three general matrices (an equation whose addends are plain matrices)
    "dscale8192": ("dscale8192", None),
    "add3_8192": ("add3_8192", "equation"),
    # plain copy of a general 8192x8192 matrix (a chain with one factor): the known-size kernel
    # that the HBM counters are calibrated against
    "copy8192": ("copy8192", None),
}
ELEMENTWISE_KERNEL = {"copy8192": "copy_structure_kernel", "dscale8192": "diag_scale_kernel", "add3_8192": "add_terms_kernel"}
SIDE_WORKLOADS = ["trmm4096", "trmm4096_transposed", "general5", "general5_left_to_right", "mixed5_tri_intermediate",
                  "mixed5_left_to_right", "batched32", "gggl256_min_mults", "gggl256_min_time", "dscale8192", "add3_8192"]

sc.CONFIGS["copy8192"] = sc.ChainConfig("copy8192", 9, (8192, 8192), (sc.GENERAL,))
sc.CONFIGS["dscale8192"] = sc.ChainConfig("dscale8192", 10, (8192, 8192, 8192), (sc.DIAGONAL, sc.GENERAL))
# three addends, each a chain of one general 8192 x 8192 factor (dims / props list the addends one after the other)
sc.CONFIGS["add3_8192"] = sc.ChainConfig("add3_8192", 11, (8192, 8192), (sc.GENERAL,))
ADD3_TERMS = 3


def kernel_sources_digest():
    import hashlib
    h = hashlib.sha256()
    # what decides the kernels and their launch geometry; the planner's host code is left out
    names = ("batched_kernel.h", "eval.hip", "launch_params.h", "product_kernel.h", "product_variant.h", "skinny_pair_kernel.h",
             "schedule.h", "small_kernels.h")
    for path in (os.path.join(ROOT, "paper_2208_10391_amd", "csrc", n) for n in names):
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_counters(workload):
    """HBM-side bytes per step and matrix-pipe utilisation from the committed counter passes
    (bench_counters.json); None for whatever was taken with other kernel sources than today's."""
    try:
        with open(COUNTERS_FILE) as f:
            table = json.load(f)
    except OSError:
        return None, None, None
    m = table.get("workloads", {}).get(workload)
    if not m or table.get("sources") != kernel_sources_digest():
        return None, None, None
    traffic = detail = None
    if m.get("fetch_bytes") is not None and m.get("write_bytes") is not None:
        traffic = m["fetch_bytes"] + m["write_bytes"]
        detail = {"fetch_bytes": m["fetch_bytes"], "write_bytes": m["write_bytes"]}
    return traffic, detail, m.get("mfma_busy")


def structural_bytes(rows, cols, prop):
    if prop in (sc.LOWER_TRI, sc.UPPER_TRI):
        return rows * (rows + 1) // 2 * 4
    if prop == sc.DIAGONAL:
        return rows * 4
    return rows * cols * 4


def algorithmic_bytes(cfg, result_prop):
    """Bytes that must cross HBM once: the structural part of every factor plus the result."""
    total = 0
    for t, p in enumerate(cfg.props):
        if p != sc.IDENTITY:
            total += structural_bytes(cfg.dims[t], cfg.dims[t + 1], p)      # (a transpose has as many)
    total += structural_bytes(cfg.dims[0], cfg.dims[-1], result_prop)
    return total * max(cfg.batch, 1)


def step_bound_ms(mom, plan):
    """Nominal floor of one evaluation, launch structure taken as given: for every binary
    product the larger of its useful FLOP at the f32 MFMA peak and its structural operand and
    result bytes at the HBM peak; products are summed (they depend on each other level by level)."""
    total = 0.0
    parts = []
    for i in range(mom.mom_plan_num_products(plan)):
        pr = mom.mom_plan_product(plan, i)
        m, k, n = pr["shape"]
        pa, pb, pc = pr["props"]
        flop = 2.0 * pr["mults"]
        byts = structural_bytes(m, k, pa) + structural_bytes(k, n, pb) + structural_bytes(m, n, pc)
        t_mfma, t_hbm = flop / (F32_MFMA_PEAK_TFLOPS * 1e12), byts / (HBM_PEAK_GBS * 1e9)
        total += max(t_mfma, t_hbm)
        parts.append({"shape": [m, k, n], "props": [pa, pb, pc], "level": pr["level"],
                      "mfma_us": t_mfma * 1e6, "hbm_us": t_hbm * 1e6})
    return total * 1e3, parts


def settle(step, min_ms=60.0, max_ms=3000.0):
    """Run the workload's own launches until the clocks have settled: windows of a few
    milliseconds each, until at least min_ms have passed and two consecutive windows agree
    within 2 % (or max_ms).  Returns (ms spent, windows, ms per step of the last window)."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record(); step(); b.record()
    torch.cuda.synchronize()
    per_window = max(4, int(6.0 / max(a.elapsed_time(b), 1e-3)))
    spent, windows, last, prev = 0.0, 0, None, None
    t0 = time.perf_counter()
    while True:
        a.record()
        for _ in range(per_window):
            step()
        b.record()
        torch.cuda.synchronize()
        prev, last = last, a.elapsed_time(b) / per_window
        windows += 1
        spent = (time.perf_counter() - t0) * 1e3
        agree = prev is not None and abs(last - prev) <= 0.02 * prev
        if (spent >= min_ms and agree) or spent >= max_ms:
            return spent, windows, last


def time_steps(step, steps, warmup):
    """settle, warm up, then `steps` calls between events and between host clocks, then single calls."""
    settle_ms, settle_windows, _ = settle(step)
    for _ in range(warmup):
        step()
    first, last = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    first.record()
    for _ in range(steps):
        step()
    last.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / steps
    dev_ms = first.elapsed_time(last) / steps
    events = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(min(steps, 50))]
    for s, e in events:
        s.record()
        step()
        e.record()
    torch.cuda.synchronize()
    per = sorted(s.elapsed_time(e) for s, e in events)
    return {"ms_per_step": wall_ms, "device_ms_per_step": dev_ms, "min_ms": per[0], "median_ms": per[len(per) // 2],
            "settle_ms": settle_ms, "settle_windows": settle_windows}


def measure_sum(mom, workload, cfg, steps, warmup):
    """The sum of ADD3_TERMS general matrices through mom_equation_eval: one element-wise launch,
    every addend read once and the sum written once."""
    rows, cols = cfg.dims
    terms = [sc.make_factor(rows, cols, sc.GENERAL, sc.factor_seed(cfg.number, t)).cuda() for t in range(ADD3_TERMS)]
    eq = mom.mom_equation_plan([((rows, cols), (sc.GENERAL,), None)] * ADD3_TERMS)
    out = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
    step = mom.bind_equation_eval(eq, [[t] for t in terms], out=out)
    rec = {"workload": workload, "plan": " + ".join("(%d)" % t for t in range(ADD3_TERMS)), "mults": 0, "useful_flop": 0.0,
           "tree_flop": 0.0, "launches_per_step": 1, "value": 0.0}
    rec.update(time_steps(step, steps, warmup))
    traffic, traffic_detail, _ = measured_counters(workload)
    byts = (ADD3_TERMS + 1) * rows * cols * 4
    ach = byts / (rec["device_ms_per_step"] * 1e-3) / 1e9
    rec["roofline"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": ach / HBM_PEAK_GBS,
                       "traffic": traffic, "traffic_detail": traffic_detail, "kernel": ELEMENTWISE_KERNEL[workload],
                       "algorithmic_bytes_per_launch": byts, "mfma_busy": None}
    return rec


def measure(mom, workload, steps, warmup, want_cpu_baseline):
    cfg_name, splits = WORKLOADS[workload]
    cfg = sc.CONFIGS[cfg_name]
    if splits == "equation":
        return measure_sum(mom, workload, cfg, steps, warmup), cfg, None
    host = sc.make_config(cfg_name)
    trans = list(cfg.trans) if cfg.trans else None
    best = mom.mom_chain_plan(cfg.dims, cfg.props, trans=trans)    # the planner's tree
    if splits == "min_time":
        plan = mom.mom_chain_plan_ex(cfg.dims, cfg.props, trans, objective=mom.MOM_PLAN_MIN_TIME)
    else:
        plan = best if splits is None else mom.mom_plan_from_splits(cfg.dims, cfg.props, splits, trans=trans)
    dev = [None if f is None else f.cuda() for f in host]
    rows, cols, rprop = plan.result
    # arguments are marshalled once; a step is one call of the C entry point
    if cfg.batch:
        out = torch.empty((cfg.batch, rows, cols), dtype=torch.float32, device="cuda")
        step = mom.bind_chain_eval_batched(plan, dev, out=out)
    else:
        out = torch.empty((rows, cols), dtype=torch.float32, device="cuda")
        ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device="cuda")
        step = mom.bind_chain_eval(plan, dev, out=out, workspace=ws)

    # useful work: what the planner's tree needs (the single TRMM is counted as n^3, the
    # non-zero half of 2*n^3, as its workload definition says); tree_flop: what THIS tree
    # executes usefully, which is more for a forced tree
    batch = max(cfg.batch, 1)
    useful = float(cfg.dims[0]) ** 3 if cfg_name.startswith("trmm4096") else 2.0 * best.cost_mults * batch
    tree_flop = useful if splits is None else 2.0 * plan.cost_mults * batch

    # The event pair sits on the launch stream (the library enqueues on torch's current stream)
    # and brackets the timed region: device time per step, which feeds the roofline; then one
    # evaluation at a time: minimum and median (the paper logs the minimum of its runs)
    timing = time_steps(step, steps, warmup)
    wall_ms, dev_ms = timing["ms_per_step"], timing["device_ms_per_step"]

    traffic, traffic_detail, mfma_busy = measured_counters(workload)
    launches = 1 if cfg.batch else mom.mom_plan_num_launches(plan)      # a whole batch is one launch
    rec = {"workload": workload, "plan": plan.string, "mults": plan.cost_mults, "useful_flop": useful,
           "tree_flop": tree_flop, "launches_per_step": launches,
           "value": useful / (wall_ms * 1e-3) / 1e9}
    rec.update(timing)
    if cfg.batch or workload in ELEMENTWISE_KERNEL:       # HBM-bound: factors in and result out, once
        byts = algorithmic_bytes(cfg, rprop)
        ach = byts / (dev_ms * 1e-3) / 1e9
        rec["roofline"] = {"bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                           "frac": ach / HBM_PEAK_GBS, "traffic": traffic, "traffic_detail": traffic_detail,
                           "kernel": "batched_chain3_right_kernel" if cfg.batch else ELEMENTWISE_KERNEL[workload],
                           "algorithmic_bytes_per_launch": byts, "mfma_busy": mfma_busy}
    else:
        # dominant kernel: product_kernel; a step's product launches are taken together (their
        # useful FLOP summed, divided by the device time of the step)
        ach = tree_flop / (dev_ms * 1e-3) / 1e12
        bound_ms, parts = step_bound_ms(mom, plan)
        rec["roofline"] = {"bound": "mfma", "achieved": ach, "peak": F32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                           "frac": ach / F32_MFMA_PEAK_TFLOPS, "traffic": traffic, "traffic_detail": traffic_detail,
                           "kernel": "product_kernel", "algorithmic_flop_per_step": tree_flop,
                           "algorithmic_bytes_per_step": algorithmic_bytes(cfg, rprop),
                           "mfma_busy": mfma_busy, "step_bound_ms": bound_ms,
                           "frac_of_step_bound": bound_ms / dev_ms, "step_bound_parts": parts}
        if splits is not None:                    # against the work the planner's tree would need
            rec["roofline"]["frac_vs_planned_tree"] = useful / (dev_ms * 1e-3) / 1e12 / F32_MFMA_PEAK_TFLOPS
    if want_cpu_baseline:
        rec["cpu_baseline"] = cpu_baseline(cfg, host, plan.splits, tree_flop, trans)
    return rec, cfg, plan


def cpu_baseline(cfg, host, splits, flop, trans=None):
    """The oracle as it stands, timed on the host cores along the same tree (f64, loops
    restricted by the properties).  For the batched workload a bounded number of chains."""
    import numpy as np
    import oracle
    np_f = [None if f is None else f.numpy() for f in host]
    if cfg.batch:
        chains = min(cfg.batch, 512)
        t0 = time.perf_counter()
        for b in range(chains):
            oracle.eval_plan(cfg.dims, cfg.props, [None if f is None else f[b] for f in np_f], splits, trans=trans)
        dt = time.perf_counter() - t0
        done = flop * chains / cfg.batch
        sample = "%d of %d chains, same tree" % (chains, cfg.batch)
    else:
        # bound the work to roughly 250 GFLOP by narrowing the last factor to a column panel
        full_cols = cfg.dims[-1]
        cols = full_cols
        while flop * cols / full_cols > 2.5e11 and cols > 64 and cfg.props[-1] == sc.GENERAL and not trans:
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
        oracle.eval_plan(dims, cfg.props, np_f, splits, trans=trans)
        dt = time.perf_counter() - t0
    return {"value": done / dt / 1e9, "unit": "GFLOP/s", "cores": oracle.max_threads(), "kind": "oracle",
            "sample": sample, "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="mixed5", choices=sorted(WORKLOADS))
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-configs", action="store_true", help="time the headline workload only")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this evaluator runs on one GPU; --gpus %d is not supported "
                 "(no sharding or collectives are part of it)" % args.gpus)
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    import paper_2208_10391_amd as mom   # fails loudly when libmom.so is missing
    mom.mom_init()

    head, cfg, plan = measure(mom, args.workload, args.steps, args.warmup,
                              not args.no_cpu_baseline and args.workload != "copy8192")

    # what the matrix pipes of this very GPU sustain with no memory traffic (register-only MFMA
    # loop of the library), best of eight launches: reported beside the nominal peak
    sink = torch.zeros(256, dtype=torch.float32, device="cuda")
    probe_tflops = 0.0
    for _ in range(8):
        ps, pe = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        ps.record()
        probe_flop = mom.mom_probe_mfma_peak(2000, sink)
        pe.record()
        torch.cuda.synchronize()
        probe_tflops = max(probe_tflops, probe_flop / (ps.elapsed_time(pe) * 1e-3) / 1e12)
    if head["roofline"]["bound"] == "mfma":
        head["roofline"]["measured_peak"] = probe_tflops
        head["roofline"]["frac_of_measured_peak"] = head["roofline"]["achieved"] / probe_tflops

    configs = []
    if not args.no_configs:
        for w in SIDE_WORKLOADS:
            if w == args.workload:
                continue
            side_steps = max(10, min(args.steps, 100))
            rec, _, _ = measure(mom, w, side_steps, min(args.warmup, 10), False)
            r = rec["roofline"]
            configs.append({"workload": w, "plan": rec["plan"], "ms": rec["device_ms_per_step"], "min_ms": rec["min_ms"],
                            "value": rec["value"], "unit": "GFLOP/s", "bound": r["bound"], "frac": r["frac"],
                            "achieved": r["achieved"], "achieved_unit": r["unit"], "mfma_busy": r["mfma_busy"],
                            "traffic": r["traffic"], "launches_per_step": rec["launches_per_step"],
                            "step_bound_ms": r.get("step_bound_ms"), "frac_vs_planned_tree": r.get("frac_vs_planned_tree"),
                            "useful_flop": rec["useful_flop"], "tree_flop": rec["tree_flop"], "steps": side_steps})
            torch.cuda.empty_cache()

    line = {
        "metric": "useful GFLOP/s per chain eval (f32) + % of MI355X f32 MFMA peak",
        "value": head["value"],
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": args.workload, "dims": list(cfg.dims), "props": list(cfg.props),
                   "batch": cfg.batch, "plan": head["plan"], "mults": head["mults"],
                   "useful_flop": head["useful_flop"], "launches_per_step": head["launches_per_step"]},
        "pct_of_f32_mfma_peak": 100.0 * head["value"] / 1e3 / F32_MFMA_PEAK_TFLOPS,
        "device_ms_per_step": head["device_ms_per_step"],
        "min_ms": head["min_ms"],
        "median_ms": head["median_ms"],
        "settle_ms": head["settle_ms"],
        "roofline": head["roofline"],
        "configs": configs,
    }
    if "cpu_baseline" in head:
        line["cpu_baseline"] = head["cpu_baseline"]
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
