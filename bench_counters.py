#!/usr/bin/env python3
"""Turn rocprofv3 counter passes of bench.py into bench_counters.json, the table bench.py
reads `roofline.traffic` and `roofline.mfma_busy` from.

The passes (one counter block per run, each in a run of its own; W = a bench.py workload,
D = any output folder, the same D for all passes):

  rocprofv3 --pmc FETCH_SIZE --output-format csv -d D/W/fetch -o p -- \
      python3 bench.py --workload W --no-configs --no-cpu-baseline --steps 10 --warmup 0 > D/W/fetch.json
  rocprofv3 --pmc WRITE_SIZE --output-format csv -d D/W/write -o p -- (same command)  > D/W/write.json
  rocprofv3 --pmc SQ_VALU_MFMA_BUSY_CYCLES GRBM_GUI_ACTIVE SQ_INSTS_VALU_MFMA_MOPS_F32 --output-format csv -d D/W/mfma -o p -- \
      (same command) > D/W/mfma.json

plus the fetch and write passes of the workload copy8192, a plain copy of 8192 x 8192 floats
whose HBM traffic is known (256 MiB each way): FETCH_SIZE and WRITE_SIZE (KiB per dispatch) are
scaled by what they read for that copy.

Then:  python3 bench_counters.py D   -> writes bench_counters.json next to bench.py and prints
the figures.  Per workload: bytes fetched / written per evaluation (all launches of the library
summed) and the fraction of the kernels' cycles in which the matrix pipes were busy
(SQ_VALU_MFMA_BUSY_CYCLES over 1024 SIMDs, against GRBM_GUI_ACTIVE over 8 XCDs, product
launches only).  The table is stamped with the digest of the kernel sources; bench.py ignores it
once they change."""
import collections
import csv
import glob
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
KNOWN_COPY_KIB = 8192 * 8192 * 4 / 1024.0
SIMDS, XCDS = 1024, 8


def read_pass(folder):
    """{counter: [(kernel name, value)]} of the library's dispatches, in dispatch order."""
    files = glob.glob(os.path.join(folder, "**", "*counter_collection.csv"), recursive=True)
    if not files:
        return None
    rows = list(csv.DictReader(open(files[0])))
    rows.sort(key=lambda r: int(r["Dispatch_Id"]))
    out = collections.defaultdict(list)
    for r in rows:
        name = r["Kernel_Name"]
        if "mom::" not in name or "probe_mfma" in name:
            continue
        out[r["Counter_Name"]].append((name, float(r["Counter_Value"])))
    return out


def bench_line(path):
    try:
        for ln in open(path):
            if ln.startswith("{"):
                return json.loads(ln)
    except OSError:
        pass
    return None


def per_step(values, launches_per_step):
    steps = len(values) / float(launches_per_step)
    return sum(v for _, v in values) / steps, steps


def main():
    if len(sys.argv) != 2:
        sys.exit(__doc__)
    top = sys.argv[1]
    sys.path.insert(0, ROOT)
    import bench
    cal_f, cal_w = read_pass(os.path.join(top, "copy8192", "fetch")), read_pass(os.path.join(top, "copy8192", "write"))
    if not cal_f or not cal_w:
        sys.exit("bench_counters.py: the copy8192 calibration passes are missing under %s" % top)
    f_vals, w_vals = [v for _, v in cal_f["FETCH_SIZE"]], [v for _, v in cal_w["WRITE_SIZE"]]
    fetch_scale = KNOWN_COPY_KIB / (sum(f_vals) / len(f_vals))
    write_scale = KNOWN_COPY_KIB / (sum(w_vals) / len(w_vals))
    print("calibration (copy8192, %.0f KiB each way): FETCH_SIZE x %.4f, WRITE_SIZE x %.4f" %
          (KNOWN_COPY_KIB, fetch_scale, write_scale))
    table = {"sources": bench.kernel_sources_digest(), "fetch_scale": fetch_scale, "write_scale": write_scale,
             "workloads": {}}
    for w in sorted(os.listdir(top)):
        if w not in bench.WORKLOADS:
            continue
        entry = {"fetch_bytes": None, "write_bytes": None, "mfma_busy": None}
        for leg, counter, scale, key in (("fetch", "FETCH_SIZE", fetch_scale, "fetch_bytes"),
                                         ("write", "WRITE_SIZE", write_scale, "write_bytes")):
            vals = read_pass(os.path.join(top, w, leg))
            line = bench_line(os.path.join(top, w, leg + ".json"))
            if not vals or not line or counter not in vals:
                continue
            kib, steps = per_step(vals[counter], line["config"]["launches_per_step"])
            entry[key] = int(round(kib * scale * 1024))
            entry[leg + "_steps"] = steps
        vals = read_pass(os.path.join(top, w, "mfma"))
        if vals and "SQ_VALU_MFMA_BUSY_CYCLES" in vals and "GRBM_GUI_ACTIVE" in vals:
            pick = [i for i, (name, _) in enumerate(vals["GRBM_GUI_ACTIVE"]) if "product_kernel" in name or "batched_chain" in name or "skinny_pair" in name]
            busy = sum(vals["SQ_VALU_MFMA_BUSY_CYCLES"][i][1] for i in pick) / SIMDS
            cycles = sum(vals["GRBM_GUI_ACTIVE"][i][1] for i in pick) / XCDS
            if cycles > 0:
                entry["mfma_busy"] = busy / cycles
                entry["mfma_dispatches"] = len(pick)
        table["workloads"][w] = entry
        print("%-26s fetch %s  write %s  mfma_busy %s" % (
            w, "%.1f MB" % (entry["fetch_bytes"] / 1e6) if entry["fetch_bytes"] is not None else "-",
            "%.1f MB" % (entry["write_bytes"] / 1e6) if entry["write_bytes"] is not None else "-",
            "%.3f" % entry["mfma_busy"] if entry["mfma_busy"] is not None else "-"))
    with open(os.path.join(ROOT, "bench_counters.json"), "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")


if __name__ == "__main__":
    main()
