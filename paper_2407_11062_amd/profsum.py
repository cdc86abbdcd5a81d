"""Turn rocprofv3 CSV output into the short text / JSON summaries kept under profiles/.

  python -m paper_2407_11062_amd.profsum trace   <prefix>_kernel_stats.csv  <out.txt>  "<command that was profiled>" [bench.json]
  python -m paper_2407_11062_amd.profsum traffic <out.json> <workload> <fetch.csv> <write.csv> <copy_fetch.csv> <copy_write.csv> <copy_bytes>

  python -m paper_2407_11062_amd.profsum counters <out.txt> "<command that was profiled>" <counter_collection.csv> [more.csv ...]

`trace`   one line per kernel (calls, total and average duration, share) from `rocprofv3 --kernel-trace --stats`,
          followed by the bench line of the same run if given.
`traffic` bytes per launch that crossed the L2 <-> memory-fabric boundary, per library kernel, from two
          `rocprofv3 --pmc` runs of the bench (FETCH_SIZE, then WRITE_SIZE; both in KiB per dispatch), each scaled by
          what the same counter reads for a plain device copy of `copy_bytes` bytes (bench.py --copy-calibration).
`traffic-rows` the same two counters for every library kernel of a run with launches of several sizes (the benchmark's
          rows): one line per kernel and grid size (work-items of the launch), so that each matrix shape stands alone.
          python -m paper_2407_11062_amd.profsum traffic-rows <out.txt> "<command>" <fetch.csv> <write.csv> <copy_fetch.csv> <copy_write.csv> <copy_bytes>
`counters` mean reading per launch of every counter in the given `rocprofv3 --pmc` CSV files, per library kernel, plus
          the MFMA pipe's share of the busy cycles where both counters are present.
"""
from __future__ import annotations

import collections
import csv
import json
import sys

# kernel-name fragment -> name the library's own timers use
KERNELS = (("k_gemm_q<", None), ("k_gemm_dw", "gemm_dw"), ("k_quantize", "quantize"), ("k_init_minmax", "init_minmax"),
           ("k_e2e_prepare", "e2e_prepare"), ("k_gemv", "gemv"), ("k_recon_loss", "recon_loss"), ("k_adamw", "adamw_update"))


def _library_kernel(name: str):
    if "k_gemm_q<" in name:
        # second template argument: false = forward (weights K-contiguous), true = dX
        args = name.split("k_gemm_q<", 1)[1].split(",")
        return "gemm_dx" if args[1].strip() == "true" else "gemm_fwd"
    if "k_gemm_qILi" in name:                       # mangled form: ...ILi<bits>ELb<0|1>E...
        return "gemm_dx" if name.split("k_gemm_qILi", 1)[1].split("ELb", 1)[1][0] == "1" else "gemm_fwd"
    for frag, label in KERNELS[1:]:
        if frag in name:
            return label
    return None


def trace(stats_csv: str, out_txt: str, command: str, bench_json: str | None = None) -> None:
    rows = list(csv.DictReader(open(stats_csv)))
    with open(out_txt, "w") as f:
        f.write("rocprofv3 kernel-trace summary (MI355X, gfx950)\ncommand: %s\n\n" % command)
        f.write("%-100s %6s %14s %12s %7s\n" % ("kernel", "calls", "total_ns", "avg_ns", "pct"))
        for r in rows:
            if float(r["Percentage"]) < 0.05:
                continue
            f.write("%-100s %6s %14s %12.0f %7s\n" % (r["Name"][:100], r["Calls"], r["TotalDurationNs"],
                                                     float(r["AverageNs"]), r["Percentage"]))
        if bench_json:
            bench = json.loads(open(bench_json).read().strip().splitlines()[-1])
            f.write("\nbench.py line of the same run (HIP-event timing inside the library, timed steps only):\n")
            keep = {k: bench[k] for k in ("value", "unit", "ms_per_step", "roofline", "kernels") if k in bench}
            f.write(json.dumps(keep, indent=1) + "\n")


def _mean_per_kernel(counter_csv: str):
    acc = collections.defaultdict(list)
    for r in csv.DictReader(open(counter_csv)):
        acc[r["Kernel_Name"]].append(float(r["Counter_Value"]))
    return {k: sum(v) / len(v) for k, v in acc.items()}, {k: len(v) for k, v in acc.items()}


def traffic(out_json, workload, fetch_csv, write_csv, copy_fetch_csv, copy_write_csv, copy_bytes) -> None:
    copy_bytes = float(copy_bytes)

    def copy_factor(path):
        mean, n = _mean_per_kernel(path)
        # the copy kernel is the one with the largest mean reading
        k = max(mean, key=lambda x: mean[x])
        return copy_bytes / (mean[k] * 1024.0), k, n[k]

    f_fac, f_k, f_n = copy_factor(copy_fetch_csv)
    w_fac, w_k, w_n = copy_factor(copy_write_csv)
    out = {"_comment": "Bytes crossing the L2 <-> memory-fabric boundary per launch (mean over the launches of one bench run): "
                       "rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE (KiB per dispatch), each scaled by what the same counter "
                       "reads for a device copy of %d bytes (FETCH_SIZE x%.3f, WRITE_SIZE x%.3f)." % (copy_bytes, f_fac, w_fac)}
    per = collections.defaultdict(lambda: {"fetch": 0.0, "write": 0.0, "n": 0})
    for path, fac, key in ((fetch_csv, f_fac, "fetch"), (write_csv, w_fac, "write")):
        acc = collections.defaultdict(list)
        for r in csv.DictReader(open(path)):
            lab = _library_kernel(r["Kernel_Name"])
            if lab:
                acc[lab].append(float(r["Counter_Value"]) * 1024.0 * fac)
        for lab, v in acc.items():
            per[lab][key] = sum(v) / len(v)
            per[lab]["n"] = len(v)
    try:                                   # other workloads already in the file stay
        prior = json.load(open(out_json))
        out.update({k: v for k, v in prior.items() if k != "_comment"})
    except (OSError, ValueError):
        pass
    out[workload] = {lab: int(round(d["fetch"] + d["write"])) for lab, d in per.items()}
    out[workload + "_detail"] = {lab: {"fetch_bytes": int(round(d["fetch"])), "write_bytes": int(round(d["write"])),
                                       "launches_sampled": d["n"]} for lab, d in per.items()}
    json.dump(out, open(out_json, "w"), indent=1)
    print(json.dumps(out, indent=1))


def _copy_factor(path, copy_bytes):
    mean, _ = _mean_per_kernel(path)
    k = max(mean, key=lambda x: mean[x])          # the copy kernel is the one with the largest mean reading
    return float(copy_bytes) / (mean[k] * 1024.0)


def traffic_rows(out_txt, command, fetch_csv, write_csv, copy_fetch_csv, copy_write_csv, copy_bytes) -> None:
    f_fac, w_fac = _copy_factor(copy_fetch_csv, copy_bytes), _copy_factor(copy_write_csv, copy_bytes)
    per = collections.defaultdict(lambda: {"fetch": [], "write": []})
    for path, fac, key in ((fetch_csv, f_fac, "fetch"), (write_csv, w_fac, "write")):
        for r in csv.DictReader(open(path)):
            lab = _library_kernel(r["Kernel_Name"])
            if lab:
                per[(lab, int(r["Grid_Size"]))][key].append(float(r["Counter_Value"]) * 1024.0 * fac)
    with open(out_txt, "w") as f:
        f.write("rocprofv3 FETCH_SIZE / WRITE_SIZE per launch (MI355X, gfx950): bytes that crossed the L2 <-> memory-fabric\n"
                "boundary, mean over the launches of one kernel at one grid size; counters scaled by what they read for a\n"
                "device copy of %d bytes (FETCH_SIZE x%.3f, WRITE_SIZE x%.3f)\n" % (int(float(copy_bytes)), f_fac, w_fac))
        f.write("command (FETCH_SIZE, then WRITE_SIZE in a run of its own): %s\n\n" % command)
        f.write("%-16s %12s %9s %14s %14s %14s\n" % ("kernel", "work-items", "launches", "fetch_bytes", "write_bytes", "total_bytes"))
        for (lab, grid) in sorted(per):
            d = per[(lab, grid)]
            fe = sum(d["fetch"]) / max(1, len(d["fetch"]))
            wr = sum(d["write"]) / max(1, len(d["write"]))
            f.write("%-16s %12d %9d %14.0f %14.0f %14.0f\n" % (lab, grid, len(d["fetch"]), fe, wr, fe + wr))
    print(open(out_txt).read())


def counters(out_txt, command, *csvs) -> None:
    acc = collections.defaultdict(lambda: collections.defaultdict(list))
    for path in csvs:
        for r in csv.DictReader(open(path)):
            lab = _library_kernel(r["Kernel_Name"])
            if lab:
                acc[lab][r["Counter_Name"]].append(float(r["Counter_Value"]))
    with open(out_txt, "w") as f:
        f.write("rocprofv3 counter summary (MI355X, gfx950): mean per launch over the launches of one bench run\n")
        f.write("command: %s\n\n" % command)
        for lab in sorted(acc):
            f.write("%s\n" % lab)
            means = {c: sum(v) / len(v) for c, v in acc[lab].items()}
            for c in sorted(means):
                f.write("  %-34s %18.0f   (%d launches)\n" % (c, means[c], len(acc[lab][c])))
            if "SQ_VALU_MFMA_BUSY_CYCLES" in means and "SQ_BUSY_CU_CYCLES" in means and means["SQ_BUSY_CU_CYCLES"] > 0:
                # MFMA busy cycles are summed over the 4 SIMDs of a CU, CU busy cycles over the CUs
                f.write("  MFMA pipe busy / (4 x CU busy cycles)  %.3f\n" % (means["SQ_VALU_MFMA_BUSY_CYCLES"] / (4.0 * means["SQ_BUSY_CU_CYCLES"])))
            f.write("\n")
    print(open(out_txt).read())


def main(argv):
    if len(argv) >= 4 and argv[0] == "trace":
        trace(*argv[1:5])
    elif len(argv) == 8 and argv[0] == "traffic":
        traffic(*argv[1:])
    elif len(argv) == 8 and argv[0] == "traffic-rows":
        traffic_rows(*argv[1:])
    elif len(argv) >= 4 and argv[0] == "counters":
        counters(*argv[1:])
    else:
        print(__doc__)
        return 2
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv[1:]))
