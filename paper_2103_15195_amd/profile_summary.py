"""Short text summaries of rocprofv3 runs of bench.py, and the per-kernel HBM traffic file that bench.py reads.

    python3 -m paper_2103_15195_amd.profile_summary --stats S.csv --fetch F.csv --write W.csv \
        --out profiles/NAME.txt --traffic profiles/traffic_NAME.txt --title "..." --commands-file cmds.txt

S.csv is the kernel_stats file of a `rocprofv3 --kernel-trace --stats --output-format csv` run; F.csv and W.csv are the
counter_collection files of two `--pmc` runs (FETCH_SIZE, then WRITE_SIZE, KiB per dispatch) of bench.py with
--calibrate-copy, which adds plain 256 MiB device copies: what the counters read for those gives the factor that turns
the counters into bytes.  The traffic file holds one line per library kernel: profiler slot name, HBM bytes per launch
(read + write), read bytes, write bytes.  Every --counters C.csv adds a table of further per-dispatch counters.
"""
from __future__ import annotations

import argparse
import collections
import csv

COPY_KIB = 262144.0          # the calibration copy moves 256 MiB in and 256 MiB out
COPY_GRID = 131072           # ... and the runtime launches it with this grid
SLOT_OF = {"sign_compress": "efsign_compress", "plane_decompress": "dense_decompress"}


def short_name(kernel: str) -> str:
    return kernel.split("(")[0].replace("void ", "")


def slot_name(kernel: str) -> str:
    """Name under which the library's own profiler (mc_profile_read) lists this kernel."""
    base = short_name(kernel).split("<")[0].split("::")[-1]
    base = base[:-2] if base.endswith("_k") else base
    return SLOT_OF.get(base, base)


def per_dispatch(path: str, counter: str | None = None):
    d = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if counter is None or r["Counter_Name"] == counter:
            d[(r["Kernel_Name"], int(r["Grid_Size"]), r["Counter_Name"])].append(float(r["Counter_Value"]))
    return d


def mean(v):
    return sum(v) / len(v)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--stats", required=True)
    ap.add_argument("--trace", help="the kernel_trace file of the same run: adds the median duration and the register count")
    ap.add_argument("--fetch")
    ap.add_argument("--write")
    ap.add_argument("--counters", action="append", default=[], help="counter_collection file of a further --pmc run (may be given more than once)")
    ap.add_argument("--out", required=True)
    ap.add_argument("--traffic")
    ap.add_argument("--title", required=True)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--commands-file", required=True, help="text file with the full commands that produced the inputs")
    a = ap.parse_args()

    L = [a.title, "", "Commands (from the repository root on one MI355X; each is a process of its own):"]
    L += ["  " + l.rstrip() for l in open(a.commands_file) if l.strip()]
    med, regs = {}, {}
    if a.trace:
        durs = collections.defaultdict(list)
        for r in csv.DictReader(open(a.trace)):
            durs[r["Kernel_Name"]].append(int(r["End_Timestamp"]) - int(r["Start_Timestamp"]))
            regs[r["Kernel_Name"]] = f"{r['VGPR_Count']:>4s} {r['LDS_Block_Size']:>6s}"
        med = {k: sorted(v)[len(v) // 2] / 1e3 for k, v in durs.items()}
    L += ["", f"Workload: {a.workload}", "", "Kernel time (--kernel-trace --stats), library kernels only:",
          f"  {'kernel':62s} {'calls':>6s} {'avg us':>9s} {'median':>9s} {'min us':>9s} {'max us':>9s} {'% of GPU time':>14s} {'VGPR':>4s} {'LDS B':>6s}"]
    for r in csv.DictReader(open(a.stats)):
        if "mc::" in r["Name"]:
            m = f"{med[r['Name']]:9.2f}" if r["Name"] in med else f"{'-':>9s}"
            L.append(f"  {short_name(r['Name']):62s} {int(r['Calls']):6d} {float(r['AverageNs']) / 1e3:9.2f} {m} {float(r['MinNs']) / 1e3:9.2f} "
                     f"{float(r['MaxNs']) / 1e3:9.2f} {float(r['Percentage']):14.2f} {regs.get(r['Name'], '')}")

    if a.fetch and a.write:
        F, Wr = per_dispatch(a.fetch, "FETCH_SIZE"), per_dispatch(a.write, "WRITE_SIZE")
        copyF = [v for (k, g, c), v in F.items() if "copyBuffer" in k and g == COPY_GRID][0]
        copyW = [v for (k, g, c), v in Wr.items() if "copyBuffer" in k and g == COPY_GRID][0]
        fscale, wscale = COPY_KIB / mean(copyF), COPY_KIB / mean(copyW)
        L += ["", "HBM traffic per launch (--pmc FETCH_SIZE / WRITE_SIZE, KiB per dispatch), scaled by what the same counter",
              "reads for a plain 256 MiB device copy (__amd_rocclr_copyBuffer, 262144 KiB in and out):",
              f"  FETCH_SIZE of the copy = {mean(copyF):.1f} -> scale {fscale:.4f};  WRITE_SIZE of the copy = {mean(copyW):.1f} -> scale {wscale:.4f}",
              f"  {'kernel':62s} {'launches':>8s} {'read MB':>10s} {'write MB':>10s} {'total MB':>10s}"]
        slots = collections.OrderedDict()
        for (k, g, c), v in sorted(F.items(), key=lambda kv: -mean(kv[1])):
            if "mc::" not in k:
                continue
            w = Wr.get((k, g, "WRITE_SIZE"), [0.0])
            rd, wr = mean(v) * fscale * 1024, mean(w) * wscale * 1024
            L.append(f"  {short_name(k):62s} {len(v):8d} {rd / 1e6:10.2f} {wr / 1e6:10.2f} {(rd + wr) / 1e6:10.2f}")
            s = slots.setdefault(slot_name(k), [0.0, 0.0, 0])
            s[0] += rd * len(v)
            s[1] += wr * len(v)
            s[2] += len(v)
        if a.traffic:
            with open(a.traffic, "w") as f:
                f.write("# HBM bytes per launch by kernel (launch-weighted mean over template instances and grid sizes), from the\n"
                        f"# FETCH_SIZE / WRITE_SIZE runs summarised in {a.out}\n# slot total_bytes read_bytes write_bytes launches\n")
                for s, (rd, wr, n) in slots.items():
                    f.write(f"{s} {(rd + wr) / n:.0f} {rd / n:.0f} {wr / n:.0f} {n}\n")

    for path in a.counters:
        Cn = per_dispatch(path)
        names = sorted({c for (_, _, c) in Cn})
        L += ["", "Further counters per launch (mean over launches; a pass of its own), by kernel and grid size:",
              "  " + f"{'kernel':62s} {'grid':>9s} " + " ".join(f"{n:>22s}" for n in names)]
        for k, g in sorted({(k, g) for (k, g, _) in Cn if "mc::" in k}):
            L.append("  " + f"{short_name(k):62s} {g:9d} " + " ".join(f"{mean(Cn[(k, g, n)]):22.0f}" if (k, g, n) in Cn else f"{'-':>22s}" for n in names))

    text = "\n".join(L) + "\n"
    open(a.out, "w").write(text)
    print(text)


if __name__ == "__main__":
    main()
