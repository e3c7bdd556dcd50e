"""Turns raw rocprofv3 output (CSV) into the short text summaries kept under profiles/.

  python -m paper_1805_10387_amd.profile_summary stats   <kernel_stats.csv> <out.txt> --title T --command C [--note N ...]
  python -m paper_1805_10387_amd.profile_summary traffic <fetch_counter_collection.csv> <write_counter_collection.csv> <out.txt>
                                                         --command-fetch C1 --command-write C2
  python -m paper_1805_10387_amd.profile_summary counters <counter_collection.csv> <out.txt> --title T --command C
  python -m paper_1805_10387_amd.profile_summary mfma     <counter_collection.csv> <out.txt> --title T --command C [--note N ...]

`traffic` also writes the two machine-readable lines bench.py reads for its `roofline.traffic` fields:
  gemm_traffic_bytes_per_launch = <bytes>      update_traffic_bytes_per_launch = <bytes>
Counter values of FETCH_SIZE / WRITE_SIZE are KiB per dispatch; each is scaled by what the same counter reads for the
256 MiB device copy bench.py issues as its calibration launch (__amd_rocclr_copyBuffer with the largest grid)."""
from __future__ import annotations

import argparse
import collections
import csv
import re


def _short(name: str) -> str:
    if "mfma_rate_kernel" in name:          # reported with its mangled name
        return "mfma_rate_kernel (probe)"
    name = name.replace("void ", "").replace("mp::", "")
    return re.sub(r"\(.*$", "", name)[:78]


def stats(a):
    rows = list(csv.DictReader(open(a.csv)))
    out = [a.title, "", "command (from /tmp, TMPDIR=/tmp, PYTHONPATH=/root/repo):", "  " + a.command, ""]
    out += list(a.note or []) + ([""] if a.note else [])
    out.append(f"{'kernel':<80}{'calls':>7}{'total_ms':>10}{'avg_us':>10}{'min_us':>10}{'max_us':>10}{'pct':>7}")
    for r in rows:
        out.append(f"{_short(r['Name']):<80}{r['Calls']:>7}{float(r['TotalDurationNs']) / 1e6:>10.3f}{float(r['AverageNs']) / 1e3:>10.2f}"
                   f"{float(r['MinNs']) / 1e3:>10.2f}{float(r['MaxNs']) / 1e3:>10.2f}{float(r['Percentage']):>7.2f}")
    gem = [r for r in rows if "gemm_" in r["Name"] and "splitk" not in r["Name"]]
    if gem:
        n = sum(int(r["Calls"]) for r in gem)
        t = sum(float(r["TotalDurationNs"]) for r in gem)
        out += ["", f"contraction kernels (gemm_kernel, gemm_dtl_kernel, grouped variants), all instances: {n} launches, {t / 1e6:.3f} ms, "
                    f"average {t / n / 1e3:.2f} us per launch"]
    open(a.out, "w").write("\n".join(out) + "\n")


def _per_kernel(path, counter):
    tot, cnt, grids = collections.defaultdict(float), collections.Counter(), {}
    seen = set()
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        k = _short(r["Kernel_Name"])
        tot[k] += float(r["Counter_Value"])
        key = (k, r["Dispatch_Id"])
        if key not in seen:
            seen.add(key)
            cnt[k] += 1
        g = int(r.get("Grid_Size", 0) or 0)
        if k.startswith("__amd_rocclr_copyBuffer"):
            grids.setdefault(r["Dispatch_Id"], [g, 0.0])
            grids[r["Dispatch_Id"]][1] += float(r["Counter_Value"])
    return tot, cnt, grids


def traffic(a):
    out = ["HBM-side traffic of the contraction kernels and the update kernel in bench.py (config 3), from two rocprofv3 --pmc runs",
           "", "commands (from /tmp, TMPDIR=/tmp, repo at /root/repo; eager launches, short run: counter collection serialises dispatches):",
           "  " + a.command_fetch, "  " + a.command_write, "",
           "Counter values are KiB per dispatch, summed per kernel below (largest first).", ""]
    res, factor = {}, {}
    for counter, path in (("FETCH_SIZE", a.fetch), ("WRITE_SIZE", a.write)):
        tot, cnt, grids = _per_kernel(path, counter)
        out.append(counter)
        out.append(f"{'kernel':<80}{'dispatches':>11}{'KiB total':>16}{'KiB/dispatch':>15}")
        for k in sorted(tot, key=lambda x: -tot[x])[:16]:
            out.append(f"{k:<80}{cnt[k]:>11}{tot[k]:>16.1f}{tot[k] / cnt[k]:>15.1f}")
        out.append("")
        cal = max(grids.values(), key=lambda v: (v[0], v[1])) if grids else None   # the 256 MiB copy: largest grid, most bytes
        factor[counter] = (262144.0 / cal[1]) if cal and cal[1] > 0 else 1.0
        res[counter] = (tot, cnt)
    out.append("calibration (the __amd_rocclr_copyBuffer dispatch with the largest grid and reading: the 256 MiB copy, 262144 KiB read and written):")
    out.append(f"  FETCH_SIZE factor {factor['FETCH_SIZE']:.4f}   WRITE_SIZE factor {factor['WRITE_SIZE']:.4f}")
    out.append("")

    def per_launch(match):
        b, n = 0.0, None
        for counter in ("FETCH_SIZE", "WRITE_SIZE"):
            tot, cnt = res[counter]
            ks = [k for k in tot if match(k)]
            launches = sum(cnt[k] for k in ks)
            n = launches if n is None else n
            if launches:
                b += sum(tot[k] for k in ks) * 1024.0 * factor[counter] / launches
        return b, n

    gb, gn = per_launch(lambda k: k.startswith("gemm_") and "splitk" not in k)
    ub, un = per_launch(lambda k: k.startswith("update_kernel"))
    out.append(f"per launch, average over the {gn} contraction launches (gemm_kernel, gemm_dtl_kernel and grouped variants): {gb / 1e6:.1f} MB")
    out.append(f"per launch of update_kernel ({un} launches): {ub / 1e6:.1f} MB")
    out.append("")
    out.append(f"gemm_traffic_bytes_per_launch = {int(gb)}")
    out.append(f"update_traffic_bytes_per_launch = {int(ub)}")
    open(a.out, "w").write("\n".join(out) + "\n")


def counters(a):
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    disp = collections.defaultdict(set)
    for r in csv.DictReader(open(a.csv)):
        k = _short(r["Kernel_Name"])
        agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
        disp[k].add(r["Dispatch_Id"])
    names = sorted({c for v in agg.values() for c in v})
    out = [a.title, "", "command (from /tmp, TMPDIR=/tmp, repo at /root/repo):", "  " + a.command, ""]
    out += list(a.note or []) + ([""] if a.note else [])
    out.append(f"{'kernel':<64}{'launches':>9}" + "".join(f"{n[-22:]:>24}" for n in names))
    for k in sorted(agg, key=lambda x: -sum(agg[x].values()))[:14]:
        out.append(f"{k[:62]:<64}{len(disp[k]):>9}" + "".join(f"{agg[k].get(n, 0.0):>24.4g}" for n in names))
    open(a.out, "w").write("\n".join(out) + "\n")


def mfma(a):
    """Derived per-kernel figures from one --pmc run holding SQ_VALU_MFMA_BUSY_CYCLES, GRBM_GUI_ACTIVE, SQ_WAIT_ANY,
    SQ_WAVE_CYCLES, SQ_ACTIVE_INST_LDS, SQ_LDS_BANK_CONFLICT and SQ_INSTS_VALU_MFMA_MOPS_F16."""
    agg = collections.defaultdict(lambda: collections.defaultdict(float))
    disp = collections.defaultdict(set)
    for r in csv.DictReader(open(a.csv)):
        k = _short(r["Kernel_Name"])
        agg[k][r["Counter_Name"]] += float(r["Counter_Value"])
        disp[k].add(r["Dispatch_Id"])
    out = [a.title, "", "command (from /tmp, TMPDIR=/tmp, repo at /root/repo; eager launches, short run: counter collection serialises dispatches):",
           "  " + a.command, "",
           "GRBM_GUI_ACTIVE is summed over the 8 XCDs, SQ_VALU_MFMA_BUSY_CYCLES over the 1024 SIMDs:",
           "  MFMA busy % = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 * 1024).",
           "wait any % = SQ_WAIT_ANY / SQ_WAVE_CYCLES, LDS active % = SQ_ACTIVE_INST_LDS / SQ_WAVE_CYCLES, bank conflicts = SQ_LDS_BANK_CONFLICT per",
           "launch.  SQ_INSTS_VALU_MFMA_MOPS_F16 x 512 is the flop count the hardware saw per launch: it equals 2 M N K of the launch.", ""]
    out.append(f"{'kernel':<62}{'launches':>9}{'GUI cyc/8':>12}{'MFMA busy %':>12}{'wait any %':>11}{'LDS act %':>10}{'bank conf':>11}{'flop':>12}")
    keep = [k for k in agg if agg[k].get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) > 0.0]
    for k in sorted(keep, key=lambda x: -agg[x]["SQ_VALU_MFMA_BUSY_CYCLES"]):
        c, n = agg[k], len(disp[k])
        gui = c["GRBM_GUI_ACTIVE"] / 8.0
        wave = max(c["SQ_WAVE_CYCLES"], 1.0)
        out.append(f"{k[:60]:<62}{n:>9}{gui / n:>12.0f}{100.0 * c['SQ_VALU_MFMA_BUSY_CYCLES'] / (gui * 1024.0):>12.1f}"
                   f"{100.0 * c['SQ_WAIT_ANY'] / wave:>11.1f}{100.0 * c['SQ_ACTIVE_INST_LDS'] / wave:>10.1f}"
                   f"{c['SQ_LDS_BANK_CONFLICT'] / n:>11.0f}{512.0 * c['SQ_INSTS_VALU_MFMA_MOPS_F16'] / n:>12.4g}")
    out += [""] + list(a.note or [])
    open(a.out, "w").write("\n".join(out) + "\n")


def main():
    ap = argparse.ArgumentParser(prog="python -m paper_1805_10387_amd.profile_summary")
    sub = ap.add_subparsers(dest="what", required=True)
    p = sub.add_parser("stats")
    p.add_argument("csv"); p.add_argument("out"); p.add_argument("--title", required=True); p.add_argument("--command", required=True)
    p.add_argument("--note", action="append")
    p.set_defaults(fn=stats)
    p = sub.add_parser("traffic")
    p.add_argument("fetch"); p.add_argument("write"); p.add_argument("out")
    p.add_argument("--command-fetch", required=True); p.add_argument("--command-write", required=True)
    p.set_defaults(fn=traffic)
    p = sub.add_parser("counters")
    p.add_argument("csv"); p.add_argument("out"); p.add_argument("--title", required=True); p.add_argument("--command", required=True)
    p.add_argument("--note", action="append")
    p.set_defaults(fn=counters)
    p = sub.add_parser("mfma")
    p.add_argument("csv"); p.add_argument("out"); p.add_argument("--title", required=True); p.add_argument("--command", required=True)
    p.add_argument("--note", action="append")
    p.set_defaults(fn=mfma)
    a = ap.parse_args()
    a.fn(a)


if __name__ == "__main__":
    main()
