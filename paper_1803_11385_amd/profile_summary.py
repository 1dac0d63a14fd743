"""Short text summaries of rocprofv3 output, as kept under profiles/.

    python3 -m paper_1803_11385_amd.profile_summary --out profiles/NAME.txt --title "..." \
        [--command "..."]... [--note "..."]... [--bench bench.json] [--stats X_kernel_stats.csv] \
        [--counters Y_counter_collection.csv ...] [--traffic]

--stats     per-kernel calls / total / average / min / max from a `--kernel-trace --stats` run
--counters  average per launch of every counter found in `--pmc` runs, plus the ratios that can be
            formed from them (matrix-pipe busy share, L1 accesses per CU and cycle, ...)
--traffic   FETCH_SIZE / WRITE_SIZE in bytes per launch, each scaled by (known bytes / counted
            bytes) of the relu_fwd_kernel launches of `bench.py --copy-calibration`, a plain copy
            of 2^24 floats; written as `kernel | launches | fetch | write | total` lines, which
            bench.py reads back as `roofline.traffic`
Every summary names the digest of the library sources it was made from (build.source_digest()).
"""
from __future__ import annotations

import argparse
import collections
import csv
import json
import re

from .build import source_digest

CALIBRATION_BYTES = float(1 << 26)      # one relu_fwd_kernel launch over 2^24 floats, each way


def short(name):
    name = re.sub(r"^void ", "", name)
    i = name.find(">(")
    name = name[: i + 1] if i >= 0 else name.split("(")[0]
    return name.replace("hch::", "")


def ours(kernel):
    return "kernel" in kernel and not kernel.startswith("__amd") and "at::" not in kernel


def stats_table(path, min_pct):
    out = [f"{'kernel':76s} {'calls':>6s} {'total_us':>10s} {'avg_us':>9s} {'pct':>6s} {'min_us':>8s} {'max_us':>8s}"]
    for r in csv.DictReader(open(path)):
        if float(r["Percentage"]) < min_pct:
            continue
        out.append(f"{short(r['Name'])[:76]:76s} {r['Calls']:>6s} {float(r['TotalDurationNs']) / 1e3:10.1f} "
                   f"{float(r['AverageNs']) / 1e3:9.2f} {float(r['Percentage']):6.2f} "
                   f"{float(r['MinNs']) / 1e3:8.2f} {float(r['MaxNs']) / 1e3:8.2f}")
    return out


def read_counters(paths):
    """kernel -> counter -> list of per-dispatch values"""
    cnt = collections.defaultdict(lambda: collections.defaultdict(list))
    for p in paths:
        for r in csv.DictReader(open(p)):
            cnt[short(r["Kernel_Name"])][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return cnt


RATIOS = (
    ("mfma_busy", ("SQ_VALU_MFMA_BUSY_CYCLES", "SQ_BUSY_CU_CYCLES"), lambda a, b: a / (4 * b),
     "SQ_VALU_MFMA_BUSY_CYCLES / (4 * SQ_BUSY_CU_CYCLES): share of a busy CU's time in which its four matrix pipes work"),
    ("lds_busy", ("SQ_LDS_IDX_ACTIVE", "SQ_BUSY_CU_CYCLES"), lambda a, b: a / b, "SQ_LDS_IDX_ACTIVE / SQ_BUSY_CU_CYCLES"),
    ("lds_conflicts", ("SQ_LDS_BANK_CONFLICT", "SQ_LDS_IDX_ACTIVE"), lambda a, b: a / b, "SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE"),
    ("waiting", ("SQ_WAIT_INST_ANY", "SQ_WAVE_CYCLES"), lambda a, b: a / b,
     "SQ_WAIT_INST_ANY / SQ_WAVE_CYCLES: share of a wave's life spent waiting for an instruction's operands"),
    ("l1_rate", ("TCP_TOTAL_CACHE_ACCESSES_sum", "GRBM_GUI_ACTIVE"), lambda a, b: a / (256 * b / 8),
     "TCP_TOTAL_CACHE_ACCESSES_sum per CU and cycle (256 CUs; cycles = GRBM_GUI_ACTIVE / 8, the counter adds up the "
     "8 XCDs); an L1 takes about one 64-byte access per cycle"),
    ("l2_hit", ("TCC_HIT_sum", "TCC_MISS_sum"), lambda a, b: a / (a + b), "TCC_HIT_sum / (TCC_HIT_sum + TCC_MISS_sum)"),
)


def counter_table(cnt, only):
    names = sorted({c for k in cnt for c in cnt[k]})
    ratios = [r for r in RATIOS if all(c in names for c in r[1])]
    out = ["averages per launch" + (":" if not ratios else "; ratios:")]
    out += [f"  {r[0]} = {r[3]}" for r in ratios]
    out.append("")
    avg = {k: {c: sum(v) / len(v) for c, v in d.items()} for k, d in cnt.items()}
    key = names[0]
    for k in sorted(avg, key=lambda k: -avg[k].get(key, 0.0) * len(cnt[k].get(key, ()))):
        if not ours(k) or (only and not any(t in k for t in only)):
            continue
        out.append(f"{k}   ({max(len(v) for v in cnt[k].values())} launches)")
        for c in names:
            if c in avg[k]:
                out.append(f"    {c:32s} {avg[k][c]:14.5g}")
        for r in ratios:
            if all(c in avg[k] and avg[k][c] > 0 for c in r[1]):
                out.append(f"    {r[0]:32s} {r[2](avg[k][r[1][0]], avg[k][r[1][1]]):14.3f}")
    return out


def traffic_table(cnt):
    factor = {}
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        cal = cnt.get("relu_fwd_kernel", {}).get(c)
        if not cal:
            raise SystemExit(f"--traffic: no relu_fwd_kernel launches with {c} (run bench.py with --copy-calibration)")
        factor[c] = CALIBRATION_BYTES * len(cal) / (sum(cal) * 1024.0)
    out = ["# counters are in KiB per dispatch; each is scaled by (known bytes / counted bytes) of the relu_fwd_kernel",
           "# launches of --copy-calibration, a plain copy of 2^24 floats (64 MiB read, 64 MiB written):",
           f"#   FETCH_SIZE factor {factor['FETCH_SIZE']:.4f}   WRITE_SIZE factor {factor['WRITE_SIZE']:.4f}",
           "# columns: kernel | launches | fetch bytes per launch | write bytes per launch | total per launch"]
    rows = []
    for k, d in cnt.items():
        if not ours(k) or "FETCH_SIZE" not in d or "WRITE_SIZE" not in d:
            continue
        fe = sum(d["FETCH_SIZE"]) / len(d["FETCH_SIZE"]) * 1024 * factor["FETCH_SIZE"]
        wr = sum(d["WRITE_SIZE"]) / len(d["WRITE_SIZE"]) * 1024 * factor["WRITE_SIZE"]
        rows.append((-(fe + wr) * len(d["FETCH_SIZE"]), f"{k} | {len(d['FETCH_SIZE'])} | {fe:.0f} | {wr:.0f} | {fe + wr:.0f}"))
    return out + [r[1] for r in sorted(rows)]


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--out", required=True)
    ap.add_argument("--title", required=True)
    ap.add_argument("--command", action="append", default=[], help="a command the summary comes from (repeatable)")
    ap.add_argument("--note", action="append", default=[])
    ap.add_argument("--bench", help="file with the JSON line bench.py printed in the profiled run")
    ap.add_argument("--stats")
    ap.add_argument("--min-pct", type=float, default=0.05)
    ap.add_argument("--counters", nargs="*", default=[])
    ap.add_argument("--only", nargs="*", default=[], help="counter tables: only kernels whose name holds one of these")
    ap.add_argument("--traffic", action="store_true")
    a = ap.parse_args()

    pre = "# " if a.traffic else ""
    out = [pre + a.title, pre + f"sources sha256/16: {source_digest()}",
           pre + "commands (from the repository root on one MI355X, library built; `cd /tmp && export TMPDIR=/tmp` first"
                 " where rocprofv3 needs a writable temporary folder, then give bench.py by its full path):"]
    out += [pre + "  " + c for c in a.command]
    out += [pre + n for n in a.note]
    if a.bench:
        line = [l for l in open(a.bench) if l.lstrip().startswith("{")][-1]
        b = json.loads(line)
        out.append("")
        if "roofline" in b:
            r = b["roofline"]
            out.append(pre + f"bench.py in that run: {b['ms_per_step']} ms/step, {b['value']} {b['unit']}; dominant kernel {r['kernel']}:")
            out.append(pre + f"  average launch {r['avg_launch_ms'] * 1000:.1f} us by HIP events, {r['achieved']} {r['unit']} = {r['frac']} of peak")
        elif "products" in b:
            out.append(pre + f"bench.py in that run ({b['metric']}; HIP events around {b['calls_timed']} calls each):")
            for k, v in b["products"].items():
                out.append(pre + f"  {k:16s} {v['ms']:.4f} ms  {v['tflops']:.1f} TFLOP/s  ({v['frac_of_mfma_peak']:.3f} of the dense MFMA peak)")
        else:
            out.append(pre + "bench.py in that run: " + json.dumps({k: v for k, v in b.items() if k != "config"}))
    if a.stats:
        out += [""] + stats_table(a.stats, a.min_pct)
    if a.counters:
        cnt = read_counters(a.counters)
        out += traffic_table(cnt) if a.traffic else [""] + counter_table(cnt, a.only)
    with open(a.out, "w") as f:
        f.write("\n".join(out) + "\n")
    print("\n".join(out))


if __name__ == "__main__":
    main()
