"""Turns rocprofv3 output (CSV) into the short summaries kept under ``profiles/``.

    python -m paper_2401_09670_amd.profile_summary kernel-stats <..._kernel_stats.csv> --out profiles/X.md \
        --title "..." --command "rocprofv3 --kernel-trace --stats ... -- python3 bench.py ..."
    python -m paper_2401_09670_amd.profile_summary traffic <fetch_counter_collection.csv> <write_counter_collection.csv> \
        --out profiles/X.md --json profiles/X.json --command "..." --command "..."
    python -m paper_2401_09670_amd.profile_summary counters <sq_counter_collection.csv> --out profiles/X.md --command "..."

Every summary is stamped with ``source_stamp()``: a hash over the kernel sources the numbers were measured
on.  ``bench.py`` compares that stamp with the sources it runs and marks the stored HBM-traffic figures as
stale when they differ.  Nothing here touches the GPU; the inputs are files a profiler run left behind.
"""
from __future__ import annotations

import argparse
import collections
import csv
import hashlib
import json
import os
import re
import subprocess
from typing import Dict, List

PKG_DIR = os.path.dirname(os.path.abspath(__file__))

# kernel class (the names bench.py reports) -> substring of the kernel's symbol
KERNEL_CLASSES = collections.OrderedDict([
    ("gemm", "gemm_dl_kernel"), ("skinny_gemm", "skinny_gemm_kernel"), ("wring_gemm", "wring_gemm_kernel"),
    ("skinny_reduce", "skinny_reduce"), ("decode_attn", "decode_attention"), ("decode_combine", "decode_combine"),
    ("prefill_attn", "prefill_attention_kernel"), ("layernorm", "layernorm_kernel"),
    ("kv_migrate", "kv_migrate_kernel"), ("kv_append", "kv_append_kernel"),
    ("calibration_copy", "copyBuffer"),
])
CALIBRATION_BYTES = 1 << 30   # bench.py --copy-calibration copies 1 GiB device to device


def source_stamp() -> str:
    """sha256 (first 16 hex digits) over the kernel sources, in name order."""
    h = hashlib.sha256()
    csrc = os.path.join(PKG_DIR, "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


def git_head() -> str:
    try:
        return subprocess.run(["git", "rev-parse", "--short=12", "HEAD"], cwd=PKG_DIR, capture_output=True,
                              text=True, check=True).stdout.strip()
    except Exception:
        return "unknown"


def _header(title: str, commands: List[str]) -> str:
    out = [f"# {title}", "",
           f"Measured on kernel sources `{source_stamp()}` (profile_summary.source_stamp), git HEAD `{git_head()}` "
           "when summarised.", "", "Command(s), on the MI355X box from /tmp with TMPDIR=/tmp:", ""]
    out += [f"    {c}" for c in commands]
    out.append("")
    return "\n".join(out)


def _classify(kernel_name: str):
    for cls, pat in KERNEL_CLASSES.items():
        if pat in kernel_name:
            return cls
    return None


# ----------------------------------------------------------------------------- kernel trace
def kernel_stats(path: str, out: str, title: str, commands: List[str], notes: List[str]):
    rows = list(csv.DictReader(open(path)))
    lines = [_header(title, commands),
             "Per-kernel summary (rocprofv3 `kernel_stats.csv`; durations in ns):", "",
             "| kernel | calls | total ns | avg ns | % | min ns | max ns |", "|---|---|---|---|---|---|---|"]
    for r in rows:
        if float(r["Percentage"]) < 0.01:
            continue
        name = r["Name"].replace("|", "/")
        if len(name) > 90:
            name = name[:87] + "..."
        lines.append(f"| `{name}` | {r['Calls']} | {r['TotalDurationNs']} | {float(r['AverageNs']):.0f} | "
                     f"{r['Percentage']} | {r['MinNs']} | {r['MaxNs']} |")

    def tot(pat):
        return sum(int(r["TotalDurationNs"]) for r in rows if re.search(pat, r["Name"]))

    def calls(pat):
        return sum(int(r["Calls"]) for r in rows if re.search(pat, r["Name"]))

    n_prefill = calls(r"prefill_attention_kernel")
    n_decode = calls(r"decode_attention")
    lines += ["", "Class totals in the terms of bench.py's `kernels` table (one GEMM launch there = one linear step of "
              "the C ABI: 4 per prefill batch and 4 per decode step; a step may be two kernels - a column-split "
              "tail, a split-K reduce pass):", "",
              "| class | steps | kernels launched | total ms | us per step |", "|---|---|---|---|---|"]
    if n_prefill:
        g = tot(r"gemm_dl_kernel")
        lines.append(f"| prefill GEMM (`gemm`) | {4 * n_prefill} | {calls(r'gemm_dl_kernel')} | {g / 1e6:.1f} | "
                     f"{g / 1e3 / (4 * n_prefill):.1f} |")
    if n_decode:
        pat = r"skinny_gemm_kernel|wring_gemm_kernel|skinny_reduce"
        d = tot(pat)
        lines.append(f"| decode GEMM (`skinny_gemm`) | {4 * n_decode} | {calls(pat)} | {d / 1e6:.1f} | "
                     f"{d / 1e3 / (4 * n_decode):.1f} |")
    for name, pat in (("prefill attention (`prefill_attn`)", r"prefill_attention_kernel"),
                      ("decode attention (`decode_attn`)", r"decode_attention|decode_combine"),
                      ("KV hand-off (`kv_migrate`)", r"kv_migrate_kernel"), ("LayerNorm (`layernorm`)", r"layernorm_kernel")):
        c_ = calls(pat.split("|")[0])
        if c_:
            lines.append(f"| {name} | {c_} | {calls(pat)} | {tot(pat) / 1e6:.1f} | {tot(pat) / 1e3 / c_:.1f} |")
    lines += ["", "bench.py's own figures are HIP-event times around each step on the same stream (they include the "
              "gap to the next launch), a few per cent above these kernel-only durations.", ""]
    for n in notes:
        lines.append(open(n).read() if os.path.exists(n) else n)
    with open(out, "w") as f:
        f.write("\n".join(lines) + "\n")


# ----------------------------------------------------------------------------- HBM traffic
def _per_class(path: str, counter: str) -> Dict[str, List[float]]:
    out = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        if r["Counter_Name"] != counter:
            continue
        cls = _classify(r["Kernel_Name"])
        if cls is None:
            continue
        v = float(r["Counter_Value"])
        if cls == "calibration_copy" and v < 1000:   # small staging copies of the set-up
            continue
        out[cls].append(v)
    return out


def traffic(fetch_csv: str, write_csv: str, out: str, json_out: str, title: str, commands: List[str]):
    f = _per_class(fetch_csv, "FETCH_SIZE")
    w = _per_class(write_csv, "WRITE_SIZE")
    cal_f, cal_w = f.get("calibration_copy"), w.get("calibration_copy")
    if not cal_f or not cal_w:
        raise SystemExit("no calibration copy in the counter files: run bench.py with --copy-calibration")
    fetch_scale = CALIBRATION_BYTES / 1024 / (sum(cal_f) / len(cal_f))
    write_scale = CALIBRATION_BYTES / 1024 / (sum(cal_w) / len(cal_w))
    res, rows = {}, []
    for cls in KERNEL_CLASSES:
        if not f.get(cls) or not w.get(cls):
            continue
        fa, wa = sum(f[cls]) / len(f[cls]), sum(w[cls]) / len(w[cls])
        res[cls] = {"launches": len(f[cls]), "fetch_KiB_raw": round(fa, 1), "write_KiB_raw": round(wa, 1),
                    "hbm_read_bytes": round(fa * 1024 * fetch_scale), "hbm_write_bytes": round(wa * 1024 * write_scale)}
        rows.append(f"| {cls} | {len(f[cls])} | {fa:.0f} | {wa:.0f} | {fa * 1024 * fetch_scale / 1e6:.1f} | "
                    f"{wa * 1024 * write_scale / 1e6:.1f} |")
    # one decode GEMM call = a weight-streaming kernel (either of the two) plus, where K is split, its reduce launch
    gemm_kernels = [k for k in ("skinny_gemm", "wring_gemm") if k in res]
    n_calls = sum(res[k]["launches"] for k in gemm_kernels)
    if n_calls:
        parts = gemm_kernels + (["skinny_reduce"] if "skinny_reduce" in res else [])
        rd = sum(res[k]["hbm_read_bytes"] * res[k]["launches"] for k in parts)
        wr = sum(res[k]["hbm_write_bytes"] * res[k]["launches"] for k in parts)
        res["decode_gemm_call"] = {"launches": n_calls, "hbm_read_bytes": round(rd / n_calls),
                                   "hbm_write_bytes": round(wr / n_calls)}
        rows.append(f"| decode GEMM call (kernel + its reduce, average of the four) | {n_calls} | - | - | "
                    f"{rd / n_calls / 1e6:.1f} | {wr / n_calls / 1e6:.1f} |")
    with open(json_out, "w") as jf:
        json.dump({"source_stamp": source_stamp(), "git_head": git_head(), "commands": commands,
                   "fetch_scale": round(fetch_scale, 4), "write_scale": round(write_scale, 4), "per_launch": res},
                  jf, indent=1)
    text = _header(title, commands) + f"""
Calibration: `--copy-calibration` runs a plain 1 GiB device-to-device copy first (1 048 576 KiB read, 1 048 576 KiB
written).  The counters read FETCH_SIZE = {sum(cal_f) / len(cal_f):.0f} KiB and WRITE_SIZE = {sum(cal_w) / len(cal_w):.0f} KiB
for it, so FETCH_SIZE is scaled by {fetch_scale:.3f} and WRITE_SIZE by {write_scale:.3f}.  (Both counters sit behind
the L2: they count what leaves an XCD, whether the last-level cache or HBM then serves it.)

| kernel class | launches | FETCH_SIZE KiB (raw avg) | WRITE_SIZE KiB (raw avg) | read MB / launch (scaled) | write MB / launch |
|---|---|---|---|---|---|
""" + "\n".join(rows) + "\n"
    with open(out, "w") as of:
        of.write(text)


# ----------------------------------------------------------------------------- SQ counters
def counters(path: str, out: str, title: str, commands: List[str]):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(path)):
        short = r["Kernel_Name"].split("(")[0].replace("void ", "")
        agg[short][r["Counter_Name"]].append(float(r["Counter_Value"]))
    XCD, SIMD, CU = 8, 1024, 256
    rows = []
    for k, v in agg.items():
        if not k.startswith("ds::") or not v.get("GRBM_GUI_ACTIVE"):
            continue
        n = len(v["GRBM_GUI_ACTIVE"])

        def avg(c):
            return sum(v[c]) / max(len(v[c]), 1)
        gui = avg("GRBM_GUI_ACTIVE") / XCD
        mf, bc, ia = avg("SQ_VALU_MFMA_BUSY_CYCLES"), avg("SQ_LDS_BANK_CONFLICT"), avg("SQ_LDS_IDX_ACTIVE")
        wc, mops = avg("SQ_WAVE_CYCLES"), avg("SQ_INSTS_VALU_MFMA_MOPS_BF16")
        rows.append((-(avg("GRBM_GUI_ACTIVE") * n),
                     f"| `{k}` | {n} | {gui:.0f} | {100 * mf / (gui * SIMD):.1f} | {mops * 512 / 1e9:.2f} | "
                     f"{100 * bc / ia if ia else 0:.1f} | {4 * wc / (gui * CU):.1f} |"))
    text = _header(title, commands) + """
Averages per launch.  `GRBM_GUI_ACTIVE` is reported summed over the 8 XCDs and is divided by 8 here (cycles of one XCD
at the clock the kernel actually ran at).  MFMA busy % = `SQ_VALU_MFMA_BUSY_CYCLES` / (cycles x 1024 SIMDs), i.e. the
fraction of the matrix-core issue slots in use at that clock; MFMA GFLOP = `SQ_INSTS_VALU_MFMA_MOPS_BF16` x 512 (flops
the matrix cores executed, to be compared with the algorithmic count); LDS conflict % = `SQ_LDS_BANK_CONFLICT` /
`SQ_LDS_IDX_ACTIVE`; waves per CU = 4 x `SQ_WAVE_CYCLES` / (cycles x 256 CUs), the mean number of resident waves.

| kernel | launches | cycles per launch | MFMA busy % | MFMA GFLOP per launch | LDS bank conflict % | mean waves per CU |
|---|---|---|---|---|---|---|
""" + "\n".join(l for _, l in sorted(rows)) + "\n"
    with open(out, "w") as of:
        of.write(text)


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    sub = ap.add_subparsers(dest="what", required=True)
    a = sub.add_parser("kernel-stats")
    a.add_argument("csv")
    a.add_argument("--note", action="append", default=[], help="text (or a file of text) appended to the summary")
    b = sub.add_parser("traffic")
    b.add_argument("fetch_csv")
    b.add_argument("write_csv")
    b.add_argument("--json", required=True)
    c = sub.add_parser("counters")
    c.add_argument("csv")
    for p in (a, b, c):
        p.add_argument("--out", required=True)
        p.add_argument("--title", default="rocprofv3 summary")
        p.add_argument("--command", action="append", default=[])
    sub.add_parser("stamp")
    args = ap.parse_args(argv)
    if args.what == "kernel-stats":
        kernel_stats(args.csv, args.out, args.title, args.command, args.note)
    elif args.what == "traffic":
        traffic(args.fetch_csv, args.write_csv, args.out, args.json, args.title, args.command)
    elif args.what == "counters":
        counters(args.csv, args.out, args.title, args.command)
    else:
        print(source_stamp())


if __name__ == "__main__":
    main()
