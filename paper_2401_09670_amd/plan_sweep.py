"""Measures what the GEMM planners choose against every plan that can be forced, shape by shape.

    python -m paper_2401_09670_amd.plan_sweep --model opt13b --out profiles/gemm_plan_sweep_opt13b.md

The library picks, per product shape, a kernel family, a tile, a split count over K and (for prefill sizes) a
column cut (``skinny_plan`` / ``wring_tiles`` / ``decode_plan`` / ``prefill_plan`` in csrc).  Some of those rules
are a model, some are measured optima for the OPT shapes.  This harness is the measurement: it loads the
development build of the library (``build.build_library(dev=True)`` -> libds_dev.so, the same sources with the
planning switches settable at run time through ``ds_dev_switch``), times ``ds_linear`` with the planner left
alone and with each alternative forced, on weights that are not resident in any cache (rotating copies, more than
600 MB in total), and writes one table.  The product library has no such switches and is never touched.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

SHAPES = {"opt13b": (5120, 20480), "opt66b": (9216, 36864), "opt175b": (12288, 49152)}
INT32_MIN = -(1 << 31)


class Harness:
    def __init__(self):
        import torch
        from . import binding, build
        if not os.path.exists(build.DEV_LIB_PATH):
            build.build_library(dev=True)
        binding.LIB_PATH = build.DEV_LIB_PATH      # this process only
        self.torch, self.binding = torch, binding
        self.lib = binding.load_library()
        self.lib.ds_dev_switch.argtypes = [ctypes.c_char_p, ctypes.c_int32]
        self.lib.ds_dev_switch.restype = ctypes.c_int32
        self.dev = torch.device("cuda:0")
        self.defaults = {}

    def switch(self, name: str, value: int):
        old = self.lib.ds_dev_switch(name.encode(), value)
        if old == INT32_MIN:
            raise RuntimeError(f"no switch {name} in the development build")
        self.defaults.setdefault(name, old)

    def reset(self):
        for name, value in self.defaults.items():
            self.lib.ds_dev_switch(name.encode(), value)

    def time_linear(self, ctx, M: int, K: int, N: int, copies):
        """Mean microseconds of ds_linear over the rotating weight copies; None if the forced plan is rejected."""
        torch = self.torch
        x = torch.empty((M, K), dtype=torch.bfloat16, device=self.dev).normal_()
        y = torch.empty((M, N), dtype=torch.bfloat16, device=self.dev)
        ws = torch.empty(max(ctx.ds_linear_workspace_bytes(M, K, N), 16) + (96 << 20), dtype=torch.uint8,
                         device=self.dev)
        R = len(copies)
        try:
            for i in range(R):
                ctx.ds_linear(x, copies[i], None, None, 0, M, K, N, y, ws)
        except self.binding.DsError:
            return None
        reps = max(3 * R, 24)
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(reps):
            ctx.ds_linear(x, copies[i % R], None, None, 0, M, K, N, y, ws)
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps * 1e3


def sweep(model: str, decode_rows, prefill_rows, log=print):
    hs = Harness()
    torch = hs.torch
    h, m = SHAPES[model]
    ctx = hs.binding.Context(h, h // 128, 128, m)
    gemms = (("QKV", h, 3 * h), ("out-proj", h, h), ("FFN-in", h, m), ("FFN-out", m, h))
    rows = []
    for name, K, N in gemms:
        R = max(2, (600 << 20) // (K * N * 2) + 1)
        copies = [torch.empty((N, K), dtype=torch.bfloat16, device=hs.dev).normal_(0, 0.02) for _ in range(R)]
        for M in decode_rows:
            hs.reset()
            plan = ctx.ds_linear_plan(M, K, N)
            t_plan = hs.time_linear(ctx, M, K, N, copies)
            forced = []
            hs.switch("g_skinny_wring", 0)
            for ntw in (1, 2, 4):
                for sp in (1, 2, 3, 4, 6, 8, 12, 16):
                    if (N // (64 * ntw)) * sp > 256 or K // sp < 256 or (M > 64 and ntw == 4) or (M > 128 and ntw > 1):
                        continue
                    hs.switch("g_skinny_force_ntw", ntw)
                    hs.switch("g_skinny_force_splits", sp)
                    t = hs.time_linear(ctx, M, K, N, copies)
                    if t is not None:
                        forced.append((t, f"ring {64 * ntw} cols x {sp} splits"))
            hs.reset()
            t_plan = min(t_plan, hs.time_linear(ctx, M, K, N, copies))   # first and last measurement of the shape
            rows.append(("decode", name, M, K, N, plan, t_plan, sorted(forced)))
            log(f"[plan_sweep] {name} M={M}: plan {t_plan:.1f} us, {len(forced)} forced plans, best "
                f"{min(forced)[0] if forced else float('nan'):.1f} us")
        for M in prefill_rows:
            hs.reset()
            plan = ctx.ds_linear_plan(M, K, N)
            t_plan = hs.time_linear(ctx, M, K, N, copies)
            forced = []
            hs.switch("g_gemm_tail_split", 0)
            for variant, (bm, bn) in ((1, (256, 160)), (2, (128, 128)), (3, (256, 256)), (5, (128, 256))):
                tiles = -(-M // bm) * -(-N // bn)
                for sp in (1, 2, 4):
                    if sp > 1 and (tiles * sp > 256 or K // (64 * sp) < 8):
                        continue
                    hs.switch("g_gemm_variant", variant)
                    hs.switch("g_gemm_splits", sp)
                    t = hs.time_linear(ctx, M, K, N, copies)
                    if t is not None:
                        forced.append((t, f"{bm}x{bn} x {sp} splits"))
            hs.reset()
            t_plan = min(t_plan, hs.time_linear(ctx, M, K, N, copies))
            rows.append(("prefill", name, M, K, N, plan, t_plan, sorted(forced)))
            log(f"[plan_sweep] {name} M={M}: plan {t_plan:.1f} us, best forced {min(forced)[0]:.1f} us")
        del copies
    return rows


def plan_text(p: dict) -> str:
    if p["streaming"]:
        s = f"streaming, {p['tile_cols']} cols per workgroup"
    else:
        s = f"{p['tile_rows']}x{p['tile_cols']} tiles"
    if p["splits"] > 1:
        s += f", {p['splits']} splits"
    if p["cut_cols"]:
        s += f", cut at column {p['cut_cols']}"
    return s


def to_markdown(model: str, rows, command: str) -> str:
    from . import profile_summary
    out = [f"# GEMM plans against forced alternatives, {model} shapes, one MI355X", "",
           f"Produced by `{command}` (development build of the library, kernel sources "
           f"`{profile_summary.source_stamp()}`); weights rotate over copies of more than 600 MB in total, so nothing "
           "is cache-resident; times are HIP-event means over at least 24 launches, in microseconds (the plan is timed "
           "before and after the forced runs of its shape and the smaller figure kept; run-to-run noise is 2-4 %).", "",
           "\"plan\" is what `ds_linear` does by itself.  For decode sizes the forced alternatives are the split-K ring "
           "kernel at every column-tile width and split count that fits one round of workgroups (where the planner "
           "itself takes the unsplit wave-private-ring kernel - 64 or 80 columns per workgroup, no splits, wide N - "
           "that is the comparison of the two families); for prefill sizes, "
           "every tile at 1, 2 and 4 splits with the column cut switched off.", "",
           "| phase | product | rows | K | N | plan | plan us | best forced | us | plan / best | next best forced |",
           "|---|---|---|---|---|---|---|---|---|---|---|"]
    worst = 0.0
    for phase, name, M, K, N, plan, t_plan, forced in rows:
        best = forced[0] if forced else (float("nan"), "-")
        nxt = ", ".join(f"{d}: {t:.1f}" for t, d in forced[1:4])
        ratio = t_plan / best[0] if forced else float("nan")
        worst = max(worst, ratio) if forced else worst
        out.append(f"| {phase} | {name} | {M} | {K} | {N} | {plan_text(plan)} | {t_plan:.1f} | {best[1]} | {best[0]:.1f} | "
                   f"{ratio:.2f} | {nxt} |")
    out += ["", f"Largest plan / best-forced ratio: {worst:.2f} (1.00 = the planner's choice is the fastest plan there is; "
            "below 1 = the planner's own combination - another kernel family, a column cut - beats every forced one).", ""]
    return "\n".join(out)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--model", default="opt13b", choices=sorted(SHAPES))
    ap.add_argument("--decode-rows", type=int, nargs="*", default=[16, 64, 128])
    ap.add_argument("--prefill-rows", type=int, nargs="*", default=[512, 1024, 2048])
    ap.add_argument("--out", default=None)
    a = ap.parse_args(argv)
    rows = sweep(a.model, a.decode_rows, a.prefill_rows)
    md = to_markdown(a.model, rows, "python -m paper_2401_09670_amd.plan_sweep "
                     + " ".join(argv if argv is not None else sys.argv[1:]))
    if a.out:
        with open(a.out, "w") as f:
            f.write(md)
    else:
        print(md)
    return 0


if __name__ == "__main__":
    sys.exit(main())
