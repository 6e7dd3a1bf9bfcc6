"""The paper's analytical latency model (App. A) fitted to this library's kernels on the GPU at hand,
with the sweeps that feed it (the throughput-vs-batch/length curves of Sec. 3.1/3.2, the saturation
length L_m of Sec. 3.1 and the prefill/decoding interference measurement of Sec. 2.3).

    python -m paper_2401_09670_amd.latency_model [--model opt13b] [--quick] [--out FILE.md]

times one decoder layer through ds_prefill / ds_decode_step (HIP kernels only), fits

    T_prefill = C1 (4 t h^2 + 2 t h m) + C2 (3 h t2 / b) + C3          (App. A.2)
    T_decode  = C4 (4 h^2 + 2 h m) + C5 (3 h t)                        (App. A.3)

by least squares and prints the constants, the residuals and the tables as markdown.
Host-side analysis only: nothing here is on the serving path.
"""
from __future__ import annotations

import argparse
import json
import sys
from typing import Sequence

import numpy as np

ATTN_BLOCK = 64  # b of App. A.2: keys per attention tile in this library's prefill attention kernel


def prefill_features(lens: Sequence[int], h: int, m: int, b: int = ATTN_BLOCK) -> np.ndarray:
    """Regressors of the prefill time of one batch (App. A.2): GEMM work, attention traffic, constant."""
    l = np.asarray(lens, dtype=np.float64)
    t, t2 = l.sum(), (l * l).sum()
    return np.array([t * (4.0 * h * h + 2.0 * h * m), 3.0 * h * t2 / b, 1.0])


def decode_features(ctx_lens: Sequence[int], h: int, m: int) -> np.ndarray:
    """Regressors of one decoding step (App. A.3): weight traffic (constant per model), KV traffic."""
    t = float(np.asarray(ctx_lens, dtype=np.float64).sum())
    return np.array([4.0 * h * h + 2.0 * h * m, 3.0 * h * t])


def fit_least_squares(features, times) -> np.ndarray:
    """Least-squares coefficients through a column-scaled QR factorisation (the regressors differ by
    ~15 orders of magnitude, so columns are normalised first)."""
    a = np.asarray(features, dtype=np.float64)
    y = np.asarray(times, dtype=np.float64)
    if a.ndim != 2 or a.shape[0] != y.shape[0] or a.shape[0] < a.shape[1]:
        raise ValueError("need at least as many measurements as coefficients")
    scale = np.sqrt((a * a).sum(axis=0))
    if np.any(scale == 0):
        raise ValueError("a regressor is identically zero")
    q, r = np.linalg.qr(a / scale)
    rhs = q.T @ y
    c = np.zeros(a.shape[1])
    for i in range(a.shape[1] - 1, -1, -1):       # back substitution
        c[i] = (rhs[i] - r[i, i + 1:] @ c[i + 1:]) / r[i, i]
    return c / scale


def relative_residuals(features, times, coeffs) -> np.ndarray:
    pred = np.asarray(features, dtype=np.float64) @ np.asarray(coeffs, dtype=np.float64)
    return (pred - np.asarray(times, dtype=np.float64)) / np.asarray(times, dtype=np.float64)


def saturation_length(lengths: Sequence[int], tokens_per_s: Sequence[float], frac: float = 0.9) -> int:
    """L_m of Sec. 3.1 read as: the shortest single-request prompt whose prefill throughput reaches
    `frac` of the best throughput seen in the sweep (beyond it, batching only adds latency)."""
    best = max(tokens_per_s)
    for l, r in sorted(zip(lengths, tokens_per_s)):
        if r >= frac * best:
            return int(l)
    return int(max(lengths))


# ------------------------------------------------------------------------------------------------
# GPU sweeps (need the HIP library and a GPU)
# ------------------------------------------------------------------------------------------------
def _time_ms(fn, torch, reps: int, warm: int = 2) -> float:
    for _ in range(warm):
        fn()
    a = torch.cuda.Event(enable_timing=True)
    b = torch.cuda.Event(enable_timing=True)
    a.record()
    for _ in range(reps):
        fn()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / reps


class _Layer:
    """One randomly initialised layer resident on the GPU plus reusable buffers."""

    def __init__(self, shape, seed: int):
        import torch
        from . import binding, synth
        self.torch, self.synth, self.shape = torch, synth, shape
        self.dev = torch.device("cuda:0")
        h, m = shape.hidden, shape.ffn
        g = torch.Generator(device="cuda")
        g.manual_seed(seed)

        def nrm(sh, std, mean=0.0):
            return torch.empty(sh, dtype=torch.float32, device=self.dev).normal_(mean, std, generator=g).to(torch.bfloat16)

        self.gen = g
        w = {"ln1_g": nrm((h,), 0.02, 1.0), "ln1_b": nrm((h,), 0.02), "w_qkv": nrm((3 * h, h), 0.02),
             "b_qkv": nrm((3 * h,), 0.02), "w_o": nrm((h, h), 0.02), "b_o": nrm((h,), 0.02),
             "ln2_g": nrm((h,), 0.02, 1.0), "ln2_b": nrm((h,), 0.02), "w_fc1": nrm((m, h), 0.02),
             "b_fc1": nrm((m,), 0.02), "w_fc2": nrm((h, m), 0.02), "b_fc2": nrm((h,), 0.02)}
        self.ctx = binding.Context(h, shape.n_heads, shape.head_dim, m, shape.block_size, shape.ln_eps)
        self.lw, self._keep = self.ctx.pack_weights(w)
        self.nrm = nrm

    def prefill_fn(self, lens):
        torch, synth, shape = self.torch, self.synth, self.shape
        h, t = shape.hidden, int(sum(lens))
        x = self.nrm((t, h), 1.0)
        cu = torch.from_numpy(synth.cu_seqlens(lens)).to(self.dev)
        y = torch.empty_like(x)
        k = torch.empty_like(x)
        v = torch.empty_like(x)
        ws = torch.empty(self.ctx.ds_prefill_workspace_bytes(t), dtype=torch.uint8, device=self.dev)
        B, mx = len(lens), int(max(lens))
        return lambda: self.ctx.ds_prefill(self.lw, x, cu, B, t, mx, y, k, v, ws)

    def decode_fn(self, B: int, ctx_len: int):
        """One decoding step of B requests that each already hold ctx_len tokens (random cache content)."""
        torch, synth, shape = self.torch, self.synth, self.shape
        h, n, s, bs = shape.hidden, shape.n_heads, shape.head_dim, shape.block_size
        bt, nblk = synth.make_block_tables([ctx_len + 1] * B, bs, 7)
        bt_d = torch.from_numpy(bt).to(self.dev)
        kc = self.nrm((nblk, n, bs, s), 1.0)
        vc = self.nrm((nblk, n, bs, s), 1.0)
        x = self.nrm((B, h), 1.0)
        y = torch.empty_like(x)
        lens = torch.full((B,), ctx_len, dtype=torch.int32, device=self.dev)
        ws = torch.empty(self.ctx.ds_decode_workspace_bytes(B, ctx_len + 1), dtype=torch.uint8, device=self.dev)
        mb = bt.shape[1]
        return lambda: self.ctx.ds_decode_step(self.lw, x, lens, bt_d, B, mb, ctx_len + 1, kc, vc, nblk, y, ws)


def run_sweeps(model: str, quick: bool, log=lambda s: None, interference_lens=None) -> dict:
    """All three sweeps on one layer of `model`.  `interference_lens` overrides the prompt lengths of the
    interference measurement (default: 128 in quick mode, 128 and 1024 otherwise)."""
    import torch
    from . import synth
    shape = {"opt13b": synth.OPT_13B, "opt66b": synth.OPT_66B, "opt175b": synth.OPT_175B, "tiny": synth.TINY}[model]
    h, m = shape.hidden, shape.ffn
    layer = _Layer(shape, 20240109)
    reps = 5 if quick else 10
    out = {"model": model, "quick": bool(quick), "hidden": h, "ffn": m, "heads": shape.n_heads, "attn_block": ATTN_BLOCK}

    # ---- prefill: throughput versus batch size and input length (Sec. 3.1) ----
    lengths = [32, 128, 512, 2048] if quick else [16, 32, 64, 128, 256, 512, 1024, 2048]
    batches = [1, 4] if quick else [1, 2, 4, 8, 16]
    pre = []
    for B in batches:
        for l in lengths:
            if B * l > 16384:
                continue
            ms = _time_ms(layer.prefill_fn([l] * B), torch, reps)
            pre.append({"batch": B, "len": l, "ms": ms, "tok_per_s": B * l / (ms * 1e-3)})
            log("prefill B=%d l=%d: %.3f ms" % (B, l, ms))
    # ragged batches so that t2 is not a function of t alone
    rag = [[2048, 64, 64, 64], [1024, 512, 256, 128, 64, 32], [1536, 512], [300, 700, 1100]]
    for lens in (rag[:2] if quick else rag):
        ms = _time_ms(layer.prefill_fn(lens), torch, reps)
        pre.append({"batch": len(lens), "len": lens, "ms": ms, "tok_per_s": sum(lens) / (ms * 1e-3)})
        log("prefill ragged %s: %.3f ms" % (lens, ms))
    out["prefill"] = pre

    def lens_of(r):
        return r["len"] if isinstance(r["len"], list) else [r["len"]] * r["batch"]

    fp = [prefill_features(lens_of(r), h, m) for r in pre]
    cp = fit_least_squares(fp, [r["ms"] * 1e-3 for r in pre])
    rp = relative_residuals(fp, [r["ms"] * 1e-3 for r in pre], cp)
    out["prefill_fit"] = {"C1_s_per_mac": cp[0], "C2_s_per_elem": cp[1], "C3_s": cp[2],
                          "max_abs_rel_residual": float(np.abs(rp).max()),
                          "median_abs_rel_residual": float(np.median(np.abs(rp))),
                          # compute-bound points only (t >= 512): the model's own premise
                          "max_abs_rel_residual_t_ge_512": float(max(abs(e) for e, r in zip(rp, pre)
                                                                      if sum(lens_of(r)) >= 512))}
    single = [r for r in pre if r["batch"] == 1 and not isinstance(r["len"], list)]
    out["L_m"] = saturation_length([r["len"] for r in single], [r["tok_per_s"] for r in single])

    # ---- decoding: throughput versus batch size and context (Sec. 3.2) ----
    dbatches = [1, 16, 128] if quick else [1, 2, 4, 8, 16, 32, 64, 128, 256]
    dctx = [128, 1024] if quick else [128, 512, 1024, 2048]
    dec = []
    for B in dbatches:
        for c in dctx:
            ms = _time_ms(layer.decode_fn(B, c), torch, reps * 2)
            dec.append({"batch": B, "ctx": c, "ms": ms, "tok_per_s": B / (ms * 1e-3)})
            log("decode B=%d ctx=%d: %.4f ms" % (B, c, ms))
    out["decode"] = dec
    fd = [decode_features([r["ctx"] + 1] * r["batch"], h, m) for r in dec]
    cd = fit_least_squares(fd, [r["ms"] * 1e-3 for r in dec])
    rd = relative_residuals(fd, [r["ms"] * 1e-3 for r in dec], cd)
    out["decode_fit"] = {"C4_s_per_elem": cd[0], "C5_s_per_elem": cd[1],
                         "max_abs_rel_residual": float(np.abs(rd).max()),
                         "median_abs_rel_residual": float(np.median(np.abs(rd)))}

    # ---- interference (Sec. 2.3): a decoding-only step versus the same step with one prefill added,
    #      serialised on the one GPU (this library never mixes the phases inside a kernel) ----
    inter = []
    for l_in in (interference_lens if interference_lens is not None else ([128] if quick else [128, 1024])):
        pf = layer.prefill_fn([l_in])
        ms_pre = _time_ms(pf, torch, reps)
        for B in ([1, 64] if quick else [1, 4, 16, 64, 128]):
            df = layer.decode_fn(B, l_in)
            ms_dec = _time_ms(df, torch, reps * 2)

            def both():
                df()
                pf()
            ms_both = _time_ms(both, torch, reps)
            inter.append({"input_len": l_in, "decode_batch": B, "decode_only_ms": ms_dec, "prefill_only_ms": ms_pre,
                          "decode_plus_one_prefill_ms": ms_both, "slowdown": ms_both / ms_dec})
            log("interference l=%d B=%d: decode %.4f ms, +prefill %.4f ms" % (l_in, B, ms_dec, ms_both))
    out["interference"] = inter
    return out


def to_markdown(res: dict) -> str:
    L = []
    L.append("# Latency model (App. A) fitted to one %s decoder layer on this GPU" % res["model"])
    L.append("")
    L.append("Produced by `python -m paper_2401_09670_amd.latency_model --model %s%s --out <this file>` on one MI355X; "
             "synthetic random weights and activations." % (res["model"], " --quick" if res.get("quick") else ""))
    L.append("")
    L.append("h = %d, m = %d, n = %d; attention block b = %d; times are per layer." % (res["hidden"], res["ffn"], res["heads"], res["attn_block"]))
    pf, df = res["prefill_fit"], res["decode_fit"]
    L.append("")
    L.append("| constant | value | meaning |")
    L.append("|---|---|---|")
    L.append("| C1 | %.4e s per multiply-accumulate | => %.0f TFLOP/s effective GEMM rate (2 flops per MAC) |" % (pf["C1_s_per_mac"], 2.0 / pf["C1_s_per_mac"] / 1e12))
    L.append("| C2 | %.4e s per element | attention term 3 h t2 / b |" % pf["C2_s_per_elem"])
    L.append("| C3 | %.2f us | fixed overhead per prefill batch-layer |" % (pf["C3_s"] * 1e6))
    L.append("| C4 | %.4e s per element | => %.0f GB/s effective weight streaming (2 bytes per element) |" % (df["C4_s_per_elem"], 2.0 / df["C4_s_per_elem"] / 1e9))
    L.append("| C5 | %.4e s per element | KV term 3 h t |" % df["C5_s_per_elem"])
    L.append("")
    L.append("Prefill fit: median |relative residual| %.1f %%, max %.1f %% (max over points with t >= 512: %.1f %%). "
             "Decoding fit: median %.1f %%, max %.1f %%." % (100 * pf["median_abs_rel_residual"], 100 * pf["max_abs_rel_residual"],
                                                            100 * pf["max_abs_rel_residual_t_ge_512"],
                                                            100 * df["median_abs_rel_residual"], 100 * df["max_abs_rel_residual"]))
    L.append("")
    L.append("Saturation length L_m (single request, 90 %% of the best prefill throughput): **%d tokens**." % res["L_m"])
    L.append("")
    L.append("## Prefill: tokens/s per layer versus batch and input length")
    L.append("")
    L.append("| batch | input length | ms | tokens/s |")
    L.append("|---|---|---|---|")
    for r in res["prefill"]:
        L.append("| %d | %s | %.3f | %.0f |" % (r["batch"], r["len"], r["ms"], r["tok_per_s"]))
    L.append("")
    L.append("## Decoding: tokens/s per layer versus batch and context")
    L.append("")
    L.append("| batch | context | ms per step | tokens/s |")
    L.append("|---|---|---|---|")
    for r in res["decode"]:
        L.append("| %d | %d | %.4f | %.0f |" % (r["batch"], r["ctx"], r["ms"], r["tok_per_s"]))
    L.append("")
    L.append("## Interference: decoding-only step versus the same step plus one prefill (serialised)")
    L.append("")
    L.append("| input length | decode batch | decode only ms | prefill only ms | decode + one prefill ms | slowdown of the decode step |")
    L.append("|---|---|---|---|---|---|")
    for r in res["interference"]:
        L.append("| %d | %d | %.4f | %.4f | %.4f | %.1fx |" % (r["input_len"], r["decode_batch"], r["decode_only_ms"],
                                                            r["prefill_only_ms"], r["decode_plus_one_prefill_ms"], r["slowdown"]))
    L.append("")
    return "\n".join(L)


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("--model", default="opt13b", choices=["tiny", "opt13b", "opt66b", "opt175b"])
    ap.add_argument("--quick", action="store_true", help="a coarse grid (a minute instead of several)")
    ap.add_argument("--out", default=None, help="write the markdown report here (default: stdout)")
    ap.add_argument("--json", default=None, help="also write the raw measurements here")
    args = ap.parse_args(argv)
    res = run_sweeps(args.model, args.quick, log=lambda s: print(s, file=sys.stderr, flush=True))
    md = to_markdown(res)
    if args.out:
        with open(args.out, "w") as f:
            f.write(md)
    else:
        print(md)
    if args.json:
        with open(args.json, "w") as f:
            json.dump(res, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
