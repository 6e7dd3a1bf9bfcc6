#!/usr/bin/env python3
"""Benchmark of the prefill -> KV hand-off -> decode hot path on one MI355X.

Workload (`opt13b-1layer-in512-out64`, the shape of the paper's Fig. 1): ONE OPT-13B
layer (h 5120, 40 heads x 128, FFN 20480, bf16).  One "step" serves a batch of
64 requests with 512 prompt tokens and 64 output tokens each:
  16 x [ ds_prefill(4 prompts x 512) + ds_kv_migrate into the paged cache ]
  64 x   ds_decode_step(B = 64, context 512 -> 576, 16-token pages)
Inputs are seeded synthetic tensors resident in HBM before the timed region.

Prints ONE JSON line: whole-step tokens/s, the per-phase numbers (prefill
tokens/s, decode TPOT, migration GB/s), per-kernel rooflines measured with HIP
events in the same run, and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--small", action="store_true", help="tiny config (debug only; not a valid bench line)")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the side measurements (keeps a profiler's per-kernel averages to the workload itself)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain 1 GiB device copy (known traffic) for calibrating rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2401_09670_amd import binding, cost, synth

    if not torch.cuda.is_available():
        print("bench.py: needs a GPU", file=sys.stderr)
        sys.exit(2)
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()

    cfg = synth.config(0 if args.small else 1)
    shape, seed = cfg["shape"], cfg["seed"]
    h, m, n, s = shape.hidden, shape.ffn, shape.n_heads, shape.head_dim
    lens = cfg["prefill_lens"]
    B_dec, steps_dec = cfg["decode_batch"], cfg["decode_steps"]
    ctx0 = cfg.get("decode_ctx0", lens[0])
    assert all(l == ctx0 for l in lens) and B_dec % len(lens) == 0
    n_prefill = B_dec // len(lens)
    t = sum(lens)
    dev = torch.device("cuda:0")

    def to_dev(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(dev).view(torch.bfloat16)

    # ---------------- inputs (resident in HBM before timing) ----------------
    t_setup = time.time()
    wbits = synth.make_layer_weights(shape, seed)
    wdev = {k: to_dev(v) for k, v in wbits.items()}
    ctx = binding.Context(h, n, s, m, shape.block_size, shape.ln_eps)
    lw, _keep = ctx.pack_weights(wdev)
    x_pre = [to_dev(synth.make_activations(t, h, seed, stream=100 + i)) for i in range(n_prefill)]
    x_dec = to_dev(synth.make_activations(steps_dec * B_dec, h, seed, stream=200)).view(steps_dec, B_dec, h)
    cu = torch.from_numpy(synth.cu_seqlens(lens)).to(dev)
    bt, nblk = synth.make_block_tables([ctx0 + steps_dec] * B_dec, shape.block_size, seed)
    bt_dev = torch.from_numpy(bt).to(dev)
    max_blocks = bt.shape[1]
    k_cache = torch.zeros(nblk, n, shape.block_size, s, dtype=torch.bfloat16, device=dev)
    v_cache = torch.zeros_like(k_cache)
    ctx_all = torch.from_numpy(
        (ctx0 + np.arange(steps_dec, dtype=np.int32))[:, None].repeat(B_dec, axis=1)).to(dev)
    y_pre = torch.empty(t, h, dtype=torch.bfloat16, device=dev)
    k_out = torch.empty(t, h, dtype=torch.bfloat16, device=dev)
    v_out = torch.empty(t, h, dtype=torch.bfloat16, device=dev)
    y_dec = torch.empty(B_dec, h, dtype=torch.bfloat16, device=dev)
    ws_pre = torch.empty(ctx.ds_prefill_workspace_bytes(t), dtype=torch.uint8, device=dev)
    ws_dec = torch.empty(ctx.ds_decode_workspace_bytes(B_dec, ctx0 + steps_dec), dtype=torch.uint8, device=dev)
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def one_step(marks=None):
        """One pass of the whole path.  `marks`, if given, receives events at the phase boundaries."""
        for i in range(n_prefill):
            ctx.ds_prefill(lw, x_pre[i], cu, len(lens), t, max(lens), y_pre, k_out, v_out, ws_pre)
            if marks is not None:
                e = ev(); e.record(); marks["prefill_end"].append(e)
            sl = slice(i * len(lens), (i + 1) * len(lens))
            ctx.ds_kv_migrate(k_out, v_out, cu, len(lens), t, max(lens), bt_dev[sl], max_blocks, k_cache, v_cache,
                              nblk)
            if marks is not None:
                e = ev(); e.record(); marks["migrate_end"].append(e)
        for j in range(steps_dec):
            ctx.ds_decode_step(lw, x_dec[j], ctx_all[j], bt_dev, B_dec, max_blocks, ctx0 + j + 1, k_cache, v_cache,
                               nblk, y_dec, ws_dec)

    if args.copy_calibration:
        a = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        b = torch.empty_like(a)
        a.fill_(1)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        del a, b

    # ---------------- warm-up, then the timed region ----------------
    for _ in range(args.warmup):
        one_step()
    step_marks = [ev() for _ in range(args.steps + 1)]   # events between the steps: recording one does not wait
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    step_marks[0].record()
    for i in range(args.steps):
        one_step()
        step_marks[i + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall * 1e3 / args.steps
    per_step = sorted(step_marks[i].elapsed_time(step_marks[i + 1]) for i in range(args.steps))
    ms_median, ms_min = per_step[len(per_step) // 2], per_step[0]
    tokens_per_step = B_dec * ctx0 + B_dec * steps_dec
    value = tokens_per_step / (ms_per_step * 1e-3)

    # ---------------- per-phase times (events at the phase boundaries, same stream) ----------------
    phase = {"prefill_ms": 0.0, "migrate_ms": 0.0, "decode_ms": 0.0}
    reps = max(1, min(args.steps, 3))
    for _ in range(reps):
        marks = {"prefill_end": [], "migrate_end": []}
        e0 = ev(); e0.record()
        one_step(marks)
        e1 = ev(); e1.record()
        torch.cuda.synchronize()
        prev = e0
        for pe, me in zip(marks["prefill_end"], marks["migrate_end"]):
            phase["prefill_ms"] += prev.elapsed_time(pe)
            phase["migrate_ms"] += pe.elapsed_time(me)
            prev = me
        phase["decode_ms"] += prev.elapsed_time(e1)
    for k in phase:
        phase[k] /= reps

    # ---------------- per-kernel-class times (HIP events around every launch) ----------------
    ctx.ds_profile_enable(True)
    for _ in range(reps):
        one_step()
    torch.cuda.synchronize()
    prof = ctx.ds_profile_collect()
    ctx.ds_profile_enable(False)

    kv_lens_steps = [[ctx0 + j + 1] * B_dec for j in range(steps_dec)]
    work = {   # algorithmic work per step of the whole path, per kernel class
        "gemm": ("mfma", n_prefill * cost.prefill_gemm_flops(t, h, m), cost.PEAK_BF16_FLOPS),
        "prefill_attn": ("mfma", n_prefill * cost.prefill_attention_flops(lens, h), cost.PEAK_BF16_FLOPS),
        "layernorm": ("hbm", (n_prefill * 2 * cost.layernorm_bytes(t, h)
                              + steps_dec * 2 * cost.layernorm_bytes(B_dec, h)), cost.PEAK_HBM_BYTES),
        "kv_migrate": ("hbm", n_prefill * cost.kv_migrate_bytes(t, h), cost.PEAK_HBM_BYTES),
        "skinny_gemm": ("hbm", steps_dec * cost.decode_gemm_bytes(B_dec, h, m), cost.PEAK_HBM_BYTES),
        "decode_attn": ("hbm", sum(cost.decode_attention_bytes(kl, h) for kl in kv_lens_steps), cost.PEAK_HBM_BYTES),
        "kv_append": ("hbm", steps_dec * cost.kv_append_bytes(B_dec, h), cost.PEAK_HBM_BYTES),
    }
    # HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (separate runs of this same
    # command, scaled by a known-size copy); the summary and its commands are kept under profiles/.
    # These are stored figures, not measured in this run: they carry the hash of the kernel sources they were
    # measured on, and are dropped (traffic = null, traffic_source.stale = true) when the sources have changed.
    traffic, traffic_source = {}, None
    tpath = os.path.join(ROOT, "profiles", "bench_opt13b_1layer_hbm_traffic.json")
    if not args.small and os.path.exists(tpath):
        from paper_2401_09670_amd import profile_summary
        with open(tpath) as f:
            stored = json.load(f)
        stale = stored.get("source_stamp") != profile_summary.source_stamp()
        traffic_source = {"file": "profiles/bench_opt13b_1layer_hbm_traffic.json",
                          "measured_on_sources": stored.get("source_stamp"), "stale": stale}
        if not stale:
            per = stored["per_launch"]
            traffic = {k: v["hbm_read_bytes"] + v["hbm_write_bytes"] for k, v in per.items()}
            if "decode_gemm_call" in per:   # the class timed as skinny_gemm = either streaming kernel + its reduce launch
                traffic["skinny_gemm"] = (per["decode_gemm_call"]["hbm_read_bytes"]
                                          + per["decode_gemm_call"]["hbm_write_bytes"])
    kernels = {}
    for name, (bound, amount, peak) in work.items():
        ms, cnt = prof[name]
        ms /= reps
        cnt //= reps
        if cnt == 0 or ms <= 0:
            continue
        rate = amount / (ms * 1e-3)
        unit_scale, unit = (1e12, "TFLOP/s") if bound == "mfma" else (1e9, "GB/s")
        kernels[name] = {"bound": bound, "achieved": round(rate / unit_scale, 2), "peak": peak / unit_scale,
                         "unit": unit, "frac": round(rate / peak, 4), "launches_per_step": int(cnt),
                         "avg_launch_us": round(ms * 1e3 / cnt, 2), "ms_per_step": round(ms, 4),
                         "algorithmic_per_launch": round(amount / cnt),
                         "traffic": traffic.get(name)}
    dominant = max(kernels, key=lambda k: kernels[k]["ms_per_step"])
    roofline = dict(kernels[dominant])
    roofline["kernel"] = dominant
    roofline["traffic_source"] = traffic_source
    roofline["timed_in"] = "a separate pass of the same steps with HIP events around every launch"

    # ---------------- phase metrics ----------------
    prefill_tok_s = n_prefill * t / (phase["prefill_ms"] * 1e-3)
    prefill_flops = n_prefill * (cost.prefill_gemm_flops(t, h, m) + cost.prefill_attention_flops(lens, h))
    decode_bytes = (work["skinny_gemm"][1] + work["decode_attn"][1] + work["kv_append"][1]
                    + steps_dec * 2 * cost.layernorm_bytes(B_dec, h))
    phases = {
        "prefill_tok_per_s_per_layer": round(prefill_tok_s, 1),
        "prefill_ms_per_batch": round(phase["prefill_ms"] / n_prefill, 4),
        "prefill_mfma_frac": round(prefill_flops / (phase["prefill_ms"] * 1e-3) / cost.PEAK_BF16_FLOPS, 4),
        "decode_tpot_ms_per_layer": round(phase["decode_ms"] / steps_dec, 4),
        "decode_tpot_ms_x_layers_projection": round(phase["decode_ms"] / steps_dec * shape.n_layers, 3),
        "decode_hbm_frac": round(decode_bytes / (phase["decode_ms"] * 1e-3) / cost.PEAK_HBM_BYTES, 4),
        "migrate_GB_per_s": round(work["kv_migrate"][1] / (phase["migrate_ms"] * 1e-3) / 1e9, 1),
        "migrate_hbm_frac": round(work["kv_migrate"][1] / (phase["migrate_ms"] * 1e-3) / cost.PEAK_HBM_BYTES, 4),
    }

    # ---------------- extra: the KV hand-off at a size that does not fit the 256 MB last-level cache ----------------
    extras = {}
    if not args.small and not args.no_extras:
        Bm, Lm = 8, 2048                      # 16384 tokens of this layer's K and V: 2 x 168 MB read + written
        tm_ = Bm * Lm
        ks = torch.empty(tm_, h, dtype=torch.bfloat16, device=dev).normal_()
        vs = torch.empty(tm_, h, dtype=torch.bfloat16, device=dev).normal_()
        btm, nblkm = synth.make_block_tables([Lm] * Bm, shape.block_size, seed + 7)
        kcm = torch.empty(nblkm, n, shape.block_size, s, dtype=torch.bfloat16, device=dev)
        vcm = torch.empty_like(kcm)
        cum = torch.from_numpy(synth.cu_seqlens([Lm] * Bm)).to(dev)
        btm_d = torch.from_numpy(btm).to(dev)
        for _ in range(2):
            ctx.ds_kv_migrate(ks, vs, cum, Bm, tm_, Lm, btm_d, btm.shape[1], kcm, vcm, nblkm)
        a, b = ev(), ev()
        a.record()
        for _ in range(5):
            ctx.ds_kv_migrate(ks, vs, cum, Bm, tm_, Lm, btm_d, btm.shape[1], kcm, vcm, nblkm)
        b.record()
        torch.cuda.synchronize()
        msm = a.elapsed_time(b) / 5
        bytes_m = cost.kv_migrate_bytes(tm_, h)
        extras["kv_migrate_16384_tokens"] = {"ms": round(msm, 4), "GB_per_s": round(bytes_m / (msm * 1e-3) / 1e9, 1),
                                             "hbm_frac": round(bytes_m / (msm * 1e-3) / cost.PEAK_HBM_BYTES, 4)}
        del ks, vs, kcm, vcm

        # The prefill GEMM under sustained load with N(0,1)-like operands versus all-zero operands of
        # the same shape: the instruction stream is identical, only the switching activity (hence the
        # power draw and the clock the chip sustains) differs.
        tq = sum(lens)
        yq = torch.empty(tq, 3 * h, dtype=torch.bfloat16, device=dev)
        for name, fill in (("random", None), ("zero", 0.0)):
            xg = torch.empty(tq, h, dtype=torch.bfloat16, device=dev)
            wg = torch.empty(3 * h, h, dtype=torch.bfloat16, device=dev)
            if fill is None:
                xg.normal_()
                wg.normal_(0.0, 0.02)
            else:
                xg.zero_()
                wg.zero_()
            for _ in range(5):
                ctx.ds_linear(xg, wg, None, None, 0, tq, h, 3 * h, yq)
            a, b = ev(), ev()
            a.record()
            for _ in range(20):
                ctx.ds_linear(xg, wg, None, None, 0, tq, h, 3 * h, yq)
            b.record()
            torch.cuda.synchronize()
            msg = a.elapsed_time(b) / 20
            fl = 2.0 * tq * h * 3 * h
            extras["gemm_qkv_%s_operands" % name] = {"ms": round(msg, 4), "TFLOP_per_s": round(fl / (msg * 1e-3) / 1e12, 1),
                                                     "mfma_frac": round(fl / (msg * 1e-3) / cost.PEAK_BF16_FLOPS, 4)}
            del xg, wg
        del yq

        # The token loop's exit (final LayerNorm + logits over OPT's 50272-entry vocabulary + greedy
        # choice) for the decode batch: one more weight-streaming pass, priced like the decode GEMMs.
        vocab = 50272
        wv = torch.empty(vocab, h, dtype=torch.bfloat16, device=dev).normal_(0.0, 0.02)
        xn = torch.empty(B_dec, h, dtype=torch.bfloat16, device=dev).normal_()
        tok = torch.empty(B_dec, dtype=torch.int32, device=dev)
        ws_tok = torch.empty(ctx.ds_next_token_workspace_bytes(B_dec, vocab), dtype=torch.uint8, device=dev)
        for _ in range(3):
            ctx.ds_next_token(xn, None, B_dec, wdev["ln1_g"], wdev["ln1_b"], wv, vocab, tok, None, ws_tok)
        a, b = ev(), ev()
        a.record()
        for _ in range(20):
            ctx.ds_next_token(xn, None, B_dec, wdev["ln1_g"], wdev["ln1_b"], wv, vocab, tok, None, ws_tok)
        b.record()
        torch.cuda.synchronize()
        mst = a.elapsed_time(b) / 20
        bytes_t = 2.0 * vocab * h + 2 * 2.0 * B_dec * h + 8.0 * B_dec
        extras["next_token_b%d_vocab%d" % (B_dec, vocab)] = {
            "ms": round(mst, 4), "GB_per_s": round(bytes_t / (mst * 1e-3) / 1e9, 1),
            "hbm_frac": round(bytes_t / (mst * 1e-3) / cost.PEAK_HBM_BYTES, 4)}
        del wv, xn

        # Grouped-query decode attention (64 query heads on 8 key/value heads, the geometry of a 70B-class
        # grouped-query model; OPT itself is multi-head): the kernel that serves a whole group per pass over
        # the pages, priced by the K/V bytes it has to read once.
        gn, gkv, gB, gctx = 64, 8, 64, 2048
        gctx_ = binding.Context(gn * s, gn, s, 4 * gn * s, shape.block_size, shape.ln_eps, gkv)
        gbt, gnblk = synth.make_block_tables([gctx] * gB, shape.block_size, seed + 9)
        gk = torch.empty(gnblk, gkv, shape.block_size, s, dtype=torch.bfloat16, device=dev).normal_()
        gv = torch.empty_like(gk).normal_()
        gq = torch.empty(gB, gn * s, dtype=torch.bfloat16, device=dev).normal_()
        go = torch.empty_like(gq)
        glens = torch.full((gB,), gctx, dtype=torch.int32, device=dev)
        gbt_d = torch.from_numpy(gbt).to(dev)
        gws = torch.empty(max(gctx_.ds_decode_workspace_bytes(gB, gctx), 256), dtype=torch.uint8, device=dev)
        for _ in range(3):
            gctx_.ds_decode_attention(gq, glens, gbt_d, gB, gbt.shape[1], gctx, gk, gv, gnblk, go, gws)
        a, b = ev(), ev()
        a.record()
        for _ in range(10):
            gctx_.ds_decode_attention(gq, glens, gbt_d, gB, gbt.shape[1], gctx, gk, gv, gnblk, go, gws)
        b.record()
        torch.cuda.synchronize()
        msa = a.elapsed_time(b) / 10
        bytes_a = 2.0 * gB * gctx * gkv * s * 2
        extras["decode_attn_gqa_n64_kv8_b64_ctx2048"] = {
            "ms": round(msa, 4), "GB_per_s": round(bytes_a / (msa * 1e-3) / 1e9, 1),
            "hbm_frac": round(bytes_a / (msa * 1e-3) / cost.PEAK_HBM_BYTES, 4)}
        del gk, gv, gq, go

    # ---------------- CPU oracle on a bounded sample of the same workload ----------------
    cpu_baseline = None
    if not args.no_cpu_baseline:
        cpu_baseline = time_oracle(np, synth, shape, seed, wbits, ctx0, B_dec, lens)

    out = {
        "metric": "prefill tok/s + decode TPOT (ms) at OPT-13B shapes, % of MFMA/HBM roofline",
        "value": round(value, 1),
        "unit": "tokens/s (prompt+generated, one OPT-13B layer: 16x prefill(4x512)+migrate, 64x decode(B=64))",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(ms_median, 4), "ms_per_step_min": round(ms_min, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg["name"], "hidden": h, "heads": n, "head_dim": s, "ffn": m, "layers": 1,
                   "prefill_batches_per_step": n_prefill, "prefill_lens": lens, "decode_batch": B_dec,
                   "decode_steps": steps_dec, "decode_ctx": [ctx0, ctx0 + steps_dec], "kv_page": shape.block_size,
                   "tokens_per_step": tokens_per_step},
        "phases": phases,
        "roofline": roofline,
        "kernels": kernels,
        "kernels_timed_in": "a separate pass of the same steps with HIP events around every launch (event overhead "
                            "included, so the classes sum to slightly more than ms_per_step); phases: a third pass with "
                            "events at the phase boundaries only",
        "extras": extras,
        "cpu_baseline": cpu_baseline,
        "setup_s": round(setup_s, 1),
    }
    print(json.dumps(out))


def time_oracle(np, synth, shape, seed, wbits, ctx0, B_dec, lens):
    """The oracle as it stands (numpy, fp32 variant = the 'plain fp32 CPU decoder layer'), timed on a
    bounded sample with the workload's own mix: 8 prefill batches (+ their hand-off) and 32 decode steps
    of the full decode batch, i.e. one prefill batch per four decode steps as in the timed step."""
    from oracle import ds_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    h, n = shape.hidden, shape.n_heads
    w = orc.weights_from_bits(wbits, np.float32)
    t = sum(lens)
    n_pre, dec_steps = 8, 32
    bt, nblk = synth.make_block_tables([ctx0 + dec_steps] * B_dec, shape.block_size, seed)
    kc = np.zeros((nblk, n, shape.block_size, shape.head_dim), dtype=np.float32)
    vc = np.zeros_like(kc)
    t_prefill = t_migrate = 0.0
    for i in range(n_pre):
        x = orc.from_bf16_bits(synth.make_activations(t, h, seed, stream=100 + i), np.float32)
        t0 = time.perf_counter()
        y, k, v = orc.layer_prefill(w, x, lens, n, shape.ln_eps)
        t_prefill += time.perf_counter() - t0
        rows = slice((i * len(lens)) % B_dec, (i * len(lens)) % B_dec + len(lens))
        t0 = time.perf_counter()
        orc.kv_migrate(k, v, lens, bt[rows], kc, vc)
        t_migrate += time.perf_counter() - t0
    for i in range(n_pre * len(lens), B_dec, len(lens)):   # untimed: give the remaining sequences a cache too
        orc.kv_migrate(k, v, lens, bt[i:i + len(lens)], kc, vc)
    xd = orc.from_bf16_bits(synth.make_activations(dec_steps * B_dec, h, seed, stream=200), np.float32)
    t0 = time.perf_counter()
    for j in range(dec_steps):
        orc.layer_decode_cached(w, xd[j * B_dec:(j + 1) * B_dec], [ctx0 + j] * B_dec, bt, kc, vc, n, shape.ln_eps)
    t_decode = time.perf_counter() - t0
    tokens = n_pre * t + dec_steps * B_dec
    total = t_prefill + t_migrate + t_decode
    return {"value": round(tokens / total, 1), "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": f"numpy fp32 oracle: {n_pre} prefill batches ({len(lens)} prompts x {ctx0} tokens each) + their "
                      f"KV hand-off + {dec_steps} decode steps at B={B_dec}, ctx {ctx0}..{ctx0 + dec_steps}",
            "prefill_tok_per_s": round(n_pre * t / t_prefill, 1),
            "decode_ms_per_step": round(t_decode / dec_steps * 1e3, 1),
            "migrate_GB_per_s": round(n_pre * 2 * 2 * t * h * 4 / t_migrate / 1e9, 3), "seconds": round(total, 2)}


if __name__ == "__main__":
    main()
