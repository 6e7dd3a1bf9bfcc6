"""GPU tests of the whole-stack loop (embedding -> L layers with per-layer KV hand-off -> first token;
continuously refilled decode batch over a paged pool).

Rounding compounds over a deep stack, so parity is gated per layer with teacher forcing: the oracle's
layer k is fed the GPU's input to layer k (and, for a decoding step, the GPU's cache pages), on the first,
middle and last layer; the hand-off is compared bit for bit against the index map on those layers."""
import numpy as np
import pytest
import torch

from oracle import ds_oracle as orc
from paper_2401_09670_amd import instance as inst
from paper_2401_09670_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-2


def _check_prefill_capture(stack, li, cap, seqs, rows_per_seq, dtype, rng):
    shape = stack.shape
    w = orc.weights_from_bits(gu.host_weights(stack._keep[li]), dtype)
    lens = cap["lens"]
    cu = synth.cu_seqlens(lens)
    hkv = shape.kv_heads * shape.head_dim
    for i in seqs:
        l, r0 = int(lens[i]), int(cu[i])
        rows = sorted(set([0, l - 1] + [int(r) for r in rng.integers(0, l, size=rows_per_seq)]))
        xs = orc.from_bf16_bits(gu.to_bits(cap["x"][r0:r0 + l]), dtype)
        yr, kr, vr = orc.layer_prefill_rows(w, xs, rows, shape.n_heads, shape.ln_eps)
        yg = gu.to_f64(cap["y"][r0:r0 + l])
        assert gu.rel_err(yg[rows], yr) < TOL, (li, i)
        assert gu.update_ok(yg[rows], yr.astype(np.float64), xs[rows].astype(np.float64)), (li, i)
        assert gu.rel_err(gu.to_f64(cap["k_out"][r0:r0 + l]), kr.reshape(l, hkv)) < TOL
        assert gu.rel_err(gu.to_f64(cap["v_out"][r0:r0 + l]), vr.reshape(l, hkv)) < TOL


def _check_decode_capture(stack, li, cap, sample, dtype):
    shape = stack.shape
    w = orc.weights_from_bits(gu.host_weights(stack._keep[li]), dtype)
    ctx, table = cap["ctx"], cap["table"]
    # the oracle's own small cache: the sampled sequences' pages as the GPU holds them (teacher forcing)
    caps = [int(ctx[i]) + 1 for i in sample]
    sbt, snblk = synth.make_block_tables(caps, 16, 77)
    okc = np.zeros((snblk, shape.kv_heads, 16, shape.head_dim), dtype=dtype)
    ovc = np.zeros_like(okc)
    for r, i in enumerate(sample):
        nb = synth.blocks_needed(caps[r], 16)
        pages = torch.from_numpy(table[i, :nb].astype(np.int64)).cuda()
        okc[sbt[r, :nb]] = orc.from_bf16_bits(gu.to_bits(cap["k_pool"][pages]), dtype)
        ovc[sbt[r, :nb]] = orc.from_bf16_bits(gu.to_bits(cap["v_pool"][pages]), dtype)
    xin = orc.from_bf16_bits(gu.to_bits(cap["x"][torch.tensor(sample).cuda()]), dtype)
    k_before = okc.copy()
    yr = orc.layer_decode_cached(w, xin, [int(ctx[i]) for i in sample], sbt, okc, ovc, shape.n_heads, shape.ln_eps)
    yg = gu.to_f64(cap["y"])[sample]
    assert gu.rel_err(yg, yr) < TOL, li
    assert gu.update_ok(yg, yr.astype(np.float64), xin.astype(np.float64)), li
    # the row the step appended: the oracle wrote its own K over the GPU's in slot ctx - they must agree
    for r, i in enumerate(sample):
        blk, slot = sbt[r, int(ctx[i]) // 16], int(ctx[i]) % 16
        assert gu.rel_err(k_before[blk, :, slot].astype(np.float64), okc[blk, :, slot].astype(np.float64)) < TOL


@pytest.mark.parametrize("n_kv,overlap", [(0, False), (2, False), (0, True)])   # multi-head; two query heads per
def test_small_stack_runs_a_workload_to_completion_with_layerwise_parity(gpu, n_kv, overlap):   # K/V head; overlapped hand-off
    shape = synth.ModelShape(hidden=512, n_heads=4, head_dim=128, ffn=2048, n_layers=4, n_kv_heads=n_kv)
    L, vocab = 4, 1024
    rng = np.random.default_rng(11)
    reqs = [inst.Request(i, int(rng.integers(1, 150)), int(rng.integers(1, 24))) for i in range(24)]
    life = [synth.blocks_needed(r.prompt_len + r.output_len - 1, 16) for r in reqs]
    pool_blocks = max(life) * 3                                   # tight: admission has to wait for pages
    stack = inst.GpuStack(shape, L, 5, pool_blocks, max_batch=6, max_prefill_tokens=256, max_ctx=max(life) * 16,
                          max_blocks_per_seq=max(life), vocab=vocab, n_pos=64, overlap_handoff=overlap)
    sched = inst.Scheduler(reqs, inst.BlockPool(pool_blocks, 5), 6, 256, 16, max(life))
    stack.capture = {0: [], 2: [], 3: []}
    raw = inst.run_workload(stack, sched)
    assert raw["finished"] == len(reqs) and sched.pool.n_free == pool_blocks
    assert sum(len(p["lens"]) for p in raw["prefills"]) == len(reqs)
    assert sum(s["batch"] for s in raw["steps"]) == sum(r.output_len - 1 for r in reqs)
    assert all(p["ms"] > 0 for p in raw["prefills"]) and all(s["ms"] > 0 for s in raw["steps"])
    res = inst.summarise(raw, shape, L, vocab)
    assert res["prefill"]["tokens"] == sum(r.prompt_len for r in reqs)
    for li, caps in stack.capture.items():
        pre = [c for c in caps if c["kind"] == "prefill"]
        dec = [c for c in caps if c["kind"] == "decode"]
        assert len(pre) == len(raw["prefills"]) and len(dec) == len(raw["steps"])
        for c in pre[:3]:
            _check_prefill_capture(stack, li, c, range(len(c["lens"])), 4, np.float64, rng)
        for c in dec[::max(1, len(dec) // 5)]:
            _check_decode_capture(stack, li, c, list(range(len(c["ctx"]))), np.float64)


@pytest.mark.parametrize("overlap", [False, True])   # hand-off in line, or on a second stream beside the next layer
def test_small_stack_handoff_is_bit_exact_in_every_captured_layer(gpu, overlap):
    shape = synth.ModelShape(hidden=512, n_heads=4, head_dim=128, ffn=2048, n_layers=3)
    lens = [33, 16, 1, 70]
    reqs = [inst.Request(i, l, 1) for i, l in enumerate(lens)]
    pool_blocks = 40
    stack = inst.GpuStack(shape, 3, 9, pool_blocks, max_batch=4, max_prefill_tokens=128, max_ctx=96,
                          max_blocks_per_seq=6, vocab=512, n_pos=128, overlap_handoff=overlap)
    stack.k_pool.fill_(3.0)
    stack.v_pool.fill_(5.0)
    sched = inst.Scheduler(reqs, inst.BlockPool(pool_blocks, 2), 4, 128, 16, 6)
    batch = sched.next_prefill_batch()
    table = sched.prefill_table(batch)
    stack.capture = {0: [], 1: [], 2: []}
    stack.prefill(lens, [s.req.rid for s in batch], table)
    torch.cuda.synchronize()
    for li in range(3):
        cap = stack.capture[li][0]
        kg, vg = gu.to_bits(stack.k_pool[li]), gu.to_bits(stack.v_pool[li])
        kref, vref = gu.to_bits(torch.full_like(stack.k_pool[li], 3.0)), gu.to_bits(torch.full_like(stack.v_pool[li], 5.0))
        orc.kv_migrate(gu.to_bits(cap["k_out"]).reshape(sum(lens), 4, -1), gu.to_bits(cap["v_out"]).reshape(sum(lens), 4, -1),
                       lens, table, kref, vref)
        assert np.array_equal(kg, kref) and np.array_equal(vg, vref)     # sentinel slots untouched too
    # the first generated token of every prompt sits in its decode row: the oracle's greedy choice from the
    # GPU's last-layer output (same precision for the decision: bf16 rows after the final LayerNorm)
    y_last = gu.to_f64(stack.capture[2][0]["y"])
    last_rows = synth.cu_seqlens(lens)[1:] - 1
    logits = orc.next_token_logits(y_last[last_rows], gu.to_f64(stack.lnf_g), gu.to_f64(stack.lnf_b),
                                   gu.to_f64(stack.tok_emb))
    want = orc.greedy(logits)
    got = stack.first_tok[:len(lens)].cpu().numpy()
    for r in range(len(lens)):
        if got[r] != want[r]:
            gap = abs(logits[r, got[r]] - logits[r, want[r]])
            assert gap <= 5e-3 * np.max(np.abs(logits[r])), (r, got[r], want[r])


def test_opt13b_40_layer_stack_first_middle_last_layer_parity(gpu):
    """The chatbot workload's real shape: 40 layers of OPT-13B, a first-come-first-served prefill batch under
    the 4096-token cap, its hand-off, and a decoding step of the admitted requests."""
    cfg = synth.config(2)
    shape, L, seed = cfg["shape"], cfg["layers"], cfg["seed"]
    reqs = inst.requests_for(cfg, 24)
    reqs = [inst.Request(r.rid, r.prompt_len, max(r.output_len, 3)) for r in reqs]
    plan = inst.plan_for(cfg, reqs, pool_gb=20.0)
    stack = inst.GpuStack(shape, L, seed, plan["pool_blocks"], 32, plan["max_prefill_tokens"], plan["max_ctx"],
                          plan["max_blocks"])
    sched = inst.Scheduler(reqs, inst.BlockPool(plan["pool_blocks"], seed), 32, plan["token_cap"], 16,
                           plan["max_blocks"])
    rng = np.random.default_rng(seed)
    layers = [0, L // 2, L - 1]
    stack.capture = {li: [] for li in layers}
    batch = sched.next_prefill_batch()
    lens = [s.req.prompt_len for s in batch]
    assert len(batch) > 4 and sum(lens) <= 4096
    table = sched.prefill_table(batch)
    stack.prefill(lens, [s.req.rid for s in batch], table)
    stack.place(sched.place_ready())
    rows = sched.decode_rows()
    assert len(rows) == len(batch)
    ctx, dtable = sched.prepare_step(rows)
    stack.decode_step(rows, ctx, dtable)
    torch.cuda.synchronize()
    shortest, longest = int(np.argmin(lens)), int(np.argmax(lens))
    for li in layers:
        pre, dec = stack.capture[li]
        assert pre["kind"] == "prefill" and dec["kind"] == "decode"
        _check_prefill_capture(stack, li, pre, [shortest, longest], 3, np.float32, rng)
        _check_decode_capture(stack, li, dec, [0, int(np.argmax(ctx))], np.float32)
    # hand-off of the last layer, whose pool nothing has touched since except the step's appended rows:
    # check the pages of a prompt that ends inside a page and of one page-aligned or long prompt
    pre = stack.capture[L - 1][0]
    cu = synth.cu_seqlens(lens)
    kg = gu.to_bits(stack.k_pool[L - 1])
    ksrc = gu.to_bits(pre["k_out"]).reshape(sum(lens), shape.kv_heads, -1)
    for i in (shortest, longest):
        for j in (0, lens[i] // 2, lens[i] - 1):
            assert np.array_equal(kg[table[i, j // 16], :, j % 16], ksrc[cu[i] + j])


def test_small_stack_decodes_preloaded_contexts(gpu):
    """Decode-only workloads (the OPT-175B stage's decode batch): contexts that no prefill here produced sit in
    pool pages as seeded random K/V; the loop decodes over them with page growth, every step checked per layer."""
    shape = synth.ModelShape(hidden=512, n_heads=4, head_dim=128, ffn=2048, n_layers=3)
    ctxs = [40, 17, 100, 1, 64, 16]
    reqs = [inst.Request(i, c, 4, preloaded=True) for i, c in enumerate(ctxs)]     # 3 decoding steps each
    life = [synth.blocks_needed(c + 3, 16) for c in ctxs]
    pool_blocks = sum(life) + 2
    stack = inst.GpuStack(shape, 3, 21, pool_blocks, max_batch=len(reqs), max_prefill_tokens=16,
                          max_ctx=max(life) * 16, max_blocks_per_seq=max(life), vocab=512, n_pos=128)
    stack.k_pool.fill_(float("nan"))          # what is not filled below must never matter
    stack.v_pool.fill_(float("-inf"))
    sched = inst.Scheduler(reqs, inst.BlockPool(pool_blocks, 3), len(reqs), 16, 16, max(life))
    stack.capture = {0: [], 2: []}
    raw = inst.run_workload(stack, sched)
    assert raw["finished"] == len(reqs) and not raw["prefills"] and len(raw["steps"]) == 3
    assert [s["batch"] for s in raw["steps"]] == [len(reqs)] * 3
    for li, caps in stack.capture.items():
        assert len(caps) == 3
        for c in caps:
            assert np.all(np.isfinite(gu.to_f64(c["y"])))
            _check_decode_capture(stack, li, c, list(range(len(ctxs))), np.float64)


def test_timing_only_mode_cycles_layers_through_fewer_pools(gpu):
    """The labelled timing-only mode (a decode batch whose KV does not fit beside the weights: layers share a
    few pools, outputs are meaningless) on a small stack: it runs every layer at the recipe's contexts, uses
    fewer pools than layers, and prices the step with the bytes of the full batch."""
    shape = synth.ModelShape(hidden=512, n_heads=4, head_dim=128, ffn=2048)
    cfg = dict(name="tiny-summarization", shape=shape, seed=99, layers=5,
               prompt=dict(kind="uniform", lo=100, hi=400), output=dict(kind="uniform", lo=4, hi=32))
    batch, steps = 12, 3
    one_layer_gb = 2 * 2 * shape.kv_heads * shape.head_dim * 16 * (batch * 28) / 1e9      # >= this batch's pages
    r = inst.timing_only_decode(cfg, batch, steps, pool_gb=2.5 * one_layer_gb)
    assert 1 <= r["pool_layers"] < cfg["layers"]
    assert r["steps"] == steps and r["mean_batch"] == batch
    assert 100 <= r["ctx_min"] <= r["ctx_max"] <= 400 + 31
    assert np.isfinite(r["tpot_ms_mean"]) and r["tpot_ms_mean"] > 0
    # the byte count behind the HBM fraction is that of all five layers at the batch's real contexts
    ctx = np.full(batch, r["mean_ctx"] - 1)
    per_step = inst.decode_bytes(ctx, shape, cfg["layers"], inst.VOCAB)
    assert abs(r["gb_per_s"] * 1e9 * r["tpot_ms_mean"] * 1e-3 / per_step - 1) < 0.05
    md = inst.timing_only_markdown(cfg, r, "cmd")
    assert "outputs meaningless" in md and "mod %d" % r["pool_layers"] in md
