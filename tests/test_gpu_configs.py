"""GPU parity at the shapes of the larger workload configurations (one layer each, real widths and
batch shapes): ragged chatbot-like prefill batches and a 128-wide decode batch at OPT-13B, long
summarization-like prompts at OPT-66B, and one OPT-175B pipeline-stage layer with 8 x 2048 prompts and a
256-wide decode batch over contexts in [128, 2048].  Weights are drawn on the device (seeded) and copied
to the host for the oracle, which computes sampled rows / sequences in float32 (fp64 would need > 30 GB for
the 175B layer); the KV hand-off is compared bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ds_oracle as orc
from paper_2401_09670_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-2


def _prefill_and_check(shape, lw, w32, lens, seed, sample_seqs, rows_per_seq=6):
    ctx = gu.make_ctx(shape)
    t, h = int(sum(lens)), shape.hidden
    x = gu.dev_normal_bits((t, h), 1.0, seed + 100)
    y = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    hkv = shape.kv_heads * shape.head_dim
    k_out = torch.empty(t, hkv, dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty_like(k_out)
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))
    ctx.ds_prefill(lw, x, gu.i32_dev(synth.cu_seqlens(lens)), len(lens), t, int(max(lens)), y, k_out, v_out, ws)
    torch.cuda.synchronize()
    cu = synth.cu_seqlens(lens)
    rng = np.random.default_rng(seed)
    for i in sample_seqs:
        l = int(lens[i])
        r0 = int(cu[i])
        rows = sorted(set([0, l - 1] + [int(r) for r in rng.integers(0, l, size=rows_per_seq)]))
        xs = orc.from_bf16_bits(gu.to_bits(x[r0:r0 + l]), np.float32)
        yr, kr, vr = orc.layer_prefill_rows(w32, xs, rows, shape.n_heads, shape.ln_eps)
        yg = gu.to_f64(y[r0:r0 + l])
        assert gu.rel_err(yg[rows], yr) < TOL, (i, l)
        assert gu.update_ok(yg[rows], yr.astype(np.float64), xs[rows].astype(np.float64)), (i, l)
        assert gu.rel_err(gu.to_f64(k_out[r0:r0 + l]), kr.reshape(l, hkv)) < TOL
        assert gu.rel_err(gu.to_f64(v_out[r0:r0 + l]), vr.reshape(l, hkv)) < TOL
    return ctx, k_out, v_out


def _migrate_and_check(ctx, shape, k_out, v_out, lens, seed, extra=1):
    t = int(sum(lens))
    bt, nblk = synth.make_block_tables([int(l) + extra for l in lens], 16, seed)
    kc = torch.full((nblk, shape.kv_heads, 16, shape.head_dim), 3.0, dtype=torch.bfloat16, device="cuda")
    vc = torch.full_like(kc, 5.0)
    ctx.ds_kv_migrate(k_out, v_out, gu.i32_dev(synth.cu_seqlens(lens)), len(lens), t, int(max(lens)), gu.i32_dev(bt),
                      bt.shape[1], kc, vc, nblk)
    torch.cuda.synchronize()
    kref, vref = gu.to_bits(torch.full_like(kc, 3.0)), gu.to_bits(torch.full_like(vc, 5.0))
    orc.kv_migrate(gu.to_bits(k_out).reshape(t, shape.kv_heads, -1), gu.to_bits(v_out).reshape(t, shape.kv_heads, -1),
                   [int(l) for l in lens], bt, kref, vref)
    assert np.array_equal(gu.to_bits(kc), kref)
    assert np.array_equal(gu.to_bits(vc), vref)


def _decode_and_check(shape, lw, w32, ctx_lens, seed, sample, steps=1):
    ctx = gu.make_ctx(shape)
    B, h, n, s = len(ctx_lens), shape.hidden, shape.n_heads, shape.head_dim
    nk = shape.kv_heads
    bt, nblk = synth.make_block_tables([int(c) + steps for c in ctx_lens], 16, seed)
    # cache contents are an input: every page filled with seeded N(0,1) values on the device
    kc = gu.dev_normal_bits((nblk, nk, 16, s), 1.0, seed + 200)
    vc = gu.dev_normal_bits((nblk, nk, 16, s), 1.0, seed + 201)
    # oracle side: its own small float32 cache holding only the sampled sequences (paging is an index map)
    sbt, snblk = synth.make_block_tables([int(ctx_lens[i]) + steps for i in sample], 16, seed + 1)
    okc = np.zeros((snblk, nk, 16, s), dtype=np.float32)
    ovc = np.zeros_like(okc)
    for r, i in enumerate(sample):
        nb = synth.blocks_needed(int(ctx_lens[i]) + steps, 16)
        okc[sbt[r, :nb]] = orc.from_bf16_bits(gu.to_bits(kc[torch.from_numpy(bt[i, :nb]).long().cuda()]), np.float32)
        ovc[sbt[r, :nb]] = orc.from_bf16_bits(gu.to_bits(vc[torch.from_numpy(bt[i, :nb]).long().cuda()]), np.float32)
    bt_d = gu.i32_dev(bt)
    max_ctx = int(max(ctx_lens)) + steps
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max_ctx))
    cl = np.array(ctx_lens, dtype=np.int32)
    for j in range(steps):
        x = gu.dev_normal_bits((B, h), 1.0, seed + 300 + j)
        y = torch.empty(B, h, dtype=torch.bfloat16, device="cuda")
        ctx.ds_decode_step(lw, x, gu.i32_dev(cl), bt_d, B, bt.shape[1], int(cl.max()) + 1, kc, vc, nblk, y, ws)
        torch.cuda.synchronize()
        xin = orc.from_bf16_bits(gu.to_bits(x[torch.tensor(sample).cuda()]), np.float32)
        yr = orc.layer_decode_cached(w32, xin, [int(cl[i]) for i in sample], sbt, okc, ovc, n, shape.ln_eps)
        yg = gu.to_f64(y)[sample]
        assert gu.rel_err(yg, yr) < TOL, j
        assert gu.update_ok(yg, yr.astype(np.float64), xin.astype(np.float64)), j
        cl = cl + 1


def test_config3_opt13b_chatbot_shapes(gpu):
    cfg = synth.config(2)
    shape, seed = cfg["shape"], cfg["seed"]
    lw, wdev = gu.dev_layer_weights(shape, seed)
    w32 = orc.weights_from_bits(gu.host_weights(wdev), np.float32)
    p = cfg["prompt"]
    lens_all = synth.lognormal_lengths(64, p["median"], p["sigma"], p["lo"], p["hi"], seed)
    batch = synth.token_capped_batches(lens_all, cfg["prefill_token_cap"])[0]     # first FCFS batch under the cap
    lens = [int(lens_all[i]) for i in batch]
    assert sum(lens) <= cfg["prefill_token_cap"] and len(lens) > 4
    shortest, longest = int(np.argmin(lens)), int(np.argmax(lens))
    ctx, k_out, v_out = _prefill_and_check(shape, lw, w32, lens, seed, [shortest, longest])
    _migrate_and_check(ctx, shape, k_out, v_out, lens, seed)
    # decode batch of 128 with chatbot-like contexts (prompt + part of the output already generated)
    o = cfg["output"]
    ctxs = synth.lognormal_lengths(cfg["decode_batch"], p["median"], p["sigma"], p["lo"], p["hi"], seed, stream=1) + \
        synth.lognormal_lengths(cfg["decode_batch"], o["median"], o["sigma"], o["lo"], o["hi"], seed, stream=2) // 2
    _decode_and_check(shape, lw, w32, ctxs, seed, [0, int(np.argmax(ctxs)), int(np.argmin(ctxs))], steps=2)


def test_config4_opt66b_summarization_shapes(gpu):
    cfg = synth.config(3)
    shape, seed = cfg["shape"], cfg["seed"]
    lw, wdev = gu.dev_layer_weights(shape, seed)
    w32 = orc.weights_from_bits(gu.host_weights(wdev), np.float32)
    p = cfg["prompt"]
    lens = [int(v) for v in synth.uniform_lengths(2, p["lo"], p["hi"], seed)]
    ctx, k_out, v_out = _prefill_and_check(shape, lw, w32, lens, seed, [int(np.argmin(lens))], rows_per_seq=4)
    _migrate_and_check(ctx, shape, k_out, v_out, lens, seed)
    o = cfg["output"]
    ctxs = synth.uniform_lengths(cfg["decode_batch"], p["lo"], p["hi"], seed, stream=1) + \
        synth.uniform_lengths(cfg["decode_batch"], o["lo"], o["hi"], seed, stream=2) // 2
    _decode_and_check(shape, lw, w32, ctxs, seed, [1, int(np.argmin(ctxs))], steps=1)


def test_config5_opt175b_stage_layer_shapes(gpu):
    cfg = synth.config(4)
    shape, seed = cfg["shape"], cfg["seed"]
    lw, wdev = gu.dev_layer_weights(shape, seed)
    w32 = orc.weights_from_bits(gu.host_weights(wdev), np.float32)
    lens = cfg["prefill_lens"]
    ctx, k_out, v_out = _prefill_and_check(shape, lw, w32, lens, seed, [5], rows_per_seq=3)
    _migrate_and_check(ctx, shape, k_out, v_out, lens, seed)
    del k_out, v_out
    c = cfg["decode_ctx"]
    ctxs = synth.uniform_lengths(cfg["decode_batch"], c["lo"], c["hi"], seed)
    _decode_and_check(shape, lw, w32, ctxs, seed, [0, int(np.argmin(ctxs))], steps=1)


def test_two_layer_stack_end_to_end(gpu):
    """Layers compose: the GPU's layer-2 output over a short ragged batch against the oracle's own two-layer
    forward (its layer 2 fed by its layer 1), plus decode steps through both layers' caches."""
    shape = synth.ModelShape(hidden=1024, n_heads=8, head_dim=128, ffn=4096, n_layers=2)
    seed, lens, steps = 909, [70, 5, 131], 2
    t, h, B = sum(lens), shape.hidden, len(lens)
    ctx = gu.make_ctx(shape)
    layers = []
    for li in range(2):
        wb = synth.make_layer_weights(shape, seed, layer=li)
        lw, keep = gu.weights_to_dev(wb)
        layers.append((lw, keep, orc.weights_from_bits(wb)))
    xbits = synth.make_activations(t, h, seed)
    cu = gu.i32_dev(synth.cu_seqlens(lens))
    bt, nblk = synth.make_block_tables([l + steps for l in lens], 16, seed)
    bt_d = gu.i32_dev(bt)
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))
    dws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(lens) + steps))
    caches, ocaches = [], []
    xg, xo = gu.to_dev(xbits), orc.from_bf16_bits(xbits)
    for lw, _, w64 in layers:
        y = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
        k_out, v_out = torch.empty_like(y), torch.empty_like(y)
        ctx.ds_prefill(lw, xg, cu, B, t, max(lens), y, k_out, v_out, ws)
        kc = torch.zeros(nblk, shape.n_heads, 16, shape.head_dim, dtype=torch.bfloat16, device="cuda")
        vc = torch.zeros_like(kc)
        ctx.ds_kv_migrate(k_out, v_out, cu, B, t, max(lens), bt_d, bt.shape[1], kc, vc, nblk)
        caches.append((kc, vc))
        yo, ko, vo = orc.layer_prefill(w64, xo, lens, shape.n_heads)
        okc = np.zeros((nblk, shape.n_heads, 16, shape.head_dim))
        ovc = np.zeros_like(okc)
        orc.kv_migrate(ko, vo, lens, bt, okc, ovc)
        ocaches.append((okc, ovc))
        xg, xo = y, yo
    torch.cuda.synchronize()
    assert gu.rel_err(gu.to_f64(xg), xo) < TOL          # two layers of bf16 rounding still inside the budget
    cl = np.array(lens, dtype=np.int32)
    for j in range(steps):
        xb = synth.make_activations(B, h, seed, stream=1 + j)
        xg, xo = gu.to_dev(xb), orc.from_bf16_bits(xb)
        for (lw, _, w64), (kc, vc), (okc, ovc) in zip(layers, caches, ocaches):
            y = torch.empty(B, h, dtype=torch.bfloat16, device="cuda")
            ctx.ds_decode_step(lw, xg, gu.i32_dev(cl), bt_d, B, bt.shape[1], int(cl.max()) + 1, kc, vc, nblk, y, dws)
            xo = orc.layer_decode_cached(w64, xo, cl, bt, okc, ovc, shape.n_heads)
            xg = y
        torch.cuda.synchronize()
        assert gu.rel_err(gu.to_f64(xg), xo) < TOL, j
        cl = cl + 1


@pytest.mark.parametrize("name,hidden,n_heads,ffn", [
    ("opt13b-tp2", 2560, 20, 10240),    # OPT-13B with h, n, m divided by 2
    ("opt66b-tp4", 2304, 18, 9216),     # OPT-66B with h, n, m divided by 4
])
def test_tensor_parallel_shard_shapes(gpu, name, hidden, n_heads, ffn):
    """The shapes one tensor-parallel shard works on under the paper's convention (App. A.1: with tensor
    parallelism h, n and m are divided by the parallel degree): widths that are not multiples of the
    GEMM tiles, on a ragged prefill batch, its hand-off and a 48-wide decode batch.  No collective is
    involved; this is the single shard's arithmetic only."""
    shape = synth.ModelShape(hidden=hidden, n_heads=n_heads, head_dim=128, ffn=ffn)
    seed = 4242 + hidden
    lw, wdev = gu.dev_layer_weights(shape, seed)
    w32 = orc.weights_from_bits(gu.host_weights(wdev), np.float32)
    lens = [700, 129, 1, 512, 33]
    ctx, k_out, v_out = _prefill_and_check(shape, lw, w32, lens, seed, [0, 2, 4])
    _migrate_and_check(ctx, shape, k_out, v_out, lens, seed)
    ctxs = synth.uniform_lengths(48, 1, 900, seed, stream=3)
    _decode_and_check(shape, lw, w32, ctxs, seed, [0, int(np.argmax(ctxs)), int(np.argmin(ctxs))], steps=2)


@pytest.mark.parametrize("hidden,n_heads,ffn,B", [
    (1024, 8, 4096, 200),     # QKV / FFN-in split over K on the tile kernel: K,V arrive through the reduce pass
    (256, 2, 1024, 150),      # too few k-tiles to split: K,V scattered by the tile kernel's own epilogue
    (2048, 16, 8192, 129),    # just past the row count where the weight-streaming kernel hands over
])
def test_decode_step_wide_batches(gpu, hidden, n_heads, ffn, B):
    """Decode batches of more than 128 rows take the MFMA tile kernel (with or without split-K); every
    fusion of the step (KV append, LayerNorm-2) must give the same layer as the oracle's."""
    shape = synth.ModelShape(hidden=hidden, n_heads=n_heads, head_dim=128, ffn=ffn)
    seed = 31337 + hidden
    lw, wdev = gu.dev_layer_weights(shape, seed)
    w64 = orc.weights_from_bits(gu.host_weights(wdev), np.float64)
    ctxs = synth.uniform_lengths(B, 1, 200, seed, stream=5)
    sample = sorted(set([0, B - 1, int(np.argmax(ctxs)), int(np.argmin(ctxs))] +
                        [int(i) for i in np.random.default_rng(seed).integers(0, B, size=12)]))
    _decode_and_check(shape, lw, w64, ctxs, seed, sample, steps=3)


@pytest.mark.parametrize("name,hidden,n_heads,n_kv,head_dim,ffn", [
    ("gqa-small", 512, 8, 2, 64, 1024),          # every row and element against the fp64 oracle
    ("mqa-small", 256, 2, 1, 128, 512),          # one key/value head for all query heads
    ("llama2-70b-like", 8192, 64, 8, 128, 28672),  # that model's attention geometry (sampled rows)
])
def test_grouped_query_attention_layer(gpu, name, hidden, n_heads, n_kv, head_dim, ffn):
    """Fewer key/value heads than query heads (grouped-query attention, named in Sec. 3.2): the QKV
    projection is (n + 2 n_kv) s wide, K/V rows and the paged cache have n_kv heads, query head j reads
    key/value head j / (n / n_kv).  Prefill, the bit-exact hand-off and decode steps of both GEMM kernels
    (64 and 150 rows)."""
    shape = synth.ModelShape(hidden=hidden, n_heads=n_heads, head_dim=head_dim, ffn=ffn, n_kv_heads=n_kv)
    seed = 777 + hidden
    lw, wdev = gu.dev_layer_weights(shape, seed)
    small = hidden <= 512
    wref = orc.weights_from_bits(gu.host_weights(wdev), np.float64 if small else np.float32)
    lens = [70, 5, 131, 1] if small else [300, 17, 129]
    ctx, k_out, v_out = _prefill_and_check(shape, lw, wref, lens, seed, list(range(len(lens))) if small else [1, 2],
                                           rows_per_seq=200 if small else 5)
    assert k_out.shape[1] == n_kv * head_dim
    _migrate_and_check(ctx, shape, k_out, v_out, lens, seed)
    for B in (64, 150):
        ctxs = synth.uniform_lengths(B, 1, 300, seed, stream=B)
        sample = list(range(B)) if small else [0, B - 1, int(np.argmax(ctxs)), int(np.argmin(ctxs))]
        _decode_and_check(shape, lw, wref, ctxs, seed + B, sample, steps=2)
