"""GPU parity: every kernel and the whole layer, through the C ABI, against the
CPU oracle on the same seeded inputs.  Gate: max|gpu-ref| / max|ref| <= 1e-2 per
tensor for floating point (bf16 storage, fp32 accumulate); bit-exact for the
KV hand-off."""
import numpy as np
import pytest
import torch

from oracle import ds_oracle as orc
from paper_2401_09670_amd import binding, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-2


def small_shape(head_dim, n_heads=4, ffn_mult=4):
    h = head_dim * n_heads
    return synth.ModelShape(hidden=h, n_heads=n_heads, head_dim=head_dim, ffn=ffn_mult * h)


# ------------------------------------------------------------------ KV hand-off
@pytest.mark.parametrize("n_heads,head_dim,lens", [
    (4, 64, [1, 16, 17, 40, 100]),
    (40, 128, [512, 33, 1, 250]),
    (9, 128, [15, 31]),
])
def test_kv_migrate_bit_exact(gpu, n_heads, head_dim, lens):
    shape = synth.ModelShape(hidden=n_heads * head_dim, n_heads=n_heads, head_dim=head_dim, ffn=n_heads * head_dim * 4)
    ctx = gu.make_ctx(shape)
    t = sum(lens)
    ks, vs = synth.make_kv_fill(t, shape, seed=11)
    bt, nblk = synth.make_block_tables(lens, 16, seed=12, spare_blocks=5)
    kc = np.full((nblk, n_heads, 16, head_dim), 0xDEAD, dtype=np.uint16)
    vc = np.full((nblk, n_heads, 16, head_dim), 0xBEEF, dtype=np.uint16)
    kc_d, vc_d = gu.to_dev(kc), gu.to_dev(vc)
    cu = synth.cu_seqlens(lens)
    ctx.ds_kv_migrate(gu.to_dev(ks), gu.to_dev(vs), gu.i32_dev(cu), len(lens), t, max(lens), gu.i32_dev(bt),
                      bt.shape[1], kc_d, vc_d, nblk)
    torch.cuda.synchronize()
    orc.kv_migrate(ks, vs, lens, bt, kc, vc)
    assert np.array_equal(gu.to_bits(kc_d), kc)      # includes the sentinel slots
    assert np.array_equal(gu.to_bits(vc_d), vc)


# ------------------------------------------------------------------ LayerNorm
@pytest.mark.parametrize("rows,h", [(37, 256), (5, 5120), (3, 12288), (2, 64)])
def test_layernorm(gpu, rows, h):
    shape = synth.ModelShape(hidden=h, n_heads=h // 64, head_dim=64, ffn=4 * h)
    ctx = gu.make_ctx(shape)
    xb = synth.make_activations(rows, h, seed=21)
    # one row with a large mean and small spread: catches a one-pass variance
    xb[0] = synth.f32_to_bf16_bits(np.float32(3.0) + synth.bf16_bits_to_f32(xb[0]) * np.float32(0.01))
    rng = np.random.Generator(np.random.Philox(key=[22, h]))
    gb = synth.f32_to_bf16_bits(1 + 0.02 * rng.standard_normal(h, dtype=np.float32))
    bb = synth.f32_to_bf16_bits(0.02 * rng.standard_normal(h, dtype=np.float32))
    out = torch.empty(rows, h, dtype=torch.bfloat16, device="cuda")
    ctx.ds_layernorm(gu.to_dev(xb), gu.to_dev(gb), gu.to_dev(bb), rows, out)
    ref = orc.layernorm(orc.from_bf16_bits(xb), orc.from_bf16_bits(gb), orc.from_bf16_bits(bb), 1e-5)
    assert gu.rel_err(gu.to_f64(out), ref) < TOL


# ------------------------------------------------------------------ GEMMs
def _linear_case(ctx, rows, in_f, out_f, bias, relu, residual, seed):
    rng = np.random.Generator(np.random.Philox(key=[seed, 7]))
    xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, in_f), dtype=np.float32))
    wb = synth.f32_to_bf16_bits(rng.standard_normal((out_f, in_f), dtype=np.float32) * 0.05)
    bb = synth.f32_to_bf16_bits(rng.standard_normal(out_f, dtype=np.float32)) if bias else None
    rb = synth.f32_to_bf16_bits(rng.standard_normal((rows, out_f), dtype=np.float32)) if residual else None
    y = torch.full((rows + 1, out_f), 7.0, dtype=torch.bfloat16, device="cuda")   # guard row
    ws = gu.workspace(ctx.ds_linear_workspace_bytes(rows, in_f, out_f))
    ctx.ds_linear(gu.to_dev(xb), gu.to_dev(wb), None if bb is None else gu.to_dev(bb),
                  None if rb is None else gu.to_dev(rb), int(relu), rows, in_f, out_f, y, ws)
    torch.cuda.synchronize()
    ref = orc.linear(orc.from_bf16_bits(xb), orc.from_bf16_bits(wb), None if bb is None else orc.from_bf16_bits(bb))
    if relu:
        ref = np.maximum(ref, 0)
    if rb is not None:
        ref = ref + orc.from_bf16_bits(rb)
    got = gu.to_f64(y)
    assert np.all(got[rows] == 7.0), "wrote past the last row"
    assert gu.rel_err(got[:rows], ref) < TOL, (rows, in_f, out_f)


@pytest.mark.parametrize("rows,in_f,out_f,bias,relu,residual", [
    (257, 256, 768, True, False, False),      # smallest tile-path case, ragged rows
    (520, 1024, 1288, True, True, False),     # several tiles, ragged rows and columns (1288 = 161*8)
    (2048, 512, 5120, True, False, True),     # the 256x160 tile with exact quantisation
    (700, 320, 160, False, False, True),      # K = 5 k-tiles, one column tile
    (1111, 192, 2048, False, True, False),
    (200, 5120, 5120, True, False, True),     # decode-sized rows on the tile kernel: split over K + reduce pass
    (129, 2048, 256, True, True, False),      # very few tiles: many splits
    (256, 4096, 1032, False, False, False),   # split-K with a ragged last column tile
    (4400, 64, 4000, True, True, False),      # 18 x 16 tiles: a ragged last group of row tiles and a tile count
                                              # that is no multiple of the 256 tiles dealt out together
    (8200, 64, 1296, False, False, True),     # 33 row tiles: two full groups of 16 and a group of one
    (2048, 64, 20480, True, True, True),      # four exact rounds of 256x160 tiles
    (3738, 128, 9216, True, False, True),     # cut at a column with ragged rows (bias and residual follow the cut)
    (1100, 512, 20480, True, True, False),    # 256x256 head, cut at column 12800, ragged rows
    (2048, 1024, 20480, True, True, False),   # two rounds of 256x256 tiles, the last 4096 columns on 256x128 tiles
    (512, 512, 15360, True, False, False),    # the 128x256 tile, unsplit
    (1024, 1024, 5120, False, False, True),   # the 128x256 tile with a residual
    (512, 5120, 5120, True, False, True),     # the 128x256 tile, K split three ways (OPT-13B out-projection at 512 rows)
    (600, 5120, 5128, True, True, False),     # the same with ragged rows and a ragged last column tile
    (1024, 20480, 5120, True, False, True),   # 256x160 tiles, K split in two (OPT-13B FFN-out at 1024 rows)
])
def test_linear_tile_path(gpu, rows, in_f, out_f, bias, relu, residual):
    ctx = gu.make_ctx(synth.TINY)
    _linear_case(ctx, rows, in_f, out_f, bias, relu, residual, seed=rows)


def test_linear_tile_path_cases_cover_every_plan_kind(gpu):
    """The cases above are there for the plans they take: this pins which ones (host-side planning only)."""
    ctx = gu.make_ctx(synth.TINY)
    plan = lambda r, k, n: ctx.ds_linear_plan(r, k, n)
    assert plan(512, 512, 15360) == dict(streaming=False, tile_rows=128, tile_cols=256, splits=1, cut_cols=0)
    assert plan(512, 5120, 5120) == dict(streaming=False, tile_rows=128, tile_cols=256, splits=3, cut_cols=0)
    assert plan(600, 5120, 5128)["splits"] > 1
    assert plan(1024, 20480, 5120) == dict(streaming=False, tile_rows=256, tile_cols=160, splits=2, cut_cols=0)
    assert plan(1100, 512, 20480)["cut_cols"] == 12800 and plan(3738, 128, 9216)["cut_cols"] > 0
    assert plan(2048, 1024, 20480)["cut_cols"] == 16384
    assert plan(2048, 512, 5120)["tile_cols"] == 160 and plan(4400, 64, 4000)["splits"] == 1


@pytest.mark.parametrize("rows,in_f,out_f,bias,relu,residual", [
    (1, 256, 768, True, False, False),
    (2, 1024, 256, True, False, True),
    (17, 512, 1032, False, True, False),      # ragged: 1032 = 16*64 + 8
    (64, 5120, 5120, True, False, True),      # split-K over workgroups
    (100, 2048, 512, True, True, False),
    (256, 1024, 384, True, False, True),
    (33, 320, 256, True, False, False),       # in_f not a multiple of 128 -> tile path
    # wide outputs, unsplit streaming kernel: one instantiation per batch size class (16 / 32 / 64 rows)
    # and column-tile width (64 columns at 10240, 80 at 20480)
    (1, 512, 10240, True, False, False), (16, 256, 20480, True, True, False), (17, 768, 10240, False, False, True),
    (32, 512, 20480, True, False, True), (33, 256, 10240, True, True, False), (9, 1024, 20480, False, False, False),
    (65, 256, 20480, True, True, False), (100, 768, 20480, False, False, True), (128, 512, 20480, True, False, True),
    (128, 512, 10240, True, False, False),    # 64-column shape above 64 rows: stays on the split-K ring kernel
])
def test_linear_skinny_path(gpu, rows, in_f, out_f, bias, relu, residual):
    ctx = gu.make_ctx(synth.TINY)
    _linear_case(ctx, rows, in_f, out_f, bias, relu, residual, seed=1000 + rows)


def test_linear_wide_products_that_need_several_rounds(gpu):
    """Few rows against very many output columns: the unsplit kernel would need three rounds of 64-column
    workgroups, each re-reading the activations, and the plan hands the product to the ring kernel with 256-column
    tiles; two rounds of 80 columns against a part-filled round of 256-column tiles stay on the unsplit kernel.
    Both paths against the oracle, and the plan as ds_linear_plan reports it."""
    ctx = gu.make_ctx(synth.TINY)
    assert ctx.ds_linear_plan(64, 1024, 49152) == dict(streaming=True, tile_rows=0, tile_cols=256, splits=1,
                                                        cut_cols=0)
    assert ctx.ds_linear_plan(64, 1024, 36864) == dict(streaming=True, tile_rows=0, tile_cols=80, splits=1,
                                                        cut_cols=0)
    assert ctx.ds_linear_plan(16, 1024, 49152)["tile_cols"] == 64      # 16 activation rows: re-reading them is cheap
    _linear_case(ctx, 64, 1024, 49152, True, True, False, seed=2001)
    _linear_case(ctx, 40, 1024, 36864, True, False, False, seed=2002)
    _linear_case(ctx, 33, 512, 27648, False, False, False, seed=2003)  # 432 workgroups of 64 columns, or 108 x 2 splits


# ------------------------------------------------------------------ attention
@pytest.mark.parametrize("head_dim,n_heads,lens", [
    (64, 4, [1, 5, 64, 129, 300]),
    (128, 3, [128, 1, 333, 17]),
    (128, 2, [1000]),
])
def test_prefill_attention(gpu, head_dim, n_heads, lens):
    shape = small_shape(head_dim, n_heads)
    ctx = gu.make_ctx(shape)
    t, h = sum(lens), shape.hidden
    qb = synth.make_activations(t, h, seed=31)
    kb = synth.make_activations(t, h, seed=32)
    vb = synth.make_activations(t, h, seed=33)
    o = torch.zeros(t, h, dtype=torch.bfloat16, device="cuda")
    ctx.ds_prefill_attention(gu.to_dev(qb), gu.to_dev(kb), gu.to_dev(vb), gu.i32_dev(synth.cu_seqlens(lens)),
                             len(lens), t, max(lens), o)
    torch.cuda.synchronize()
    q, k, v = (orc.from_bf16_bits(a).reshape(t, n_heads, head_dim) for a in (qb, kb, vb))
    ref = np.empty_like(q)
    r0 = 0
    for l in lens:
        ref[r0:r0 + l] = orc.attention_rows(q[r0:r0 + l], np.arange(l), k[r0:r0 + l], v[r0:r0 + l])
        r0 += l
    assert gu.rel_err(gu.to_f64(o).reshape(t, n_heads, head_dim), ref) < TOL


@pytest.mark.parametrize("n_heads,head_dim", [(64, 128), (128, 64)])
def test_prefill_attention_two_query_tiles_per_workgroup(gpu, n_heads, head_dim):
    """A batch whose K/V (192 MB) no longer fits the last-level cache beside everything else: the launch then runs
    a pair's workgroups back to back, each taking query tile nq-1-r and then tile r.  Ragged on purpose: an odd
    tile count (the middle tile has no mirror image), a one-token and a one-tile request between long ones, a
    last tile of one row.  Sampled rows of every request against the oracle, all heads."""
    lens = [3000, 129, 1, 2100, 640]
    shape = small_shape(head_dim, n_heads)
    ctx = gu.make_ctx(shape)
    t, h = sum(lens), shape.hidden
    assert 4 * t * h > 160e6                      # the size from which the launcher takes this order
    qb = synth.make_activations(t, h, seed=41)
    kb = synth.make_activations(t, h, seed=42)
    vb = synth.make_activations(t, h, seed=43)
    o = torch.full((t, h), 7.0, dtype=torch.bfloat16, device="cuda")
    ctx.ds_prefill_attention(gu.to_dev(qb), gu.to_dev(kb), gu.to_dev(vb), gu.i32_dev(synth.cu_seqlens(lens)),
                             len(lens), t, max(lens), o)
    torch.cuda.synchronize()
    got = gu.to_f64(o).reshape(t, n_heads, head_dim)
    r0 = 0
    for l in lens:
        rows = sorted({r for r in (0, 1, 31, 32, 127, 128, 129, 255, 256, 1023, 1024, 1407, 1408, 1535, 1536,
                                   l // 2, l - 130, l - 129, l - 128, l - 2, l - 1) if 0 <= r < l})
        sl = slice(r0, r0 + l)
        q, k, v = (orc.from_bf16_bits(a[sl]).reshape(l, n_heads, head_dim) for a in (qb, kb, vb))
        ref = orc.attention_rows(q[rows], np.array(rows), k, v)
        assert gu.rel_err(got[sl][rows], ref) < TOL, l
        assert gu.rel_err_rows(got[sl][rows].reshape(len(rows) * n_heads, -1), ref.reshape(len(rows) * n_heads, -1)) < 2 * TOL, l
        r0 += l
    assert torch.isfinite(o.float()).all()        # every row was written


@pytest.mark.parametrize("head_dim,n_heads,kv_lens", [
    (64, 4, [1, 16, 17, 100, 600]),
    (128, 5, [512, 513, 31, 2]),
    (128, 2, [3000]),                       # few (sequence, head) pairs -> KV axis split over workgroups
    (64, 1, [2047, 5]),
])
def test_decode_attention(gpu, head_dim, n_heads, kv_lens):
    shape = small_shape(head_dim, n_heads)
    ctx = gu.make_ctx(shape)
    B, h = len(kv_lens), shape.hidden
    bt, nblk = synth.make_block_tables(kv_lens, 16, seed=41)
    kf, vf = synth.make_kv_fill(sum(kv_lens), shape, seed=42)
    # slots no sequence owns (the tail of a last page, spare pages) hold what a pool's memory may hold after
    # earlier use: NaN and -Inf bit patterns.  Their attention weight is 0, and they must not leak (0 * NaN)
    kc = np.full((nblk, n_heads, 16, head_dim), 0x7FC0, dtype=np.uint16)
    vc = np.full_like(kc, 0xFF80)
    orc.kv_migrate(kf, vf, kv_lens, bt, kc, vc)       # cache contents are an input here
    qb = synth.make_activations(B, h, seed=43)
    o = torch.zeros(B, h, dtype=torch.bfloat16, device="cuda")
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(kv_lens)))
    ctx.ds_decode_attention(gu.to_dev(qb), gu.i32_dev(kv_lens), gu.i32_dev(bt), B, bt.shape[1], max(kv_lens),
                            gu.to_dev(kc), gu.to_dev(vc), nblk, o, ws)
    torch.cuda.synchronize()
    q = orc.from_bf16_bits(qb).reshape(B, n_heads, head_dim)
    cu = synth.cu_seqlens(kv_lens)
    ref = np.empty_like(q)
    for i, l in enumerate(kv_lens):
        ks = orc.from_bf16_bits(kf[cu[i]:cu[i] + l])
        vs = orc.from_bf16_bits(vf[cu[i]:cu[i] + l])
        ref[i] = orc.attention_rows(q[i:i + 1], np.array([l - 1]), ks, vs)[0]
    assert gu.rel_err(gu.to_f64(o).reshape(B, n_heads, head_dim), ref) < TOL


@pytest.mark.parametrize("n_heads,n_kv,kv_lens", [
    (8, 4, [1, 16, 17, 33, 100, 600]),        # 2 query heads per key/value head; odd and even page counts
    (8, 2, [512, 513, 31, 2, 48]),            # 4 per group
    (16, 2, [3000]),                          # 8 per group, one sequence: KV axis split over workgroups
    (10, 2, [2047, 5, 129]),                  # 5 per group (not a power of two): padded head columns stay out
    (16, 1, [300, 40]),                       # 16 per group = a full tile of heads
    (6, 1, [777]),                            # splits with an odd number of pages per split
    (32, 1, [100, 33, 530]),                  # 32 per group: wider than a tile of heads, the per-head kernel serves it
])
def test_decode_attention_grouped_query(gpu, n_heads, n_kv, kv_lens):
    """Query head j reads key/value head j / (n / n_kv) (grouped-query attention, Sec. 3.2); head size 128 takes
    the kernel that serves a whole group per pass over the pages."""
    head_dim = 128
    shape = synth.ModelShape(hidden=n_heads * head_dim, n_heads=n_heads, head_dim=head_dim, ffn=256,
                             n_kv_heads=n_kv)
    ctx = gu.make_ctx(shape)
    B, h = len(kv_lens), shape.hidden
    bt, nblk = synth.make_block_tables(kv_lens, 16, seed=51)
    kf, vf = synth.make_kv_fill(sum(kv_lens), shape, seed=52)
    kc = np.full((nblk, n_kv, 16, head_dim), 0x7FC0, dtype=np.uint16)     # unowned slots: NaN / -Inf
    vc = np.full_like(kc, 0xFF80)
    orc.kv_migrate(kf, vf, kv_lens, bt, kc, vc)
    qb = synth.make_activations(B, h, seed=53)
    o = torch.zeros(B, h, dtype=torch.bfloat16, device="cuda")
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(kv_lens)))
    ctx.ds_decode_attention(gu.to_dev(qb), gu.i32_dev(kv_lens), gu.i32_dev(bt), B, bt.shape[1], max(kv_lens),
                            gu.to_dev(kc), gu.to_dev(vc), nblk, o, ws)
    torch.cuda.synchronize()
    q = orc.from_bf16_bits(qb).reshape(B, n_heads, head_dim)
    cu = synth.cu_seqlens(kv_lens)
    ref = np.empty_like(q)
    for i, l in enumerate(kv_lens):
        ks = orc.from_bf16_bits(kf[cu[i]:cu[i] + l])
        vs = orc.from_bf16_bits(vf[cu[i]:cu[i] + l])
        ref[i] = orc.attention_rows(q[i:i + 1], np.array([l - 1]), ks, vs)[0]
    got = gu.to_f64(o).reshape(B, n_heads, head_dim)
    assert np.all(np.isfinite(got))
    assert gu.rel_err(got, ref) < TOL
    for i in range(B):                       # per sequence too: a short one must not hide behind a long one
        assert gu.rel_err(got[i], ref[i]) < TOL, (i, kv_lens[i])


# ------------------------------------------------------------------ whole path, config 1 (tiny), every element
def run_path(shape, wbits, xbits, lens, steps, seed, decode_x):
    """prefill -> migrate -> `steps` decode steps on the GPU; returns device results as numpy."""
    ctx = gu.make_ctx(shape)
    lw, keep = gu.weights_to_dev(wbits)
    B, t, h = len(lens), sum(lens), shape.hidden
    cu = gu.i32_dev(synth.cu_seqlens(lens))
    x = gu.to_dev(xbits)
    y = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    k_out = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    v_out = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))
    ctx.ds_prefill(lw, x, cu, B, t, max(lens), y, k_out, v_out, ws)
    bt, nblk = synth.make_block_tables([l + steps for l in lens], shape.block_size, seed)
    # the pool starts out as used memory may look (NaN / -Inf everywhere): only slots the path itself has
    # written may ever influence a result
    kc = torch.full((nblk, shape.n_heads, 16, shape.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    vc = torch.full_like(kc, float("-inf"))
    bt_d = gu.i32_dev(bt)
    ctx.ds_kv_migrate(k_out, v_out, cu, B, t, max(lens), bt_d, bt.shape[1], kc, vc, nblk)
    ctx_lens = np.array(lens, dtype=np.int32)
    dws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(lens) + steps))
    ys = []
    for step in range(steps):
        yd = torch.empty(B, h, dtype=torch.bfloat16, device="cuda")
        ctx.ds_decode_step(lw, gu.to_dev(decode_x[step]), gu.i32_dev(ctx_lens), bt_d, B, bt.shape[1],
                           int(ctx_lens.max()) + 1, kc, vc, nblk, yd, dws)
        ys.append(gu.to_f64(yd))
        ctx_lens = ctx_lens + 1
    torch.cuda.synchronize()
    return dict(y=gu.to_f64(y), k=gu.to_f64(k_out), v=gu.to_f64(v_out), kc=gu.to_bits(kc), vc=gu.to_bits(vc),
                k_bits=gu.to_bits(k_out), v_bits=gu.to_bits(v_out), decode=ys, bt=bt, nblk=nblk)


def test_config1_whole_path_every_element(gpu):
    cfg = synth.config(0)
    shape, seed, lens, steps = cfg["shape"], cfg["seed"], cfg["prefill_lens"], cfg["decode_steps"]
    wbits = synth.make_layer_weights(shape, seed)
    xbits = synth.make_activations(sum(lens), shape.hidden, seed)
    dx = [synth.make_activations(len(lens), shape.hidden, seed, stream=1 + s) for s in range(steps)]
    got = run_path(shape, wbits, xbits, lens, steps, seed, dx)

    w = orc.weights_from_bits(wbits)
    y, k, v = orc.layer_prefill(w, orc.from_bf16_bits(xbits), lens, shape.n_heads)
    t = sum(lens)
    assert gu.rel_err(got["y"], y) < TOL
    xin = orc.from_bf16_bits(xbits)          # the residual input dominates y: also gate the layer's own update
    assert gu.update_ok(got["y"], y, xin)
    assert gu.rel_err(got["k"], k.reshape(t, -1)) < TOL
    assert gu.rel_err(got["v"], v.reshape(t, -1)) < TOL
    # decode: the oracle keeps its own fp64 cache, started from its own prefill K,V
    kc = np.zeros((got["nblk"], shape.n_heads, 16, shape.head_dim))
    vc = np.zeros_like(kc)
    orc.kv_migrate(k, v, lens, got["bt"], kc, vc)
    ctx_lens = list(lens)
    for step in range(steps):
        xd = orc.from_bf16_bits(dx[step])
        yr = orc.layer_decode_cached(w, xd, ctx_lens, got["bt"], kc, vc, shape.n_heads)
        assert gu.rel_err(got["decode"][step], yr) < TOL, step
        assert gu.update_ok(got["decode"][step], yr, xd), step
        ctx_lens = [c + 1 for c in ctx_lens]
    # the GPU cache after the run: prefill rows are bit-identical to k_out/v_out, appended rows match the oracle
    kc_bits = np.zeros((got["nblk"], shape.n_heads, 16, shape.head_dim), dtype=np.uint16)
    vc_bits = np.zeros_like(kc_bits)
    orc.kv_migrate(got["k_bits"].reshape(t, shape.n_heads, -1), got["v_bits"].reshape(t, shape.n_heads, -1), lens,
                   got["bt"], kc_bits, vc_bits)
    for i, l in enumerate(lens):
        g = orc.kv_gather(got["kc"], got["bt"][i], l + steps)
        assert np.array_equal(g[:l], orc.kv_gather(kc_bits, got["bt"][i], l))
        ref_new = orc.kv_gather(kc, got["bt"][i], l + steps)[l:]
        assert gu.rel_err(orc.from_bf16_bits(g[l:]), ref_new) < TOL
        gv = orc.kv_gather(got["vc"], got["bt"][i], l + steps)
        assert np.array_equal(gv[:l], orc.kv_gather(vc_bits, got["bt"][i], l))
        assert gu.rel_err(orc.from_bf16_bits(gv[l:]), orc.kv_gather(vc, got["bt"][i], l + steps)[l:]) < TOL


def test_ragged_layer_small(gpu):
    """Ragged prompts (1 token, one tile + 1, several tiles) through prefill -> migrate -> 3 decode steps."""
    shape = synth.ModelShape(hidden=512, n_heads=4, head_dim=128, ffn=1024)
    lens, steps, seed = [1, 129, 300, 16], 3, 77
    wbits = synth.make_layer_weights(shape, seed)
    wbits["b_o"] = None            # a NULL bias
    xbits = synth.make_activations(sum(lens), shape.hidden, seed)
    dx = [synth.make_activations(len(lens), shape.hidden, seed, stream=1 + s) for s in range(steps)]
    got = run_path(shape, {k: v for k, v in wbits.items() if v is not None}, xbits, lens, steps, seed, dx)
    w = orc.weights_from_bits({k: v for k, v in wbits.items() if v is not None})
    y, k, v = orc.layer_prefill(w, orc.from_bf16_bits(xbits), lens, shape.n_heads)
    assert gu.rel_err(got["y"], y) < TOL
    kc = np.zeros((got["nblk"], shape.n_heads, 16, shape.head_dim))
    vc = np.zeros_like(kc)
    orc.kv_migrate(k, v, lens, got["bt"], kc, vc)
    ctx_lens = list(lens)
    for step in range(steps):
        yr = orc.layer_decode_cached(w, orc.from_bf16_bits(dx[step]), ctx_lens, got["bt"], kc, vc, shape.n_heads)
        assert gu.rel_err(got["decode"][step], yr) < TOL, step
        ctx_lens = [c + 1 for c in ctx_lens]


def test_decode_equals_prefill_last_row_on_gpu(gpu):
    """The invariant the method rests on, checked on the GPU path itself: decoding token l with the
    cache of tokens 0..l-1 gives the same row as prefilling l+1 tokens."""
    shape = synth.TINY
    seed, l = 5, 47
    wbits = synth.make_layer_weights(shape, seed)
    xbits = synth.make_activations(l + 1, shape.hidden, seed)
    got_a = run_path(shape, wbits, xbits[:l], [l], 1, seed, [xbits[l:l + 1]])
    got_b = run_path(shape, wbits, xbits, [l + 1], 0, seed, [])
    assert gu.rel_err(got_a["decode"][0][0], got_b["y"][l]) < TOL


# ------------------------------------------------------------------ HIP graph capture
def test_decode_step_replays_identically_from_a_hip_graph(gpu):
    """A serving loop replays the decode step from a captured graph.  The step allocates nothing,
    never synchronises and records no memset, so a capture (after one eager warm-up that sets the
    kernels' LDS attributes) must replay bit-identically: three replays, each after eager work of its own
    that changes the inputs, compared with the eager result on the same inputs."""
    shape = synth.ModelShape(hidden=1024, n_heads=8, head_dim=128, ffn=4096)
    seed, B, ctx0 = 4711, 24, 70
    ctx = gu.make_ctx(shape)
    lw, keep = gu.weights_to_dev(synth.make_layer_weights(shape, seed))
    bt, nblk = synth.make_block_tables([ctx0 + 8] * B, 16, seed)
    bt_d = gu.i32_dev(bt)
    kfill, vfill = synth.make_kv_fill(nblk * 16, shape, seed)
    kc0 = gu.to_dev(kfill).view(nblk, 16, shape.n_heads, shape.head_dim).permute(0, 2, 1, 3).contiguous()
    vc0 = gu.to_dev(vfill).view(nblk, 16, shape.n_heads, shape.head_dim).permute(0, 2, 1, 3).contiguous()
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, ctx0 + 8))
    x = torch.empty(B, shape.hidden, dtype=torch.bfloat16, device="cuda")
    lens = torch.empty(B, dtype=torch.int32, device="cuda")
    kc, vc = kc0.clone(), vc0.clone()
    y = torch.empty_like(x)

    def step():
        ctx.ds_decode_step(lw, x, lens, bt_d, B, bt.shape[1], ctx0 + 8, kc, vc, nblk, y, ws)

    def eager(j):
        x.copy_(gu.to_dev(synth.make_activations(B, shape.hidden, seed, stream=10 + j)))
        lens.fill_(ctx0 + j)
        kc.copy_(kc0)
        vc.copy_(vc0)

    eager(0)
    step()                                  # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for j in range(1, 4):
        eager(j)
        step()
        torch.cuda.synchronize()
        want_y, want_k, want_v = y.clone(), kc.clone(), vc.clone()
        eager(j)                            # same inputs again, caches restored
        y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want_y), j
        assert torch.equal(kc, want_k) and torch.equal(vc, want_v), j


def test_prefill_and_handoff_replay_identically_from_a_hip_graph(gpu):
    """The prefill pass and the KV hand-off behind it, captured together: ragged prompts (tile, split-K and
    ragged-page paths), three replays, each after eager work that changes the input and clears the outputs."""
    shape = synth.ModelShape(hidden=1024, n_heads=8, head_dim=128, ffn=4096)
    seed, lens = 1812, [300, 77, 513]
    t, h = sum(lens), shape.hidden
    ctx = gu.make_ctx(shape)
    lw, keep = gu.weights_to_dev(synth.make_layer_weights(shape, seed))
    cu = gu.i32_dev(synth.cu_seqlens(lens))
    bt, nblk = synth.make_block_tables([l + 16 for l in lens], 16, seed)
    bt_d = gu.i32_dev(bt)
    x = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    y, k_out, v_out = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
    kc = torch.empty(nblk, shape.n_heads, 16, shape.head_dim, dtype=torch.bfloat16, device="cuda")
    vc = torch.empty_like(kc)
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))

    def step():
        ctx.ds_prefill(lw, x, cu, len(lens), t, max(lens), y, k_out, v_out, ws)
        ctx.ds_kv_migrate(k_out, v_out, cu, len(lens), t, max(lens), bt_d, bt.shape[1], kc, vc, nblk)

    def eager(j):
        x.copy_(gu.to_dev(synth.make_activations(t, h, seed, stream=40 + j)))
        for buf in (y, k_out, v_out, kc, vc):
            buf.fill_(float(j))

    eager(0)
    step()                                  # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for j in range(1, 4):
        eager(j)
        step()
        torch.cuda.synchronize()
        want = [b.clone() for b in (y, k_out, v_out, kc, vc)]
        eager(j)
        graph.replay()
        torch.cuda.synchronize()
        for got, w, name in zip((y, k_out, v_out, kc, vc), want, ("y", "k_out", "v_out", "k_cache", "v_cache")):
            assert torch.equal(got, w), (j, name)
