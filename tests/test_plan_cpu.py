"""Host-side planning of the linear steps (no GPU): which kernel, tile and split count a product gets.  The
expected plans for the OPT-13B products are the measured optima of a sweep over forced (tile, splits) pairs
with weights not resident in any cache; the rest are properties any plan must have."""
import pytest

from paper_2401_09670_amd import binding

H, M_FFN = 5120, 20480
PRODUCTS = {"qkv": (H, 3 * H), "out": (H, H), "ffn_in": (H, M_FFN), "ffn_out": (M_FFN, H)}


@pytest.fixture(scope="module")
def ctx():
    return binding.Context(H, 40, 128, M_FFN)


def _plan(ctx, rows, name):
    k, n = PRODUCTS[name]
    return ctx.ds_linear_plan(rows, k, n)


def test_decode_sized_products_stream_the_weights(ctx):
    for rows in (1, 16, 64, 128):
        for name in PRODUCTS:
            assert _plan(ctx, rows, name)["streaming"]
    assert not _plan(ctx, 129, "qkv")["streaming"]


def test_opt13b_prefill_plans_at_the_bench_shape(ctx):
    """2048 tokens (4 x 512): the tiles fill their rounds, nothing is split."""
    assert _plan(ctx, 2048, "qkv") == dict(streaming=False, tile_rows=256, tile_cols=256, splits=1, cut_cols=0)
    assert _plan(ctx, 2048, "out") == dict(streaming=False, tile_rows=256, tile_cols=160, splits=1, cut_cols=0)
    # two whole rounds of 256x256 tiles over 16384 columns, the other 4096 columns as one round of 256x160
    assert _plan(ctx, 2048, "ffn_in") == dict(streaming=False, tile_rows=256, tile_cols=256, splits=1, cut_cols=16384)
    assert _plan(ctx, 2048, "ffn_out") == dict(streaming=False, tile_rows=256, tile_cols=160, splits=1, cut_cols=0)


def test_short_prefill_batches_fill_the_chip(ctx):
    """512 and 1024 tokens: the narrow products (5120 output columns) split K until a round is full; the wide
    ones change tile shape instead (Sec. 3.1: how few tokens saturate the GPU)."""
    assert _plan(ctx, 512, "qkv") == dict(streaming=False, tile_rows=128, tile_cols=256, splits=1, cut_cols=0)
    assert _plan(ctx, 512, "ffn_in") == dict(streaming=False, tile_rows=256, tile_cols=160, splits=1, cut_cols=0)
    assert _plan(ctx, 512, "ffn_out") == dict(streaming=False, tile_rows=256, tile_cols=160, splits=4, cut_cols=0)
    assert _plan(ctx, 512, "out")["splits"] == 3
    assert _plan(ctx, 1024, "out") == dict(streaming=False, tile_rows=256, tile_cols=160, splits=2, cut_cols=0)
    assert _plan(ctx, 1024, "ffn_out") == dict(streaming=False, tile_rows=256, tile_cols=160, splits=2, cut_cols=0)
    for rows in (512, 1024):
        for name in PRODUCTS:
            p = _plan(ctx, rows, name)
            k, n = PRODUCTS[name]
            wgs = -(-rows // p["tile_rows"]) * -(-n // p["tile_cols"]) * p["splits"]
            assert wgs >= 190, (rows, name, p)          # at least three quarters of the 256 compute units


@pytest.mark.parametrize("rows", [257, 300, 512, 777, 1024, 1536, 2048, 3738, 4096, 16384])
@pytest.mark.parametrize("k,n", [(5120, 15360), (5120, 5120), (20480, 5120), (9216, 36864), (36864, 9216),
                                 (12288, 12288), (49152, 12288), (256, 768), (64, 4000)])
def test_plan_invariants(ctx, rows, k, n):
    p = ctx.ds_linear_plan(rows, k, n)
    assert not p["streaming"]
    assert (p["tile_rows"], p["tile_cols"]) in {(256, 256), (256, 160), (128, 256), (128, 128), (64, 128)}
    assert 1 <= p["splits"] <= 32
    if p["splits"] > 1:
        assert k // 64 // p["splits"] >= 8                # every split keeps at least 8 k-tiles
        tiles = -(-rows // p["tile_rows"]) * -(-n // p["tile_cols"])
        assert tiles * p["splits"] <= 256 and p["cut_cols"] == 0     # a split launch stays within one round
        # the workspace the call asks for is exactly the partial sums
        assert ctx.ds_linear_workspace_bytes(rows, k, n) == p["splits"] * rows * n * 4
    else:
        assert ctx.ds_linear_workspace_bytes(rows, k, n) == 0
    if p["cut_cols"]:
        assert 0 < p["cut_cols"] < n and p["cut_cols"] % p["tile_cols"] == 0
        head = -(-rows // p["tile_rows"]) * (p["cut_cols"] // p["tile_cols"])
        assert head % 256 == 0 or head <= 256              # the head: whole rounds, or a single one


def test_workspace_sized_for_a_maximum_serves_smaller_batches(ctx):
    big = ctx.ds_prefill_workspace_bytes(2048)
    for t in (257, 512, 1000, 1024, 1536, 2047):
        assert ctx.ds_prefill_workspace_bytes(t) <= big


def test_wide_decode_products_leave_the_unsplit_kernel_when_it_would_need_several_rounds(ctx):
    """64 rows: three rounds of 64-column workgroups re-read the activations three times over (OPT-175B FFN-in),
    two rounds of 64 columns lose to 108 x 2 workgroups of 256 (OPT-66B QKV); two rounds of 80 columns against a
    part-filled round of 256-column tiles stay (OPT-175B QKV, OPT-66B FFN-in), and so does everything at 16 rows."""
    assert ctx.ds_linear_plan(64, 12288, 49152) == dict(streaming=True, tile_rows=0, tile_cols=256, splits=1, cut_cols=0)
    assert ctx.ds_linear_plan(64, 9216, 27648) == dict(streaming=True, tile_rows=0, tile_cols=256, splits=2, cut_cols=0)
    for k, n in ((12288, 36864), (9216, 36864)):
        assert ctx.ds_linear_plan(64, k, n)["tile_cols"] == 80
    for k, n in ((12288, 49152), (9216, 27648)):
        assert ctx.ds_linear_plan(16, k, n) == dict(streaming=True, tile_rows=0, tile_cols=64, splits=1, cut_cols=0)
    # the OPT-13B products fit one round unsplit: 64 and 80 columns per workgroup
    assert ctx.ds_linear_plan(64, 5120, 15360)["tile_cols"] == 64 and ctx.ds_linear_plan(64, 5120, 20480)["tile_cols"] == 80
