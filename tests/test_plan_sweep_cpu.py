"""Host-side pieces of the plan sweep harness (the sweep itself needs a GPU and the development build)."""
from paper_2401_09670_amd import plan_sweep


def test_plan_text_names_what_the_plan_does():
    assert plan_sweep.plan_text(dict(streaming=True, tile_rows=0, tile_cols=80, splits=1, cut_cols=0)) == \
        "streaming, 80 cols per workgroup"
    assert plan_sweep.plan_text(dict(streaming=True, tile_rows=0, tile_cols=128, splits=6, cut_cols=0)) == \
        "streaming, 128 cols per workgroup, 6 splits"
    assert plan_sweep.plan_text(dict(streaming=False, tile_rows=256, tile_cols=256, splits=1, cut_cols=16384)) == \
        "256x256 tiles, cut at column 16384"


def test_markdown_reports_the_worst_ratio_and_every_row():
    plan = dict(streaming=False, tile_rows=256, tile_cols=160, splits=1, cut_cols=0)
    rows = [("prefill", "out-proj", 2048, 5120, 5120, plan, 94.0, [(95.0, "256x160 x 1 splits"), (118.0, "256x256 x 1 splits")]),
            ("decode", "FFN-in", 128, 5120, 20480, dict(plan, streaming=True, tile_rows=0, tile_cols=80), 55.0, []),
            ("decode", "QKV", 64, 5120, 15360, dict(plan, streaming=True, tile_rows=0, tile_cols=64), 44.0,
             [(40.0, "ring 64 cols x 1 splits")])]
    md = plan_sweep.to_markdown("opt13b", rows, "python -m paper_2401_09670_amd.plan_sweep --model opt13b")
    lines = [l for l in md.splitlines() if l.startswith("| prefill") or l.startswith("| decode")]
    assert len(lines) == 3
    assert "| 0.99 |" in lines[0] and "256x256 x 1 splits: 118.0" in lines[0]
    assert "| nan |" in lines[1]                      # nothing could be forced for that shape
    assert "Largest plan / best-forced ratio: 1.10" in md


def test_shapes_are_the_three_opt_models():
    assert plan_sweep.SHAPES == {"opt13b": (5120, 20480), "opt66b": (9216, 36864), "opt175b": (12288, 49152)}
