"""ds_decode_step_static (the decode step whose scratch is a static device array: no workspace argument,
no allocation) against ds_decode_step on the same inputs, through the C ABI: two calls in a row, the second
on a smaller batch, so that whatever the first left in the shared array is there when the second runs."""
import numpy as np
import pytest
import torch

from paper_2401_09670_amd import binding, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _case(ctx, lw, shape, seed, ctx_lens):
    B, h = len(ctx_lens), shape.hidden
    cap = [int(c) + 1 for c in ctx_lens]
    bt, nblk = synth.make_block_tables(cap, 16, seed)
    kfill, vfill = synth.make_kv_fill(nblk * 16, shape, seed)
    kc0 = gu.to_dev(kfill).view(nblk, 16, shape.kv_heads, shape.head_dim).permute(0, 2, 1, 3).contiguous()
    vc0 = gu.to_dev(vfill).view(nblk, 16, shape.kv_heads, shape.head_dim).permute(0, 2, 1, 3).contiguous()
    x = gu.to_dev(synth.make_activations(B, h, seed, stream=3))
    lens_d, bt_d = gu.i32_dev(ctx_lens), gu.i32_dev(bt)
    max_ctx = max(cap)
    return dict(B=B, x=x, lens=lens_d, bt=bt_d, max_blocks=bt.shape[1], max_ctx=max_ctx, kc0=kc0, vc0=vc0,
                nblk=nblk)


def _run(ctx, lw, c, static):
    kc, vc = c["kc0"].clone(), c["vc0"].clone()
    y = torch.full((c["B"], c["x"].shape[1]), 3.0, dtype=torch.bfloat16, device="cuda")
    if static:
        ctx.ds_decode_step_static(lw, c["x"], c["lens"], c["bt"], c["B"], c["max_blocks"], c["max_ctx"], kc, vc,
                                  c["nblk"], y)
    else:
        ws = gu.workspace(ctx.ds_decode_workspace_bytes(c["B"], c["max_ctx"]))
        ctx.ds_decode_step(lw, c["x"], c["lens"], c["bt"], c["B"], c["max_blocks"], c["max_ctx"], kc, vc, c["nblk"],
                           y, ws)
    torch.cuda.synchronize()
    return y, kc, vc


def test_static_scratch_decode_step_matches_workspace_decode_step(gpu):
    shape = synth.ModelShape(hidden=1024, n_heads=8, head_dim=128, ffn=4096)
    seed = 31337
    ctx = gu.make_ctx(shape)
    lw, keep = gu.weights_to_dev(synth.make_layer_weights(shape, seed))
    # first call: 40 sequences with long contexts (split-K partials and attention partials in the scratch);
    # second call: 3 short sequences (other kernels, other split counts, a much smaller footprint)
    first = _case(ctx, lw, shape, seed, [700 + 13 * i for i in range(40)])
    second = _case(ctx, lw, shape, seed + 1, [5, 31, 16])
    assert ctx.ds_decode_workspace_bytes(first["B"], first["max_ctx"]) <= binding.STATIC_SCRATCH_BYTES
    want1 = _run(ctx, lw, first, static=False)
    want2 = _run(ctx, lw, second, static=False)
    got1 = _run(ctx, lw, first, static=True)
    got2 = _run(ctx, lw, second, static=True)
    for got, want, name in ((got1, want1, "first"), (got2, want2, "second")):
        assert torch.isfinite(got[0].float()).all(), name
        # same kernels on the same inputs, only the scratch address differs: bit-identical
        assert torch.equal(got[0], want[0]), name
        assert torch.equal(got[1], want[1]) and torch.equal(got[2], want[2]), name
    # and once more in the other order, with a second context sharing the device's array
    ctx_b = gu.make_ctx(shape)
    got2b = _run(ctx_b, lw, second, static=True)
    got1b = _run(ctx_b, lw, first, static=True)
    assert torch.equal(got2b[0], want2[0]) and torch.equal(got1b[0], want1[0])


def test_static_scratch_decode_step_replays_from_a_hip_graph(gpu):
    """What the entry point is for: a decode step captured into a HIP graph with no workspace to carry.  Three
    replays, each after eager work that changes the inputs, against ds_decode_step run eagerly on the same inputs."""
    shape = synth.ModelShape(hidden=1024, n_heads=8, head_dim=128, ffn=4096)
    seed = 2718
    ctx = gu.make_ctx(shape)
    lw, keep = gu.weights_to_dev(synth.make_layer_weights(shape, seed))
    c = _case(ctx, lw, shape, seed, [200 + 7 * i for i in range(24)])
    x, lens = c["x"].clone(), c["lens"].clone()
    kc, vc = c["kc0"].clone(), c["vc0"].clone()
    y = torch.empty_like(x)
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(c["B"], c["max_ctx"]))

    def static_step():
        ctx.ds_decode_step_static(lw, x, lens, c["bt"], c["B"], c["max_blocks"], c["max_ctx"], kc, vc, c["nblk"], y)

    def eager(j):
        x.copy_(gu.to_dev(synth.make_activations(c["B"], shape.hidden, seed, stream=20 + j)))
        lens.copy_(c["lens"] - j)           # shorter contexts: still inside every sequence's pages
        kc.copy_(c["kc0"])
        vc.copy_(c["vc0"])
        y.zero_()

    eager(0)
    static_step()                           # warm-up outside the capture
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            static_step()
    torch.cuda.synchronize()
    for j in range(1, 4):
        eager(j)
        ctx.ds_decode_step(lw, x, lens, c["bt"], c["B"], c["max_blocks"], c["max_ctx"], kc, vc, c["nblk"], y, ws)
        torch.cuda.synchronize()
        want_y, want_k, want_v = y.clone(), kc.clone(), vc.clone()
        eager(j)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want_y), j
        assert torch.equal(kc, want_k) and torch.equal(vc, want_v), j


def test_static_scratch_rejects_what_does_not_fit(gpu):
    shape = synth.OPT_13B
    ctx = gu.make_ctx(shape)
    B, max_ctx = 256, 2064
    assert ctx.ds_decode_workspace_bytes(B, max_ctx) > binding.STATIC_SCRATCH_BYTES
    # the size check comes before anything is dereferenced or launched: small dummy buffers suffice
    d = torch.zeros(4096, dtype=torch.bfloat16, device="cuda")
    names = [n for n, _ in binding.LayerWeights._fields_]
    lw, keep = binding.Context.pack_weights({n: d for n in names})
    i = torch.zeros(4096, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.DsError) as e:
        ctx.ds_decode_step_static(lw, d, i, i, B, 130, max_ctx, d, d, 8, d[2048:])
    assert e.value.status == 3 and "static" in str(e.value)
