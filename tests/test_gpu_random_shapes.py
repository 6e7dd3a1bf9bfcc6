"""Seeded sweep of GEMM and attention shapes (valid inputs only) against the oracle: the launch plans
choose among four tile shapes, two kernels, split-K or not and several fused epilogues, and a sweep
reaches combinations the hand-picked cases do not.  Every output buffer carries a guard row that
must stay untouched."""
import numpy as np
import pytest
import torch

from oracle import ds_oracle as orc
from paper_2401_09670_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-2


def _cases(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        rows = int(rng.choice([1, 3, 16, 63, 64, 65, 127, 128, 129, 200, 256, 257, 400, 640, 1000]))
        in_f = int(rng.choice([64, 128, 192, 256, 320, 512, 1024, 2048, 4096]))
        out_f = int(rng.choice([8, 24, 64, 128, 160, 168, 256, 520, 1024, 1288, 2048, 3072, 5120]))
        if rows * in_f * out_f > 3e9:
            continue
        out.append((rows, in_f, out_f, bool(rng.integers(2)), bool(rng.integers(2)), bool(rng.integers(2))))
    return out


@pytest.mark.parametrize("rows,in_f,out_f,bias,relu,residual", _cases(48, 2401))
def test_linear_random_shapes(gpu, rows, in_f, out_f, bias, relu, residual):
    ctx = gu.make_ctx(synth.TINY)
    rng = np.random.Generator(np.random.Philox(key=[rows * 7 + in_f, out_f]))
    xb = synth.f32_to_bf16_bits(rng.standard_normal((rows, in_f), dtype=np.float32))
    wb = synth.f32_to_bf16_bits(rng.standard_normal((out_f, in_f), dtype=np.float32) * 0.05)
    bb = synth.f32_to_bf16_bits(rng.standard_normal(out_f, dtype=np.float32)) if bias else None
    rb = synth.f32_to_bf16_bits(rng.standard_normal((rows, out_f), dtype=np.float32)) if residual else None
    y = torch.full((rows + 1, out_f), 7.0, dtype=torch.bfloat16, device="cuda")
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
    scale = max(float(np.max(np.abs(ref))), 1e-3)
    assert float(np.max(np.abs(got[:rows] - ref))) / scale < TOL


def _attention_cases(count, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        head_dim = int(rng.choice([64, 128]))
        n_kv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 4]))
        nseq = int(rng.integers(1, 6))
        lens = [int(v) for v in rng.choice([1, 2, 15, 16, 17, 63, 64, 65, 127, 128, 129, 255, 300, 513], size=nseq)]
        out.append((head_dim, n_kv * group, n_kv, lens))
    return out


@pytest.mark.parametrize("head_dim,n_heads,n_kv,lens", _attention_cases(16, 9670))
def test_attention_random_shapes(gpu, head_dim, n_heads, n_kv, lens):
    """Prefill attention, then a decode step's attention over the handed-over cache, ragged lengths."""
    shape = synth.ModelShape(hidden=n_heads * head_dim, n_heads=n_heads, head_dim=head_dim, ffn=64 * n_heads,
                             n_kv_heads=n_kv)
    ctx = gu.make_ctx(shape)
    t, h, hk = sum(lens), n_heads * head_dim, n_kv * head_dim
    q = gu.dev_normal_bits((t, h), 1.0, 1 + t)
    k = gu.dev_normal_bits((t, hk), 1.0, 2 + t)
    v = gu.dev_normal_bits((t, hk), 1.0, 3 + t)
    o = torch.full((t + 1, h), 7.0, dtype=torch.bfloat16, device="cuda")
    cu = synth.cu_seqlens(lens)
    ctx.ds_prefill_attention(q, k, v, gu.i32_dev(cu), len(lens), t, max(lens), o)
    torch.cuda.synchronize()
    q64 = gu.to_f64(q).reshape(t, n_heads, head_dim)
    k64 = gu.to_f64(k).reshape(t, n_kv, head_dim)
    v64 = gu.to_f64(v).reshape(t, n_kv, head_dim)
    got = gu.to_f64(o)
    assert np.all(got[t] == 7.0)
    for i, l in enumerate(lens):
        sl = slice(int(cu[i]), int(cu[i]) + l)
        ref = orc.attention_rows(q64[sl], np.arange(l), k64[sl], v64[sl]).reshape(l, h)
        assert gu.rel_err(got[sl], ref) < TOL, (i, l)
    # hand the K/V over and attend with one fresh query per request over all of its tokens
    bt, nblk = synth.make_block_tables(lens, 16, 5 + t)
    kc = torch.zeros(nblk, n_kv, 16, head_dim, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    ctx.ds_kv_migrate(k, v, gu.i32_dev(cu), len(lens), t, max(lens), gu.i32_dev(bt), bt.shape[1], kc, vc, nblk)
    B = len(lens)
    qd = gu.dev_normal_bits((B, h), 1.0, 4 + t)
    od = torch.full((B + 1, h), 7.0, dtype=torch.bfloat16, device="cuda")
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(lens)))
    ctx.ds_decode_attention(qd, gu.i32_dev(lens), gu.i32_dev(bt), B, bt.shape[1], max(lens), kc, vc, nblk, od, ws)
    torch.cuda.synchronize()
    gd = gu.to_f64(od)
    assert np.all(gd[B] == 7.0)
    qd64 = gu.to_f64(qd).reshape(B, n_heads, head_dim)
    for i, l in enumerate(lens):
        sl = slice(int(cu[i]), int(cu[i]) + l)
        ref = orc.attention_rows(qd64[i:i + 1], np.array([l - 1]), k64[sl], v64[sl]).reshape(h)
        assert gu.rel_err(gd[i], ref) < TOL, (i, l)
