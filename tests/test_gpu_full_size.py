"""GPU parity at the benchmark's full size (one OPT-13B layer, 4 prompts x 512
tokens, decode batch 64 at context 512, 16-token pages), in the launch
configuration bench.py times.  The oracle computes sampled outputs one by one:
sampled rows of one prompt (all of its K,V), sampled sequences of the decode
batch; the KV hand-off is compared bit for bit over the whole cache."""
import numpy as np
import pytest
import torch

from oracle import ds_oracle as orc
from paper_2401_09670_amd import synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
TOL = 1e-2


@pytest.fixture(scope="module")
def cfg2(gpu):
    cfg = synth.config(1)
    shape, seed = cfg["shape"], cfg["seed"]
    wbits = synth.make_layer_weights(shape, seed)
    lw, keep = gu.weights_to_dev(wbits)
    ctx = gu.make_ctx(shape)
    return dict(cfg=cfg, shape=shape, seed=seed, wbits=wbits, lw=lw, keep=keep, ctx=ctx,
                w64=orc.weights_from_bits(wbits))


def test_prefill_full_size_sampled_rows(cfg2):
    shape, seed, ctx = cfg2["shape"], cfg2["seed"], cfg2["ctx"]
    lens = cfg2["cfg"]["prefill_lens"]
    t, h = sum(lens), shape.hidden
    xbits = synth.make_activations(t, h, seed, stream=100)
    y = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    k_out, v_out = torch.empty_like(y), torch.empty_like(y)
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))
    ctx.ds_prefill(cfg2["lw"], gu.to_dev(xbits), gu.i32_dev(synth.cu_seqlens(lens)), len(lens), t, max(lens), y,
                   k_out, v_out, ws)
    torch.cuda.synchronize()
    # 32 rows of every prompt: both ends, both sides of every 128-row tile edge of the attention kernel, and a
    # seeded draw of the rest; the prompt's K and V are compared in full
    rng = np.random.Generator(np.random.Philox(key=[seed, 77]))
    yg_all, kg_all, vg_all = gu.to_f64(y), gu.to_f64(k_out), gu.to_f64(v_out)
    for seq in range(len(lens)):
        r0, l = sum(lens[:seq]), lens[seq]
        fixed = [0, 1, 63, 64, 127, 128, 255, 256, 383, 384, l - 2, l - 1]
        extra = [int(r) for r in rng.permutation(l) if int(r) not in fixed][:32 - len(fixed)]
        rows = sorted(fixed + extra)
        assert len(rows) == 32
        yr, kr, vr = orc.layer_prefill_rows(cfg2["w64"], orc.from_bf16_bits(xbits[r0:r0 + l]), rows,
                                            shape.n_heads, shape.ln_eps)
        yg = yg_all[r0:r0 + l]
        assert gu.rel_err(yg[rows], yr) < TOL, seq
        assert gu.rel_err_rows(yg[rows], yr) < TOL, seq
        # the layer's own contribution (output minus the residual input) is checked too: the residual
        # stream dominates y, so this is the sharper test of attention + FFN
        xin = orc.from_bf16_bits(xbits[r0:r0 + l])[rows]
        assert gu.update_ok(yg[rows], yr, xin), seq
        assert gu.rel_err(kg_all[r0:r0 + l], kr.reshape(l, h)) < TOL, seq
        assert gu.rel_err(vg_all[r0:r0 + l], vr.reshape(l, h)) < TOL, seq
        # per (token, head) rows of K and V as well: one wrong head must not hide in the tensor's maximum
        assert gu.rel_err_rows(kg_all[r0:r0 + l].reshape(l * shape.n_heads, -1), kr.reshape(l * shape.n_heads, -1)) < 2 * TOL
        assert gu.rel_err_rows(vg_all[r0:r0 + l].reshape(l * shape.n_heads, -1), vr.reshape(l * shape.n_heads, -1)) < 2 * TOL


def test_migrate_full_size_bit_exact(cfg2):
    shape, seed, ctx = cfg2["shape"], cfg2["seed"], cfg2["ctx"]
    lens = cfg2["cfg"]["prefill_lens"]
    t = sum(lens)
    ks, vs = synth.make_kv_fill(t, shape, seed, stream=1)
    bt, nblk = synth.make_block_tables([l + 64 for l in lens], 16, seed)
    kc = np.full((nblk, shape.n_heads, 16, shape.head_dim), 0x7FC1, dtype=np.uint16)
    vc = np.full_like(kc, 0x7FC2)
    kc_d, vc_d = gu.to_dev(kc), gu.to_dev(vc)
    ctx.ds_kv_migrate(gu.to_dev(ks), gu.to_dev(vs), gu.i32_dev(synth.cu_seqlens(lens)), len(lens), t, max(lens),
                      gu.i32_dev(bt), bt.shape[1], kc_d, vc_d, nblk)
    torch.cuda.synchronize()
    orc.kv_migrate(ks, vs, lens, bt, kc, vc)
    assert np.array_equal(gu.to_bits(kc_d), kc)
    assert np.array_equal(gu.to_bits(vc_d), vc)


def test_decode_full_size_sampled_sequences(cfg2):
    shape, seed, ctx = cfg2["shape"], cfg2["seed"], cfg2["ctx"]
    B, ctx0, steps = cfg2["cfg"]["decode_batch"], cfg2["cfg"]["decode_ctx0"], 2
    h, n, s = shape.hidden, shape.n_heads, shape.head_dim
    # cache contents are an input: 8 distinct synthetic sequences, tiled over the batch
    kf8, vf8 = synth.make_kv_fill(8 * ctx0, shape, seed, stream=2)
    bt, nblk = synth.make_block_tables([ctx0 + 64] * B, 16, seed)
    kc = np.zeros((nblk, n, 16, s), dtype=np.uint16)
    vc = np.zeros_like(kc)
    src = lambda a, i: a[(i % 8) * ctx0:(i % 8 + 1) * ctx0]
    for i in range(B):
        orc.kv_migrate(src(kf8, i), src(vf8, i), [ctx0], bt[i:i + 1], kc, vc)
    kc_d, vc_d, bt_d = gu.to_dev(kc), gu.to_dev(vc), gu.i32_dev(bt)
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, ctx0 + 64))
    xs = [synth.make_activations(B, h, seed, stream=300 + j) for j in range(steps)]
    ys = []
    for j in range(steps):
        y = torch.empty(B, h, dtype=torch.bfloat16, device="cuda")
        ctx.ds_decode_step(cfg2["lw"], gu.to_dev(xs[j]), gu.i32_dev([ctx0 + j] * B), bt_d, B, bt.shape[1],
                           ctx0 + j + 1, kc_d, vc_d, nblk, y, ws)
        ys.append(gu.to_f64(y))
    torch.cuda.synchronize()

    sample = [0, 9, 18, 27, 31, 40, 54, 63]     # 8 of the 64 sequences, all 8 distinct cache contents
    sbt, snblk = synth.make_block_tables([ctx0 + steps] * len(sample), 16, seed + 1)
    okc = np.zeros((snblk, n, 16, s))
    ovc = np.zeros_like(okc)
    for r, i in enumerate(sample):
        orc.kv_migrate(orc.from_bf16_bits(src(kf8, i)), orc.from_bf16_bits(src(vf8, i)), [ctx0], sbt[r:r + 1], okc, ovc)
    for j in range(steps):
        xin = orc.from_bf16_bits(xs[j][sample])
        yr = orc.layer_decode_cached(cfg2["w64"], xin, [ctx0 + j] * len(sample), sbt, okc, ovc, n, shape.ln_eps)
        assert gu.rel_err(ys[j][sample], yr) < TOL, j
        assert gu.rel_err_rows(ys[j][sample], yr) < TOL, j
        assert gu.update_ok(ys[j][sample], yr, xin), j
    # the appended K,V rows of the sampled sequences
    got_k = gu.to_bits(kc_d)
    for r, i in enumerate(sample):
        new_g = orc.from_bf16_bits(orc.kv_gather(got_k, bt[i], ctx0 + steps)[ctx0:])
        new_r = orc.kv_gather(okc, sbt[r], ctx0 + steps)[ctx0:]
        assert gu.rel_err(new_g, new_r) < TOL
