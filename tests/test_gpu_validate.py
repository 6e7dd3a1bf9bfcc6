"""The debug validation of device index arrays (DS_ERR_BOUNDS) and the defined results of degenerate
inputs.  Every bad input here is caught on the host, before any kernel is launched: the calls return a
status, nothing on the GPU is given an out-of-range index."""
import numpy as np
import pytest
import torch

from oracle import ds_oracle as orc
from paper_2401_09670_amd import binding, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu
DS_ERR_BOUNDS = 5
SHAPE = synth.TINY


def _prefill_args(lens):
    t, h = sum(lens), SHAPE.hidden
    x = gu.to_dev(synth.make_activations(t, h, seed=3))
    y = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    return t, x, y, torch.empty_like(y), torch.empty_like(y)


def _expect_bounds(call, text):
    with pytest.raises(binding.DsError) as e:
        call()
    assert e.value.status == DS_ERR_BOUNDS, str(e.value)
    assert text in str(e.value), str(e.value)


@pytest.mark.parametrize("cu,max_seqlen,text", [
    ([1, 20, 40], 39, "cu_seqlens[0]"),          # does not start at 0
    ([0, 30, 25, 40], 30, "not increasing"),     # a negative length
    ([0, 20, 20, 40], 20, "not increasing"),     # an empty prompt
    ([0, 20, 39], 20, "must be t"),              # does not end at t
    ([0, 35, 40], 30, "max_seqlen"),             # a prompt longer than the bound the grid was sized for
])
def test_prefill_rejects_bad_cu_seqlens(gpu, cu, max_seqlen, text):
    ctx = gu.make_ctx(SHAPE)
    ctx.ds_set_validate(True)
    lw, keep = gu.weights_to_dev(synth.make_layer_weights(SHAPE, 1))
    t, x, y, k, v = _prefill_args([40])
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))
    B = len(cu) - 1
    _expect_bounds(lambda: ctx.ds_prefill(lw, x, gu.i32_dev(cu), B, t, max_seqlen, y, k, v, ws), text)
    q = x
    _expect_bounds(lambda: ctx.ds_prefill_attention(q, q, q, gu.i32_dev(cu), B, t, max_seqlen, y), text)


def test_validation_off_by_default_and_switchable(gpu, monkeypatch):
    lens = [20, 20]
    lw, keep = gu.weights_to_dev(synth.make_layer_weights(SHAPE, 1))
    t, x, y, k, v = _prefill_args(lens)
    good = gu.i32_dev(synth.cu_seqlens(lens))
    short = gu.i32_dev([0, 20, 39])            # harmless for the kernels (one row less), caught only by validation
    ctx = gu.make_ctx(SHAPE)
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))
    ctx.ds_prefill(lw, x, short, 2, t, 20, y, k, v, ws)          # default: not looked at
    ctx.ds_prefill(lw, x, good, 2, t, 20, y, k, v, ws)
    torch.cuda.synchronize()
    want = y.clone()
    monkeypatch.setenv("DS_DEBUG_VALIDATE", "1")
    ctx2 = gu.make_ctx(SHAPE)                  # the environment switch is read when the context is created
    _expect_bounds(lambda: ctx2.ds_prefill(lw, x, short, 2, t, 20, y, k, v, ws), "must be t")
    y.zero_()
    ctx2.ds_prefill(lw, x, good, 2, t, 20, y, k, v, ws)          # valid input: same result with validation on
    torch.cuda.synchronize()
    assert torch.equal(y, want)
    ctx2.ds_set_validate(False)
    ctx2.ds_prefill(lw, x, short, 2, t, 20, y, k, v, ws)


def test_kv_migrate_rejects_bad_block_ids(gpu):
    ctx = gu.make_ctx(SHAPE)
    ctx.ds_set_validate(True)
    lens = [33, 16]
    t = sum(lens)
    ks, vs = synth.make_kv_fill(t, SHAPE, seed=5)
    bt, nblk = synth.make_block_tables(lens, 16, seed=6)
    kc = torch.zeros(nblk, SHAPE.n_heads, 16, SHAPE.head_dim, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    cu = gu.i32_dev(synth.cu_seqlens(lens))

    def call(table, nb=nblk, maxb=None):
        ctx.ds_kv_migrate(gu.to_dev(ks), gu.to_dev(vs), cu, len(lens), t, max(lens), gu.i32_dev(table),
                          table.shape[1] if maxb is None else maxb, kc, vc, nb)

    bad = bt.copy(); bad[0, 2] = nblk              # one past the pool
    _expect_bounds(lambda: call(bad), "block_tables[0][2]")
    bad = bt.copy(); bad[1, 0] = -1                # a page the sequence needs is marked unused
    _expect_bounds(lambda: call(bad), "block_tables[1][0]")
    _expect_bounds(lambda: call(bt, nb=int(bt.max())), "outside")   # pool smaller than the ids in use
    call(bt)                                       # the valid table passes and is bit-exact
    torch.cuda.synchronize()
    kref = np.zeros((nblk, SHAPE.n_heads, 16, SHAPE.head_dim), dtype=np.uint16)
    vref = np.zeros_like(kref)
    orc.kv_migrate(ks, vs, lens, bt, kref, vref)
    assert np.array_equal(gu.to_bits(kc), kref) and np.array_equal(gu.to_bits(vc), vref)


def test_decode_rejects_bad_lengths_and_tables(gpu):
    ctx = gu.make_ctx(SHAPE)
    ctx.ds_set_validate(True)
    lw, keep = gu.weights_to_dev(synth.make_layer_weights(SHAPE, 1))
    B, h = 3, SHAPE.hidden
    ctx_lens = np.array([20, 47, 5], dtype=np.int32)
    bt, nblk = synth.make_block_tables([int(c) + 1 for c in ctx_lens], 16, seed=8)
    kc = torch.zeros(nblk, SHAPE.n_heads, 16, SHAPE.head_dim, dtype=torch.bfloat16, device="cuda")
    vc = torch.zeros_like(kc)
    x = gu.to_dev(synth.make_activations(B, h, seed=9))
    y = torch.empty(B, h, dtype=torch.bfloat16, device="cuda")
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, 48))

    def step(lens, table, max_ctx=48, nb=nblk):
        ctx.ds_decode_step(lw, x, gu.i32_dev(lens), gu.i32_dev(table), B, table.shape[1], max_ctx, kc, vc, nb, y, ws)

    # max_ctx below a real context: without validation the tail pages of that sequence would be dropped silently
    _expect_bounds(lambda: step(ctx_lens, bt, max_ctx=40), "sequence 1")
    _expect_bounds(lambda: step(np.array([20, -1, 5], dtype=np.int32), bt), "sequence 1")
    bad = bt.copy(); bad[2, 0] = nblk + 7
    _expect_bounds(lambda: step(ctx_lens, bad), "block_tables[2][0]")
    bad = bt.copy(); bad[1, 2] = -1                # the page the new token's K,V would be appended to
    _expect_bounds(lambda: step(ctx_lens, bad), "block_tables[1][2]")
    step(ctx_lens, bt)                             # valid
    q = torch.zeros(B, h, dtype=torch.bfloat16, device="cuda")
    _expect_bounds(lambda: ctx.ds_decode_attention(q, gu.i32_dev([21, 49, 6]), gu.i32_dev(bt), B, bt.shape[1], 48,
                                                   kc, vc, nblk, y, ws), "sequence 1")
    torch.cuda.synchronize()


@pytest.mark.parametrize("head_dim,n_heads,n_kv", [(128, 4, 4), (64, 4, 4), (128, 8, 2)])
def test_decode_attention_zero_length_gives_zero(gpu, head_dim, n_heads, n_kv):
    """A sequence with no cached token has nothing to attend over: its output is 0 (not 0/0), with and
    without a split of the KV axis, and its neighbours are unaffected."""
    shape = synth.ModelShape(hidden=n_heads * head_dim, n_heads=n_heads, head_dim=head_dim, ffn=256,
                             n_kv_heads=n_kv)
    ctx = gu.make_ctx(shape)
    for kv_lens in ([0, 37], [2000, 0]):       # the second case splits the KV axis over workgroups
        B, h = len(kv_lens), shape.hidden
        real = [max(l, 1) for l in kv_lens]    # a table row needs a page even for the empty sequence
        bt, nblk = synth.make_block_tables(real, 16, seed=13)
        kf, vf = synth.make_kv_fill(sum(real), shape, seed=14)
        kc = np.full((nblk, n_kv, 16, head_dim), 0x7FC0, dtype=np.uint16)
        vc = np.full_like(kc, 0xFF80)
        orc.kv_migrate(kf, vf, real, bt, kc, vc)
        qb = synth.make_activations(B, h, seed=15)
        o = torch.full((B, h), 7.0, dtype=torch.bfloat16, device="cuda")
        ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(kv_lens)))
        ctx.ds_decode_attention(gu.to_dev(qb), gu.i32_dev(kv_lens), gu.i32_dev(bt), B, bt.shape[1], max(kv_lens),
                                gu.to_dev(kc), gu.to_dev(vc), nblk, o, ws)
        torch.cuda.synchronize()
        got = gu.to_f64(o).reshape(B, n_heads, head_dim)
        q = orc.from_bf16_bits(qb).reshape(B, n_heads, head_dim)
        cu = synth.cu_seqlens(real)
        for i, l in enumerate(kv_lens):
            if l == 0:
                assert np.all(got[i] == 0.0)
            else:
                ref = orc.attention_rows(q[i:i + 1], np.array([l - 1]), orc.from_bf16_bits(kf[cu[i]:cu[i] + l]),
                                         orc.from_bf16_bits(vf[cu[i]:cu[i] + l]))[0]
                assert gu.rel_err(got[i], ref) < 1e-2


@pytest.mark.parametrize("head_dim,n_heads,lens", [(128, 2, [1, 63, 64, 65, 300, 700]), (64, 4, [17, 129, 512])])
def test_attention_weights_sum_to_one_on_the_gpu(gpu, head_dim, n_heads, lens):
    """Pins the softmax denominators of both attention kernels directly: with every value row equal to all
    ones, each output element is the sum of the row's attention weights, which is 1 whatever q and k are
    (one bf16 rounding of the probabilities in the prefill kernel, one of the result)."""
    shape = synth.ModelShape(hidden=n_heads * head_dim, n_heads=n_heads, head_dim=head_dim, ffn=256)
    ctx = gu.make_ctx(shape)
    t, h = sum(lens), shape.hidden
    q = gu.to_dev(synth.make_activations(t, h, seed=61))
    k = gu.to_dev(synth.make_activations(t, h, seed=62))
    ones = torch.ones(t, h, dtype=torch.bfloat16, device="cuda")
    o = torch.zeros(t, h, dtype=torch.bfloat16, device="cuda")
    ctx.ds_prefill_attention(q, k, ones, gu.i32_dev(synth.cu_seqlens(lens)), len(lens), t, max(lens), o)
    torch.cuda.synchronize()
    assert float((o.float() - 1.0).abs().max()) <= 2.0 ** -7      # 2 bf16 roundings near 1

    B = len(lens)
    bt, nblk = synth.make_block_tables(lens, 16, seed=63)
    kf, _ = synth.make_kv_fill(t, shape, seed=64)
    kc = np.zeros((nblk, n_heads, 16, head_dim), dtype=np.uint16)
    vc = np.zeros_like(kc)
    one_bits = np.full((t, n_heads, head_dim), 0x3F80, dtype=np.uint16)
    orc.kv_migrate(kf, one_bits, lens, bt, kc, vc)
    qd = gu.to_dev(synth.make_activations(B, h, seed=65))
    od = torch.zeros(B, h, dtype=torch.bfloat16, device="cuda")
    ws = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(lens)))
    ctx.ds_decode_attention(qd, gu.i32_dev(lens), gu.i32_dev(bt), B, bt.shape[1], max(lens), gu.to_dev(kc),
                            gu.to_dev(vc), nblk, od, ws)
    torch.cuda.synchronize()
    assert float((od.float() - 1.0).abs().max()) <= 2.0 ** -8     # fp32 weights, one bf16 rounding of the result
