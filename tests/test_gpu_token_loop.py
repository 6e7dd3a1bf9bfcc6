"""GPU parity of the two ends of the token loop (Sec. 2.1): the embedding gather and the greedy choice
of the next token (final LayerNorm -> logits over the vocabulary -> argmax), against the oracle.

The argmax is an integer decided by floating point.  Both sides decide at the same precision (hidden
rows rounded to bf16 after the LayerNorm); what remains is the accumulation order and rare 1-ulp
differences of that rounding.  So the test demands the same id, or - where the ids differ - that the
oracle's logits of the two ids are within 5e-3 of the row's largest |logit| (a valid alternative), and
it always checks the returned logit value.  Exact ties (duplicated vocabulary rows) must go to the lowest
id."""
import numpy as np
import pytest
import torch

from oracle import ds_oracle as orc
from paper_2401_09670_amd import binding, synth
from tests import gpu_util as gu

pytestmark = pytest.mark.gpu


def _ctx(h, n_heads, head_dim, ffn):
    return binding.Context(h, n_heads, head_dim, ffn, 16, 1e-5)


@pytest.mark.parametrize("h,vocab,n_pos,rows,with_pos", [
    (256, 1000, 64, 1, True), (256, 1000, 64, 37, True), (256, 1000, 64, 300, False),
    (5120, 50272, 2050, 2048, True),
])
def test_embed(h, vocab, n_pos, rows, with_pos):
    ctx = _ctx(h, h // 64, 64, 4 * h) if h == 256 else _ctx(h, 40, 128, 4 * h)
    te = gu.dev_normal_bits((vocab, h), 0.05, 1)
    pe = gu.dev_normal_bits((n_pos, h), 0.05, 2) if with_pos else None
    rng = np.random.default_rng(3)
    ids = rng.integers(0, vocab, size=rows)
    pos = rng.integers(0, n_pos, size=rows)
    ids[0], ids[-1] = 0, vocab - 1                      # both ends of the table
    pos[0], pos[-1] = n_pos - 1, 0
    x = torch.full((rows, h), 7.0, dtype=torch.bfloat16, device="cuda")
    ctx.ds_embed(gu.i32_dev(ids), gu.i32_dev(pos) if with_pos else None, te, vocab, pe, n_pos if with_pos else 0,
                 rows, x)
    torch.cuda.synchronize()
    ref = orc.embed(gu.to_f64(te), gu.to_f64(pe) if with_pos else None, ids, pos)
    got = gu.to_f64(x)
    if with_pos:   # one bf16 rounding of the sum
        assert np.all(np.abs(got - ref) <= 2.0 ** -8 * np.abs(ref) + 1e-30)
    else:          # a pure copy
        assert np.array_equal(got, ref)


def test_embed_clamps_out_of_range_ids():
    h, vocab, n_pos = 256, 100, 10
    ctx = _ctx(h, 4, 64, 1024)
    te, pe = gu.dev_normal_bits((vocab, h), 0.05, 1), gu.dev_normal_bits((n_pos, h), 0.05, 2)
    x = torch.empty(4, h, dtype=torch.bfloat16, device="cuda")
    ctx.ds_embed(gu.i32_dev([-5, vocab + 3, 0, vocab - 1]), gu.i32_dev([n_pos + 9, -1, 0, n_pos - 1]), te, vocab, pe,
                 n_pos, 4, x)
    y = torch.empty_like(x)
    ctx.ds_embed(gu.i32_dev([0, vocab - 1, 0, vocab - 1]), gu.i32_dev([n_pos - 1, 0, 0, n_pos - 1]), te, vocab, pe,
                 n_pos, 4, y)
    torch.cuda.synchronize()
    assert torch.equal(x, y)


def _check_choice(tok, best, logits):
    """tok/best from the GPU, logits from the oracle ([rows, vocab] float64)."""
    want = orc.greedy(logits)
    top = np.max(np.abs(logits), axis=1)
    r = np.arange(logits.shape[0])
    assert np.all((tok >= 0) & (tok < logits.shape[1]))
    gap = logits[r, want] - logits[r, tok]
    assert np.all(gap <= 5e-3 * top), (np.max(gap / top), int(np.sum(tok != want)))
    assert np.all(np.abs(best - logits[r, want]) <= 1e-2 * top)
    return int(np.sum(tok != want))


def _oracle_logits(xs_bits, g, b, w_dev, eps):
    """Oracle logits for a few rows; the vocabulary matrix is brought over in pieces."""
    a = orc.round_to_bf16(orc.layernorm(orc.from_bf16_bits(xs_bits), g, b, eps))
    out = []
    for v0 in range(0, w_dev.shape[0], 8192):
        out.append(a @ gu.to_f64(w_dev[v0:v0 + 8192]).T)
    return np.concatenate(out, axis=1)


@pytest.mark.parametrize("h,vocab,rows,gather", [
    (256, 1000, 1, False), (256, 1000, 5, True), (256, 1000, 64, False), (256, 1000, 100, True),
    (256, 8, 3, False), (512, 50272, 256, False),
])
def test_next_token_small(h, vocab, rows, gather):
    ctx = _ctx(h, h // 64, 64, 4 * h)
    x_rows = rows * 3 if gather else rows
    x = gu.dev_normal_bits((x_rows, h), 1.0, 21)
    g, b = gu.dev_normal_bits((h,), 0.05, 22, 1.0), gu.dev_normal_bits((h,), 0.05, 23)
    w = gu.dev_normal_bits((vocab, h), 0.05, 24)
    idx = np.random.default_rng(5).permutation(x_rows)[:rows] if gather else None
    tok = torch.full((rows,), -7, dtype=torch.int32, device="cuda")
    best = torch.zeros(rows, dtype=torch.float32, device="cuda")
    ws = gu.workspace(ctx.ds_next_token_workspace_bytes(rows, vocab))
    ctx.ds_next_token(x, gu.i32_dev(idx) if gather else None, rows, g, b, w, vocab, tok, best, ws)
    torch.cuda.synchronize()
    xs = gu.to_bits(x)[idx] if gather else gu.to_bits(x)
    logits = _oracle_logits(xs, gu.to_f64(g), gu.to_f64(b), w, 1e-5)
    _check_choice(tok.cpu().numpy(), best.cpu().numpy().astype(np.float64), logits)


def test_next_token_ties_go_to_lowest_id():
    h, vocab, rows = 256, 4096, 16
    ctx = _ctx(h, 4, 64, 1024)
    x = gu.dev_normal_bits((rows, h), 1.0, 31)
    g, b = gu.dev_normal_bits((h,), 0.05, 32, 1.0), gu.dev_normal_bits((h,), 0.05, 33)
    w = gu.dev_normal_bits((vocab, h), 0.05, 34)
    ws = gu.workspace(ctx.ds_next_token_workspace_bytes(rows, vocab))
    tok = torch.empty(rows, dtype=torch.int32, device="cuda")
    ctx.ds_next_token(x, None, rows, g, b, w, vocab, tok, None, ws)
    torch.cuda.synchronize()
    first = tok.cpu().numpy().copy()
    # plant an exact copy of every row's winning vocabulary row far away (another column block), once
    # above and once below the winner's id: the choice must be the lowest of the equal ids
    w2 = w.clone()
    expect = first.copy()
    for r, t in enumerate(first):
        twin = (int(t) + 1500 + 7 * r) % vocab
        if twin in first or twin in expect:
            continue
        w2[twin] = w[int(t)]
        expect[r] = min(int(t), twin)
    tok2 = torch.empty(rows, dtype=torch.int32, device="cuda")
    best2 = torch.empty(rows, dtype=torch.float32, device="cuda")
    ctx.ds_next_token(x, None, rows, g, b, w2, vocab, tok2, best2, ws)
    torch.cuda.synchronize()
    assert np.array_equal(tok2.cpu().numpy(), expect)
    assert np.any(expect != first)          # some twin really sat below its original


def test_next_token_opt13b_vocab_after_prefill_rows():
    """OPT-13B width and OPT's vocabulary (50272 ids, Sec. 6.1), rows picked like the last positions of a
    packed prefill batch, and a 64-wide decode batch."""
    h, vocab = 5120, 50272
    ctx = _ctx(h, 40, 128, 20480)
    g, b = gu.dev_normal_bits((h,), 0.02, 42, 1.0), gu.dev_normal_bits((h,), 0.02, 43)
    w = gu.dev_normal_bits((vocab, h), 0.02, 44)
    lens = [512, 37, 300, 1]
    last = (synth.cu_seqlens(lens)[1:] - 1).astype(np.int32)
    x = gu.dev_normal_bits((int(sum(lens)), h), 1.0, 41)
    for rows, idx, xsrc in ((len(lens), last, x), (64, None, gu.dev_normal_bits((64, h), 1.0, 45))):
        tok = torch.empty(rows, dtype=torch.int32, device="cuda")
        best = torch.empty(rows, dtype=torch.float32, device="cuda")
        ws = gu.workspace(ctx.ds_next_token_workspace_bytes(rows, vocab))
        ctx.ds_next_token(xsrc, gu.i32_dev(idx) if idx is not None else None, rows, g, b, w, vocab, tok, best, ws)
        torch.cuda.synchronize()
        sample = np.arange(rows) if rows <= 8 else np.array([0, 1, 17, 31, 32, 63])
        xs = gu.to_bits(xsrc)[idx] if idx is not None else gu.to_bits(xsrc)
        logits = _oracle_logits(xs[sample], gu.to_f64(g), gu.to_f64(b), w, 1e-5)
        _check_choice(tok.cpu().numpy()[sample], best.cpu().numpy().astype(np.float64)[sample], logits)


def test_token_loop_arguments_are_checked():
    ctx = _ctx(256, 4, 64, 1024)
    x = torch.zeros(4, 256, dtype=torch.bfloat16, device="cuda")
    g = torch.ones(256, dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(64, 256, dtype=torch.bfloat16, device="cuda")
    tok = torch.zeros(4, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.DsError):      # workspace too small
        ctx.ds_next_token(x, None, 4, g, g, w, 64, tok, None, torch.empty(16, dtype=torch.uint8, device="cuda"))
    with pytest.raises(binding.DsError):      # vocab not a multiple of 8
        ctx.ds_next_token(x, None, 4, g, g, w, 60, tok, None, gu.workspace(1 << 20))
    with pytest.raises(binding.DsError):      # too many rows for one call
        ctx.ds_next_token(x, None, 257, g, g, w, 64, tok, None, gu.workspace(1 << 20))
    with pytest.raises(binding.DsError):      # position table without positions
        ctx.ds_embed(gu.i32_dev([0]), None, w, 64, w, 64, 1, x)


def test_greedy_generation_two_layers_end_to_end():
    """The closed loop on a tiny two-layer model: embed the prompts, prefill both layers, hand the KV
    over, choose the first token, then six decoding steps that each embed the previous choice.  The
    oracle recomputes every step from the whole token history (the definition the KV cache only
    short-cuts, Sec. 2.1), fed with the tokens the GPU chose; each GPU choice must be the oracle's, or a
    near-tie of it (3e-2 of the largest |logit|: two layers of bf16 intermediates lie in between)."""
    shape, vocab, steps = synth.TINY, 512, 6
    h, n = shape.hidden, shape.n_heads
    lens = [19, 33, 7]
    B, t = len(lens), sum(lens)
    n_pos = max(lens) + steps + 2
    ctx = gu.make_ctx(shape)
    layers_bits = [synth.make_layer_weights(shape, 77, layer=i) for i in range(2)]
    layers_dev = [gu.weights_to_dev(wb) for wb in layers_bits]
    layers_ref = [orc.weights_from_bits(wb) for wb in layers_bits]
    te, pe = gu.dev_normal_bits((vocab, h), 0.5, 71), gu.dev_normal_bits((n_pos, h), 0.5, 72)
    lg, lb = gu.dev_normal_bits((h,), 0.05, 73, 1.0), gu.dev_normal_bits((h,), 0.05, 74)
    te_r, pe_r, lg_r, lb_r = gu.to_f64(te), gu.to_f64(pe), gu.to_f64(lg), gu.to_f64(lb)
    rng = np.random.default_rng(75)
    prompts = [rng.integers(0, vocab, size=l) for l in lens]

    # ---- GPU: prefill ----
    cu = synth.cu_seqlens(lens)
    ids = np.concatenate(prompts)
    pos = np.concatenate([np.arange(l) + 2 for l in lens])       # OPT numbers positions from 2
    x = torch.empty(t, h, dtype=torch.bfloat16, device="cuda")
    ctx.ds_embed(gu.i32_dev(ids), gu.i32_dev(pos), te, vocab, pe, n_pos, t, x)
    bt, nblk = synth.make_block_tables([l + steps for l in lens], 16, 76)
    bt_d = gu.i32_dev(bt)
    caches = []
    ws = gu.workspace(ctx.ds_prefill_workspace_bytes(t))
    for lw, _keep in layers_dev:
        y, k_out, v_out = torch.empty_like(x), torch.empty_like(x), torch.empty_like(x)
        ctx.ds_prefill(lw, x, gu.i32_dev(cu), B, t, max(lens), y, k_out, v_out, ws)
        kc = torch.zeros(nblk, n, 16, shape.head_dim, dtype=torch.bfloat16, device="cuda")
        vc = torch.zeros_like(kc)
        ctx.ds_kv_migrate(k_out, v_out, gu.i32_dev(cu), B, t, max(lens), bt_d, bt.shape[1], kc, vc, nblk)
        caches.append((kc, vc))
        x = y
    tok = torch.empty(B, dtype=torch.int32, device="cuda")
    best = torch.empty(B, dtype=torch.float32, device="cuda")
    ws_tok = gu.workspace(ctx.ds_next_token_workspace_bytes(B, vocab))
    ctx.ds_next_token(x, gu.i32_dev(cu[1:] - 1), B, lg, lb, te, vocab, tok, best, ws_tok)   # tied vocabulary matrix
    torch.cuda.synchronize()
    chosen = [tok.cpu().numpy().copy()]
    bests = [best.cpu().numpy().astype(np.float64)]

    # ---- GPU: decoding steps ----
    ws_dec = gu.workspace(ctx.ds_decode_workspace_bytes(B, max(lens) + steps))
    ctx_lens = np.array(lens, dtype=np.int32)
    for _ in range(steps):
        xd = torch.empty(B, h, dtype=torch.bfloat16, device="cuda")
        ctx.ds_embed(tok, gu.i32_dev(ctx_lens + 2), te, vocab, pe, n_pos, B, xd)
        for (lw, _keep), (kc, vc) in zip(layers_dev, caches):
            yd = torch.empty_like(xd)
            ctx.ds_decode_step(lw, xd, gu.i32_dev(ctx_lens), bt_d, B, bt.shape[1], int(ctx_lens.max()) + 1, kc, vc,
                               nblk, yd, ws_dec)
            xd = yd
        ctx_lens = ctx_lens + 1
        tok = torch.empty(B, dtype=torch.int32, device="cuda")
        best = torch.empty(B, dtype=torch.float32, device="cuda")
        ctx.ds_next_token(xd, None, B, lg, lb, te, vocab, tok, best, ws_tok)
        torch.cuda.synchronize()
        chosen.append(tok.cpu().numpy().copy())
        bests.append(best.cpu().numpy().astype(np.float64))

    # ---- oracle: every step from the full history, teacher-forced with the GPU's tokens ----
    differing = 0
    for step in range(steps + 1):
        logits = []
        for i in range(B):
            hist = np.concatenate([prompts[i]] + [np.array([chosen[s][i]]) for s in range(step)])
            xr = orc.embed(te_r, pe_r, hist, np.arange(len(hist)) + 2)
            for w in layers_ref:
                xr, _, _ = orc.layer_prefill(w, xr, [len(hist)], n, shape.ln_eps)
            logits.append(orc.next_token_logits(xr[-1:], lg_r, lb_r, te_r, shape.ln_eps)[0])
        logits = np.array(logits)
        want = orc.greedy(logits)
        top = np.max(np.abs(logits), axis=1)
        r = np.arange(B)
        gap = logits[r, want] - logits[r, chosen[step]]
        assert np.all(gap <= 3e-2 * top), (step, gap / top)
        assert np.all(np.abs(bests[step] - logits[r, want]) <= 3e-2 * top), step
        differing += int(np.sum(want != chosen[step]))
    assert differing <= 2     # near-ties are rare; most choices must coincide exactly
