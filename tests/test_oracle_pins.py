"""Pins for the CPU oracle: closed forms, invariants, another library's
routines, scalar brute force and the sizes the paper prints.  No GPU."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import ds_oracle as orc
from paper_2401_09670_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_values.txt")


def golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        kv = line.split("|")[0]
        k, v = kv.split("=", 1)
        out[k.strip()] = v.strip()
    return out


def rnd(shape, seed, scale=1.0):
    return np.random.default_rng(seed).standard_normal(shape) * scale


def tiny_weights(h, m, seed, scale=0.2):
    r = np.random.default_rng(seed)
    g = lambda *s: r.standard_normal(s) * scale
    return dict(ln1_g=1 + g(h), ln1_b=g(h), w_qkv=g(3 * h, h), b_qkv=g(3 * h), w_o=g(h, h), b_o=g(h),
                ln2_g=1 + g(h), ln2_b=g(h), w_fc1=g(m, h), b_fc1=g(m), w_fc2=g(h, m), b_fc2=g(h))


# ------------------------------------------------------------------ number format
def test_bf16_bits_roundtrip_and_rne():
    # exactly representable values survive; ties round to even mantissa
    vals = np.array([1.0, -2.5, 0.0, 3.140625, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8], dtype=np.float32)
    bits = synth.f32_to_bf16_bits(vals)
    back = orc.from_bf16_bits(bits)
    assert back[0] == 1.0 and back[1] == -2.5 and back[2] == 0.0 and back[3] == 3.140625
    assert back[4] == 1.0                 # tie -> even (1.0)
    assert back[5] == 1.0 + 2 ** -6       # tie -> even (1 + 4*2^-8)
    t = torch.tensor(vals).to(torch.bfloat16)
    assert np.array_equal(t.view(torch.int16).numpy().view(np.uint16), bits)
    assert np.array_equal(orc.from_bf16_bits(bits, np.float32), t.float().numpy())


# ------------------------------------------------------------------ LayerNorm
def test_layernorm_constant_row_gives_beta():
    h = 64
    g, b = rnd(h, 1), rnd(h, 2)
    x = np.full((3, h), 7.25)
    assert np.allclose(orc.layernorm(x, g, b), np.broadcast_to(b, (3, h)), atol=1e-12)


def test_layernorm_moments_closed_form():
    h, eps = 512, 1e-5
    x = rnd((5, h), 3, 3.0) + 1.7
    out = orc.layernorm(x, np.ones(h), np.zeros(h), eps)
    var = x.var(axis=1)           # numpy's biased variance
    assert np.allclose(out.mean(axis=1), 0, atol=1e-12)
    assert np.allclose(out.var(axis=1), var / (var + eps), rtol=1e-12)


def test_layernorm_matches_torch():
    h = 96
    x, g, b = rnd((7, h), 4), rnd(h, 5), rnd(h, 6)
    ref = F.layer_norm(torch.tensor(x), (h,), torch.tensor(g), torch.tensor(b), 1e-5).numpy()
    assert np.allclose(orc.layernorm(x, g, b, 1e-5), ref, rtol=1e-12, atol=1e-12)


# ------------------------------------------------------------------ linear
def test_linear_scalar_bruteforce_and_orientation():
    x, w, b = rnd((3, 5), 7), rnd((4, 5), 8), rnd(4, 9)    # non-square: a transposed operand cannot pass
    ref = np.zeros((3, 4))
    for r in range(3):
        for o in range(4):
            acc = 0.0
            for i in range(5):
                acc += x[r, i] * w[o, i]
            ref[r, o] = acc + b[o]
    assert np.allclose(orc.linear(x, w, b), ref, rtol=1e-13)
    assert np.allclose(orc.linear(x, w, None), ref - b, rtol=1e-12, atol=1e-13)


def test_linear_identity_and_onehot():
    x = rnd((4, 6), 10)
    assert np.array_equal(orc.linear(x, np.eye(6), None), x)
    w = np.zeros((2, 6)); w[0, 4] = 1; w[1, 1] = 1          # output o picks input column
    assert np.array_equal(orc.linear(x, w, None), x[:, [4, 1]])
    assert np.allclose(orc.linear(F.linear(torch.tensor(x), torch.tensor(w)).numpy(), np.eye(2), None),
                       x[:, [4, 1]])


# ------------------------------------------------------------------ attention
def test_softmax_rows_sum_to_one_and_future_is_zero():
    l, n, s = 37, 3, 16
    q, k = rnd((l, n, s), 11), rnd((l, n, s), 12)
    p = orc.attention_probs(q, np.arange(l), k)
    assert np.all(np.abs(p.sum(axis=2) - 1) < 1e-12)
    assert np.all(p >= 0)
    for r in range(l):
        assert np.all(p[:, r, r + 1:] == 0)
        assert np.all(p[:, r, :r + 1] > 0)


def test_attention_single_key_returns_v0():
    q, k, v = rnd((1, 2, 8), 13), rnd((1, 2, 8), 14), rnd((1, 2, 8), 15)
    assert np.allclose(orc.attention_rows(q, np.array([0]), k, v), v, rtol=0, atol=1e-15)


def test_attention_equal_keys_gives_running_mean():
    l, n, s = 9, 2, 8
    q, v = rnd((l, n, s), 16), rnd((l, n, s), 17)
    k = np.broadcast_to(rnd((1, n, s), 18), (l, n, s)).copy()
    o = orc.attention_rows(q, np.arange(l), k, v)
    ref = np.cumsum(v, axis=0) / np.arange(1, l + 1).reshape(l, 1, 1)
    assert np.allclose(o, ref, rtol=1e-12, atol=1e-13)


def test_attention_scalar_bruteforce():
    l, n, s = 6, 2, 4
    q, k, v = rnd((l, n, s), 19), rnd((l, n, s), 20), rnd((l, n, s), 21)
    ref = np.zeros((l, n, s))
    for j in range(n):
        for r in range(l):
            e = [sum(q[r, j, d] * k[c, j, d] for d in range(s)) / math.sqrt(s) for c in range(r + 1)]
            mx = max(e)
            w = [math.exp(v_ - mx) for v_ in e]
            z = sum(w)
            for d in range(s):
                ref[r, j, d] = sum(w[c] / z * v[c, j, d] for c in range(r + 1))
    assert np.allclose(orc.attention_rows(q, np.arange(l), k, v), ref, rtol=1e-12, atol=1e-14)


def test_attention_matches_torch_sdpa_causal():
    l, n, s = 45, 4, 32
    q, k, v = rnd((l, n, s), 22), rnd((l, n, s), 23), rnd((l, n, s), 24)
    tq, tk, tv = (torch.tensor(a).permute(1, 0, 2).unsqueeze(0) for a in (q, k, v))
    ref = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(orc.attention_rows(q, np.arange(l), k, v), ref, rtol=1e-10, atol=1e-12)


def test_attention_rows_subset_equals_full():
    l, n, s = 20, 2, 8
    q, k, v = rnd((l, n, s), 25), rnd((l, n, s), 26), rnd((l, n, s), 27)
    full = orc.attention_rows(q, np.arange(l), k, v)
    rows = np.array([0, 7, 19])
    assert np.allclose(orc.attention_rows(q[rows], rows, k, v), full[rows], rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ whole layer
def scalar_layer(w, x, n, eps):
    """The layer from its definition, in scalar Python, for one request."""
    l, h = len(x), len(x[0])
    s = h // n
    m = len(w["w_fc1"])

    def ln(row, g, b):
        mu = sum(row) / h
        var = sum((v - mu) ** 2 for v in row) / h
        return [(row[i] - mu) / math.sqrt(var + eps) * g[i] + b[i] for i in range(h)]

    def lin(row, W, b):
        return [sum(row[i] * W[o][i] for i in range(len(row))) + b[o] for o in range(len(W))]

    a = [ln(x[r], w["ln1_g"], w["ln1_b"]) for r in range(l)]
    qkv = [lin(a[r], w["w_qkv"], w["b_qkv"]) for r in range(l)]
    y = []
    for r in range(l):
        o = [0.0] * h
        for j in range(n):
            qv = qkv[r][j * s:(j + 1) * s]
            e = []
            for c in range(r + 1):
                kv = qkv[c][h + j * s:h + (j + 1) * s]
                e.append(sum(qv[d] * kv[d] for d in range(s)) / math.sqrt(s))
            mx = max(e)
            p = [math.exp(v - mx) for v in e]
            z = sum(p)
            for d in range(s):
                o[j * s + d] = sum(p[c] / z * qkv[c][2 * h + j * s + d] for c in range(r + 1))
        proj = lin(o, w["w_o"], w["b_o"])
        x1 = [x[r][i] + proj[i] for i in range(h)]
        f = ln(x1, w["ln2_g"], w["ln2_b"])
        u = [max(0.0, v) for v in lin(f, w["w_fc1"], w["b_fc1"])]
        d2 = lin(u, w["w_fc2"], w["b_fc2"])
        y.append([x1[i] + d2[i] for i in range(h)])
    return np.array(y), np.array([row[h:2 * h] for row in qkv]), np.array([row[2 * h:] for row in qkv])


def test_layer_prefill_scalar_bruteforce():
    h, n, m, l = 8, 2, 12, 5
    w = tiny_weights(h, m, 30, scale=0.5)
    x = rnd((l, h), 31)
    wl = {k: v.tolist() for k, v in w.items()}
    ry, rk, rv = scalar_layer(wl, x.tolist(), n, 1e-5)
    y, k, v = orc.layer_prefill(w, x, [l], n, 1e-5)
    assert np.allclose(y, ry, rtol=1e-11, atol=1e-12)
    assert np.allclose(k.reshape(l, h), rk, rtol=1e-12, atol=1e-13)
    assert np.allclose(v.reshape(l, h), rv, rtol=1e-12, atol=1e-13)


def test_layer_requests_are_independent_and_causal():
    h, n, m = 32, 4, 64
    w = tiny_weights(h, m, 32)
    xa, xb = rnd((7, h), 33), rnd((11, h), 34)
    y, k, v = orc.layer_prefill(w, np.concatenate([xa, xb]), [7, 11], n)
    ya, ka, _ = orc.layer_prefill(w, xa, [7], n)
    yb, _, vb = orc.layer_prefill(w, xb, [11], n)
    assert np.allclose(y[:7], ya, rtol=1e-12, atol=1e-13) and np.allclose(y[7:], yb, rtol=1e-12, atol=1e-13)
    assert np.allclose(k[:7], ka, rtol=1e-12, atol=1e-13) and np.allclose(v[7:], vb, rtol=1e-12, atol=1e-13)
    # causality: changing rows > r leaves rows <= r bit-identical
    xb2 = xb.copy(); xb2[6:] += 3.0
    yb2, _, _ = orc.layer_prefill(w, xb2, [11], n)
    assert np.array_equal(yb2[:6], yb[:6])
    assert not np.allclose(yb2[6:], yb[6:])


def test_layer_zero_ffn_out_gives_x1_and_relu_matters():
    h, n, m = 16, 2, 32
    w = tiny_weights(h, m, 35)
    x = rnd((4, h), 36)
    w0 = dict(w); w0["w_fc2"] = np.zeros_like(w["w_fc2"]); w0["b_fc2"] = np.zeros(h)
    y0, k, v = orc.layer_prefill(w0, x, [4], n)
    a = orc.layernorm(x, w["ln1_g"], w["ln1_b"])
    qkv = orc.linear(a, w["w_qkv"], w["b_qkv"])
    o = orc.attention_rows(qkv[:, :h].reshape(4, n, -1), np.arange(4), k, v).reshape(4, h)
    assert np.allclose(y0, x + orc.linear(o, w["w_o"], w["b_o"]), rtol=1e-12, atol=1e-13)
    # with W1 = -|W1| and large negative bias every FFN unit is cut off by the ReLU: y = x1 + b2
    wn = dict(w); wn["w_fc1"] = np.zeros_like(w["w_fc1"]); wn["b_fc1"] = -np.ones(m)
    yn, _, _ = orc.layer_prefill(wn, x, [4], n)
    assert np.allclose(yn, y0 + w["b_fc2"], rtol=1e-12, atol=1e-13)


def test_layer_prefill_rows_matches_full():
    h, n, m, l = 32, 2, 64, 13
    w = tiny_weights(h, m, 37)
    x = rnd((l, h), 38)
    y, k, v = orc.layer_prefill(w, x, [l], n)
    rows = [0, 5, 12]
    yr, kr, vr = orc.layer_prefill_rows(w, x, rows, n)
    assert np.allclose(yr, y[rows], rtol=1e-12, atol=1e-13)
    assert np.allclose(kr, k, rtol=1e-12, atol=1e-14) and np.allclose(vr, v, rtol=1e-12, atol=1e-14)


def test_layer_fp32_close_to_fp64():
    shape = synth.TINY
    wb = synth.make_layer_weights(shape, 5)
    xb = synth.make_activations(64, shape.hidden, 5)
    y64, _, _ = orc.layer_prefill(orc.weights_from_bits(wb), orc.from_bf16_bits(xb), [32, 32], shape.n_heads)
    y32, _, _ = orc.layer_prefill(orc.weights_from_bits(wb, np.float32), orc.from_bf16_bits(xb, np.float32),
                                  [32, 32], shape.n_heads)
    assert y32.dtype == np.float32
    assert np.max(np.abs(y32 - y64)) / np.max(np.abs(y64)) < 1e-5


# ------------------------------------------------------------------ migration and paging
def test_kv_migrate_index_map_sentinel_and_roundtrip():
    n, s, bs = 3, 8, 16
    lens = [1, 16, 17, 40]
    t = sum(lens)
    bt, nblk = synth.make_block_tables(lens, bs, seed=3)
    ks = np.arange(t * n * s, dtype=np.uint16).reshape(t, n, s)
    vs = (ks + 40000).astype(np.uint16)
    kc = np.full((nblk, n, bs, s), 0xDEAD, dtype=np.uint16)
    vc = np.full((nblk, n, bs, s), 0xBEEF, dtype=np.uint16)
    orc.kv_migrate(ks, vs, lens, bt, kc, vc)
    cu = synth.cu_seqlens(lens)
    touched = np.zeros((nblk, bs), dtype=bool)
    for i, l in enumerate(lens):
        for j in range(l):
            for hd in range(n):
                for d in range(s):
                    assert kc[bt[i][j // bs]][hd][j % bs][d] == ks[cu[i] + j][hd][d]
                    assert vc[bt[i][j // bs]][hd][j % bs][d] == vs[cu[i] + j][hd][d]
            touched[bt[i][j // bs], j % bs] = True
        assert np.array_equal(orc.kv_gather(kc, bt[i], l), ks[cu[i]:cu[i] + l])
    assert touched.sum() == t
    assert np.all(kc.transpose(0, 2, 1, 3)[~touched] == 0xDEAD)
    assert np.all(vc.transpose(0, 2, 1, 3)[~touched] == 0xBEEF)


def _prefill_into_cache(w, shape, xs, lens, bt, nblk, caps):
    y, k, v = orc.layer_prefill(w, xs, lens, shape.n_heads)
    kc = np.zeros((nblk, shape.n_heads, shape.block_size, shape.head_dim))
    vc = np.zeros_like(kc)
    orc.kv_migrate(k, v, lens, bt, kc, vc)
    return kc, vc


def test_decode_cached_equals_recompute_equals_prefill_last_row():
    """Config-1 shape: 2 prompts of 32 tokens, pages of 16, 8 decode steps."""
    shape = synth.TINY
    cfg = synth.config(0)
    w = orc.weights_from_bits(synth.make_layer_weights(shape, cfg["seed"]))
    lens = cfg["prefill_lens"]
    steps = cfg["decode_steps"]
    xs = orc.from_bf16_bits(synth.make_activations(sum(lens), shape.hidden, cfg["seed"]))
    bt, nblk = synth.make_block_tables([l + steps for l in lens], shape.block_size, cfg["seed"])
    kc, vc = _prefill_into_cache(w, shape, xs, lens, bt, nblk, None)
    hist = [xs[:32], xs[32:]]
    ctx = list(lens)
    for step in range(steps):
        xn = orc.from_bf16_bits(synth.make_activations(2, shape.hidden, cfg["seed"], stream=1 + step))
        y = orc.layer_decode_cached(w, xn, ctx, bt, kc, vc, shape.n_heads)
        for i in range(2):
            yr = orc.layer_decode_recompute(w, hist[i], xn[i], shape.n_heads)
            assert np.max(np.abs(y[i] - yr)) < 1e-10 * max(1.0, np.max(np.abs(yr)))
            full = np.concatenate([hist[i], xn[i:i + 1]])
            yp, _, _ = orc.layer_prefill(w, full, [len(full)], shape.n_heads)
            assert np.array_equal(yp[-1], yr)
            hist[i] = full
            ctx[i] += 1
    assert ctx == [40, 40]


def test_decode_invariant_under_block_permutation_and_padding():
    shape = synth.ModelShape(hidden=32, n_heads=2, head_dim=16, ffn=64, block_size=16)
    w = tiny_weights(32, 64, 40)
    lens = [5, 33, 16]
    xs = rnd((sum(lens), 32), 41)
    xn = rnd((3, 32), 42)
    outs = []
    for seed, spare, shuffle in [(1, 0, False), (2, 3, True), (3, 11, True)]:
        bt, nblk = synth.make_block_tables([l + 1 for l in lens], 16, seed, spare_blocks=spare, shuffle=shuffle)
        kc, vc = _prefill_into_cache(w, shape, xs, lens, bt, nblk, None)
        outs.append(orc.layer_decode_cached(w, xn, lens, bt, kc, vc, 2))
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])


# ------------------------------------------------------------------ counts vs the paper's printed figures
def test_counts_match_paper_values():
    g = golden()
    s66, s13, s175 = synth.OPT_66B, synth.OPT_13B, synth.OPT_175B
    kv_req = orc.kv_bytes_per_token(s66.hidden, s66.n_layers) * 512
    assert abs(kv_req / 2 ** 30 - float(g["kv_request_GB_opt66b_512tok"])) < 0.01
    assert abs(kv_req / 2 ** 30 * 10 - float(g["kv_bandwidth_GBps_at_10rps"])) < 0.1
    for shp, key in [(s13, "model_GB_opt13b"), (s66, "model_GB_opt66b"), (s175, "model_GB_opt175b")]:
        gb = orc.layer_matrix_params(shp.hidden, shp.ffn) * shp.n_layers * 2 / 1e9
        assert 0.96 * float(g[key]) < gb < float(g[key])      # + embeddings, LN, biases make up the rest
    for B, h, m in [(64, 5120, 20480), (256, 12288, 49152), (1, 256, 1024)]:
        assert orc.decode_gemm_traffic_elems(B, h, m) == 8 * B * h + 4 * h * h + 2 * h * m + 2 * B * m
        assert orc.prefill_gemm_flops(B, h, m) == 2 * (4 * B * h * h + 2 * B * h * m)
    # App. A.2: per head 2 s l^2 flops against 3 s l (l/b) memory -> AI = 2b/3
    for b, key in [(16, "flash_ai_b16"), (32, "flash_ai_b32")]:
        l, s, n = 512, 128, 40
        flops = orc.prefill_attention_flops([l], n * s)
        mem = n * 3 * s * l * (l / b)
        assert abs(flops / mem - float(g[key])) < 0.01
    assert orc.decode_attention_kv_elems([511, 0], 5120) == 2 * 5120 * 513


# ---------------------------------------------------------------------------------------------
# Token loop ends (Sec. 2.1): embedding, logits, greedy choice
# ---------------------------------------------------------------------------------------------
def test_embed_is_one_hot_matmul():
    rng = np.random.default_rng(11)
    V, P, h, rows = 37, 19, 24, 13
    te, pe = rng.normal(size=(V, h)), rng.normal(size=(P, h))
    ids, pos = rng.integers(0, V, size=rows), rng.integers(0, P, size=rows)
    got = orc.embed(te, pe, ids, pos)
    onehot_t = np.zeros((rows, V)); onehot_t[np.arange(rows), ids] = 1.0
    onehot_p = np.zeros((rows, P)); onehot_p[np.arange(rows), pos] = 1.0
    assert np.allclose(got, onehot_t @ te + onehot_p @ pe, rtol=0, atol=1e-14)
    assert np.array_equal(orc.embed(te, None, ids, None), te[ids])
    # a repeated id gives identical rows; position 0 and token 0 are ordinary entries
    assert np.array_equal(orc.embed(te, pe, [0, 0], [0, 0])[0], te[0] + pe[0])


def test_round_to_bf16_hand_values_and_torch():
    # 8 significant bits: spacing 2^-7 in [1,2).  Ties go to the even neighbour.
    cases = {1.0: 1.0, 1.0 + 2.0 ** -8: 1.0,                 # tie between 1 and 1+2^-7 -> even (1.0)
             1.0 + 3 * 2.0 ** -8: 1.0 + 2 * 2.0 ** -7,       # tie between 1+2^-7 and 1+2^-6 -> even (1+2^-6)
             1.0 + 2.0 ** -8 + 2.0 ** -20: 1.0 + 2.0 ** -7,  # just above the tie -> up
             -3.14159: -3.140625, 1000.0: 1000.0, 1001.0: 1000.0, 1003.0: 1004.0, 0.1: 0.10009765625}
    for x, want in cases.items():
        assert orc.round_to_bf16(np.array([x]))[0] == want, x
    rng = np.random.default_rng(12)
    x = (rng.normal(size=5000) * np.exp(rng.uniform(-20, 20, size=5000))).astype(np.float32)
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(orc.round_to_bf16(x), want)
    assert orc.round_to_bf16(np.array([0.0]))[0] == 0.0


def test_next_token_logits_against_torch_and_special_cases():
    rng = np.random.default_rng(13)
    rows, h, V = 7, 64, 101
    x = rng.normal(size=(rows, h)); g = 1 + 0.1 * rng.normal(size=h); b = 0.1 * rng.normal(size=h)
    w = rng.normal(size=(V, h))
    got = orc.next_token_logits(x, g, b, w, 1e-5, hidden_in_bf16=False)
    tx = torch.from_numpy(x)
    want = torch.nn.functional.linear(
        torch.nn.functional.layer_norm(tx, (h,), torch.from_numpy(g), torch.from_numpy(b), 1e-5),
        torch.from_numpy(w)).numpy()
    assert np.allclose(got, want, rtol=1e-11, atol=1e-11)
    # rounding the hidden rows moves a logit by at most sum |w| * half-ulp of the hidden values
    got_r = orc.next_token_logits(x, g, b, w, 1e-5, hidden_in_bf16=True)
    a = orc.layernorm(x, g, b, 1e-5)
    bound = (np.abs(a) * 2.0 ** -8) @ np.abs(w).T
    assert np.all(np.abs(got_r - got) <= bound + 1e-12) and np.any(got_r != got)
    # zero gain: every row normalises to the shift vector, so all rows get the same logits b w^T
    z = orc.next_token_logits(x, np.zeros(h), b, w, 1e-5, hidden_in_bf16=False)
    assert np.allclose(z, np.tile(b @ w.T, (rows, 1)), atol=1e-12)


def test_greedy_brute_force_and_ties():
    rng = np.random.default_rng(14)
    logits = rng.normal(size=(9, 300))
    logits[2, 17] = logits[2, 250] = 50.0            # tie -> lowest id
    logits[3, :] = 1.0                               # all equal -> id 0
    logits[4, 299] = 99.0                            # maximum in the last column
    want = []
    for r in range(logits.shape[0]):
        best = 0
        for j in range(1, logits.shape[1]):
            if logits[r, j] > logits[r, best]:
                best = j
        want.append(best)
    got = orc.greedy(logits)
    assert got.tolist() == want and got[2] == 17 and got[3] == 0 and got[4] == 299


# ---------------------------------------------------------------------------------------------
# Grouped-query attention (fewer key/value heads than query heads; Sec. 3.2 names it)
# ---------------------------------------------------------------------------------------------
def _repeat_kv_weights(w, n, n_kv, s):
    """The multi-head layer that a grouped-query layer is by definition equal to: every key/value
    head's projection rows copied to each query head of its group."""
    h, hk, g = n * s, n_kv * s, n // n_kv
    wq, wk, wv = w["w_qkv"][:h], w["w_qkv"][h:h + hk], w["w_qkv"][h + hk:]
    bq, bk, bv = w["b_qkv"][:h], w["b_qkv"][h:h + hk], w["b_qkv"][h + hk:]
    rep_rows = lambda m: np.repeat(m.reshape(n_kv, s, -1), g, axis=0).reshape(n * s, -1)
    rep_vec = lambda v: np.repeat(v.reshape(n_kv, s), g, axis=0).reshape(n * s)
    out = dict(w)
    out["w_qkv"] = np.concatenate([wq, rep_rows(wk), rep_rows(wv)], axis=0)
    out["b_qkv"] = np.concatenate([bq, rep_vec(bk), rep_vec(bv)])
    return out


def test_gqa_layer_equals_multi_head_layer_with_repeated_kv_heads():
    shape = synth.ModelShape(hidden=64, n_heads=8, head_dim=8, ffn=96, n_kv_heads=2)
    w = orc.weights_from_bits(synth.make_layer_weights(shape, 5))
    assert w["w_qkv"].shape == ((8 + 2 * 2) * 8, 64)
    lens = [5, 1, 9]
    x = orc.from_bf16_bits(synth.make_activations(sum(lens), 64, 5))
    y, k, v = orc.layer_prefill(w, x, lens, 8)
    assert k.shape == (15, 2, 8) and v.shape == (15, 2, 8)
    w_mha = _repeat_kv_weights(w, 8, 2, 8)
    y2, k2, v2 = orc.layer_prefill(w_mha, x, lens, 8)
    assert np.allclose(y, y2, rtol=0, atol=1e-13)
    assert np.array_equal(k2[:, ::4], k) and np.array_equal(k2[:, 3::4], k)   # group of 4 shares one head
    # row-sampled form and the decode forms agree with it as well
    yr, kr, vr = orc.layer_prefill_rows(w, x[:5], [0, 4], 8)
    assert np.allclose(yr, y[[0, 4]], atol=1e-13) and np.allclose(kr, k[:5], atol=1e-13) and kr.shape == (5, 2, 8)
    hist, new = x[6:14], x[14]
    want = orc.layer_decode_recompute(w_mha, hist, new, 8)
    assert np.allclose(orc.layer_decode_recompute(w, hist, new, 8), want, atol=1e-13)
    bt, nblk = synth.make_block_tables([9], 16, 3)
    kc = np.zeros((nblk, 2, 16, 8)); vc = np.zeros_like(kc)
    orc.kv_migrate(k[6:14], v[6:14], [8], bt, kc, vc)
    got = orc.layer_decode_cached(w, new.reshape(1, -1), [8], bt, kc, vc, 8)
    assert np.allclose(got[0], want, atol=1e-13)


def test_gqa_attention_against_torch_sdpa_with_repeated_heads():
    rng = np.random.default_rng(21)
    l, n, n_kv, s = 11, 6, 3, 16
    q, k, v = rng.normal(size=(l, n, s)), rng.normal(size=(l, n_kv, s)), rng.normal(size=(l, n_kv, s))
    got = orc.attention_rows(q, np.arange(l), k, v)
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(k, n // n_kv, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(v, n // n_kv, axis=1)).permute(1, 0, 2)[None]
    want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    assert np.allclose(got, want, atol=1e-12)
    # one key/value head for all query heads (multi-query attention) is the extreme case
    got1 = orc.attention_rows(q, np.arange(l), k[:, :1], v[:, :1])
    for j in range(n):
        assert np.allclose(got1[:, j], orc.attention_rows(q[:, j:j + 1], np.arange(l), k[:, :1], v[:, :1])[:, 0])
