"""CPU oracle for the prefill / KV-migrate / decode hot path.  TEST INFRASTRUCTURE.

This file is the slow, plain definition the HIP kernels are checked against.
Only tests, the smoke check and the benchmark's ``cpu_baseline`` leg may use
it; the product path never does.  It shares no code with the GPU path and
imports nothing from the package.

What it computes (numpy, float64 unless ``dtype`` says otherwise):

* An OPT-style pre-LayerNorm decoder layer (paper Sec. 6.1 names OPT; the four
  GEMM shapes are the tables of App. A.2 / A.3; symbols are App. A.1):
      a  = LN(x; g1, b1)
      [q|k|v] = a W_qkv^T + b_qkv              (t,h) x (h,3h)
      o  = per-request causal softmax(q k^T / sqrt(s)) v, per head (App. A.2:
           attention only operates among the tokens of one request)
      x1 = x + o W_o^T + b_o                   (t,h) x (h,h)
      f  = LN(x1; g2, b2)
      u  = relu(f W_1^T + b_1)                 (t,h) x (h,m)
      y  = x1 + u W_2^T + b_2                  (t,m) x (m,h)
  Matrices are held ``[out, in]``; ``w_qkv`` rows are ``[Q|K|V]``, each part
  ordered ``head*s + d``.  The K and V parts may have fewer heads than Q
  (grouped-query attention, named in Sec. 3.2): ``w_qkv`` is then
  ``[(n + 2 n_kv) s, h]`` and query head j uses key/value head ``j // (n/n_kv)``;
  n_kv is read off the matrix shape.
* The decode step (App. A.3): the same layer for one new row per request whose
  attention runs over the request's cached keys/values plus its own.  Because
  the KV cache exists only to avoid recomputation (Sec. 2.1), the defining
  form is ``layer_decode_recompute`` (run the whole history, keep the last
  row); ``layer_decode_cached`` reads the earlier rows' K,V through a block
  table from a paged cache (Sec. 5 uses PagedAttention) and must agree with it.
* The KV hand-off (Sec. 3.3 / 4.3): a pure index map from the prefill side's
  contiguous per-token K,V rows into ``[num_blocks, n, block_size, s]`` pages.
* The two ends of the token loop (Sec. 2.1: tokens in, one new token out per pass): ``embed``
  (token row + learned position row, OPT being the model family of Sec. 6.1) and
  ``next_token_logits`` / ``greedy`` (final LayerNorm, logits against the vocabulary matrix,
  largest logit, lowest id among equals).
* Size/traffic counts used to price the kernels, pinned to figures the paper
  prints (Sec. 3.3 KV size, Table 1 model sizes, App. A.3 decode traffic).

Pinning status: every function here is pinned by tests/test_oracle_pins.py
(closed forms, invariants, library routines of a different library, scalar
brute force, the paper's printed sizes).  The paper prints no activations, so
whole-layer numerics are pinned by those invariants only, not by paper values.
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence

import numpy as np


# ---------------------------------------------------------------------------
# number format
# ---------------------------------------------------------------------------
def from_bf16_bits(bits: np.ndarray, dtype=np.float64) -> np.ndarray:
    """bf16 bit patterns (uint16) -> exact value in ``dtype``."""
    u = np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(dtype)


def weights_from_bits(wbits: Dict[str, np.ndarray], dtype=np.float64) -> Dict[str, np.ndarray]:
    return {k: from_bf16_bits(v, dtype) for k, v in wbits.items()}


# ---------------------------------------------------------------------------
# layer pieces
# ---------------------------------------------------------------------------
def layernorm(x: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float = 1e-5) -> np.ndarray:
    """Per-row LayerNorm with biased variance over the hidden dimension."""
    mu = x.mean(axis=-1, keepdims=True)
    d = x - mu
    var = (d * d).mean(axis=-1, keepdims=True)
    return d / np.sqrt(var + eps) * gamma + beta


def linear(x: np.ndarray, w: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    """``x[rows,in] @ w[out,in]^T + b`` (GEMM tables of App. A.2 / A.3)."""
    y = x @ w.T
    if b is not None:
        y = y + b
    return y


def attention_probs(q_rows: np.ndarray, pos: np.ndarray, k: np.ndarray) -> np.ndarray:
    """Softmax weights ``[n, R, l]``: query row r (at position ``pos[r]``) over
    keys ``0..pos[r]``; keys after ``pos[r]`` get weight exactly 0."""
    R, n, s = q_rows.shape
    l = k.shape[0]
    g = n // k.shape[1]  # query heads per key/value head (1 = ordinary multi-head attention)
    pos = np.asarray(pos).reshape(R, 1)
    allowed = np.arange(l).reshape(1, l) <= pos
    p = np.zeros((n, R, l), dtype=q_rows.dtype)
    for j in range(n):
        e = (q_rows[:, j, :] @ k[:, j // g, :].T) / math.sqrt(s)
        e = np.where(allowed, e, -np.inf)
        e = e - e.max(axis=1, keepdims=True)
        w = np.exp(e)
        p[j] = w / w.sum(axis=1, keepdims=True)
    return p


def attention_rows(q_rows: np.ndarray, pos: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """``o[r, j, :] = sum_c p[j, r, c] v[c, j, :]`` for one request.

    ``q_rows[R,n,s]`` are queries at positions ``pos[R]`` of a request whose
    keys/values are ``k, v[l,n,s]``.  Prefill uses all rows (pos = 0..l-1),
    a decode step uses one row (pos = l-1).

    With fewer key/value heads than query heads (``k, v[l,n_kv,s]``, n_kv
    dividing n: grouped-query attention, which Sec. 3.2 names as a way to
    shrink the KV cache) query head j reads key/value head ``j // (n / n_kv)``."""
    p = attention_probs(q_rows, pos, k)
    R, n, s = q_rows.shape
    g = n // v.shape[1]
    o = np.empty((R, n, s), dtype=q_rows.dtype)
    for j in range(n):
        o[:, j, :] = p[j] @ v[:, j // g, :]
    return o


def _split_qkv(qkv: np.ndarray, n: int, s: int):
    """Columns are [Q: n heads | K: n_kv heads | V: n_kv heads]; n_kv follows from the width."""
    h = n * s
    rows = qkv.shape[0]
    n_kv = (qkv.shape[1] // s - n) // 2
    assert (n + 2 * n_kv) * s == qkv.shape[1] and n % n_kv == 0
    hk = n_kv * s
    q = qkv[:, 0:h].reshape(rows, n, s)
    k = qkv[:, h:h + hk].reshape(rows, n_kv, s)
    v = qkv[:, h + hk:h + 2 * hk].reshape(rows, n_kv, s)
    return q, k, v


def _post_attention(w, x_rows, o_rows, eps):
    """Steps after attention for the given rows: out-proj + residual, LN2, FFN + residual."""
    rows = x_rows.shape[0]
    x1 = x_rows + linear(o_rows.reshape(rows, -1), w["w_o"], w.get("b_o"))
    f = layernorm(x1, w["ln2_g"], w["ln2_b"], eps)
    u = np.maximum(linear(f, w["w_fc1"], w.get("b_fc1")), 0)
    return x1 + linear(u, w["w_fc2"], w.get("b_fc2"))


# ---------------------------------------------------------------------------
# prefill
# ---------------------------------------------------------------------------
def layer_prefill(w: Dict[str, np.ndarray], x: np.ndarray, seq_lens: Sequence[int],
                  n_heads: int, eps: float = 1e-5):
    """One layer over packed prompts ``x[t,h]``; returns ``(y[t,h], k[t,n,s], v[t,n,s])``."""
    t, h = x.shape
    s = h // n_heads
    assert int(np.sum(seq_lens)) == t
    a = layernorm(x, w["ln1_g"], w["ln1_b"], eps)
    q, k, v = _split_qkv(linear(a, w["w_qkv"], w.get("b_qkv")), n_heads, s)
    o = np.empty_like(q)
    r0 = 0
    for l in seq_lens:
        l = int(l)
        sl = slice(r0, r0 + l)
        o[sl] = attention_rows(q[sl], np.arange(l), k[sl], v[sl])
        r0 += l
    y = _post_attention(w, x, o, eps)
    return y, np.ascontiguousarray(k), np.ascontiguousarray(v)


def layer_prefill_rows(w: Dict[str, np.ndarray], x_seq: np.ndarray, rows: Sequence[int],
                       n_heads: int, eps: float = 1e-5):
    """The same definition for ONE request ``x_seq[l,h]``, finishing only the
    sampled ``rows``: K,V are computed for every row of the request (they are
    needed by later rows), the rest of the layer only for ``rows``.
    Returns ``(y_rows[R,h], k[l,n,s], v[l,n,s])``."""
    l, h = x_seq.shape
    s = h // n_heads
    rows = np.asarray(rows, dtype=np.int64)
    a = layernorm(x_seq, w["ln1_g"], w["ln1_b"], eps)
    bq = w.get("b_qkv")
    kv = linear(a, w["w_qkv"][h:], None if bq is None else bq[h:])
    hk = kv.shape[1] // 2                      # n_kv * s
    k = kv[:, :hk].reshape(l, hk // s, s)
    v = kv[:, hk:].reshape(l, hk // s, s)
    q = linear(a[rows], w["w_qkv"][:h], None if bq is None else bq[:h]).reshape(len(rows), n_heads, s)
    o = attention_rows(q, rows, k, v)
    y = _post_attention(w, x_seq[rows], o, eps)
    return y, np.ascontiguousarray(k), np.ascontiguousarray(v)


# ---------------------------------------------------------------------------
# KV hand-off: contiguous rows -> paged blocks
# ---------------------------------------------------------------------------
def kv_migrate(k_src: np.ndarray, v_src: np.ndarray, seq_lens: Sequence[int],
               block_tables: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray) -> None:
    """Token j of request i goes to page ``block_tables[i, j // bs]``, slot ``j % bs``.

    ``k_src, v_src[t,n,s]``; ``k_cache, v_cache[num_blocks,n,bs,s]`` are updated
    in place.  Works on any element type (bit patterns included); slots that no
    token maps to are left untouched."""
    bs = k_cache.shape[2]
    r = 0
    for i, l in enumerate(seq_lens):
        for j in range(int(l)):
            blk = int(block_tables[i, j // bs])
            assert 0 <= blk < k_cache.shape[0]
            k_cache[blk, :, j % bs, :] = k_src[r]
            v_cache[blk, :, j % bs, :] = v_src[r]
            r += 1


def kv_gather(cache: np.ndarray, block_table_row: np.ndarray, length: int) -> np.ndarray:
    """Inverse view: the first ``length`` tokens of one request as ``[length,n,s]``."""
    bs = cache.shape[2]
    out = np.empty((length, cache.shape[1], cache.shape[3]), dtype=cache.dtype)
    for j in range(length):
        out[j] = cache[int(block_table_row[j // bs]), :, j % bs, :]
    return out


# ---------------------------------------------------------------------------
# decode step
# ---------------------------------------------------------------------------
def layer_decode_recompute(w: Dict[str, np.ndarray], history: np.ndarray, x_new: np.ndarray,
                           n_heads: int, eps: float = 1e-5) -> np.ndarray:
    """Defining form for one request: run the layer over ``[history; x_new]``
    as a prompt and return the last row ``[h]``."""
    xs = np.concatenate([history, x_new.reshape(1, -1)], axis=0)
    y, _, _ = layer_prefill(w, xs, [xs.shape[0]], n_heads, eps)
    return y[-1]


def layer_decode_cached(w: Dict[str, np.ndarray], x: np.ndarray, ctx_lens: Sequence[int],
                        block_tables: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray,
                        n_heads: int, eps: float = 1e-5) -> np.ndarray:
    """One decode step for a batch ``x[B,h]``.

    Request i already has ``ctx_lens[i]`` tokens in the paged cache.  The new
    row's k,v are written at position ``ctx_lens[i]`` (page
    ``block_tables[i, ctx // bs]``, slot ``ctx % bs``), then its query attends
    over ``ctx_lens[i] + 1`` keys.  Returns ``y[B,h]``; caches updated in place."""
    B, h = x.shape
    s = h // n_heads
    bs = k_cache.shape[2]
    a = layernorm(x, w["ln1_g"], w["ln1_b"], eps)
    q, k, v = _split_qkv(linear(a, w["w_qkv"], w.get("b_qkv")), n_heads, s)
    o = np.empty_like(q)
    for i in range(B):
        c = int(ctx_lens[i])
        blk = int(block_tables[i, c // bs])
        assert 0 <= blk < k_cache.shape[0]
        k_cache[blk, :, c % bs, :] = k[i]
        v_cache[blk, :, c % bs, :] = v[i]
        ks = kv_gather(k_cache, block_tables[i], c + 1)
        vs = kv_gather(v_cache, block_tables[i], c + 1)
        o[i] = attention_rows(q[i:i + 1], np.array([c]), ks, vs)[0]
    return _post_attention(w, x, o, eps)


# ---------------------------------------------------------------------------
# counts (sizes, flops, traffic)
# ---------------------------------------------------------------------------
# ---------------------------------------------------------------------------------------------
# Token loop ends (Sec. 2.1)
# ---------------------------------------------------------------------------------------------
def embed(tok_emb: np.ndarray, pos_emb: Optional[np.ndarray], token_ids: Sequence[int],
          positions: Optional[Sequence[int]]) -> np.ndarray:
    """x[r] = tok_emb[token_ids[r]] + pos_emb[positions[r]] (no position term without a table)."""
    x = np.array([tok_emb[int(i)] for i in token_ids], dtype=tok_emb.dtype)
    if pos_emb is not None:
        x = x + np.array([pos_emb[int(j)] for j in positions], dtype=pos_emb.dtype)
    return x


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest value with an 8-bit significand (1 implicit + 7 stored bits), ties to even; same dtype
    out.  Written with frexp/rint so that it does not share the bit tricks of any other rounding
    routine in this repository.  (Finite normal-range inputs; that is all the tests feed it.)"""
    x = np.asarray(x)
    mant, expo = np.frexp(x.astype(np.float64))      # x = mant * 2**expo, 0.5 <= |mant| < 1
    q = np.rint(mant * 256.0) / 256.0                # 8 significant bits; rint rounds ties to even
    return np.ldexp(q, expo).astype(x.dtype)


def next_token_logits(x_rows: np.ndarray, ln_g: np.ndarray, ln_b: np.ndarray, w_vocab: np.ndarray,
                      eps: float = 1e-5, hidden_in_bf16: bool = True) -> np.ndarray:
    """logits = LN(x_rows) w_vocab^T.  With ``hidden_in_bf16`` the normalised rows are rounded to
    bf16 before the product: that is the precision in which the GPU path takes the greedy decision
    (its LayerNorm writes bf16), and an argmax has to be compared at the decision's precision."""
    a = layernorm(x_rows, ln_g, ln_b, eps)
    if hidden_in_bf16:
        a = round_to_bf16(a)
    return a @ w_vocab.T


def greedy(logits: np.ndarray) -> np.ndarray:
    """Per row the id of the largest logit; among equal logits the lowest id (numpy's argmax returns
    the first occurrence of the maximum)."""
    return np.argmax(logits, axis=1).astype(np.int64)


# ---------------------------------------------------------------------------------------------
def layer_matrix_params(h: int, m: int) -> int:
    """Elements of the four weight matrices of one layer: 4h^2 + 2hm (App. A.3)."""
    return 4 * h * h + 2 * h * m


def kv_bytes_per_token(h: int, n_layers: int, bytes_per_elem: int = 2) -> int:
    """K and V rows of one token over all layers (Sec. 3.3)."""
    return 2 * h * n_layers * bytes_per_elem


def prefill_gemm_flops(t: int, h: int, m: int) -> int:
    """True multiply-add flops of the four prefill GEMMs: 2 t (4h^2 + 2hm)
    (App. A.2 prints the multiply-accumulate count 4th^2 + 2thm)."""
    return 2 * t * layer_matrix_params(h, m)


def prefill_attention_flops(seq_lens: Sequence[int], h: int) -> int:
    """Causal attention flops summed over heads: ~2 s l^2 per head (App. A.2),
    i.e. 2 h t_2 with t_2 = sum l_i^2."""
    return int(2 * h * sum(int(l) * int(l) for l in seq_lens))


def decode_gemm_traffic_elems(B: int, h: int, m: int) -> int:
    """Elements read+written by the four decode GEMMs (App. A.3), derived per
    GEMM as input + weight + output."""
    qkv = B * h + h * 3 * h + B * 3 * h
    out = B * h + h * h + B * h
    fc1 = B * h + h * m + B * m
    fc2 = B * m + m * h + B * h
    return qkv + out + fc1 + fc2


def decode_attention_kv_elems(ctx_lens: Sequence[int], h: int) -> int:
    """K and V elements a decode step must read: 2 h sum(ctx_i + 1)."""
    return int(2 * h * sum(int(c) + 1 for c in ctx_lens))
