"""Seeded synthetic inputs for the prefill / KV-migrate / decode hot path.

This module only *draws inputs*: weights, activations, sequence lengths and
block tables.  It contains none of the method's arithmetic (no LayerNorm, no
GEMM, no attention, no paging logic beyond handing out block ids) and is the
one module that both the GPU tests and the CPU oracle's tests may share.

Everything is returned as numpy arrays.  Tensors that live in HBM as bf16 are
returned as ``uint16`` arrays holding the bf16 bit patterns, so the GPU path
and the CPU oracle start from exactly the same bits.

Shapes follow the paper's symbols (App. A.1): ``h`` hidden size, ``n`` heads,
``s`` head size, ``m`` FFN size, ``B`` batch, ``l_i`` lengths, ``t = sum l_i``.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Sequence

import numpy as np

BASE_SEED = 20240109  # + config index


@dataclasses.dataclass(frozen=True)
class ModelShape:
    """One decoder layer's dimensions (App. A.1 symbols)."""

    hidden: int      # h
    n_heads: int     # n
    head_dim: int    # s, h = n * s
    ffn: int         # m
    block_size: int = 16   # tokens per KV page
    n_layers: int = 1
    ln_eps: float = 1e-5
    n_kv_heads: int = 0    # key/value heads; 0 = as many as query heads (multi-head attention)

    def __post_init__(self):
        assert self.hidden == self.n_heads * self.head_dim
        assert self.n_heads % self.kv_heads == 0

    @property
    def kv_heads(self) -> int:
        return self.n_kv_heads or self.n_heads

    @property
    def qkv_width(self) -> int:
        """Output features of the QKV projection: (n + 2 n_kv) s."""
        return (self.n_heads + 2 * self.kv_heads) * self.head_dim


TINY = ModelShape(hidden=256, n_heads=4, head_dim=64, ffn=1024)
OPT_13B = ModelShape(hidden=5120, n_heads=40, head_dim=128, ffn=20480, n_layers=40)
OPT_66B = ModelShape(hidden=9216, n_heads=72, head_dim=128, ffn=36864, n_layers=64)
OPT_175B = ModelShape(hidden=12288, n_heads=96, head_dim=128, ffn=49152, n_layers=96)


# ---------------------------------------------------------------------------
# bf16 bit patterns (a number format, not part of the method)
# ---------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even); returns uint16 bits."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounding = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + rounding) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def _normal_bf16(rng: np.random.Generator, shape, mean: float, std: float) -> np.ndarray:
    """N(mean, std) drawn in float32 in bounded chunks, rounded to bf16 bits."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for lo in range(0, n, step):
        hi = min(n, lo + step)
        v = rng.standard_normal(hi - lo, dtype=np.float32)
        v *= np.float32(std)
        if mean != 0.0:
            v += np.float32(mean)
        out[lo:hi] = f32_to_bf16_bits(v)
    return out.reshape(shape)


# ---------------------------------------------------------------------------
# weights and activations
# ---------------------------------------------------------------------------
WEIGHT_NAMES = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o",
                "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


def make_layer_weights(shape: ModelShape, seed: int, layer: int = 0) -> Dict[str, np.ndarray]:
    """One layer's parameters as bf16 bits.

    Matrices are stored ``[out_features, in_features]`` row-major (the
    reduction dimension is contiguous).  ``w_qkv`` rows are ordered
    ``[Q | K | V]`` and, within each third, ``head * s + d``.
    Big matrices and biases ~ N(0, 0.02); LayerNorm gain ~ 1 + N(0, 0.02),
    LayerNorm shift ~ N(0, 0.02), so every term of the layer is exercised.
    """
    h, m = shape.hidden, shape.ffn
    rng = np.random.Generator(np.random.Philox(key=[seed, 1000 + layer]))
    w = {}
    w["ln1_g"] = _normal_bf16(rng, (h,), 1.0, 0.02)
    w["ln1_b"] = _normal_bf16(rng, (h,), 0.0, 0.02)
    w["w_qkv"] = _normal_bf16(rng, (shape.qkv_width, h), 0.0, 0.02)
    w["b_qkv"] = _normal_bf16(rng, (shape.qkv_width,), 0.0, 0.02)
    w["w_o"] = _normal_bf16(rng, (h, h), 0.0, 0.02)
    w["b_o"] = _normal_bf16(rng, (h,), 0.0, 0.02)
    w["ln2_g"] = _normal_bf16(rng, (h,), 1.0, 0.02)
    w["ln2_b"] = _normal_bf16(rng, (h,), 0.0, 0.02)
    w["w_fc1"] = _normal_bf16(rng, (m, h), 0.0, 0.02)
    w["b_fc1"] = _normal_bf16(rng, (m,), 0.0, 0.02)
    w["w_fc2"] = _normal_bf16(rng, (h, m), 0.0, 0.02)
    w["b_fc2"] = _normal_bf16(rng, (h,), 0.0, 0.02)
    return w


def make_activations(rows: int, hidden: int, seed: int, stream: int = 0) -> np.ndarray:
    """``[rows, hidden]`` N(0, 1) activations as bf16 bits."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 2000 + stream]))
    return _normal_bf16(rng, (rows, hidden), 0.0, 1.0)


def make_kv_fill(tokens: int, shape: ModelShape, seed: int, stream: int = 0):
    """``[tokens, n, s]`` N(0, 1) K and V rows (bf16 bits) for pre-filling a cache."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 3000 + stream]))
    k = _normal_bf16(rng, (tokens, shape.kv_heads, shape.head_dim), 0.0, 1.0)
    v = _normal_bf16(rng, (tokens, shape.kv_heads, shape.head_dim), 0.0, 1.0)
    return k, v


# ---------------------------------------------------------------------------
# sequence lengths and block tables
# ---------------------------------------------------------------------------
def cu_seqlens(seq_lens: Sequence[int]) -> np.ndarray:
    cu = np.zeros(len(seq_lens) + 1, dtype=np.int32)
    cu[1:] = np.cumsum(np.asarray(seq_lens, dtype=np.int64))
    return cu


def blocks_needed(tokens: int, block_size: int) -> int:
    return (tokens + block_size - 1) // block_size


def make_block_tables(capacities: Sequence[int], block_size: int, seed: int,
                      spare_blocks: int = 3, shuffle: bool = True):
    """Hand out physical KV pages for sequences that may grow to ``capacities[i]`` tokens.

    Returns ``(block_tables[B, max_blocks] int32 with -1 for unused entries,
    num_blocks)``.  Physical ids are a seeded permutation of
    ``range(num_blocks)`` (``spare_blocks`` ids stay unused), so pages of one
    sequence are neither contiguous nor ordered.
    """
    per_seq = [blocks_needed(int(c), block_size) for c in capacities]
    max_blocks = max(per_seq) if per_seq else 0
    total = int(sum(per_seq))
    num_blocks = total + spare_blocks
    rng = np.random.Generator(np.random.Philox(key=[seed, 4000]))
    ids = rng.permutation(num_blocks) if shuffle else np.arange(num_blocks)
    bt = np.full((len(per_seq), max_blocks), -1, dtype=np.int32)
    pos = 0
    for i, nb in enumerate(per_seq):
        bt[i, :nb] = ids[pos:pos + nb]
        pos += nb
    return bt, num_blocks


def lognormal_lengths(count: int, median: float, sigma: float, lo: int, hi: int,
                      seed: int, stream: int = 0) -> np.ndarray:
    """round(clip(LogNormal(ln median, sigma), lo, hi)) — chatbot-like lengths."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 5000 + stream]))
    v = np.exp(rng.normal(np.log(median), sigma, size=count))
    return np.clip(np.rint(v), lo, hi).astype(np.int32)


def uniform_lengths(count: int, lo: int, hi: int, seed: int, stream: int = 0) -> np.ndarray:
    """Integers uniform in [lo, hi] — summarization-like lengths / decode contexts."""
    rng = np.random.Generator(np.random.Philox(key=[seed, 6000 + stream]))
    return rng.integers(lo, hi + 1, size=count).astype(np.int32)


def token_capped_batches(lengths: Sequence[int], cap: int) -> List[List[int]]:
    """First-come-first-served prompt batches with ``sum(l) <= cap`` (a prompt
    longer than ``cap`` runs alone).  Returns lists of request indices."""
    batches, cur, tot = [], [], 0
    for i, l in enumerate(lengths):
        l = int(l)
        if cur and tot + l > cap:
            batches.append(cur)
            cur, tot = [], 0
        cur.append(i)
        tot += l
    if cur:
        batches.append(cur)
    return batches


# ---------------------------------------------------------------------------
# the benchmark configurations as concrete recipes
# ---------------------------------------------------------------------------
def config(index: int) -> dict:
    """Concrete synthetic recipe for workload ``index`` (0-based)."""
    seed = BASE_SEED + index + 1
    if index == 0:
        return dict(name="tiny-1layer", shape=TINY, seed=seed, layers=1,
                    prefill_lens=[32, 32], decode_batch=2, decode_steps=8)
    if index == 1:
        return dict(name="opt13b-1layer-in512-out64", shape=OPT_13B, seed=seed, layers=1,
                    prefill_lens=[512] * 4, decode_batch=64, decode_ctx0=512, decode_steps=64)
    if index == 2:
        return dict(name="opt13b-40layer-chatbot", shape=OPT_13B, seed=seed, layers=40,
                    prompt=dict(kind="lognormal", median=256, sigma=0.8, lo=16, hi=2048),
                    output=dict(kind="lognormal", median=128, sigma=0.8, lo=1, hi=1024),
                    prefill_token_cap=4096, decode_batch=128)
    if index == 3:
        return dict(name="opt66b-64layer-summarization", shape=OPT_66B, seed=seed, layers=64,
                    prompt=dict(kind="uniform", lo=1024, hi=4096),
                    output=dict(kind="uniform", lo=16, hi=256), decode_batch=64)
    if index == 4:
        return dict(name="opt175b-8layer-stage", shape=OPT_175B, seed=seed, layers=8,
                    prefill_lens=[2048] * 8, decode_batch=256,
                    decode_ctx=dict(kind="uniform", lo=128, hi=2048), decode_steps=32)
    raise ValueError(index)
