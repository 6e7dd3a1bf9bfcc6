"""Algorithmic work of each kernel class, used to price measurements against
the MI355X rooflines.  Counts follow App. A of the paper (true flops = 2 x its
multiply-accumulate counts; K and V read once each for decode attention)."""
from __future__ import annotations

from typing import Sequence

# MI355X published peaks
PEAK_BF16_FLOPS = 2.5e15      # dense bf16 MFMA
PEAK_HBM_BYTES = 8.0e12       # HBM3E


def layer_matrix_params(h: int, m: int) -> int:
    return 4 * h * h + 2 * h * m


def prefill_gemm_flops(t: int, h: int, m: int) -> int:
    """QKV + Attn-Output + FFN-Input + FFN-Output GEMMs over t tokens (App. A.2)."""
    return 2 * t * layer_matrix_params(h, m)


def prefill_attention_flops(seq_lens: Sequence[int], h: int) -> int:
    """Causal attention, all heads: 2 h sum(l_i^2) (App. A.2; the masked half is not counted)."""
    return int(2 * h * sum(int(l) ** 2 for l in seq_lens))


def layernorm_bytes(rows: int, h: int) -> int:
    return 2 * rows * h * 2


def kv_migrate_bytes(t: int, h: int) -> int:
    """K and V rows read once and written once."""
    return 2 * (2 * t * h * 2)


def decode_gemm_bytes(B: int, h: int, m: int) -> int:
    """Weights once + activations in/out of the four GEMMs (App. A.3: 8Bh + 4h^2 + 2hm + 2Bm elements)."""
    return 2 * (8 * B * h + layer_matrix_params(h, m) + 2 * B * m)


def decode_attention_bytes(kv_lens: Sequence[int], h: int) -> int:
    """K and V of every attended token once (2 h elements per token)."""
    return int(2 * h * 2 * sum(int(l) for l in kv_lens))


def kv_append_bytes(B: int, h: int) -> int:
    return 2 * (2 * B * h * 2)
