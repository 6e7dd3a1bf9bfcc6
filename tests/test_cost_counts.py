"""The package's work counts (cost.py, what bench.py prices its measurements with) against the oracle's
counts, which tests/test_oracle_pins.py pins to the numbers the paper prints (App. A.2 / A.3, Sec. 3.3)."""
import pytest

from oracle import ds_oracle as orc
from paper_2401_09670_amd import cost

SHAPES = [(256, 1024), (5120, 20480), (9216, 36864), (12288, 49152)]


@pytest.mark.parametrize("h,m", SHAPES)
def test_gemm_and_attention_counts_agree(h, m):
    assert cost.layer_matrix_params(h, m) == orc.layer_matrix_params(h, m)
    for t in (1, 64, 2048, 16384):
        assert cost.prefill_gemm_flops(t, h, m) == orc.prefill_gemm_flops(t, h, m)
    for lens in ([512] * 4, [1, 17, 300], [2048] * 8):
        assert cost.prefill_attention_flops(lens, h) == orc.prefill_attention_flops(lens, h)


@pytest.mark.parametrize("h,m", SHAPES)
def test_decode_byte_counts_agree(h, m):
    for B in (1, 64, 256):
        # bf16: two bytes per element of App. A.3's 8Bh + 4h^2 + 2hm + 2Bm
        assert cost.decode_gemm_bytes(B, h, m) == 2 * orc.decode_gemm_traffic_elems(B, h, m)
        ctx = [100 + 7 * i for i in range(B)]
        # cost.py takes the attended lengths (context + the new token), the oracle the contexts before the step
        assert cost.decode_attention_bytes([c + 1 for c in ctx], h) == 2 * orc.decode_attention_kv_elems(ctx, h)


def test_copy_counts_are_the_kv_rows_moved():
    h, t, B = 5120, 2048, 64
    per_token_one_layer = orc.kv_bytes_per_token(h, 1)          # K and V rows of one token, bf16
    assert cost.kv_migrate_bytes(t, h) == 2 * t * per_token_one_layer      # read once, written once
    assert cost.kv_append_bytes(B, h) == 2 * B * per_token_one_layer
    assert cost.layernorm_bytes(t, h) == 2 * t * h * 2                     # a bf16 row in, a bf16 row out
