"""The C-ABI library loads and exports what include/ds.h declares; host-side
argument checks work without a GPU (no kernel is launched here)."""
import ctypes
import os
import re

import pytest

from paper_2401_09670_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ds.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ds_[a-z_]+)\s*\(", text)))


def test_header_symbols_all_exported():
    lib = binding.load_library()
    syms = declared_symbols()
    assert set(syms) == set(binding.EXPORTS)
    for s in syms:
        assert hasattr(lib, s), s


def test_create_validates_config():
    lib = binding.load_library()
    h = ctypes.c_void_p()
    bad = [dict(hidden=256, n_heads=4, head_dim=32, ffn=1024, block_size=16, ln_eps=1e-5),   # head_dim
           dict(hidden=256, n_heads=4, head_dim=64, ffn=1024, block_size=32, ln_eps=1e-5),   # page size
           dict(hidden=250, n_heads=4, head_dim=64, ffn=1024, block_size=16, ln_eps=1e-5),   # h != n*s
           dict(hidden=256, n_heads=4, head_dim=64, ffn=1000, block_size=16, ln_eps=1e-5),   # ffn % 64
           dict(hidden=256, n_heads=4, head_dim=64, ffn=1024, block_size=16, ln_eps=0.0),
           dict(hidden=256, n_heads=4, head_dim=64, ffn=1024, block_size=16, ln_eps=1e-5, n_kv_heads=3),   # 4 % 3
           dict(hidden=256, n_heads=4, head_dim=64, ffn=1024, block_size=16, ln_eps=1e-5, n_kv_heads=8),   # > n
           dict(hidden=256, n_heads=4, head_dim=64, ffn=1024, block_size=16, ln_eps=1e-5, n_kv_heads=-1)]
    for kw in bad:
        cfg = binding.ModelCfg(**kw)
        assert lib.ds_create(ctypes.byref(cfg), ctypes.byref(h)) != binding.DS_OK
        assert not h.value
    assert lib.ds_create(None, ctypes.byref(h)) == 1
    for n_kv in (0, 1, 2, 4):   # 0 = as many as query heads; divisors of n = grouped-query attention
        binding.Context(256, 4, 64, 1024, n_kv_heads=n_kv).close()
    # fewer key/value heads shrink the QKV projection, hence the decode workspace
    assert binding.Context(256, 4, 64, 1024, n_kv_heads=1).ds_decode_workspace_bytes(8, 64) < \
        binding.Context(256, 4, 64, 1024).ds_decode_workspace_bytes(8, 64)


def test_host_argument_checks_return_status():
    ctx = binding.Context(256, 4, 64, 1024)
    assert ctx.ds_prefill_workspace_bytes(64) > 0
    assert ctx.ds_decode_workspace_bytes(2, 48) > 0
    assert ctx.ds_prefill_workspace_bytes(0) == 0
    lib = ctx.lib
    # NULL pointers are rejected before anything touches the device
    st = lib.ds_kv_migrate(ctx.handle, None, None, None, 1, 16, 16, None, 1, None, None, 4, None)
    assert st == 1 and b"NULL" in lib.ds_last_error(ctx.handle)
    st = lib.ds_layernorm(ctx.handle, None, None, None, 4, None, None)
    assert st == 1
    lw = binding.LayerWeights()
    st = lib.ds_prefill(ctx.handle, ctypes.byref(lw), None, None, 1, 16, 16, None, None, None, None, 0, None)
    assert st == 1
    # inconsistent sizes: 3 blocks of 16 cannot hold 64 tokens
    st = lib.ds_kv_migrate(ctx.handle, 16, 16, 16, 1, 64, 64, 16, 3, 16, 16, 8, None)
    assert st == 1 and b"does not fit" in lib.ds_last_error(ctx.handle)
    # misaligned pointer
    st = lib.ds_kv_migrate(ctx.handle, 8, 16, 16, 1, 64, 64, 16, 4, 16, 16, 8, None)
    assert st == 1 and b"aligned" in lib.ds_last_error(ctx.handle)
    ctx.close()


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libds.so")
    with pytest.raises(RuntimeError):
        binding.Context(256, 4, 64, 1024)


@pytest.mark.parametrize("hidden,n_heads,head_dim,ffn,n_kv", [
    (256, 4, 64, 1024, 0), (5120, 40, 128, 20480, 0), (8192, 64, 128, 28672, 8), (2048, 16, 128, 4096, 1),
])
def test_workspace_for_a_maximum_serves_every_smaller_call(hidden, n_heads, head_dim, ffn, n_kv):
    """A caller sizes one workspace for its largest batch; smaller batches may split K or the KV axis over
    more workgroups (more partial sums), and must still fit."""
    ctx = binding.Context(hidden, n_heads, head_dim, ffn, n_kv_heads=n_kv)
    for max_batch, max_ctx in ((1, 16), (7, 300), (64, 4096), (256, 2048)):
        cap = ctx.ds_decode_workspace_bytes(max_batch, max_ctx)
        assert cap > 0
        for b in sorted(b for b in {1, 2, 3, max_batch // 2, max_batch - 1, max_batch} if 1 <= b <= max_batch):
            for c in (1, max_ctx // 3 or 1, max_ctx):
                assert ctx.ds_decode_workspace_bytes(b, c) <= cap, (max_batch, max_ctx, b, c)
    for max_tokens in (1, 100, 2048, 5000):
        cap = ctx.ds_prefill_workspace_bytes(max_tokens)
        for t in sorted({1, max_tokens // 2 or 1, max_tokens}):
            assert ctx.ds_prefill_workspace_bytes(t) <= cap
