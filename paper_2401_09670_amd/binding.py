"""ctypes binding of libds.so — argument marshalling only.

Every function here has the name and argument order of its C counterpart in
``include/ds.h`` (minus the context, which ``Context`` carries).  Tensors are
torch CUDA tensors used purely as device buffers: the binding passes
``data_ptr()`` and sizes, and the current torch stream as the HIP stream.
There is no CPU fallback: if the library cannot be loaded, calls raise.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Tuple

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(PKG_DIR, "libds.so")

DS_OK = 0
STATIC_SCRATCH_BYTES = 32 << 20   # DS_STATIC_SCRATCH_BYTES of include/ds.h
STATUS_NAMES = {0: "DS_OK", 1: "DS_ERR_INVALID_ARG", 2: "DS_ERR_UNSUPPORTED", 3: "DS_ERR_WORKSPACE",
                4: "DS_ERR_HIP", 5: "DS_ERR_BOUNDS"}
KERNEL_CLASSES = ("layernorm", "gemm", "prefill_attn", "kv_migrate", "skinny_gemm", "decode_attn", "kv_append",
                  "token_io")

# every symbol include/ds.h declares
EXPORTS = ("ds_create", "ds_destroy", "ds_last_error", "ds_set_validate", "ds_prefill_workspace_bytes",
           "ds_decode_workspace_bytes", "ds_prefill", "ds_kv_migrate", "ds_decode_step", "ds_decode_step_static",
           "ds_layernorm",
           "ds_linear_workspace_bytes", "ds_linear_plan", "ds_linear", "ds_prefill_attention", "ds_decode_attention",
           "ds_embed", "ds_next_token_workspace_bytes", "ds_next_token", "ds_profile_enable", "ds_profile_collect")


class DsError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{STATUS_NAMES.get(status, status)}: {text}")
        self.status = status


class ModelCfg(ctypes.Structure):
    _fields_ = [("hidden", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("ffn", ctypes.c_int32), ("block_size", ctypes.c_int32), ("ln_eps", ctypes.c_float),
                ("n_kv_heads", ctypes.c_int32)]


class LayerWeights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_void_p) for n in
                ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b",
                 "w_fc1", "b_fc1", "w_fc2", "b_fc2")]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libds.so (built in-tree by ``build.build_library``); raises if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() "
                           "(there is no fallback path)")
    # torch ships a HIP runtime of its own under the same library name: it has to be the one in the process
    # before libds.so asks for it, or torch later finds the system's copy loaded in its place (seen as a
    # segmentation fault at torch's first GPU call when this library was loaded first)
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    lib.ds_create.argtypes = [ctypes.POINTER(ModelCfg), ctypes.POINTER(vp)]
    lib.ds_create.restype = ctypes.c_int
    lib.ds_destroy.argtypes = [vp]
    lib.ds_destroy.restype = None
    lib.ds_last_error.argtypes = [vp]
    lib.ds_last_error.restype = ctypes.c_char_p
    lib.ds_set_validate.argtypes = [vp, i32]
    lib.ds_set_validate.restype = ctypes.c_int
    lib.ds_prefill_workspace_bytes.argtypes = [vp, i32]
    lib.ds_prefill_workspace_bytes.restype = sz
    lib.ds_decode_workspace_bytes.argtypes = [vp, i32, i32]
    lib.ds_decode_workspace_bytes.restype = sz
    lib.ds_prefill.argtypes = [vp, ctypes.POINTER(LayerWeights), vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    lib.ds_prefill.restype = ctypes.c_int
    lib.ds_kv_migrate.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, i32, vp, vp, i32, vp]
    lib.ds_kv_migrate.restype = ctypes.c_int
    lib.ds_decode_step.argtypes = [vp, ctypes.POINTER(LayerWeights), vp, vp, vp, i32, i32, i32, vp, vp, i32,
                                   vp, vp, sz, vp]
    lib.ds_decode_step.restype = ctypes.c_int
    lib.ds_decode_step_static.argtypes = [vp, ctypes.POINTER(LayerWeights), vp, vp, vp, i32, i32, i32, vp, vp, i32,
                                          vp, vp]
    lib.ds_decode_step_static.restype = ctypes.c_int
    lib.ds_layernorm.argtypes = [vp, vp, vp, vp, i32, vp, vp]
    lib.ds_layernorm.restype = ctypes.c_int
    lib.ds_linear_workspace_bytes.argtypes = [vp, i32, i32, i32]
    lib.ds_linear_workspace_bytes.restype = sz
    lib.ds_linear_plan.argtypes = [vp, i32, i32, i32] + [ctypes.POINTER(ctypes.c_int32)] * 5
    lib.ds_linear_plan.restype = ctypes.c_int
    lib.ds_linear.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, vp, sz, vp]
    lib.ds_linear.restype = ctypes.c_int
    lib.ds_prefill_attention.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, vp, vp]
    lib.ds_prefill_attention.restype = ctypes.c_int
    lib.ds_decode_attention.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, vp, i32, vp, vp, sz, vp]
    lib.ds_decode_attention.restype = ctypes.c_int
    lib.ds_embed.argtypes = [vp, vp, vp, vp, i32, vp, i32, i32, vp, vp]
    lib.ds_embed.restype = ctypes.c_int
    lib.ds_next_token_workspace_bytes.argtypes = [vp, i32, i32]
    lib.ds_next_token_workspace_bytes.restype = sz
    lib.ds_next_token.argtypes = [vp, vp, vp, i32, vp, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.ds_next_token.restype = ctypes.c_int
    lib.ds_profile_enable.argtypes = [vp, i32]
    lib.ds_profile_enable.restype = ctypes.c_int
    lib.ds_profile_collect.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64)]
    lib.ds_profile_collect.restype = ctypes.c_int
    _lib = lib
    return lib


def _ptr(t) -> Optional[int]:
    """Device (or NULL) pointer of a torch tensor."""
    if t is None:
        return None
    return t.data_ptr()


def _stream() -> Optional[int]:
    import torch
    s = torch.cuda.current_stream().cuda_stream
    return s if s else None


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


class Context:
    """``ds_ctx`` for one layer shape; methods mirror the C entry points."""

    def __init__(self, hidden: int, n_heads: int, head_dim: int, ffn: int, block_size: int = 16,
                 ln_eps: float = 1e-5, n_kv_heads: int = 0):
        self.lib = load_library()
        self.cfg = ModelCfg(hidden, n_heads, head_dim, ffn, block_size, ln_eps, n_kv_heads)
        self.handle = ctypes.c_void_p()
        st = self.lib.ds_create(ctypes.byref(self.cfg), ctypes.byref(self.handle))
        if st != DS_OK:
            self.handle = ctypes.c_void_p()
            raise DsError(st, "ds_create rejected the configuration")

    def close(self):
        if getattr(self, "handle", None) and self.handle.value:
            self.lib.ds_destroy(self.handle)
            self.handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, st: int):
        if st != DS_OK:
            raise DsError(st, self.lib.ds_last_error(self.handle).decode())

    @staticmethod
    def pack_weights(w: Dict[str, "object"]) -> Tuple[LayerWeights, dict]:
        """dict of device tensors (missing / None bias = NULL) -> (struct, keep-alive dict)."""
        lw = LayerWeights()
        for name, _ in LayerWeights._fields_:
            setattr(lw, name, _ptr(w.get(name)))
        return lw, w

    def ds_set_validate(self, on: bool):
        self._check(self.lib.ds_set_validate(self.handle, 1 if on else 0))

    # ---- sizes ----
    def ds_prefill_workspace_bytes(self, max_tokens: int) -> int:
        return self.lib.ds_prefill_workspace_bytes(self.handle, max_tokens)

    def ds_decode_workspace_bytes(self, max_batch: int, max_ctx: int) -> int:
        return self.lib.ds_decode_workspace_bytes(self.handle, max_batch, max_ctx)

    def ds_linear_workspace_bytes(self, rows: int, in_f: int, out_f: int) -> int:
        return self.lib.ds_linear_workspace_bytes(self.handle, rows, in_f, out_f)

    # ---- the three calls of the path ----
    def ds_prefill(self, weights: LayerWeights, x, cu_seqlens, B: int, t: int, max_seqlen: int, y, k_out, v_out,
                   workspace):
        self._check(self.lib.ds_prefill(self.handle, ctypes.byref(weights), _ptr(x), _ptr(cu_seqlens), B, t,
                                        max_seqlen, _ptr(y), _ptr(k_out), _ptr(v_out), _ptr(workspace),
                                        _nbytes(workspace), _stream()))

    def ds_kv_migrate(self, k_src, v_src, cu_seqlens, B: int, t: int, max_seqlen: int, block_tables,
                      max_blocks_per_seq: int, k_cache, v_cache, num_blocks: int):
        self._check(self.lib.ds_kv_migrate(self.handle, _ptr(k_src), _ptr(v_src), _ptr(cu_seqlens), B, t,
                                           max_seqlen, _ptr(block_tables), max_blocks_per_seq, _ptr(k_cache),
                                           _ptr(v_cache), num_blocks, _stream()))

    def ds_decode_step(self, weights: LayerWeights, x, ctx_lens, block_tables, B: int, max_blocks_per_seq: int,
                       max_ctx: int, k_cache, v_cache, num_blocks: int, y, workspace):
        self._check(self.lib.ds_decode_step(self.handle, ctypes.byref(weights), _ptr(x), _ptr(ctx_lens),
                                            _ptr(block_tables), B, max_blocks_per_seq, max_ctx, _ptr(k_cache),
                                            _ptr(v_cache), num_blocks, _ptr(y), _ptr(workspace),
                                            _nbytes(workspace), _stream()))

    def ds_decode_step_static(self, weights: LayerWeights, x, ctx_lens, block_tables, B: int,
                              max_blocks_per_seq: int, max_ctx: int, k_cache, v_cache, num_blocks: int, y):
        self._check(self.lib.ds_decode_step_static(self.handle, ctypes.byref(weights), _ptr(x), _ptr(ctx_lens),
                                                   _ptr(block_tables), B, max_blocks_per_seq, max_ctx,
                                                   _ptr(k_cache), _ptr(v_cache), num_blocks, _ptr(y), _stream()))

    # ---- single steps ----
    def ds_layernorm(self, x, gamma, beta, rows: int, out):
        self._check(self.lib.ds_layernorm(self.handle, _ptr(x), _ptr(gamma), _ptr(beta), rows, _ptr(out),
                                          _stream()))

    def ds_linear_plan(self, rows: int, in_f: int, out_f: int) -> dict:
        v = [ctypes.c_int32() for _ in range(5)]
        self._check(self.lib.ds_linear_plan(self.handle, rows, in_f, out_f, *[ctypes.byref(a) for a in v]))
        return dict(streaming=bool(v[0].value), tile_rows=v[1].value, tile_cols=v[2].value, splits=v[3].value,
                    cut_cols=v[4].value)

    def ds_linear(self, x, w, bias, residual, relu: int, rows: int, in_f: int, out_f: int, y, workspace=None):
        self._check(self.lib.ds_linear(self.handle, _ptr(x), _ptr(w), _ptr(bias), _ptr(residual), relu, rows,
                                       in_f, out_f, _ptr(y), _ptr(workspace), _nbytes(workspace), _stream()))

    def ds_prefill_attention(self, q, k, v, cu_seqlens, B: int, t: int, max_seqlen: int, o):
        self._check(self.lib.ds_prefill_attention(self.handle, _ptr(q), _ptr(k), _ptr(v), _ptr(cu_seqlens), B, t,
                                                  max_seqlen, _ptr(o), _stream()))

    def ds_decode_attention(self, q, kv_lens, block_tables, B: int, max_blocks_per_seq: int, max_kv_len: int,
                            k_cache, v_cache, num_blocks: int, o, workspace=None):
        self._check(self.lib.ds_decode_attention(self.handle, _ptr(q), _ptr(kv_lens), _ptr(block_tables), B,
                                                 max_blocks_per_seq, max_kv_len, _ptr(k_cache), _ptr(v_cache),
                                                 num_blocks, _ptr(o), _ptr(workspace), _nbytes(workspace),
                                                 _stream()))

    # ---- the two ends of the token loop ----
    def ds_embed(self, token_ids, positions, tok_emb, vocab: int, pos_emb, n_pos: int, rows: int, x):
        self._check(self.lib.ds_embed(self.handle, _ptr(token_ids), _ptr(positions), _ptr(tok_emb), vocab,
                                      _ptr(pos_emb), n_pos, rows, _ptr(x), _stream()))

    def ds_next_token_workspace_bytes(self, rows: int, vocab: int) -> int:
        return self.lib.ds_next_token_workspace_bytes(self.handle, rows, vocab)

    def ds_next_token(self, x, row_index, rows: int, ln_g, ln_b, w_vocab, vocab: int, next_token, best_logit,
                      workspace):
        self._check(self.lib.ds_next_token(self.handle, _ptr(x), _ptr(row_index), rows, _ptr(ln_g), _ptr(ln_b),
                                           _ptr(w_vocab), vocab, _ptr(next_token), _ptr(best_logit),
                                           _ptr(workspace), _nbytes(workspace), _stream()))

    # ---- timing ----
    def ds_profile_enable(self, on: bool):
        self._check(self.lib.ds_profile_enable(self.handle, 1 if on else 0))

    def ds_profile_collect(self):
        n = len(KERNEL_CLASSES)
        ms = (ctypes.c_double * n)()
        cnt = (ctypes.c_int64 * n)()
        self._check(self.lib.ds_profile_collect(self.handle, ms, cnt))
        return {k: (ms[i], cnt[i]) for i, k in enumerate(KERNEL_CLASSES)}
