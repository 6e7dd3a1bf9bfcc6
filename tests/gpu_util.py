"""Helpers for the GPU parity tests: numpy bf16 bit patterns <-> device tensors."""
import numpy as np
import torch

from paper_2401_09670_amd import binding


def to_dev(bits: np.ndarray) -> torch.Tensor:
    """uint16 bf16 bit patterns -> bf16 CUDA tensor with identical bits."""
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    return t.cuda().view(torch.bfloat16)


def to_bits(t: torch.Tensor) -> np.ndarray:
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def i32_dev(a) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()


def weights_to_dev(wbits: dict):
    dev = {k: to_dev(v) for k, v in wbits.items()}
    lw, keep = binding.Context.pack_weights(dev)
    return lw, keep


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max|gpu - ref| / max|ref| over one tensor: the parity gate (<= 1e-2)."""
    return float(np.max(np.abs(gpu - ref)) / np.max(np.abs(ref)))


def make_ctx(shape) -> binding.Context:
    return binding.Context(shape.hidden, shape.n_heads, shape.head_dim, shape.ffn, shape.block_size, shape.ln_eps)


def workspace(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def update_ok(y_gpu: np.ndarray, y_ref: np.ndarray, x_in: np.ndarray) -> bool:
    """Gate on the layer's own contribution y - x (the residual input dominates y, so this is the
    sharper check of attention + FFN).  The residual stream is rounded to bf16 twice on the GPU
    (x1 and y), each within 2^-9 of its magnitude; on top of that the update gets the 1e-2 budget."""
    upd_ref = y_ref - x_in
    bound = 2 * 2.0 ** -9 * np.max(np.abs(y_ref)) + 1e-2 * np.max(np.abs(upd_ref))
    return bool(np.max(np.abs((y_gpu - x_in) - upd_ref)) <= bound)
