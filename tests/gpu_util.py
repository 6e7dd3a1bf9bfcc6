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


def rel_err_rows(gpu: np.ndarray, ref: np.ndarray) -> float:
    """The same metric taken row by row (rows = first axis) and maximised: a row of small magnitude that is
    entirely wrong cannot hide behind a large row elsewhere in the tensor."""
    g = gpu.reshape(gpu.shape[0], -1)
    r = ref.reshape(ref.shape[0], -1)
    return float(np.max(np.max(np.abs(g - r), axis=1) / np.max(np.abs(r), axis=1)))


def make_ctx(shape) -> binding.Context:
    return binding.Context(shape.hidden, shape.n_heads, shape.head_dim, shape.ffn, shape.block_size, shape.ln_eps,
                           shape.n_kv_heads)


def workspace(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device="cuda")


def update_ok(y_gpu: np.ndarray, y_ref: np.ndarray, x_in: np.ndarray) -> bool:
    """Gate on the layer's own contribution y - x (the residual input dominates y, so this is the
    sharper check of attention + FFN).  The residual stream is rounded to bf16 twice on the GPU
    (x1 and y), each within half a unit in the last place of its magnitude - for |v| in [2^e, 2^(e+1)) that is
    2^(e-8), between 2^-9 |v| and 2^-8 |v| - taken at the largest magnitude; on top of that the update gets the
    1e-2 budget."""
    upd_ref = y_ref - x_in
    half_ulp = 2.0 ** (np.floor(np.log2(np.max(np.abs(y_ref)))) - 8)
    bound = 2 * half_ulp + 1e-2 * np.max(np.abs(upd_ref))
    return bool(np.max(np.abs((y_gpu - x_in) - upd_ref)) <= bound)


def dev_normal_bits(shape, std: float, seed: int, mean: float = 0.0) -> torch.Tensor:
    """Seeded N(mean, std) bf16 tensor generated ON the device (for inputs too large to draw on the
    host).  The oracle receives the same bits through a device-to-host copy of what it needs."""
    g = torch.Generator(device="cuda")
    g.manual_seed(int(seed))
    t = torch.empty(shape, dtype=torch.float32, device="cuda")
    t.normal_(mean, std, generator=g)
    return t.to(torch.bfloat16)


def dev_layer_weights(shape, seed: int):
    """One layer's parameters drawn on the device with the recipe of synth.make_layer_weights.
    Returns (struct for the C ABI, dict of device tensors)."""
    h, m = shape.hidden, shape.ffn
    w = {
        "ln1_g": dev_normal_bits((h,), 0.02, seed + 1, 1.0), "ln1_b": dev_normal_bits((h,), 0.02, seed + 2),
        "w_qkv": dev_normal_bits((shape.qkv_width, h), 0.02, seed + 3),
        "b_qkv": dev_normal_bits((shape.qkv_width,), 0.02, seed + 4),
        "w_o": dev_normal_bits((h, h), 0.02, seed + 5), "b_o": dev_normal_bits((h,), 0.02, seed + 6),
        "ln2_g": dev_normal_bits((h,), 0.02, seed + 7, 1.0), "ln2_b": dev_normal_bits((h,), 0.02, seed + 8),
        "w_fc1": dev_normal_bits((m, h), 0.02, seed + 9), "b_fc1": dev_normal_bits((m,), 0.02, seed + 10),
        "w_fc2": dev_normal_bits((h, m), 0.02, seed + 11), "b_fc2": dev_normal_bits((h,), 0.02, seed + 12),
    }
    lw, keep = binding.Context.pack_weights(w)
    return lw, keep


def host_weights(wdev: dict) -> dict:
    """Device weights -> numpy bf16 bit patterns (what the oracle consumes)."""
    return {k: to_bits(v) for k, v in wdev.items()}
