"""Small conversions used by the tests (no method arithmetic)."""
import numpy as np
import torch


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """torch tensor (any float dtype) -> uint16 bf16 bit patterns (rne)."""
    t = t.detach().to("cpu").to(torch.bfloat16).contiguous()
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_f64(u: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> exact float64 values."""
    u32 = u.astype(np.uint32) << 16
    return u32.view(np.float32).astype(np.float64)


def f32_to_bits(a) -> np.ndarray:
    return bf16_bits(torch.tensor(np.asarray(a, dtype=np.float32)))
