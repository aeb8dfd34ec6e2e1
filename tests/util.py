"""Small helpers shared by the tests (no method arithmetic)."""
import numpy as np
import torch


def bf16_u16(x) -> np.ndarray:
    """Round a float array to bf16 (nearest even) and return the raw uint16 bit patterns."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.contiguous().view(torch.int16).numpy().view(np.uint16).copy()


def u16_f64(u) -> np.ndarray:
    """Widen raw bf16 bit patterns exactly to float64."""
    u = np.ascontiguousarray(u, dtype=np.uint16)
    return (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def u16_torch(u, device="cpu") -> torch.Tensor:
    """Raw uint16 bit patterns -> torch.bfloat16 tensor."""
    u = np.ascontiguousarray(u, dtype=np.uint16)
    return torch.from_numpy(u.view(np.int16).copy()).view(torch.bfloat16).to(device)
