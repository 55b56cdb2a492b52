"""Shared helpers for the parity tests (no method arithmetic)."""
import numpy as np
import torch

# Per-step gates on W, M, V (relative Frobenius error against the fp64 oracle).
TOL = {"f32": 1e-5, "bf16": 2e-2}
TDT = {"f32": torch.float32, "bf16": torch.bfloat16}


def to64(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def relF(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    d = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (d if d > 0 else 1.0))


def dev(a, dtype, device="cuda"):
    """fp64 numpy (already representable in dtype) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(TDT[dtype] if isinstance(dtype, str) else dtype).to(device).contiguous()


def strided(t, pad):
    """Copy of t living inside a wider buffer, so its leading dimension is cols + pad.  The pad holds
    NaN (floating dtypes): a kernel that lets anything beyond a row's end into a result shows up."""
    fill = float("nan") if t.dtype.is_floating_point else 0
    buf = torch.full((t.shape[0], t.shape[1] + pad), fill, dtype=t.dtype, device=t.device)
    view = buf[:, : t.shape[1]]
    view.copy_(t)
    return view


def f32(x):
    """The value the C ABI receives for a float hyper-parameter; the oracle is given the same number."""
    return float(np.float32(x))
