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


def bf16_ulp(x):
    """Spacing of bf16 numbers at |x| (8 significant bits), as fp64."""
    ax = np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


def check_bf16_weights(W_dev, W_orc, W_before, steps, lr, alpha, where=None, expect_moved=True):
    """Per-entry gate on bf16 weights after `steps` steps from W_before (all fp64 arrays of bf16 values;
    W_orc = the oracle's stored weights, rounded to bf16 after every step).  relF on W cannot see the
    update (one step moves W by well under a per cent of its norm), so every entry is bounded: a rounding
    that falls the other way costs one ulp per step (ulp at the larger of old and new weight), and an
    entry of R within rounding distance of zero may flip the sign of its N on the first step after
    zero moments, which moves a weight by a small fraction of lr*alpha.  Nearly all entries are
    identical: the device rounds N to bf16 before the back-projection (N is stored in the tensor's dtype), the
    oracle does not, so the two updates differ by about 2^-9 of their size and a weight lands on the other
    side of a rounding boundary with probability about 2 * 2^-9 |dW| / ulp per step (0.4 % at the paper's
    lr*alpha = 2.5e-4, ten times that at lr = 1e-2).  And the device moved (about) as many weights as the
    oracle did."""
    ulp = np.maximum(bf16_ulp(W_orc), bf16_ulp(W_before))
    err = np.abs(W_dev - W_orc)
    assert np.all(err <= steps * ulp + 0.1 * lr * alpha), (where, float(err.max()), float((steps * ulp).max()))
    same = float(np.mean(W_dev == W_orc))
    per_step = 0.005 + 2.0 ** -8 * float(np.median(np.abs(W_orc - W_before)) / steps / np.median(ulp))
    assert same >= 1.0 - steps * per_step, (where, same, per_step)
    moved_orc = float(np.mean(W_orc != W_before))
    moved_dev = float(np.mean(W_dev != W_before))
    if expect_moved:
        assert moved_orc > 0.2, (where, moved_orc)       # the comparison is not vacuous
    assert moved_dev >= 0.9 * moved_orc - 0.01, (where, moved_dev, moved_orc)
    return same, moved_dev
