"""Pins for the oracle's storage rounding (nearest-even fp64 -> bf16 / fp32)."""
import numpy as np
import torch

from oracle import galore_oracle as orc


def test_f32_matches_numpy_cast():
    rng = np.random.default_rng(3)
    x = rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, 20000)
    np.testing.assert_array_equal(orc.round_storage(x, "f32"), x.astype(np.float32).astype(np.float64))


def test_bf16_matches_torch_cast_on_f32_values():
    # torch rounds fp32 -> bf16 to nearest even; on fp32-representable inputs both must agree.
    rng = np.random.default_rng(4)
    x = (rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, 20000)).astype(np.float32)
    ref = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    np.testing.assert_array_equal(orc.round_storage(x.astype(np.float64), "bf16"), ref)


def test_bf16_ties_to_even_and_no_double_rounding():
    # bf16 has 8 significand bits: spacing at 1.0 is 2^-7.
    u = 2.0 ** -7
    x = np.array([1 + u / 2, 1 + 3 * u / 2, 1 + u / 2 + 2.0 ** -40, 1 + u / 2 - 2.0 ** -40, -(1 + u / 2)])
    want = np.array([1.0, 1 + 2 * u, 1 + u, 1.0, -1.0])
    np.testing.assert_array_equal(orc.round_storage(x, "bf16"), want)


def test_bf16_subnormal_and_overflow():
    tiny = 2.0 ** -133  # smallest bf16 subnormal
    x = np.array([tiny, tiny * 0.49, tiny * 1.5, 3.4e38, 0.0])
    got = orc.round_storage(x, "bf16")
    assert got[0] == tiny and got[1] == 0.0 and got[2] == 2 * tiny and np.isinf(got[3]) and got[4] == 0.0
