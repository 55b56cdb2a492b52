"""Per-layer weight updates from autograd hooks (Sec. 4.3: update a layer's weights as soon as its
gradients exist, then drop them) against the same steps issued by hand after a plain backward pass."""
import pytest
import torch

from paper_2403_03507_amd import binding as gb
from paper_2403_03507_amd.hooks import PerLayerGaLore

pytestmark = pytest.mark.gpu


class Block(torch.nn.Module):
    def __init__(self, d, f, dtype):
        super().__init__()
        self.up = torch.nn.Linear(d, f, bias=False, dtype=dtype, device="cuda")
        self.gate = torch.nn.Linear(d, f, bias=False, dtype=dtype, device="cuda")
        self.down = torch.nn.Linear(f, d, bias=False, dtype=dtype, device="cuda")

    def forward(self, x):
        return x + self.down(torch.nn.functional.silu(self.gate(x)) * self.up(x))


def _model(seed, dtype):
    torch.manual_seed(seed)
    return torch.nn.Sequential(*[Block(256, 512, dtype) for _ in range(3)])


def _layers(model):
    return [[b.up.weight, b.gate.weight, b.down.weight] for b in model]


@pytest.mark.parametrize("overlap", [False, True])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_hook_driven_updates_equal_manual_steps_bitwise(dtype, overlap):
    rank, lr, steps = 32, 1e-2, 3
    xs = [torch.randn(64, 256, device="cuda", generator=torch.Generator("cuda").manual_seed(100 + s)).to(dtype) for s in range(steps)]

    hooked = _model(7, dtype)
    drv = PerLayerGaLore(_layers(hooked), rank, lr, overlap_calls=overlap, update_gap=2, refresh_iters=3)
    for s in range(steps):
        hooked(xs[s]).float().pow(2).mean().backward()
        drv.finish()
        assert all(p.grad is None for l in _layers(hooked) for p in l)   # gradients were dropped layer by layer
    torch.cuda.synchronize()

    manual = _model(7, dtype)
    flat = [p for l in _layers(manual) for p in l]
    opt = gb.GaLore([p.data for p in flat], rank, update_gap=2, refresh_iters=3)
    for s in range(steps):
        manual(xs[s]).float().pow(2).mean().backward()
        for li in reversed(range(3)):                                     # the order backward reaches the blocks
            ps = flat[3 * li: 3 * li + 3]
            opt.step([p.data for p in ps], [p.grad for p in ps], lr, first=3 * li)
        for p in flat:
            p.grad = None
    torch.cuda.synchronize()

    for a, b in zip([p for l in _layers(hooked) for p in l], flat):
        assert torch.equal(a.data, b.data)
    for x, y in zip(drv.opt.M + drv.opt.V + drv.opt.proj, opt.M + opt.V + opt.proj):
        assert torch.equal(x, y)
    drv.close()
    opt.close()


def test_overhead_script_runs_on_a_small_stack():
    from paper_2403_03507_amd import llama_overhead
    out = llama_overhead.main(["--d", "256", "--f", "512", "--heads", "4", "--layers", "2", "--rank", "64", "--batch", "2",
                               "--seq", "64", "--reps", "1"])
    assert out["ms_forward_backward"] > 0 and out["ms_with_galore"] > 0 and out["tokens_per_s_with_galore"] > 0
