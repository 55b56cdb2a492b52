"""galore_step_static (the entry point that allocates nothing: transients in the library's static device array)
against galore_step, through the C ABI: two calls in a row, the second with a smaller input, bit for bit; the size
limit; the refusal of a step that is due for a refresh."""
import pytest
import torch

from paper_2403_03507_amd import binding as gb
from paper_2403_03507_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _setup(specs, rank, **kw):
    W = [wl.make_weight(m, n, 900 + i, dt).cuda() for i, ((m, n), dt) in enumerate(specs)]
    opt = gb.GaLore(W, rank, auto_refresh=False, **kw)
    for i, ((m, n), dt) in enumerate(specs):
        opt.proj[i].copy_(wl.random_orthonormal(min(m, n), rank, 950 + i).to(wl.TORCH_DTYPE[dt]))
    return W, opt


@pytest.mark.parametrize("fused_adam", [False, True])
def test_static_scratch_step_equals_workspace_step_on_two_calls_in_a_row(fused_adam):
    # call 1: four tensors (both orientations, bf16 and fp32, one with an odd row length: padded copy of G and the
    # any-alignment weight update); call 2, right behind it on the same stream: one small tensor, so most of the array
    # still holds call 1's transients
    specs = [((256, 688), "bf16"), ((688, 256), "bf16"), ((128, 333), "bf16"), ((320, 256), "f32"), ((64, 96), "bf16")]
    rank = 64
    srcs = [wl.GradientSource(m, n, 970 + i, "lowrank", dtype=dt) for i, ((m, n), dt) in enumerate(specs)]
    Wa, a = _setup(specs, rank)
    Wb, b = _setup(specs, rank)
    a.set_fused_adam(fused_adam)      # Adam in the projection's epilogue (the aligned bf16 tensors) or as its own kernel
    b.set_fused_adam(fused_adam)
    for step in range(3):
        G = [s.grad(step).cuda() for s in srcs]
        a.step(Wa[:4], G[:4], 1e-2, first=0)
        a.step(Wa[4:], G[4:], 1e-2, first=4)
        b.step_static(Wb[:4], G[:4], 1e-2, first=0)
        b.step_static(Wb[4:], G[4:], 1e-2, first=4)          # smaller input, no synchronisation in between
        torch.cuda.synchronize()
        for i in range(len(specs)):
            assert b.get_step(i) == a.get_step(i) == step + 1
            assert torch.equal(Wa[i], Wb[i]), (step, i)
            assert torch.equal(a.M[i], b.M[i]) and torch.equal(a.V[i], b.V[i]), (step, i)
    # the workspace path keeps working on the context that used the static path, and the other way round
    G = [s.grad(7).cuda() for s in srcs]
    a.step_static(Wa, G, 1e-2)
    b.step(Wb, G, 1e-2)
    torch.cuda.synchronize()
    for i in range(len(specs)):
        assert torch.equal(Wa[i], Wb[i]) and torch.equal(a.M[i], b.M[i]) and torch.equal(a.V[i], b.V[i])
    a.close()
    b.close()


def test_static_scratch_groups_split_when_the_array_is_full():
    # 1024 x 6144 at r = 1024: 24 + 12 MiB of transients per tensor, so three of them do not fit 80 MiB together and
    # the call runs as two launch groups that reuse the array in stream order
    specs = [((1024, 6144), "bf16")] * 3
    rank = 1024
    srcs = [wl.GradientSource(m, n, 990 + i, "lowrank", dtype=dt, device="cuda") for i, ((m, n), dt) in enumerate(specs)]
    Wa, a = _setup(specs, rank)
    Wb, b = _setup(specs, rank)
    for step in range(2):
        G = [s.grad(step) for s in srcs]
        a.step(Wa, G, 1e-2)
        b.step_static(Wb, G, 1e-2)
    torch.cuda.synchronize()
    for i in range(3):
        assert torch.equal(Wa[i], Wb[i]) and torch.equal(a.M[i], b.M[i]) and torch.equal(a.V[i], b.V[i])
    a.close()
    b.close()


def test_static_scratch_rejects_what_it_cannot_hold_and_steps_due_for_a_refresh():
    # 1024 x 16384 at r = 1024 needs 64 + 32 MiB of transients: beyond the array
    W = [torch.full((1024, 16384), 0.5, dtype=torch.bfloat16, device="cuda")]
    big = gb.GaLore(W, 1024, auto_refresh=False)
    G = [torch.ones_like(w) for w in W]
    with pytest.raises(gb.GaloreError) as e:
        big.step_static(W[:1], G[:1], 1e-2)
    assert e.value.status == 6 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert big.get_step(0) == 0 and torch.all(W[0] == 0.5) and torch.all(big.M[0] == 0)   # nothing ran
    big.close()
    # auto_refresh on: the first step (t = 0) is due for a refresh and is refused; after galore_step took it, the
    # following steps run from the array until the next refresh falls due
    specs = [((256, 688), "bf16"), ((688, 256), "bf16")]
    Wa = [wl.make_weight(m, n, 900 + i, dt).cuda() for i, ((m, n), dt) in enumerate(specs)]
    Wb = [w.clone() for w in Wa]
    srcs = [wl.GradientSource(m, n, 970 + i, "gapped", dtype=dt, gap_rank=32) for i, ((m, n), dt) in enumerate(specs)]
    a = gb.GaLore(Wa, 32, update_gap=3, refresh_iters=3)
    b = gb.GaLore(Wb, 32, update_gap=3, refresh_iters=3)
    for step in range(5):
        G = [s.grad(step).cuda() for s in srcs]
        a.step(Wa, G, 1e-2)
        if step % 3 == 0:
            with pytest.raises(gb.GaloreError) as e:
                b.step_static(Wb, G, 1e-2)
            assert e.value.status == 9
            assert b.get_step(0) == step
            b.step(Wb, G, 1e-2)
        else:
            b.step_static(Wb, G, 1e-2)
    torch.cuda.synchronize()
    for i in range(2):
        assert torch.equal(Wa[i], Wb[i]) and torch.equal(a.M[i], b.M[i]) and torch.equal(a.proj[i], b.proj[i])
    a.close()
    b.close()
