"""Timing of GaLore with Adafactor on the three tensor shapes of a LLaMA-7B layer (r = 1024, bf16 weights):
`python -m paper_2403_03507_amd.adafactor_timing` prints, per shape, the time of a whole galore_adafactor_step (one
tensor per call) and of the update block alone (galore_adafactor) with the rate at which it moves its algorithmic bytes
(three reads of R, M in and out, N out).  Synthetic data, given projectors, HIP events around 20 calls after 3 warm-up calls."""
import torch

from . import binding as gb
from . import workloads as wl


def main(rank=1024, reps=20):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps

    for (m, n) in [(4096, 4096), (4096, 11008), (11008, 4096)]:
        g = torch.Generator(device="cuda")
        g.manual_seed(1)
        W = (torch.randn(m, n, generator=g, device="cuda") * 0.02).to(torch.bfloat16)
        G = (torch.randn(m, n, generator=g, device="cuda") * 0.01).to(torch.bfloat16)
        opt = gb.GaLoreAdafactor(W, rank, auto_refresh=False)
        opt.proj.copy_(wl.random_orthonormal(min(m, n), rank, 5, device="cuda").to(torch.bfloat16))
        step_ms = timed(lambda: opt.step(W, G, 1e-3))
        rows, cols = (rank, n) if m <= n else (m, rank)
        R = torch.randn(rows, cols, device="cuda")
        M = torch.zeros(rows, cols, device="cuda")
        row, col = torch.zeros(rows, device="cuda"), torch.zeros(cols, device="cuda")
        N = torch.empty(rows, cols, dtype=torch.bfloat16, device="cuda")
        ws = torch.empty(8 << 20, dtype=torch.uint8, device="cuda")
        block_ms = timed(lambda: gb.galore_adafactor(R, M, row, col, N, 0.9, 2, ws))
        nbytes = rows * cols * (3 * 4 + 8 + 2)
        print("%5d x %5d  step %.3f ms   update block %.3f ms = %.0f GB/s of its %.0f MB"
              % (m, n, step_ms, block_ms, nbytes / block_ms / 1e6, nbytes / 1e6), flush=True)


if __name__ == "__main__":
    main()
