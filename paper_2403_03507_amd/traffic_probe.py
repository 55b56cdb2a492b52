"""Workload for rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (HBM traffic of the step kernels).

Runs a few steps of the library on LLaMA-7B-shaped layer sets with a given projector (no
refresh: its thousands of tiny launches would only slow the counter run down), strictly serial,
followed by one 1 GiB device-to-device copy whose traffic is known exactly (2^30 bytes read,
2^30 bytes written) and calibrates the counters.  Usage (on the GPU machine, from the repo root):

    rocprofv3 --pmc FETCH_SIZE --output-format csv -d /tmp/pmc_f -o f -- python3 paper_2403_03507_amd/traffic_probe.py
    rocprofv3 --pmc WRITE_SIZE --output-format csv -d /tmp/pmc_w -o w -- python3 paper_2403_03507_amd/traffic_probe.py
"""
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_2403_03507_amd import binding as gb  # noqa: E402
from paper_2403_03507_amd import workloads as wl  # noqa: E402


def main(layers=3, steps=2):
    torch.cuda.set_device(0)
    c = wl.CONFIGS["llama7b"]
    shapes = wl.layer_shapes(c["d"], c["f"])
    r = c["rank"]
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    W = [(torch.randn(m, n, generator=gen, device="cuda") * 0.02).to(torch.bfloat16) for _ in range(layers) for (m, n) in shapes]
    G = [(torch.randn(m, n, generator=gen, device="cuda") * 0.01).to(torch.bfloat16) for _ in range(layers) for (m, n) in shapes]
    opt = gb.GaLore(W, r, auto_refresh=False)
    gb.galore_set_concurrency(opt.ctx, 1)
    for p in opt.proj:  # traffic does not depend on the values: a scaled Gaussian block stands in for a projector
        p.copy_((torch.randn(p.shape, generator=gen, device="cuda") / 64).to(torch.bfloat16))
    n7 = len(shapes)
    for s in range(steps):
        for l in reversed(range(layers)):
            opt.step(W[n7 * l: n7 * (l + 1)], G[n7 * l: n7 * (l + 1)], 1e-3, first=n7 * l)
        torch.cuda.synchronize()
        print("step", s, "done", flush=True)
    src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    dst.copy_(src)
    torch.cuda.synchronize()
    print("copy done", flush=True)


if __name__ == "__main__":
    main()
