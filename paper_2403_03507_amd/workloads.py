"""Seeded synthetic workloads: LLaMA-shaped weight/gradient stacks.

Input generation only.  Nothing here performs any part of the optimizer step:
the HIP library and the CPU oracle are both handed the tensors made here, so
both consume identical bits.  Shapes follow the LLaMA sizes in the paper's
hyper-parameter table (App. C); gradients are "low-rank signal + Gaussian
noise" or "power-law spectrum + noise", standing in for the C4 gradients the
paper trained on (Sec. 3.2 argues such gradients become low-rank).
"""
import math

import torch

# name -> (layers, hidden d, ffn f, rank, update_gap T, dtype, gradient kind, kind params)
CONFIGS = {
    "llama60m": dict(layers=1, d=512, f=1376, rank=128, update_gap=5, dtype="f32",
                     grad="lowrank", signal_rank=32, sigma0=10.0, decay=0.8, noise=0.01),
    "llama130m": dict(layers=12, d=768, f=2048, rank=256, update_gap=200, dtype="bf16",
                      grad="lowrank", signal_rank=64, sigma0=10.0, decay=0.9, noise=0.01),
    "llama350m": dict(layers=24, d=1024, f=2736, rank=256, update_gap=200, dtype="bf16",
                      grad="powerlaw", noise=1e-3),
    "llama1b": dict(layers=24, d=2048, f=5461, rank=512, update_gap=200, dtype="bf16",
                    grad="lowrank", signal_rank=128, sigma0=10.0, decay=0.95, noise=0.01),
    "llama7b": dict(layers=32, d=4096, f=11008, rank=1024, update_gap=200, dtype="bf16",
                    grad="powerlaw", noise=1e-3),
}
DEFAULTS = dict(scale=0.25, lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.0)

TORCH_DTYPE = {"f32": torch.float32, "bf16": torch.bfloat16}


def layer_shapes(d, f):
    """The seven GaLore matrices of one LLaMA layer: q, k, v, o, gate, up, down."""
    return [(d, d)] * 4 + [(d, f)] * 2 + [(f, d)]


def stack_shapes(cfg):
    c = CONFIGS[cfg] if isinstance(cfg, str) else cfg
    return [s for _ in range(c["layers"]) for s in layer_shapes(c["d"], c["f"])]


def _gen(seed, device):
    g = torch.Generator(device=device)
    g.manual_seed(int(seed) & 0x7FFFFFFFFFFFFFFF)
    return g


def _key(*parts):
    """Mix integers into one 63-bit seed (splitmix-style), so every (tensor, step) has its own stream."""
    x = 0x9E3779B97F4A7C15
    for p in parts:
        x ^= (int(p) + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2)) & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    return x & 0x7FFFFFFFFFFFFFFF


def make_weight(m, n, seed, dtype="f32", device="cpu", std=0.02):
    g = _gen(_key(seed, 1, m, n), device)
    w = torch.randn(m, n, generator=g, device=device, dtype=torch.float32) * std
    return w.to(TORCH_DTYPE[dtype]).contiguous()


def random_orthonormal(rows, cols, seed, device="cpu"):
    """rows x cols matrix with orthonormal columns (QR of a Gaussian), fp32."""
    assert cols <= rows
    g = _gen(_key(seed, 2, rows, cols), device)
    a = torch.randn(rows, cols, generator=g, device=device, dtype=torch.float32)
    q, r = torch.linalg.qr(a)
    return (q * torch.sign(torch.diagonal(r)).unsqueeze(0)).contiguous()


class GradientSource:
    """Per-tensor gradient stream: fixed singular factors, fresh noise every step."""

    def __init__(self, m, n, seed, kind, device="cpu", dtype="f32", signal_rank=32,
                 sigma0=10.0, decay=0.8, noise=0.01, max_components=1024, gap_rank=None,
                 gap_ratio=4.0):
        self.m, self.n, self.seed, self.kind = m, n, seed, kind
        self.device, self.dtype, self.noise = device, dtype, noise
        k_full = min(m, n)
        if kind == "lowrank":
            k = min(signal_rank, k_full)
            sig = sigma0 * decay ** torch.arange(k, dtype=torch.float32)
        elif kind == "powerlaw":
            # sigma_i = C / i with C = 1e-2 sqrt(mn); components beyond max_components lie
            # far under the noise floor noise*(sqrt(m)+sqrt(n)) and are dropped.
            k = min(k_full, max_components)
            sig = 1e-2 * math.sqrt(m * n) / torch.arange(1, k + 1, dtype=torch.float32)
        elif kind == "gapped":
            # exactly gap_rank signal directions, geometric from sigma0 down to sigma0/20,
            # then nothing but noise whose spectral norm stays under sigma_r / gap_ratio.
            k = gap_rank
            sig = sigma0 * (1.0 / 20.0) ** (torch.arange(k, dtype=torch.float32) / max(k - 1, 1))
            self.noise = float(sig[-1]) / gap_ratio / (math.sqrt(m) + math.sqrt(n)) / 1.1
        else:
            raise ValueError(kind)
        self.sigma = sig.to(device)
        self.U = random_orthonormal(m, k, _key(seed, 11), device)
        self.V = random_orthonormal(n, k, _key(seed, 12), device)
        self.US = (self.U * self.sigma.unsqueeze(0)).contiguous()

    def grad(self, step):
        g = _gen(_key(self.seed, 3, step), self.device)
        out = torch.randn(self.m, self.n, generator=g, device=self.device, dtype=torch.float32)
        out.mul_(self.noise)
        out.addmm_(self.US, self.V.t())
        return out.to(TORCH_DTYPE[self.dtype]).contiguous()


def make_sources(cfg, seed=0, device="cpu", layers=None):
    """One GradientSource per tensor of the stack.  Singular factors are shared per shape
    (one Haar pair per distinct (m, n)), as a full pair per tensor would only cost time."""
    c = dict(CONFIGS[cfg]) if isinstance(cfg, str) else dict(cfg)
    if layers is not None:
        c["layers"] = layers
    shapes = stack_shapes(c)
    cache, out = {}, []
    for i, (m, n) in enumerate(shapes):
        kw = dict(kind=c["grad"], device=device, dtype=c["dtype"], noise=c["noise"])
        for k in ("signal_rank", "sigma0", "decay"):
            if k in c:
                kw[k] = c[k]
        if (m, n) not in cache:
            cache[(m, n)] = GradientSource(m, n, _key(seed, m, n), **kw)
        base = cache[(m, n)]
        src = GradientSource.__new__(GradientSource)
        src.__dict__.update(base.__dict__)
        src.seed = _key(seed, 100 + i)
        out.append(src)
    return out
