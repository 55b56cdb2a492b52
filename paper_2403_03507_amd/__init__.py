"""GaLore optimizer step (arXiv 2403.03507, Algorithm 2) as hand-written gfx950 HIP kernels.

``binding`` is the thin ctypes face of ``libgalore.so`` (the C ABI declared in
``include/galore.h``); ``workloads`` makes the seeded synthetic inputs.
"""
