"""Build-time assumptions of the hand-scheduled GEMM, checked on the compiler's own assembly output
of this repository's source (no GPU needed).

The weight-update kernel lets its early W prefetch stay in flight across one barrier with
`s_waitcnt vmcnt(8)`: that is only right if the compiler emits exactly 8 vector-memory loads for
the 8 prefetched slices, after the tile loads of the same K step.  A compiler that merged, split
or moved those loads would silently break the wait count; this test would catch it."""
import os
import re
import shutil
import subprocess

import pytest

from conftest import ROOT

HIPCC = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_early_weight_prefetch_is_exactly_eight_loads():
    # the check itself is part of the build (the library is not linked when it fails); here it runs on its own
    from paper_2403_03507_amd import build as lib_build
    assert lib_build.check_weight_prefetch_assembly() == 3


@pytest.mark.skipif(not os.path.exists(HIPCC), reason="hipcc not available")
def test_large_tile_kernel_refuses_operands_beyond_its_32_bit_offsets(tmp_path):
    # The large-tile GEMM addresses an operand with 32-bit byte offsets from its first element, so the
    # host has to route operands of 4 GiB or more to the general kernel (64-bit offsets).  Host code only.
    src = tmp_path / "fits.hip"
    src.write_text(r'''
#include "gemm_mfma_dl.hpp"
#include <cstdio>
using namespace galore;
static GemmGroup one(int M, int N, int K, int lda, int ldb) {
  GemmGroup g{}; g.count = 1;
  GemmProblem& p = g.p[0];
  p.A = reinterpret_cast<const void*>(0x1000); p.B = reinterpret_cast<const void*>(0x2000); p.C = reinterpret_cast<void*>(0x3000);
  p.M = M; p.N = N; p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = N;
  return g;
}
int main() {
  // A as [M][K], B as [N][K], both contiguous along K
  printf("%d", (int)group_fits_dl(one(4096, 4096, 1024, 1024, 1024), true, true, Epilogue::ApplyW));          // ordinary
  printf("%d", (int)group_fits_dl(one(1 << 20, 4096, 1024, 2048, 1024), true, true, Epilogue::ApplyW));       // A: 2^20 x 2048 x 2 B = 4 GiB
  printf("%d", (int)group_fits_dl(one((1 << 20) - 1, 4096, 1024, 2048, 1024), true, true, Epilogue::ApplyW));  // just under
  printf("%d", (int)group_fits_dl(one(4096, 1 << 21, 1024, 1024, 1024), true, true, Epilogue::ApplyW));       // B: 4 GiB
  // B as [K][N]: K rows of ldb elements
  printf("%d\n", (int)group_fits_dl(one(1024, 8192, 1 << 18, 1 << 18, 8192), true, false, Epilogue::StoreF32)); // B: 2^18 x 8192 x 2 B = 4 GiB
  return 0;
}
''')
    exe = str(tmp_path / "fits")
    inc = os.path.join(ROOT, "paper_2403_03507_amd", "csrc")
    subprocess.check_call([HIPCC, "--offload-arch=gfx950", "-O1", "-std=c++17", "-I", inc, "-Xclang", "-target-feature",
                           "-Xclang", "-packed-fp32-ops", "-o", exe, str(src)], stderr=subprocess.DEVNULL)
    assert subprocess.check_output([exe]).decode().strip() == "10100"


def test_three_bf16_parts_hold_an_fp32_number_exactly():
    # The refresh multiplies fp32 matrices on the bf16 matrix cores after splitting every entry into
    # hi + mid + lo (each rounded to nearest even, the remainder formed in fp32).  The claim behind it:
    # the three parts reproduce the fp32 number exactly (8 significant bits apiece), and the six partial
    # products the kernel keeps miss the full product by less than 2^-22 of it.  Checked here with
    # torch's own bf16 rounding on the CPU (same arithmetic as the kernel's split3).
    import torch
    g = torch.Generator().manual_seed(0)
    x = torch.cat([torch.randn(200000, generator=g) * s for s in (1e-20, 1e-6, 1.0, 1e6, 1e20)] +
                  [torch.tensor([0.0, 1.0, -1.0, 3.0e38, -3.0e38, 1.1754944e-38 * 2 ** 20, 0.1, 1.0 + 2 ** -23, 1.0 - 2 ** -24])])

    def split(v):
        hi = v.bfloat16().float()
        r1 = v - hi
        mid = r1.bfloat16().float()
        lo = (r1 - mid).bfloat16().float()
        return hi, mid, lo

    hi, mid, lo = split(x)
    assert torch.equal((hi.double() + mid.double() + lo.double()).float(), x)
    assert torch.equal(hi.double() + mid.double() + lo.double(), x.double())     # not merely after rounding
    y = x[torch.randperm(x.numel(), generator=g)]
    yh, ym, yl = split(y)
    kept = (hi.double() * yh.double() + hi.double() * ym.double() + mid.double() * yh.double() + mid.double() * ym.double()
            + hi.double() * yl.double() + lo.double() * yh.double())
    full = x.double() * y.double()
    ok = full != 0
    assert float(((kept - full).abs()[ok] / full.abs()[ok]).max()) <= 2.0 ** -22
