// Host side of the grouped projection GEMM (gemm_proj_dl.hpp): tile plan, the split of the tiles that do not
// fill a round of the persistent grid into K pieces, and the two launches (GEMM, sum of the partial tiles).
#include "gemm_dispatch.hpp"
#include "gemm_proj_dl.hpp"

namespace galore {

bool proj_problem_fits(const ProjProblem& p) {
  GemmGroup one{};
  one.count = 1;
  GemmProblem& q = one.p[0];
  q.A = p.A; q.B = p.B; q.C = p.R;
  q.M = p.M; q.N = p.N; q.K = p.K;
  q.lda = p.lda; q.ldb = p.ldb; q.ldc = p.ldr;
  return group_fits_dl(one, true, p.b_kcontig != 0, Epilogue::StoreF32, CfgDl::BK);
}

hipError_t launch_proj_group(ProjGroup& g, float* slabs, size_t slab_bytes, hipStream_t stream, bool fuse_adam) {
  using Cfg = CfgDl;
  if (g.count <= 0) return hipSuccess;
  if (g.count > kMaxGroup) return hipErrorInvalidValue;
  int total = 0, min_kt = 1 << 30;
  for (int i = 0; i < g.count; ++i) {
    ProjProblem& p = g.p[i];
    if (!proj_problem_fits(p)) return hipErrorInvalidValue;
    if (fuse_adam && (!p.Mo || !p.Vo || !p.Nout || p.cols_valid < 1 || p.cols_valid > p.N || p.ldm < p.cols_valid ||
                      p.ldn < (p.n_transposed ? p.M : p.cols_valid) || (uint64_t)p.M * (uint64_t)p.ldm * 4 > 0xFFFFFFFFull))
      return hipErrorInvalidValue;
    p.tile_begin = total;
    p.tiles_m = (p.M + Cfg::BM - 1) / Cfg::BM;
    p.tiles_n = (p.N + Cfg::BN - 1) / Cfg::BN;
    total += p.tiles_m * p.tiles_n;
    min_kt = p.K / Cfg::BK < min_kt ? p.K / Cfg::BK : min_kt;
  }
  if (total == 0) return hipSuccess;
  g.total_tiles = total;
  const int cus = dl_grid_size(1 << 20);  // one workgroup per CU, a multiple of 8
  // Whole rounds of the grid run whole tiles.  What is left over after at least one whole round would occupy `rem`
  // CUs for a whole tile time while the others idle: cut every leftover tile into K pieces of at least 4 K steps, as
  // many as there are CUs to take them (at most 16, and only what the slab area holds).  A launch of less than one
  // round is left alone: measured on the 130M / 350M stacks, cutting ALL its tiles costs more in slab traffic and
  // in the second launch than the fuller chip gains (0.47 against 0.33 ms and 1.20 against 0.97 ms per step).
  int regular = total / cus * cus;
  const int rem = total - regular;
  int pieces = 1;
  if (rem > 0 && regular > 0) {
    pieces = cus / rem;
    if (pieces > min_kt / 4) pieces = min_kt / 4;
    if (pieces > 16) pieces = 16;
    const size_t slab_tile = (size_t)Cfg::BM * Cfg::BN * sizeof(float);
    if (!slabs) slab_bytes = 0;
    if ((size_t)rem * (size_t)pieces * slab_tile > slab_bytes) pieces = (int)(slab_bytes / slab_tile / (size_t)rem);
  }
  if (pieces < 2) {  // not worth it, or no room: the leftover tiles run as a last, partly filled round
    pieces = 1;
    regular = total;
  }
  g.regular_tiles = regular;
  g.pieces = pieces;
  g.slabs = slabs;
  const int split_items = (total - regular) * pieces;
  const int grid = dl_grid_size(regular > split_items ? regular : split_items);

  using AOp = DlOperand<true, Cfg::BM, Cfg::BK, Cfg::NW>;
  using BOp = DlOperand<true, Cfg::BN, Cfg::BK, Cfg::NW>;
  constexpr size_t smem = (size_t)Cfg::STAGES * (AOp::TILE_BYTES + BOp::TILE_BYTES) +
                          (size_t)Cfg::NW * 8 * (Cfg::WN + 8) * sizeof(float);  // tile ring + epilogue strips
  static_assert(smem <= 160 * 1024, "tile ring and strips do not fit the 160 KB LDS");
  auto kern = fuse_adam ? proj_dl_kernel<Cfg, true> : proj_dl_kernel<Cfg, false>;
  static bool attr_set[2] = {false, false};
  if (!attr_set[fuse_adam]) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set[fuse_adam] = true;
  }
  hipLaunchKernelGGL(kern, dim3(grid), dim3(Cfg::NT), smem, stream, g);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (total > regular) {
    if (fuse_adam) hipLaunchKernelGGL((proj_reduce_kernel<Cfg, true>), dim3(64, total - regular), dim3(256), 0, stream, g);
    else hipLaunchKernelGGL((proj_reduce_kernel<Cfg, false>), dim3(64, total - regular), dim3(256), 0, stream, g);
    e = hipGetLastError();
  }
  return e;
}

}  // namespace galore
