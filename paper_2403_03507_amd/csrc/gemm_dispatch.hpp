// Layout / epilogue dispatch shared by the per-dtype GEMM translation units.
#pragma once
#include <type_traits>

#include "gemm_mfma.hpp"
#include "gemm_mfma_dl.hpp"

namespace galore {

using CfgDefault = TileCfg<128, 128, 32, 2, 2>;
// Large tile of the direct-to-LDS kernel.  Measured alternatives on the 7B shapes were slower:
// 4 waves of 128x128 (one wave per SIMD cannot overlap its LDS reads with MFMAs), 256x128 and
// 128x128 tiles (more LDS and L2 traffic per flop).
using CfgDl = DlCfg<256, 256, 64, 2, 4, 2>;  // 8 waves of 128 x 64, two 64 KB stages

// A group is split by what each problem allows: problems that meet the large-tile kernel's
// alignment rules go there together, the rest to the general kernel (aligned and element-aligned
// problems apart), so one odd-shaped tensor does not drag its whole group onto the slow path.
template <class T, bool AK, bool BKC, Epilogue EPI>
inline hipError_t launch_gemm_layout(GemmGroup& g, hipStream_t stream) {
  GemmGroup dl{}, dlw{}, al{}, un{};  // dlw: weight updates whose W has an odd row length or alignment
  for (int i = 0; i < g.count; ++i) {
    GemmGroup one{};
    one.count = 1;
    one.p[0] = g.p[i];
    bool to_dl = false, to_dlw = false;
    if constexpr (std::is_same<T, __bf16>::value) {
      to_dl = group_fits_dl(one, AK, BKC, EPI, CfgDl::BK);
      if constexpr (EPI == Epilogue::ApplyW && BKC) to_dlw = !to_dl && group_fits_dl(one, AK, BKC, EPI, CfgDl::BK, true);
    }
    GemmGroup& dst = to_dl ? dl : to_dlw ? dlw : (group_is_aligned<T>(one, AK, BKC) ? al : un);
    dst.p[dst.count++] = g.p[i];
  }
  if constexpr (std::is_same<T, __bf16>::value) {
    if (dl.count > 0) {
      plan_tiles<CfgDl>(dl);
      if (dl.total_tiles > 0) {
        hipError_t e = launch_gemm_dl_instance<AK, BKC, EPI, CfgDl>(dl, stream);
        if (e != hipSuccess) return e;
      }
    }
    if constexpr (EPI == Epilogue::ApplyW && BKC) {
      if (dlw.count > 0) {
        plan_tiles<CfgDl>(dlw);
        if (dlw.total_tiles > 0) {
          hipError_t e = launch_gemm_dl_instance<AK, BKC, EPI, CfgDl, true>(dlw, stream);
          if (e != hipSuccess) return e;
        }
      }
    }
  }
  if (al.count > 0) {
    plan_tiles<CfgDefault>(al);
    if (al.total_tiles > 0) {
      hipError_t e = launch_gemm_instance<T, AK, BKC, true, EPI, CfgDefault>(al, stream);
      if (e != hipSuccess) return e;
    }
  }
  if (un.count > 0) {
    plan_tiles<CfgDefault>(un);
    if (un.total_tiles > 0) return launch_gemm_instance<T, AK, BKC, false, EPI, CfgDefault>(un, stream);
  }
  return hipSuccess;
}

// The layout / epilogue combinations the library uses:
//   (K,X) Store   : R = P^T G with A = the transposed projector copy ; fp32 also C Q and Q S of the refresh
//   (K,K) Store   : R = G Q   with B = the transposed projector copy
//   (K,K) ApplyW  : W -= P N^T^T (N stored transposed) and W -= N Q^T
//   (K,X) ApplyW  : kept for callers that hold N untransposed
//   (K,K) StoreSym: C = G G^T
//   (X,X) StoreSym: C = G^T G
template <class T>
inline hipError_t launch_gemm_typed(GemmGroup& g, bool ak, bool bk, Epilogue epi, hipStream_t stream) {
  if (epi == Epilogue::StoreF32) {
    if (ak && !bk) return launch_gemm_layout<T, true, false, Epilogue::StoreF32>(g, stream);
    if (ak && bk) return launch_gemm_layout<T, true, true, Epilogue::StoreF32>(g, stream);
  } else if (epi == Epilogue::ApplyW) {
    if (ak && !bk) return launch_gemm_layout<T, true, false, Epilogue::ApplyW>(g, stream);
    if (ak && bk) return launch_gemm_layout<T, true, true, Epilogue::ApplyW>(g, stream);
  } else if (epi == Epilogue::StoreSymF32) {
    if (ak && bk) return launch_gemm_layout<T, true, true, Epilogue::StoreSymF32>(g, stream);
    if (!ak && !bk) return launch_gemm_layout<T, false, false, Epilogue::StoreSymF32>(g, stream);
  }
  return hipErrorInvalidValue;
}

hipError_t launch_gemm_bf16(GemmGroup& g, bool ak, bool bk, Epilogue epi, hipStream_t stream);
hipError_t launch_gemm_f32(GemmGroup& g, bool ak, bool bk, Epilogue epi, hipStream_t stream);

}  // namespace galore
