// Layout / epilogue dispatch shared by the per-dtype GEMM translation units.
#pragma once
#include <type_traits>

#include "gemm_mfma.hpp"
#include "gemm_mfma_dl.hpp"

// Build-time choice of the large-tile configuration (tuning knob; 0 disables the kernel).
#ifndef GALORE_DL_VARIANT
#define GALORE_DL_VARIANT 2
#endif

namespace galore {

using CfgDefault = TileCfg<128, 128, 32, 2, 2>;
// Measured on the 7B shapes (projection / back-projection TFLOP/s of a single 4096x11008 tensor):
//   1: 256x256x64, 4 waves (128x128 each)  746 / 650     2: 256x256x64, 8 waves (128x64 each)  876 / 894
//   3: 256x128x32, 4 waves, 3 stages       828 / 699     4: 128x128x64, 4 waves                878 / 711
#if GALORE_DL_VARIANT == 1
using CfgDl = DlCfg<256, 256, 64, 2, 2, 2>;
#elif GALORE_DL_VARIANT == 2
using CfgDl = DlCfg<256, 256, 64, 2, 4, 2>;
#elif GALORE_DL_VARIANT == 3
using CfgDl = DlCfg<256, 128, 32, 2, 2, 3>;
#elif GALORE_DL_VARIANT == 4
using CfgDl = DlCfg<128, 128, 64, 2, 2, 2>;
#elif GALORE_DL_VARIANT == 5
using CfgDl = DlCfg<256, 128, 64, 2, 2, 3>;
#elif GALORE_DL_VARIANT == 6
using CfgDl = DlCfg<256, 128, 64, 4, 2, 3>;
#elif GALORE_DL_VARIANT == 7
using CfgDl = DlCfg<128, 256, 64, 2, 4, 3>;
#elif GALORE_DL_VARIANT == 8
using CfgDl = DlCfg<128, 256, 64, 1, 4, 3>;
#endif

template <class T, bool AK, bool BKC, Epilogue EPI>
inline hipError_t launch_gemm_layout(GemmGroup& g, hipStream_t stream) {
#if GALORE_DL_VARIANT > 0
  if constexpr (std::is_same<T, __bf16>::value) {
    if (group_fits_dl(g, AK, BKC, EPI, CfgDl::BK)) {
      plan_tiles<CfgDl>(g);
      if (g.total_tiles == 0) return hipSuccess;
      return launch_gemm_dl_instance<AK, BKC, EPI, CfgDl>(g, stream);
    }
  }
#endif
  plan_tiles<CfgDefault>(g);
  if (g.total_tiles == 0) return hipSuccess;
  if (group_is_aligned<T>(g, AK, BKC))
    return launch_gemm_instance<T, AK, BKC, true, EPI, CfgDefault>(g, stream);
  return launch_gemm_instance<T, AK, BKC, false, EPI, CfgDefault>(g, stream);
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
