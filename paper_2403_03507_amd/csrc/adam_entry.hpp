// The update block of Algorithm 2 for one entry, shared by the Adam kernels and by the projection GEMM's
// fused epilogue so that both paths evaluate the very same fp32 expression (bit-identical M, V, N).
#pragma once
#include <hip/hip_runtime.h>

namespace galore {

__device__ __forceinline__ float adam_entry(float g, float& m, float& v, float beta1, float beta2,
                                            float eps, float inv_c1, float inv_c2) {
  // Every operation is written out and rounded once (no contraction left to the compiler), so that the expression
  // means the same in every kernel it is inlined into.
#pragma clang fp contract(off)
  const float gm = (1.f - beta1) * g;
  m = __builtin_fmaf(beta1, m, gm);
  float gv = (1.f - beta2) * g;
  gv = gv * g;
  v = __builtin_fmaf(beta2, v, gv);
  const float mh = m * inv_c1;
  const float vh = v * inv_c2;
  const float den = sqrtf(vh) + eps;
  return mh / den;
}

}  // namespace galore
