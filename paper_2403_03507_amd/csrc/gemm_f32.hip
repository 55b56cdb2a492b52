// fp32-operand instances of the grouped MFMA GEMM, and the dtype dispatch.
#include "gemm_dispatch.hpp"

namespace galore {
hipError_t launch_gemm_f32(GemmGroup& g, bool ak, bool bk, Epilogue epi, hipStream_t stream) {
  return launch_gemm_typed<float>(g, ak, bk, epi, stream);
}

hipError_t launch_gemm_group(GemmGroup& g, DType dt, bool a_kcontig, bool b_kcontig, Epilogue epi,
                             hipStream_t stream) {
  if (g.count <= 0) return hipSuccess;
  if (g.count > kMaxGroup) return hipErrorInvalidValue;
  return dt == DType::BF16 ? launch_gemm_bf16(g, a_kcontig, b_kcontig, epi, stream)
                           : launch_gemm_f32(g, a_kcontig, b_kcontig, epi, stream);
}
}  // namespace galore
