// bf16-operand instances of the grouped MFMA GEMM.
#include "gemm_dispatch.hpp"

namespace galore {
hipError_t launch_gemm_bf16(GemmGroup& g, bool ak, bool bk, Epilogue epi, hipStream_t stream) {
  return launch_gemm_typed<__bf16>(g, ak, bk, epi, stream);
}
}  // namespace galore
