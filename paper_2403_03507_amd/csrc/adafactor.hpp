// Adafactor with first-order statistics on one projected gradient (kernels in adafactor.hip).
#pragma once
#include "common.hpp"

namespace galore {

// R rows x cols fp32 (row stride ldr); M rows x cols fp32 dense; rowv (rows), colv (cols) fp32; N rows x cols in n_dtype,
// dense.  `scratch` holds adafactor_scratch_floats(rows, cols) floats of partial sums (fixed reduction order, no atomics).
struct AdafactorProblem {
  const float* R;
  float* M;
  float* rowv;
  float* colv;
  void* N;
  float* scratch;
  int rows, cols, ldr;
  float beta1, beta2t;   // momentum; decay rate 1 - k^decay_pow of this step
  float eps1, clip_d;
};
size_t adafactor_scratch_floats(int rows, int cols);
hipError_t launch_adafactor(const AdafactorProblem& p, DType n_dtype, hipStream_t stream);

}  // namespace galore
