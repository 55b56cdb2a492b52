// Small kernels of the two-sided rule (Definition 3.6: G~ = P rho(P^T G Q) Q^T): storage-dtype
// copies of fp32 intermediates that feed the next matrix product, and the unit-length rows that
// turn P^T G = S_r V_r^T into V_r^T when the partner projector is formed (Sec. 3.3, SVD equation).
#include "common.hpp"

namespace galore {
namespace {

template <class T> __device__ __forceinline__ T from_f32(float x) { return (T)x; }

// dst (rows x cols, leading dimension ldd, dtype T) <- src (rows x cols dense fp32), round to nearest even
template <class T>
__global__ __launch_bounds__(256) void cast_rows_kernel(const float* __restrict__ src, T* __restrict__ dst, int rows, int cols, int ldd) {
  const int64_t total = (int64_t)rows * cols;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < total; e += stride) {
    const int i = (int)(e / cols), j = (int)(e - (int64_t)i * cols);
    dst[(size_t)i * ldd + j] = from_f32<T>(src[e]);
  }
}

// dst row i <- src row i / |src row i|  (zero row stays zero); one workgroup per row
template <class T>
__global__ __launch_bounds__(256) void normalize_rows_kernel(const float* __restrict__ src, T* __restrict__ dst, int cols, int ldd) {
  __shared__ float red[4];
  const float* row = src + (size_t)blockIdx.x * cols;
  float s = 0.f;
  for (int j = threadIdx.x; j < cols; j += 256) s += row[j] * row[j];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  const float nrm2 = (red[0] + red[1]) + (red[2] + red[3]);   // fixed order: the same bits in every thread
  const float inv = nrm2 > 0.f ? 1.0f / sqrtf(nrm2) : 0.f;
  T* out = dst + (size_t)blockIdx.x * ldd;
  for (int j = threadIdx.x; j < cols; j += 256) out[j] = from_f32<T>(row[j] * inv);
}

}  // namespace

hipError_t launch_cast_rows(const float* src, void* dst, int rows, int cols, int ldd, DType dt, hipStream_t stream) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  const int64_t total = (int64_t)rows * cols;
  const unsigned blocks = (unsigned)((total + 256 * 8 - 1) / (256 * 8) > 4096 ? 4096 : (total + 256 * 8 - 1) / (256 * 8));
  if (dt == DType::BF16) hipLaunchKernelGGL(cast_rows_kernel<__bf16>, dim3(blocks), dim3(256), 0, stream, src, static_cast<__bf16*>(dst), rows, cols, ldd);
  else hipLaunchKernelGGL(cast_rows_kernel<float>, dim3(blocks), dim3(256), 0, stream, src, static_cast<float*>(dst), rows, cols, ldd);
  return hipGetLastError();
}

hipError_t launch_normalize_rows(const float* src, void* dst, int rows, int cols, int ldd, DType dt, hipStream_t stream) {
  if (rows <= 0 || cols <= 0) return hipSuccess;
  if (dt == DType::BF16) hipLaunchKernelGGL(normalize_rows_kernel<__bf16>, dim3(rows), dim3(256), 0, stream, src, static_cast<__bf16*>(dst), cols, ldd);
  else hipLaunchKernelGGL(normalize_rows_kernel<float>, dim3(rows), dim3(256), 0, stream, src, static_cast<float*>(dst), cols, ldd);
  return hipGetLastError();
}

}  // namespace galore
