// Adafactor with first-order statistics as the optimizer of the projected gradient (the optimizer Sec. 4.3 and Sec. 5 of
// the paper name next to Adam; the paper prints no equations, so this is the published Adafactor update for a matrix,
// with the learning rate left to the caller as in Algorithm 2):
//   rowv_i <- b2 rowv_i + (1 - b2) sum_j (R_ij^2 + eps1),  colv_j <- b2 colv_j + (1 - b2) sum_i (R_ij^2 + eps1),  b2 = 1 - k^-0.8
//   Vhat_ij = rowv_i colv_j / sum_i rowv_i,  U = R / sqrt(Vhat),  Uhat = U / max(1, RMS(U) / d)
//   M <- b1 M + (1 - b1) Uhat,  N = M
// Six launches, three passes over R: partial sums of the squares by rows and by columns; the statistics; their total;
// partial sums of U^2; the clipping factor; the update.  Every sum has a fixed order (partials per workgroup, added in index order by one
// workgroup): no atomics, bit-identical from run to run.  Bound by memory traffic: 3 reads of R, one read and write of M,
// one write of N.
#include "adafactor.hpp"

namespace galore {
namespace {

constexpr int kAfCols = 256;  // columns per workgroup (one per thread)
constexpr int kAfRows = 32;   // rows per workgroup

__device__ __forceinline__ float af_wave_sum(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// scratch layout (floats): rowpart [cb][rows] | colpart [rb][cols] | blockpart [rb * cb] | scal [4]: total of rowv, clip factor
struct AfScratch {
  float* rowpart;
  float* colpart;
  float* blockpart;
  float* scal;
  int cb, rb;
};
__host__ __device__ inline AfScratch af_scratch(float* base, int rows, int cols) {
  AfScratch s;
  s.cb = (cols + kAfCols - 1) / kAfCols;
  s.rb = (rows + kAfRows - 1) / kAfRows;
  s.rowpart = base;
  s.colpart = s.rowpart + (size_t)s.cb * rows;
  s.blockpart = s.colpart + (size_t)s.rb * cols;
  s.scal = s.blockpart + (size_t)s.rb * s.cb;
  return s;
}

// pass 1: sums of R^2 + eps1 over this workgroup's 256 columns for each of its 32 rows, and over its 32 rows for each column.
// A thread owns a column: its 32 loads are independent (clamped addresses, masked afterwards) and all in flight together.
// Column sums stay in the thread; for the row sums the squares cross an LDS tile and 8 threads per row add 32 columns
// each, then each other (fixed order).
__global__ __launch_bounds__(kAfCols) void adafactor_sums_kernel(const AdafactorProblem p) {
  __shared__ float tile[kAfRows][kAfCols + 1];
  const AfScratch s = af_scratch(p.scratch, p.rows, p.cols);
  const int tid = threadIdx.x;
  const int c = blockIdx.x * kAfCols + tid;
  const int row0 = blockIdx.y * kAfRows;
  const bool cok = c < p.cols;
  const int cc = cok ? c : p.cols - 1;
  float x[kAfRows];
#pragma unroll
  for (int rl = 0; rl < kAfRows; ++rl) {
    const int row = row0 + rl < p.rows ? row0 + rl : p.rows - 1;
    x[rl] = p.R[(size_t)row * p.ldr + cc];
  }
  float colacc = 0.f;
#pragma unroll
  for (int rl = 0; rl < kAfRows; ++rl) {
    const float q = (cok && row0 + rl < p.rows) ? x[rl] * x[rl] + p.eps1 : 0.f;
    colacc += q;
    tile[rl][tid] = q;
  }
  if (cok) s.colpart[(size_t)blockIdx.y * p.cols + c] = colacc;
  __syncthreads();
  const int rl = tid >> 3, part = tid & 7;
  float a = 0.f;
#pragma unroll
  for (int j = 0; j < kAfCols / 8; ++j) a += tile[rl][part + 8 * j];
  a += __shfl_xor(a, 1, 64);
  a += __shfl_xor(a, 2, 64);
  a += __shfl_xor(a, 4, 64);
  if (part == 0 && row0 + rl < p.rows) s.rowpart[(size_t)blockIdx.x * p.rows + row0 + rl] = a;
}

// sum of `count` values f(i), i = 0 .. count - 1, over one workgroup of 1024 threads, in a fixed order; every thread gets it
template <class F> __device__ __forceinline__ float af_block_total(int count, F f, float* red) {
  float a = 0.f;
  for (int i = threadIdx.x; i < count; i += 1024) a += f(i);
  a = af_wave_sum(a);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = a;
  __syncthreads();
  float t = 0.f;
  for (int w = 0; w < 16; ++w) t += red[w];
  return t;
}

// the statistics: partial sums added in index order (loads in batches of eight), then the decayed averages; one thread per
// row statistic (idx < rows) or column statistic
__global__ __launch_bounds__(256) void adafactor_stats_kernel(const AdafactorProblem p) {
  const AfScratch s = af_scratch(p.scratch, p.rows, p.cols);
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= p.rows + p.cols) return;
  const bool is_row = idx < p.rows;
  const int i = is_row ? idx : idx - p.rows;
  const float* part = is_row ? s.rowpart + i : s.colpart + i;
  const size_t stride = is_row ? p.rows : p.cols;
  const int count = is_row ? s.cb : s.rb;
  float a = 0.f;
#pragma unroll 8
  for (int b = 0; b < count; ++b) a += part[(size_t)b * stride];
  float* stat = is_row ? p.rowv + i : p.colv + i;
  *stat = p.beta2t * *stat + (1.f - p.beta2t) * a;
}

// the total of the row statistics
__global__ __launch_bounds__(1024) void adafactor_total_kernel(const AdafactorProblem p) {
  __shared__ float red[16];
  const AfScratch s = af_scratch(p.scratch, p.rows, p.cols);
  const float total = af_block_total(p.rows, [&](int i) { return p.rowv[i]; }, red);
  if (threadIdx.x == 0) s.scal[0] = total;
}

// U_ij = R_ij / sqrt(rowv_i colv_j / total); the association keeps the quotient colv_j / total (of order 1 / rows) away
// from the underflow that rowv_i colv_j could reach for tiny gradients
__device__ __forceinline__ float af_u(float x, float rv, float cv_over_total) { return x / sqrtf(rv * cv_over_total); }

// pass 2: sum of U^2 over this workgroup's tile
__global__ __launch_bounds__(kAfCols) void adafactor_rms_kernel(const AdafactorProblem p) {
  __shared__ float sm[4];
  const AfScratch s = af_scratch(p.scratch, p.rows, p.cols);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = blockIdx.x * kAfCols + tid;
  const int row0 = blockIdx.y * kAfRows;
  const float total = s.scal[0];
  float acc = 0.f;
  {
    const bool cok = c < p.cols;
    const int cc = cok ? c : p.cols - 1;
    const float cvt = p.colv[cc] / total;
    float x[kAfRows], rv[kAfRows];
#pragma unroll
    for (int rl = 0; rl < kAfRows; ++rl) {        // independent loads from clamped addresses, masked below
      const int row = row0 + rl < p.rows ? row0 + rl : p.rows - 1;
      x[rl] = p.R[(size_t)row * p.ldr + cc];
      rv[rl] = p.rowv[row];
    }
#pragma unroll
    for (int rl = 0; rl < kAfRows; ++rl) {
      const float u = af_u(x[rl], rv[rl], cvt);
      acc += (cok && row0 + rl < p.rows) ? u * u : 0.f;
    }
  }
  acc = af_wave_sum(acc);
  if (lane == 0) sm[wave] = acc;
  __syncthreads();
  if (tid == 0) s.blockpart[blockIdx.y * s.cb + blockIdx.x] = ((sm[0] + sm[1]) + sm[2]) + sm[3];
}

// the clipping factor 1 / max(1, RMS(U) / d)
__global__ __launch_bounds__(1024) void adafactor_clip_kernel(const AdafactorProblem p) {
  __shared__ float red[16];
  const AfScratch s = af_scratch(p.scratch, p.rows, p.cols);
  const float sumsq = af_block_total(s.rb * s.cb, [&](int i) { return s.blockpart[i]; }, red);
  if (threadIdx.x == 0) {
    const float rms = sqrtf(sumsq / ((float)p.rows * (float)p.cols));
    const float over = rms / p.clip_d;
    s.scal[1] = 1.f / (over > 1.f ? over : 1.f);
  }
}

// pass 3: Uhat, the momentum, N
template <class TN>
__global__ __launch_bounds__(kAfCols) void adafactor_update_kernel(const AdafactorProblem p) {
  const AfScratch s = af_scratch(p.scratch, p.rows, p.cols);
  const int c = blockIdx.x * kAfCols + threadIdx.x;
  const int row0 = blockIdx.y * kAfRows;
  if (c >= p.cols) return;
  const float total = s.scal[0], factor = s.scal[1];
  const float cvt = p.colv[c] / total;
  TN* N = static_cast<TN*>(p.N);
  float x[kAfRows], rv[kAfRows], mo[kAfRows];
#pragma unroll
  for (int rl = 0; rl < kAfRows; ++rl) {          // independent loads from clamped addresses
    const int row = row0 + rl < p.rows ? row0 + rl : p.rows - 1;
    x[rl] = p.R[(size_t)row * p.ldr + c];
    rv[rl] = p.rowv[row];
    mo[rl] = p.M[(size_t)row * p.cols + c];
  }
#pragma unroll
  for (int rl = 0; rl < kAfRows; ++rl) {
    const int row = row0 + rl;
    if (row < p.rows) {
      const float uhat = af_u(x[rl], rv[rl], cvt) * factor;
      const size_t e = (size_t)row * p.cols + c;
      const float m = p.beta1 * mo[rl] + (1.f - p.beta1) * uhat;
      p.M[e] = m;
      N[e] = (TN)m;
    }
  }
}

}  // namespace

size_t adafactor_scratch_floats(int rows, int cols) {
  const AfScratch s = af_scratch(nullptr, rows, cols);
  return (size_t)(s.scal - s.rowpart) + 4;
}

hipError_t launch_adafactor(const AdafactorProblem& p, DType n_dtype, hipStream_t stream) {
  if (p.rows < 1 || p.cols < 1 || p.ldr < p.cols || !p.R || !p.M || !p.rowv || !p.colv || !p.N || !p.scratch) return hipErrorInvalidValue;
  const AfScratch s = af_scratch(p.scratch, p.rows, p.cols);
  if (s.rb > 65535) return hipErrorInvalidValue;   // grid.y
  const dim3 grid(s.cb, s.rb);
  hipLaunchKernelGGL(adafactor_sums_kernel, grid, dim3(kAfCols), 0, stream, p);
  hipLaunchKernelGGL(adafactor_stats_kernel, dim3((p.rows + p.cols + 255) / 256), dim3(256), 0, stream, p);
  hipLaunchKernelGGL(adafactor_total_kernel, dim3(1), dim3(1024), 0, stream, p);
  hipLaunchKernelGGL(adafactor_rms_kernel, grid, dim3(kAfCols), 0, stream, p);
  hipLaunchKernelGGL(adafactor_clip_kernel, dim3(1), dim3(1024), 0, stream, p);
  if (n_dtype == DType::BF16) hipLaunchKernelGGL(adafactor_update_kernel<__bf16>, grid, dim3(kAfCols), 0, stream, p);
  else hipLaunchKernelGGL(adafactor_update_kernel<float>, grid, dim3(kAfCols), 0, stream, p);
  return hipGetLastError();
}

}  // namespace galore
