// Fused low-rank Adam (Algorithm 2, update block): one pass over R, M, V that updates the
// fp32 moments in place, applies the bias correction and writes the normalised update N
// in the dtype the back-projection GEMM consumes.  Pure streaming: 16-byte vectors; R, M and V
// are read and M, V written with non-temporal accesses (each is touched once per step and the
// stack's moments are far larger than the caches), N is written normally because the
// back-projection GEMM reads it next.  Measured at 7B: 0.210 -> 0.204 ms per layer set.
#include "adam_entry.hpp"
#include "common.hpp"

namespace galore {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ void store_n(float* N, int64_t i, f32x4 n) { *reinterpret_cast<f32x4*>(N + i) = n; }
__device__ __forceinline__ void store_n(__bf16* N, int64_t i, f32x4 n) {
  bf16x4 o;
  o[0] = (__bf16)n[0]; o[1] = (__bf16)n[1]; o[2] = (__bf16)n[2]; o[3] = (__bf16)n[3];
  *reinterpret_cast<bf16x4*>(N + i) = o;
}

template <class TN>
__global__ __launch_bounds__(256) void adam_group_kernel(const AdamGroup grp) {
  const AdamProblem& pr = grp.p[blockIdx.y];
  const float beta1 = grp.beta1, beta2 = grp.beta2, eps = grp.eps;
  const float ic1 = pr.inv_c1, ic2 = pr.inv_c2;
  const float* __restrict__ R = pr.R;
  float* __restrict__ M = pr.M;
  float* __restrict__ V = pr.V;
  TN* __restrict__ N = static_cast<TN*>(pr.N);
  const int64_t count = pr.count;
  const int64_t nvec = count >> 2;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nvec; q += stride) {
    const int64_t i = q << 2;
    const f32x4 g = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(R + i));
    f32x4 m = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(M + i));
    f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(V + i));
    f32x4 n;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float me = m[e], ve = v[e];
      n[e] = adam_entry(g[e], me, ve, beta1, beta2, eps, ic1, ic2);
      m[e] = me; v[e] = ve;
    }
    __builtin_nontemporal_store(m, reinterpret_cast<f32x4*>(M + i));
    __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(V + i));
    store_n(N, i, n);
  }
  // ragged tail (count not a multiple of 4)
  if (blockIdx.x == 0) {
    const int64_t i = (nvec << 2) + threadIdx.x;
    if (threadIdx.x < 4 && i < count) {
      float me = M[i], ve = V[i];
      const float n = adam_entry(R[i], me, ve, beta1, beta2, eps, ic1, ic2);
      M[i] = me; V[i] = ve;
      N[i] = (TN)n;
    }
  }
}

// Same update, but N is written transposed (cols x rows): the back-projection GEMM then finds
// its contraction index contiguous in memory.  One block per 64 x 64 tile: R, M, V are read and
// M, V written row-wise with 16-byte vectors, N goes through a padded LDS tile and leaves
// column-wise, again as 16-byte vectors.  Ragged or unaligned tiles take an element-wise path.
// 16-byte access to four floats that are only 4-byte aligned (rows of odd length): the compiler picks
// the widest access the target allows at that alignment
__device__ __forceinline__ f32x4 load4(const float* p) { f32x4 v; __builtin_memcpy(&v, p, sizeof v); return v; }
__device__ __forceinline__ void store4(float* p, f32x4 v) { __builtin_memcpy(p, &v, sizeof v); }

// RAGGED: some tile of the launch is not a full, aligned 64 x 64 tile.  The variant without that path needs 48 registers
// per lane instead of 55 (bf16 N), which is what lets a wavefront of it share a SIMD with the two wavefronts of the
// projection GEMM (2 x 232 of the 512 registers per lane): the Adam pass of one call then runs on the CUs that the
// projection of the next call occupies.
template <class TN, bool RAGGED>
__global__ __launch_bounds__(256) void adam_transpose_group_kernel(const AdamGroup grp) {
  constexpr int TS = 64;
  constexpr int VEC = 16 / sizeof(TN);          // N elements per 16 bytes
  __shared__ __align__(16) TN tile[TS][TS + VEC];  // tile[j][i] = N[i][j]
  const AdamProblem& pr = grp.p[blockIdx.y];
  const int rows = pr.rows, cols = pr.cols, ldr = pr.ldr;
  const int tiles_c = (cols + TS - 1) / TS;
  const int ntiles = tiles_c * ((rows + TS - 1) / TS);
  const float beta1 = grp.beta1, beta2 = grp.beta2, eps = grp.eps;
  const float ic1 = pr.inv_c1, ic2 = pr.inv_c2;
  const float* __restrict__ R = pr.R;
  float* __restrict__ M = pr.M;
  float* __restrict__ V = pr.V;
  TN* __restrict__ N = static_cast<TN*>(pr.N);
  const bool cols4 = cols % 4 == 0 && ldr % 4 == 0 && ((reinterpret_cast<uintptr_t>(R) | reinterpret_cast<uintptr_t>(M) | reinterpret_cast<uintptr_t>(V)) & 15) == 0;
  const bool aligned = rows % VEC == 0;  // rows of N^T stay 16-byte aligned; R, M, V rows may be of any length
  for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const int i0 = (t / tiles_c) * TS, j0 = (t % tiles_c) * TS;
    const bool full = aligned && i0 + TS <= rows && j0 + TS <= cols;
    if (full) {
      // tile origin as a (wave-uniform) pointer, in-tile offsets in 32 bits: fewer address registers per lane
      const float* __restrict__ Rt = R + ((size_t)i0 * ldr + j0);
      float* __restrict__ Mt = M + ((size_t)i0 * cols + j0);
      float* __restrict__ Vt = V + ((size_t)i0 * cols + j0);
#pragma unroll 1
      for (int ps = 0; ps < 4; ++ps) {
        const int i = ps * 16 + (threadIdx.x >> 4), j = (threadIdx.x & 15) * 4;
        const int idx = i * cols + j;
        const int ridx = i * ldr + j;
        f32x4 g, m, v;
        if (cols4) {
          g = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Rt + ridx));
          m = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Mt + idx));
          v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(Vt + idx));
        } else {
          g = load4(Rt + ridx); m = load4(Mt + idx); v = load4(Vt + idx);
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          float me = m[e], ve = v[e];
          tile[j + e][i] = (TN)adam_entry(g[e], me, ve, beta1, beta2, eps, ic1, ic2);
          m[e] = me; v[e] = ve;
        }
        if (cols4) {
          __builtin_nontemporal_store(m, reinterpret_cast<f32x4*>(Mt + idx));
          __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(Vt + idx));
        } else {
          store4(Mt + idx, m);
          store4(Vt + idx, v);
        }
      }
      __syncthreads();
      constexpr int LPR = TS / VEC;        // lanes per output row
      constexpr int RPP = 256 / LPR;       // output rows per pass
#pragma unroll
      for (int ps = 0; ps < TS / RPP; ++ps) {
        const int j = ps * RPP + threadIdx.x / LPR, i = (threadIdx.x % LPR) * VEC;
        *reinterpret_cast<uint4*>(N + (size_t)(j0 + j) * rows + i0 + i) = *reinterpret_cast<const uint4*>(&tile[j][i]);
      }
      __syncthreads();
    } else if constexpr (RAGGED) {
      for (int e = threadIdx.x; e < TS * TS; e += 256) {
        const int i = e / TS, j = e % TS;
        if (i0 + i < rows && j0 + j < cols) {
          const size_t idx = (size_t)(i0 + i) * cols + j0 + j;
          float me = M[idx], ve = V[idx];
          const float n = adam_entry(R[(size_t)(i0 + i) * ldr + j0 + j], me, ve, beta1, beta2, eps, ic1, ic2);
          M[idx] = me; V[idx] = ve;
          N[(size_t)(j0 + j) * rows + i0 + i] = (TN)n;
        }
      }
    }
  }
}

hipError_t launch_adam_group(const AdamGroup& g, DType n_dtype, hipStream_t stream) {
  if (g.count <= 0) return hipSuccess;
  if (g.count > kMaxGroup) return hipErrorInvalidValue;
  for (int i = 0; i < g.count; ++i)  // padded rows of R are a feature of the transposing kernel only
    if (g.p[i].ldr < g.p[i].cols || (!g.p[0].transpose_n && g.p[i].ldr != g.p[i].cols)) return hipErrorInvalidValue;
  if (g.p[0].transpose_n) {
    int64_t maxtiles = 0;
    for (int i = 0; i < g.count; ++i) {
      const int64_t t = (int64_t)((g.p[i].rows + 63) / 64) * ((g.p[i].cols + 63) / 64);
      maxtiles = t > maxtiles ? t : maxtiles;
    }
    if (maxtiles == 0) return hipSuccess;
    const dim3 grid((unsigned)(maxtiles > 4096 ? 4096 : maxtiles), (unsigned)g.count);
    // every tile of every problem full and 16-byte aligned on the N side: the lean variant
    bool ragged = false;
    for (int i = 0; i < g.count; ++i) ragged = ragged || g.p[i].rows % 64 != 0 || g.p[i].cols % 64 != 0;
    if (n_dtype == DType::BF16) {
      if (ragged) hipLaunchKernelGGL((adam_transpose_group_kernel<__bf16, true>), grid, dim3(256), 0, stream, g);
      else hipLaunchKernelGGL((adam_transpose_group_kernel<__bf16, false>), grid, dim3(256), 0, stream, g);
    } else {
      if (ragged) hipLaunchKernelGGL((adam_transpose_group_kernel<float, true>), grid, dim3(256), 0, stream, g);
      else hipLaunchKernelGGL((adam_transpose_group_kernel<float, false>), grid, dim3(256), 0, stream, g);
    }
    return hipGetLastError();
  }
  int64_t maxcount = 0;
  for (int i = 0; i < g.count; ++i) maxcount = g.p[i].count > maxcount ? g.p[i].count : maxcount;
  if (maxcount == 0) return hipSuccess;
  // 4 elements per thread per trip; enough blocks for ~4 trips each, capped to fill the chip a few times over
  int64_t blocks = (maxcount / 4 + 256 * 4 - 1) / (256 * 4);
  if (blocks < 1) blocks = 1;
  if (blocks > 2048) blocks = 2048;
  dim3 grid((unsigned)blocks, (unsigned)g.count);
  if (n_dtype == DType::BF16) hipLaunchKernelGGL(adam_group_kernel<__bf16>, grid, dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(adam_group_kernel<float>, grid, dim3(256), 0, stream, g);
  return hipGetLastError();
}

// One aligned 16-byte piece of dst per thread and trip; the source piece is read with whatever
// alignment its row has (memcpy lets the compiler pick the widest access the target allows there).
__global__ __launch_bounds__(256) void pad_rows_kernel(const PadGroup grp) {
  const PadProblem& pr = grp.p[blockIdx.y];
  const __bf16* __restrict__ src = static_cast<const __bf16*>(pr.src);
  __bf16* __restrict__ dst = static_cast<__bf16*>(pr.dst);
  const int cols = pr.cols, cpr = pr.ldd / 8;  // pieces per row
  const int64_t pieces = (int64_t)pr.rows * cpr;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t c = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; c < pieces; c += stride) {
    const int64_t row = c / cpr;
    const int col = (int)(c % cpr) * 8;
    const __bf16* s = src + row * pr.lds + col;
    uint4 v;
    if (col + 8 <= cols) {
      __builtin_memcpy(&v, s, sizeof(uint4));
    } else {
      __bf16 tmp[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) tmp[e] = col + e < cols ? s[e] : (__bf16)0.f;
      __builtin_memcpy(&v, tmp, sizeof(uint4));
    }
    *reinterpret_cast<uint4*>(dst + row * pr.ldd + col) = v;
  }
}

hipError_t launch_pad_rows_group(const PadGroup& g, hipStream_t stream) {
  if (g.count <= 0) return hipSuccess;
  if (g.count > kMaxGroup) return hipErrorInvalidValue;
  int64_t most = 0;
  for (int i = 0; i < g.count; ++i) {
    const PadProblem& p = g.p[i];
    if (p.rows < 1 || p.cols < 1 || p.ldd < p.cols || p.ldd % 8 != 0 || p.lds < p.cols || (reinterpret_cast<uintptr_t>(p.dst) & 15))
      return hipErrorInvalidValue;
    const int64_t pieces = (int64_t)p.rows * (p.ldd / 8);
    most = pieces > most ? pieces : most;
  }
  int64_t blocks = (most + 256 * 4 - 1) / (256 * 4);
  if (blocks < 1) blocks = 1;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(pad_rows_kernel, dim3((unsigned)blocks, (unsigned)g.count), dim3(256), 0, stream, g);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void fill_zero_kernel(unsigned char* p, size_t bytes) {
  const size_t nvec = bytes / 16;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  const size_t first = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint4* pv = reinterpret_cast<uint4*>(p);
  for (size_t i = first; i < nvec; i += stride) pv[i] = make_uint4(0u, 0u, 0u, 0u);
  const size_t tail = nvec * 16 + first;  // fewer than 16 trailing bytes
  if (tail < bytes) p[tail] = 0;
}

// Zero `bytes` at a 16-byte-aligned pointer with a plain kernel (not a memset node), so the
// call can be recorded in a HIP graph like every other piece of the library's work.
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t stream) {
  if (bytes == 0) return hipSuccess;
  size_t blocks = (bytes / 16 + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(fill_zero_kernel, dim3((unsigned)blocks), dim3(256), 0, stream,
                     static_cast<unsigned char*>(ptr), bytes);
  return hipGetLastError();
}

// dst (cols x rows) = src^T through a padded 64 x 64 LDS tile; element-wise, any shape / stride.
template <class T>
__global__ __launch_bounds__(256) void transpose_group_kernel(const TransposeGroup grp) {
  constexpr int TS = 64;
  __shared__ T tile[TS][TS + 2];
  const TransposeProblem& pr = grp.p[blockIdx.y];
  const T* __restrict__ src = static_cast<const T*>(pr.src);
  T* __restrict__ dst = static_cast<T*>(pr.dst);
  const int tiles_c = (pr.cols + TS - 1) / TS;
  const int ntiles = tiles_c * ((pr.rows + TS - 1) / TS);
  for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const int i0 = (t / tiles_c) * TS, j0 = (t % tiles_c) * TS;
    for (int e = threadIdx.x; e < TS * TS; e += 256) {
      const int i = e / TS, j = e % TS;
      if (i0 + i < pr.rows && j0 + j < pr.cols) tile[i][j] = src[(size_t)(i0 + i) * pr.lds + j0 + j];
    }
    __syncthreads();
    for (int e = threadIdx.x; e < TS * TS; e += 256) {
      const int j = e / TS, i = e % TS;
      if (i0 + i < pr.rows && j0 + j < pr.cols) dst[(size_t)(j0 + j) * pr.ldd + i0 + i] = tile[i][j];
    }
    __syncthreads();
  }
}

hipError_t launch_transpose_group(const TransposeGroup& g, DType dt, hipStream_t stream) {
  if (g.count <= 0) return hipSuccess;
  if (g.count > kMaxGroup) return hipErrorInvalidValue;
  int64_t maxtiles = 0;
  for (int i = 0; i < g.count; ++i) {
    const int64_t t = (int64_t)((g.p[i].rows + 63) / 64) * ((g.p[i].cols + 63) / 64);
    maxtiles = t > maxtiles ? t : maxtiles;
  }
  if (maxtiles == 0) return hipSuccess;
  const dim3 grid((unsigned)(maxtiles > 2048 ? 2048 : maxtiles), (unsigned)g.count);
  if (dt == DType::BF16) hipLaunchKernelGGL(transpose_group_kernel<__bf16>, grid, dim3(256), 0, stream, g);
  else hipLaunchKernelGGL(transpose_group_kernel<float>, grid, dim3(256), 0, stream, g);
  return hipGetLastError();
}

}  // namespace galore
