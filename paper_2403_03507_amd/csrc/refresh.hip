// Subspace refresh (Algorithm 2, refresh branch; Sec. 3.3 SVD equation for P_t, Q_t).
//
// The paper takes P = U[:, :r] from an SVD of the gradient.  Here the leading singular
// vectors of the short side are computed from the Gram matrix C = G G^T (or G^T G), whose
// eigenvectors they are, by blocked orthogonal iteration:
//     Q <- Gaussian (k x r);  repeat iters times: Z = C Q ; Q = qr(Z).Q
// followed by a Rayleigh-Ritz step B = Q^T C Q = S L S^T, P = Q S, columns ordered by
// decreasing L, each column signed so that its largest-magnitude entry is positive.
//   * Gram and the tall GEMMs run on the grouped MFMA GEMM; Zt = Qt C runs on the bf16 matrix cores with both
//     operands split into three bf16 parts (as accurate as an fp32 product; split_rows_kernel below).
//   * QR (refresh_qr.hip) is Householder in panels of 8 reflectors held in registers inside macro panels of 32
//     columns; the rest of the matrix sees a macro panel once, in compact WY form on the fp32 matrix cores.
//   * The r x r eigenproblem (refresh_ritz.hip) is solved by one-sided (Hestenes) Jacobi on the rows of B, blocked:
//     a workgroup forms the 32 x 32 Gram matrix of two 16-row blocks on the matrix cores straight from global
//     memory, rotates on the Gram matrix alone and applies the accumulated 32 x 32 rotation to its rows of B and
//     of the eigenvector matrix; block pairs follow a round-robin schedule, one launch per round of disjoint pairs.
// This file holds the driver (refresh_group), the workspace layout, the start blocks, the operand split and the
// final sign rule / store.
// The iteration blocks are kept TRANSPOSED in memory (Qt, Zt: r x k row-major), so that a
// column of Z - the thing a Householder reflector works on - is a contiguous row and every
// access below is coalesced; C is symmetric, so Zt = Qt C needs no transposed GEMM either.
// All tensors of a group advance in lock-step (blockIdx.y = tensor), nothing syncs the host,
// iteration counts are fixed, and no atomics are used, so results are reproducible bit for bit.
#include "refresh_common.hpp"

namespace galore {
namespace rf {

// Whether Zt = Qt C of a tensor with short side k runs on the bf16 matrix cores with split operands
// (below).  The fp32 matrix-core product stays for short sides that the large-tile bf16 kernel
// cannot take (6k has to be a multiple of its K step of 64) or that are too small to matter.
bool split_products(int64_t k, int64_t r) {
  static const bool off = [] { const char* e = getenv("GALORE_REFRESH_FP32_PRODUCTS"); return e && e[0] == '1'; }();
  return !off && k % 32 == 0 && k >= 512 && r >= 8;
}

Layout layout_for(int64_t k, int64_t r) {
  Layout L{};
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align_up(bytes); return o; };
  L.C = take((size_t)k * k * 4);
  L.Q = take((size_t)k * r * 4);
  L.Z = take((size_t)k * r * 4);
  L.Bw = take((size_t)r * r * 4);
  L.Jt = take((size_t)r * r * 4);
  L.S = take((size_t)r * r * 4);
  L.tau = take((size_t)r * 4);
  L.vscale = take((size_t)r * 4);
  L.vclean = take((size_t)((r + 31) / 32 * 32) * k * 4);
  L.tmat = take((size_t)((r + 31) / 32) * 1024 * 4);
  L.tpart = take((size_t)8 * 1024 * 4);
  L.wpart = take((size_t)((r + 31) / 32 + 1) * 4 * 1024 * 4);
  L.lambda = take((size_t)r * 4);
  L.order = take((size_t)r * 4);
  L.sweep_flag = take((size_t)(kJacobiSweeps + 1) * 4);
  L.group = take(sizeof(RefreshGroup));  // the descriptor table of the group this tensor leads
  const bool split = split_products(k, r);
  L.Csplit = take(split ? (size_t)k * 6 * k * 2 : 0);
  L.Qsplit = take(split ? (size_t)r * 6 * k * 2 : 0);
  L.total = off;
  return L;
}

}  // namespace rf

using namespace rf;

namespace {

// x = hi + mid + lo exactly: each part is a bf16 (8 significant bits), the three together hold the
// 24 significant bits of an fp32 number (every difference below is exact in fp32).
__device__ __forceinline__ void split3(float x, __bf16& hi, __bf16& mid, __bf16& lo) {
  hi = (__bf16)x;
  const float r1 = x - (float)hi;
  mid = (__bf16)r1;
  lo = (__bf16)(r1 - (float)mid);
}

// Split-bf16 form of the fp32 product Zt = Qt C.  With a = ah + am + al and c = ch + cm + cl,
//   a c = ah ch + ah cm + am ch + am cm + ah cl + al ch + (am cl + al cm + al cl),
// and the bracket is below 2^-23 |a c|: the six kept products, accumulated in fp32 by the bf16 matrix
// cores, are as accurate as one fp32 multiply-add, at more than twice the rate of the fp32 matrix
// cores on this chip (6 bf16 passes at ~1.1 PFLOP/s against one fp32 pass at ~0.09).  The six
// products become ONE bf16 GEMM over a contraction index of length 6k: operand rows are the
// parts laid side by side, in the orders [hi hi mid mid hi lo] (Qt) and [hi mid hi mid lo hi] (C).
// IS_C: source is C (k x k, symmetric, so row n serves as column n), else Qt (r x k).
template <bool IS_C>
__global__ __launch_bounds__(256) void split_rows_kernel(const RefreshGroup* __restrict__ gp) {
  const RefreshGroup& grp = *gp;
  const RefreshTensor& t = grp.t[blockIdx.y];
  if (!t.split) return;
  const int k = t.k;
  const int rows = IS_C ? k : grp.r;
  const float* __restrict__ src = IS_C ? t.C : t.Q;
  __bf16* __restrict__ dst = IS_C ? t.Csplit : t.Qsplit;
  const int64_t nvec = (int64_t)rows * (k >> 3);  // pieces of 8 consecutive elements (k is a multiple of 32)
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
  typedef float f32x4_t __attribute__((ext_vector_type(4)));
  for (int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; q < nvec; q += stride) {
    const int row = (int)(q / (k >> 3)), col = (int)(q % (k >> 3)) << 3;
    const float* p = src + (size_t)row * k + col;
    const f32x4_t x0 = *reinterpret_cast<const f32x4_t*>(p), x1 = *reinterpret_cast<const f32x4_t*>(p + 4);
    bf16x8_t part[3];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      __bf16 h, m, l;
      split3(e < 4 ? x0[e] : x1[e - 4], h, m, l);
      part[0][e] = h; part[1][e] = m; part[2][e] = l;
    }
    __bf16* out = dst + (size_t)row * 6 * k + col;
    constexpr int order_q[6] = {0, 0, 1, 1, 0, 2}, order_c[6] = {0, 1, 0, 1, 2, 0};
#pragma unroll
    for (int sgm = 0; sgm < 6; ++sgm)
      *reinterpret_cast<bf16x8_t*>(out + (size_t)sgm * k) = part[IS_C ? order_c[sgm] : order_q[sgm]];
  }
}

// Copy the descriptor table into device memory (one launch per refresh).
__global__ __launch_bounds__(256) void upload_group_kernel(const RefreshGroup grp, RefreshGroup* dst) {
  static_assert(sizeof(RefreshGroup) % 4 == 0, "copied as 32-bit words");
  const uint32_t* src = reinterpret_cast<const uint32_t*>(&grp);
  uint32_t* out = reinterpret_cast<uint32_t*>(dst);
  for (int i = threadIdx.x; i < (int)(sizeof(RefreshGroup) / 4); i += blockDim.x) out[i] = src[i];
}

// ---- counter-based Gaussian start block ----------------------------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t z) {
  z += 0x9E3779B97F4A7C15ull;
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  return z ^ (z >> 31);
}

__global__ __launch_bounds__(256) void gaussian_fill_kernel(const RefreshGroup grp) {
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int64_t count = (int64_t)t.k * grp.r;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
    const uint64_t h = mix64(t.seed ^ mix64((uint64_t)i));
    const float u1 = (float)((h >> 40) + 1) * (1.0f / 16777216.0f);  // (0, 1]
    const float u2 = (float)(h & 0xFFFFFF) * (1.0f / 16777216.0f);   // [0, 1)
    t.Q[i] = sqrtf(-2.0f * logf(u1)) * cosf(6.28318530718f * u2);
  }
}

// Warm start: the iteration block is the previous projector, Qt <- proj_t widened to fp32.
__global__ __launch_bounds__(256) void projector_start_kernel(const RefreshGroup grp) {
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int64_t count = (int64_t)t.k * grp.r;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride) {
    const int64_t row = i / t.k, col = i - row * t.k;
    const int64_t src = row * t.ldpt + col;
    t.Q[i] = t.proj_is_bf16 ? (float)static_cast<const __bf16*>(t.proj_t)[src] : static_cast<const float*>(t.proj_t)[src];
  }
}

// proj_t[c][:] = sign * Zt[c][:] with the sign chosen so the entry of largest magnitude (lowest
// index on ties) is positive; stored in the projector's dtype (round to nearest even for bf16).
// One block per projector column (= row of Zt).
template <class T>
__global__ __launch_bounds__(256) void finalize_projector_kernel(const RefreshGroup grp) {
  __shared__ float bestv[256];
  __shared__ int besti[256];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int k = t.k, c = blockIdx.x;
  const float* __restrict__ z = t.Z + (size_t)c * k;
  float bv = -1.f; int bi = 0x7fffffff;
  for (int row = threadIdx.x; row < k; row += 256) {
    const float x = fabsf(z[row]);
    if (x > bv) { bv = x; bi = row; }  // rows ascend per thread: first maximum kept
  }
  bestv[threadIdx.x] = bv; besti[threadIdx.x] = bi;
  __syncthreads();
  for (int o = 128; o > 0; o >>= 1) {
    if (threadIdx.x < o) {
      const float x = bestv[threadIdx.x + o]; const int y = besti[threadIdx.x + o];
      if (x > bestv[threadIdx.x] || (x == bestv[threadIdx.x] && y < besti[threadIdx.x])) { bestv[threadIdx.x] = x; besti[threadIdx.x] = y; }
    }
    __syncthreads();
  }
  // No entry compares greater than the start value when all of them are NaN (a gradient with
  // non-finite entries): the index is still the sentinel then, and row 0 serves as well as any.
  const int pick = besti[0] < k ? besti[0] : 0;
  const float sgn = z[pick] < 0.f ? -1.f : 1.f;
  T* P = static_cast<T*>(t.proj_t) + (size_t)c * t.ldpt;
  for (int row = threadIdx.x; row < k; row += 256) P[row] = (T)(sgn * z[row]);
}

}  // namespace

size_t refresh_workspace_bytes(int64_t kdim, int64_t r) { return layout_for(kdim, r).total; }

hipError_t refresh_group(const std::vector<RefreshItem>& items, int r, int iters, bool warm_start, bool crowded, hipStream_t stream) {
  const int n = (int)items.size();
  if (n == 0) return hipSuccess;
  if (n > kMaxGroup) return hipErrorInvalidValue;

  RefreshGroup grp{};
  grp.count = n;
  grp.r = r;
  int64_t kmax = 0;
  for (int i = 0; i < n; ++i) {
    const RefreshItem& it = items[i];
    const int64_t k = it.rows <= it.cols ? it.rows : it.cols;
    const Layout L = layout_for(k, r);
    RefreshTensor& t = grp.t[i];
    t.C = reinterpret_cast<float*>(it.ws + L.C);
    t.Q = reinterpret_cast<float*>(it.ws + L.Q);
    t.Z = reinterpret_cast<float*>(it.ws + L.Z);
    t.Bw = reinterpret_cast<float*>(it.ws + L.Bw);
    t.Jt = reinterpret_cast<float*>(it.ws + L.Jt);
    t.S = reinterpret_cast<float*>(it.ws + L.S);
    t.tau = reinterpret_cast<float*>(it.ws + L.tau);
    t.vscale = reinterpret_cast<float*>(it.ws + L.vscale);
    t.vclean = reinterpret_cast<float*>(it.ws + L.vclean);
    t.tmat = reinterpret_cast<float*>(it.ws + L.tmat);
    t.tpart = reinterpret_cast<float*>(it.ws + L.tpart);
    t.wpart = reinterpret_cast<float*>(it.ws + L.wpart);
    t.lambda = reinterpret_cast<float*>(it.ws + L.lambda);
    t.order = reinterpret_cast<int32_t*>(it.ws + L.order);
    t.sweep_flag = reinterpret_cast<int32_t*>(it.ws + L.sweep_flag);
    t.proj_t = it.proj_t;
    t.k = (int32_t)k;
    t.ldpt = (int32_t)it.ldpt;
    t.seed = it.seed;
    t.proj_is_bf16 = it.dt == DType::BF16;
    t.split = split_products(k, r) ? 1 : 0;
    t.Csplit = reinterpret_cast<__bf16*>(it.ws + L.Csplit);
    t.Qsplit = reinterpret_cast<__bf16*>(it.ws + L.Qsplit);
    kmax = k > kmax ? k : kmax;
  }

  RefreshGroup* dgrp;
  {
    const RefreshItem& lead = items[0];
    dgrp = reinterpret_cast<RefreshGroup*>(lead.ws + layout_for(lead.rows <= lead.cols ? lead.rows : lead.cols, r).group);
    hipLaunchKernelGGL(upload_group_kernel, dim3(1), dim3(256), 0, stream, grp, dgrp);
    GALORE_RETURN_IF(hipGetLastError());
  }

  // Gram matrix of the short side, split by (dtype, orientation).
  for (int dti = 0; dti < 2; ++dti)
    for (int left = 1; left >= 0; --left) {
      const DType dt = dti == 0 ? DType::F32 : DType::BF16;
      GemmGroup g{};
      for (int i = 0; i < n; ++i) {
        const RefreshItem& it = items[i];
        if (it.dt != dt || (int)(it.rows <= it.cols) != left) continue;
        GemmProblem& p = g.p[g.count++];
        p.A = it.G; p.B = it.G; p.lda = (int)it.ldg; p.ldb = (int)it.ldg;
        p.M = p.N = grp.t[i].k;
        p.K = (int)(left ? it.cols : it.rows);
        p.C = grp.t[i].C; p.ldc = grp.t[i].k;
      }
      // LEFT: C = G G^T, both operands [row][K] ; RIGHT: C = G^T G, both operands [K][col]
      GALORE_RETURN_IF(launch_gemm_group(g, dt, left != 0, left != 0, Epilogue::StoreSymF32, stream));
    }

  const dim3 fill_grid(blocks_for(kmax * r, 256 * 8, 1024), n);
  if (warm_start) hipLaunchKernelGGL(projector_start_kernel, fill_grid, dim3(256), 0, stream, grp);
  else hipLaunchKernelGGL(gaussian_fill_kernel, fill_grid, dim3(256), 0, stream, grp);
  GALORE_RETURN_IF(hipGetLastError());

  bool any_split = false;
  for (int i = 0; i < n; ++i) any_split = any_split || grp.t[i].split;
  if (any_split) {  // C is complete: lay out its three bf16 parts once per refresh
    hipLaunchKernelGGL(split_rows_kernel<true>, dim3(blocks_for(kmax * kmax / 8, 256, 4096), n), dim3(256), 0, stream, dgrp);
    GALORE_RETURN_IF(hipGetLastError());
  }

  auto gemm_f32 = [&](int which) -> hipError_t {
    GemmGroup g{};
    if (which == 0 && any_split) {
      // tensors whose product runs on the bf16 matrix cores: split Qt, then one (K,K) GEMM over 6k
      hipLaunchKernelGGL(split_rows_kernel<false>, dim3(blocks_for(kmax * r / 8, 256, 4096), n), dim3(256), 0, stream, dgrp);
      GALORE_RETURN_IF(hipGetLastError());
      GemmGroup gs{};
      for (int i = 0; i < n; ++i) {
        const RefreshTensor& t = grp.t[i];
        GemmProblem& p = t.split ? gs.p[gs.count++] : g.p[g.count++];
        if (t.split) {
          p.A = t.Qsplit; p.lda = 6 * t.k; p.B = t.Csplit; p.ldb = 6 * t.k; p.M = r; p.N = t.k; p.K = 6 * t.k; p.C = t.Z; p.ldc = t.k;
        } else {
          p.A = t.Q; p.lda = t.k; p.B = t.C; p.ldb = t.k; p.M = r; p.N = t.k; p.K = t.k; p.C = t.Z; p.ldc = t.k;
        }
      }
      GALORE_RETURN_IF(launch_gemm_group(gs, DType::BF16, true, true, Epilogue::StoreF32, stream));
      if (g.count == 0) return hipSuccess;
      return launch_gemm_group(g, DType::F32, true, false, Epilogue::StoreF32, stream);
    }
    g.count = n;
    for (int i = 0; i < n; ++i) {
      const RefreshTensor& t = grp.t[i];
      GemmProblem& p = g.p[i];
      if (which == 0) {         // Zt (r x k) = Qt C     (C symmetric)
        p.A = t.Q; p.lda = t.k; p.B = t.C; p.ldb = t.k; p.M = r; p.N = t.k; p.K = t.k; p.C = t.Z; p.ldc = t.k;
      } else if (which == 1) {  // Bw (r x r) = Qt Zt^T = Q^T C Q
        p.A = t.Q; p.lda = t.k; p.B = t.Z; p.ldb = t.k; p.M = r; p.N = r; p.K = t.k; p.C = t.Bw; p.ldc = r;
      } else {                  // Zt (r x k) = St Qt = (Q S)^T
        p.A = t.S; p.lda = r; p.B = t.Q; p.ldb = t.k; p.M = r; p.N = t.k; p.K = r; p.C = t.Z; p.ldc = t.k;
      }
    }
    return launch_gemm_group(g, DType::F32, true, which == 1, Epilogue::StoreF32, stream);
  };

  for (int it = 0; it < iters; ++it) {
    GALORE_RETURN_IF(gemm_f32(0));
    GALORE_RETURN_IF(launch_householder_qr(grp, dgrp, kmax, stream));
  }

  // Rayleigh-Ritz
  GALORE_RETURN_IF(gemm_f32(0));
  GALORE_RETURN_IF(gemm_f32(1));
  GALORE_RETURN_IF(launch_ritz_solve(grp, dgrp, crowded, stream));
  GALORE_RETURN_IF(gemm_f32(2));

  // sign convention + store in the projector dtype, split by dtype
  for (int dti = 0; dti < 2; ++dti) {
    const DType dt = dti == 0 ? DType::F32 : DType::BF16;
    RefreshGroup sub{};
    sub.r = r;
    for (int i = 0; i < n; ++i)
      if (items[i].dt == dt) sub.t[sub.count++] = grp.t[i];
    if (sub.count == 0) continue;
    const dim3 grid(r, sub.count);
    if (dt == DType::F32) hipLaunchKernelGGL(finalize_projector_kernel<float>, grid, dim3(256), 0, stream, sub);
    else hipLaunchKernelGGL(finalize_projector_kernel<__bf16>, grid, dim3(256), 0, stream, sub);
    GALORE_RETURN_IF(hipGetLastError());
    // the projector proper (k x r) is the transpose of what was just written
    TransposeGroup tg{};
    for (int i = 0; i < n; ++i) {
      if (items[i].dt != dt) continue;
      TransposeProblem& p = tg.p[tg.count++];
      p.src = items[i].proj_t; p.lds = (int)items[i].ldpt;
      p.dst = items[i].proj; p.ldd = (int)items[i].ldp;
      p.rows = r; p.cols = grp.t[i].k;
    }
    GALORE_RETURN_IF(launch_transpose_group(tg, dt, stream));
  }
  return hipSuccess;
}

}  // namespace galore
