// Shared pieces of the subspace refresh (Algorithm 2, refresh branch; Sec. 3.3 SVD equation): the per-tensor
// descriptor table the kernels read, workspace layout, tuning constants, block reductions, and the entry points
// of the two long launch sequences (Householder QR in refresh_qr.hip, Rayleigh-Ritz eigen-solve in
// refresh_ritz.hip) that the driver in refresh.hip strings together.
#pragma once
#include <cstdlib>
#include <type_traits>

#include "refresh.hpp"

namespace galore {
namespace rf {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

constexpr int kJacobiSweeps = 10;   // upper bound; sweeps after convergence return at once
constexpr float kJacobiTol = 1e-5f;  // |b_p.b_q| <= tol |b_p||b_q|: a few times the rounding floor of an fp32 dot of length r
// A sweep whose largest rotation stayed below this level is the last one (Gram-matrix kernel): inner
// products of long fp32 rows keep crossing kJacobiTol by rounding alone, so "no rotation at all" is
// rarely reached although the result has stopped changing.
constexpr float kJacobiStopTol = 4e-5f;
constexpr int kNB = 8;               // reflectors per Householder panel (block_sum_vec sums 8 values)
constexpr int kRPT = 4;              // rows per thread in the panel kernels (1024 threads): k - j0 <= 4096
constexpr int kSW = 8;               // columns per block in the blocked reflector application

struct RefreshTensor {
  float* C;      // k x k Gram matrix
  float* Q;      // Qt: r x k, the iteration block transposed
  float* Z;      // Zt: r x k, product block / factored reflectors / fp32 projector, transposed
  float* Bw;     // r x r Rayleigh-Ritz matrix, rotated in place
  float* Jt;     // r x r accumulated rotations (rows = eigenvectors)
  float* S;      // St: r x r, rows = eigenvectors, ordered by decreasing Ritz value, unit length
  float* tau;    // r
  float* vscale; // r
  float* vclean; // round_up(r, 32) x k: reflectors as plain vectors (unit diagonal, zeros above, scaled), transposed
  float* tmat;   // (r / 32 macro panels) x 32 x 32: triangular factors T of the compact WY form
  float* tpart;  // 8 x 32 x 32: shares of V^T V of the macro panel being prepared
  float* wpart;  // (r / 32 + 1) x 4 x 32 x 32: shares of w = x V^T, per block of 32 target rows and slice of positions
  float* lambda; // r
  int32_t* order;// r : order[i] = output column of eigenvector i
  int32_t* sweep_flag;  // kJacobiSweeps + 1 : sweep s rotated something
  void* proj_t;  // output, r x k, ld ldpt (the projector itself is its transpose)
  int32_t k;
  int32_t ldpt;
  uint64_t seed;
  int32_t proj_is_bf16;  // dtype of proj_t
  int32_t split;         // Zt = Qt C runs as a bf16 product of three-way split operands (see split3)
  __bf16* Csplit;        // k x 6k: row n = [hi | mid | hi | mid | lo | hi] parts of row n of C
  __bf16* Qsplit;        // r x 6k: row i = [hi | hi | mid | mid | hi | lo] parts of row i of Qt
};

// The kernels of the long launch sequences (QR panels, Jacobi rounds: about two thousand launches per
// refresh) read this table from device memory through a pointer; the few one-off kernels take it by
// value.  By value every launch would put 2.3 KB into the runtime's kernel-argument ring, whose few MB
// then hold only some hundred launches: the host thread ends up waiting for the GPU launch by launch
// for the whole refresh instead of running ahead of it.
struct RefreshGroup {
  int32_t count;
  int32_t r;
  RefreshTensor t[kMaxGroup];
};

struct Layout {
  size_t C, Q, Z, Bw, Jt, S, tau, vscale, vclean, tmat, tpart, wpart, lambda, order, sweep_flag, group, Csplit, Qsplit, total;
};

bool split_products(int64_t k, int64_t r);
Layout layout_for(int64_t k, int64_t r);

inline unsigned blocks_for(int64_t count, int per_block, unsigned cap) {
  int64_t b = (count + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > cap) b = cap;
  return (unsigned)b;
}

#define GALORE_RETURN_IF(e_)            \
  do {                                  \
    hipError_t _e = (e_);               \
    if (_e != hipSuccess) return _e;    \
  } while (0)

// Householder QR of Zt (r x k per tensor, transposed layout) of every tensor of the group, reflectors left in Zt,
// then Qt <- the orthonormal factor (refresh_qr.hip).  dgrp: the group's table in device memory; kmax: largest short side.
hipError_t launch_householder_qr(const RefreshGroup& grp, const RefreshGroup* dgrp, int64_t kmax, hipStream_t stream);
// Eigen-decomposition of the symmetric r x r matrix in Bw by blocked one-sided Jacobi, eigenvectors ordered by
// decreasing Ritz value and normalised into S (refresh_ritz.hip).
hipError_t launch_ritz_solve(const RefreshGroup& grp, const RefreshGroup* dgrp, bool crowded, hipStream_t stream);

namespace {

// ---- block reductions (wavefront shuffles, then LDS across the waves) ------------------------
// Sum over the 64 lanes of a wavefront; every lane gets the result.  Data-parallel-primitive
// moves inside the VALU (quad permutes, row mirrors, row broadcasts) instead of LDS-crossbar
// shuffles: six dependent adds of a few cycles each where six ds_bpermute round trips took
// well over a hundred cycles apiece.
__device__ __forceinline__ float wave_sum(float v) {
  auto dpp = [](float x, auto ctrl, auto row_mask) {
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), decltype(ctrl)::value,
                                                                 decltype(row_mask)::value, 0xF, false));
  };
  using std::integral_constant;
  v += dpp(v, integral_constant<int, 0xB1>{}, integral_constant<int, 0xF>{});   // quad_perm [1,0,3,2]
  v += dpp(v, integral_constant<int, 0x4E>{}, integral_constant<int, 0xF>{});   // quad_perm [2,3,0,1]
  v += dpp(v, integral_constant<int, 0x141>{}, integral_constant<int, 0xF>{});  // row_half_mirror
  v += dpp(v, integral_constant<int, 0x140>{}, integral_constant<int, 0xF>{});  // row_mirror: each row of 16 holds its sum
  v += dpp(v, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{});  // row_bcast15 into rows 1 and 3
  v += dpp(v, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{});  // row_bcast31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// Sum over all threads of the block; every thread gets the result.  `red` holds >= 16 floats.
__device__ __forceinline__ float block_sum(float v, float* red) {
  v = wave_sum(v);
  const int wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[wave] = v;
  __syncthreads();
  float s = 0.f;
  for (int w = 0; w < nw; ++w) s += red[w];
  return s;
}

// which 0: Qt <- [I_r 0] (r x k);  which 1: Jt <- I_r and the sweep flags <- 0
__global__ __launch_bounds__(256) void identity_fill_kernel(const RefreshGroup* __restrict__ gp, int which) {
  const RefreshGroup& grp = *gp;
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  if (which == 1 && blockIdx.x == 0 && threadIdx.x <= kJacobiSweeps) t.sweep_flag[threadIdx.x] = 0;
  float* X = which == 0 ? t.Q : t.Jt;
  const int64_t width = which == 0 ? t.k : r;
  const int64_t count = width * r;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
    X[i] = (i / width == i % width) ? 1.f : 0.f;
}

}  // namespace
}  // namespace rf
}  // namespace galore
