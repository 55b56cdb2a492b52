// Subspace refresh (Algorithm 2, refresh branch; Sec. 3.3 SVD equation for P_t, Q_t).
//
// The paper takes P = U[:, :r] from an SVD of the gradient.  Here the leading singular
// vectors of the short side are computed from the Gram matrix C = G G^T (or G^T G), whose
// eigenvectors they are, by blocked orthogonal iteration:
//     Q <- Gaussian (k x r);  repeat iters times: Z = C Q ; Q = qr(Z).Q
// followed by a Rayleigh-Ritz step B = Q^T C Q = S L S^T, P = Q S, columns ordered by
// decreasing L, each column signed so that its largest-magnitude entry is positive.
//   * Gram and the tall GEMMs run on the grouped MFMA GEMM.
//   * QR is Householder in panels of 8 reflectors: one block per tensor factors a panel held in
//     registers (wavefront shuffle + LDS reductions for the norms and inner products), then
//     blocks of 8 trailing columns apply the 8 reflectors to register-resident data, so each
//     panel costs one read and one write of the trailing matrix; Q is formed by applying the
//     panels to [I; 0] backwards.  Short sides beyond 4096 fall back to one launch per reflector.
//   * The r x r eigenproblem is solved by one-sided (Hestenes) Jacobi on the rows of B, blocked:
//     a workgroup holds two blocks of 16 whole rows in LDS, orthogonalises them against each
//     other and applies the accumulated 32 x 32 rotation to the eigenvector rows; block pairs
//     follow a round-robin schedule, one launch per round of disjoint pairs.  (Rows longer than
//     LDS allows fall back to one launch per round of row pairs.)
// The iteration blocks are kept TRANSPOSED in memory (Qt, Zt: r x k row-major), so that a
// column of Z - the thing a Householder reflector works on - is a contiguous row and every
// access below is coalesced; C is symmetric, so Zt = Qt C needs no transposed GEMM either.
// All tensors of a group advance in lock-step (blockIdx.y = tensor), nothing syncs the host,
// iteration counts are fixed, and no atomics are used, so results are reproducible bit for bit.
#include "refresh.hpp"
#include <cstdlib>

#include <type_traits>

namespace galore {

namespace {

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

// ---- Householder reflector j applied to 32 columns (fallback for short sides beyond 4096) -------
// Element (row, col) of Z lives at Zt[col * k + row].  Column j (rows > j) holds the unscaled
// reflector, v_j = 1, v_row = Z[row][j] * vscale_j.  H_j = I - tau_j v v^T is applied to columns
// col_begin + 32 blockIdx.x + (0..31) of the target, rows >= j.  Each column is handled by one
// 32-lane half-wave striding over the rows, so the inner product is a plain shuffle reduction.
// COMPUTE: derive tau_j and vscale_j from column j first (factoring; target == Z, col_begin = j + 1)
// and let block 0 publish them; otherwise read them (forming Q).
template <bool COMPUTE>
__global__ __launch_bounds__(1024) void householder_strip_kernel(const RefreshGroup* __restrict__ gp, int j, int col_begin,
                                                                 int target_is_q) {
  const RefreshGroup& grp = *gp;
  __shared__ float red1[16];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r, k = t.k;
  const float* __restrict__ vcol = t.Z + (size_t)j * k;  // column j of Z
  const int cg = threadIdx.x >> 5, l32 = threadIdx.x & 31;
  const int col = col_begin + 32 * blockIdx.x + cg;
  const bool active = col < r;
  float* __restrict__ xcol = (target_is_q ? t.Q : t.Z) + (size_t)(active ? col : 0) * k;

  float tau, vs;
  if (COMPUTE) {
    float part = 0.f;
    for (int row = j + 1 + threadIdx.x; row < k; row += 1024) part += vcol[row] * vcol[row];
    const float sigma = block_sum(part, red1);
    const float x0 = vcol[j];
    if (sigma == 0.f) {
      tau = 0.f; vs = 0.f;
    } else {
      const float beta = -copysignf(sqrtf(x0 * x0 + sigma), x0);
      tau = (beta - x0) / beta;
      vs = 1.0f / (x0 - beta);
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) { t.tau[j] = tau; t.vscale[j] = vs; }
  } else {
    tau = t.tau[j]; vs = t.vscale[j];
  }
  if (tau == 0.f || !active) return;  // H_j = I, or a column past the matrix (whole half-wave)

  float part = 0.f;
  for (int row = j + 1 + l32; row < k; row += 32) part += vcol[row] * xcol[row];
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) part += __shfl_xor(part, o, 32);
  const float tw = tau * (xcol[j] + vs * part);
  const float tws = tw * vs;
  for (int row = j + 1 + l32; row < k; row += 32) xcol[row] -= vcol[row] * tws;
  if (l32 == 0) xcol[j] -= tw;
}

// ---- blocked Householder (panels of kNB reflectors), for k <= 1024 * kRPT -----------------------
// Thread t of the 1024-thread block owns rows j0 + t + 1024 s (s < kRPT) and keeps them in
// registers, so a panel is read and written once however many reflectors touch it.

// Sum 8 values over the block of 16 waves; every thread gets all sums.  One barrier per call: red holds
// two areas of 16 x 8 floats that successive calls use alternately (phase), so a wave may write its
// partial sums of call n + 1 while slower waves still read those of call n, and the area of call n is
// written again only after the barrier of call n + 1, which every reader of call n has passed.  Behind
// the barrier every wave adds the 16 partial sums itself: lane 8 w + c takes waves w and w + 8 of value c,
// three exchange steps add over w, and lanes 0 .. 7 then hold the eight sums (same bits in every wave).
__device__ __forceinline__ void block_sum_vec(float (&v)[8], float* red, int& phase) {
#pragma unroll
  for (int c = 0; c < 8; ++c) v[c] = wave_sum(v[c]);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  float* buf = red + phase * 128;
  phase ^= 1;
  if (lane == 0) {
#pragma unroll
    for (int c = 0; c < 8; ++c) buf[wave * 8 + c] = v[c];
  }
  __syncthreads();
  float a = buf[lane] + buf[64 + lane];
  a += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, a), 0x128, 0xF, 0xF, false));  // row_ror:8, lane ^ 8
  a += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 16) << 2, __builtin_bit_cast(int, a)));
  a += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, __builtin_bit_cast(int, a)));
#pragma unroll
  for (int c = 0; c < 8; ++c) v[c] = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, a), c));
}

// Factor columns [j0, j0 + nb) of Z below row j0: LAPACK-style reflectors, column j keeps the
// unscaled vector below its diagonal, tau_j and the scale 1 / (x0 - beta) go to side arrays.
__global__ __launch_bounds__(1024) void householder_panel_kernel(const RefreshGroup* __restrict__ gp, int j0, int nb) {
  const RefreshGroup& grp = *gp;
  __shared__ float red[2 * 16 * kNB];
  int red_phase = 0;
  __shared__ float bc[kNB + 1];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int k = t.k;
  float* __restrict__ Z = t.Z;  // element (row, col) at Z[col * k + row]
  float* const tau_out = t.tau;        // fetched from the table here, not inside thread 0's branch of every reflector round
  float* const vscale_out = t.vscale;
  const int tid = threadIdx.x;
  float x[kRPT][kNB];
#pragma unroll
  for (int s = 0; s < kRPT; ++s) {
    const int row = j0 + tid + 1024 * s;
#pragma unroll
    for (int c = 0; c < kNB; ++c) x[s][c] = (row < k && c < nb) ? Z[(size_t)(j0 + c) * k + row] : 0.f;
  }
#pragma unroll
  for (int i = 0; i < kNB; ++i) {
    if (i >= nb) break;
    const int j = j0 + i;
    // dot products of column i (rows > j) with itself and with the later panel columns
    float d[kNB];
#pragma unroll
    for (int c = 0; c < kNB; ++c) {
      float a = 0.f;
      if (c >= i) {
#pragma unroll
        for (int s = 0; s < kRPT; ++s)
          if (j0 + tid + 1024 * s > j) a += x[s][i] * x[s][c];
      }
      d[c] = a;
    }
    if (tid == i) {  // owner of row j publishes that row of the panel
#pragma unroll
      for (int c = 0; c < kNB; ++c) bc[c] = x[0][c];
    }
    block_sum_vec(d, red, red_phase);  // its barriers also publish bc
    const float x0 = bc[i];
    const float sigma = d[i];
    float tau = 0.f, vs = 0.f;
    if (sigma != 0.f) {
      const float beta = -copysignf(sqrtf(x0 * x0 + sigma), x0);
      tau = (beta - x0) / beta;
      vs = 1.0f / (x0 - beta);
    }
    if (tid == 0) { tau_out[j] = tau; vscale_out[j] = vs; }
    if (tau != 0.f) {
#pragma unroll
      for (int c = 0; c < kNB; ++c) {
        if (c <= i) continue;
        const float tw = tau * (bc[c] + vs * d[c]);
#pragma unroll
        for (int s = 0; s < kRPT; ++s) {
          const int row = j0 + tid + 1024 * s;
          if (row == j) x[s][c] -= tw;
          else if (row > j) x[s][c] -= tw * vs * x[s][i];
        }
      }
    }
    __syncthreads();  // bc is rewritten in the next round
  }
#pragma unroll
  for (int s = 0; s < kRPT; ++s) {
    const int row = j0 + tid + 1024 * s;
    if (row < k) {
#pragma unroll
      for (int c = 0; c < kNB; ++c)
        if (c < nb) Z[(size_t)(j0 + c) * k + row] = x[s][c];
    }
  }
}

// Apply the nb reflectors of panel j0 (stored in Z) to columns col_begin + kSW blockIdx.x + (0..kSW-1)
// of the target (Z itself while factoring, Q while forming the orthogonal factor), rows >= j0,
// in forward order (H_nb-1 ... H_0 X: factoring) or reverse order (H_0 ... H_nb-1 X: forming Q).
// With factor_next (factoring only), workgroup 0 - whose columns are the next panel - goes on to factor
// them while it still holds them in registers, exactly as householder_panel_kernel would: one launch and
// one trip of the panel through memory less per panel.
__global__ __launch_bounds__(1024) void householder_block_apply_kernel(const RefreshGroup* __restrict__ gp, int j0, int nb, int col_begin,
                                                                       int target_is_q, int reverse, int col_end, int factor_next) {
  const RefreshGroup& grp = *gp;
  static_assert(kSW == kNB, "the fused factorisation treats a workgroup's columns as one panel");
  __shared__ float red[2 * 16 * kSW];
  int red_phase = 0;
  __shared__ float bc[kNB + 1];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int k = t.k;
  const float* __restrict__ Zv = t.Z;
  float* __restrict__ X = target_is_q ? t.Q : t.Z;
  const int tid = threadIdx.x;
  const int c0 = col_begin + kSW * blockIdx.x;
  // v[s][ii]: entry of the ii-th reflector IN APPLICATION ORDER (unit diagonal, zeros above it)
  float v[kRPT][kNB], x[kRPT][kSW];
  // Every load below is unconditional, from an address that is valid whatever the guards say (the
  // guards only select afterwards): written as "if (inside) load", each of the 32 reflector entries
  // became a branch with its own scalar load, vector load and full wait, one after the other, and
  // those round trips were two thirds of this kernel's time.
  int jref[kNB];
  float vsc[kNB], taus[kNB];
  float* const vscale_p = t.vscale;   // both also written by the fused factorisation below
  float* const tau_p = t.tau;
#pragma unroll
  for (int ii = 0; ii < kNB; ++ii) {
    jref[ii] = ii < nb ? j0 + (reverse ? nb - 1 - ii : ii) : j0;
    vsc[ii] = vscale_p[jref[ii]];
    const float tau_any = tau_p[jref[ii]];
    taus[ii] = ii < nb ? tau_any : 0.f;
  }
#pragma unroll
  for (int s = 0; s < kRPT; ++s) {
    const int row = j0 + tid + 1024 * s;
    const int row_ok = row < k ? row : j0;  // j0 < k always
#pragma unroll
    for (int ii = 0; ii < kNB; ++ii) {
      // select by arithmetic (raw is finite wherever the matrix is): a select on the loaded value lets the
      // compiler sink the load back under a branch
      const float raw = Zv[(size_t)jref[ii] * k + row_ok];
      const int j = jref[ii];
      const bool in = row < k && ii < nb;
      v[s][ii] = __builtin_fmaf(raw, (in && row > j) ? vsc[ii] : 0.f, (in && row == j) ? 1.f : 0.f);
    }
#pragma unroll
    for (int c = 0; c < kSW; ++c) {
      const int col = c0 + c < col_end ? c0 + c : c0;  // c0 < col_end: the grid covers [col_begin, col_end)
      const float raw = X[(size_t)col * k + row_ok];
      x[s][c] = raw * ((row < k && c0 + c < col_end) ? 1.f : 0.f);
    }
  }
#pragma unroll
  for (int ii = 0; ii < kNB; ++ii) {
    if (ii >= nb) break;
    const float tau = taus[ii];
    if (tau == 0.f) continue;  // uniform over the block
    float w[kSW];
#pragma unroll
    for (int c = 0; c < kSW; ++c) {
      float a = 0.f;
#pragma unroll
      for (int s = 0; s < kRPT; ++s) a += v[s][ii] * x[s][c];
      w[c] = a;
    }
    block_sum_vec(w, red, red_phase);
#pragma unroll
    for (int s = 0; s < kRPT; ++s) {
      const float tv = tau * v[s][ii];
#pragma unroll
      for (int c = 0; c < kSW; ++c) x[s][c] -= tv * w[c];
    }
  }
  if (factor_next && blockIdx.x == 0) {
    // columns c0 .. c0 + nbn - 1 are the next panel; thread tid still owns rows j0 + tid + 1024 s
    const int nbn = col_end - c0 < kNB ? col_end - c0 : kNB;
#pragma unroll
    for (int i = 0; i < kNB; ++i) {
      if (i >= nbn) break;
      const int j = c0 + i;
      float d[kNB];
#pragma unroll
      for (int c = 0; c < kNB; ++c) {
        float a = 0.f;
        if (c >= i) {
#pragma unroll
          for (int s = 0; s < kRPT; ++s)
            if (j0 + tid + 1024 * s > j) a += x[s][i] * x[s][c];
        }
        d[c] = a;
      }
      if (tid == j - j0) {  // owner of row j (j - j0 < 2 kNB) publishes that row of the panel
#pragma unroll
        for (int c = 0; c < kNB; ++c) bc[c] = x[0][c];
      }
      block_sum_vec(d, red, red_phase);  // its barriers also publish bc
      const float x0 = bc[i];
      const float sigma = d[i];
      float tau = 0.f, vs = 0.f;
      if (sigma != 0.f) {
        const float beta = -copysignf(sqrtf(x0 * x0 + sigma), x0);
        tau = (beta - x0) / beta;
        vs = 1.0f / (x0 - beta);
      }
      if (tid == 0) { tau_p[j] = tau; vscale_p[j] = vs; }
      if (tau != 0.f) {
#pragma unroll
        for (int c = 0; c < kNB; ++c) {
          if (c <= i) continue;
          const float tw = tau * (bc[c] + vs * d[c]);
#pragma unroll
          for (int s = 0; s < kRPT; ++s) {
            const int row = j0 + tid + 1024 * s;
            if (row == j) x[s][c] -= tw;
            else if (row > j) x[s][c] -= tw * vs * x[s][i];
          }
        }
      }
      __syncthreads();  // bc is rewritten in the next round
    }
  }
#pragma unroll
  for (int s = 0; s < kRPT; ++s) {
    const int row = j0 + tid + 1024 * s;
    if (row < k) {
#pragma unroll
      for (int c = 0; c < kSW; ++c)
        if (c0 + c < col_end) X[(size_t)(c0 + c) * k + row] = x[s][c];
    }
  }
}

// Partial inner products for a 16 x 16 block on the matrix cores: lane (i = lane % 16, g = lane / 16)
// holds row i of A and row i of B; every group of 16 positions base + 16 S .. + 15 contributes
// sum_p A[i][p] B[j][p] through four v_mfma_f32_16x16x4_f32 (lane group g supplies positions
// 4 g .. 4 g + 3 of the group, the same for A and B).  This wave takes groups kq, kq + 4, ...
// Rows that do not exist (aok / bok false) count as zero.  limit - base need not be a multiple of 16,
// but every 4-float piece is entirely inside or outside [base, limit).  Eight groups are loaded
// before they are consumed, so the loop is not bound by one load latency per group.
typedef float gf4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ gf4 gram_partial(const float* __restrict__ arow, bool aok, const float* __restrict__ brow, bool bok,
                                            int base, int limit, int kq, int g) {
  gf4 acc = {0.f, 0.f, 0.f, 0.f};
  const gf4 zero = {0.f, 0.f, 0.f, 0.f};
  const int ngroups = (limit - base + 15) >> 4;
  const int nfull = (limit - base) >> 4;      // groups with all 16 positions inside
  int S = kq;
  for (; S + 28 < nfull; S += 32) {
    gf4 a[8], b[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const int pos = base + 16 * (S + 4 * u) + 4 * g;
      a[u] = *reinterpret_cast<const gf4*>(arow + pos);
      b[u] = *reinterpret_cast<const gf4*>(brow + pos);
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const gf4 au = aok ? a[u] : zero, bu = bok ? b[u] : zero;
#pragma unroll
      for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(au[e], bu[e], acc, 0, 0, 0);
    }
  }
  for (; S < ngroups; S += 4) {
    const int pos = base + 16 * S + 4 * g;
    gf4 a = zero, b = zero;
    if (pos < limit) {
      a = *reinterpret_cast<const gf4*>(arow + pos);
      b = *reinterpret_cast<const gf4*>(brow + pos);
    }
    if (!aok) a = zero;
    if (!bok) b = zero;
#pragma unroll
    for (int e = 0; e < 4; ++e) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], acc, 0, 0, 0);
  }
  return acc;
}

// ---- compact WY form of a macro panel of up to 32 reflectors ---------------------------------------
// H_0 H_1 ... H_{nb-1} = I - V T V^T with T upper triangular (T_jj = tau_j,
// T_{0:j,j} = -tau_j T_{0:j,0:j} V_{:,0:j}^T v_j).  With it the trailing matrix is updated once per 32
// reflectors, by matrix products on the matrix cores, instead of once per 8 with reductions.
typedef float wf4 __attribute__((ext_vector_type(4)));
constexpr int kWY = 32;

// Slice blockIdx.x of kWYSlices of the positions >= J0: write the reflectors of macro panel J0 as plain
// vectors into vclean (rows beyond nb are zero) and form this slice's share of S = V^T V on the
// matrix cores (left in tpart; wy_tfactor_kernel adds the shares).
constexpr int kWYSlices = 8;
__global__ __launch_bounds__(1024) void wy_gram_kernel(const RefreshGroup* __restrict__ gp, int J0, int nb) {
  const RefreshGroup& grp = *gp;
  __shared__ float stage[16 * 256];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int k = t.k;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // slice of the positions, in units of 16 so that every 16-byte piece belongs to one slice
  const int units = (k - J0 + 15) >> 4;
  const int per = (units + kWYSlices - 1) / kWYSlices;
  const int p_begin = J0 + 16 * per * blockIdx.x;
  const int p_end = min(k, p_begin + 16 * per);
  for (int j = wave; j < kWY; j += 16) {
    const int col = J0 + j;                   // reflector index = row of Zt
    const float vs = j < nb ? t.vscale[col] : 0.f;
    const float* src = t.Z + (size_t)(j < nb ? col : 0) * k;
    float* dst = t.vclean + (size_t)col * k;
    for (int pos = p_begin + 4 * lane; pos < p_end; pos += 256) {
      wf4 v = {0.f, 0.f, 0.f, 0.f};
      if (j < nb) {
        const wf4 z = *reinterpret_cast<const wf4*>(src + pos);
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = pos + e > col ? z[e] * vs : (pos + e == col ? 1.f : 0.f);
      }
      *reinterpret_cast<wf4*>(dst + pos) = v;
    }
  }
  __syncthreads();  // the rows written above are read back below by other waves of this workgroup
  {
    const int I0 = (wave & 1) * 16, Jb = ((wave >> 1) & 1) * 16, kq = wave >> 2;
    const int i = lane & 15, g = lane >> 4;
    const float* arow = t.vclean + (size_t)(J0 + I0 + i) * k;
    const float* brow = t.vclean + (size_t)(J0 + Jb + i) * k;
    wf4 acc = {0.f, 0.f, 0.f, 0.f};
    if (p_begin < p_end) acc = gram_partial(arow, true, brow, true, p_begin, p_end, kq, g);
#pragma unroll
    for (int v = 0; v < 4; ++v) stage[wave * 256 + (4 * g + v) * 16 + i] = acc[v];
  }
  __syncthreads();
  {
    const int i = tid >> 5, j = tid & 31;
    const int blk = (i >> 4) | ((j >> 4) << 1);
    float sum = 0.f;
#pragma unroll
    for (int kq = 0; kq < 4; ++kq) sum += stage[(blk + 4 * kq) * 256 + (i & 15) * 16 + (j & 15)];
    t.tpart[blockIdx.x * (kWY * kWY) + tid] = sum;
  }
}

// One workgroup per tensor: S = sum of the slices' shares (one entry per thread, so the shares arrive in
// one memory round trip), then the first 32 lanes build T column by column; lane i owns row i of T in
// registers.
__global__ __launch_bounds__(1024) void wy_tfactor_kernel(const RefreshGroup* __restrict__ gp, int J0, int nb) {
  const RefreshGroup& grp = *gp;
  __shared__ float Sm[kWY * (kWY + 1)];
  __shared__ float taus[kWY];   // fetched once: a global load inside the column loop would cost its latency 32 times
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int lane = threadIdx.x;
  if (lane < kWY) taus[lane] = lane < nb ? t.tau[J0 + lane] : 0.f;
  {
    const int e = lane;   // 1024 threads, 32 x 32 entries
    float sum = 0.f;
#pragma unroll
    for (int sl = 0; sl < kWYSlices; ++sl) sum += t.tpart[sl * (kWY * kWY) + e];
    Sm[(e >> 5) * (kWY + 1) + (e & 31)] = sum;
  }
  __syncthreads();
  if (lane < kWY) {
    const int i = lane;
    float trow[kWY];
#pragma unroll
    for (int j = 0; j < kWY; ++j) trow[j] = 0.f;
    // fully unrolled: every register index is static and column j only touches entries l < j
#pragma unroll
    for (int j = 0; j < kWY; ++j) {
      const float tau = taus[j];
      float acc = 0.f;
#pragma unroll
      for (int l = 0; l < j; ++l) acc += trow[l] * Sm[l * (kWY + 1) + j];  // trow[l] = 0 unless i <= l
      trow[j] = i == j ? tau : (i < j ? -tau * acc : 0.f);
    }
    float* out = t.tmat + (size_t)(J0 / kWY) * (kWY * kWY);
#pragma unroll
    for (int j = 0; j < kWY; ++j) out[i * kWY + j] = trow[j];
  }
}

// Apply macro panel J0 to the target (rows col_begin .. col_end-1 of the transposed storage), positions
// >= J0:  x <- x - V Tf^T (V^T x)  with Tf = T when factoring (Q_p^T x) and T^T when forming Q (Q_p x);
// in row form w = x V^T, y = w Tf, x -= y V.  Two launches over a grid of (32 target rows) x (slice of
// the positions) x (tensor), so that late macro panels, which have few target rows left, still fill the
// chip, and no workgroup has to pull more than a few hundred KB through its CU's L2 port:
//   wy_project_kernel  this slice's share of w (32 x 32) into wpart;
//   wy_update_kernel   w = sum of the shares, y = w Tf, then x -= y V on this slice of the positions.
constexpr int kWYApplySlices = 4;
__device__ __forceinline__ void wy_slice(int J0, int k, int s, int& p_begin, int& p_end) {
  const int units = (k - J0 + 63) >> 6;  // slices are whole 64-position chunks (one wave trip of the update)
  const int per = (units + kWYApplySlices - 1) / kWYApplySlices;
  p_begin = J0 + 64 * per * s;
  p_end = min(k, p_begin + 64 * per);
}

__global__ __launch_bounds__(1024) void wy_project_kernel(const RefreshGroup* __restrict__ gp, int J0, int col_begin, int col_end,
                                                          int target_is_q) {
  const RefreshGroup& grp = *gp;
  __shared__ float stage[16 * 4 * 256];  // per wave: its shares of the four 16 x 16 blocks of w
  const RefreshTensor& t = grp.t[blockIdx.z];
  const int k = t.k;
  const float* __restrict__ X = target_is_q ? t.Q : t.Z;
  const float* __restrict__ V = t.vclean + (size_t)J0 * k;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c0 = col_begin + kWY * blockIdx.x;
  int p_begin, p_end;
  wy_slice(J0, k, blockIdx.y, p_begin, p_end);
  // Wave w takes the groups of 16 positions w, w + 16, ... of the slice and, for each, one 16-byte piece
  // of target rows i and 16 + i and of reflectors i and 16 + i (lane (i = lane % 16, g = lane / 16) supplies
  // positions 4 g .. 4 g + 3 of the group): four pieces feed the four block products, where a block per
  // wave over a quarter of the slice loaded two pieces per product, in two batches.  All loads of a batch
  // (4 groups, the whole share at full slice length) leave before the first MFMA, unconditionally from
  // clamped addresses; target rows and positions that do not exist are masked to zero afterwards.
  {
    const int i = lane & 15, g = lane >> 4;
    const int xr0 = c0 + i, xr1 = c0 + 16 + i;
    const bool ok0 = xr0 < col_end, ok1 = xr1 < col_end;
    const float* x0 = X + (size_t)(ok0 ? xr0 : col_begin) * k;
    const float* x1 = X + (size_t)(ok1 ? xr1 : col_begin) * k;
    const float* v0 = V + (size_t)i * k;
    const float* v1 = V + (size_t)(16 + i) * k;
    const float m0 = ok0 ? 1.f : 0.f, m1 = ok1 ? 1.f : 0.f;
    const wf4 zero = {0.f, 0.f, 0.f, 0.f};
    wf4 a00 = zero, a01 = zero, a10 = zero, a11 = zero;  // a[I][Jb]: target rows 16 I .., reflectors 16 Jb ..
    const int ngroups = p_begin < p_end ? (p_end - p_begin + 15) >> 4 : 0;
    for (int S0 = wave; S0 < ngroups; S0 += 4 * 16) {
      wf4 px0[4], px1[4], pv0[4], pv1[4];
      float mk[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int pos = p_begin + 16 * (S0 + 16 * u) + 4 * g;
        const bool ok = pos < p_end;   // slice ends are multiples of 4: a piece is inside or outside as a whole
        const int ps = ok ? pos : p_begin;
        mk[u] = ok ? 1.f : 0.f;
        px0[u] = *reinterpret_cast<const wf4*>(x0 + ps);
        px1[u] = *reinterpret_cast<const wf4*>(x1 + ps);
        pv0[u] = *reinterpret_cast<const wf4*>(v0 + ps);
        pv1[u] = *reinterpret_cast<const wf4*>(v1 + ps);
      }
      __builtin_amdgcn_sched_barrier(0);  // all 16 loads first
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        px0[u] *= m0 * mk[u];
        px1[u] *= m1 * mk[u];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          a00 = __builtin_amdgcn_mfma_f32_16x16x4f32(px0[u][e], pv0[u][e], a00, 0, 0, 0);
          a01 = __builtin_amdgcn_mfma_f32_16x16x4f32(px0[u][e], pv1[u][e], a01, 0, 0, 0);
          a10 = __builtin_amdgcn_mfma_f32_16x16x4f32(px1[u][e], pv0[u][e], a10, 0, 0, 0);
          a11 = __builtin_amdgcn_mfma_f32_16x16x4f32(px1[u][e], pv1[u][e], a11, 0, 0, 0);
        }
      }
    }
    // block index I + 2 Jb, element (row 4 g + v, column i) of the block
#pragma unroll
    for (int v = 0; v < 4; ++v) {
      stage[(wave * 4 + 0) * 256 + (4 * g + v) * 16 + i] = a00[v];
      stage[(wave * 4 + 1) * 256 + (4 * g + v) * 16 + i] = a10[v];
      stage[(wave * 4 + 2) * 256 + (4 * g + v) * 16 + i] = a01[v];
      stage[(wave * 4 + 3) * 256 + (4 * g + v) * 16 + i] = a11[v];
    }
  }
  __syncthreads();
  {
    const int i = tid >> 5, j = tid & 31;
    const int blk = (i >> 4) | ((j >> 4) << 1);
    float sum = 0.f;
#pragma unroll
    for (int w = 0; w < 16; ++w) sum += stage[(w * 4 + blk) * 256 + (i & 15) * 16 + (j & 15)];
    t.wpart[((size_t)blockIdx.x * kWYApplySlices + blockIdx.y) * (kWY * kWY) + tid] = sum;  // entry (i, j)
  }
}

// NW = wavefronts per workgroup: the work is laid out for 16 (one entry of the 32 x 32 products per thread
// of 1024, 64 positions per wavefront and trip); with 8 every wavefront takes two shares, and the lanes
// may use up to 256 registers, which the 16 pieces in flight per trip need (under the 128 of a
// 1024-thread workgroup the scheduler issued the loads one by one, each with a wait of its own).
constexpr int kWYUpdateWaves = 8;
template <int NW>
__global__ __launch_bounds__(64 * NW) void wy_update_kernel(const RefreshGroup* __restrict__ gp, int J0, int col_begin, int col_end,
                                                            int target_is_q, int backward) {
  const RefreshGroup& grp = *gp;
  constexpr int VW = 16 / NW;
  __shared__ float Wm[kWY * (kWY + 1)];
  __shared__ float Ym[kWY * (kWY + 1)];
  __shared__ float Tf[kWY * (kWY + 1)];
  const RefreshTensor& t = grp.t[blockIdx.z];
  const int k = t.k;
  float* __restrict__ X = target_is_q ? t.Q : t.Z;
  const float* __restrict__ V = t.vclean + (size_t)J0 * k;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c0 = col_begin + kWY * blockIdx.x;
  int p_begin, p_end;
  wy_slice(J0, k, blockIdx.y, p_begin, p_end);
  if (p_begin >= p_end) return;  // uniform
#pragma unroll
  for (int sh = 0; sh < VW; ++sh) {
    const float* T = t.tmat + (size_t)(J0 / kWY) * (kWY * kWY);
    const int vt = tid + 64 * NW * sh;
    const int i = vt >> 5, j = vt & 31;
    Tf[i * (kWY + 1) + j] = backward ? T[j * kWY + i] : T[i * kWY + j];
    float sum = 0.f;
#pragma unroll
    for (int sl = 0; sl < kWYApplySlices; ++sl) sum += t.wpart[((size_t)blockIdx.x * kWYApplySlices + sl) * (kWY * kWY) + vt];
    Wm[i * (kWY + 1) + j] = sum;
  }
  __syncthreads();
#pragma unroll
  for (int sh = 0; sh < VW; ++sh) {
    const int vt = tid + 64 * NW * sh;
    const int i = vt >> 5, j = vt & 31;
    float y = 0.f;
#pragma unroll 8
    for (int l = 0; l < kWY; ++l) y += Wm[i * (kWY + 1) + l] * Tf[l * (kWY + 1) + j];
    Ym[i * (kWY + 1) + j] = y;
  }
  __syncthreads();
  // x -= y V on this slice: acc starts as x, A = -y, B = V
  {
    const int i = lane & 15, g = lane >> 4;
    float ya[2][8];
    int xrow[2][4];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
      for (int sidx = 0; sidx < 8; ++sidx) ya[h][sidx] = -Ym[(16 * h + i) * (kWY + 1) + 4 * sidx + g];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int xr = c0 + 16 * h + 4 * g + v;
        xrow[h][v] = xr < col_end ? xr : -1;
      }
    }
    // 64 positions per trip: lane (i, g) owns positions pos0 .. pos0 + 3 (one 16-byte access per row),
    // position pos0 + c belongs to MFMA column block c, so block c holds positions {n0 + 4 n + c}.
    // All loads of a trip are issued before its MFMAs.
    for (int n0 = p_begin + 64 * wave; n0 < p_end; n0 += 64 * NW) {
      const int pos0 = n0 + 4 * i;
      const bool pok = pos0 < p_end;          // slice ends are multiples of 4: a piece is inside or outside as a whole
      wf4 b[8];
      wf4 x[2][4];
      const wf4 zero = {0.f, 0.f, 0.f, 0.f};
      // All 16 loads are unconditional, from clamped addresses: a lane whose positions lie beyond the slice
      // reads the slice's first positions, a target row that does not exist is read from row c0 (always
      // valid).  Nothing is masked: in these MFMAs a lane's pieces only reach the outputs of its own
      // positions and each output row only depends on its own input row, and those outputs are not
      // stored.  Guarded loads ("inside ? load : 0") compiled to a region and a full wait per load.
      const int pos_ok = pok ? pos0 : p_begin;   // p_begin < p_end here; both are multiples of 4
#pragma unroll
      for (int sidx = 0; sidx < 8; ++sidx) b[sidx] = *reinterpret_cast<const wf4*>(V + (size_t)(4 * sidx + g) * k + pos_ok);
#pragma unroll
      for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int v = 0; v < 4; ++v) {
          const int xr = xrow[h][v] >= 0 ? xrow[h][v] : c0;
          x[h][v] = *reinterpret_cast<const wf4*>(X + (size_t)xr * k + pos_ok);
        }
      __builtin_amdgcn_sched_barrier(0);  // all 16 loads first: the scheduler would otherwise thread them through the MFMAs, a wait apiece
      (void)zero;
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        wf4 acc[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
#pragma unroll
          for (int v = 0; v < 4; ++v) acc[c][v] = x[h][v][c];
#pragma unroll
          for (int sidx = 0; sidx < 8; ++sidx) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(ya[h][sidx], b[sidx][c], acc[c], 0, 0, 0);
        }
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (xrow[h][v] >= 0 && pok) {
            const wf4 o = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
            *reinterpret_cast<wf4*>(X + (size_t)xrow[h][v] * k + pos0) = o;
          }
      }
    }
  }
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

// ---- one-sided Jacobi on the rows of Bw ----------------------------------------------------------
// Round `round` of a round-robin tournament over n = r (+1 if odd) players: pair s = 0 is
// (n-1, round); pair s > 0 is ((round + s) mod (n-1), (round - s) mod (n-1)).
__global__ __launch_bounds__(256) void jacobi_round_kernel(const RefreshGroup* __restrict__ gp, int round, int n, int sweep) {
  const RefreshGroup& grp = *gp;
  __shared__ float red[3][4];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  if (sweep > 0 && t.sweep_flag[sweep - 1] == 0) return;  // the previous sweep rotated nothing: converged
  const int s = blockIdx.x;
  int p, q;
  if (s == 0) { p = n - 1; q = round; }
  else { p = (round + s) % (n - 1); q = (round - s + (n - 1)) % (n - 1); }
  if (p >= r || q >= r) return;  // bye
  if (p > q) { const int x = p; p = q; q = x; }
  float* bp = t.Bw + (size_t)p * r;
  float* bq = t.Bw + (size_t)q * r;
  float a = 0.f, b = 0.f, c = 0.f;
  for (int i = threadIdx.x; i < r; i += 256) {
    const float x = bp[i], y = bq[i];
    a += x * x; b += y * y; c += x * y;
  }
  a = wave_sum(a); b = wave_sum(b); c = wave_sum(c);
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { red[0][wave] = a; red[1][wave] = b; red[2][wave] = c; }
  __syncthreads();
  a = red[0][0] + red[0][1] + red[0][2] + red[0][3];
  b = red[1][0] + red[1][1] + red[1][2] + red[1][3];
  c = red[2][0] + red[2][1] + red[2][2] + red[2][3];
  if (a == 0.f || b == 0.f) return;
  if (fabsf(c) <= kJacobiTol * sqrtf(a) * sqrtf(b)) return;
  const float zeta = (b - a) / (2.f * c);
  const float tt = copysignf(1.f, zeta) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta));
  const float cs = 1.f / sqrtf(1.f + tt * tt);
  const float sn = cs * tt;
  if (threadIdx.x == 0) t.sweep_flag[sweep] = 1;  // idempotent plain store, no atomics
  float* jp = t.Jt + (size_t)p * r;
  float* jq = t.Jt + (size_t)q * r;
  for (int i = threadIdx.x; i < r; i += 256) {
    const float x = bp[i], y = bq[i];
    bp[i] = cs * x - sn * y;
    bq[i] = sn * x + cs * y;
    const float u = jp[i], v = jq[i];
    jp[i] = cs * u - sn * v;
    jq[i] = sn * u + cs * v;
  }
}

// ---- block one-sided Jacobi ------------------------------------------------------------------
// The rows of Bw are cut into blocks of `b` rows.  One workgroup takes a pair of blocks (2b rows,
// whole rows, in LDS), orthogonalises those rows against each other with `kInnerSweeps` sweeps of
// the same Hestenes rotations (round-robin over the 2b rows, one row pair per wave and round),
// accumulates the 2b x 2b product of the rotations, writes the rows back and applies the product
// to the matching rows of Jt.  Block pairs of one launch are disjoint (round-robin over the
// blocks), so a sweep over all pairs of rows costs (blocks - 1) launches that each read and write
// Bw and Jt once, instead of (r - 1) launches.
constexpr int kInnerSweeps = 1;
#ifndef GALORE_GRAM_INNER
#define GALORE_GRAM_INNER 1
#endif
constexpr int kGramInnerSweeps = GALORE_GRAM_INNER;  // inner sweeps of the Gram-maintained block round
constexpr int kJacobiMaxR = 1280;  // longest row the register-resident inner loop is unrolled for (5 float4 per lane and row)

typedef float jf4 __attribute__((ext_vector_type(4)));

template <int B>  // rows per block (16 or 8); 2B rows are orthogonalised against each other
__global__ __launch_bounds__(1024) void jacobi_block_round_kernel(const RefreshGroup* __restrict__ gp, int round, int nplayers, int sweep) {
  const RefreshGroup& grp = *gp;
  constexpr int R2 = 2 * B;
  extern __shared__ __align__(16) float jsm[];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  if (sweep > 0 && t.sweep_flag[sweep - 1] == 0) return;  // converged
  const int nblocks = (r + B - 1) / B;
  const int s = blockIdx.x;
  int bi, bj;
  if (s == 0) { bi = nplayers - 1; bj = round; }
  else { bi = (round + s) % (nplayers - 1); bj = (round - s + (nplayers - 1)) % (nplayers - 1); }
  if (bi > bj) { const int x = bi; bi = bj; bj = x; }
  if (bi >= nblocks) return;                // both absent
  const int rp = (r + 3) & ~3;               // LDS row pitch: rows padded with zeros to a multiple of 4
  const int nv = rp >> 2;                    // float4 per row
  float* X = jsm;                            // [2B][rp]
  float* RotT = jsm + (size_t)R2 * rp;       // [2B][2B], RotT[j][i] = Rot[i][j]
  __shared__ int rotated;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // local row ls -> row of Bw, or -1 when the row does not exist (ragged last block, bye block)
  auto grow = [&](int ls) {
    const int g = ls < B ? bi * B + ls : bj * B + (ls - B);
    return ((ls < B || bj < nblocks) && g < r) ? g : -1;
  };
  const bool vec_ok = (r & 3) == 0;          // global rows are 16-byte aligned

  // each wave moves rows wave, wave + 16, ... with 16-byte accesses
  for (int ls = wave; ls < R2; ls += 16) {
    const int g = grow(ls);
    jf4* dst = reinterpret_cast<jf4*>(X + (size_t)ls * rp);
    if (g >= 0 && vec_ok) {
      const jf4* src = reinterpret_cast<const jf4*>(t.Bw + (size_t)g * r);
      for (int e = lane; e < nv; e += 64) dst[e] = src[e];
    } else {
      for (int e = lane; e < rp; e += 64) X[(size_t)ls * rp + e] = (g >= 0 && e < r) ? t.Bw[(size_t)g * r + e] : 0.f;
    }
  }
  for (int e = tid; e < R2 * R2; e += 1024) RotT[e] = ((e / R2) == (e % R2)) ? 1.f : 0.f;
  if (tid == 0) rotated = 0;
  __syncthreads();

  constexpr int NV = kJacobiMaxR / 256;      // float4 per lane per row, upper bound
  const bool row_ok = wave < B;
  for (int isw = 0; isw < kInnerSweeps; ++isw)
    for (int ir = 0; ir < R2 - 1; ++ir) {
      if (row_ok) {
        int p, q;
        if (wave == 0) { p = R2 - 1; q = ir; }
        else { p = (ir + wave) % (R2 - 1); q = (ir + (R2 - 1) - wave) % (R2 - 1); }
        if (p > q) { const int x = p; p = q; q = x; }
        if (grow(p) >= 0 && grow(q) >= 0) {          // wave-uniform
          jf4* xp = reinterpret_cast<jf4*>(X + (size_t)p * rp);
          jf4* xq = reinterpret_cast<jf4*>(X + (size_t)q * rp);
          jf4 u[NV], v[NV];
          float a = 0.f, bb = 0.f, c = 0.f;
#pragma unroll
          for (int i = 0; i < NV; ++i) {
            const int e = lane + 64 * i;
            if (e < nv) { u[i] = xp[e]; v[i] = xq[e]; }
            else { u[i] = jf4{0.f, 0.f, 0.f, 0.f}; v[i] = u[i]; }
#pragma unroll
            for (int k = 0; k < 4; ++k) { a += u[i][k] * u[i][k]; bb += v[i][k] * v[i][k]; c += u[i][k] * v[i][k]; }
          }
          a = wave_sum(a); bb = wave_sum(bb); c = wave_sum(c);
          if (a != 0.f && bb != 0.f && c * c > (kJacobiTol * kJacobiTol) * a * bb) {
            const float zeta = (bb - a) / (2.f * c);
            const float tt = copysignf(1.f, zeta) / (fabsf(zeta) + sqrtf(1.f + zeta * zeta));
            const float cs = 1.f / sqrtf(1.f + tt * tt);
            const float sn = cs * tt;
#pragma unroll
            for (int i = 0; i < NV; ++i) {
              const int e = lane + 64 * i;
              if (e < nv) {
                xp[e] = cs * u[i] - sn * v[i];
                xq[e] = sn * u[i] + cs * v[i];
              }
            }
            if (lane < R2) {  // rows p, q of Rot = columns p, q of RotT
              const float uu = RotT[lane * R2 + p], vv = RotT[lane * R2 + q];
              RotT[lane * R2 + p] = cs * uu - sn * vv;
              RotT[lane * R2 + q] = sn * uu + cs * vv;
            }
            if (lane == 0) rotated = 1;
          }
        }
      }
      __syncthreads();
    }

  if (rotated == 0) return;  // nothing changed: leave Bw, Jt and the sweep flag alone (uniform)
  if (tid == 0) t.sweep_flag[sweep] = 1;  // idempotent plain store, no atomics
  for (int ls = wave; ls < R2; ls += 16) {
    const int g = grow(ls);
    if (g < 0) continue;
    const jf4* src = reinterpret_cast<const jf4*>(X + (size_t)ls * rp);
    if (vec_ok) {
      jf4* dst = reinterpret_cast<jf4*>(t.Bw + (size_t)g * r);
      for (int e = lane; e < nv; e += 64) dst[e] = src[e];
    } else {
      for (int e = lane; e < r; e += 64) t.Bw[(size_t)g * r + e] = X[(size_t)ls * rp + e];
    }
  }
  // Jt rows <- Rot * Jt rows, one column per thread; RotT[j][:] is read as broadcast float4
  int gr[R2];
#pragma unroll
  for (int j = 0; j < R2; ++j) gr[j] = grow(j);
  for (int c = tid; c < r; c += 1024) {
    float acc[R2];
#pragma unroll
    for (int i = 0; i < R2; ++i) acc[i] = 0.f;
#pragma unroll 4
    for (int j = 0; j < R2; ++j) {
      if (gr[j] < 0) continue;
      const float x = t.Jt[(size_t)gr[j] * r + c];
      const jf4* rt = reinterpret_cast<const jf4*>(RotT + j * R2);
#pragma unroll
      for (int i4 = 0; i4 < R2 / 4; ++i4) {
        const jf4 w = rt[i4];
#pragma unroll
        for (int k = 0; k < 4; ++k) acc[4 * i4 + k] += w[k] * x;
      }
    }
#pragma unroll
    for (int i = 0; i < R2; ++i)
      if (gr[i] >= 0) t.Jt[(size_t)gr[i] * r + c] = acc[i];
  }
}

// Block round on the Gram matrix.  The 32 rows of a block pair are never staged in LDS:
//   1. G = X X^T (32 x 32) is formed on the matrix cores (v_mfma_f32_16x16x4_f32) straight from
//      global memory;
//   2. one inner sweep (31 rounds of 16 disjoint row pairs) works on G alone: every rotation reads
//      its three inner products from G, the 16 rotations of a round update it together as
//      G <- J^T G J (one entry per thread) and are accumulated into the 32 x 32 product Rot;
//   3. X <- Rot X and the matching rows of the eigenvector matrix Jt <- Rot Jt are two small
//      matrix products on the matrix cores, 16 columns per wave at a time, in place.
// Needs r % 4 == 0 (16-byte row segments); no limit on r.
typedef float jf4m __attribute__((ext_vector_type(4)));
constexpr int kGramB = 16, kGramR2 = 32;
constexpr int kGramSlices = 8;  // column slices of the Gram phase of the block round

// Y (32 rows picked by rows[], length r) <- Rot Y, in place.  rot[h][s] = Rot[16 h + i][4 s + g]
// for lane (i = lane % 16, g = lane / 16).  A wave owns whole columns, so it reads all 32 inputs
// of a column before it writes any.
__device__ __forceinline__ void gram_apply_rotation(float* __restrict__ Y, int r, const int (&rows)[8], const int (&out_rows)[2][4],
                                                    const float (&rot)[2][8], int wave, int lane, int nwaves) {
  const int j = lane & 15;
  // 64 columns per trip: lane (j, g) owns columns col0 .. col0 + 3 (one 16-byte access per row), column
  // col0 + c belongs to MFMA column block c.  r is a multiple of 4, so a piece is inside or outside as
  // a whole.  All loads of a trip are issued before its MFMAs.
  const jf4m zero = {0.f, 0.f, 0.f, 0.f};
  for (int n0 = 64 * wave; n0 < r; n0 += 64 * nwaves) {
    const int col0 = n0 + 4 * j;
    const bool cok = col0 < r;
    jf4m b[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) b[s] = (rows[s] >= 0 && cok) ? *reinterpret_cast<const jf4m*>(Y + (size_t)rows[s] * r + col0) : zero;
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      jf4m acc[4];
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        acc[c] = zero;
#pragma unroll
        for (int s = 0; s < 8; ++s) acc[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(rot[h][s], b[s][c], acc[c], 0, 0, 0);
      }
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (out_rows[h][v] >= 0 && cok) {
          const jf4m o = {acc[0][v], acc[1][v], acc[2][v], acc[3][v]};
          *reinterpret_cast<jf4m*>(Y + (size_t)out_rows[h][v] * r + col0) = o;
        }
    }
  }
}

// NW = wavefronts per workgroup.  The work is laid out in 16 shares (two Gram rows per share and inner
// round, one entry per lane); a wavefront takes 16 / NW of them and 16 / NW workgroups fit a CU (<= 128
// registers per lane).  An inner round is bound by latency (one LDS round trip, the reciprocal / square
// root chain, one barrier), so fewer wavefronts cost little.  Measured when an inner round still took
// two barriers, per 7B layer set: a refresh alone 84.0 / 84.2 / 90.6 ms with NW = 16 / 8 / 4; three
// refreshes in flight (the launches of this kernel then outnumber the CUs, and the memory phases of one
// workgroup overlap with the inner rounds of its neighbours on the CU) 53.3 / 50.8 / 48.9 ms.  Hence 8
// alone and 4 when crowded.
template <int NW>
__global__ __launch_bounds__(64 * NW, 16 / NW) void jacobi_gram_round_kernel(const RefreshGroup* __restrict__ gp, int round, int nplayers, int sweep) {
  const RefreshGroup& grp = *gp;
  constexpr int B = kGramB, R2 = kGramR2, GP = R2 + 1;
  constexpr int VW = 16 / NW;  // shares ("virtual wavefronts") per wavefront
  __shared__ float Gm[2][R2 * GP];
  __shared__ float Rot[R2 * GP];             // Rot[i][k]: new row i = sum_k Rot[i][k] old row k
  __shared__ float stage[kGramSlices * 3 * 256];  // per column slice: the partial blocks (0,0), (0,1), (1,1), 16 x 16 each; later the second buffer of Rot
  static_assert(kGramSlices * 3 * 256 >= R2 * GP, "the staging area doubles as the second rotation buffer");
  __shared__ int rotated;      // some rotation was applied: Bw and Jt have to be updated
  __shared__ int significant;  // some rotation was above the stopping level: another sweep is due
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  if (sweep > 0 && t.sweep_flag[sweep - 1] == 0) return;  // converged
  const int nblocks = (r + B - 1) / B;
  const int s = blockIdx.x;
  int bi, bj;
  if (s == 0) { bi = nplayers - 1; bj = round; }
  else { bi = (round + s) % (nplayers - 1); bj = (round - s + (nplayers - 1)) % (nplayers - 1); }
  if (bi > bj) { const int x = bi; bi = bj; bj = x; }
  if (bi >= nblocks) return;                // both absent
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // local row ls -> row of Bw, or -1 when the row does not exist (ragged last block, bye block)
  auto grow = [&](int ls) {
    const int g = ls < B ? bi * B + ls : bj * B + (ls - B);
    return ((ls < B || bj < nblocks) && g < r) ? g : -1;
  };

  // 1. Gram matrix.  The columns are dealt in groups of 16 to kGramSlices slices (group S belongs to
  // slice S mod kGramSlices; the number of slices is fixed so that the result does not depend on NW).  A
  // wavefront takes whole slices: for each it loads, per group, one 16-byte piece of row i and one of row
  // 16 + i (MFMA operand lane (i = lane % 16, g = lane / 16) supplies columns 4 g .. 4 g + 3 of the group) and
  // feeds three block products with them: (0,0), (0,1) and (1,1); block (1,0) is the transpose of (0,1).
  // All loads of a slice (8 groups at r = 1024) are in flight together: one exposed memory round trip
  // where block-by-block products of a quarter of the columns each needed four, for half the bytes.
  {
    const int i = lane & 15, g = lane >> 4;
    const int g0 = grow(i), g1 = grow(16 + i);
    const float* x0 = t.Bw + (size_t)(g0 >= 0 ? g0 : 0) * r;
    const float* x1 = t.Bw + (size_t)(g1 >= 0 ? g1 : 0) * r;
    const float m0 = g0 >= 0 ? 1.f : 0.f, m1 = g1 >= 0 ? 1.f : 0.f;   // rows that do not exist count as zero
    const int ngroups = (r + 15) >> 4;
    const jf4m zero = {0.f, 0.f, 0.f, 0.f};
    for (int sl = wave; sl < kGramSlices; sl += NW) {
      jf4m a00 = zero, a01 = zero, a11 = zero;
      for (int S0 = sl; S0 < ngroups; S0 += 8 * kGramSlices) {
        jf4m p0[8], p1[8];
        float msk0[8], msk1[8];
        // unconditional loads from clamped addresses, masked by arithmetic (the matrix is finite wherever
        // the gradient is): a guarded load would cost a branch and a wait of its own
#pragma unroll
        for (int u = 0; u < 8; ++u) {
          const int pos = 16 * (S0 + kGramSlices * u) + 4 * g;
          const bool ok = pos < r;   // r is a multiple of 4: a piece is inside or outside as a whole
          const int ps = ok ? pos : 0;
          const float mk = ok ? 1.f : 0.f;
          p0[u] = *reinterpret_cast<const jf4m*>(x0 + ps);
          p1[u] = *reinterpret_cast<const jf4m*>(x1 + ps);
          msk0[u] = m0 * mk; msk1[u] = m1 * mk;
        }
        __builtin_amdgcn_sched_barrier(0);  // all 16 loads first: the scheduler would otherwise thread them through the MFMAs, a wait apiece
#pragma unroll
        for (int u = 0; u < 8; ++u) { p0[u] *= msk0[u]; p1[u] *= msk1[u]; }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            a00 = __builtin_amdgcn_mfma_f32_16x16x4f32(p0[u][e], p0[u][e], a00, 0, 0, 0);
            a01 = __builtin_amdgcn_mfma_f32_16x16x4f32(p0[u][e], p1[u][e], a01, 0, 0, 0);
            a11 = __builtin_amdgcn_mfma_f32_16x16x4f32(p1[u][e], p1[u][e], a11, 0, 0, 0);
          }
      }
      // element (row 4 g + v, column i) of each block
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        stage[(sl * 3 + 0) * 256 + (4 * g + v) * 16 + i] = a00[v];
        stage[(sl * 3 + 1) * 256 + (4 * g + v) * 16 + i] = a01[v];
        stage[(sl * 3 + 2) * 256 + (4 * g + v) * 16 + i] = a11[v];
      }
    }
  }
  if (tid == 0) { rotated = 0; significant = 0; }
  __syncthreads();
#pragma unroll
  for (int sh = 0; sh < VW; ++sh) {
    const int vt = tid + 64 * NW * sh;
    const int i = vt >> 5, j = vt & 31;
    // entry (i, j) lives in block (i / 16, j / 16); the lower-left block is read from the upper-right one, transposed
    const int bI = i >> 4, bJ = j >> 4;
    const int b3 = bI == bJ ? 2 * bI : 1;
    const int rr = (bI > bJ ? j : i) & 15, cc = (bI > bJ ? i : j) & 15;
    float sum = 0.f;
#pragma unroll
    for (int sl = 0; sl < kGramSlices; ++sl) sum += stage[(sl * 3 + b3) * 256 + rr * 16 + cc];
    Gm[0][i * GP + j] = sum;
    Rot[i * GP + j] = i == j ? 1.f : 0.f;
  }
  __syncthreads();

  // 2. inner sweeps on the Gram matrix.  One barrier and one LDS round trip per inner round: the pairing
  // of a round is arithmetic (mate()), so every lane derives the rotation of the pair that holds its
  // column j from three Gram entries by itself (the 32 columns of a wavefront cover all 16 pairs; the
  // lanes of a pair read the same entries in the same order, so they agree to the bit), the two rows a
  // wavefront updates per share take theirs from the lanes whose column has that number, and G and the
  // accumulated rotation are both updated entry by entry from one buffer into the other.
  int cur = 0;
  // Round 0 of a sweep pairs every block exactly once: there the inner sweep covers all pairs of the
  // 32 rows (31 rounds), which also rotates the pairs INSIDE each block once per sweep.  The other
  // rounds only need the 16 x 16 pairs between the two blocks: 16 rounds of (i, 16 + (i + ir) % 16).
  const int j = lane & 31;
  const unsigned exist = (unsigned)__ballot(grow(lane & 31) >= 0);  // bit x: local row x exists
  const int wave_u = __builtin_amdgcn_readfirstlane(wave);
  const bool upper = lane >= 32;
  // the two pairings are compiled apart (the choice is uniform), so each inner loop carries only its own index arithmetic
  auto inner_sweeps = [&](auto all_pairs_t) {
  constexpr bool all_pairs = decltype(all_pairs_t)::value;
  constexpr int inner_rounds = all_pairs ? R2 - 1 : B;
  for (int isw = 0; isw < kGramInnerSweeps; ++isw)
    for (int ir = 0; ir < inner_rounds; ++ir) {
      const float* G = Gm[cur];
      float* Gn = Gm[cur ^ 1];
      const float* Rc = cur ? stage : Rot;   // the staging area of the Gram phase is free by now
      float* Rn = cur ? Rot : stage;
      // the row that row x is paired with in this inner round (selects only: no divergent branches)
      auto mate = [&](int x) {
        // round robin of 32 players: row 31 stays, rows with p + q = 2 ir (mod 31) meet
        int y = 2 * ir - x;
        y += y < 0 ? R2 - 1 : 0;
        y -= y >= R2 - 1 ? R2 - 1 : 0;
        y = x == ir ? R2 - 1 : y;
        y = x == R2 - 1 ? ir : y;
        const int z = x < B ? B + ((x + ir) & (B - 1)) : ((x - B - ir) & (B - 1));
        if constexpr (all_pairs) return y;
        else return z;
      };
      const int pj = mate(j);
      const int p = j < pj ? j : pj, q = j < pj ? pj : j;
      // every LDS read of the round is issued here, ahead of the arithmetic: one round trip
      const float a = G[p * GP + p], bb = G[q * GP + q], c = G[p * GP + q];
      float gij[VW], gipj[VW], gpij[VW], gpipj[VW], rij[VW], rpij[VW];
#pragma unroll
      for (int sh = 0; sh < VW; ++sh) {
        const int i = 2 * (wave_u + NW * sh) + (upper ? 1 : 0);  // lanes 0 .. 31 update row i0, lanes 32 .. 63 row i0 + 1
        const int pi = mate(i);
        gij[sh] = G[i * GP + j]; gipj[sh] = G[i * GP + pj]; gpij[sh] = G[pi * GP + j]; gpipj[sh] = G[pi * GP + pj];
        rij[sh] = Rc[i * GP + j]; rpij[sh] = Rc[pi * GP + j];
      }
      __builtin_amdgcn_sched_barrier(0);
      const bool rot = ((exist >> p) & (exist >> q) & 1u) != 0 && a > 0.f && bb > 0.f && c * c > (kJacobiTol * kJacobiTol) * a * bb;
      // hardware reciprocal / square-root approximations (1 ulp): a rotation with c^2 + s^2 = 1 to
      // within a few ulps is all that is needed, and this chain is the latency of every inner round.
      // Computed by every lane and selected afterwards (a pair that is not rotated may divide by zero).
      const float zeta = (bb - a) * __builtin_amdgcn_rcpf(2.f * c);
      const float tt = copysignf(1.f, zeta) * __builtin_amdgcn_rcpf(fabsf(zeta) + __builtin_amdgcn_sqrtf(1.f + zeta * zeta));
      const float cs0 = __builtin_amdgcn_rsqf(1.f + tt * tt);
      const float cs = rot ? cs0 : 1.f, sn = rot ? cs0 * tt : 0.f;
      // new row x = alpha_x * row x + beta_x * row mate(x): (cs, -sn) for the lower row of a pair, (cs, sn) for the upper
      const float aj = cs, bj2 = j == p ? -sn : sn;
      if (wave == 0 && rot) {  // same value from every lane that writes
        rotated = 1;
        if (c * c > (kJacobiStopTol * kJacobiStopTol) * a * bb) significant = 1;
      }
#pragma unroll
      for (int sh = 0; sh < VW; ++sh) {
        const int i0 = 2 * (wave_u + NW * sh);
        const float al0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(aj), i0));
        const float al1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(aj), i0 + 1));
        const float be0 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bj2), i0));
        const float be1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(bj2), i0 + 1));
        const int i = i0 + (upper ? 1 : 0);
        const float ai = upper ? al1 : al0, bi2 = upper ? be1 : be0;
        Gn[i * GP + j] = ai * (aj * gij[sh] + bj2 * gipj[sh]) + bi2 * (aj * gpij[sh] + bj2 * gpipj[sh]);
        Rn[i * GP + j] = ai * rij[sh] + bi2 * rpij[sh];
      }
      __syncthreads();
      cur ^= 1;
    }
  };
  if (round == 0) inner_sweeps(std::true_type{});
  else inner_sweeps(std::false_type{});

  if (rotated == 0) return;  // nothing changed: leave Bw, Jt and the sweep flag alone (uniform)
  if (tid == 0 && significant) t.sweep_flag[sweep] = 1;  // idempotent plain store, no atomics

  // 3. apply the accumulated rotation to the rows of Bw and of Jt
  {
    const int i = lane & 15, g = lane >> 4;
    const float* Rf = cur ? stage : Rot;
    float rot[2][8];
    int rows[8], out_rows[2][4];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int sidx = 0; sidx < 8; ++sidx) rot[h][sidx] = Rf[(16 * h + i) * GP + 4 * sidx + g];
#pragma unroll
    for (int sidx = 0; sidx < 8; ++sidx) rows[sidx] = grow(4 * sidx + g);
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
      for (int v = 0; v < 4; ++v) out_rows[h][v] = grow(16 * h + 4 * g + v);
    gram_apply_rotation(t.Bw, r, rows, out_rows, rot, wave, lane, NW);
    gram_apply_rotation(t.Jt, r, rows, out_rows, rot, wave, lane, NW);
  }
}

// lambda_i = |row i of Bw| ; order[i] = number of rows that come before row i when sorted by
// decreasing lambda (ties: lower index first).  The thousands of fp32 rotations let the length
// of each accumulated eigenvector drift by a few 1e-6; tau[i] (free by now) gets 1 / |row i of Jt|
// so the vectors are rescaled to unit length when they are copied out.
__global__ __launch_bounds__(256) void ritz_values_kernel(const RefreshGroup grp) {
  __shared__ float red[2][4];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r, i = blockIdx.x;
  float a = 0.f, b = 0.f;
  for (int c = threadIdx.x; c < r; c += 256) {
    const float x = t.Bw[(size_t)i * r + c], y = t.Jt[(size_t)i * r + c];
    a += x * x; b += y * y;
  }
  a = wave_sum(a); b = wave_sum(b);
  if ((threadIdx.x & 63) == 0) { red[0][threadIdx.x >> 6] = a; red[1][threadIdx.x >> 6] = b; }
  __syncthreads();
  if (threadIdx.x == 0) {
    t.lambda[i] = sqrtf(red[0][0] + red[0][1] + red[0][2] + red[0][3]);
    t.tau[i] = 1.0f / sqrtf(red[1][0] + red[1][1] + red[1][2] + red[1][3]);
  }
}

__global__ __launch_bounds__(256) void ritz_order_kernel(const RefreshGroup grp) {
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < r; i += gridDim.x * blockDim.x) {
    const float li = t.lambda[i];
    int before = 0;
    for (int j = 0; j < r; ++j) {
      const float lj = t.lambda[j];
      before += (lj > li || (lj == li && j < i)) ? 1 : 0;
    }
    t.order[i] = before;
  }
}

// St[order[i]][:] = Jt[i][:] / |Jt[i]|
__global__ __launch_bounds__(256) void ritz_vectors_kernel(const RefreshGroup grp) {
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  const int64_t count = (int64_t)r * r;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
    const int i = (int)(e / r), kk = (int)(e % r);
    t.S[(size_t)t.order[i] * r + kk] = t.Jt[e] * t.tau[i];
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

  bool wy_ok = true;  // compact WY path: 16-byte pieces of the transposed rows
  for (int i = 0; i < n; ++i) wy_ok = wy_ok && grp.t[i].k % 4 == 0;
  for (int it = 0; it < iters; ++it) {
    GALORE_RETURN_IF(gemm_f32(0));
    // Householder QR of Z
    if (kmax <= 1024 * kRPT) {
      // blocked: factor a panel of kNB columns, apply its reflectors to the trailing columns
      if (wy_ok) {
        // two levels: inside a macro panel of 32 columns the 8-column panels update only the macro
        // panel; the rest of the matrix is updated once per macro panel in compact WY form
        for (int J0 = 0; J0 < r; J0 += kWY) {
          const int nb32 = r - J0 < kWY ? r - J0 : kWY;
          for (int j0 = J0; j0 < J0 + nb32; j0 += kNB) {
            const int nb = J0 + nb32 - j0 < kNB ? J0 + nb32 - j0 : kNB;
            // the first panel of a macro panel has its own launch; the others are factored by workgroup 0
            // of the previous panel's update, which holds their columns in registers anyway
            if (j0 == J0) hipLaunchKernelGGL(householder_panel_kernel, dim3(1, n), dim3(1024), 0, stream, dgrp, j0, nb);
            const int inner = J0 + nb32 - (j0 + nb);
            if (inner > 0)
              hipLaunchKernelGGL(householder_block_apply_kernel, dim3((inner + kSW - 1) / kSW, n), dim3(1024), 0, stream, dgrp,
                                 j0, nb, j0 + nb, 0, 0, J0 + nb32, 1);
          }
          hipLaunchKernelGGL(wy_gram_kernel, dim3(kWYSlices, n), dim3(1024), 0, stream, dgrp, J0, nb32);
          hipLaunchKernelGGL(wy_tfactor_kernel, dim3(1, n), dim3(kWY * kWY), 0, stream, dgrp, J0, nb32);
          const int trailing = r - (J0 + nb32);
          if (trailing > 0) {
            const dim3 grid((trailing + kWY - 1) / kWY, kWYApplySlices, n);
            hipLaunchKernelGGL(wy_project_kernel, grid, dim3(1024), 0, stream, dgrp, J0, J0 + nb32, r, 0);
            hipLaunchKernelGGL(wy_update_kernel<kWYUpdateWaves>, grid, dim3(64 * kWYUpdateWaves), 0, stream, dgrp, J0, J0 + nb32, r, 0, 0);
          }
        }
        GALORE_RETURN_IF(hipGetLastError());
        hipLaunchKernelGGL(identity_fill_kernel, fill_grid, dim3(256), 0, stream, dgrp, 0);
        for (int J0 = (r - 1) / kWY * kWY; J0 >= 0; J0 -= kWY) {
          const dim3 grid((r - J0 + kWY - 1) / kWY, kWYApplySlices, n);
          hipLaunchKernelGGL(wy_project_kernel, grid, dim3(1024), 0, stream, dgrp, J0, J0, r, 1);
          hipLaunchKernelGGL(wy_update_kernel<kWYUpdateWaves>, grid, dim3(64 * kWYUpdateWaves), 0, stream, dgrp, J0, J0, r, 1, 1);
        }
        GALORE_RETURN_IF(hipGetLastError());
        continue;
      }
      for (int j0 = 0; j0 < r; j0 += kNB) {
        const int nb = r - j0 < kNB ? r - j0 : kNB;
        hipLaunchKernelGGL(householder_panel_kernel, dim3(1, n), dim3(1024), 0, stream, dgrp, j0, nb);
        const int ncols = r - (j0 + nb);
        if (ncols > 0)
          hipLaunchKernelGGL(householder_block_apply_kernel, dim3((ncols + kSW - 1) / kSW, n), dim3(1024), 0, stream, dgrp,
                             j0, nb, j0 + nb, 0, 0, r, 0);
      }
      GALORE_RETURN_IF(hipGetLastError());
      hipLaunchKernelGGL(identity_fill_kernel, fill_grid, dim3(256), 0, stream, dgrp, 0);
      const int last = (r - 1) / kNB * kNB;
      for (int j0 = last; j0 >= 0; j0 -= kNB) {
        const int nb = r - j0 < kNB ? r - j0 : kNB;
        hipLaunchKernelGGL(householder_block_apply_kernel, dim3((r - j0 + kSW - 1) / kSW, n), dim3(1024), 0, stream, dgrp,
                           j0, nb, j0, 1, 1, r, 0);
      }
      GALORE_RETURN_IF(hipGetLastError());
    } else {
      // tall fallback (short side beyond the register-resident panel): reflector by reflector
      for (int j = 0; j < r; ++j) {
        const int ncols = r - (j + 1);
        const dim3 grid(ncols > 0 ? (ncols + 31) / 32 : 1, n);
        hipLaunchKernelGGL(householder_strip_kernel<true>, grid, dim3(1024), 0, stream, dgrp, j, j + 1, 0);
      }
      GALORE_RETURN_IF(hipGetLastError());
      hipLaunchKernelGGL(identity_fill_kernel, fill_grid, dim3(256), 0, stream, dgrp, 0);
      for (int j = r - 1; j >= 0; --j) {
        const dim3 grid((r - j + 31) / 32, n);
        hipLaunchKernelGGL(householder_strip_kernel<false>, grid, dim3(1024), 0, stream, dgrp, j, j, 1);
      }
      GALORE_RETURN_IF(hipGetLastError());
    }
  }

  // Rayleigh-Ritz
  GALORE_RETURN_IF(gemm_f32(0));
  GALORE_RETURN_IF(gemm_f32(1));
  hipLaunchKernelGGL(identity_fill_kernel, dim3(blocks_for((int64_t)r * r, 256 * 8, 1024), n), dim3(256), 0, stream, dgrp, 1);
  // rows per block so that two blocks of whole rows (plus the 2b x 2b rotation product) fit in LDS
  int jb = 0;
  for (int cand : {16, 8})
    if (jb == 0 && (size_t)2 * cand * ((r + 3) & ~3) * 4 + (size_t)4 * cand * cand * 4 <= 150 * 1024) jb = cand;
  if (r > kJacobiMaxR) jb = 0;  // the inner loop keeps a row pair in registers, unrolled for rows up to kJacobiMaxR
  const bool use_gram = r % 4 == 0 && r >= 4;  // the Gram-matrix kernel stages no rows: any such r
  if (use_gram) jb = kGramB;
  if (r > 1 && jb > 0) {
    const size_t smem = (size_t)2 * jb * ((r + 3) & ~3) * 4 + (size_t)4 * jb * jb * 4;
    static bool attr_set = false;
    if (!attr_set) {
      GALORE_RETURN_IF(hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi_block_round_kernel<16>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
      GALORE_RETURN_IF(hipFuncSetAttribute(reinterpret_cast<const void*>(jacobi_block_round_kernel<8>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
      attr_set = true;
    }
    const int nblocks = (r + jb - 1) / jb;
    const int players = (nblocks % 2 == 0) ? nblocks : nblocks + 1;   // >= 2
    for (int sweep = 0; sweep < kJacobiSweeps; ++sweep)
      for (int round = 0; round < players - 1; ++round)
        if (use_gram)
          if (crowded) hipLaunchKernelGGL(jacobi_gram_round_kernel<4>, dim3(players / 2, n), dim3(256), 0, stream, dgrp, round, players, sweep);
          else hipLaunchKernelGGL(jacobi_gram_round_kernel<8>, dim3(players / 2, n), dim3(512), 0, stream, dgrp, round, players, sweep);
        else if (jb == 16)
          hipLaunchKernelGGL(jacobi_block_round_kernel<16>, dim3(players / 2, n), dim3(1024), smem, stream, dgrp, round, players, sweep);
        else
          hipLaunchKernelGGL(jacobi_block_round_kernel<8>, dim3(players / 2, n), dim3(1024), smem, stream, dgrp, round, players, sweep);
  } else if (r > 1) {  // rows too long for LDS: one launch per round of row pairs
    const int players = (r % 2 == 0) ? r : r + 1;
    for (int sweep = 0; sweep < kJacobiSweeps; ++sweep)
      for (int round = 0; round < players - 1; ++round)
        hipLaunchKernelGGL(jacobi_round_kernel, dim3(players / 2, n), dim3(256), 0, stream, dgrp, round, players, sweep);
  }
  GALORE_RETURN_IF(hipGetLastError());
  hipLaunchKernelGGL(ritz_values_kernel, dim3(r, n), dim3(256), 0, stream, grp);
  hipLaunchKernelGGL(ritz_order_kernel, dim3((r + 255) / 256, n), dim3(256), 0, stream, grp);
  hipLaunchKernelGGL(ritz_vectors_kernel, dim3(blocks_for((int64_t)r * r, 256 * 8, 1024), n), dim3(256), 0, stream, grp);
  GALORE_RETURN_IF(hipGetLastError());
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
