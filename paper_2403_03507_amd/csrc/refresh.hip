// Subspace refresh (Algorithm 2, refresh branch; Sec. 3.3 SVD equation for P_t, Q_t).
//
// The paper takes P = U[:, :r] from an SVD of the gradient.  Here the leading singular
// vectors of the short side are computed from the Gram matrix C = G G^T (or G^T G), whose
// eigenvectors they are, by blocked orthogonal iteration:
//     Q <- Gaussian (k x r);  repeat iters times: Z = C Q ; Q = qr(Z).Q
// followed by a Rayleigh-Ritz step B = Q^T C Q = S L S^T, P = Q S, columns ordered by
// decreasing L, each column signed so that its largest-magnitude entry is positive.
//   * Gram and the tall GEMMs run on the grouped MFMA GEMM.
//   * QR is Householder, one reflector per launch: every block rebuilds the reflector of
//     column j with a wavefront (DPP shuffle) + LDS reduction and applies it to its own strip
//     of 32 trailing columns; Q is then formed by applying the reflectors to [I; 0] backwards.
//   * The r x r eigenproblem is solved by one-sided (Hestenes) Jacobi on the rows of B with
//     round-robin pair ordering, one launch per round of r/2 disjoint pairs.
// All tensors of a group advance in lock-step (blockIdx.y = tensor), nothing syncs the host,
// iteration counts are fixed, and no atomics are used, so results are reproducible bit for bit.
#include "refresh.hpp"

namespace galore {

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

constexpr int kJacobiSweeps = 10;
constexpr float kJacobiTol = 1e-7f;

struct RefreshTensor {
  float* C;      // k x k Gram matrix
  float* Q;      // k x r iteration block
  float* Z;      // k x r product block / factored reflectors / fp32 projector
  float* Bw;     // r x r Rayleigh-Ritz matrix, rotated in place
  float* Jt;     // r x r accumulated rotations (rows = eigenvectors)
  float* S;      // r x r eigenvectors as columns, ordered
  float* tau;    // r
  float* vscale; // r
  float* lambda; // r
  int32_t* order;// r : order[i] = output column of eigenvector i
  void* proj;    // output, k x r, ld ldp
  int32_t k;
  int32_t ldp;
  uint64_t seed;
};

struct RefreshGroup {
  int32_t count;
  int32_t r;
  RefreshTensor t[kMaxGroup];
};

struct Layout {
  size_t C, Q, Z, Bw, Jt, S, tau, vscale, lambda, order, total;
};

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
  L.lambda = take((size_t)r * 4);
  L.order = take((size_t)r * 4);
  L.total = off;
  return L;
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

// ---- block reductions (wavefront shuffles, then LDS across the waves) ------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
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

// ---- Householder reflector j applied to a strip of 32 columns --------------------------------
// V holds the (unscaled) reflector of column j in rows >= j of its column j: v_j = 1,
// v_row = V[row][j] * vscale_j.  H_j = I - tau_j v v^T is applied to columns
// col_begin + 32 blockIdx.x + (0..31) of the target matrix, rows >= j.
// COMPUTE: derive tau_j and vscale_j from column j first (QR factorisation; target == V and
// col_begin = j + 1) and let block 0 publish them; otherwise read them (forming Q).
template <bool COMPUTE>
__global__ __launch_bounds__(1024) void householder_strip_kernel(const RefreshGroup grp, int j, int col_begin,
                                                                 int target_is_q) {
  __shared__ float red[32][33];
  __shared__ float red1[16];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r, k = t.k;
  const float* __restrict__ V = t.Z;
  float* __restrict__ X = target_is_q ? t.Q : t.Z;
  const int c = threadIdx.x & 31, rg = threadIdx.x >> 5;
  const int col = col_begin + 32 * blockIdx.x + c;
  const bool active = col < r;

  float tau, vs;
  if (COMPUTE) {
    float part = 0.f;
    for (int row = j + 1 + threadIdx.x; row < k; row += 1024) {
      const float x = V[(size_t)row * r + j];
      part += x * x;
    }
    const float sigma = block_sum(part, red1);
    const float x0 = V[(size_t)j * r + j];
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
  if (tau == 0.f) return;  // H_j = I (uniform over the block)

  // w_c = X[j][col] + vs * sum_{row > j} V[row][j] X[row][col]
  float part = 0.f;
  if (active)
    for (int row = j + 1 + rg; row < k; row += 32) part += V[(size_t)row * r + j] * X[(size_t)row * r + col];
  red[rg][c] = part;
  __syncthreads();
  if (rg == 0) {
    float s = 0.f;
#pragma unroll
    for (int g = 0; g < 32; ++g) s += red[g][c];
    red[0][c] = active ? X[(size_t)j * r + col] + vs * s : 0.f;
  }
  __syncthreads();
  const float w = red[0][c];
  if (!active) return;
  const float tw = tau * w;
  if (rg == 0) X[(size_t)j * r + col] -= tw;
  const float tws = tw * vs;
  for (int row = j + 1 + rg; row < k; row += 32) X[(size_t)row * r + col] -= V[(size_t)row * r + j] * tws;
}

// Q <- [I_r ; 0]
__global__ __launch_bounds__(256) void identity_fill_kernel(const RefreshGroup grp, int which /*0: Q, 1: Jt*/) {
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  float* X = which == 0 ? t.Q : t.Jt;
  const int64_t count = (int64_t)(which == 0 ? t.k : r) * r;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += stride)
    X[i] = (i / r == i % r) ? 1.f : 0.f;
}

// ---- one-sided Jacobi on the rows of Bw ----------------------------------------------------------
// Round `round` of a round-robin tournament over n = r (+1 if odd) players: pair s = 0 is
// (n-1, round); pair s > 0 is ((round + s) mod (n-1), (round - s) mod (n-1)).
__global__ __launch_bounds__(256) void jacobi_round_kernel(const RefreshGroup grp, int round, int n) {
  __shared__ float red[3][4];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
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

// S[kk][order[i]] = Jt[i][kk] / |Jt[i]|
__global__ __launch_bounds__(256) void ritz_vectors_kernel(const RefreshGroup grp) {
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r;
  const int64_t count = (int64_t)r * r;
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; e < count; e += stride) {
    const int i = (int)(e / r), kk = (int)(e % r);
    t.S[(size_t)kk * r + t.order[i]] = t.Jt[e] * t.tau[i];
  }
}

// proj[:, col] = sign * Z[:, col] with sign chosen so the entry of largest magnitude (lowest row
// on ties) is positive; stored in the projector's dtype (round to nearest even for bf16).
template <class T>
__global__ __launch_bounds__(1024) void finalize_projector_kernel(const RefreshGroup grp) {
  __shared__ float bestv[32][33];
  __shared__ int bestr[32][33];
  const RefreshTensor& t = grp.t[blockIdx.y];
  const int r = grp.r, k = t.k;
  const int c = threadIdx.x & 31, rg = threadIdx.x >> 5;
  const int col = 32 * blockIdx.x + c;
  const bool active = col < r;
  float bv = -1.f; int br = 0x7fffffff;
  if (active)
    for (int row = rg; row < k; row += 32) {
      const float x = fabsf(t.Z[(size_t)row * r + col]);
      if (x > bv) { bv = x; br = row; }   // rows ascend per thread: first maximum kept
    }
  bestv[rg][c] = bv; bestr[rg][c] = br;
  __syncthreads();
  if (rg == 0) {
    float v = bestv[0][c]; int rw = bestr[0][c];
    for (int g = 1; g < 32; ++g) {
      const float x = bestv[g][c]; const int y = bestr[g][c];
      if (x > v || (x == v && y < rw)) { v = x; rw = y; }
    }
    bestr[0][c] = rw;
  }
  __syncthreads();
  if (!active) return;
  const int arg = bestr[0][c];
  const float sgn = t.Z[(size_t)arg * r + col] < 0.f ? -1.f : 1.f;
  T* P = static_cast<T*>(t.proj);
  for (int row = rg; row < k; row += 32) P[(size_t)row * t.ldp + col] = (T)(sgn * t.Z[(size_t)row * r + col]);
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

hipError_t refresh_group(const std::vector<RefreshItem>& items, int r, int iters, hipStream_t stream) {
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
    t.lambda = reinterpret_cast<float*>(it.ws + L.lambda);
    t.order = reinterpret_cast<int32_t*>(it.ws + L.order);
    t.proj = it.proj;
    t.k = (int32_t)k;
    t.ldp = (int32_t)it.ldp;
    t.seed = it.seed;
    kmax = k > kmax ? k : kmax;
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
  hipLaunchKernelGGL(gaussian_fill_kernel, fill_grid, dim3(256), 0, stream, grp);
  GALORE_RETURN_IF(hipGetLastError());

  auto gemm_f32 = [&](int which) -> hipError_t {
    GemmGroup g{};
    g.count = n;
    for (int i = 0; i < n; ++i) {
      const RefreshTensor& t = grp.t[i];
      GemmProblem& p = g.p[i];
      if (which == 0) {         // Z (k x r) = C Q
        p.A = t.C; p.lda = t.k; p.B = t.Q; p.ldb = r; p.M = t.k; p.N = r; p.K = t.k; p.C = t.Z; p.ldc = r;
      } else if (which == 1) {  // Bw (r x r) = Q^T Z
        p.A = t.Q; p.lda = r; p.B = t.Z; p.ldb = r; p.M = r; p.N = r; p.K = t.k; p.C = t.Bw; p.ldc = r;
      } else {                  // Z (k x r) = Q S
        p.A = t.Q; p.lda = r; p.B = t.S; p.ldb = r; p.M = t.k; p.N = r; p.K = r; p.C = t.Z; p.ldc = r;
      }
    }
    return launch_gemm_group(g, DType::F32, which != 1, false, Epilogue::StoreF32, stream);
  };

  for (int it = 0; it < iters; ++it) {
    GALORE_RETURN_IF(gemm_f32(0));
    // Householder QR of Z, reflector by reflector
    for (int j = 0; j < r; ++j) {
      const int ncols = r - (j + 1);
      const dim3 grid(ncols > 0 ? (ncols + 31) / 32 : 1, n);
      hipLaunchKernelGGL(householder_strip_kernel<true>, grid, dim3(1024), 0, stream, grp, j, j + 1, 0);
    }
    GALORE_RETURN_IF(hipGetLastError());
    hipLaunchKernelGGL(identity_fill_kernel, fill_grid, dim3(256), 0, stream, grp, 0);
    for (int j = r - 1; j >= 0; --j) {
      const dim3 grid((r - j + 31) / 32, n);
      hipLaunchKernelGGL(householder_strip_kernel<false>, grid, dim3(1024), 0, stream, grp, j, j, 1);
    }
    GALORE_RETURN_IF(hipGetLastError());
  }

  // Rayleigh-Ritz
  GALORE_RETURN_IF(gemm_f32(0));
  GALORE_RETURN_IF(gemm_f32(1));
  hipLaunchKernelGGL(identity_fill_kernel, dim3(blocks_for((int64_t)r * r, 256 * 8, 1024), n), dim3(256), 0, stream, grp, 1);
  const int players = (r % 2 == 0) ? r : r + 1;
  if (r > 1)
    for (int sweep = 0; sweep < kJacobiSweeps; ++sweep)
      for (int round = 0; round < players - 1; ++round)
        hipLaunchKernelGGL(jacobi_round_kernel, dim3(players / 2, n), dim3(256), 0, stream, grp, round, players);
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
    const dim3 grid((r + 31) / 32, sub.count);
    if (dt == DType::F32) hipLaunchKernelGGL(finalize_projector_kernel<float>, grid, dim3(1024), 0, stream, sub);
    else hipLaunchKernelGGL(finalize_projector_kernel<__bf16>, grid, dim3(1024), 0, stream, sub);
    GALORE_RETURN_IF(hipGetLastError());
  }
  return hipSuccess;
}

}  // namespace galore
