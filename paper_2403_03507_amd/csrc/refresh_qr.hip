// Householder QR of the iteration block of the subspace refresh (Algorithm 2, refresh branch): Q = qr(Z).Q for the
// transposed blocks Zt, Qt (r x k).  Two levels: panels of 8 reflectors factored and applied with the panel in
// registers inside a macro panel of 32 columns; the rest of the matrix sees a macro panel once, in compact WY form
// I - V T V^T on the fp32 matrix cores.  Q is formed by applying the macro panels to [I 0] backwards.  Short sides
// beyond 4096 (or not a multiple of 4) fall back to simpler paths.  All tensors of a group advance in lock-step
// (blockIdx.y = tensor); no atomics, fixed reduction orders.
#include "refresh_common.hpp"

namespace galore {
namespace rf {
namespace {

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

}  // namespace

hipError_t launch_householder_qr(const RefreshGroup& grp, const RefreshGroup* dgrp, int64_t kmax, hipStream_t stream) {
  const int n = grp.count, r = grp.r;
  const dim3 fill_grid(blocks_for(kmax * r, 256 * 8, 1024), n);
  bool wy_ok = true;  // compact WY path: 16-byte pieces of the transposed rows
  for (int i = 0; i < n; ++i) wy_ok = wy_ok && grp.t[i].k % 4 == 0;
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
      return hipSuccess;
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
  return hipSuccess;
}

}  // namespace rf
}  // namespace galore
