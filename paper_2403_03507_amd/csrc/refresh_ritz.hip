// Rayleigh-Ritz eigen-solve of the subspace refresh (Algorithm 2, refresh branch): the symmetric r x r matrix
// B = Q^T C Q is diagonalised by one-sided (Hestenes) Jacobi on its rows, in blocks: a round pairs two 16-row
// blocks (round robin over blocks); a workgroup forms the 32 x 32 Gram matrix of its rows on the matrix cores,
// runs its inner rounds on the Gram matrix alone, accumulates the 32 x 32 rotation product and applies it to its
// rows of B and of the eigenvector matrix as two small matrix products (rows are never staged in LDS).  Up to 10
// sweeps; sweeps after convergence return at once.  Then Ritz values, their order, and unit-length eigenvectors.
#include "refresh_common.hpp"

namespace galore {
namespace rf {
namespace {

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

}  // namespace

hipError_t launch_ritz_solve(const RefreshGroup& grp, const RefreshGroup* dgrp, bool crowded, hipStream_t stream) {
  const int n = grp.count, r = grp.r;
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
  return hipGetLastError();
}

}  // namespace rf
}  // namespace galore
