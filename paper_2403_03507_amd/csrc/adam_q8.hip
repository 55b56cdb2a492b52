// Low-rank Adam (Algorithm 2, update block) with 8-bit block-wise moments, the storage Sec. 4.3
// of the paper takes from 8-bit optimizers.  The paper prints no number format; this one is the
// library's own:
//   * block = 256 consecutive elements of a row, one fp32 scale per block (max |m|, max v);
//   * first moment  : sign | 4 exponent bits e | 3 mantissa bits f, magnitude (1 + f/8) 2^(e-15)
//                     for e > 0 and (f/8) 2^-14 for e = 0, times the scale (largest used: 1);
//   * second moment : 5 exponent bits | 3 mantissa bits, (1 + f/8) 2^(e-31) / (f/8) 2^-30;
//   * decode = magnitude * scale; encode = round min(|x| * (1 / scale), 1) to the nearest magnitude
//     (one reciprocal per block, one multiplication per element), ties to the even mantissa field.
// One pass: decode, update in fp32 (every operation rounded once, fused multiply-adds where
// written), form N from the unquantised new moments, take the block maxima over the wavefront,
// encode.  One wavefront owns one block (4 elements per lane), so the maxima are wavefront
// reductions and nothing but N's transposition needs LDS.
#include <type_traits>

#include "common.hpp"

namespace galore {
namespace {

typedef float q_f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 q_bf16x4 __attribute__((ext_vector_type(4)));

template <int EBITS> __device__ __forceinline__ float q8_magnitude(unsigned code) {  // code without sign
  constexpr int bias = (1 << EBITS) - 1;
  // (1 + f/8) 2^(e-bias) = (8 + f) 2^(e-bias-3) for e > 0, (f/8) 2^(1-bias) = f 2^(1-bias-3) for e = 0:
  // an integer of at most 4 bits scaled by a power of two, exact either way
  const unsigned e = code >> 3, f = code & 7u;
  const unsigned mant = e ? 8u + f : f;
  const int ex = (int)(e ? e : 1u) - (bias + 3);
  return __builtin_ldexpf((float)mant, ex);
}

// y in [0, 1] -> code of the nearest magnitude; round-to-nearest-even on a 3-bit mantissa is
// exactly "nearest, ties to the even mantissa field", binade changes included.  For a normal
// magnitude the rounding is one integer addition on the bits of y: adding 0x7FFFF plus the lowest
// kept bit carries into the kept mantissa bit exactly when the dropped part is above one half, or
// equal to it with the kept field odd, and a mantissa that rounds up to 8 carries on into the exponent.
template <int EBITS> __device__ __forceinline__ unsigned q8_encode_magnitude(float y) {
  constexpr int bias = (1 << EBITS) - 1;
  constexpr int emin = 1 - bias;                    // exponent of the smallest normal magnitude
  const unsigned bits = __float_as_uint(y);
  const unsigned kept = (bits + 0x7FFFFu + ((bits >> 20) & 1u)) >> 20;   // (biased exponent << 3) | f after rounding
  const unsigned normal = kept - ((unsigned)(127 - bias) << 3);           // (e << 3) | f
  // below the smallest normal: uniform steps of 2^(emin-3); 8 steps reach the smallest normal (code 8)
  const unsigned sub = (unsigned)__builtin_rintf(y * __builtin_ldexpf(1.0f, 3 - emin));
  return y >= __builtin_ldexpf(1.0f, emin) ? normal : sub;   // y < 2^-40 rounds to 0 in the second form
}

// Maximum over the 64 lanes of a wavefront, every lane gets it.  Data-parallel-primitive moves inside
// the VALU (quad permutes, row mirrors, row broadcasts) instead of six LDS-crossbar shuffles; lanes a
// row mask excludes see their own value again.  The maximum does not depend on the order.
__device__ __forceinline__ float wave_max(float x) {
  auto dpp = [](float v, auto ctrl, auto row_mask) {
    const int b = __builtin_bit_cast(int, v);
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(b, b, decltype(ctrl)::value, decltype(row_mask)::value, 0xF, false));
  };
  using std::integral_constant;
  x = fmaxf(x, dpp(x, integral_constant<int, 0xB1>{}, integral_constant<int, 0xF>{}));   // quad_perm [1,0,3,2]
  x = fmaxf(x, dpp(x, integral_constant<int, 0x4E>{}, integral_constant<int, 0xF>{}));   // quad_perm [2,3,0,1]
  x = fmaxf(x, dpp(x, integral_constant<int, 0x141>{}, integral_constant<int, 0xF>{}));  // row_half_mirror
  x = fmaxf(x, dpp(x, integral_constant<int, 0x140>{}, integral_constant<int, 0xF>{}));  // row_mirror: each row of 16 holds its maximum
  x = fmaxf(x, dpp(x, integral_constant<int, 0x142>{}, integral_constant<int, 0xA>{}));  // row_bcast15 into rows 1 and 3
  x = fmaxf(x, dpp(x, integral_constant<int, 0x143>{}, integral_constant<int, 0xC>{}));  // row_bcast31 into rows 2 and 3
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), 63));
}

__device__ __forceinline__ void store_n4(float* N, size_t i, q_f32x4 n) { *reinterpret_cast<q_f32x4*>(N + i) = n; }
__device__ __forceinline__ void store_n4(__bf16* N, size_t i, q_f32x4 n) {
  q_bf16x4 o;
  o[0] = (__bf16)n[0]; o[1] = (__bf16)n[1]; o[2] = (__bf16)n[2]; o[3] = (__bf16)n[3];
  *reinterpret_cast<q_bf16x4*>(N + i) = o;
}

// One workgroup of 4 wavefronts per tile of TR rows x 256 columns; wavefront w takes rows
// w, w + 4, ...; lane l takes columns 4 l .. 4 l + 3 of the block.
template <class TN, bool TRANSPOSE>
__global__ __launch_bounds__(256) void adam_q8_group_kernel(const AdamQ8Group grp) {
#pragma clang fp contract(off)
  constexpr int TR = 32;
  constexpr int PAD = 16 / sizeof(TN);
  __shared__ __align__(16) TN tile[TRANSPOSE ? 256 : 1][TRANSPOSE ? TR + PAD : 1];  // tile[column][row] = N[row][column]
  const AdamQ8Problem& pr = grp.p[blockIdx.y];
  const int rows = pr.rows, cols = pr.cols;
  const int tiles_c = cols >> 8;
  const int ntiles = tiles_c * ((rows + TR - 1) / TR);
  const float beta1 = grp.beta1, beta2 = grp.beta2, omb1 = grp.omb1, omb2 = grp.omb2, eps = grp.eps;
  const float ic1 = pr.inv_c1, ic2 = pr.inv_c2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  TN* __restrict__ N = static_cast<TN*>(pr.N);
  for (int t = blockIdx.x; t < ntiles; t += gridDim.x) {
    const int i0 = (t / tiles_c) * TR, j0 = (t % tiles_c) << 8;
    for (int rl = wave; rl < TR; rl += 4) {
      const int i = i0 + rl;
      if (i >= rows) break;                             // wave-uniform
      const size_t base = (size_t)i * cols + j0;
      const size_t idx = base + 4 * lane;
      const size_t blk = base >> 8;
      const q_f32x4 g = *reinterpret_cast<const q_f32x4*>(pr.R + idx);
      const unsigned cm = *reinterpret_cast<const unsigned*>(pr.Mc + idx);
      const unsigned cv = *reinterpret_cast<const unsigned*>(pr.Vc + idx);
      const float sm = pr.Ms[blk], sv = pr.Vs[blk];
      float m[4], v[4];
      q_f32x4 n;
      float amax = 0.f, vmax = 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const unsigned bm = (cm >> (8 * e)) & 0xFFu, bv = (cv >> (8 * e)) & 0xFFu;
        float m_old = q8_magnitude<4>(bm & 0x7Fu) * sm;
        if (bm & 0x80u) m_old = -m_old;
        const float v_old = q8_magnitude<5>(bv) * sv;
        const float gm = omb1 * g[e];
        m[e] = __builtin_fmaf(beta1, m_old, gm);
        float gv = omb2 * g[e];
        gv = gv * g[e];
        v[e] = __builtin_fmaf(beta2, v_old, gv);
        const float mh = m[e] * ic1;
        const float vh = v[e] * ic2;
        const float den = __builtin_sqrtf(vh) + eps;
        n[e] = mh / den;
        amax = fmaxf(amax, fabsf(m[e]));
        vmax = fmaxf(vmax, v[e]);
      }
      amax = wave_max(amax);
      vmax = wave_max(vmax);
      unsigned om = 0u, ov = 0u;
      const float inv_m = amax != 0.f ? 1.0f / amax : 0.f;   // one correctly rounded division per block
      const float inv_v = vmax != 0.f ? 1.0f / vmax : 0.f;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        unsigned bm = 0u, bv = 0u;
        if (amax != 0.f && m[e] != 0.f) bm = (m[e] < 0.f ? 0x80u : 0u) | q8_encode_magnitude<4>(fminf(fabsf(m[e]) * inv_m, 1.0f));
        if (vmax != 0.f && v[e] > 0.f) bv = q8_encode_magnitude<5>(fminf(v[e] * inv_v, 1.0f));
        om |= bm << (8 * e);
        ov |= bv << (8 * e);
      }
      *reinterpret_cast<unsigned*>(pr.Mc + idx) = om;
      *reinterpret_cast<unsigned*>(pr.Vc + idx) = ov;
      if (lane == 0) { pr.Ms[blk] = amax; pr.Vs[blk] = vmax; }
      if (TRANSPOSE) {
#pragma unroll
        for (int e = 0; e < 4; ++e) tile[4 * lane + e][rl] = (TN)n[e];
      } else {
        store_n4(N, idx, n);
      }
    }
    if (TRANSPOSE) {
      __syncthreads();
      // column j0 + threadIdx.x of the tile = TR consecutive entries of row j0 + threadIdx.x of N^T
      const int j = j0 + threadIdx.x;
      TN* dst = N + (size_t)j * rows + i0;
      if (i0 + TR <= rows && (rows * sizeof(TN)) % 16 == 0) {
        constexpr int VEC = 16 / sizeof(TN);
#pragma unroll
        for (int q = 0; q < TR / VEC; ++q)
          *reinterpret_cast<uint4*>(dst + q * VEC) = *reinterpret_cast<const uint4*>(&tile[threadIdx.x][q * VEC]);
      } else {
        for (int rl = 0; rl < TR && i0 + rl < rows; ++rl) dst[rl] = tile[threadIdx.x][rl];
      }
      __syncthreads();
    }
  }
}

}  // namespace

hipError_t launch_adam_q8_group(const AdamQ8Group& g, DType n_dtype, hipStream_t stream) {
  if (g.count <= 0) return hipSuccess;
  if (g.count > kMaxGroup) return hipErrorInvalidValue;
  int64_t maxtiles = 0;
  for (int i = 0; i < g.count; ++i) {
    if (g.p[i].cols % 256 != 0 || g.p[i].rows < 1) return hipErrorInvalidValue;
    if (g.p[i].transpose_n != g.p[0].transpose_n) return hipErrorInvalidValue;
    const int64_t t = (int64_t)((g.p[i].rows + 31) / 32) * (g.p[i].cols / 256);
    maxtiles = t > maxtiles ? t : maxtiles;
  }
  const dim3 grid((unsigned)(maxtiles > 8192 ? 8192 : maxtiles), (unsigned)g.count);
  const bool tr = g.p[0].transpose_n != 0;
  if (n_dtype == DType::BF16) {
    if (tr) hipLaunchKernelGGL((adam_q8_group_kernel<__bf16, true>), grid, dim3(256), 0, stream, g);
    else hipLaunchKernelGGL((adam_q8_group_kernel<__bf16, false>), grid, dim3(256), 0, stream, g);
  } else {
    if (tr) hipLaunchKernelGGL((adam_q8_group_kernel<float, true>), grid, dim3(256), 0, stream, g);
    else hipLaunchKernelGGL((adam_q8_group_kernel<float, false>), grid, dim3(256), 0, stream, g);
  }
  return hipGetLastError();
}

}  // namespace galore
