// Grouped, LDS-tiled MFMA GEMM for gfx950 (wave64), fp32 accumulate.
//
// One launch covers up to kMaxGroup independent problems C = A * B; a block finds its
// problem and tile from a table in the kernel arguments.  Operand tiles are staged
// global -> registers -> LDS in the layout they have in memory (16-byte vectors along the
// contiguous index), double-buffered, and turned into MFMA fragments on the LDS read:
//   * operand contiguous along K ("KCONTIG"): each lane reads its 8 (bf16) / 4 (fp32)
//     consecutive k values with one 16-byte LDS read;
//   * operand contiguous along its M or N index ("XCONTIG"): bf16 fragments are gathered with
//     the LDS transpose read (ds_read_b64_tr_b16), fp32 fragments with dword reads.
// bf16 uses v_mfma_f32_32x32x16_bf16, fp32 uses v_mfma_f32_32x32x2_f32 (four per 8-k group,
// with the k order inside the group permuted identically for A and B).
#pragma once
#include "common.hpp"

namespace galore {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <class T> struct ElemTraits;
template <> struct ElemTraits<__bf16> {
  static constexpr int VEC = 8;     // elements per 16-byte vector
  static constexpr int KSTEP = 16;  // k extent of one fragment
  static constexpr int PADK = 8;    // LDS row padding (elements), KCONTIG tiles
  static constexpr int PADX = 32;   // LDS row padding (elements), XCONTIG tiles
};
template <> struct ElemTraits<float> {
  static constexpr int VEC = 4;
  static constexpr int KSTEP = 8;
  static constexpr int PADK = 4;
  static constexpr int PADX = 8;
};

template <int BM_, int BN_, int BK_, int WGM_, int WGN_> struct TileCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_;
  static constexpr int NT = 64 * WGM * WGN;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32x32");
};

// ---- one operand tile: global -> registers -> LDS ------------------------------------------
template <class T, bool KCONTIG, int BX, int BK, int NT, bool ALIGNED> struct OperandTile {
  using ET = ElemTraits<T>;
  static constexpr int VEC = ET::VEC;
  static constexpr int OUTER = KCONTIG ? BX : BK;
  static constexpr int INNER = KCONTIG ? BK : BX;
  static constexpr int PITCH = INNER + (KCONTIG ? ET::PADK : ET::PADX);
  static constexpr int CH_ROW = INNER / VEC;
  static constexpr int TOTAL = OUTER * CH_ROW;
  static constexpr int PER_THREAD = TOTAL / NT;
  static constexpr int LDS_ELEMS = OUTER * PITCH;
  static_assert(TOTAL % NT == 0, "tile chunks must divide evenly over the block");
  static_assert((PITCH * sizeof(T)) % 16 == 0, "LDS rows must stay 16-byte aligned");

  uint4 regs[PER_THREAD];

  // x0 / k0: first x (M or N index) and first k of the tile; X / K: problem extents.
  __device__ __forceinline__ void load_global(const T* __restrict__ base, int ld, int x0, int k0,
                                              int X, int K, int tid) {
    const int o0 = KCONTIG ? x0 : k0, i0 = KCONTIG ? k0 : x0;
    const int olim = KCONTIG ? X : K, ilim = KCONTIG ? K : X;
#pragma unroll
    for (int it = 0; it < PER_THREAD; ++it) {
      const int c = tid + it * NT;
      const int o = o0 + c / CH_ROW;
      const int i = i0 + (c % CH_ROW) * VEC;
      uint4 v = make_uint4(0u, 0u, 0u, 0u);
      if (ALIGNED) {
        if (o < olim && i < ilim) v = *reinterpret_cast<const uint4*>(base + (size_t)o * ld + i);
      } else {
        if (o < olim) {
          const T* src = base + (size_t)o * ld + i;
          if (i + VEC <= ilim) {
            // whole 16-byte piece inside the row, but only element-aligned: memcpy lets the compiler
            // pick the widest access the target allows at that alignment
            __builtin_memcpy(&v, src, sizeof(uint4));
          } else {
            T tmp[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) tmp[e] = (i + e < ilim) ? src[e] : T(0);
            v = *reinterpret_cast<const uint4*>(tmp);
          }
        }
      }
      regs[it] = v;
    }
  }

  __device__ __forceinline__ void store_lds(T* lds, int tid) const {
#pragma unroll
    for (int it = 0; it < PER_THREAD; ++it) {
      const int c = tid + it * NT;
      *reinterpret_cast<uint4*>(lds + (c / CH_ROW) * PITCH + (c % CH_ROW) * VEC) = regs[it];
    }
  }
};

// ---- fragments -------------------------------------------------------------------------------
template <class T> struct Frag;

template <> struct Frag<__bf16> {
  bf16x8 v;
  // KCONTIG tile: lane (i = lane % 32, kg = lane / 32) takes k = kk + 8 kg .. + 7 of row x + i.
  template <int PITCH> __device__ __forceinline__ void load_k(const __bf16* lds, int x, int kk, int lane) {
    v = *reinterpret_cast<const bf16x8*>(lds + (x + (lane & 31)) * PITCH + kk + 8 * (lane >> 5));
  }
  // XCONTIG tile (rows are k): within each 16-lane group the transpose read hands lane i the four
  // k values of column i from a 4 (k) x 16 (x) block; lane s of the group supplies row s / 4,
  // columns 4 (s % 4) .. + 3.  Two reads give the 8 consecutive k of this lane's column.
  template <int PITCH> __device__ __forceinline__ void load_x(const __bf16* lds, int x, int kk, int lane) {
    const int s = lane & 15, g = lane >> 4;
    const __bf16* p = lds + (kk + 8 * (g >> 1) + (s >> 2)) * PITCH + x + 16 * (g & 1) + 4 * (s & 3);
    typedef s16x4 __attribute__((address_space(3))) * lds_v4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p + 4 * PITCH));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    const s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    v = __builtin_bit_cast(bf16x8, both);
  }
  static __device__ __forceinline__ void mma(f32x16& acc, const Frag& a, const Frag& b) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a.v, b.v, acc, 0, 0, 0);
  }
};

template <> struct Frag<float> {
  float v[4];  // k = kk + 4 kg + s for s = 0..3 (same permutation for A and B)
  template <int PITCH> __device__ __forceinline__ void load_k(const float* lds, int x, int kk, int lane) {
    const f32x4 t = *reinterpret_cast<const f32x4*>(lds + (x + (lane & 31)) * PITCH + kk + 4 * (lane >> 5));
    v[0] = t[0]; v[1] = t[1]; v[2] = t[2]; v[3] = t[3];
  }
  template <int PITCH> __device__ __forceinline__ void load_x(const float* lds, int x, int kk, int lane) {
    const float* p = lds + (kk + 4 * (lane >> 5)) * PITCH + x + (lane & 31);
#pragma unroll
    for (int s = 0; s < 4; ++s) v[s] = p[s * PITCH];
  }
  static __device__ __forceinline__ void mma(f32x16& acc, const Frag& a, const Frag& b) {
#pragma unroll
    for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.v[s], b.v[s], acc, 0, 0, 0);
  }
};

// Blocks are handed to the 8 XCDs round-robin by block id; give every XCD a contiguous run
// of logical tiles so neighbouring tiles (which share operand panels) share an L2.
__device__ __forceinline__ int xcd_contiguous_block_id(int bid, int nblocks) {
  const int xcd = bid & 7, q = bid >> 3;
  const int base = nblocks >> 3, rem = nblocks & 7;
  return xcd * base + (xcd < rem ? xcd : rem) + q;
}

// Tile id -> (tm, tn).  Tiles are numbered in bands of 4 tile-rows, and inside a band down the
// rows first, so any 32 consecutive ids (what the CUs of one XCD work on at a time) form a
// 4 x 8 patch of the output: they share 4 A panels and 8 B panels instead of streaming 32 + 32
// panels through the XCD's L2.
__device__ __forceinline__ void tile_coords(int t, int tiles_m, int tiles_n, int& tm, int& tn) {
  constexpr int kBand = 4;
  const int per_band = kBand * tiles_n;
  const int band = t / per_band;
  const int first = band * kBand;
  const int height = tiles_m - first < kBand ? tiles_m - first : kBand;
  const int in_band = t - band * per_band;
  tm = first + in_band % height;
  tn = in_band / height;
}

template <class T> __device__ __forceinline__ float to_f32(T x) { return (float)x; }

// ---- the kernel --------------------------------------------------------------------------------
template <class T, bool AK, bool BKC, bool ALIGNED, Epilogue EPI, class Cfg>
__global__ __launch_bounds__(Cfg::NT) void gemm_group_kernel(const GemmGroup grp) {
  using ET = ElemTraits<T>;
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, NT = Cfg::NT;
  constexpr int TM = Cfg::TM, TN = Cfg::TN;
  using ATile = OperandTile<T, AK, BM, BK, NT, ALIGNED>;
  using BTile = OperandTile<T, BKC, BN, BK, NT, ALIGNED>;
  static_assert(BK % ET::KSTEP == 0, "BK must be a multiple of the fragment k extent");

  extern __shared__ __align__(16) unsigned char smem_raw[];
  T* As[2];
  T* Bs[2];
  As[0] = reinterpret_cast<T*>(smem_raw);
  As[1] = As[0] + ATile::LDS_ELEMS;
  Bs[0] = As[1] + ATile::LDS_ELEMS;
  Bs[1] = Bs[0] + BTile::LDS_ELEMS;

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int wm0 = (wave % Cfg::WGM) * Cfg::WM;
  const int wn0 = (wave / Cfg::WGM) * Cfg::WN;

  const int bid = xcd_contiguous_block_id(blockIdx.x, gridDim.x);
  int pi = 0;
  for (int i = 1; i < grp.count; ++i)
    if (bid >= grp.p[i].tile_begin) pi = i;
  const GemmProblem& pr = grp.p[pi];
  int tm, tn;
  tile_coords(bid - pr.tile_begin, pr.tiles_m, pr.tiles_n, tm, tn);
  if (EPI == Epilogue::StoreSymF32 && tm > tn) return;
  const int m0 = tm * BM, n0 = tn * BN;
  const int M = pr.M, N = pr.N, K = pr.K;
  const T* __restrict__ A = static_cast<const T*>(pr.A);
  const T* __restrict__ B = static_cast<const T*>(pr.B);

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  ATile ta;
  BTile tb;
  const int KT = (K + BK - 1) / BK;
  ta.load_global(A, pr.lda, m0, 0, M, K, tid);
  tb.load_global(B, pr.ldb, n0, 0, N, K, tid);
  ta.store_lds(As[0], tid);
  tb.store_lds(Bs[0], tid);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) {
      ta.load_global(A, pr.lda, m0, (kt + 1) * BK, M, K, tid);
      tb.load_global(B, pr.ldb, n0, (kt + 1) * BK, N, K, tid);
    }
    const T* as = As[cur];
    const T* bs = Bs[cur];
#pragma unroll
    for (int kk = 0; kk < BK; kk += ET::KSTEP) {
      Frag<T> fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        if (AK) fa[i].template load_k<ATile::PITCH>(as, wm0 + 32 * i, kk, lane);
        else fa[i].template load_x<ATile::PITCH>(as, wm0 + 32 * i, kk, lane);
      }
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        if (BKC) fb[j].template load_k<BTile::PITCH>(bs, wn0 + 32 * j, kk, lane);
        else fb[j].template load_x<BTile::PITCH>(bs, wn0 + 32 * j, kk, lane);
      }
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) Frag<T>::mma(acc[i][j], fa[i], fb[j]);
    }
    if (kt + 1 < KT) {
      ta.store_lds(As[cur ^ 1], tid);
      tb.store_lds(Bs[cur ^ 1], tid);
    }
    __syncthreads();
  }

  // Epilogue.  Accumulator register v of lane l in a 32x32 MFMA tile is element
  // (row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32).
  const int ldc = pr.ldc;
  if (EPI == Epilogue::ApplyW) {
    // Weight update.  The 16 old weights of a 32 x 32 tile are all read before the first one is written
    // back: as one read-modify-write per element, every load had to wait for the store before it (the
    // compiler cannot tell that the addresses differ), 64 memory round trips in a row per thread.  Rows
    // and columns beyond the matrix are read from its last row / column (in bounds) and not written.
    T* W = static_cast<T*>(pr.C);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn0 + 32 * j + (lane & 31);
        const int col_ok = col < N ? col : N - 1;
        float w_old[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm0 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          w_old[v] = to_f32(W[(size_t)(row < M ? row : M - 1) * ldc + col_ok]);
        }
        __builtin_amdgcn_sched_barrier(0);  // the loads first, in one batch
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int row = m0 + wm0 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
          if (row < M && col < N) W[(size_t)row * ldc + col] = (T)(pr.s0 * w_old[v] - pr.s1 * acc[i][j][v]);
        }
      }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm0 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
        const int col = n0 + wn0 + 32 * j + (lane & 31);
        if (row < M && col < N) {
          const float a = acc[i][j][v];
          if (EPI == Epilogue::StoreF32) {
            static_cast<float*>(pr.C)[(size_t)row * ldc + col] = a;
          } else if (EPI == Epilogue::StoreSymF32) {
            float* C = static_cast<float*>(pr.C);
            C[(size_t)row * ldc + col] = a;
            if (tm != tn) C[(size_t)col * ldc + row] = a;
          } else {
            T* W = static_cast<T*>(pr.C);
            const size_t idx = (size_t)row * ldc + col;
            W[idx] = (T)(pr.s0 * to_f32(W[idx]) - pr.s1 * a);
          }
        }
      }
}

template <class T, bool AK, bool BKC, bool ALIGNED, Epilogue EPI, class Cfg>
inline hipError_t launch_gemm_instance(const GemmGroup& g, hipStream_t stream) {
  using ATile = OperandTile<T, AK, Cfg::BM, Cfg::BK, Cfg::NT, ALIGNED>;
  using BTile = OperandTile<T, BKC, Cfg::BN, Cfg::BK, Cfg::NT, ALIGNED>;
  constexpr size_t smem = 2 * (ATile::LDS_ELEMS + BTile::LDS_ELEMS) * sizeof(T);
  static_assert(smem <= 160 * 1024, "tile does not fit the 160 KB LDS");
  auto kern = gemm_group_kernel<T, AK, BKC, ALIGNED, EPI, Cfg>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(g.total_tiles), dim3(Cfg::NT), smem, stream, g);
  return hipGetLastError();
}

// Fills tile_begin / tiles_m / total_tiles for tile size BM x BN.
template <class Cfg> inline void plan_tiles(GemmGroup& g) {
  int total = 0;
  for (int i = 0; i < g.count; ++i) {
    GemmProblem& p = g.p[i];
    p.tile_begin = total;
    p.tiles_m = (p.M + Cfg::BM - 1) / Cfg::BM;
    p.tiles_n = (p.N + Cfg::BN - 1) / Cfg::BN;
    total += p.tiles_m * p.tiles_n;
  }
  g.total_tiles = total;
}

// 16-byte vector loads are legal when bases, strides and inner extents allow them.
template <class T> inline bool group_is_aligned(const GemmGroup& g, bool ak, bool bk) {
  constexpr int VEC = ElemTraits<T>::VEC;
  for (int i = 0; i < g.count; ++i) {
    const GemmProblem& p = g.p[i];
    if ((reinterpret_cast<uintptr_t>(p.A) | reinterpret_cast<uintptr_t>(p.B)) & 15) return false;
    if (p.lda % VEC || p.ldb % VEC) return false;
    if ((ak ? p.K : p.M) % VEC) return false;
    if ((bk ? p.K : p.N) % VEC) return false;
  }
  return true;
}

}  // namespace galore
