// Large-tile bf16 MFMA GEMM with direct global -> LDS loads (gfx950), used when every
// operand is 16-byte aligned and K is a multiple of the K step.
//
// Differences from the generic kernel in gemm_mfma.hpp:
//   * tiles go from global memory straight into LDS with global_load_lds_dwordx4 (each wave
//     instruction deposits 64 x 16 bytes contiguously at a wave-uniform LDS address), so no
//     VGPRs are spent on staging and a tile can be in flight while the previous one is consumed;
//   * LDS rows are unpadded; bank conflicts are avoided by an XOR swizzle that is applied by
//     choosing WHICH 16-byte piece of global memory each lane fetches:
//       - K-contiguous tile (rows of 64 k = 8 pieces): piece p of row x sits at p ^ ((x >> 1) & 7)
//         (rows of 32 k = 4 pieces: p ^ ((x >> 2) & 3));
//       - tile contiguous along its M/N index (rows are k): column c of row k sits at c ^ (32 (k & 3));
//     both make the ds_read_b128 / ds_read_b64_tr_b16 fragment reads conflict-free;
//   * rows past the matrix edge are fetched from the clamped (last valid) row / column and
//     never stored, so no masking is needed in the main loop;
//   * a STAGES-deep ring of tiles with one workgroup barrier per K step of 32 or 64.
#pragma once
#include "gemm_mfma.hpp"

namespace galore {

template <int BM_, int BN_, int BK_, int WGM_, int WGN_, int STAGES_> struct DlCfg {
  static constexpr int BM = BM_, BN = BN_, BK = BK_, WGM = WGM_, WGN = WGN_, STAGES = STAGES_;
  static_assert(BK == 32 || BK == 64, "K step is 32 or 64");
  static constexpr int NW = WGM * WGN;
  static constexpr int NT = 64 * NW;
  static constexpr int WM = BM / WGM, WN = BN / WGN;
  static constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(WM % 32 == 0 && WN % 32 == 0, "wave tile must be a multiple of 32x32");
};

typedef const void __attribute__((address_space(1))) * gptr_t;
typedef void __attribute__((address_space(3))) * lptr_t;

// s_waitcnt that waits only for vector-memory operations: at most `n` may stay outstanding.
template <int N> __device__ __forceinline__ void wait_vmcnt() {
  constexpr int imm = (N & 0xF) | ((N >> 4) << 14) | (7 << 4) | (15 << 8);
  __builtin_amdgcn_s_waitcnt(imm);
}

template <bool KCONTIG, int BX, int BK, int NW> struct DlOperand {
  static constexpr int TILE_BYTES = BX * BK * 2;
  static constexpr int CHUNKS = TILE_BYTES / 1024;  // one wave instruction fills 1 KB
  static constexpr int PER_WAVE = CHUNKS / NW;
  static constexpr int ROW_BYTES = KCONTIG ? BK * 2 : BX * 2;
  static_assert(CHUNKS % NW == 0, "tile chunks must divide evenly over the waves");
  static_assert(KCONTIG || BX >= 128, "index-contiguous tiles need rows of at least 128 elements");

  // Byte offsets (relative to the tile's first k) of the PER_WAVE 16-byte pieces this lane
  // fetches for every K step; computed once per block.  X = extent of the M/N index.
  unsigned voff[PER_WAVE];
  __device__ __forceinline__ void plan(int ld, int x0, int X, int wave, int lane) {
#pragma unroll
    for (int it = 0; it < PER_WAVE; ++it) {
      const int c = wave + it * NW;
      if (KCONTIG) {
        // BK = 64: rows of 8 pieces, 8 rows per chunk; BK = 32: rows of 4 pieces, 16 rows per chunk
        const int row = BK == 64 ? 8 * c + (lane >> 3) : 16 * c + (lane >> 2);
        const int p = BK == 64 ? (lane & 7) ^ ((row >> 1) & 7) : (lane & 3) ^ ((row >> 2) & 3);
        int xr = x0 + row;
        xr = xr < X ? xr : X - 1;
        voff[it] = ((unsigned)xr * (unsigned)ld + p * 8) * 2u;
      } else {
        constexpr int PPR = BX / 8;          // 16-byte pieces per row
        constexpr int RPC = 64 / PPR;        // rows per 1 KB chunk
        const int row = RPC * c + lane / PPR;
        const int p = (lane % PPR) ^ (4 * (row & 3));
        int xc = x0 + p * 8;
        xc = xc <= X - 8 ? xc : X - 8;
        voff[it] = ((unsigned)row * (unsigned)ld + xc) * 2u;
      }
    }
  }

  // Issue this wave's loads of one tile: `src` points at the tile's first k (wave-uniform),
  // `lds_tile` is the LDS byte address of the tile.  The instruction is written in assembly so
  // that the compiler does not see an LDS write it would fence every later LDS read against
  // (it would wait for ALL outstanding loads, the prefetched tile included); ordering against
  // the fragment reads is provided by the vmcnt waits and the barrier of the main loop.
  __device__ __forceinline__ void issue(const void* src, unsigned lds_tile, int wave) const {
#pragma unroll
    for (int it = 0; it < PER_WAVE; ++it) {
      const unsigned dst = __builtin_amdgcn_readfirstlane(lds_tile + (wave + it * NW) * 1024);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                   :: "s"(dst), "v"(voff[it]), "s"(src) : "memory");
    }
  }

  // Fragment of the 32-wide block starting at x (multiple of 32) for k = kk .. kk + 15.
  static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds_tile, int x, int kk, int lane) {
    if (KCONTIG) {
      const int i = lane & 31;
      const int pc = (2 * (kk >> 4) + (lane >> 5)) ^ (BK == 64 ? (i >> 1) & 7 : (i >> 2) & 3);
      return *reinterpret_cast<const bf16x8*>(lds_tile + (x + i) * ROW_BYTES + pc * 16);
    } else {
      const int s = lane & 15, g = lane >> 4;
      const int rho = (s >> 2) & 3;
      const int col = (x + 16 * (g & 1) + 4 * (s & 3)) ^ (32 * rho);
      const unsigned char* p = lds_tile + (kk + 8 * (g >> 1) + (s >> 2)) * ROW_BYTES + col * 2;
      typedef s16x4 __attribute__((address_space(3))) * lds_v4;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p));
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4)(p + 4 * ROW_BYTES));
      return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  }
};

template <bool AK, bool BKC, Epilogue EPI, class Cfg>
__global__ __launch_bounds__(Cfg::NT) void gemm_dl_kernel(const GemmGroup grp) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, NW = Cfg::NW, S = Cfg::STAGES;
  constexpr int TM = Cfg::TM, TN = Cfg::TN;
  using AOp = DlOperand<AK, BM, BK, NW>;
  using BOp = DlOperand<BKC, BN, BK, NW>;
  constexpr int STAGE_BYTES = AOp::TILE_BYTES + BOp::TILE_BYTES;
  constexpr int LOADS = AOp::PER_WAVE + BOp::PER_WAVE;  // vector-memory ops per wave per tile
  static_assert((S - 2) * LOADS <= 63, "too many loads in flight for the wait counter");

  extern __shared__ __align__(1024) unsigned char smem_dl[];

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
  const int M = pr.M, N = pr.N;
  const __bf16* __restrict__ A = static_cast<const __bf16*>(pr.A);
  const __bf16* __restrict__ B = static_cast<const __bf16*>(pr.B);
  const int KT = pr.K / BK;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  AOp opa;
  BOp opb;
  opa.plan(pr.lda, m0, M, wave, lane);
  opb.plan(pr.ldb, n0, N, wave, lane);
  const size_t a_step = AK ? (size_t)BK * 2 : (size_t)BK * pr.lda * 2;  // bytes per K step
  const size_t b_step = BKC ? (size_t)BK * 2 : (size_t)BK * pr.ldb * 2;
  const unsigned lds0 = (unsigned)(uintptr_t)smem_dl;
  auto issue_tile = [&](int kt) {
    const unsigned st = lds0 + (kt % S) * STAGE_BYTES;
    opa.issue(reinterpret_cast<const unsigned char*>(A) + kt * a_step, st, wave);
    opb.issue(reinterpret_cast<const unsigned char*>(B) + kt * b_step, st + AOp::TILE_BYTES, wave);
  };

  // Epilogue geometry (see below): after a trip through LDS each lane owns 8 consecutive
  // columns of row (32 i + ps RPP + rr) of its wave's tile.
  constexpr int WN = Cfg::WN;
  constexpr int PITCH = WN + 8;
  constexpr int LPR = WN / 8;        // lanes per row
  constexpr int RPP = 64 / LPR;      // rows per pass
  constexpr int PASSES = 32 / RPP;
  const int ldc = pr.ldc;
  const int rr = lane / LPR, cc = (lane % LPR) * 8;
  const int col = n0 + wn0 + cc;
  // The weight update reads W; those loads are issued during the last K step so their latency
  // hides behind its MFMAs instead of sitting in front of the epilogue.
  bf16x8 wpre[TM][PASSES];
  bool wok[TM][PASSES];

  // prologue: S - 1 tiles in flight (empty groups keep the wait counts uniform)
#pragma unroll
  for (int s = 0; s < S - 1; ++s)
    if (s < KT) issue_tile(s);

  for (int kt = 0; kt < KT; ++kt) {
    // tile kt has landed once at most the loads of the younger tiles are outstanding
    if (kt + S - 2 < KT) wait_vmcnt<(S - 2) * LOADS>();
    else wait_vmcnt<0>();
    __syncthreads();  // everyone's pieces of tile kt are visible; everyone is done with tile kt - 1
    if (kt + S - 1 < KT) issue_tile(kt + S - 1);  // refills the stage consumed at kt - 1
    if (EPI == Epilogue::ApplyW && kt == KT - 1) {
      const __bf16* W = static_cast<const __bf16*>(pr.C);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
          const int row = m0 + wm0 + 32 * i + ps * RPP + rr;
          wok[i][ps] = row < M && col < N;
          if (wok[i][ps]) wpre[i][ps] = *reinterpret_cast<const bf16x8*>(W + (size_t)row * ldc + col);
        }
    }

    const unsigned char* as = smem_dl + (kt % S) * STAGE_BYTES;
    const unsigned char* bs = as + AOp::TILE_BYTES;
#pragma unroll
    for (int kk = 0; kk < BK; kk += 16) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = AOp::frag(as, wm0 + 32 * i, kk, lane);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = BOp::frag(bs, wn0 + 32 * j, kk, lane);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
  }

  // ---- epilogue: accumulators -> wave-private LDS strip -> row-contiguous 16/32-byte accesses ----
  // An MFMA accumulator holds one column and 16 scattered rows per lane, which would make every
  // global access 2 or 4 bytes wide.  Each wave therefore parks a 32-row strip of its tile in LDS
  // (fp32, row pitch WN + 8 so both the column-wise writes and the row-wise reads spread over
  // the banks) and re-reads it with 8 consecutive columns per lane.
  static_assert(NW * 32 * PITCH * 4 <= S * STAGE_BYTES, "epilogue strips must fit the tile ring");
  __syncthreads();  // every wave has finished reading the last tile
  float* strip = reinterpret_cast<float*>(smem_dl) + wave * (32 * PITCH);
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        strip[(8 * (v >> 2) + 4 * (lane >> 5) + (v & 3)) * PITCH + 32 * j + (lane & 31)] = acc[i][j][v];
    f32x4 lo[PASSES], hi[PASSES];
#pragma unroll
    for (int ps = 0; ps < PASSES; ++ps) {
      const float* src = strip + (ps * RPP + rr) * PITCH + cc;
      lo[ps] = *reinterpret_cast<const f32x4*>(src);
      hi[ps] = *reinterpret_cast<const f32x4*>(src + 4);
    }
    if (EPI == Epilogue::ApplyW) {
      __bf16* W = static_cast<__bf16*>(pr.C);
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) {
        if (!wok[i][ps]) continue;
        const int row = m0 + wm0 + 32 * i + ps * RPP + rr;
        bf16x8 o;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          o[e] = (__bf16)(pr.s0 * (float)wpre[i][ps][e] - pr.s1 * lo[ps][e]);
          o[e + 4] = (__bf16)(pr.s0 * (float)wpre[i][ps][e + 4] - pr.s1 * hi[ps][e]);
        }
        *reinterpret_cast<bf16x8*>(W + (size_t)row * ldc + col) = o;
      }
    } else {
      float* C = static_cast<float*>(pr.C);
#pragma unroll
      for (int ps = 0; ps < PASSES; ++ps) {
        const int row = m0 + wm0 + 32 * i + ps * RPP + rr;
        if (row < M && col < N) {
          float* dst = C + (size_t)row * ldc + col;
          *reinterpret_cast<f32x4*>(dst) = lo[ps];
          *reinterpret_cast<f32x4*>(dst + 4) = hi[ps];
          if (EPI == Epilogue::StoreSymF32 && tm != tn) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              C[(size_t)(col + e) * ldc + row] = lo[ps][e];
              C[(size_t)(col + e + 4) * ldc + row] = hi[ps][e];
            }
          }
        }
      }
    }
  }
}

template <bool AK, bool BKC, Epilogue EPI, class Cfg>
inline hipError_t launch_gemm_dl_instance(const GemmGroup& g, hipStream_t stream) {
  using AOp = DlOperand<AK, Cfg::BM, Cfg::BK, Cfg::NW>;
  using BOp = DlOperand<BKC, Cfg::BN, Cfg::BK, Cfg::NW>;
  constexpr size_t smem = (size_t)Cfg::STAGES * (AOp::TILE_BYTES + BOp::TILE_BYTES);
  static_assert(smem <= 160 * 1024, "tile ring does not fit the 160 KB LDS");
  auto kern = gemm_dl_kernel<AK, BKC, EPI, Cfg>;
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

// The direct-load kernel needs 16-byte alignment of both operands and of the output (its
// epilogue moves 8 consecutive columns per lane), K a multiple of 64, N a multiple of 8, and at
// least 8 valid elements along each M/N index (for the edge clamp).
inline bool group_fits_dl(const GemmGroup& g, bool ak, bool bk, Epilogue epi, int bk_step = 64) {
  if (!group_is_aligned<__bf16>(g, ak, bk)) return false;
  const int c_vec = epi == Epilogue::ApplyW ? 8 : 4;  // elements per 16 bytes of the output
  for (int i = 0; i < g.count; ++i) {
    const GemmProblem& p = g.p[i];
    if (p.K % bk_step != 0 || p.K < bk_step) return false;
    if (p.M < 8 || p.N < 8 || p.N % 8 != 0) return false;
    if ((reinterpret_cast<uintptr_t>(p.C) & 15) || p.ldc % c_vec != 0) return false;
  }
  return true;
}

}  // namespace galore
