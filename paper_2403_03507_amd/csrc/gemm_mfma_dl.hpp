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

typedef int i32x4 __attribute__((ext_vector_type(4)));
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
  __device__ __forceinline__ void plan(int ld, int x0, int X, int wave, int lane) { plan_into(voff, ld, x0, X, wave, lane); }
  // The same plan into an array the caller owns (a kernel that switches layouts between tiles keeps one).
  static __device__ __forceinline__ void plan_into(unsigned (&voff)[PER_WAVE], int ld, int x0, int X, int wave, int lane) {
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
  // STREAM marks the loads non-temporal: for an operand whose panels are used once by the
  // workgroups that share them and not again soon, so that they do not displace the other
  // operand's panels (which the XCD needs again in its next round) from L2.
  template <bool STREAM> __device__ __forceinline__ void issue(const void* src, unsigned lds_tile, int wave) const {
    issue_from<STREAM>(voff, src, lds_tile, wave);
  }
  template <bool STREAM>
  static __device__ __forceinline__ void issue_from(const unsigned (&voff)[PER_WAVE], const void* src, unsigned lds_tile, int wave) {
#pragma unroll
    for (int it = 0; it < PER_WAVE; ++it) {
      const unsigned dst = __builtin_amdgcn_readfirstlane(lds_tile + (wave + it * NW) * 1024);
      if (STREAM)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 nt"
                     :: "s"(dst), "v"(voff[it]), "s"(src) : "memory");
      else
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

// One tile of the launch, as seen by the workgroup that computes it (all wave-uniform).
struct DlTile {
  int pi;      // problem index
  int m0, n0;  // first row / column
  int tm, tn;
  int round;   // which pass of the persistent grid produced it
};

// Persistent kernel: the grid has at most one workgroup per CU and workgroup b walks the tiles
// of its XCD's share with stride G/8.  The K steps of consecutive tiles form ONE stream through
// the two-stage LDS ring: the first K step of the next tile is requested while the last K step of
// the current tile is multiplied, so its latency (and the whole epilogue) hides behind MFMAs and
// stores, and no workgroup launch sits between two tiles.  The epilogue parks 8-row strips of the
// accumulators in a wave-private LDS area OUTSIDE the ring, so it never waits for the ring.
// W_ANY (weight update only): the output may have any row length, leading dimension and element
// alignment.  Its 16-byte pieces are then read and written at element alignment, and the piece that
// straddles the end of a row is updated element by element.
template <bool AK, bool BKC, Epilogue EPI, class Cfg, bool W_ANY = false>
__global__ __launch_bounds__(Cfg::NT) void gemm_dl_kernel(const GemmGroup grp) {
  static_assert(!W_ANY || EPI == Epilogue::ApplyW, "W_ANY is a variant of the weight update");
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, NW = Cfg::NW, S = Cfg::STAGES;
  constexpr int TM = Cfg::TM, TN = Cfg::TN, WN = Cfg::WN;
  using AOp = DlOperand<AK, BM, BK, NW>;
  using BOp = DlOperand<BKC, BN, BK, NW>;
  constexpr int STAGE_BYTES = AOp::TILE_BYTES + BOp::TILE_BYTES;
  constexpr int RING_BYTES = S * STAGE_BYTES;
  // Measured on the 7B shapes: streaming G in the LEFT projection (its panels are shared by the
  // four tile rows of a band at the same time and never needed again) -2.7 %; streaming the B
  // panels of the weight update +9 % (slower), G of the RIGHT projection no change.
  constexpr bool STREAM_A = false;
  constexpr bool STREAM_B = EPI == Epilogue::StoreF32 && AK && !BKC;
  static_assert(S == 2, "the cross-tile stream is written for a two-stage ring");
  static_assert(BK == 64, "the pipelined main loop is written out for four 16-k substeps per K step");
  static_assert(WN == 64 || WN == 128, "the strip epilogue covers 8 rows with one or two passes of the wave");
  constexpr int PITCH = WN + 8;           // floats; 4 PITCH = 32 (mod 64) spreads the two half-waves over the banks
  constexpr int STRIP_FLOATS = 8 * PITCH;
  constexpr int LPR = WN / 8;             // lanes per strip row (8 columns each)
  constexpr int RPP = 64 / LPR;           // rows per pass
  constexpr int PASSES = 8 / RPP;

  extern __shared__ __align__(1024) unsigned char smem_dl[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave % Cfg::WGM) * Cfg::WM;
  const int wn0 = (wave / Cfg::WGM) * Cfg::WN;

  // Workgroups are dealt to the XCDs round-robin (blockIdx % 8).  XCD x owns one contiguous eighth
  // of the launch's tile ids and its G/8 workgroups walk it side by side, so the tiles an XCD works
  // on at a time are consecutive (see tile_coords) and every XCD has the same amount of work.
  const int per_xcd = gridDim.x >> 3;
  const int xcd = blockIdx.x & 7, q_in_xcd = blockIdx.x >> 3;
  const int share = grp.total_tiles >> 3, extra = grp.total_tiles & 7;
  const int first_id = xcd * share + (xcd < extra ? xcd : extra);
  const int n_ids = share + (xcd < extra ? 1 : 0);
  auto locate = [&](int round, DlTile& t) -> bool {
    for (;; ++round) {
      const int idx = round * per_xcd + q_in_xcd;
      if (idx >= n_ids) return false;
      const int id = first_id + idx;
      int pi = 0;
      for (int i = 1; i < grp.count; ++i)
        if (id >= grp.p[i].tile_begin) pi = i;
      int tm, tn;
      tile_coords(id - grp.p[pi].tile_begin, grp.p[pi].tiles_m, grp.p[pi].tiles_n, tm, tn);
      if (EPI == Epilogue::StoreSymF32 && tm > tn) continue;  // the mirror tile writes this one
      t.pi = pi; t.m0 = tm * BM; t.n0 = tn * BN; t.tm = tm; t.tn = tn; t.round = round;
      return true;
    }
  };

  DlTile cur;
  if (!locate(0, cur)) return;

  // load side: plan and source of the tile whose K steps are being requested
  AOp opa;
  BOp opb;
  const unsigned char* a_src = nullptr;
  const unsigned char* b_src = nullptr;
  size_t a_step = 0, b_step = 0;  // bytes per K step
  auto bind = [&](const DlTile& t) {
    const GemmProblem& p = grp.p[t.pi];
    opa.plan(p.lda, t.m0, p.M, wave, lane);
    opb.plan(p.ldb, t.n0, p.N, wave, lane);
    a_src = static_cast<const unsigned char*>(p.A);
    b_src = static_cast<const unsigned char*>(p.B);
    a_step = AK ? (size_t)BK * 2 : (size_t)BK * p.lda * 2;
    b_step = BKC ? (size_t)BK * 2 : (size_t)BK * p.ldb * 2;
  };
  const unsigned lds0 = (unsigned)(uintptr_t)smem_dl;
  auto issue_step = [&](int kt, int stage) {
    const unsigned st = lds0 + stage * STAGE_BYTES;
    opa.template issue<STREAM_A>(a_src + kt * a_step, st, wave);
    opb.template issue<STREAM_B>(b_src + kt * b_step, st + AOp::TILE_BYTES, wave);
  };

  // epilogue geometry: a strip is 8 rows x WN columns of the wave's tile (accumulator registers
  // 4q .. 4q+3 of every 32x32 block); after the trip through LDS each lane owns 8 consecutive
  // columns of a row, i.e. 16-byte (bf16) or 32-byte (fp32) contiguous global accesses.
  float* strip = reinterpret_cast<float*>(smem_dl + RING_BYTES) + wave * STRIP_FLOATS;
  const int rr = lane / LPR, cc = (lane % LPR) * 8;

  bind(cur);
  issue_step(0, 0);
  int g = 0;  // K steps consumed so far, over all tiles: step g lives in stage g & 1

  for (;;) {
    const GemmProblem& pr = grp.p[cur.pi];
    const int M = pr.M, N = pr.N, ldc = pr.ldc;
    const int KT = pr.K / BK;
    const int row0 = cur.m0 + wm0 + rr;
    const int col = cur.n0 + wn0 + cc;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    auto multiply_step = [&](int stage) {
      const unsigned char* as = smem_dl + stage * STAGE_BYTES;
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
    };

    // The weight update reads the W tile.  Its loads are issued in two halves during the last two
    // K steps (block rows 0 .. TM/2-1 first: the epilogue needs them first), so that their
    // latency hides behind MFMAs instead of sitting in front of the epilogue.  Every slice is
    // exactly one load instruction (lanes outside the matrix read a clamped address): the wait
    // of the last K step counts on that.
    bf16x8 wpre[TM][4][PASSES];
    constexpr int W_EARLY = (TM / 2) * 4 * PASSES;  // load instructions of the first half
    auto fetch_w = [&](int i_begin, int i_end) {
      const __bf16* W = static_cast<const __bf16*>(pr.C);
      const int colc = (W_ANY ? col + 8 <= N : col < N) ? col : 0;  // W_ANY: whole pieces only (a row holds at least 8 elements)
#pragma unroll
      for (int i = 0; i < TM; ++i)
        if (i >= i_begin && i < i_end) {
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int ps = 0; ps < PASSES; ++ps) {
              const int row = row0 + 32 * i + 8 * q + RPP * ps;
              // W is read once and written once per step: non-temporal accesses keep it from
              // displacing the operand panels that the XCD's other workgroups still need in L2
              const __bf16* wsrc = W + (size_t)(row < M ? row : M - 1) * ldc + colc;
              if (W_ANY) __builtin_memcpy(&wpre[i][q][ps], wsrc, sizeof(bf16x8));  // element-aligned; still one load instruction
              else wpre[i][q][ps] = __builtin_bit_cast(bf16x8, __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(wsrc)));
            }
        }
    };

    // All K steps but the last two run software-pipelined: the fragments of the next 16 k are read
    // from LDS while the MFMAs of the current 16 k execute, and the MFMAs of a step's last 16 k are
    // deferred past the next step's barrier, so the matrix cores have work during the barrier, the
    // load issue and the first LDS reads of every step.
    // At the top of a step everything this wave requested has landed (vmcnt also covers the
    // previous epilogue's stores) and its own LDS reads of the other stage have returned; after
    // the barrier every wave's pieces of step g are visible and the other stage can be refilled.
    const int n_main = KT - 2;
    if (n_main > 0) {
      bf16x8 fa0[TM], fb0[TN], fa1[TM], fb1[TN];
      auto read_frags = [&](int stage, int kk, bf16x8 (&fa)[TM], bf16x8 (&fb)[TN]) {
        const unsigned char* as = smem_dl + stage * STAGE_BYTES;
        const unsigned char* bs = as + AOp::TILE_BYTES;
#pragma unroll
        for (int i = 0; i < TM; ++i) fa[i] = AOp::frag(as, wm0 + 32 * i, kk, lane);
#pragma unroll
        for (int j = 0; j < TN; ++j) fb[j] = BOp::frag(bs, wn0 + 32 * j, kk, lane);
      };
      auto mma = [&](const bf16x8 (&fa)[TM], const bf16x8 (&fb)[TN]) {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int j = 0; j < TN; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
      };
      // scheduling hint: alternate one LDS read with one MFMA, then the remaining MFMAs
      constexpr int NREADS = TM * (AK ? 1 : 2) + TN * (BKC ? 1 : 2);
      constexpr int NPAIR = NREADS < TM * TN ? NREADS : TM * TN;
      auto interleave = [&]() {
#pragma unroll
        for (int t = 0; t < NPAIR; ++t) {
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
        }
        if (NREADS > NPAIR) __builtin_amdgcn_sched_group_barrier(0x100, NREADS - NPAIR, 0);
        if (TM * TN > NPAIR) __builtin_amdgcn_sched_group_barrier(0x008, TM * TN - NPAIR, 0);
      };

      wait_vmcnt<0>();
      __syncthreads();
      issue_step(1, (g + 1) & 1);
      read_frags(g & 1, 0, fa0, fb0);
      read_frags(g & 1, 16, fa1, fb1); mma(fa0, fb0); interleave();
      read_frags(g & 1, 32, fa0, fb0); mma(fa1, fb1); interleave();
      read_frags(g & 1, 48, fa1, fb1); mma(fa0, fb0); interleave();
      ++g;
      for (int kt = 1; kt < n_main; ++kt) {
        __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) and lgkmcnt(0)
        __syncthreads();
        issue_step(kt + 1, (g + 1) & 1);
        read_frags(g & 1, 0, fa0, fb0); mma(fa1, fb1); interleave();
        read_frags(g & 1, 16, fa1, fb1); mma(fa0, fb0); interleave();
        read_frags(g & 1, 32, fa0, fb0); mma(fa1, fb1); interleave();
        read_frags(g & 1, 48, fa1, fb1); mma(fa0, fb0); interleave();
        ++g;
      }
      mma(fa1, fb1);
    }
    bool w_early = false;
    if (KT >= 2) {  // step KT - 2
      __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) and lgkmcnt(0)
      __syncthreads();
      issue_step(KT - 1, (g + 1) & 1);
      if (EPI == Epilogue::ApplyW) {
        fetch_w(0, TM / 2);
        w_early = true;
      }
      multiply_step(g & 1);
      ++g;
    }

    // Last K step: the tile loads are older than the early W loads and vmcnt retires in issue
    // order, so they have landed once at most W_EARLY operations are outstanding.  The first K
    // step of the next tile is requested here, so the epilogue and the tile switch hide behind it.
    if (w_early) wait_vmcnt<W_EARLY>();
    else wait_vmcnt<0>();
    __syncthreads();
    DlTile nxt;
    const bool have_next = locate(cur.round + 1, nxt);
    if (have_next) {
      bind(nxt);
      issue_step(0, (g + 1) & 1);
    }
    if (EPI == Epilogue::ApplyW) fetch_w(w_early ? TM / 2 : 0, TM);
    multiply_step(g & 1);
    ++g;

    // ---- epilogue: accumulators -> wave-private LDS strip -> row-contiguous global accesses ----
    // An MFMA accumulator holds one column and 16 scattered rows per lane, which would make every
    // global access 2 or 4 bytes wide.  LDS operations of one wave execute in order, so the strip
    // can be rewritten right after it was read without a wait.
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int c = 0; c < 4; ++c)
            strip[(4 * (lane >> 5) + c) * PITCH + 32 * j + (lane & 31)] = acc[i][j][4 * q + c];
#pragma unroll
        for (int ps = 0; ps < PASSES; ++ps) {
          const float* src = strip + (rr + RPP * ps) * PITCH + cc;
          const f32x4 lo = *reinterpret_cast<const f32x4*>(src);
          const f32x4 hi = *reinterpret_cast<const f32x4*>(src + 4);
          const int row = row0 + 32 * i + 8 * q + RPP * ps;
          if (row >= M || col >= N) continue;
          if (EPI == Epilogue::ApplyW) {
            __bf16* W = static_cast<__bf16*>(pr.C);
            __bf16* wdst = W + (size_t)row * ldc + col;
            if (W_ANY && col + 8 > N) {  // the piece that straddles the end of the row: its old weights were not prefetched
#pragma unroll
              for (int e = 0; e < 8; ++e)
                if (col + e < N) wdst[e] = (__bf16)(pr.s0 * (float)wdst[e] - pr.s1 * (e < 4 ? lo[e & 3] : hi[e & 3]));
              continue;
            }
            bf16x8 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              o[e] = (__bf16)(pr.s0 * (float)wpre[i][q][ps][e] - pr.s1 * lo[e]);
              o[e + 4] = (__bf16)(pr.s0 * (float)wpre[i][q][ps][e + 4] - pr.s1 * hi[e]);
            }
            if (W_ANY) __builtin_memcpy(wdst, &o, sizeof(bf16x8));
            else __builtin_nontemporal_store(__builtin_bit_cast(i32x4, o), reinterpret_cast<i32x4*>(wdst));
          } else {
            float* C = static_cast<float*>(pr.C);
            float* dst = C + (size_t)row * ldc + col;
            *reinterpret_cast<f32x4*>(dst) = lo;
            *reinterpret_cast<f32x4*>(dst + 4) = hi;
            if (EPI == Epilogue::StoreSymF32 && cur.tm != cur.tn) {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                C[(size_t)(col + e) * ldc + row] = lo[e];
                C[(size_t)(col + e + 4) * ldc + row] = hi[e];
              }
            }
          }
        }
      }
    }

    if (!have_next) break;
    cur = nxt;
  }
}

// Number of workgroups of the persistent grid: one per CU, a multiple of 8 (one share per XCD).
inline int dl_grid_size(int total_tiles) {
  static int cus = 0;
  if (cus == 0) {
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess && prop.multiProcessorCount >= 8)
      cus = prop.multiProcessorCount & ~7;
    else
      cus = 256;
  }
  const int want = (total_tiles + 7) & ~7;
  return want < cus ? want : cus;
}

template <bool AK, bool BKC, Epilogue EPI, class Cfg, bool W_ANY = false>
inline hipError_t launch_gemm_dl_instance(const GemmGroup& g, hipStream_t stream) {
  using AOp = DlOperand<AK, Cfg::BM, Cfg::BK, Cfg::NW>;
  using BOp = DlOperand<BKC, Cfg::BN, Cfg::BK, Cfg::NW>;
  constexpr size_t smem = (size_t)Cfg::STAGES * (AOp::TILE_BYTES + BOp::TILE_BYTES) +
                          (size_t)Cfg::NW * 8 * (Cfg::WN + 8) * sizeof(float);  // tile ring + epilogue strips
  static_assert(smem <= 160 * 1024, "tile ring and strips do not fit the 160 KB LDS");
  auto kern = gemm_dl_kernel<AK, BKC, EPI, Cfg, W_ANY>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  hipLaunchKernelGGL(kern, dim3(dl_grid_size(g.total_tiles)), dim3(Cfg::NT), smem, stream, g);
  return hipGetLastError();
}

// The direct-load kernel needs 16-byte alignment of both operands and of the output (its
// epilogue moves 8 consecutive columns per lane), K a multiple of 64, N a multiple of 8, and at
// least 8 valid elements along each M/N index (for the edge clamp).
// With w_any (the weight update with B contiguous along K: no operand is cut into pieces along N)
// the output may have any row length, leading dimension and element alignment.
inline bool group_fits_dl(const GemmGroup& g, bool ak, bool bk, Epilogue epi, int bk_step = 64, bool w_any = false) {
  if (!group_is_aligned<__bf16>(g, ak, bk)) return false;
  if (w_any && (epi != Epilogue::ApplyW || !bk)) return false;
  const int c_vec = epi == Epilogue::ApplyW ? 8 : 4;  // elements per 16 bytes of the output
  for (int i = 0; i < g.count; ++i) {
    const GemmProblem& p = g.p[i];
    if (p.K % bk_step != 0 || p.K < bk_step) return false;
    if (p.M < 8 || p.N < 8 || (!w_any && p.N % 8 != 0)) return false;
    if (w_any ? (p.ldc < p.N || (reinterpret_cast<uintptr_t>(p.C) & 1)) : ((reinterpret_cast<uintptr_t>(p.C) & 15) || p.ldc % c_vec != 0)) return false;
    // the tile loads address an operand with 32-bit byte offsets from its first element
    const uint64_t a_outer = ak ? (uint64_t)p.M : (uint64_t)p.K, b_outer = bk ? (uint64_t)p.N : (uint64_t)p.K;
    if (a_outer * (uint64_t)p.lda * 2 > 0xFFFFFFFFull || b_outer * (uint64_t)p.ldb * 2 > 0xFFFFFFFFull) return false;
  }
  return true;
}

}  // namespace galore
