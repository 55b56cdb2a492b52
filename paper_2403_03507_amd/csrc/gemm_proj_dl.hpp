// Projection GEMM of the GaLore step, R = P^T G and R = G Q in ONE persistent launch (gfx950, bf16 operands,
// fp32 result).  Built from the parts of the large-tile kernel in gemm_mfma_dl.hpp (direct global -> LDS tile
// loads, swizzled unpadded LDS rows, two-stage ring, 256 x 256 x 64 tiles of 8 waves, strip epilogue) with three
// differences that matter for this stage of Algorithm 2:
//   * the layout of the B operand is a field of each problem, not a template parameter: LEFT tensors (B = G,
//     contiguous along N, LDS transpose reads) and RIGHT tensors (B = the transposed projector, contiguous along
//     K) share the launch, so the 172 tiles of a 7B layer's RIGHT tensor no longer run alone on 256 CUs;
//   * a work item is a tile AND a range of K steps.  The tiles that fill whole rounds of the grid run over the
//     whole K range and store R.  The tiles left over (4 of 772 for a 7B layer, every tile of a small stack) are
//     cut into `pieces` K ranges, one item each, spread over the CUs; each piece stores its partial tile in a
//     slab and proj_reduce_kernel adds the slabs in a fixed order afterwards (no atomics, no waiting between
//     workgroups, bit-identical from run to run);
//   * the K steps of consecutive items form one stream through the ring, as in the large-tile kernel;
//   * FUSE: the update block of Algorithm 2 (moments, bias correction, N) runs in the epilogue on the
//     accumulators themselves, so R never travels to memory and back (8 of the 22 bytes per entry the separate
//     Adam kernel moves).  The accumulator layout serves as it is: a lane holds one column and groups of four
//     consecutive rows, so M and V are read and written as 128-byte row segments per half-wave, and N leaves
//     transposed (LEFT tensors) as 8-byte pieces of four consecutive r, or row-wise (RIGHT tensors).
#pragma once
#include <type_traits>

#include "adam_entry.hpp"
#include "gemm_mfma_dl.hpp"

namespace galore {

// One work item as seen by the workgroup that computes it (all wave-uniform).
struct ProjItem {
  int pi;        // problem
  int m0, n0;    // tile origin
  int k0, k1;    // K steps [k0, k1)
  float* dst;    // where element (0, 0) of the tile goes
  int ldc;       // row stride of dst
  int rows, cols;  // valid extent from the tile origin (may exceed the tile)
  int bkc;       // layout of B
  int kind;      // kWhole or kPiece
  int seq;       // position in the workgroup's item sequence
};
enum : int { kWhole = 0, kPiece = 1 };

template <class Cfg, bool FUSE>
__global__ __launch_bounds__(Cfg::NT) void proj_dl_kernel(const ProjGroup grp) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN, BK = Cfg::BK, NW = Cfg::NW, S = Cfg::STAGES;
  constexpr int TM = Cfg::TM, TN = Cfg::TN, WN = Cfg::WN;
  using AOp = DlOperand<true, BM, BK, NW>;
  using BOpK = DlOperand<true, BN, BK, NW>;
  using BOpX = DlOperand<false, BN, BK, NW>;
  static_assert(BOpK::TILE_BYTES == BOpX::TILE_BYTES && BOpK::PER_WAVE == BOpX::PER_WAVE, "both layouts fill the same stage");
  constexpr int STAGE_BYTES = AOp::TILE_BYTES + BOpK::TILE_BYTES;
  constexpr int RING_BYTES = S * STAGE_BYTES;
  static_assert(S == 2 && BK == 64, "written for a two-stage ring of 64-wide K steps");
  static_assert(WN == 64 || WN == 128, "the strip epilogue covers 8 rows with one or two passes of the wave");
  constexpr int PITCH = WN + 8;
  constexpr int STRIP_FLOATS = 8 * PITCH;
  constexpr int LPR = WN / 8;
  constexpr int RPP = 64 / LPR;
  constexpr int PASSES = 8 / RPP;

  extern __shared__ __align__(1024) unsigned char smem_dl[];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm0 = (wave % Cfg::WGM) * Cfg::WM;
  const int wn0 = (wave / Cfg::WGM) * Cfg::WN;

  // ---- work items of this workgroup: at most one split piece, then its share of the regular tiles ----
  const int regular = grp.regular_tiles;
  const int n_split_items = (grp.total_tiles - regular) * grp.pieces;
  const int per_xcd = gridDim.x >> 3;
  const int xcd = blockIdx.x & 7, q_in_xcd = blockIdx.x >> 3;
  const int share = regular >> 3, extra = regular & 7;
  const int first_id = xcd * share + (xcd < extra ? xcd : extra);
  const int n_ids = share + (xcd < extra ? 1 : 0);
  auto tile_item = [&](int id, ProjItem& t) {
    int pi = 0;
    for (int i = 1; i < grp.count; ++i)
      if (id >= grp.p[i].tile_begin) pi = i;
    const ProjProblem& p = grp.p[pi];
    int tm, tn;
    tile_coords(id - p.tile_begin, p.tiles_m, p.tiles_n, tm, tn);
    t.pi = pi; t.m0 = tm * BM; t.n0 = tn * BN;
    t.k0 = 0; t.k1 = p.K / BK;
    t.dst = p.R + (size_t)t.m0 * p.ldr + t.n0;
    t.ldc = p.ldr;
    t.rows = p.M - t.m0; t.cols = p.N - t.n0;
    t.bkc = p.b_kcontig;
  };
  // Item sequence of this workgroup: [piece] one K piece of a leftover tile (blockIdx < n_split_items), whose partial
  // tile goes to a row-major slab; then its regular tiles, round after round.
  const int has_piece = (int)blockIdx.x < n_split_items ? 1 : 0;
  const int n_rounds = q_in_xcd < n_ids ? (n_ids - q_in_xcd + per_xcd - 1) / per_xcd : 0;
  auto item_at = [&](int seq, ProjItem& t) -> bool {
    t.seq = seq;
    if (has_piece && seq == 0) {
      const int j = blockIdx.x;
      tile_item(regular + j / grp.pieces, t);
      const int sp = j % grp.pieces, KT = t.k1;
      t.k0 = (int)((long long)sp * KT / grp.pieces);
      t.k1 = (int)((long long)(sp + 1) * KT / grp.pieces);
      t.dst = grp.slabs + (size_t)j * (BM * BN);
      t.ldc = BN;
      t.kind = kPiece;
      return true;
    }
    const int s = seq - has_piece;  // position among the regular items
    if (s >= n_rounds) return false;
    tile_item(first_id + s * per_xcd + q_in_xcd, t);
    t.kind = kWhole;
    return true;
  };

  ProjItem cur;
  if (!item_at(0, cur)) return;

  // ---- load side ----
  AOp opa;
  unsigned bvoff[BOpK::PER_WAVE];  // one plan for B, whichever layout the tile being requested has
  int ld_bkc = 1;  // layout of the tile whose K steps are being requested
  const unsigned char* a_src = nullptr;
  const unsigned char* b_src = nullptr;
  size_t a_step = 0, b_step = 0;
  auto bind = [&](const ProjItem& t) {
    const ProjProblem& p = grp.p[t.pi];
    opa.plan(p.lda, t.m0, p.M, wave, lane);
    ld_bkc = t.bkc;
    if (ld_bkc) BOpK::plan_into(bvoff, p.ldb, t.n0, p.N, wave, lane);
    else BOpX::plan_into(bvoff, p.ldb, t.n0, p.N, wave, lane);
    a_src = static_cast<const unsigned char*>(p.A);
    b_src = static_cast<const unsigned char*>(p.B);
    a_step = (size_t)BK * 2;
    b_step = ld_bkc ? (size_t)BK * 2 : (size_t)BK * p.ldb * 2;
  };
  const unsigned lds0 = (unsigned)(uintptr_t)smem_dl;
  // G of a LEFT tensor is shared by the four tile rows of a band at the same time and never needed again:
  // streamed, so that it does not displace the projector panels from L2
  auto issue_step_as = [&](auto layout, int kt, int stage) {  // layout known at compile time: inside an item's K loop
    constexpr bool BKC = decltype(layout)::value;
    const unsigned st = lds0 + stage * STAGE_BYTES;
    opa.template issue<false>(a_src + kt * a_step, st, wave);
    if (BKC) BOpK::template issue_from<false>(bvoff, b_src + kt * b_step, st + AOp::TILE_BYTES, wave);
    else BOpX::template issue_from<true>(bvoff, b_src + kt * b_step, st + AOp::TILE_BYTES, wave);
  };
  auto issue_step = [&](int kt, int stage) {  // layout of the tile last bound
    if (ld_bkc) issue_step_as(std::true_type{}, kt, stage);
    else issue_step_as(std::false_type{}, kt, stage);
  };

  bind(cur);
  issue_step(cur.k0, 0);
  int g = 0;  // K steps consumed so far, over all items: step g lives in stage g & 1

  for (;;) {
    ProjItem nxt;
    const bool have_next = item_at(cur.seq + 1, nxt);
    const int L = cur.k1 - cur.k0;

    f32x16 acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // The K steps of an item, software-pipelined as in the large-tile kernel: the fragments of the next 16 k are
    // read from LDS while the MFMAs of the current 16 k execute, and the MFMAs of a step's last 16 k are deferred
    // past the next step's barrier.  At the top of a step everything this wave requested has landed and its own
    // LDS reads of the other stage have returned; after the barrier the other stage can be refilled.
    auto run = [&](auto layout) {
      constexpr bool BKC = decltype(layout)::value;
      using BOp = typename std::conditional<BKC, BOpK, BOpX>::type;
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
      constexpr int NREADS = TM + TN * (BKC ? 1 : 2);
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
      auto request_next = [&](int s) {
        if (s + 1 < L) {
          issue_step_as(layout, cur.k0 + s + 1, (g + 1) & 1);
        } else if (have_next) {  // the first K step of the next item: its latency and this item's epilogue hide behind it
          bind(nxt);
          issue_step(nxt.k0, (g + 1) & 1);
        }
      };

      __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) and lgkmcnt(0)
      __syncthreads();
      request_next(0);
      read_frags(g & 1, 0, fa0, fb0);
      read_frags(g & 1, 16, fa1, fb1); mma(fa0, fb0); interleave();
      read_frags(g & 1, 32, fa0, fb0); mma(fa1, fb1); interleave();
      read_frags(g & 1, 48, fa1, fb1); mma(fa0, fb0); interleave();
      ++g;
      for (int s = 1; s < L; ++s) {
        __builtin_amdgcn_s_waitcnt(0x0070);
        __syncthreads();
        request_next(s);
        read_frags(g & 1, 0, fa0, fb0); mma(fa1, fb1); interleave();
        read_frags(g & 1, 16, fa1, fb1); mma(fa0, fb0); interleave();
        read_frags(g & 1, 32, fa0, fb0); mma(fa1, fb1); interleave();
        read_frags(g & 1, 48, fa1, fb1); mma(fa0, fb0); interleave();
        ++g;
      }
      mma(fa1, fb1);
    };
    if (cur.bkc) run(std::true_type{});
    else run(std::false_type{});

    if (FUSE && cur.kind != kPiece) {
      // ---- fused epilogue: Adam on the accumulators (tiles summed over their whole K range; pieces go to their slabs below) ----
      const ProjProblem& p = grp.p[cur.pi];
      float* Mp = p.Mo;
      float* Vp = p.Vo;
      __bf16* Np = static_cast<__bf16*>(p.Nout);
      const int ldm = p.ldm, ldn = p.ldn;
      const int rows = cur.rows, colsv = p.cols_valid - cur.n0;
      const float b1 = grp.beta1, b2 = grp.beta2, eps = grp.eps, ic1 = p.inv_c1, ic2 = p.inv_c2;
      const bool ntr = p.n_transposed != 0;
      const bool nvec = ntr && (ldn & 3) == 0 && (reinterpret_cast<uintptr_t>(Np) & 7) == 0;
      // (lane-dependent values of the epilogue are derived behind a compiler barrier: hoisted out of the item loop
      // they would stay live across the K loop, whose register budget has no room for them)
      int le = lane;
      asm volatile("" : "+v"(le));
      const int lrow = wm0 + 4 * (le >> 5), lcol = wn0 + (le & 31);
      // entry (i, q, j, c) of this lane: row lrow + 32 i + 8 q + c, column lcol + 32 j
      // 32-bit element offsets from uniform base pointers (the launcher checks that the moments span < 2^32 bytes):
      // one lane-dependent register, everything that varies with (i, q, j, c) is wave-uniform
      const unsigned mv0 = (unsigned)(cur.m0 + lrow) * (unsigned)ldm + (unsigned)(cur.n0 + lcol);
      const unsigned mv_safe = (unsigned)cur.m0 * (unsigned)ldm + (unsigned)cur.n0;  // the tile's first entry: always inside
      // The moments come from HBM, one group of entries ahead of the update (DEPTH = 2).  The epilogue is then a chain
      // of 16 memory round trips per tile (measured: 56 us, 20 GB/s per CU); more groups in flight need registers the
      // kernel does not have (DEPTH = 4 spills and measured slower).
      constexpr int DEPTH = 2;
      float mb[DEPTH][TN * 4], vb[DEPTH][TN * 4];
      auto fetch = [&](int i, int q, float (&m)[TN * 4], float (&v)[TN * 4]) {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const int ro = 32 * i + 8 * q + c;
            const bool ok = lrow + ro < rows && lcol + 32 * j < colsv;  // lanes outside the matrix read the safe entry and store nothing
            const unsigned off = ok ? mv0 + (unsigned)ro * (unsigned)ldm + 32u * j : mv_safe;
            m[j * 4 + c] = __builtin_nontemporal_load(Mp + off);
            v[j * 4 + c] = __builtin_nontemporal_load(Vp + off);
          }
      };
      auto apply = [&](int i, int q, float (&m)[TN * 4], float (&v)[TN * 4]) {
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          const int col = lcol + 32 * j;
          const int row0 = lrow + 32 * i + 8 * q;
          float n[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            float me = m[j * 4 + c], ve = v[j * 4 + c];
            n[c] = adam_entry(acc[i][j][4 * q + c], me, ve, b1, b2, eps, ic1, ic2);
            if (row0 + c < rows && col < colsv) {
              const unsigned off = mv0 + (unsigned)(32 * i + 8 * q + c) * (unsigned)ldm + 32u * j;
              __builtin_nontemporal_store(me, Mp + off);
              __builtin_nontemporal_store(ve, Vp + off);
            }
          }
          if (col >= colsv) continue;
          if (ntr) {  // N^T[col][row]: four consecutive rows are 8 contiguous bytes
            __bf16* dst = Np + (size_t)(cur.n0 + col) * ldn + cur.m0 + row0;
            if (nvec && row0 + 3 < rows) {
              bf16x4 o;
              o[0] = (__bf16)n[0]; o[1] = (__bf16)n[1]; o[2] = (__bf16)n[2]; o[3] = (__bf16)n[3];
              *reinterpret_cast<bf16x4*>(dst) = o;
            } else {
#pragma unroll
              for (int c = 0; c < 4; ++c)
                if (row0 + c < rows) dst[c] = (__bf16)n[c];
            }
          } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
              if (row0 + c < rows) Np[(size_t)(cur.m0 + row0 + c) * ldn + cur.n0 + col] = (__bf16)n[c];
          }
        }
      };
      // the moments of the next group of entries are in flight while this group is updated
#pragma unroll
      for (int gq = 0; gq < DEPTH - 1; ++gq) fetch(gq >> 2, gq & 3, mb[gq], vb[gq]);
#pragma unroll
      for (int gq = 0; gq < TM * 4; ++gq) {
        constexpr int AHEAD = DEPTH - 1;
        if (gq + AHEAD < TM * 4) fetch((gq + AHEAD) >> 2, (gq + AHEAD) & 3, mb[(gq + AHEAD) % DEPTH], vb[(gq + AHEAD) % DEPTH]);
        __builtin_amdgcn_sched_barrier(0);  // keep the loads ahead of the update they overlap with
        apply(gq >> 2, gq & 3, mb[gq % DEPTH], vb[gq % DEPTH]);
      }
    } else {
    // ---- epilogue: accumulators -> wave-private LDS strip -> 32 contiguous bytes per lane ----
    // (the strip area lies outside the ring, which keeps receiving the next item's first K step meanwhile;
    // LDS operations of one wave execute in order, so the strip can be rewritten right after it was read)
      int le = lane;
      asm volatile("" : "+v"(le));
      float* strip = reinterpret_cast<float*>(smem_dl + RING_BYTES) + wave * STRIP_FLOATS;
      const int rr = le / LPR, cc = (le % LPR) * 8;
      float* dst0 = cur.dst;
      const int ldc = cur.ldc;
      const int col = wn0 + cc;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
#pragma unroll
          for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int c = 0; c < 4; ++c)
              strip[(4 * (le >> 5) + c) * PITCH + 32 * j + (le & 31)] = acc[i][j][4 * q + c];
#pragma unroll
          for (int ps = 0; ps < PASSES; ++ps) {
            const float* src = strip + (rr + RPP * ps) * PITCH + cc;
            const f32x4 lo = *reinterpret_cast<const f32x4*>(src);
            const f32x4 hi = *reinterpret_cast<const f32x4*>(src + 4);
            const int row = wm0 + rr + 32 * i + 8 * q + RPP * ps;
            if (row >= cur.rows || col >= cur.cols) continue;
            float* dst = dst0 + (size_t)row * ldc + col;
            *reinterpret_cast<f32x4*>(dst) = lo;
            *reinterpret_cast<f32x4*>(dst + 4) = hi;
          }
        }
      }
    }

    if (!have_next) break;
    cur = nxt;
  }
}

// R tile = sum of its `pieces` slabs, in slab order.  blockIdx.y = split tile, blockIdx.x strides over the tile.
// FUSE: the sums go into the update block of Algorithm 2 instead of into R (same expression as everywhere else).
template <class Cfg, bool FUSE>
__global__ __launch_bounds__(256) void proj_reduce_kernel(const ProjGroup grp) {
  constexpr int BM = Cfg::BM, BN = Cfg::BN;
  const int id = grp.regular_tiles + blockIdx.y;
  int pi = 0;
  for (int i = 1; i < grp.count; ++i)
    if (id >= grp.p[i].tile_begin) pi = i;
  const ProjProblem& p = grp.p[pi];
  int tm, tn;
  tile_coords(id - p.tile_begin, p.tiles_m, p.tiles_n, tm, tn);
  const int m0 = tm * BM, n0 = tn * BN;
  const int rows = p.M - m0 < BM ? p.M - m0 : BM;
  const int cols = p.N - n0 < BN ? p.N - n0 : BN;  // a multiple of 4 (N is a multiple of 8)
  const float* slab = grp.slabs + (size_t)blockIdx.y * grp.pieces * (BM * BN);
  for (int e = blockIdx.x * 256 + threadIdx.x; e < BM * BN / 4; e += gridDim.x * 256) {
    const int row = e / (BN / 4), c4 = (e % (BN / 4)) * 4;
    if (row >= rows || c4 >= cols) continue;
    // all slabs of the entry are requested together (a slab index beyond `pieces` re-reads slab 0 and is not
    // added): one memory round trip instead of one per slab; the sum keeps the slab order
    constexpr int kMaxPieces = 16;
    f32x4 x[kMaxPieces];
#pragma unroll
    for (int s = 0; s < kMaxPieces; ++s)
      x[s] = *reinterpret_cast<const f32x4*>(slab + (size_t)(s < grp.pieces ? s : 0) * (BM * BN) + (size_t)row * BN + c4);
    f32x4 sum = x[0];
#pragma unroll
    for (int s = 1; s < kMaxPieces; ++s)
      if (s < grp.pieces) { sum[0] += x[s][0]; sum[1] += x[s][1]; sum[2] += x[s][2]; sum[3] += x[s][3]; }
    if (FUSE) {
      __bf16* Np = static_cast<__bf16*>(p.Nout);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const int col = n0 + c4 + c;
        if (col >= p.cols_valid) continue;
        const size_t idx = (size_t)(m0 + row) * p.ldm + col;
        float me = p.Mo[idx], ve = p.Vo[idx];
        const float n = adam_entry(sum[c], me, ve, grp.beta1, grp.beta2, grp.eps, p.inv_c1, p.inv_c2);
        p.Mo[idx] = me; p.Vo[idx] = ve;
        if (p.n_transposed) Np[(size_t)col * p.ldn + m0 + row] = (__bf16)n;
        else Np[(size_t)(m0 + row) * p.ldn + col] = (__bf16)n;
      }
    } else {
      *reinterpret_cast<f32x4*>(p.R + (size_t)(m0 + row) * p.ldr + n0 + c4) = sum;
    }
  }
}

}  // namespace galore
