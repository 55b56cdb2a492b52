// Shared declarations of the GaLore HIP library (gfx950 only): grouped-launch
// descriptors passed by value as kernel arguments, and the host launchers the C ABI calls.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace galore {

constexpr int kMaxGroup = 16;  // problems per grouped launch (descriptor table lives in kernarg)

enum class DType : int32_t { F32 = 0, BF16 = 1 };

inline size_t dtype_size(DType d) { return d == DType::F32 ? 4 : 2; }

// ---- grouped GEMM ------------------------------------------------------------------------
// C[M x N] (+epilogue) = A * B, fp32 accumulate.  A is read as a_kcontig ? [M][K] : [K][M],
// B as b_kcontig ? [N][K] : [K][N]; lda/ldb are the strides (elements) of the outer index.
struct GemmProblem {
  const void* A;
  const void* B;
  void* C;        // output / in-place operand of the epilogue
  void* aux0;     // epilogue extra pointers
  void* aux1;
  void* aux2;
  int32_t M, N, K;
  int32_t lda, ldb, ldc;
  int32_t tile_begin;  // first block of this problem in the launch
  int32_t tiles_m;     // tiles along M and N; tile ids are decoded by tile_coords()
  int32_t tiles_n;
  float s0, s1, s2, s3;  // epilogue scalars
};

struct GemmGroup {
  int32_t count;
  int32_t total_tiles;
  GemmProblem p[kMaxGroup];
};

enum class Epilogue : int32_t {
  StoreF32 = 0,   // C (fp32) = acc
  ApplyW = 1,     // C (T) = s0 * C - s1 * acc            (weight update, s0 = 1 - lr*wd, s1 = lr*alpha)
  StoreSymF32 = 2 // C (fp32) = acc, written to (i,j) and (j,i); tiles with tm > tn skipped (M == N)
};

// Launch one grouped GEMM on `stream`.  All problems share dtype / layouts / epilogue.
// Host fills everything except tile_begin / tiles_m / total_tiles.
hipError_t launch_gemm_group(GemmGroup& g, DType dt, bool a_kcontig, bool b_kcontig, Epilogue epi,
                             hipStream_t stream);

// ---- grouped projection GEMM (bf16 operands, fp32 result): R = A * B with A as [M][K] -------------------
// LEFT tensors:  A = the transposed projector (r x m), B = G as [K = m][N = n]  (b_kcontig = 0)
// RIGHT tensors: A = G (m x n),                       B = the transposed projector as [N = r][K = n] (b_kcontig = 1)
struct ProjProblem {
  const void* A;
  const void* B;
  float* R;       // M x N, row stride ldr
  int32_t M, N, K;
  int32_t lda, ldb, ldr;
  int32_t b_kcontig;
  int32_t tile_begin, tiles_m, tiles_n;  // filled by the launcher
  // Adam in the epilogue (launch_proj_group with fuse_adam): R is not stored; the tile's entries go straight
  // into the update block of Algorithm 2.  Mo, Vo: fp32 moments with R's shape (row stride ldm, cols_valid <= N
  // columns: R may carry padded columns); Nout: bf16, n_transposed ? cols_valid x M (row stride ldn) : M x cols_valid.
  float* Mo;
  float* Vo;
  void* Nout;
  int32_t ldm, ldn, cols_valid, n_transposed;
  float inv_c1, inv_c2;
};

struct ProjGroup {
  int32_t count;
  int32_t total_tiles;
  int32_t regular_tiles;  // tiles [0, regular_tiles) run over their whole K range on the persistent grid
  int32_t pieces;         // the remaining tiles are cut into this many K ranges, one work item each
  float* slabs;           // partial tiles of the pieces (tile-local row-major, fp32), summed by the reduce kernel
  float beta1, beta2, eps;  // fused Adam only
  ProjProblem p[kMaxGroup];
};

// True if the problem meets the kernel's rules (16-byte aligned operands and rows, K a multiple of 64, ...);
// problems that do not go through launch_gemm_group.
bool proj_problem_fits(const ProjProblem& p);
// Launch one grouped projection; every problem must fit.  `slabs` (256-byte aligned, slab_bytes long, may be
// NULL / 0) is scratch for the partial tiles; without enough of it the launch simply runs whole tiles only.
// fuse_adam: every problem carries Mo, Vo, Nout, ...; M, V are updated and N written by the GEMM's epilogue (and by
// the kernel that sums the partial tiles), R is left untouched.
hipError_t launch_proj_group(ProjGroup& g, float* slabs, size_t slab_bytes, hipStream_t stream, bool fuse_adam = false);

// ---- grouped low-rank Adam -----------------------------------------------------------------
struct AdamProblem {
  const float* R;
  float* M;
  float* V;
  void* N;        // fp32 or bf16
  int64_t count;  // rows * cols
  int32_t rows;   // shape of R, M, V (M, V dense, row-major)
  int32_t cols;
  int32_t ldr;    // row stride of R, >= cols (only the transposing kernel takes R with padded rows; else ldr == cols)
  int32_t transpose_n;  // 0: N has R's layout; 1: N is stored transposed (cols x rows)
  float inv_c1;   // 1 / (1 - beta1^k)
  float inv_c2;   // 1 / (1 - beta2^k)
};

struct AdamGroup {
  int32_t count;
  float beta1, beta2, eps;
  AdamProblem p[kMaxGroup];
};

// All problems of a group share n_dtype and transpose_n.
hipError_t launch_adam_group(const AdamGroup& g, DType n_dtype, hipStream_t stream);

// ---- grouped low-rank Adam with 8-bit block-wise moments ------------------------------------------
// Moments are stored as one byte per element plus one fp32 scale per block of 256 consecutive
// elements of the row-major matrix; cols must be a multiple of 256 so that a block never
// straddles two rows.
struct AdamQ8Problem {
  const float* R;
  uint8_t* Mc;     // first-moment codes: sign, 4 exponent bits, 3 mantissa bits
  uint8_t* Vc;     // second-moment codes: 5 exponent bits, 3 mantissa bits
  float* Ms;       // per block: max |m|
  float* Vs;       // per block: max v
  void* N;         // fp32 or bf16
  int32_t rows;    // shape of R and of the code matrices (dense, row-major)
  int32_t cols;
  int32_t transpose_n;
  float inv_c1, inv_c2;
};

struct AdamQ8Group {
  int32_t count;
  float beta1, beta2;
  float omb1, omb2;  // 1 - beta, formed in fp32 on the host
  float eps;
  AdamQ8Problem p[kMaxGroup];
};

hipError_t launch_adam_q8_group(const AdamQ8Group& g, DType n_dtype, hipStream_t stream);

// ---- grouped matrix transpose (projector k x r -> r x k) ------------------------------------
struct TransposeProblem {
  const void* src;  // rows x cols, leading dimension lds
  void* dst;        // cols x rows, leading dimension ldd
  int32_t rows, cols, lds, ldd;
};
struct TransposeGroup {
  int32_t count;
  TransposeProblem p[kMaxGroup];
};
hipError_t launch_transpose_group(const TransposeGroup& g, DType dt, hipStream_t stream);

// ---- grouped row padding (bf16): dst (rows x ldd, 16-byte aligned, ldd % 8 == 0) <- src (rows x cols, any
// row stride and element alignment), columns cols .. ldd - 1 zero ------------------------------
struct PadProblem {
  const void* src;
  void* dst;
  int32_t rows, cols, lds, ldd;
};
struct PadGroup {
  int32_t count;
  PadProblem p[kMaxGroup];
};
hipError_t launch_pad_rows_group(const PadGroup& g, hipStream_t stream);

// ---- small utilities -----------------------------------------------------------------------
hipError_t launch_fill_zero(void* ptr, size_t bytes, hipStream_t stream);
// dst (rows x cols, leading dimension ldd, dtype dt) <- src (dense fp32), rounded to nearest even
hipError_t launch_cast_rows(const float* src, void* dst, int rows, int cols, int ldd, DType dt, hipStream_t stream);
// the same with every row scaled to unit Euclidean length (a zero row stays zero)
hipError_t launch_normalize_rows(const float* src, void* dst, int rows, int cols, int ldd, DType dt, hipStream_t stream);

}  // namespace galore
