// Host-side helpers shared by the translation units of the C ABI (api.hip: context and step; api_stages.hip: the
// stateless stage calls; api_two_sided.hip: the two-sided rule of Definition 3.6): status / message plumbing and
// the argument checks every entry point runs before it launches anything.
#pragma once
#include "../../include/galore.h"
#include "common.hpp"

#include <cstddef>

struct galore_ctx;

namespace galore {
namespace api {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Records the message (in ctx when given, and in the calling thread's slot read by galore_last_error(NULL)) and returns s.
galore_status fail(galore_ctx* ctx, galore_status s, const char* fmt, ...);
galore_status hip_fail(galore_ctx* ctx, hipError_t e, const char* where);
galore_status check_hparams(galore_ctx* ctx, const galore_hparams* hp);
galore_status check_matrix(galore_ctx* ctx, const galore_tensor& t, const char* what, int idx, bool need_data, bool allow_u8 = false);
galore_status check_weight_shape(galore_ctx* ctx, const galore_hparams& hp, const galore_tensor& w, int idx);

// One problem on the grouped kernels (the context-free calls work on one tensor at a time).
// C (fp32, M x N dense) = A B with A as [M][K]; B as [N][K] (b_kcontig) or [K][N]
inline hipError_t single_gemm_store(DType dt, const void* A, int lda, const void* B, int ldb, bool b_kcontig, float* C, int M, int N, int K,
                          hipStream_t stream) {
  GemmGroup g{};
  g.count = 1;
  GemmProblem& p = g.p[0];
  p.A = A; p.lda = lda; p.B = B; p.ldb = ldb;
  p.M = M; p.N = N; p.K = K;
  p.C = C; p.ldc = N;
  return launch_gemm_group(g, dt, true, b_kcontig, Epilogue::StoreF32, stream);
}

inline hipError_t single_transpose(DType dt, const void* src, int rows, int cols, int lds, void* dst, int ldd, hipStream_t stream) {
  TransposeGroup g{};
  g.count = 1;
  g.p[0].src = src; g.p[0].rows = rows; g.p[0].cols = cols; g.p[0].lds = lds;
  g.p[0].dst = dst; g.p[0].ldd = ldd;
  return launch_transpose_group(g, dt, stream);
}

}  // namespace api
}  // namespace galore
