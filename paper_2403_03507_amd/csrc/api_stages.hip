// The stateless stage calls of the C ABI: the three per-step stages of Algorithm 2 (and the projector transpose) on
// one tensor, through the same launchers galore_step uses.  Validation, then one grouped launch of one problem.
#include "api_internal.hpp"

#include <cmath>

using namespace galore;
using namespace galore::api;

extern "C" {

// ---- stateless stage calls ---------------------------------------------------------------------

galore_status galore_transpose(const galore_tensor* src, const galore_tensor* dst, void* hip_stream) {
  if (!src || !dst) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  galore_status s;
  if ((s = check_matrix(nullptr, *src, "src", 0, true)) || (s = check_matrix(nullptr, *dst, "dst", 0, true))) return s;
  if (src->dtype != dst->dtype) return fail(nullptr, GALORE_ERR_DTYPE, "src and dst dtypes differ");
  if (dst->rows != src->cols || dst->cols != src->rows) return fail(nullptr, GALORE_ERR_SHAPE, "dst must be cols x rows of src");
  TransposeGroup g{};
  g.count = 1;
  g.p[0].src = src->data; g.p[0].lds = (int)src->ld; g.p[0].dst = dst->data; g.p[0].ldd = (int)dst->ld;
  g.p[0].rows = (int)src->rows; g.p[0].cols = (int)src->cols;
  hipError_t e = launch_transpose_group(g, (DType)src->dtype, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "transpose launch");
}

galore_status galore_project(const galore_tensor* proj_t, const galore_tensor* G, const galore_tensor* R, void* hip_stream) {
  if (!proj_t || !G || !R) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  galore_status s;
  if ((s = check_matrix(nullptr, *proj_t, "proj_t", 0, true)) || (s = check_matrix(nullptr, *G, "G", 0, true)) ||
      (s = check_matrix(nullptr, *R, "R", 0, true)))
    return s;
  if (proj_t->dtype != G->dtype) return fail(nullptr, GALORE_ERR_DTYPE, "proj_t and G dtypes differ");
  if (R->dtype != GALORE_F32) return fail(nullptr, GALORE_ERR_DTYPE, "R must be fp32");
  const bool left = G->rows <= G->cols;
  const int64_t r = proj_t->rows;
  if (r > (left ? G->rows : G->cols)) return fail(nullptr, GALORE_ERR_RANK, "rank exceeds the short side");
  if (proj_t->cols != (left ? G->rows : G->cols)) return fail(nullptr, GALORE_ERR_SHAPE, "proj_t cols must equal the short side of G");
  if (R->rows != (left ? r : G->rows) || R->cols != (left ? G->cols : r))
    return fail(nullptr, GALORE_ERR_SHAPE, "R has the wrong shape");
  GemmGroup g{};
  g.count = 1;
  GemmProblem& p = g.p[0];
  if (left) {
    p.A = proj_t->data; p.lda = (int)proj_t->ld; p.B = G->data; p.ldb = (int)G->ld;
    p.M = (int)r; p.N = (int)G->cols; p.K = (int)G->rows;
  } else {
    p.A = G->data; p.lda = (int)G->ld; p.B = proj_t->data; p.ldb = (int)proj_t->ld;
    p.M = (int)G->rows; p.N = (int)r; p.K = (int)G->cols;
  }
  p.C = R->data; p.ldc = (int)R->ld;
  // the kernel galore_step uses for this tensor: the grouped projection where its rules are met, else the general GEMM
  ProjGroup pg{};
  ProjProblem& q = pg.p[0];
  q.A = p.A; q.B = p.B; q.R = static_cast<float*>(p.C);
  q.M = p.M; q.N = p.N; q.K = p.K; q.lda = p.lda; q.ldb = p.ldb; q.ldr = p.ldc;
  q.b_kcontig = left ? 0 : 1;
  hipError_t e;
  if ((DType)G->dtype == DType::BF16 && proj_problem_fits(q)) {
    pg.count = 1;
    e = launch_proj_group(pg, nullptr, 0, static_cast<hipStream_t>(hip_stream));
  } else {
    e = launch_gemm_group(g, (DType)G->dtype, true, !left, Epilogue::StoreF32, static_cast<hipStream_t>(hip_stream));
  }
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "projection GEMM launch");
}

galore_status galore_adam(const galore_tensor* R, const galore_tensor* M, const galore_tensor* V, const galore_tensor* N,
                          int32_t transpose_n, float beta1, float beta2, float eps, int64_t k, void* hip_stream) {
  if (!R || !M || !V || !N) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  const galore_tensor* all[4] = {R, M, V, N};
  const char* names[4] = {"R", "M", "V", "N"};
  for (int i = 0; i < 4; ++i) {
    galore_status s = check_matrix(nullptr, *all[i], names[i], 0, true);
    if (s) return s;
    const bool tr = i == 3 && transpose_n;
    if (all[i]->rows != (tr ? R->cols : R->rows) || all[i]->cols != (tr ? R->rows : R->cols) || all[i]->ld != all[i]->cols)
      return fail(nullptr, GALORE_ERR_SHAPE, "%s must be dense with R's shape%s", names[i], tr ? " transposed" : "");
    if (i < 3 && all[i]->dtype != GALORE_F32) return fail(nullptr, GALORE_ERR_DTYPE, "%s must be fp32", names[i]);
    if (reinterpret_cast<uintptr_t>(all[i]->data) & 15) return fail(nullptr, GALORE_ERR_ALIGN, "%s must be 16-byte aligned", names[i]);
  }
  if (k < 1) return fail(nullptr, GALORE_ERR_INVALID_ARG, "k must be >= 1");
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
    return fail(nullptr, GALORE_ERR_INVALID_ARG, "betas / eps out of range");
  AdamGroup g{};
  g.count = 1; g.beta1 = beta1; g.beta2 = beta2; g.eps = eps;
  AdamProblem& p = g.p[0];
  p.R = static_cast<const float*>(R->data); p.M = static_cast<float*>(M->data); p.V = static_cast<float*>(V->data);
  p.N = N->data; p.count = R->rows * R->cols;
  p.rows = (int)R->rows; p.cols = (int)R->cols; p.ldr = (int)R->cols; p.transpose_n = transpose_n ? 1 : 0;
  p.inv_c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)k)));
  p.inv_c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)k)));
  hipError_t e = launch_adam_group(g, (DType)N->dtype, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "Adam launch");
}

galore_status galore_adam_q8(const galore_tensor* R, const galore_tensor* Mc, const galore_tensor* Vc,
                             const galore_tensor* Ms, const galore_tensor* Vs, const galore_tensor* N,
                             int32_t transpose_n, float beta1, float beta2, float eps, int64_t k, void* hip_stream) {
  if (!R || !Mc || !Vc || !Ms || !Vs || !N) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  const galore_tensor* all[6] = {R, Mc, Vc, N, Ms, Vs};
  const char* names[6] = {"R", "Mc", "Vc", "N", "Ms", "Vs"};
  for (int i = 0; i < 6; ++i) {
    galore_status s = check_matrix(nullptr, *all[i], names[i], 0, true, i == 1 || i == 2);
    if (s) return s;
    if (all[i]->ld != all[i]->cols) return fail(nullptr, GALORE_ERR_SHAPE, "%s must be dense", names[i]);
    if (reinterpret_cast<uintptr_t>(all[i]->data) & 15) return fail(nullptr, GALORE_ERR_ALIGN, "%s must be 16-byte aligned", names[i]);
  }
  if (R->dtype != GALORE_F32 || Ms->dtype != GALORE_F32 || Vs->dtype != GALORE_F32) return fail(nullptr, GALORE_ERR_DTYPE, "R, Ms, Vs must be fp32");
  if (Mc->dtype != GALORE_U8 || Vc->dtype != GALORE_U8) return fail(nullptr, GALORE_ERR_DTYPE, "Mc, Vc must be 8-bit codes");
  if (R->cols % 256 != 0) return fail(nullptr, GALORE_ERR_UNIMPLEMENTED, "8-bit moments need rows of a multiple of 256 elements");
  for (int i = 1; i < 3; ++i)
    if (all[i]->rows != R->rows || all[i]->cols != R->cols) return fail(nullptr, GALORE_ERR_SHAPE, "%s must have R's shape", names[i]);
  for (int i = 4; i < 6; ++i)
    if (all[i]->rows != R->rows || all[i]->cols != R->cols / 256) return fail(nullptr, GALORE_ERR_SHAPE, "%s must be rows x cols/256 of R", names[i]);
  if (N->rows != (transpose_n ? R->cols : R->rows) || N->cols != (transpose_n ? R->rows : R->cols))
    return fail(nullptr, GALORE_ERR_SHAPE, "N must have R's shape%s", transpose_n ? " transposed" : "");
  if (k < 1) return fail(nullptr, GALORE_ERR_INVALID_ARG, "k must be >= 1");
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f))
    return fail(nullptr, GALORE_ERR_INVALID_ARG, "betas / eps out of range");
  AdamQ8Group g{};
  g.count = 1; g.beta1 = beta1; g.beta2 = beta2; g.omb1 = 1.0f - beta1; g.omb2 = 1.0f - beta2; g.eps = eps;
  AdamQ8Problem& p = g.p[0];
  p.R = static_cast<const float*>(R->data);
  p.Mc = static_cast<uint8_t*>(Mc->data); p.Vc = static_cast<uint8_t*>(Vc->data);
  p.Ms = static_cast<float*>(Ms->data); p.Vs = static_cast<float*>(Vs->data);
  p.N = N->data; p.rows = (int)R->rows; p.cols = (int)R->cols; p.transpose_n = transpose_n ? 1 : 0;
  p.inv_c1 = (float)(1.0 / (1.0 - std::pow((double)beta1, (double)k)));
  p.inv_c2 = (float)(1.0 / (1.0 - std::pow((double)beta2, (double)k)));
  hipError_t e = launch_adam_q8_group(g, (DType)N->dtype, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "Adam launch");
}

galore_status galore_project_back(const galore_tensor* proj, const galore_tensor* N, const galore_tensor* W, float lr,
                                  float scale, float weight_decay, void* hip_stream) {
  if (!proj || !N || !W) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  galore_status s;
  if ((s = check_matrix(nullptr, *proj, "proj", 0, true)) || (s = check_matrix(nullptr, *N, "N", 0, true)) ||
      (s = check_matrix(nullptr, *W, "W", 0, true)))
    return s;
  if (proj->dtype != W->dtype || N->dtype != W->dtype) return fail(nullptr, GALORE_ERR_DTYPE, "proj, N and W dtypes must agree");
  const bool left = W->rows <= W->cols;
  const int64_t r = proj->cols;
  if (r > (left ? W->rows : W->cols)) return fail(nullptr, GALORE_ERR_RANK, "rank exceeds the short side");
  if (proj->rows != (left ? W->rows : W->cols)) return fail(nullptr, GALORE_ERR_SHAPE, "proj rows must equal the short side of W");
  if (N->rows != (left ? W->cols : W->rows) || N->cols != r)
    return fail(nullptr, GALORE_ERR_SHAPE, "N must be max(rows, cols) x r");
  GemmGroup g{};
  g.count = 1;
  GemmProblem& p = g.p[0];
  if (left) {
    p.A = proj->data; p.lda = (int)proj->ld; p.B = N->data; p.ldb = (int)N->ld;
  } else {
    p.A = N->data; p.lda = (int)N->ld; p.B = proj->data; p.ldb = (int)proj->ld;
  }
  p.M = (int)W->rows; p.N = (int)W->cols; p.K = (int)r;
  p.C = W->data; p.ldc = (int)W->ld;
  p.s0 = 1.f - lr * weight_decay;
  p.s1 = lr * scale;
  hipError_t e = launch_gemm_group(g, (DType)W->dtype, true, true, Epilogue::ApplyW, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "back-projection GEMM launch");
}

}  // extern "C"
