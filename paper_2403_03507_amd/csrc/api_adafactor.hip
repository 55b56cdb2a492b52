// GaLore with Adafactor (first-order statistics on) as the optimizer of the projected gradient, behind the C ABI: a
// composition of the library's kernels for one tensor, no context (the paper names this combination in Sec. 4.3 and
// Sec. 5 and prints no equations for it; adafactor.hip states the update that is used).
#include "adafactor.hpp"
#include "api_internal.hpp"
#include "refresh.hpp"

#include <cmath>
#include <vector>

using namespace galore;
using namespace galore::api;

namespace {

constexpr double kDecayPow = -0.8;   // decay rate of the second-moment statistics: 1 - k^-0.8
constexpr float kEps1 = 1e-30f;      // added to every squared gradient entry
constexpr float kClip = 1.0f;        // clipping threshold d on RMS(U)

struct AdafactorLayout {
  size_t pt, R, nn, nt, scratch, step_total;   // step
  size_t rws, r_pt, refresh_total;             // refresh (overlays the step's region)
  size_t total;
};

AdafactorLayout adafactor_layout(int64_t m, int64_t n, int64_t r, DType dt) {
  AdafactorLayout L{};
  const size_t s = dtype_size(dt);
  const int64_t k = m <= n ? m : n, l = m <= n ? n : m;
  const int64_t mrows = m <= n ? r : m, mcols = m <= n ? n : r;    // shape of R, M, N
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
  L.pt = take((size_t)r * k * s);
  L.R = take((size_t)mrows * mcols * 4);
  L.nn = take((size_t)mrows * mcols * s);
  L.nt = take((size_t)l * r * s);
  L.scratch = take(adafactor_scratch_floats((int)mrows, (int)mcols) * 4);
  L.step_total = off;
  off = 0;
  L.rws = take(refresh_workspace_bytes(k, r));
  L.r_pt = take((size_t)r * k * s);
  L.refresh_total = off;
  L.total = L.step_total > L.refresh_total ? L.step_total : L.refresh_total;
  return L;
}

galore_status check_workspace(const void* workspace, size_t workspace_bytes, size_t need) {
  if (!workspace) return fail(nullptr, GALORE_ERR_WORKSPACE, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return fail(nullptr, GALORE_ERR_ALIGN, "workspace must be 256-byte aligned");
  if (workspace_bytes < need) return fail(nullptr, GALORE_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
  return GALORE_OK;
}

// M rows x cols fp32 dense, the statistics as dense fp32 vectors of rows and of cols entries
galore_status check_moment_and_statistics(const galore_tensor& M, const galore_tensor& row, const galore_tensor& col, int64_t rows, int64_t cols) {
  galore_status s;
  if ((s = check_matrix(nullptr, M, "m", 0, true)) || (s = check_matrix(nullptr, row, "row", 0, true)) || (s = check_matrix(nullptr, col, "col", 0, true)))
    return s;
  if (M.dtype != GALORE_F32 || row.dtype != GALORE_F32 || col.dtype != GALORE_F32) return fail(nullptr, GALORE_ERR_DTYPE, "Adafactor state is fp32");
  if (M.rows != rows || M.cols != cols || M.ld != cols) return fail(nullptr, GALORE_ERR_STATE, "m must be %lld x %lld, dense", (long long)rows, (long long)cols);
  if (row.rows != 1 || row.cols != rows) return fail(nullptr, GALORE_ERR_STATE, "row must be 1 x %lld", (long long)rows);
  if (col.rows != 1 || col.cols != cols) return fail(nullptr, GALORE_ERR_STATE, "col must be 1 x %lld", (long long)cols);
  return GALORE_OK;
}

galore_status check_adafactor(const galore_hparams* hp, const galore_tensor* W, const galore_tensor* G, const galore_adafactor_state* S,
                              const void* workspace, size_t workspace_bytes) {
  galore_status s = check_hparams(nullptr, hp);
  if (s) return s;
  if (!W || !S) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  if ((s = check_weight_shape(nullptr, *hp, *W, 0))) return s;
  if (G) {
    if ((s = check_matrix(nullptr, *G, "G", 0, true))) return s;
    if (G->rows != W->rows || G->cols != W->cols) return fail(nullptr, GALORE_ERR_SHAPE, "G must have W's shape");
    if (G->dtype != W->dtype) return fail(nullptr, GALORE_ERR_DTYPE, "G and W dtypes must agree");
  }
  const int64_t m = W->rows, n = W->cols, r = hp->rank;
  const bool left = m <= n;
  if ((s = check_matrix(nullptr, S->proj, "state.proj", 0, true))) return s;
  if (S->proj.rows != (left ? m : n) || S->proj.cols != r) return fail(nullptr, GALORE_ERR_STATE, "state.proj must be min(rows, cols) x rank");
  if (S->proj.dtype != W->dtype) return fail(nullptr, GALORE_ERR_DTYPE, "projector dtype must equal W's");
  if ((s = check_moment_and_statistics(S->m, S->row, S->col, left ? r : m, left ? n : r))) return s;
  return check_workspace(workspace, workspace_bytes, adafactor_layout(m, n, r, (DType)W->dtype).total);
}

}  // namespace

extern "C" {

galore_status galore_adafactor_workspace_bytes(const galore_hparams* hp, const galore_tensor* W, size_t* out_bytes) {
  galore_status s = check_hparams(nullptr, hp);
  if (s) return s;
  if (!W || !out_bytes) return fail(nullptr, GALORE_ERR_INVALID_ARG, "W / out_bytes is NULL");
  if ((s = check_weight_shape(nullptr, *hp, *W, 0))) return s;
  *out_bytes = adafactor_layout(W->rows, W->cols, hp->rank, (DType)W->dtype).total;
  return GALORE_OK;
}

galore_status galore_adafactor(const galore_tensor* R, const galore_tensor* M, const galore_tensor* row, const galore_tensor* col,
                               const galore_tensor* N, float beta1, int64_t k, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!R || !M || !row || !col || !N) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  galore_status s;
  if ((s = check_matrix(nullptr, *R, "R", 0, true)) || (s = check_matrix(nullptr, *N, "N", 0, true))) return s;
  if (R->dtype != GALORE_F32) return fail(nullptr, GALORE_ERR_DTYPE, "R is fp32");
  if (N->dtype != GALORE_F32 && N->dtype != GALORE_BF16) return fail(nullptr, GALORE_ERR_DTYPE, "N is fp32 or bf16");
  if (N->rows != R->rows || N->cols != R->cols || N->ld != N->cols) return fail(nullptr, GALORE_ERR_SHAPE, "N has R's shape, dense");
  if ((s = check_moment_and_statistics(*M, *row, *col, R->rows, R->cols))) return s;
  if (!(beta1 >= 0.f && beta1 < 1.f)) return fail(nullptr, GALORE_ERR_INVALID_ARG, "beta1 outside [0, 1)");
  if (k < 1) return fail(nullptr, GALORE_ERR_INVALID_ARG, "k < 1");
  if (R->rows > INT32_MAX || R->cols > INT32_MAX || R->ld > INT32_MAX) return fail(nullptr, GALORE_ERR_SHAPE, "R too large");
  if ((s = check_workspace(workspace, workspace_bytes, adafactor_scratch_floats((int)R->rows, (int)R->cols) * 4))) return s;
  AdafactorProblem p{};
  p.R = static_cast<const float*>(R->data);
  p.M = static_cast<float*>(M->data);
  p.rowv = static_cast<float*>(row->data);
  p.colv = static_cast<float*>(col->data);
  p.N = N->data;
  p.scratch = static_cast<float*>(workspace);
  p.rows = (int)R->rows; p.cols = (int)R->cols; p.ldr = (int)R->ld;
  p.beta1 = beta1;
  p.beta2t = (float)(1.0 - std::pow((double)k, kDecayPow));
  p.eps1 = kEps1; p.clip_d = kClip;
  const hipError_t e = launch_adafactor(p, (DType)N->dtype, static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "Adafactor launch");
}

galore_status galore_adafactor_refresh(const galore_hparams* hp, const galore_tensor* G, const galore_adafactor_state* S,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!G) return fail(nullptr, GALORE_ERR_INVALID_ARG, "G is NULL");
  galore_tensor shape = *G;   // the weight has the gradient's shape and dtype
  galore_status s = check_adafactor(hp, &shape, G, S, workspace, workspace_bytes);
  if (s) return s;
  const DType dt = (DType)G->dtype;
  const int m = (int)G->rows, n = (int)G->cols, r = hp->rank;
  const AdafactorLayout L = adafactor_layout(m, n, r, dt);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  RefreshItem it{};   // the projector of the short side, as in Algorithm 2's refresh branch
  it.G = G->data; it.ldg = G->ld; it.rows = m; it.cols = n; it.dt = dt;
  it.proj = S->proj.data;
  it.ldp = S->proj.ld;
  it.proj_t = ws + L.r_pt;
  it.ldpt = m <= n ? m : n;
  it.ws = ws + L.rws;
  it.seed = hp->seed + 0x9E3779B97F4A7C15ull;
  const hipError_t e = refresh_group(std::vector<RefreshItem>{it}, r, hp->refresh_iters, /*warm_start=*/false, /*crowded=*/false,
                                     static_cast<hipStream_t>(hip_stream));
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "subspace refresh");
}

galore_status galore_adafactor_step(const galore_hparams* hp, const galore_tensor* W, const galore_tensor* G,
                                    const galore_adafactor_state* S, int64_t t, float lr,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!G) return fail(nullptr, GALORE_ERR_INVALID_ARG, "G is NULL");
  galore_status s = check_adafactor(hp, W, G, S, workspace, workspace_bytes);
  if (s) return s;
  if (!W->data) return fail(nullptr, GALORE_ERR_INVALID_ARG, "W.data is NULL");
  if (t < 0) return fail(nullptr, GALORE_ERR_INVALID_ARG, "t < 0");
  if (hp->auto_refresh && t % hp->update_gap == 0) {  // Algorithm 2's refresh test, on this step's gradient
    s = galore_adafactor_refresh(hp, G, S, workspace, workspace_bytes, hip_stream);
    if (s) return s;
  }
  const DType dt = (DType)W->dtype;
  const int m = (int)W->rows, n = (int)W->cols, r = hp->rank;
  const bool left = m <= n;
  const int k = left ? m : n;
  const int mrows = left ? r : m, mcols = left ? n : r;
  const AdafactorLayout L = adafactor_layout(m, n, r, dt);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  float* R = reinterpret_cast<float*>(ws + L.R);
  // projection (Algorithm 2, projection line): both layouts want the projector with the contraction index contiguous
  hipError_t e = single_transpose(dt, S->proj.data, k, r, (int)S->proj.ld, ws + L.pt, k, stream);
  if (e == hipSuccess) {
    if (left) e = single_gemm_store(dt, ws + L.pt, k, G->data, (int)G->ld, false, R, r, n, m, stream);     // R (r x n) = P^T G
    else e = single_gemm_store(dt, G->data, (int)G->ld, ws + L.pt, k, true, R, m, r, n, stream);           // R (m x r) = G Q
  }
  if (e != hipSuccess) return hip_fail(nullptr, e, "projection");
  // the optimizer of the projected gradient, step k = t + 1
  {
    AdafactorProblem p{};
    p.R = R;
    p.M = static_cast<float*>(S->m.data);
    p.rowv = static_cast<float*>(S->row.data);
    p.colv = static_cast<float*>(S->col.data);
    p.N = ws + L.nn;
    p.scratch = reinterpret_cast<float*>(ws + L.scratch);
    p.rows = mrows; p.cols = mcols; p.ldr = mcols;
    p.beta1 = hp->beta1;
    p.beta2t = (float)(1.0 - std::pow((double)(t + 1), kDecayPow));
    p.eps1 = kEps1; p.clip_d = kClip;
    e = launch_adafactor(p, dt, stream);
    if (e != hipSuccess) return hip_fail(nullptr, e, "Adafactor launch");
  }
  // W <- (1 - lr wd) W - lr alpha (P N | N Q^T) in the epilogue of the product (Algorithm 2, last lines); the kernel
  // reads N as (long side) x r, i.e. transposed for a LEFT tensor
  const void* Nl = ws + L.nn;
  if (left) {
    e = single_transpose(dt, ws + L.nn, r, n, n, ws + L.nt, r, stream);
    if (e != hipSuccess) return hip_fail(nullptr, e, "transpose of N");
    Nl = ws + L.nt;
  }
  GemmGroup g{};
  g.count = 1;
  GemmProblem& p = g.p[0];
  if (left) { p.A = S->proj.data; p.lda = (int)S->proj.ld; p.B = Nl; p.ldb = r; }
  else { p.A = Nl; p.lda = r; p.B = S->proj.data; p.ldb = (int)S->proj.ld; }
  p.M = m; p.N = n; p.K = r;
  p.C = W->data; p.ldc = (int)W->ld;
  p.s0 = 1.f - lr * hp->weight_decay;
  p.s1 = lr * hp->scale;
  e = launch_gemm_group(g, dt, true, true, Epilogue::ApplyW, stream);
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "weight update");
}

}  // extern "C"
