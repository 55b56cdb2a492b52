// Two-sided projection (Sec. 3.3, Definition 3.6) behind the C ABI: a composition of the library's kernels for one
// tensor, no context.
#include "api_internal.hpp"
#include "refresh.hpp"

#include <cmath>
#include <vector>

using namespace galore;
using namespace galore::api;

namespace {

struct TwoSidedLayout {
  // step
  size_t pt, t1, t1c, R, nn, t2, t2c, step_total;
  // refresh (overlays the step's region: the two never run at once on one workspace)
  size_t rws, r_pt, r_t1, r_qt, r_tg, r_tgt, refresh_total;
  size_t total;
};

TwoSidedLayout two_sided_layout(int64_t m, int64_t n, int64_t r, DType dt) {
  TwoSidedLayout L{};
  const size_t s = dtype_size(dt);
  size_t off = 0;
  auto take = [&](size_t bytes) { const size_t o = off; off += align_up(bytes); return o; };
  L.pt = take((size_t)r * m * s);
  L.t1 = take((size_t)r * n * 4);
  L.t1c = dt == DType::F32 ? L.t1 : take((size_t)r * n * s);
  L.R = take((size_t)r * r * 4);
  L.nn = take((size_t)r * r * s);
  L.t2 = take((size_t)n * r * 4);
  L.t2c = dt == DType::F32 ? L.t2 : take((size_t)n * r * s);
  L.step_total = off;
  off = 0;
  L.rws = take(refresh_workspace_bytes(m <= n ? m : n, r));
  L.r_pt = take((size_t)r * m * s);
  L.r_qt = take((size_t)r * n * s);
  if (m <= n) {
    L.r_t1 = take((size_t)r * n * 4);
  } else {
    L.r_tg = take((size_t)m * r * 4);
    L.r_tgt = take((size_t)r * m * 4);
  }
  L.refresh_total = off;
  L.total = L.step_total > L.refresh_total ? L.step_total : L.refresh_total;
  return L;
}

galore_status check_two_sided(const galore_hparams* hp, const galore_tensor* W, const galore_tensor* G,
                              const galore_two_sided_state* S, const void* workspace, size_t workspace_bytes) {
  galore_status s = check_hparams(nullptr, hp);
  if (s) return s;
  if (!W || !S) return fail(nullptr, GALORE_ERR_INVALID_ARG, "NULL argument");
  if ((s = check_weight_shape(nullptr, *hp, *W, 0))) return s;
  if (G) {
    if ((s = check_matrix(nullptr, *G, "G", 0, true))) return s;
    if (G->rows != W->rows || G->cols != W->cols) return fail(nullptr, GALORE_ERR_SHAPE, "G must have W's shape");
    if (G->dtype != W->dtype) return fail(nullptr, GALORE_ERR_DTYPE, "G and W dtypes must agree");
  }
  const int64_t r = hp->rank;
  if ((s = check_matrix(nullptr, S->p, "state.p", 0, true)) || (s = check_matrix(nullptr, S->q, "state.q", 0, true)) ||
      (s = check_matrix(nullptr, S->m, "state.m", 0, true)) || (s = check_matrix(nullptr, S->v, "state.v", 0, true)))
    return s;
  if (S->p.rows != W->rows || S->p.cols != r) return fail(nullptr, GALORE_ERR_STATE, "state.p must be rows(W) x rank");
  if (S->q.rows != W->cols || S->q.cols != r) return fail(nullptr, GALORE_ERR_STATE, "state.q must be cols(W) x rank");
  if (S->p.dtype != W->dtype || S->q.dtype != W->dtype) return fail(nullptr, GALORE_ERR_DTYPE, "projector dtypes must equal W's");
  for (const galore_tensor* mv : {&S->m, &S->v}) {
    if (mv->dtype != GALORE_F32) return fail(nullptr, GALORE_ERR_DTYPE, "two-sided moments are fp32");
    if (mv->rows != r || mv->cols != r || mv->ld != r) return fail(nullptr, GALORE_ERR_STATE, "two-sided moments are rank x rank, dense");
  }
  if (!workspace) return fail(nullptr, GALORE_ERR_WORKSPACE, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign != 0) return fail(nullptr, GALORE_ERR_ALIGN, "workspace must be 256-byte aligned");
  const size_t need = two_sided_layout(W->rows, W->cols, r, (DType)W->dtype).total;
  if (workspace_bytes < need)
    return fail(nullptr, GALORE_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
  return GALORE_OK;
}

}  // namespace

extern "C" {

galore_status galore_two_sided_workspace_bytes(const galore_hparams* hp, const galore_tensor* W, size_t* out_bytes) {
  galore_status s = check_hparams(nullptr, hp);
  if (s) return s;
  if (!W || !out_bytes) return fail(nullptr, GALORE_ERR_INVALID_ARG, "W / out_bytes is NULL");
  if ((s = check_weight_shape(nullptr, *hp, *W, 0))) return s;
  *out_bytes = two_sided_layout(W->rows, W->cols, hp->rank, (DType)W->dtype).total;
  return GALORE_OK;
}

galore_status galore_two_sided_step(const galore_hparams* hp, const galore_tensor* W, const galore_tensor* G,
                                    const galore_two_sided_state* S, int64_t t, float lr,
                                    void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!G) return fail(nullptr, GALORE_ERR_INVALID_ARG, "G is NULL");
  galore_status s = check_two_sided(hp, W, G, S, workspace, workspace_bytes);
  if (s) return s;
  if (!W->data) return fail(nullptr, GALORE_ERR_INVALID_ARG, "W.data is NULL");
  if (t < 0) return fail(nullptr, GALORE_ERR_INVALID_ARG, "t < 0");
  if (hp->auto_refresh && t % hp->update_gap == 0) {  // Algorithm 2's refresh test, on this step's gradient
    s = galore_two_sided_refresh(hp, G, S, workspace, workspace_bytes, hip_stream);
    if (s) return s;
  }
  const DType dt = (DType)W->dtype;
  const int m = (int)W->rows, n = (int)W->cols, r = hp->rank;
  const TwoSidedLayout L = two_sided_layout(m, n, r, dt);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  float* T1 = reinterpret_cast<float*>(ws + L.t1);
  float* R = reinterpret_cast<float*>(ws + L.R);
  float* T2 = reinterpret_cast<float*>(ws + L.t2);
  hipError_t e;
  // T1 (r x n) = P^T G, then R (r x r) = T1 Q: every product reads its operands in the storage dtype
  e = single_transpose(dt, S->p.data, m, r, (int)S->p.ld, ws + L.pt, m, stream);
  if (e == hipSuccess) e = single_gemm_store(dt, ws + L.pt, m, G->data, (int)G->ld, false, T1, r, n, m, stream);
  if (e == hipSuccess && dt != DType::F32) e = launch_cast_rows(T1, ws + L.t1c, r, n, n, dt, stream);
  if (e == hipSuccess) e = single_gemm_store(dt, ws + L.t1c, n, S->q.data, (int)S->q.ld, false, R, r, r, n, stream);
  if (e != hipSuccess) return hip_fail(nullptr, e, "two-sided projection");
  // Adam on R (Algorithm 2, update block), k = t + 1
  {
    AdamGroup g{};
    g.count = 1;
    g.beta1 = hp->beta1; g.beta2 = hp->beta2; g.eps = hp->eps;
    const double k = (double)(t + 1);
    AdamProblem& p = g.p[0];
    p.R = R;
    p.M = static_cast<float*>(S->m.data);
    p.V = static_cast<float*>(S->v.data);
    p.N = ws + L.nn;
    p.rows = r; p.cols = r; p.ldr = r; p.count = (int64_t)r * r;
    p.transpose_n = 0;
    p.inv_c1 = (float)(1.0 / (1.0 - std::pow((double)hp->beta1, k)));
    p.inv_c2 = (float)(1.0 / (1.0 - std::pow((double)hp->beta2, k)));
    e = launch_adam_group(g, dt, stream);
    if (e != hipSuccess) return hip_fail(nullptr, e, "two-sided Adam");
  }
  // T2 (n x r) = Q N^T, then W <- (1 - lr wd) W - lr alpha P T2^T in the epilogue of the last product
  e = single_gemm_store(dt, S->q.data, (int)S->q.ld, ws + L.nn, r, true, T2, n, r, r, stream);
  if (e == hipSuccess && dt != DType::F32) e = launch_cast_rows(T2, ws + L.t2c, n, r, r, dt, stream);
  if (e == hipSuccess) {
    GemmGroup g{};
    g.count = 1;
    GemmProblem& p = g.p[0];
    p.A = S->p.data; p.lda = (int)S->p.ld;
    p.B = ws + L.t2c; p.ldb = r;
    p.M = m; p.N = n; p.K = r;
    p.C = W->data; p.ldc = (int)W->ld;
    p.s0 = 1.f - lr * hp->weight_decay;
    p.s1 = lr * hp->scale;
    e = launch_gemm_group(g, dt, true, true, Epilogue::ApplyW, stream);
  }
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "two-sided weight update");
}

galore_status galore_two_sided_refresh(const galore_hparams* hp, const galore_tensor* G, const galore_two_sided_state* S,
                                       void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!G) return fail(nullptr, GALORE_ERR_INVALID_ARG, "G is NULL");
  galore_tensor shape = *G;   // the weight has the gradient's shape and dtype
  galore_status s = check_two_sided(hp, &shape, G, S, workspace, workspace_bytes);
  if (s) return s;
  const DType dt = (DType)G->dtype;
  const int m = (int)G->rows, n = (int)G->cols, r = hp->rank;
  const bool left = m <= n;
  const TwoSidedLayout L = two_sided_layout(m, n, r, dt);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  // the projector of the short side, as in Algorithm 2's refresh branch (writes it and its transpose)
  RefreshItem it{};
  it.G = G->data; it.ldg = G->ld; it.rows = m; it.cols = n; it.dt = dt;
  it.proj = left ? S->p.data : S->q.data;
  it.ldp = left ? S->p.ld : S->q.ld;
  it.proj_t = ws + (left ? L.r_pt : L.r_qt);
  it.ldpt = left ? m : n;
  it.ws = ws + L.rws;
  it.seed = hp->seed + 0x9E3779B97F4A7C15ull;
  hipError_t e = refresh_group(std::vector<RefreshItem>{it}, r, hp->refresh_iters, /*warm_start=*/false, /*crowded=*/false, stream);
  if (e != hipSuccess) return hip_fail(nullptr, e, "subspace refresh");
  if (left) {
    // rows of P^T G are s_i v_i^T: unit length makes them Q^T
    float* T1 = reinterpret_cast<float*>(ws + L.r_t1);
    e = single_gemm_store(dt, ws + L.r_pt, m, G->data, (int)G->ld, false, T1, r, n, m, stream);
    if (e == hipSuccess) e = launch_normalize_rows(T1, ws + L.r_qt, r, n, n, dt, stream);
    if (e == hipSuccess) e = single_transpose(dt, ws + L.r_qt, r, n, n, S->q.data, (int)S->q.ld, stream);
  } else {
    // columns of G Q are s_i u_i
    float* Tg = reinterpret_cast<float*>(ws + L.r_tg);
    float* Tgt = reinterpret_cast<float*>(ws + L.r_tgt);
    e = single_gemm_store(dt, G->data, (int)G->ld, ws + L.r_qt, n, true, Tg, m, r, n, stream);
    if (e == hipSuccess) e = single_transpose(DType::F32, Tg, m, r, r, Tgt, m, stream);
    if (e == hipSuccess) e = launch_normalize_rows(Tgt, ws + L.r_pt, r, m, m, dt, stream);
    if (e == hipSuccess) e = single_transpose(dt, ws + L.r_pt, r, m, m, S->p.data, (int)S->p.ld, stream);
  }
  return e == hipSuccess ? GALORE_OK : hip_fail(nullptr, e, "partner projector");
}

}  // extern "C"
