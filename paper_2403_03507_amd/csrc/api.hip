// Host side of the C ABI: context, validation, chunking of tensor lists into grouped
// launches, and the per-step orchestration of Algorithm 2.  No kernels here.
#include "api_internal.hpp"
#include "refresh.hpp"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <mutex>
#include <new>
#include <algorithm>
#include <string>
#include <vector>

using namespace galore;
using namespace galore::api;

// Device memory of galore_step_static, the entry point for callers that cannot allocate: the
// transients R, N (and the padded copy of G) of one launch group live here instead of in the
// caller's workspace.  Every GPU the library runs on holds its own copy of the array at its own
// address; host code never uses the array's name as an address, only the per-device pointer that
// hipGetSymbolAddress returned.
constexpr size_t kStaticScratchBytes = (size_t)80 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

thread_local std::string g_last_error;

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};  // per device: address of that device's copy of `scratch`

// Address of the current device's scratch array (resolved once per device, with that device current).
hipError_t static_scratch_ptr(unsigned char** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<unsigned char*>(g_scratch_ptr[dev]);
  return hipSuccess;
}

struct TensorInfo {
  int64_t rows, cols;
  DType dt;
  bool left;       // rows <= cols: projector on the left (P^T G), else on the right (G Q)
  int64_t kdim;    // short side = rows of the projector
  int64_t ldim;    // long side
  galore_state st;
  int64_t t;
  bool proj_t_valid;  // state.proj_t mirrors state.proj (only trusted when the library owns the projector)
  bool refreshed;     // the projector in state.proj_t was written by a refresh of this context
  bool q8;            // moments stored as 8-bit codes with block scales
};

}  // namespace

struct ProfRecord {
  hipEvent_t begin, end;
  int stage;
};

constexpr int kLibStreams = 3;  // library-owned streams per context

struct galore_ctx {
  galore_hparams hp;
  std::vector<TensorInfo> tensors;
  unsigned char* ws;
  size_t ws_bytes;
  hipStream_t stream;
  std::string err;
  bool profiling = false;
  std::vector<ProfRecord> records;
  std::vector<hipEvent_t> event_pool;
  // Concurrency inside one galore_step call: the tensors of a call are split into up to
  // `lanes` independent chains (project -> Adam -> project back) that run on the caller's
  // stream and on library-owned streams (default priority), forked and joined with events.
  int lanes = 3;
  hipStream_t aux[kLibStreams] = {};
  hipEvent_t fork_ev = nullptr;
  hipEvent_t join_ev[kLibStreams] = {};
  // Overlap of consecutive calls (galore_set_call_overlap): every call (chunk) runs as ONE chain on
  // one of the first `slots` library streams, taking turns, and the context's stream is not made to
  // wait until galore_join.  The chunk on stream h uses share h of the workspace (one of `slots`
  // equal parts), so stream order alone protects the workspace.
  bool fused_adam = false;        // Adam in the epilogue of the projection launch (galore_set_fused_adam)
  bool merged_projection = true;  // LEFT and RIGHT projections of the large-tile kernel in one launch (see gemm_proj_dl.hpp)
  bool overlap_calls = false;
  int slots = 2;
  bool unjoined = false;          // library streams hold work the context's stream has not waited for
  int parity = 0;                 // the library stream (and workspace share) the next overlapped call takes
  std::vector<char> in_flight;    // per tensor: 0, or 1 + the library stream its last chain ran on
};

namespace galore {
namespace api {

bool valid_dtype(int32_t d, bool allow_u8) { return d == GALORE_F32 || d == GALORE_BF16 || (allow_u8 && d == GALORE_U8); }

galore_status fail(galore_ctx* ctx, galore_status s, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (ctx) ctx->err = buf;
  g_last_error = buf;
  return s;
}

galore_status check_hparams(galore_ctx* ctx, const galore_hparams* hp) {
  if (!hp) return fail(ctx, GALORE_ERR_INVALID_ARG, "hparams is NULL");
  if (hp->rank < 1) return fail(ctx, GALORE_ERR_RANK, "rank %d < 1", hp->rank);
  if (hp->update_gap < 1) return fail(ctx, GALORE_ERR_INVALID_ARG, "update_gap %d < 1", hp->update_gap);
  if (!(hp->beta1 >= 0.f && hp->beta1 < 1.f) || !(hp->beta2 >= 0.f && hp->beta2 < 1.f))
    return fail(ctx, GALORE_ERR_INVALID_ARG, "betas must lie in [0, 1)");
  if (!(hp->eps >= 0.f) || !std::isfinite(hp->scale) || !(hp->weight_decay >= 0.f))
    return fail(ctx, GALORE_ERR_INVALID_ARG, "eps / scale / weight_decay out of range");
  if (hp->refresh_iters < 1) return fail(ctx, GALORE_ERR_INVALID_ARG, "refresh_iters %d < 1", hp->refresh_iters);
  if (hp->refresh_warm_iters < 0) return fail(ctx, GALORE_ERR_INVALID_ARG, "refresh_warm_iters %d < 0", hp->refresh_warm_iters);
  return GALORE_OK;
}

galore_status check_matrix(galore_ctx* ctx, const galore_tensor& t, const char* what, int idx, bool need_data,
                           bool allow_u8) {
  if (need_data && !t.data) return fail(ctx, GALORE_ERR_INVALID_ARG, "%s[%d].data is NULL", what, idx);
  if (t.rows < 1 || t.cols < 1) return fail(ctx, GALORE_ERR_SHAPE, "%s[%d] has empty shape %lld x %lld", what, idx,
                                            (long long)t.rows, (long long)t.cols);
  if (t.ld < t.cols) return fail(ctx, GALORE_ERR_SHAPE, "%s[%d].ld %lld < cols %lld", what, idx, (long long)t.ld,
                                 (long long)t.cols);
  if (t.rows > INT32_MAX / 2 || t.ld > INT32_MAX / 2)
    return fail(ctx, GALORE_ERR_SHAPE, "%s[%d] dimension too large", what, idx);
  if (!valid_dtype(t.dtype, allow_u8)) return fail(ctx, GALORE_ERR_DTYPE, "%s[%d].dtype %d not allowed here", what, idx, t.dtype);
  return GALORE_OK;
}

galore_status check_weight_shape(galore_ctx* ctx, const galore_hparams& hp, const galore_tensor& w, int idx) {
  galore_status s = check_matrix(ctx, w, "W", idx, false);
  if (s) return s;
  const int64_t k = w.rows <= w.cols ? w.rows : w.cols;
  if (hp.rank > k) return fail(ctx, GALORE_ERR_RANK, "rank %d exceeds min(rows, cols) = %lld of W[%d]", hp.rank,
                               (long long)k, idx);
  return GALORE_OK;
}

galore_status hip_fail(galore_ctx* ctx, hipError_t e, const char* where) {
  if (e == hipErrorNotSupported) return fail(ctx, GALORE_ERR_UNIMPLEMENTED, "%s: not implemented", where);
  return fail(ctx, GALORE_ERR_HIP, "%s: %s", where, hipGetErrorString(e));
}

}  // namespace api
}  // namespace galore

namespace {



// The large-tile GEMM moves aligned 16-byte pieces, so G of a LEFT bf16 tensor (contiguous along n, the
// GEMM's N index) cannot feed it when n is not a multiple of 8: its rows start at odd element offsets.
// The projection of such a tensor reads a copy of G with the rows padded to a multiple of 8 (zeros) and
// writes R with the same padded row length; the copy costs one pass over G and buys the 256 x 256 tiles.
// Returns the row length of R: ldim itself when nothing is padded.
int64_t projected_row_length(bool left, int64_t kdim, int64_t ldim, DType dt) {
  const bool pad = left && dt == DType::BF16 && ldim % 8 != 0 && ldim >= 8 && kdim % 64 == 0;
  return pad ? (ldim + 7) / 8 * 8 : ldim;
}
size_t step_r_bytes(bool left, int64_t kdim, int64_t ldim, int64_t r, DType dt) {
  return align_up((size_t)r * projected_row_length(left, kdim, ldim, dt) * 4);
}
size_t step_n_bytes(int64_t ldim, int64_t r, DType dt) { return align_up((size_t)r * ldim * dtype_size(dt)); }
size_t step_gpad_bytes(bool left, int64_t kdim, int64_t ldim, DType dt) {
  const int64_t ldp = projected_row_length(left, kdim, ldim, dt);
  return ldp == ldim ? 0 : align_up((size_t)kdim * ldp * dtype_size(dt));
}
size_t step_need(bool left, int64_t kdim, int64_t ldim, int64_t r, DType dt) {
  return step_r_bytes(left, kdim, ldim, r, dt) + step_n_bytes(ldim, r, dt) + step_gpad_bytes(left, kdim, ldim, dt);
}

size_t tensor_need(const galore_hparams& hp, bool left, int64_t kdim, int64_t ldim, DType dt) {
  const size_t a = step_need(left, kdim, ldim, hp.rank, dt);
  const size_t b = refresh_workspace_bytes(kdim, hp.rank);
  return a > b ? a : b;
}





// Event bracket around one kernel group while profiling is on.
struct ProfScope {
  galore_ctx* ctx;
  hipStream_t stream;
  ProfRecord rec{};
  bool live = false;
  ProfScope(galore_ctx* c, int stage, bool nonempty, hipStream_t st = nullptr) : ctx(c), stream(st ? st : c->stream) {
    if (!c->profiling || !nonempty) return;
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
      if (!c->event_pool.empty()) { ev[i] = c->event_pool.back(); c->event_pool.pop_back(); }
      else if (hipEventCreate(&ev[i]) != hipSuccess) { if (i == 1) c->event_pool.push_back(ev[0]); return; }
    }
    rec.begin = ev[0]; rec.end = ev[1]; rec.stage = stage;
    live = hipEventRecord(rec.begin, stream) == hipSuccess;
  }
  ~ProfScope() {
    if (!live) return;
    (void)hipEventRecord(rec.end, stream);
    ctx->records.push_back(rec);
  }
};

// ---- one chunk of the step: tensors idx[0..n) with their W, G -------------------------------
struct StepItem {
  int tensor;
  const galore_tensor* W;
  const galore_tensor* G;
  float* R;
  void* N;
  void* Gpad;    // copy of G with padded rows (see projected_row_length), or nullptr
  int64_t ldr;   // row length of R
};

galore_status run_chain(galore_ctx* ctx, const std::vector<StepItem>& items, float lr, hipStream_t stream,
                        float* slabs = nullptr, size_t slab_bytes = 0) {
  const galore_hparams& hp = ctx->hp;
  const int r = hp.rank;
  // The list may mix dtypes; launches are split by dtype (and by orientation where layouts differ).
  for (int dti = 0; dti < 2; ++dti) {
    const DType dt = dti == 0 ? DType::F32 : DType::BF16;
    // proj_t <- proj^T where the library cannot vouch for the copy it has
    {
      TransposeGroup g{};
      for (const StepItem& it : items) {
        TensorInfo& ti = ctx->tensors[it.tensor];
        if (ti.dt != dt || (hp.auto_refresh && ti.proj_t_valid)) continue;
        TransposeProblem& p = g.p[g.count++];
        p.src = ti.st.proj.data; p.lds = (int)ti.st.proj.ld;
        p.dst = ti.st.proj_t.data; p.ldd = (int)ti.st.proj_t.ld;
        p.rows = (int)ti.kdim; p.cols = r;
        ti.proj_t_valid = true;
      }
      ProfScope prof(ctx, GALORE_STAGE_TRANSPOSE, g.count > 0, stream);
      hipError_t e = launch_transpose_group(g, dt, stream);
      if (e != hipSuccess) return hip_fail(ctx, e, "projector transpose launch");
    }
    // K1: project.  Both operands are read from layouts in which as much as possible is
    // contiguous along the contraction index; only G of a LEFT tensor is not.  bf16 tensors that meet the
    // large-tile kernel's rules go into ONE launch, LEFT and RIGHT together (the layout of B is a field of
    // each problem there); the rest take the general kernel, one launch per orientation.
    std::vector<char> adam_done(items.size(), 0);  // tensors whose Adam ran inside the projection launch
    {
      ProjGroup pg{}, pgf{};   // pgf: with the update block of Algorithm 2 in the epilogue (galore_set_fused_adam)
      pgf.beta1 = hp.beta1; pgf.beta2 = hp.beta2; pgf.eps = hp.eps;
      GemmGroup rest[2] = {};  // [0] RIGHT, [1] LEFT
      PadGroup pads{};
      for (int left = 1; left >= 0; --left) {
        for (size_t ii = 0; ii < items.size(); ++ii) {
          const StepItem& it = items[ii];
          const TensorInfo& ti = ctx->tensors[it.tensor];
          if (ti.dt != dt || (int)ti.left != left) continue;
          GemmProblem p{};
          if (left && it.Gpad) {  // the same product on the padded copy: the extra columns of G and of R are zero
            PadProblem& q = pads.p[pads.count++];
            q.src = it.G->data; q.lds = (int)it.G->ld;
            q.dst = it.Gpad; q.ldd = (int)it.ldr;
            q.rows = (int)ti.rows; q.cols = (int)ti.cols;
            p.A = ti.st.proj_t.data; p.lda = (int)ti.st.proj_t.ld;
            p.B = it.Gpad; p.ldb = (int)it.ldr;
            p.M = r; p.N = (int)it.ldr; p.K = (int)ti.rows;
            p.C = it.R; p.ldc = (int)it.ldr;
          } else if (left) {  // R (r x n) = P^T G : A = proj_t as [M=r][K=m], B = G as [K=m][N=n]
            p.A = ti.st.proj_t.data; p.lda = (int)ti.st.proj_t.ld;
            p.B = it.G->data; p.ldb = (int)it.G->ld;
            p.M = r; p.N = (int)ti.cols; p.K = (int)ti.rows;
            p.C = it.R; p.ldc = (int)ti.cols;
          } else {     // R (m x r) = G Q : A = G as [M=m][K=n], B = proj_t as [N=r][K=n]
            p.A = it.G->data; p.lda = (int)it.G->ld;
            p.B = ti.st.proj_t.data; p.ldb = (int)ti.st.proj_t.ld;
            p.M = (int)ti.rows; p.N = r; p.K = (int)ti.cols;
            p.C = it.R; p.ldc = r;
          }
          ProjProblem q{};
          q.A = p.A; q.B = p.B; q.R = static_cast<float*>(p.C);
          q.M = p.M; q.N = p.N; q.K = p.K; q.lda = p.lda; q.ldb = p.ldb; q.ldr = p.ldc;
          q.b_kcontig = left ? 0 : 1;
          if (dt == DType::BF16 && ctx->merged_projection && proj_problem_fits(q)) {
            if (ctx->fused_adam && !ti.q8) {
              const double k = (double)(ti.t + 1);
              q.Mo = static_cast<float*>(ti.st.m.data);
              q.Vo = static_cast<float*>(ti.st.v.data);
              q.Nout = it.N;
              q.ldm = q.cols_valid = left ? (int)ti.cols : r;   // M, V are dense; R may carry padded columns
              q.ldn = r;                                         // N is always (long side) x r
              q.n_transposed = left;
              q.inv_c1 = (float)(1.0 / (1.0 - std::pow((double)hp.beta1, k)));
              q.inv_c2 = (float)(1.0 / (1.0 - std::pow((double)hp.beta2, k)));
              pgf.p[pgf.count++] = q;
              adam_done[ii] = 1;
            } else {
              pg.p[pg.count++] = q;
            }
          } else {
            rest[left].p[rest[left].count++] = p;
          }
        }
      }
      {
        ProfScope prof(ctx, GALORE_STAGE_PROJECT_LEFT, pg.count + pgf.count + rest[1].count > 0, stream);
        hipError_t e = launch_pad_rows_group(pads, stream);
        if (e != hipSuccess) return hip_fail(ctx, e, "row padding launch");
        e = launch_proj_group(pgf, slabs, slab_bytes, stream, /*fuse_adam=*/true);
        if (e == hipSuccess) e = launch_proj_group(pg, slabs, slab_bytes, stream);
        if (e == hipSuccess) e = launch_gemm_group(rest[1], dt, /*a_kcontig=*/true, /*b_kcontig=*/false, Epilogue::StoreF32, stream);
        if (e != hipSuccess) return hip_fail(ctx, e, "projection GEMM launch");
      }
      {
        ProfScope prof(ctx, GALORE_STAGE_PROJECT_RIGHT, rest[0].count > 0, stream);
        hipError_t e = launch_gemm_group(rest[0], dt, /*a_kcontig=*/true, /*b_kcontig=*/true, Epilogue::StoreF32, stream);
        if (e != hipSuccess) return hip_fail(ctx, e, "projection GEMM launch");
      }
    }
    // K2: Adam on R.  N always leaves as (long side) x r: transposed for LEFT tensors.
    for (int left = 1; left >= 0; --left) {
      AdamGroup g{};
      AdamQ8Group g8{};
      g.beta1 = hp.beta1; g.beta2 = hp.beta2; g.eps = hp.eps;
      g8.beta1 = hp.beta1; g8.beta2 = hp.beta2; g8.eps = hp.eps;
      g8.omb1 = 1.0f - hp.beta1; g8.omb2 = 1.0f - hp.beta2;
      for (size_t ii = 0; ii < items.size(); ++ii) {
        const StepItem& it = items[ii];
        const TensorInfo& ti = ctx->tensors[it.tensor];
        if (ti.dt != dt || (int)ti.left != left || adam_done[ii]) continue;
        const double k = (double)(ti.t + 1);
        const float ic1 = (float)(1.0 / (1.0 - std::pow((double)hp.beta1, k)));
        const float ic2 = (float)(1.0 / (1.0 - std::pow((double)hp.beta2, k)));
        if (ti.q8) {
          AdamQ8Problem& p = g8.p[g8.count++];
          p.R = it.R;
          p.Mc = static_cast<uint8_t*>(ti.st.m.data); p.Vc = static_cast<uint8_t*>(ti.st.v.data);
          p.Ms = static_cast<float*>(ti.st.m_scale.data); p.Vs = static_cast<float*>(ti.st.v_scale.data);
          p.N = it.N;
          p.rows = left ? r : (int)ti.rows;
          p.cols = left ? (int)ti.cols : r;
          p.transpose_n = left;
          p.inv_c1 = ic1; p.inv_c2 = ic2;
          continue;
        }
        AdamProblem& p = g.p[g.count++];
        p.R = it.R;
        p.M = static_cast<float*>(ti.st.m.data);
        p.V = static_cast<float*>(ti.st.v.data);
        p.N = it.N;
        p.rows = left ? r : (int)ti.rows;
        p.cols = left ? (int)ti.cols : r;
        p.ldr = left ? (int)it.ldr : r;
        p.count = (int64_t)r * ti.ldim;
        p.transpose_n = left;
        p.inv_c1 = ic1;
        p.inv_c2 = ic2;
      }
      ProfScope prof(ctx, GALORE_STAGE_ADAM, g.count + g8.count > 0, stream);
      hipError_t e = launch_adam_group(g, dt, stream);
      if (e == hipSuccess) e = launch_adam_q8_group(g8, dt, stream);
      if (e != hipSuccess) return hip_fail(ctx, e, "Adam launch");
    }
    // K3: project back + apply; with N as (long side) x r both orientations share one layout
    // (A and B contiguous along r), hence one launch.
    {
      GemmGroup g{};
      for (const StepItem& it : items) {
        const TensorInfo& ti = ctx->tensors[it.tensor];
        if (ti.dt != dt) continue;
        GemmProblem& p = g.p[g.count++];
        if (ti.left) {  // W (m x n) -= P N : A = P as [M=m][K=r], B = N^T as [N=n][K=r]
          p.A = ti.st.proj.data; p.lda = (int)ti.st.proj.ld;
          p.B = it.N; p.ldb = r;
        } else {        // W (m x n) -= N Q^T : A = N as [M=m][K=r], B = Q as [N=n][K=r]
          p.A = it.N; p.lda = r;
          p.B = ti.st.proj.data; p.ldb = (int)ti.st.proj.ld;
        }
        p.M = (int)ti.rows; p.N = (int)ti.cols; p.K = r;
        p.C = it.W->data; p.ldc = (int)it.W->ld;
        p.s0 = 1.f - lr * hp.weight_decay;
        p.s1 = lr * hp.scale;
      }
      ProfScope prof(ctx, GALORE_STAGE_BACK, g.count > 0, stream);
      hipError_t e = launch_gemm_group(g, dt, /*a_kcontig=*/true, /*b_kcontig=*/true, Epilogue::ApplyW, stream);
      if (e != hipSuccess) return hip_fail(ctx, e, "back-projection GEMM launch");
    }
  }
  return GALORE_OK;
}

// Make the context's stream wait for everything the library streams hold.
galore_status join_all(galore_ctx* ctx) {
  galore_status st = GALORE_OK;
  for (int c = 0; c < kLibStreams; ++c) {
    if (!ctx->aux[c] || !ctx->join_ev[c]) continue;
    hipError_t e = hipEventRecord(ctx->join_ev[c], ctx->aux[c]);
    if (e == hipSuccess) e = hipStreamWaitEvent(ctx->stream, ctx->join_ev[c], 0);
    if (e != hipSuccess && st == GALORE_OK) st = hip_fail(ctx, e, "joining streams");
  }
  ctx->unjoined = false;
  std::fill(ctx->in_flight.begin(), ctx->in_flight.end(), 0);
  return st;
}

// the part of the workspace one overlapped call may use
size_t workspace_share(const galore_ctx* ctx) { return (ctx->ws_bytes / (size_t)ctx->slots) & ~(size_t)255; }
bool library_streams_ready(const galore_ctx* ctx) {
  for (int c = 0; c < kLibStreams; ++c)
    if (!ctx->aux[c] || !ctx->join_ev[c]) return false;
  return ctx->fork_ev != nullptr;
}

// One chunk of the step: carve the workspace, split the tensors into chains of similar cost and
// run the chains concurrently.  Chains touch disjoint tensors and disjoint workspace regions.
galore_status run_step_chunk(galore_ctx* ctx, std::vector<StepItem>& items, float lr) {
  const int r = ctx->hp.rank;
  size_t need = 0;
  for (const StepItem& it : items) {
    const TensorInfo& ti = ctx->tensors[it.tensor];
    need += step_need(ti.left, ti.kdim, ti.ldim, r, ti.dt);
  }
  const bool overlap = ctx->overlap_calls && library_streams_ready(ctx) && need <= workspace_share(ctx);
  if (ctx->unjoined) {
    // Order everything first when this chunk cannot run on a library stream, or when one of its
    // tensors is still in flight on the OTHER library stream.
    bool clash = !overlap;
    for (const StepItem& it : items) clash = clash || (ctx->in_flight[it.tensor] != 0 && ctx->in_flight[it.tensor] != 1 + ctx->parity);
    if (clash) {
      galore_status s = join_all(ctx);
      if (s) return s;
    }
  }
  size_t off = overlap ? (size_t)ctx->parity * workspace_share(ctx) : 0;
  for (StepItem& it : items) {
    const TensorInfo& ti = ctx->tensors[it.tensor];
    it.R = reinterpret_cast<float*>(ctx->ws + off);
    off += step_r_bytes(ti.left, ti.kdim, ti.ldim, r, ti.dt);
    it.N = ctx->ws + off;
    off += step_n_bytes(ti.ldim, r, ti.dt);
    const size_t gp = step_gpad_bytes(ti.left, ti.kdim, ti.ldim, ti.dt);
    it.Gpad = gp ? ctx->ws + off : nullptr;
    off += gp;
    it.ldr = projected_row_length(ti.left, ti.kdim, ti.ldim, ti.dt);
  }
  // What is left of this call's part of the workspace holds the partial tiles of the projection GEMM
  // (at most 64 MiB per chain are of use: one 256 x 256 fp32 tile per CU).
  const size_t region_end = overlap ? (size_t)(ctx->parity + 1) * workspace_share(ctx) : ctx->ws_bytes;
  const size_t slab_off = align_up(off);
  size_t slab_avail = region_end > slab_off ? region_end - slab_off : 0;
  constexpr size_t kSlabMax = (size_t)64 << 20;
  if (overlap) {
    const int h = ctx->parity;
    hipError_t e = hipEventRecord(ctx->fork_ev, ctx->stream);  // inputs produced on the context's stream are ready
    if (e == hipSuccess) e = hipStreamWaitEvent(ctx->aux[h], ctx->fork_ev, 0);
    if (e != hipSuccess) return hip_fail(ctx, e, "forking streams");
    const galore_status st = run_chain(ctx, items, lr, ctx->aux[h], reinterpret_cast<float*>(ctx->ws + slab_off),
                                       slab_avail < kSlabMax ? slab_avail : kSlabMax);
    for (const StepItem& it : items) ctx->in_flight[it.tensor] = (char)(1 + h);
    ctx->unjoined = true;
    ctx->parity = (ctx->parity + 1) % ctx->slots;
    if (st != GALORE_OK) (void)join_all(ctx);  // keep the context's stream ordered after a failed launch
    return st;
  }
  int lanes = ctx->lanes;
  if (lanes > 1 && !library_streams_ready(ctx)) lanes = 1;
  if ((int)items.size() < 2) lanes = 1;
  if (lanes <= 1)
    return run_chain(ctx, items, lr, ctx->stream, reinterpret_cast<float*>(ctx->ws + slab_off), slab_avail < kSlabMax ? slab_avail : kSlabMax);

  // Greedy balance by cost (m n, as r is shared): heaviest tensor first, always into the lightest chain.
  std::vector<int> order(items.size());
  for (size_t i = 0; i < items.size(); ++i) order[i] = (int)i;
  auto cost = [&](int i) { const TensorInfo& ti = ctx->tensors[items[i].tensor]; return (double)ti.rows * (double)ti.cols; };
  for (size_t a = 1; a < order.size(); ++a)  // insertion sort, descending cost, stable
    for (size_t b = a; b > 0 && cost(order[b]) > cost(order[b - 1]); --b) { const int x = order[b]; order[b] = order[b - 1]; order[b - 1] = x; }
  std::vector<StepItem> chain[3];
  double load[3] = {0, 0, 0};
  for (int i : order) {
    int best = 0;
    for (int c = 1; c < lanes; ++c)
      if (load[c] < load[best]) best = c;
    chain[best].push_back(items[i]);
    load[best] += cost(i);
  }
  hipError_t e = hipEventRecord(ctx->fork_ev, ctx->stream);
  for (int c = 1; c < lanes && e == hipSuccess; ++c)
    if (!chain[c].empty()) e = hipStreamWaitEvent(ctx->aux[c - 1], ctx->fork_ev, 0);
  if (e != hipSuccess) return hip_fail(ctx, e, "forking streams");
  galore_status st = GALORE_OK;
  for (int c = 0; c < lanes && st == GALORE_OK; ++c)
    if (!chain[c].empty()) {
      size_t part = (slab_avail / (size_t)lanes) & ~(size_t)255;  // every chain its own slab area
      st = run_chain(ctx, chain[c], lr, c == 0 ? ctx->stream : ctx->aux[c - 1],
                     reinterpret_cast<float*>(ctx->ws + slab_off + (size_t)c * part), part < kSlabMax ? part : kSlabMax);
    }
  // always join, also after a failed launch, so the caller's stream stays ordered after our streams
  for (int c = 1; c < lanes; ++c) {
    if (chain[c].empty()) continue;
    e = hipEventRecord(ctx->join_ev[c - 1], ctx->aux[c - 1]);
    if (e == hipSuccess) e = hipStreamWaitEvent(ctx->stream, ctx->join_ev[c - 1], 0);
    if (e != hipSuccess && st == GALORE_OK) st = hip_fail(ctx, e, "joining streams");
  }
  return st;
}

galore_status check_step_tensor(galore_ctx* ctx, const TensorInfo& ti, const galore_tensor& x, const char* what, int i) {
  galore_status s = check_matrix(ctx, x, what, i, true);
  if (s) return s;
  if (x.rows != ti.rows || x.cols != ti.cols)
    return fail(ctx, GALORE_ERR_SHAPE, "%s[%d] is %lld x %lld but the tensor was initialised as %lld x %lld", what, i,
                (long long)x.rows, (long long)x.cols, (long long)ti.rows, (long long)ti.cols);
  if ((DType)x.dtype != ti.dt) return fail(ctx, GALORE_ERR_DTYPE, "%s[%d] dtype differs from init", what, i);
  return GALORE_OK;
}

// Argument checks shared by galore_step and galore_step_static; nothing is enqueued on failure.
galore_status check_step_args(galore_ctx* ctx, const galore_tensor* W, const galore_tensor* G, int32_t first, int32_t count, float lr) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  const int n = (int)ctx->tensors.size();
  if (first < 0 || count < 0 || first > n || count > n - first)
    return fail(ctx, GALORE_ERR_INVALID_ARG, "range [%d, %d+%d) outside the %d tensors", first, first, count, n);
  if (count == 0) return GALORE_OK;
  if (!W || !G) return fail(ctx, GALORE_ERR_INVALID_ARG, "W or G is NULL");
  if (!std::isfinite(lr)) return fail(ctx, GALORE_ERR_INVALID_ARG, "lr is not finite");
  for (int i = 0; i < count; ++i) {
    const TensorInfo& ti = ctx->tensors[first + i];
    galore_status s = check_step_tensor(ctx, ti, W[i], "W", i);
    if (s) return s;
    s = check_step_tensor(ctx, ti, G[i], "G", i);
    if (s) return s;
  }
  return GALORE_OK;
}

galore_status run_refresh(galore_ctx* ctx, const galore_tensor* G, int32_t first, const std::vector<int>& local,
                          hipStream_t stream, unsigned char* ws, size_t ws_bytes) {
  // local: indices i (relative to `first`) of tensors to refresh, in order; [ws, ws + ws_bytes) is the
  // part of the workspace this refresh may use, `stream` the stream it runs on.
  // Tensors that start from their previous projector (see galore_hparams::refresh_warm_iters) run a
  // different number of iterations than those that start from the Gaussian block: two passes.
  const bool warm_allowed = ctx->hp.refresh_warm_iters > 0 && ctx->hp.auto_refresh;
  std::vector<int> lists[2];  // decided before anything runs: a cold refresh marks its tensors refreshed
  for (int i : local) lists[warm_allowed && ctx->tensors[first + i].refreshed ? 1 : 0].push_back(i);
  for (int pass = 0; pass < 2; ++pass) {
    const bool warm = pass == 1;
    const std::vector<int>& todo = lists[pass];
    size_t pos = 0;
    while (pos < todo.size()) {
      std::vector<RefreshItem> chunk;
      std::vector<int> chunk_tensors;
      size_t used = 0;
      while (pos < todo.size() && (int)chunk.size() < kMaxGroup) {
        const int i = todo[pos];
        TensorInfo& ti = ctx->tensors[first + i];
        const size_t need = refresh_workspace_bytes(ti.kdim, ctx->hp.rank);
        if (!chunk.empty() && used + need > ws_bytes) break;
        RefreshItem it{};
        it.G = G[i].data; it.ldg = G[i].ld; it.rows = ti.rows; it.cols = ti.cols;
        it.dt = ti.dt;
        it.proj = ti.st.proj.data; it.ldp = ti.st.proj.ld;
        it.proj_t = ti.st.proj_t.data; it.ldpt = ti.st.proj_t.ld;
        it.ws = ws + used;
        it.seed = ctx->hp.seed + 0x9E3779B97F4A7C15ull * (uint64_t)(first + i + 1);
        chunk.push_back(it);
        chunk_tensors.push_back(first + i);
        used += need;
        ++pos;
      }
      ProfScope prof(ctx, GALORE_STAGE_REFRESH, true, stream);
      hipError_t e = refresh_group(chunk, ctx->hp.rank, warm ? ctx->hp.refresh_warm_iters : ctx->hp.refresh_iters, warm,
                                   /*crowded=*/stream != ctx->stream, stream);
      if (e != hipSuccess) return hip_fail(ctx, e, "subspace refresh");
      for (int idx : chunk_tensors) {
        ctx->tensors[idx].proj_t_valid = true;  // the refresh writes proj and proj_t
        ctx->tensors[idx].refreshed = true;
      }
    }
  }
  return GALORE_OK;
}

}  // namespace

extern "C" {

const char* galore_status_string(galore_status s) {
  switch (s) {
    case GALORE_OK: return "ok";
    case GALORE_ERR_INVALID_ARG: return "invalid argument";
    case GALORE_ERR_SHAPE: return "shape mismatch";
    case GALORE_ERR_DTYPE: return "unsupported dtype";
    case GALORE_ERR_RANK: return "rank out of range";
    case GALORE_ERR_ALIGN: return "pointer alignment";
    case GALORE_ERR_WORKSPACE: return "workspace too small";
    case GALORE_ERR_STATE: return "state does not fit the tensor";
    case GALORE_ERR_HIP: return "HIP error";
    case GALORE_ERR_UNIMPLEMENTED: return "not implemented";
  }
  return "unknown status";
}

galore_status galore_workspace_bytes(const galore_hparams* hp, const galore_tensor* W, int32_t n_tensors,
                                     size_t* out_bytes) {
  galore_status s = check_hparams(nullptr, hp);
  if (s) return s;
  if (!W || !out_bytes || n_tensors < 1) return fail(nullptr, GALORE_ERR_INVALID_ARG, "W / out_bytes NULL or n_tensors < 1");
  std::vector<size_t> need(n_tensors);
  for (int i = 0; i < n_tensors; ++i) {
    s = check_weight_shape(nullptr, *hp, W[i], i);
    if (s) return s;
    const bool left = W[i].rows <= W[i].cols;
    need[i] = tensor_need(*hp, left, left ? W[i].rows : W[i].cols, left ? W[i].cols : W[i].rows, (DType)W[i].dtype);
  }
  size_t best = 0;
  for (int i = 0; i < n_tensors; ++i) {
    size_t sum = 0;
    for (int j = i; j < n_tensors && j < i + 8; ++j) sum += need[j];
    best = sum > best ? sum : best;
  }
  *out_bytes = best;
  return GALORE_OK;
}

galore_status galore_init(galore_ctx** out, const galore_hparams* hp, const galore_tensor* W, const galore_state* S,
                          int32_t n_tensors, void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (!out) return fail(nullptr, GALORE_ERR_INVALID_ARG, "out is NULL");
  *out = nullptr;
  galore_status s = check_hparams(nullptr, hp);
  if (s) return s;
  if (!W || !S || n_tensors < 1) return fail(nullptr, GALORE_ERR_INVALID_ARG, "W / S NULL or n_tensors < 1");
  if (!workspace) return fail(nullptr, GALORE_ERR_INVALID_ARG, "workspace is NULL");
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign)
    return fail(nullptr, GALORE_ERR_ALIGN, "workspace must be %zu-byte aligned", kAlign);

  std::vector<TensorInfo> infos(n_tensors);
  const int64_t r = hp->rank;
  for (int i = 0; i < n_tensors; ++i) {
    s = check_weight_shape(nullptr, *hp, W[i], i);
    if (s) return s;
    TensorInfo& ti = infos[i];
    ti.rows = W[i].rows; ti.cols = W[i].cols; ti.dt = (DType)W[i].dtype;
    ti.left = ti.rows <= ti.cols;
    ti.kdim = ti.left ? ti.rows : ti.cols;
    ti.ldim = ti.left ? ti.cols : ti.rows;
    ti.st = S[i];
    ti.t = 0;
    const galore_tensor& p = S[i].proj;
    s = check_matrix(nullptr, p, "S.proj", i, true);
    if (s) return s;
    if (p.rows != ti.kdim || p.cols != r)
      return fail(nullptr, GALORE_ERR_SHAPE, "S[%d].proj must be %lld x %lld", i, (long long)ti.kdim, (long long)r);
    if ((DType)p.dtype != ti.dt) return fail(nullptr, GALORE_ERR_DTYPE, "S[%d].proj dtype must equal the weight dtype", i);
    const galore_tensor& pt = S[i].proj_t;
    s = check_matrix(nullptr, pt, "S.proj_t", i, true);
    if (s) return s;
    if (pt.rows != r || pt.cols != ti.kdim)
      return fail(nullptr, GALORE_ERR_SHAPE, "S[%d].proj_t must be %lld x %lld", i, (long long)r, (long long)ti.kdim);
    if ((DType)pt.dtype != ti.dt) return fail(nullptr, GALORE_ERR_DTYPE, "S[%d].proj_t dtype must equal the weight dtype", i);
    ti.proj_t_valid = false;
    ti.refreshed = false;
    const int64_t mr = ti.left ? r : ti.rows, mc = ti.left ? ti.cols : r;
    const galore_tensor* mv[2] = {&S[i].m, &S[i].v};
    ti.q8 = S[i].m.dtype == GALORE_U8 || S[i].v.dtype == GALORE_U8;
    for (int q = 0; q < 2; ++q) {
      const galore_tensor& x = *mv[q];
      s = check_matrix(nullptr, x, q ? "S.v" : "S.m", i, true, true);
      if (s) return s;
      if (x.dtype != (ti.q8 ? GALORE_U8 : GALORE_F32))
        return fail(nullptr, GALORE_ERR_DTYPE, "S[%d] moments must both be fp32 or both be 8-bit codes", i);
      if (x.rows != mr || x.cols != mc || x.ld != mc)
        return fail(nullptr, GALORE_ERR_SHAPE, "S[%d] moments must be dense %lld x %lld", i, (long long)mr, (long long)mc);
      if (reinterpret_cast<uintptr_t>(x.data) & 15)
        return fail(nullptr, GALORE_ERR_ALIGN, "S[%d] moments must be 16-byte aligned", i);
    }
    if (ti.q8) {
      if (mc % 256 != 0)
        return fail(nullptr, GALORE_ERR_UNIMPLEMENTED, "S[%d]: 8-bit moments need rows of a multiple of 256 elements, got %lld", i,
                    (long long)mc);
      const galore_tensor* sc[2] = {&S[i].m_scale, &S[i].v_scale};
      for (int q = 0; q < 2; ++q) {
        const galore_tensor& x = *sc[q];
        s = check_matrix(nullptr, x, q ? "S.v_scale" : "S.m_scale", i, true);
        if (s) return s;
        if (x.dtype != GALORE_F32) return fail(nullptr, GALORE_ERR_DTYPE, "S[%d] moment scales must be fp32", i);
        if (x.rows != mr || x.cols != mc / 256 || x.ld != x.cols)
          return fail(nullptr, GALORE_ERR_SHAPE, "S[%d] moment scales must be dense %lld x %lld", i, (long long)mr, (long long)(mc / 256));
      }
    }
    if (tensor_need(*hp, ti.left, ti.kdim, ti.ldim, ti.dt) > workspace_bytes)
      return fail(nullptr, GALORE_ERR_WORKSPACE, "workspace of %zu bytes cannot hold tensor %d (needs %zu)", workspace_bytes,
                  i, tensor_need(*hp, ti.left, ti.kdim, ti.ldim, ti.dt));
  }

  galore_ctx* ctx = new (std::nothrow) galore_ctx;
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "out of host memory");
  ctx->hp = *hp;
  ctx->tensors = std::move(infos);
  ctx->ws = static_cast<unsigned char*>(workspace);
  ctx->ws_bytes = workspace_bytes;
  ctx->stream = static_cast<hipStream_t>(hip_stream);
  ctx->in_flight.assign(ctx->tensors.size(), 0);
  {
    hipError_t e = hipSuccess;
    for (int i = 0; i < kLibStreams && e == hipSuccess; ++i) {
      e = hipStreamCreateWithFlags(&ctx->aux[i], hipStreamNonBlocking);
      if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->join_ev[i], hipEventDisableTiming);
    }
    if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->fork_ev, hipEventDisableTiming);
    if (e != hipSuccess) {
      galore_status st = hip_fail(nullptr, e, "creating streams");
      galore_destroy(ctx);
      return st;
    }
  }
  {  // set-up of galore_step_static: this device's address of the static scratch array
    unsigned char* sp = nullptr;
    hipError_t e = static_scratch_ptr(&sp);
    if (e != hipSuccess) {
      galore_status st = hip_fail(nullptr, e, "resolving the static scratch array");
      galore_destroy(ctx);
      return st;
    }
  }
  // M_0 = V_0 = 0 (Algorithm 2, initialisation)
  for (const TensorInfo& ti : ctx->tensors) {
    const size_t bytes = (size_t)r * ti.ldim * (ti.q8 ? 1 : 4);  // code 0 decodes to 0
    hipError_t e = launch_fill_zero(ti.st.m.data, bytes, ctx->stream);
    if (e == hipSuccess) e = launch_fill_zero(ti.st.v.data, bytes, ctx->stream);
    if (ti.q8 && e == hipSuccess) e = launch_fill_zero(ti.st.m_scale.data, (size_t)r * ti.ldim / 256 * 4, ctx->stream);
    if (ti.q8 && e == hipSuccess) e = launch_fill_zero(ti.st.v_scale.data, (size_t)r * ti.ldim / 256 * 4, ctx->stream);
    if (e != hipSuccess) {
      galore_status st = hip_fail(nullptr, e, "zero-filling moments");
      galore_destroy(ctx);  // also releases the library streams and events
      return st;
    }
  }
  *out = ctx;
  return GALORE_OK;
}

galore_status galore_step(galore_ctx* ctx, const galore_tensor* W, const galore_tensor* G, int32_t first, int32_t count,
                          float lr) {
  galore_status s0 = check_step_args(ctx, W, G, first, count, lr);
  if (s0) return s0;
  if (count == 0) return GALORE_OK;
  // Refresh branch of Algorithm 2: t mod T == 0, on this step's gradient, before projecting.
  if (ctx->hp.auto_refresh) {
    std::vector<int> due;
    for (int i = 0; i < count; ++i)
      if (ctx->tensors[first + i].t % ctx->hp.update_gap == 0) due.push_back(i);
    if (!due.empty()) {
      size_t rneed = 0;
      for (int i : due) rneed += refresh_workspace_bytes(ctx->tensors[first + i].kdim, ctx->hp.rank);
      const int h = ctx->parity;
      // With overlapping calls the refresh runs where this call's step will run: on library stream h,
      // in share h of the workspace (the step's transients follow there on the same stream), if it fits.
      const bool on_library_stream = ctx->overlap_calls && library_streams_ready(ctx) &&
                                     (int)due.size() <= kMaxGroup && rneed <= workspace_share(ctx);
      bool clash = !on_library_stream;  // otherwise: the context's stream and the whole workspace
      for (int i : due) clash = clash || (ctx->in_flight[first + i] != 0 && ctx->in_flight[first + i] != 1 + h);
      if (ctx->unjoined && clash) {
        galore_status s = join_all(ctx);
        if (s) return s;
      }
      if (on_library_stream) {
        hipError_t e = hipEventRecord(ctx->fork_ev, ctx->stream);  // the gradients are ready on the context's stream
        if (e == hipSuccess) e = hipStreamWaitEvent(ctx->aux[h], ctx->fork_ev, 0);
        if (e != hipSuccess) return hip_fail(ctx, e, "forking streams");
        for (int i : due) ctx->in_flight[first + i] = (char)(1 + h);
        ctx->unjoined = true;
        galore_status s = run_refresh(ctx, G, first, due, ctx->aux[h], ctx->ws + (size_t)h * workspace_share(ctx), workspace_share(ctx));
        if (s) { (void)join_all(ctx); return s; }
      } else {
        galore_status s = run_refresh(ctx, G, first, due, ctx->stream, ctx->ws, ctx->ws_bytes);
        if (s) return s;
      }
    }
  }
  // with overlapping calls a chunk has to fit one call's share of the workspace
  const size_t limit = ctx->overlap_calls ? workspace_share(ctx) : ctx->ws_bytes;
  int pos = 0;
  while (pos < count) {
    std::vector<StepItem> items;
    size_t used = 0;
    while (pos < count && (int)items.size() < kMaxGroup) {
      const TensorInfo& ti = ctx->tensors[first + pos];
      const size_t need = step_need(ti.left, ti.kdim, ti.ldim, ctx->hp.rank, ti.dt);
      if (!items.empty() && used + need > limit) break;
      items.push_back(StepItem{first + pos, &W[pos], &G[pos], nullptr, nullptr, nullptr, ti.ldim});
      used += need;
      ++pos;
    }
    galore_status s = run_step_chunk(ctx, items, lr);
    if (s) return s;
  }
  for (int i = 0; i < count; ++i) ctx->tensors[first + i].t += 1;
  return GALORE_OK;
}

galore_status galore_step_static(galore_ctx* ctx, const galore_tensor* W, const galore_tensor* G, int32_t first,
                                 int32_t count, float lr) {
  galore_status s = check_step_args(ctx, W, G, first, count, lr);
  if (s) return s;
  if (count == 0) return GALORE_OK;
  if (ctx->profiling) return fail(ctx, GALORE_ERR_INVALID_ARG, "galore_step_static cannot run between galore_profile_start and _stop (the brackets create events)");
  const int r = ctx->hp.rank;
  for (int i = 0; i < count; ++i) {
    const TensorInfo& ti = ctx->tensors[first + i];
    if (ctx->hp.auto_refresh && ti.t % ctx->hp.update_gap == 0)
      return fail(ctx, GALORE_ERR_UNIMPLEMENTED, "tensor %d is due for a subspace refresh (t = %lld, T = %d), whose working set of %zu bytes "
                  "exceeds the static scratch array: take this step with galore_step", first + i, (long long)ti.t, ctx->hp.update_gap,
                  refresh_workspace_bytes(ti.kdim, r));
    const size_t need = step_need(ti.left, ti.kdim, ti.ldim, r, ti.dt);
    if (need > kStaticScratchBytes)
      return fail(ctx, GALORE_ERR_WORKSPACE, "tensor %d needs %zu bytes of transients, the static scratch array holds %zu", first + i, need,
                  kStaticScratchBytes);
  }
  unsigned char* sp = nullptr;
  hipError_t e = static_scratch_ptr(&sp);  // this device's copy of the array; never the array's name
  if (e != hipSuccess) return hip_fail(ctx, e, "resolving the static scratch array");
  if (ctx->unjoined) {  // overlapped calls may still hold these tensors on a library stream
    s = join_all(ctx);
    if (s) return s;
  }
  // Launch groups of as many consecutive tensors as fit the array, one chain on the context's stream.
  // Stream order protects the array between groups and between calls on this stream.
  int pos = 0;
  while (pos < count) {
    std::vector<StepItem> items;
    size_t off = 0;
    while (pos < count && (int)items.size() < kMaxGroup) {
      const TensorInfo& ti = ctx->tensors[first + pos];
      const size_t need = step_need(ti.left, ti.kdim, ti.ldim, r, ti.dt);
      if (off + need > kStaticScratchBytes) break;
      StepItem it{first + pos, &W[pos], &G[pos], nullptr, nullptr, nullptr, ti.ldim};
      it.R = reinterpret_cast<float*>(sp + off);
      off += step_r_bytes(ti.left, ti.kdim, ti.ldim, r, ti.dt);
      it.N = sp + off;
      off += step_n_bytes(ti.ldim, r, ti.dt);
      const size_t gp = step_gpad_bytes(ti.left, ti.kdim, ti.ldim, ti.dt);
      it.Gpad = gp ? sp + off : nullptr;
      off += gp;
      it.ldr = projected_row_length(ti.left, ti.kdim, ti.ldim, ti.dt);
      items.push_back(it);
      ++pos;
    }
    const size_t slab_off = align_up(off);  // what is left of the array holds the projection's partial tiles
    s = run_chain(ctx, items, lr, ctx->stream, reinterpret_cast<float*>(sp + slab_off),
                  kStaticScratchBytes > slab_off ? kStaticScratchBytes - slab_off : 0);
    if (s) return s;
  }
  for (int i = 0; i < count; ++i) ctx->tensors[first + i].t += 1;
  return GALORE_OK;
}

galore_status galore_refresh_subspace(galore_ctx* ctx, const galore_tensor* G, int32_t first, int32_t count) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  const int n = (int)ctx->tensors.size();
  if (first < 0 || count < 0 || first > n || count > n - first)
    return fail(ctx, GALORE_ERR_INVALID_ARG, "range [%d, %d+%d) outside the %d tensors", first, first, count, n);
  if (count == 0) return GALORE_OK;
  if (!G) return fail(ctx, GALORE_ERR_INVALID_ARG, "G is NULL");
  std::vector<int> all(count);
  for (int i = 0; i < count; ++i) {
    galore_status s = check_step_tensor(ctx, ctx->tensors[first + i], G[i], "G", i);
    if (s) return s;
    all[i] = i;
  }
  if (ctx->unjoined) {
    galore_status s = join_all(ctx);
    if (s) return s;
  }
  return run_refresh(ctx, G, first, all, ctx->stream, ctx->ws, ctx->ws_bytes);
}

galore_status galore_get_step(const galore_ctx* ctx, int32_t tensor, int64_t* t) {
  if (!ctx || !t) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx or t is NULL");
  if (tensor < 0 || tensor >= (int)ctx->tensors.size())
    return fail(nullptr, GALORE_ERR_INVALID_ARG, "tensor index %d out of range", tensor);
  *t = ctx->tensors[tensor].t;
  return GALORE_OK;
}

galore_status galore_set_step(galore_ctx* ctx, int32_t tensor, int64_t t) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  if (tensor < 0 || tensor >= (int)ctx->tensors.size())
    return fail(ctx, GALORE_ERR_INVALID_ARG, "tensor index %d out of range", tensor);
  if (t < 0) return fail(ctx, GALORE_ERR_INVALID_ARG, "step counter must be >= 0");
  ctx->tensors[tensor].t = t;
  ctx->tensors[tensor].proj_t_valid = false;  // a resumed projector was written by the caller
  ctx->tensors[tensor].refreshed = false;
  return GALORE_OK;
}

const char* galore_last_error(const galore_ctx* ctx) { return ctx ? ctx->err.c_str() : g_last_error.c_str(); }

void galore_destroy(galore_ctx* ctx) {
  if (!ctx) return;
  for (ProfRecord& r : ctx->records) { (void)hipEventDestroy(r.begin); (void)hipEventDestroy(r.end); }
  for (hipEvent_t e : ctx->event_pool) (void)hipEventDestroy(e);
  for (int i = 0; i < kLibStreams; ++i) {
    if (ctx->aux[i]) { (void)hipStreamSynchronize(ctx->aux[i]); (void)hipStreamDestroy(ctx->aux[i]); }
    if (ctx->join_ev[i]) (void)hipEventDestroy(ctx->join_ev[i]);
  }
  if (ctx->fork_ev) (void)hipEventDestroy(ctx->fork_ev);
  delete ctx;
}

galore_status galore_set_concurrency(galore_ctx* ctx, int32_t lanes) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  if (lanes < 1 || lanes > 3) return fail(ctx, GALORE_ERR_INVALID_ARG, "lanes must be 1, 2 or 3");
  ctx->lanes = lanes;
  return GALORE_OK;
}

galore_status galore_set_fused_adam(galore_ctx* ctx, int32_t on) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  ctx->fused_adam = on != 0;
  return GALORE_OK;
}

galore_status galore_set_call_overlap(galore_ctx* ctx, int32_t on) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  if (on < 0 || on > kLibStreams) return fail(ctx, GALORE_ERR_INVALID_ARG, "on must be 0 ... %d", kLibStreams);
  const int slots = on <= 2 ? 2 : on;
  // turning it off, or changing how the workspace is divided, orders everything first
  if (ctx->unjoined && (on == 0 || slots != ctx->slots)) {
    galore_status s = join_all(ctx);
    if (s) return s;
  }
  ctx->overlap_calls = on != 0;
  if (slots != ctx->slots) { ctx->slots = slots; ctx->parity = 0; }
  return GALORE_OK;
}

galore_status galore_join(galore_ctx* ctx) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  if (!ctx->unjoined) return GALORE_OK;
  return join_all(ctx);
}

galore_status galore_get_stream(const galore_ctx* ctx, int32_t which, void** out_stream) {
  if (!ctx || !out_stream) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx or out_stream is NULL");
  if (which < 0 || which >= kLibStreams) return fail(nullptr, GALORE_ERR_INVALID_ARG, "which must be 0 ... %d", kLibStreams - 1);
  *out_stream = ctx->aux[which];
  return GALORE_OK;
}

galore_status galore_profile_start(galore_ctx* ctx) {
  if (!ctx) return fail(nullptr, GALORE_ERR_INVALID_ARG, "ctx is NULL");
  for (ProfRecord& r : ctx->records) { ctx->event_pool.push_back(r.begin); ctx->event_pool.push_back(r.end); }
  ctx->records.clear();
  ctx->profiling = true;
  return GALORE_OK;
}

galore_status galore_profile_stop(galore_ctx* ctx, double* ms, int64_t* launches) {
  if (!ctx || !ms || !launches) return fail(ctx, GALORE_ERR_INVALID_ARG, "NULL argument");
  ctx->profiling = false;
  for (int i = 0; i < GALORE_STAGE_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
  galore_status st = GALORE_OK;
  for (ProfRecord& r : ctx->records) {
    float t = 0.f;
    hipError_t e = hipEventSynchronize(r.end);
    if (e == hipSuccess) e = hipEventElapsedTime(&t, r.begin, r.end);
    if (e != hipSuccess) st = hip_fail(ctx, e, "reading profile events");
    else { ms[r.stage] += t; launches[r.stage] += 1; }
    ctx->event_pool.push_back(r.begin);
    ctx->event_pool.push_back(r.end);
  }
  ctx->records.clear();
  return st;
}

}  // extern "C"
