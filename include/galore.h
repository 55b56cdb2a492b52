/*
 * galore.h - C ABI of the MI355X (gfx950) GaLore optimizer-step library.
 *
 * The library performs, for a list of 2-D weights, the step of "Adam with GaLore"
 * (arXiv 2403.03507, Algorithm 2):
 *
 *     if t mod T == 0:  P <- leading r singular vectors of G          (refresh)
 *     R = P^T G                                                       (project)
 *     M <- b1 M + (1-b1) R ;  V <- b2 V + (1-b2) R^2                  (Adam moments)
 *     N = (M / (1-b1^k)) / (sqrt(V / (1-b2^k)) + eps),  k = t+1       (normalised update)
 *     W <- (1 - lr*wd) W - lr * alpha * P N                           (project back + apply)
 *     t <- t+1
 *
 * Orientation (Sec. 4.2, one-sided projection): a tensor with rows <= cols is LEFT
 * (projector P is rows x r; R, M, V, N are r x cols); a tensor with rows > cols is
 * RIGHT (projector Q is cols x r; R = G Q, M, V, N are rows x r; update is N Q^T).
 *
 * Conventions common to every call
 *   - All tensor data pointers are DEVICE pointers (HIP global memory of the current
 *     device), row-major, leading dimension `ld` in elements (ld >= cols).  They are
 *     BORROWED: the library never allocates, frees or keeps device memory of its own
 *     except through the caller's workspace (one exception, stated there: the static
 *     device array that galore_step_static uses in place of the workspace).  Argument structs and arrays of structs
 *     are HOST memory and are copied during the call.
 *   - The gradient is the positive gradient of the loss; the update is subtracted.
 *     (The paper negates the gradient and adds; the trajectory is the same.)
 *   - Work is enqueued on the HIP stream given to galore_init (or to the stateless
 *     stage calls) and the call returns without synchronising.
 *   - Every call returns a galore_status.  Arguments are validated on the host before
 *     anything is launched; on a validation error nothing has been enqueued.
 *   - Results are deterministic: no atomics, fixed reduction order.
 */
#ifndef GALORE_H
#define GALORE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GALORE_OK = 0,
  GALORE_ERR_INVALID_ARG = 1, /* null pointer, bad count/range, bad hyper-parameter */
  GALORE_ERR_SHAPE = 2,       /* tensor shapes inconsistent with each other / with init */
  GALORE_ERR_DTYPE = 3,       /* dtype combination not supported */
  GALORE_ERR_RANK = 4,        /* rank outside 1..min(rows, cols) */
  GALORE_ERR_ALIGN = 5,       /* state / workspace pointer not 16-byte aligned */
  GALORE_ERR_WORKSPACE = 6,   /* workspace too small for even one tensor */
  GALORE_ERR_STATE = 7,       /* a state argument that does not fit its tensor (the two-sided calls: shapes of p, q, m, v).
                                 Not a check of call order: with auto_refresh = 0 the projector contents are the
                                 caller's, and the library cannot tell an unwritten projector from a written one */
  GALORE_ERR_HIP = 8,         /* a HIP runtime call or kernel launch failed */
  GALORE_ERR_UNIMPLEMENTED = 9
} galore_status;

typedef enum { GALORE_F32 = 0, GALORE_BF16 = 1, GALORE_U8 = 2 /* 8-bit moment codes only */ } galore_dtype;

/* A row-major matrix in device memory.  BORROWED. */
typedef struct {
  void* data;   /* device pointer */
  int64_t rows;
  int64_t cols;
  int64_t ld;   /* elements between consecutive rows, >= cols */
  int32_t dtype; /* galore_dtype */
} galore_tensor;

/* Optimizer state of one weight.  BORROWED, caller-allocated, survives across steps.
 *   proj   : P (rows x r) for LEFT, Q (cols x r) for RIGHT; dtype = dtype of W.
 *   m, v   : fp32, r x cols (LEFT) or rows x r (RIGHT), ld == cols, 16-byte aligned.
 *   proj_t : r x min(rows, cols), dtype of W: the projector transposed.  Derived data that
 *            the library maintains (rewritten after every refresh, and from proj at every
 *            step when auto_refresh == 0), kept so that both GEMMs of the step read the
 *            projector with its contraction index contiguous.  Its initial contents do not
 *            matter and a checkpoint need not save it.
 * proj, m, v hold min(rows,cols)*r + 2*max(rows,cols)*r elements, the paper's mr + 2nr
 * (Sec. 4.2); proj_t adds another min(rows,cols)*r.
 *
 * 8-bit moments (the "8-bit GaLore" of Sec. 4.3; the number format is this library's own, the
 * paper prints none): give m and v dtype GALORE_U8 (same shapes, one byte per element) and set
 *   m_scale, v_scale : fp32, (rows of m) x (cols of m / 256), ld == cols: one scale per block of
 *                      256 consecutive elements of a row (max |m| and max v of the block).
 * m code: sign | 4 exponent bits e | 3 mantissa bits f, magnitude (1 + f/8) 2^(e-15) for e > 0,
 * (f/8) 2^-14 for e = 0; v code: 5 exponent bits | 3 mantissa bits, (1 + f/8) 2^(e-31) and
 * (f/8) 2^-30; value = magnitude * scale; quantisation rounds min(|x| * (1 / scale), 1) to the
 * nearest magnitude, ties to the even mantissa field.  Needs cols of m to be a multiple of 256
 * (GALORE_ERR_UNIMPLEMENTED otherwise).  With fp32 moments m_scale and v_scale are ignored
 * (data may be NULL). */
typedef struct {
  galore_tensor proj;
  galore_tensor m;
  galore_tensor v;
  galore_tensor proj_t;
  galore_tensor m_scale;
  galore_tensor v_scale;
} galore_state;

/* Hyper-parameters (Algorithm 2 inputs; Sec. 4.4).  Paper defaults: update_gap 200,
 * scale 0.25, betas (0.9, 0.999), eps 1e-8. */
typedef struct {
  int32_t rank;          /* r */
  int32_t update_gap;    /* T, >= 1 */
  float scale;           /* alpha */
  float beta1;
  float beta2;
  float eps;
  float weight_decay;    /* decoupled, multiplies lr only (not alpha); 0 = Algorithm 2 as printed */
  int32_t refresh_iters; /* subspace iterations per refresh, >= 1 */
  int32_t auto_refresh;  /* 1: galore_step refreshes the projector itself when t mod T == 0;
                            0: the caller owns the projector contents (writes state.proj or
                               calls galore_refresh_subspace) */
  int32_t refresh_warm_iters; /* 0: every refresh starts from the seeded Gaussian block and runs
                            refresh_iters iterations.  > 0 (needs auto_refresh = 1): a tensor whose
                            projector was written by an earlier refresh of this context starts the
                            iteration from that projector and runs this many iterations instead
                            (this build's option, not the paper's, which calls an exact SVD: the
                            iteration converges to the same top-r vectors from any start of full
                            rank, and needs fewer rounds when the gradients of consecutive refreshes
                            span nearby subspaces); galore_set_step makes the tensor's next refresh
                            a cold one again.  >= 0 */
  uint64_t seed;         /* seed of the Gaussian start block of the first refresh */
} galore_hparams;

typedef struct galore_ctx galore_ctx; /* opaque; OWNED by the library; host memory only */

/* Human-readable text for a status code (static storage). */
const char* galore_status_string(galore_status s);

/* Workspace, in bytes, that lets one call process up to 8 consecutive tensors of the
 * list per kernel launch (transients R and N of the step, plus, for a bf16 tensor with
 * rows <= cols, rows a multiple of 64 and cols not a multiple of 8, a copy of G with its rows
 * padded to a multiple of 8 elements, which the projection then reads instead of G; Gram
 * matrix, iteration blocks and reflector storage of the refresh).  Any 256-byte-aligned workspace at least as
 * large as the largest single-tensor need is accepted by galore_init; a smaller one
 * only means more, smaller launches.  What a call's transients leave free of its share of the
 * workspace also serves, up to 64 MiB, as the area for the partial tiles of projection tiles that are cut
 * along K (see galore_set_concurrency); without room for them nothing is cut.  No device access. */
galore_status galore_workspace_bytes(const galore_hparams* hp, const galore_tensor* W,
                                     int32_t n_tensors, size_t* out_bytes);

/* Create a context for a list of n_tensors weights and their states (Algorithm 2,
 * initialisation lines): validates everything, records shapes and state pointers,
 * zero-fills every M and V on `hip_stream` (hipStream_t, may be NULL for the default
 * stream) and sets every step counter t to 0.  Projectors are left untouched.
 * The W entries are used for shape/dtype only; data pointers are given per step.
 * On error *out is NULL. */
galore_status galore_init(galore_ctx** out, const galore_hparams* hp, const galore_tensor* W,
                          const galore_state* S, int32_t n_tensors, void* workspace,
                          size_t workspace_bytes, void* hip_stream);

/* One optimizer step (the loop body of Algorithm 2) for tensors first..first+count-1 of
 * the list, in list order.  W[i], G[i] (i = 0..count-1) describe tensor first+i; shapes and
 * dtypes must match those given at init.  W is updated in place; G is read only.  With
 * auto_refresh, tensors whose counter satisfies t mod T == 0 first get a new projector
 * from this G.  Each tensor's counter advances by one.  Calling with a sub-range lets a
 * training loop update one layer at a time during back-propagation (Sec. 4.3). */
galore_status galore_step(galore_ctx* ctx, const galore_tensor* W, const galore_tensor* G,
                          int32_t first, int32_t count, float lr);

/* galore_step for callers that cannot allocate device memory or size a workspace at call time: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * same kernels and bit-identical results, but the transients of the step (R, N and, for a bf16 tensor
 * with an odd row length, the padded copy of G) live in a file-scope device array of the library,
 * 80 MiB on every GPU the library runs on, held until the process ends, instead of the caller's
 * workspace; the call allocates nothing (no hipMalloc / hipFree, no events, no streams).  The tensors
 * run as one chain on the context's stream, in launch groups of as many consecutive tensors as fit
 * the array (galore_set_concurrency and galore_set_call_overlap do not apply; pending overlapped
 * calls are joined first).
 * Limits: GALORE_ERR_WORKSPACE if one tensor's transients exceed the array (4 r max(rows, cols) bytes
 * of R plus s r max(rows, cols) of N, s = element size of W; every tensor of the LLaMA 60M ... 7B
 * stacks at the paper's ranks fits); GALORE_ERR_UNIMPLEMENTED if auto_refresh is on and a tensor of
 * the call is due for a subspace refresh (t mod T == 0: the refresh needs hundreds of MB; take that
 * step with galore_step); GALORE_ERR_INVALID_ARG between galore_profile_start and _stop.  On any
 * error nothing has been enqueued and no counter has advanced.
 * Every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (other streams,
 * other contexts, other threads) race on it.  Calls on one stream are ordered by the stream. */
galore_status galore_step_static(galore_ctx* ctx, const galore_tensor* W, const galore_tensor* G,
                                 int32_t first, int32_t count, float lr);

/* Recompute the projectors of tensors first..first+count-1 from the gradients G
 * (Algorithm 2, refresh branch; Sec. 3.3 SVD equation): the leading r left (LEFT) or right
 * (RIGHT) singular vectors of G, obtained from the Gram matrix of the short side by
 * blocked subspace iteration with Householder QR and a final Rayleigh-Ritz rotation, so
 * columns are ordered by decreasing singular value; each column's sign makes its
 * largest-magnitude entry positive.  Writes state.proj and its transposed copy state.proj_t; M, V, W
 * and t are untouched.
 * A gradient of rank below r (the zero matrix included) gets an orthonormal projector whose
 * span holds all of G; which vectors complete it is not determined by G.  The Gram matrix is
 * formed in fp32: entries of G beyond about 1e17 in magnitude overflow it, and such a gradient,
 * like one with inf or NaN entries, yields a projector (and, in galore_step, moments and weights)
 * with non-finite entries; no error is reported and no kernel misbehaves, the caller is
 * expected to skip steps whose gradients are not finite.
 * Environment: GALORE_REFRESH_FP32_PRODUCTS=1 (read once per process) makes the iteration's
 * products Qt C run on the fp32 matrix cores instead of as split-bf16 products of the same
 * accuracy; it exists for comparison and changes workspace needs, so set it before the first call. */
galore_status galore_refresh_subspace(galore_ctx* ctx, const galore_tensor* G, int32_t first,
                                      int32_t count);

/* Number of independent chains (1..3, default 3) into which one galore_step call splits its
 * tensors.  Chains run project -> Adam -> project back for disjoint tensors on the context's
 * stream and on up to two library-owned streams of default priority, forked from and joined
 * back into the context's stream with events inside the call, so tail waves of one GEMM and the
 * bandwidth-bound Adam pass overlap with another chain's MFMA work.  1 = strictly serial on the
 * context's stream.  W, M, V agree between settings to the fp32 rounding of R, and bit for bit whenever
 * the projection launches cut no tile into K pieces (short sides under 512) or cut the same tiles
 * the same way: the projection sums the K range of a tile that does not fill a round of the chip
 * in pieces, and which tiles those are depends on what shares the launch.  For one setting and one
 * sequence of calls results are bit-identical from run to run. */
galore_status galore_set_concurrency(galore_ctx* ctx, int32_t lanes);

/* Adam inside the projection (off by default; 1 = on).  When on, a bf16 tensor with fp32 moments whose
 * projection runs on the large-tile kernel gets the update block of Algorithm 2 (moments, bias correction,
 * N) computed in that GEMM's epilogue, on the accumulators: R is never written to memory and read back,
 * and the step of such a tensor is two kernels instead of three.  Other tensors (fp32, 8-bit moments,
 * shapes the large-tile kernel does not take) keep the separate Adam kernel.  Both paths evaluate the
 * same fp32 expression on the same R: W, M, V are bit-identical between the two settings. */
galore_status galore_set_fused_adam(galore_ctx* ctx, int32_t on);

/* Overlap of consecutive calls (off by default; on = 0 off, 1 or 2 = two calls in flight, 3 =
 * three).  When on, every galore_step call runs as ONE chain (all its tensors grouped in each
 * kernel launch) on one of `on` library-owned streams of default priority, taking turns from call
 * to call.  The stream waits for the context's stream at the start of the call (so gradients
 * produced there are ready) but is NOT joined back into it at the end: the bandwidth-bound Adam
 * pass and the GEMM tails of one call overlap with the GEMMs of the next one (per-layer calls of
 * one optimizer step), and so do the many short launches of the subspace refreshes of consecutive
 * calls.  Call c uses share (c mod on) of the workspace, one of `on` equal parts, so its step runs
 * this way only if the transients of its tensors fit one share, and a refresh that is due only if
 * its working set fits one share (a workspace of `on` times galore_workspace_bytes always
 * suffices); otherwise, and whenever a tensor of the call is still in flight on another
 * stream, the library joins first and proceeds as without overlap.  The caller must call
 * galore_join() before work on the context's stream (or the host) reads or writes W, M, V or the
 * projectors of tensors passed since the last join, and must not overwrite their G buffers before
 * it.  galore_set_concurrency does not apply to overlapped calls.  Results depend on the setting as
 * described for galore_set_concurrency (fp32 rounding of R at most).  Turning it off, or changing the
 * number of calls in flight, joins.
 * Errors: GALORE_ERR_INVALID_ARG for on outside 0 ... 3. */
galore_status galore_set_call_overlap(galore_ctx* ctx, int32_t on);

/* Make the context's stream wait for everything the library streams hold (no host wait).
 * A no-op when nothing is pending. */
galore_status galore_join(galore_ctx* ctx);

/* The three library-owned HIP streams (which = 0, 1, 2), for callers whose allocator must know which
 * streams still read a gradient buffer it is about to recycle (with overlapped calls the library
 * reads G on these streams after galore_step has returned).  The streams stay owned by the
 * library and die with the context. */
galore_status galore_get_stream(const galore_ctx* ctx, int32_t which, void** out_stream);

/* Step counter t of one tensor (number of steps taken); set is for checkpoint resume. */
galore_status galore_get_step(const galore_ctx* ctx, int32_t tensor, int64_t* t);
galore_status galore_set_step(galore_ctx* ctx, int32_t tensor, int64_t t);

/* Message of the last failing call on this context ("" if none).  With ctx == NULL,
 * the message of the last failing galore_init / stateless call of this thread. */
const char* galore_last_error(const galore_ctx* ctx);

/* Free the host-side context.  Device memory is the caller's. */
void galore_destroy(galore_ctx* ctx);

/* ---- Stateless stage calls: the three per-step stages of Algorithm 2 on one tensor. ----
 * They run the same kernels galore_step runs and exist so each stage can be checked and
 * timed alone. */

/* dst (cols x rows) = src^T, same dtype.  galore_step uses it to derive state.proj_t. */
galore_status galore_transpose(const galore_tensor* src, const galore_tensor* dst, void* hip_stream);

/* R = P^T G (LEFT) or G Q (RIGHT) (Algorithm 2, projection line).  proj_t is the TRANSPOSED
 * projector, r x min(rows, cols), dtype of G.  R is fp32, r x cols or rows x r, ld == its cols. */
galore_status galore_project(const galore_tensor* proj_t, const galore_tensor* G,
                             const galore_tensor* R, void* hip_stream);

/* Adam on the projected gradient (Algorithm 2, update block): updates fp32 M, V (R's shape,
 * dense) in place and writes N (fp32 or bf16, dense).  With transpose_n == 0, N has R's shape;
 * with transpose_n != 0, N is stored transposed (R.cols x R.rows), which is what
 * galore_project_back expects for a LEFT tensor.  k >= 1 is the 1-based step used by the
 * bias correction. */
galore_status galore_adam(const galore_tensor* R, const galore_tensor* M, const galore_tensor* V,
                          const galore_tensor* N, int32_t transpose_n, float beta1, float beta2,
                          float eps, int64_t k, void* hip_stream);

/* The same stage with 8-bit moments (see galore_state): Mc, Vc are GALORE_U8 with R's shape,
 * Ms, Vs fp32 (R rows) x (R cols / 256); R's cols must be a multiple of 256.  Codes and scales
 * are updated in place; N as in galore_adam. */
galore_status galore_adam_q8(const galore_tensor* R, const galore_tensor* Mc, const galore_tensor* Vc,
                             const galore_tensor* Ms, const galore_tensor* Vs, const galore_tensor* N,
                             int32_t transpose_n, float beta1, float beta2, float eps, int64_t k, void* hip_stream);

/* W <- (1 - lr*weight_decay) W - lr*scale * (P N  or  N Q^T) (Algorithm 2, last lines),
 * applied inside the GEMM epilogue; the full-size update is never stored.  N is
 * max(rows, cols) x r for both orientations (i.e. transposed for a LEFT tensor), dense.
 * N dtype == proj dtype == W dtype. */
galore_status galore_project_back(const galore_tensor* proj, const galore_tensor* N,
                                  const galore_tensor* W, float lr, float scale,
                                  float weight_decay, void* hip_stream);

/* ---- Two-sided projection (Sec. 3.3, Definition 3.6) ----
 * The general rule the paper states before it drops one projector for memory (Sec. 4.2):
 *     G~ = P rho(P^T G Q) Q^T,   P = [u_1..u_r] (m x r),  Q = [v_1..v_r] (n x r)  of  G = U S V^T,
 * with rho = the Adam map of Algorithm 2's update block on the r x r matrix R = P^T G Q:
 *     W <- (1 - lr*weight_decay) W - lr*scale * P N Q^T.
 * State per tensor: mr + nr + 2 r^2 elements.  One tensor per call, no context: the caller keeps
 * the step count t (0-based, as in galore_get_step) and clears M, V before the first step.
 * All tensors are BORROWED device memory, row-major; p, q have W's dtype, m, v are fp32, r x r, dense.
 * The calls enqueue on hip_stream and return; errors as for the other calls (galore_last_error(NULL)). */
typedef struct {
  galore_tensor p;   /* m x r */
  galore_tensor q;   /* n x r */
  galore_tensor m;   /* r x r, fp32, ld == r */
  galore_tensor v;   /* r x r, fp32, ld == r */
} galore_two_sided_state;

/* Bytes of device workspace (256-byte aligned) the two calls below need for a weight of W's shape
 * and dtype; uses hp->rank. */
galore_status galore_two_sided_workspace_bytes(const galore_hparams* hp, const galore_tensor* W, size_t* out_bytes);

/* One step: R = P^T G Q, Adam on R with bias correction for step k = t + 1, weight update in the
 * epilogue of the last product (the m x n update is never stored).  With hp->auto_refresh and
 * t a multiple of hp->update_gap, the projectors are first recomputed from this G (the refresh test
 * of Algorithm 2).  Uses hp->scale, beta1, beta2, eps, weight_decay. */
galore_status galore_two_sided_step(const galore_hparams* hp, const galore_tensor* W, const galore_tensor* G,
                                    const galore_two_sided_state* S, int64_t t, float lr,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* Both projectors from G (SVD equation of Sec. 3.3).  The projector of the short side is the one
 * galore_refresh_subspace computes (canonical signs); each vector of the other side is the one the
 * decomposition pairs with it, v_i = G^T u_i / s_i (u_i = G v_i / s_i), formed as a unit-length row
 * of P^T G (column of G Q).  Uses hp->rank, refresh_iters, seed.  M, V are not touched. */
galore_status galore_two_sided_refresh(const galore_hparams* hp, const galore_tensor* G,
                                       const galore_two_sided_state* S,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- GaLore with Adafactor (Sec. 4.3, Sec. 5: Adafactor with first-order statistics) ----
 * The paper applies the projection to Adafactor as it does to Adam and prints no equations for it; the update
 * used here is the published Adafactor update for a matrix (factored second moment, update clipping, decay rate
 * 1 - k^-0.8, momentum) on the projected gradient R (r x cols for rows <= cols, rows x r otherwise), with the
 * learning rate left to the caller as in Algorithm 2 (no relative step size, no parameter scaling), k = t + 1:
 *     b2 = 1 - k^-0.8
 *     row_i <- b2 row_i + (1 - b2) sum_j (R_ij^2 + 1e-30) ;  col_j <- b2 col_j + (1 - b2) sum_i (R_ij^2 + 1e-30)
 *     Vhat_ij = row_i col_j / sum_i row_i ;  U = R / sqrt(Vhat) ;  Uhat = U / max(1, RMS(U))
 *     M <- beta1 M + (1 - beta1) Uhat ;  N = M
 *     W <- (1 - lr*weight_decay) W - lr*scale * P N   (N Q^T for rows > cols)
 * State per tensor: min(rows, cols) r + max(rows, cols) r + r + max(rows, cols) elements, against the
 * min r + 2 max r of Adam.  One tensor per call, no context: the caller keeps the step count t (0-based) and
 * clears m, row and col before the first step.  All tensors are BORROWED device memory, row-major; proj has W's
 * dtype; m, row, col are fp32 and dense.  The calls enqueue on hip_stream and return; errors as for the other
 * calls (galore_last_error(NULL)).  Uses hp->rank, scale, beta1, weight_decay, update_gap, auto_refresh,
 * refresh_iters, seed (beta2 and eps are Adam's and are not used).  Deterministic: every sum has a fixed order. */
typedef struct {
  galore_tensor proj;  /* P (rows x r) for rows <= cols, Q (cols x r) otherwise */
  galore_tensor m;     /* first moment of the clipped update: r x cols or rows x r, ld == its cols */
  galore_tensor row;   /* 1 x (rows of m): decayed row sums of R^2 */
  galore_tensor col;   /* 1 x (cols of m): decayed column sums of R^2 */
} galore_adafactor_state;

/* Bytes of device workspace (256-byte aligned) the step and the refresh below need for a weight of W's shape
 * and dtype; uses hp->rank. */
galore_status galore_adafactor_workspace_bytes(const galore_hparams* hp, const galore_tensor* W, size_t* out_bytes);

/* One step: R = P^T G (or G Q), the update above for step k = t + 1, weight update in the epilogue of the
 * back-projection (the rows x cols update is never stored).  With hp->auto_refresh and t a multiple of
 * hp->update_gap, the projector is first recomputed from this G (the refresh test of Algorithm 2). */
galore_status galore_adafactor_step(const galore_hparams* hp, const galore_tensor* W, const galore_tensor* G,
                                    const galore_adafactor_state* S, int64_t t, float lr,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/* The projector from G, exactly as galore_refresh_subspace computes it.  m, row, col are not touched. */
galore_status galore_adafactor_refresh(const galore_hparams* hp, const galore_tensor* G, const galore_adafactor_state* S,
                                       void* workspace, size_t workspace_bytes, void* hip_stream);

/* Stage call: the update block alone.  R fp32 (rows x cols, any ld); M fp32 dense, R's shape; row 1 x rows, col
 * 1 x cols, fp32; N fp32 or bf16, R's shape, dense; k >= 1 the 1-based step.  Updates M, row, col in place and
 * writes N.  workspace: 256-byte aligned, at least 4 * (ceil(cols / 256) * rows + ceil(rows / 32) * (cols +
 * ceil(cols / 256)) + 4) bytes of partial sums. */
galore_status galore_adafactor(const galore_tensor* R, const galore_tensor* M, const galore_tensor* row, const galore_tensor* col,
                               const galore_tensor* N, float beta1, int64_t k, void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- Instrumentation (measurement only, no part of the method) ----
 * Between galore_profile_start and galore_profile_stop every kernel group that galore_step or
 * galore_refresh_subspace enqueues is bracketed by a pair of HIP events on the context's
 * stream.  galore_profile_stop waits for the recorded work, then returns per stage the summed
 * device time in milliseconds and the number of bracketed launches (arrays of
 * GALORE_STAGE_COUNT entries, host memory).  A refresh counts as one launch per tensor group. */
typedef enum {
  GALORE_STAGE_PROJECT_LEFT = 0,   /* the grouped projection launch: R = P^T G, and R = G Q of the tensors that share it
                                      (bf16 tensors on the large-tile kernel: both orientations in one launch) */
  GALORE_STAGE_PROJECT_RIGHT = 1,  /* R = G Q of tensors on the general kernel (fp32, odd shapes) */
  GALORE_STAGE_ADAM = 2,           /* fused low-rank Adam (one launch per orientation) */
  GALORE_STAGE_BACK = 3,           /* W -= lr*alpha*(P N | N Q^T)  (GEMM + weight epilogue) */
  GALORE_STAGE_TRANSPOSE = 4,      /* proj -> proj_t */
  GALORE_STAGE_REFRESH = 5,        /* whole subspace refresh of a tensor group */
  GALORE_STAGE_COUNT = 6
} galore_stage;

galore_status galore_profile_start(galore_ctx* ctx);
galore_status galore_profile_stop(galore_ctx* ctx, double* ms, int64_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* GALORE_H */
