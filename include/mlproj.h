/*
 * mlproj -- bi-level and tri-level projection onto the l_{1,q} ball on one AMD
 * MI355X (gfx950), after Perez & Barlaud, "Multi-level projection with
 * exponential parallel speedup" (arXiv 2405.02086).
 *
 * For a matrix Y in R^{n x m} whose columns y_j are the groups, the bi-level
 * projection BP^{1,q}_eta (Sec. 3, Eq. 5-9, Alg. 1) is three steps:
 *   1. v_j = ||y_j||_q                       (column aggregate, Sec. 3)
 *   2. u   = P^1_eta(v)                      (Euclidean projection of v onto the
 *                                             l1 ball of radius eta, Eq. 6-7)
 *   3. x_j = P^q_{u_j}(y_j) for every j      (per-column projection, Eq. 8-9)
 *
 * GENERAL CONVENTIONS (all entry points)
 *  - Pure C ABI.  Every pointer named "device" is GPU global memory of the
 *    current HIP device; `stream` is a hipStream_t passed as void* (NULL = the
 *    default stream).  Calls only enqueue work on `stream` and return; they never
 *    synchronise, never copy to the host and never allocate or free memory.
 *  - Matrices are dense row-major fp32 (the *_stored entry points also take
 *    bf16 and fp16): element (i, j) of an n x m matrix is Y[i*m + j].  Tensors
 *    are dense C-order, of the same element types.
 *  - The caller owns every buffer.  X may alias Y exactly (in-place); any other
 *    overlap between buffers is undefined.  Y must hold finite values.
 *  - `workspace`: device scratch of at least mlproj_workspace_bytes(...) bytes,
 *    256-byte aligned.  Its contents on entry do not matter (no clearing is
 *    needed, ever).  One workspace serves one call at a time: two calls that may
 *    overlap on the GPU (different streams) need two workspaces.  A workspace
 *    sized for one shape serves any call whose own requirement is not larger.
 *  - After a call has completed on the stream, the first bytes of the workspace
 *    hold a mlproj_result record (threshold tau, norm, active count, ...).
 *  - v_out / u_out: optional device arrays (NULL to skip) that receive the
 *    aggregate v and the radii u, rounded to fp32.
 *  - Return value: MLPROJ_OK or a negative mlproj_status.  All argument checks
 *    run on the host before anything is enqueued; on error nothing was enqueued.
 *  - eta >= 0 (Sec. 4.1).  eta = 0 gives X = 0.  ||Y||_{1,q} <= eta gives X = Y
 *    bit for bit.  A group is kept iff v_j > tau.
 */
#ifndef MLPROJ_H
#define MLPROJ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum mlproj_status {
  MLPROJ_OK = 0,
  MLPROJ_ERR_NULL_POINTER = -1,   /* a required pointer is NULL                       */
  MLPROJ_ERR_BAD_DIMENSION = -2,  /* a dimension is <= 0                              */
  MLPROJ_ERR_TOO_LARGE = -3,      /* element count or a dimension exceeds the limits  */
  MLPROJ_ERR_BAD_RADIUS = -4,     /* eta is negative, NaN or infinite                 */
  MLPROJ_ERR_WORKSPACE = -5,      /* workspace too small or misaligned                */
  MLPROJ_ERR_BAD_VARIANT = -6,    /* unknown variant / norm selector                  */
  MLPROJ_ERR_ALIGNMENT = -7,      /* Y or X not aligned to the element size            */
  MLPROJ_ERR_LAUNCH = -8,         /* the HIP runtime refused a kernel launch of this call  */
  MLPROJ_ERR_NO_ALLOC_LIMIT = -9  /* bilevel_proj_l1inf_no_alloc: the input needs more scratch than the built-in buffer */
} mlproj_status;

/* Which projection a workspace is sized for. */
typedef enum mlproj_variant {
  MLPROJ_L1INF = 0,     /* bilevel_proj_l1inf,      dims (n, m, 1)     */
  MLPROJ_L11 = 1,       /* bilevel_proj_l11,        dims (n, m, 1)     */
  MLPROJ_L12 = 2,       /* bilevel_proj_l12,        dims (n, m, 1)     */
  MLPROJ_L1INFINF = 3   /* trilevel_proj_l1infinf,  dims (d0, d1, d2)  */
} mlproj_variant;

/* Inner norms of the multi-level projection. */
typedef enum mlproj_norm {
  MLPROJ_NORM_INF = 0,
  MLPROJ_NORM_L1 = 1,
  MLPROJ_NORM_L2 = 2
} mlproj_norm;

/* Outer norm p of the generic BP^{p,q} / MP^nu entry points. */
typedef enum mlproj_outer {
  MLPROJ_OUTER_L1 = 0,
  MLPROJ_OUTER_L2 = 1,
  MLPROJ_OUTER_LINF = 2
} mlproj_outer;

/* Element type of Y and X in bilevel_proj_stored.  The 16-bit formats are storage only: each
 * element is widened exactly to fp32 on load, all arithmetic is the fp32 / fp64 of the fp32
 * entry points, and X is rounded to nearest (ties to even) on store.                       */
typedef enum mlproj_storage {
  MLPROJ_STORE_F32 = 0,
  MLPROJ_STORE_BF16 = 1,  /* upper half of IEEE binary32: 8 exponent, 7 fraction bits */
  MLPROJ_STORE_F16 = 2    /* IEEE binary16 */
} mlproj_storage;

/* Record left at offset 0 of the workspace by every projection / norm call.
 * The outer projection acts on every aggregate as u_j = min(cap, scale * max(v_j - tau, 0));
 * with a weighted l1 ball as outer norm (the *_weighted entry points) as
 * u_j = scale * max(v_j - tau w_j, 0), where norm = sum_j w_j v_j and scale is 1, or 0 with eta = 0. */
typedef struct mlproj_result {
  double tau;            /* p = 1: threshold of u = P^1_eta(v); 0 inside the ball and for p = 2, inf */
  double norm;           /* ||Y||_{p,q} of the input (fp64); mlproj_norm_l1q: sum_j v_j              */
  double vmax;           /* max_j v_j                                                                 */
  double scale;          /* p = 2: eta / ||v||_2 when outside the ball; 1 otherwise                   */
  double cap;            /* p = inf: eta when outside the ball; +inf otherwise                        */
  uint32_t n_active;     /* number of groups with u_j > 0                                             */
  uint32_t inside_ball;  /* 1 when ||Y||_{1,q} <= eta (X = Y)                                         */
  uint32_t search_iters; /* fixed-point iterations the search for tau took                            */
  uint32_t inner_sweeps; /* l1,1 only: lock-step passes over Y the per-column threshold searches took */
  uint32_t inner_pending;/* l1,1 only: columns whose inner search had not converged; always 0, since  */
                         /* the finishing pass closes every column exactly                           */
  uint32_t inner_finished;/* l1,1 only: columns the lock-step passes left to the column-wise pass (all */
                         /* kept columns when a call runs no lock-step pass at all)                   */
  uint32_t reserved[2];
} mlproj_result;

/* Library version: a number that grows with every change of the kernels. */
int mlproj_version(void);

/* Static, human-readable text for a status code. */
const char* mlproj_status_string(int status);

/* Per-kernel timing aid.  Between mlproj_trace_begin and mlproj_trace_end, every projection
 * or norm call made by the calling thread records one of the caller's HIP events
 * (events[0], events[1], ... each a hipEvent_t created by the caller) on its stream before
 * each kernel it launches and one after the last kernel; recording stops silently when
 * `capacity` events are used.  mlproj_trace_end closes the trace and returns how many events
 * were recorded.  Off by default; adds nothing to calls made outside a trace.              */
int mlproj_trace_begin(void** events /* host array of hipEvent_t */, int capacity);
int mlproj_trace_end(void);

/* TEST AND TUNING HOOKS -- not part of the projection interface.  The two setters below change a
 * process-wide value (an atomic, read once when a call is enqueued; calls already enqueued keep
 * what they read).  Neither changes any result: both only move time around.  A caller that never
 * calls them gets the defaults, and the projection entry points themselves keep no state.
 *
 * mlproj_set_l11_sweeps -- MLPROJ_L11 (Alg. 3): how many lock-step passes over Y a call enqueues
 * for the per-column threshold searches before the column-wise finishing pass closes whatever is
 * still open.  1..16, or 0 for the default, which grows with the number of rows (none up to 1024
 * rows, or up to 4096 rows when the matrix has at most 4M elements; else 3 at 4096, 6 at 16384,
 * 12 beyond 131072): the finishing pass costs more per column the taller the matrix.  With the
 * default, a matrix of at most 4096 rows and 64M elements (32M in 16-bit storage) whose rows are
 * 16-byte aligned is not swept at all: one kernel keeps 16 whole columns per workgroup in
 * registers (a stripe whose columns are all dropped is zeroed with most of it unread), finds their
 * thresholds there and maps from the same registers (fp32: also up to 8192 rows, 8 columns per
 * workgroup, while there are no more such stripes than compute units); any forced value keeps
 * the sweeps.  The
 * thresholds are exact for any value.  Returns the previous value, or MLPROJ_ERR_BAD_DIMENSION
 * for a value outside 0..16.                                                                */
int mlproj_set_l11_sweeps(int sweeps);

/* mlproj_stripe_of_workgroup -- the column-stripe kernels of MLPROJ_L11 (16 or 8 whole columns per
 * workgroup: the one-pass kernel for short matrices and the finishing pass) deal their stripes so
 * that runs of 4 neighbouring stripes, which share cache lines of Y, run on one of the chip's 8
 * XCDs (workgroup b goes to XCD b mod 8): returns the stripe that workgroup `workgroup` of
 * `stripes` takes, a permutation of 0 .. stripes-1; -1 for arguments out of range.  Host only,
 * touches no GPU: here so that the permutation can be checked without one.                    */
int mlproj_stripe_of_workgroup(long long workgroup, long long stripes);

/* mlproj_set_search_spin_limit -- vectors of more than 32768 groups are searched (Eq. 6-7) by up
 * to 64 workgroups that exchange their sums every round, which needs all of them running at
 * once.  On an idle GPU they are; on a GPU that other streams keep full some may have to wait
 * for a free compute unit.  So the exchange is bounded: a workgroup that has polled `polls`
 * times for another's numbers gives up, everybody leaves, and a one-workgroup kernel enqueued
 * behind does the search instead -- every kernel ends either way and the result is the same.
 * What a caller on a shared GPU sees is a call that takes a fraction of a millisecond longer
 * (the default, 256 polls of 1-2 us each, plus the one-workgroup search), never a stall.
 * 0 makes the several-workgroup search give up at once (which is how the tests exercise the
 * kernel behind it).  The same number, capped at 64, is the patience of the one-pass tri-level
 * kernel (see trilevel_proj_l1infinf): with 0 its workgroups never wait for one another.
 * Returns the previous value, or MLPROJ_ERR_BAD_DIMENSION for a value outside 0..4194304.    */
int mlproj_set_search_spin_limit(int polls);

/* Bytes of workspace a call of `variant` on dims (d0, d1, d2) needs; bi-level
 * variants take d0 = n, d1 = m, d2 = 1.  Host-only, touches no GPU.  The size is a few
 * MiB plus 8-16 bytes per column; MLPROJ_L11 adds up to about 1 KiB per column for the
 * lists of its per-column threshold searches and a few MiB for the partial results of its
 * aggregate pass.                                                                */
int mlproj_workspace_bytes(int variant, long long d0, long long d1, long long d2,
                           size_t* bytes_out /* host */);

/* ||Y||_{1,q} = sum_j ||y_j||_q (Sec. 2, Eq. 1-2 with p = 1; Eq. 10 for q = inf).
 * q_variant is MLPROJ_L1INF, MLPROJ_L11 or MLPROJ_L12.  The fp64 norm is written to
 * norm_out[0] (device) and to the workspace record; v_out optionally gets v.      */
int mlproj_norm_l1q(const float* Y /* device, n*m */, long long n, long long m, int q_variant,
                    void* workspace /* device */, size_t workspace_bytes,
                    double* norm_out /* device, 1; may be NULL */,
                    float* v_out /* device, m; may be NULL */, void* stream);

/* BP^{1,inf}_eta (Sec. 4.1, Eq. 13, Alg. 2): v_j = max_i |Y_ij| (exact), u = P^1_eta(v),
 * X_ij = sign(Y_ij) * min(|Y_ij|, u_j).                                                */
int bilevel_proj_l1inf(const float* Y /* device, n*m */, float* X /* device, n*m */,
                       long long n, long long m, float eta,
                       void* workspace /* device */, size_t workspace_bytes,
                       float* v_out /* device, m; may be NULL */,
                       float* u_out /* device, m; may be NULL */, void* stream);

/* bilevel_proj_l1inf for callers that cannot allocate device memory and so cannot bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The same kernels and the same results as bilevel_proj_l1inf, bit for bit, with the workspace
 * taken from a fixed buffer of MLPROJ_NO_ALLOC_SCRATCH_BYTES inside the library's device image
 * (each GPU the library is used on holds that buffer until the process ends).  The call itself
 * allocates and frees nothing, on the host or on the device; the first call on a device looks
 * the buffer's address up once.
 *  - Limit: inputs whose workspace (mlproj_workspace_bytes(MLPROJ_L1INF, n, m, 1): about
 *    16 bytes per column plus at most 1 MiB) exceeds the buffer are refused with
 *    MLPROJ_ERR_NO_ALLOC_LIMIT before anything is enqueued.  Every matrix of up to 262144
 *    columns fits, whatever its number of rows.
 *  - The device that `stream` belongs to must be the current device of the calling thread.
 *  - All calls on one GPU share the one buffer: calls that may overlap on the GPU (different
 *    streams, or graphs replayed side by side) race on it.  Order them, or use
 *    bilevel_proj_l1inf with a workspace each.  Nothing in the buffer has to be cleared between
 *    calls; the result record of the last call is not exposed.
 *  - Y, X, v_out, u_out, eta and the other error codes: as bilevel_proj_l1inf.               */
#define MLPROJ_NO_ALLOC_SCRATCH_BYTES (6u << 20)
int bilevel_proj_l1inf_no_alloc(const float* Y /* device, n*m */, float* X /* device, n*m */,
                                long long n, long long m, float eta,
                                float* v_out /* device, m; may be NULL */,
                                float* u_out /* device, m; may be NULL */, void* stream);

/* BP^{1,1}_eta (Sec. 4.3.1, Eq. 14, Alg. 3): v_j = sum_i |Y_ij|, u = P^1_eta(v),
 * x_j = P^1_{u_j}(y_j), i.e. X_ij = sign(Y_ij) * max(|Y_ij| - tau_j, 0) with the
 * per-column threshold tau_j that makes ||x_j||_1 = u_j.                          */
int bilevel_proj_l11(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes,
                     float* v_out, float* u_out, void* stream);

/* BP^{1,2}_eta (Sec. 4.3.2, Eq. 15, Alg. 4): v_j = ||y_j||_2, u = P^1_eta(v),
 * x_j = y_j * u_j / v_j (x_j = 0 when v_j = 0).                                   */
int bilevel_proj_l12(const float* Y, float* X, long long n, long long m, float eta,
                     void* workspace, size_t workspace_bytes,
                     float* v_out, float* u_out, void* stream);

/* BP^{p,q}_eta for a general outer norm (Alg. 1; Sec. 3 names the l1, l2 and l_inf balls as
 * outer projections with known linear-time algorithms): v_j = ||y_j||_q with q given by
 * `variant` (MLPROJ_L1INF, MLPROJ_L11, MLPROJ_L12), u = P^p_eta(v) with p = outer_norm
 * (a mlproj_outer: soft threshold, rescale by eta/||v||_2, or cap at eta), x_j = P^q_{u_j}(y_j).
 * outer_norm = MLPROJ_OUTER_L1 is exactly bilevel_proj_l1inf / _l11 / _l12.                   */
int bilevel_proj_pq(int outer_norm, int variant, const float* Y /* device, n*m */,
                    float* X /* device, n*m */, long long n, long long m, float eta,
                    void* workspace /* device */, size_t workspace_bytes,
                    float* v_out /* device, m; may be NULL */,
                    float* u_out /* device, m; may be NULL */, void* stream);

/* bilevel_proj_pq on a matrix stored in fp32, bf16 or fp16 (a mlproj_storage), for training
 * loops that keep weights in 16 bits and prune by column (the use Sec. 6.3 makes of the
 * projection): Alg. 1 unchanged, computed on the widened values; only X is rounded to the
 * storage format.  v_out and u_out stay fp32.  mask_out[j] = 1 when column j is kept
 * (u_j > 0, decided in fp64) and 0 when the projection zeroes it.  Y and X must be aligned to
 * the element size; the 16-byte accesses need 16-byte aligned pointers and m a multiple of
 * 16 / element size, other inputs take an element-wise path.  X may alias Y.  The workspace
 * size is mlproj_workspace_bytes(variant, n, m, 1) for every storage type.                  */
int bilevel_proj_stored(int storage, int outer_norm, int variant,
                        const void* Y /* device, n*m elements */, void* X /* device, n*m elements */,
                        long long n, long long m, float eta,
                        void* workspace /* device */, size_t workspace_bytes,
                        float* v_out /* device, m; may be NULL */,
                        float* u_out /* device, m; may be NULL */,
                        unsigned char* mask_out /* device, m; may be NULL */, void* stream);

/* BP^{p,q}_eta with the weighted l1 ball as outer norm, p = l_w1 (Sec. 3 lists it beside l1, l2
 * and l_inf as an outer projection with a linear-time algorithm): v_j = ||y_j||_q as in
 * bilevel_proj_stored, u = the Euclidean projection of v onto {u : sum_j w_j |u_j| <= eta}, that
 * is u_j = max(v_j - tau w_j, 0) with tau = 0 when sum_j w_j v_j <= eta and otherwise the root of
 * sum_j w_j max(v_j - tau w_j, 0) = eta; then x_j = P^q_{u_j}(y_j) (Eq. 8-9).  A larger w_j makes
 * column j dearer to keep.  weights: m floats in device memory, read only, every one positive
 * and finite (not checked: the call still ends with other values, with an unspecified result).
 * The result record holds tau, norm = sum_j w_j v_j, vmax = max v_j, n_active = #{u_j > 0}; with
 * eta = 0, tau = max_j v_j / w_j and X = 0.  All other arguments, the workspace size, alignment
 * rules and error codes are those of bilevel_proj_stored; a NULL weights pointer is
 * MLPROJ_ERR_NULL_POINTER.  With all weights 1 the result equals the plain l1 outer norm's to
 * rounding (the threshold search sums in another order).                                    */
int bilevel_proj_weighted(int storage, int variant,
                          const void* Y /* device, n*m elements */, void* X /* device, n*m elements */,
                          long long n, long long m, float eta,
                          const float* weights /* device, m */,
                          void* workspace /* device */, size_t workspace_bytes,
                          float* v_out /* device, m; may be NULL */,
                          float* u_out /* device, m; may be NULL */,
                          unsigned char* mask_out /* device, m; may be NULL */, void* stream);

/* MP^nu_eta (Sec. 5.2, Def. 5.2, Alg. 6) with the weighted l1 ball as outermost norm: the
 * multi-level projection of multilevel_proj_stored, except that the top aggregate w (one entry
 * per group of axis 0) is projected onto {u : sum_a weights[a] |u_a| <= eta} as in
 * bilevel_proj_weighted (Sec. 3): u_a = max(w_a - tau weights[a], 0).  weights: dims[0] floats in
 * device memory, read only, positive and finite (not checked).  Covers the tri-level l1,inf,inf
 * projection as norms = {INF, INF}.  All other arguments, the workspace size
 * (mlproj_multilevel_workspace_bytes), alignment rules and error codes are those of
 * multilevel_proj_stored; a NULL weights pointer is MLPROJ_ERR_NULL_POINTER.               */
int multilevel_proj_weighted(int storage, const void* Y /* device */, void* X /* device */, int ndim,
                             const long long* dims /* host, ndim */, const int* norms /* host, ndim-1, innermost first */,
                             float eta, const float* weights /* device, dims[0] */,
                             void* workspace /* device */, size_t workspace_bytes,
                             float* v_out /* device, dims[0]; may be NULL */,
                             float* u_out /* device, dims[0]; may be NULL */, void* stream);

/* One problem of a batch: the arguments of bilevel_proj_stored for one matrix. */
typedef struct mlproj_problem {
  const void* Y;              /* device, n*m elements                               */
  void* X;                    /* device, n*m elements; may alias Y                  */
  long long n, m;
  float eta;
  void* workspace;            /* device; its own for every problem of the batch     */
  size_t workspace_bytes;     /* at least mlproj_workspace_bytes(variant, n, m, 1)  */
  float* v_out;               /* device, m; may be NULL                             */
  float* u_out;               /* device, m; may be NULL                             */
  unsigned char* mask_out;    /* device, m; may be NULL                             */
} mlproj_problem;

/* `count` independent bi-level projections that share storage type, outer norm and variant
 * (the weight matrices a training loop projects after a step, Sec. 6.3), with the results of
 * `count` calls of bilevel_proj_stored, bit for bit.  Matrices of at most 16384 columns share
 * their kernel launches, 16 matrices at a time (three launches for all of them instead of
 * three each, which is what small matrices cost; MLPROJ_L11 shares the launches of its
 * per-column searches the same way; MLPROJ_L1INF and MLPROJ_L12 matrices of at most 128 KiB
 * take a single launch for all of them, in place or not); wider ones are enqueued one after
 * another behind them.
 * `problems` is a host array, read before
 * the call returns; all of it is checked before anything is enqueued.  Outputs of different
 * problems must not overlap.                                                                 */
int bilevel_proj_batch(int storage, int outer_norm, int variant, int count,
                       const mlproj_problem* problems /* host */, void* stream);

/* The two halves of a bi-level call, for callers that want the radii before (or without)
 * writing X.  bilevel_radii computes the aggregate v and u = P^1_eta(v) of Alg. 1 (for
 * MLPROJ_L11 also the per-column thresholds Alg. 3 needs) and leaves the outcome in the
 * workspace; bilevel_apply then maps the columns, x_j = P^q_{u_j}(y_j), from that workspace,
 * on the same Y, n, m and variant.  bilevel_proj_* is exactly bilevel_radii then bilevel_apply. */
int bilevel_radii(int variant, const float* Y /* device, n*m */, long long n, long long m, float eta,
                  void* workspace /* device */, size_t workspace_bytes,
                  float* v_out /* device, m; may be NULL */, void* stream);
int bilevel_apply(int variant, const float* Y /* device, n*m */, float* X /* device, n*m */,
                  long long n, long long m, void* workspace /* device */, size_t workspace_bytes,
                  float* u_out /* device, m; may be NULL */, void* stream);

/* TP^{1,inf,inf}_eta (Sec. 5.1, Def. 5.1, Alg. 5; iterative form in the appendix) on a
 * C-order tensor Y[a][b][c] of shape (d0, d1, d2).  Groups live on axis 0: the inner
 * aggregate is V_ab = max_c |Y_abc|, the outer one w_a = max_b V_ab, u = P^1_eta(w), and
 * each fibre Y_ab. is clipped to min(V_ab, u_a) -- which equals clipping it to u_a.
 * (The paper indexes its tensor (c, n, m) and keeps groups on the last axis; that is this
 * function applied to the transposed tensor, or bilevel_proj_l1inf on the (c*n) x m
 * reshape.)  v_out / u_out have d0 entries (w and u).
 * A tensor of at most 256 slabs (d0) and 64 MiB whose slabs are 16-byte aligned is projected in
 * one pass over memory: every workgroup keeps its share of Y in registers between the aggregate
 * and the clip, and the workgroups exchange their maxima inside the kernel.  That is fastest when
 * all of them run at once, as they do on an otherwise idle GPU; on a GPU that other streams keep
 * full a workgroup that has waited (at most 64 polls, about 0.1 ms) computes the missing maxima
 * itself, so the call gets slower but never stalls, and the result is the same.  Other tensors
 * take a chain of three kernels.                                                      */
int trilevel_proj_l1infinf(const float* Y /* device, d0*d1*d2 */, float* X /* device, same */,
                           long long d0, long long d1, long long d2, float eta,
                           void* workspace, size_t workspace_bytes,
                           float* v_out /* device, d0; may be NULL */,
                           float* u_out /* device, d0; may be NULL */, void* stream);

/* trilevel_proj_l1infinf on a tensor stored in fp32, bf16 or fp16 (a mlproj_storage, as in
 * bilevel_proj_stored: the 16-bit formats are storage only and X is rounded to nearest-even),
 * with an optional mask of the kept slabs: mask_out[a] = 1 when u_a > 0.                      */
int trilevel_proj_stored(int storage, const void* Y /* device, d0*d1*d2 elements */,
                         void* X /* device, d0*d1*d2 elements */,
                         long long d0, long long d1, long long d2, float eta,
                         void* workspace /* device */, size_t workspace_bytes,
                         float* v_out /* device, d0; may be NULL */,
                         float* u_out /* device, d0; may be NULL */,
                         unsigned char* mask_out /* device, d0; may be NULL */, void* stream);

/* MP^nu_eta (Sec. 5.2, Def. 5.2, Alg. 6; iterative form in the appendix) on a C-order tensor of
 * shape dims[0..ndim-1] (2 <= ndim <= 8) with single-axis inner norms and the l1 norm outside.
 * Groups live on axis 0.  norms[0] aggregates the last axis, norms[1] the one before, ... ,
 * norms[ndim-2] aggregates axis 1 (each MLPROJ_NORM_INF, _L1 or _L2); the resulting length-dims[0]
 * vector is projected onto the l1 ball of radius eta, and on the way back every fibre of every
 * level is projected onto the ball (of that level's norm) whose radius is the matching entry of
 * the level above.  In the paper's notation, which keeps the groups on the last axis and
 * aggregates the first axes first, this is nu = ((norms[0]), ..., (norms[ndim-2]), (1)) on the
 * tensor with its axes reversed: ndim = 3 with two MLPROJ_NORM_INF is the tri-level
 * l1,inf,inf, three MLPROJ_NORM_L1 levels give the l1,1,1 of Sec. 6.1, ndim = 2 is the bi-level
 * projection of the transposed matrix.  dims and norms are host arrays; v_out / u_out have
 * dims[0] entries.  The workspace comes from mlproj_multilevel_workspace_bytes.            */
int mlproj_multilevel_workspace_bytes(int ndim, const long long* dims /* host */,
                                      size_t* bytes_out /* host */);
int multilevel_proj(const float* Y /* device */, float* X /* device, same size */, int ndim,
                    const long long* dims /* host, ndim */, const int* norms /* host, ndim-1 */,
                    float eta, void* workspace /* device */, size_t workspace_bytes,
                    float* v_out /* device, dims[0]; may be NULL */,
                    float* u_out /* device, dims[0]; may be NULL */, void* stream);

/* multilevel_proj with the outermost norm p = outer_norm (a mlproj_outer) instead of l1. */
int multilevel_proj_p(int outer_norm, const float* Y, float* X, int ndim, const long long* dims,
                      const int* norms, float eta, void* workspace, size_t workspace_bytes,
                      float* v_out, float* u_out, void* stream);

/* multilevel_proj_p on a tensor stored in fp32, bf16 or fp16 (a mlproj_storage, as in
 * bilevel_proj_stored: the 16-bit formats are storage only; every level above the tensor is
 * kept in fp64 and X is rounded to nearest-even once, on store).  Y and X must be aligned to
 * the element size; 16-byte aligned pointers and a last axis that is a multiple of 16 bytes
 * take the wide path.                                                                      */
int multilevel_proj_stored(int storage, int outer_norm, const void* Y /* device */,
                           void* X /* device, same size and type */, int ndim,
                           const long long* dims /* host, ndim */,
                           const int* norms /* host, ndim-1 */, float eta,
                           void* workspace /* device */, size_t workspace_bytes,
                           float* v_out /* device, dims[0]; may be NULL */,
                           float* u_out /* device, dims[0]; may be NULL */, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* MLPROJ_H */
