/*
 * lordo.h -- C ABI of the MI355X (gfx950) LoRDO per-matrix optimizer library.
 *
 * The library runs, for a set of weight matrices W_i in R^{p_i x q_i}, the hot path of
 * LoRDO: the low-rank local step (Sec. 2 low-rank update; Alg. 1 inner loop), the
 * periodic subspace refresh with rotation of both moments (Sec. 2 "ComputeProjection";
 * Alg. 1 sync branch, rotation lines) and the infrequent outer step on the
 * pseudo-gradient (Alg. 1 sync branch; App. A.1-A.2; App. D.4-D.5).
 *
 * Conventions for every entry point
 *   - All matrices are dense, row-major and contiguous: element (a, b) of a p x q matrix
 *     is at index a*q + b.  Notation is the paper's: p rows, q columns, rank r,
 *     projection Q (p x r), low-rank gradient g = Q^T G (r x q), moments u, v (r x q).
 *   - "device" pointers are HIP device addresses; "host" pointers are ordinary host
 *     memory.  Arrays of pointers (`void* const*`) are HOST arrays of length n holding
 *     one DEVICE pointer per matrix, in the order of the shapes given to lordo_init.
 *   - The caller owns and allocates every buffer, including the arena the library keeps
 *     its state in; the library never allocates or frees device memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls only
 *     enqueue work on it and return; they do not synchronise, except lordo_init,
 *     lordo_poll_status and lordo_destroy.  All calls on one context must be issued
 *     on one stream, or be ordered by the caller.
 *   - Return value: LORDO_OK or a negative LORDO_E* code; lordo_strerror gives text.
 *     Argument and state errors are detected before anything is enqueued.  A numerical
 *     breakdown inside a kernel (non-positive Cholesky pivot) is latched in device
 *     memory and reported by lordo_poll_status as LORDO_ENUMERIC.  While it is latched,
 *     lordo_refresh_subspace*, lordo_init_projection leave the projection and the
 *     moments as they were (the refresh that broke down included): the optimizer goes
 *     on in the old subspace until the caller polls, which clears the latch.
 *   - Stream capture: the compute calls enqueue kernels only (no allocation, no memset, no
 *     host synchronisation), so they can be recorded into a HIP graph.  The step count and
 *     the bias corrections 1 - beta^t derived from it live in device memory and are advanced
 *     by a kernel at the head of every local step, so a recorded lordo_local_step counts its
 *     REPLAYS: replaying it k times is k local steps (on whatever the gradient buffers hold
 *     at each replay).  The learning rate and the gradient scale travel as kernel arguments:
 *     a replay uses the values of the recording.  lordo_get_step returns the number of
 *     local steps ISSUED through the API (recording counts once, replays do not); after
 *     replays, tell the context with lordo_set_step before a call that depends on it on the
 *     host (a refresh skips the moment rotation while that count is 0).  lordo_set_step
 *     takes effect at the head of the next compute call: do not record that call.  The first
 *     launch of a kernel raises its shared-memory limit with a host-side runtime call, which
 *     a capturing stream does not allow: issue a call once before recording it.
 *   - A context belongs to the GPU that was current at lordo_init (the arena and the matrices live there): every call
 *     that enqueues work on it must be made with that GPU current, and returns LORDO_ESTATE otherwise.
 *   - There is no CPU fallback: without a GPU every compute call returns LORDO_EHIP.
 */
#ifndef LORDO_H
#define LORDO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LORDO_OK        0
#define LORDO_EINVAL   (-1)   /* null pointer, bad shape, r > p, unknown dtype, unsupported option */
#define LORDO_ENOMEM   (-2)   /* arena smaller than lordo_workspace_bytes                           */
#define LORDO_EHIP     (-3)   /* HIP runtime error (message on stderr)                               */
#define LORDO_ESTATE   (-4)   /* call not valid in the current state                                 */
#define LORDO_ENUMERIC (-5)   /* numerical breakdown latched by a kernel                             */

#define LORDO_F32  0
#define LORDO_BF16 1

/* selectors of lordo_get_state / lordo_set_state; shapes of the plain fp32 buffers exchanged */
#define LORDO_STATE_Q       0   /* p x r  projection                                   */
#define LORDO_STATE_U       1   /* r x q  first moment                                 */
#define LORDO_STATE_V       2   /* r x q  second moment                                */
#define LORDO_STATE_ANCHOR  3   /* p x q  x_{t-K_x}, the model at the last outer step  */
#define LORDO_STATE_MOM     4   /* p x q  outer momentum b (only if outer_momentum!=0) */
#define LORDO_STATE_GLOW    5   /* r x q  g of the last local step (read only; scratch of a refresh)         */
#define LORDO_STATE_NUPD    6   /* r x q  bracketed update N of the last local step (read only; scratch of a
                                          refresh and of lordo_outer_step_lowrank) */
#define LORDO_STATE_ERR     7   /* p x q  error-feedback residual E (only if error_feedback != 0) */
#define LORDO_STATE_UPLINK  8   /* r x q  up-link buffer A (only if uplink_buffer != 0)           */
#define LORDO_STATE_RITZ    9   /* r      Ritz values of the last refresh, descending: the singular values of the source
                                          restricted to span(Q) (read only; only if rayleigh_ritz != 0, after a refresh) */

typedef struct lordo_ctx lordo_ctx;

/* One weight matrix: rows p, cols q, rank r; requires r <= 4096, p, q <= 2^20, max(p, q) * r < 2^29 and
 * max((p + 256) * q, p * (q + 256)) < 2^30: a matrix is addressed with 32-bit byte offsets, so the fp32 array and one
 * tile beyond it stay below 4 GiB.  A matrix for which that product reaches 2^29 (2 GiB in fp32) must have p and q
 * multiples of 256 and side 0: the kernels mask what lies outside a ragged matrix with offsets that are out of range
 * only below 2 GiB.  LORDO_EINVAL otherwise.
 *   side 0  projection on the left, as the paper writes it (Sec. 2: Q is p x r, the moments r x q); 1 <= r <= p.
 *   side 1  projection on the right, the choice that keeps Q and the moments small for a tall matrix (p > q):
 *           g = (s G) Q_R with Q_R q x r, moments p x r, W <- W - eta N Q_R^T, and the refresh takes the right
 *           singular subspace of its source.  This is Sec. 2 applied to the transpose of the matrix, and the library
 *           runs it as exactly that on the caller's row-major p x q arrays (W, G, Src, Delta keep their layout):
 *           every low-rank array of such a matrix is the one of the TRANSPOSED problem, i.e. Q is q x r, the r x q
 *           states (u, v, g, N) are r x p, Omega is p x r and the block of lordo_init_projection q x r.
 *           1 <= r <= q.  Every update case; in the "Full-Rank QHM" case the scale of the gradient term runs over the
 *           rows of W, s_i = mean over the rank of sqrt(v^_ik) + eps (the columns of the transposed problem).  With
 *           error feedback or full-rank QHM: columns a multiple of 4, 16-byte aligned W.  The products of a refresh
 *           with the source run in the library's generic grouped GEMM, also for the left-projected matrices of the
 *           same context. */
typedef struct {
  int64_t rows;
  int64_t cols;
  int32_t rank;
  int32_t side;
} lordo_shape;

/* Hyper-parameters (Alg. 1 "Require").  Scalars are double so that 1-beta and
 * 1-beta^t are formed from the same decimal values a float64 reference uses. */
typedef struct {
  double  beta1, beta2, eps;     /* moment decay rates; eps is added outside the root (Sec. 2)        */
  int32_t bias_correction;       /* 1: u/(1-beta1^t), v/(1-beta2^t) as in Sec. 2; 0: as Alg. 1 prints  */
  int32_t qhm_mode;              /* Alg. 1 update cases: 0 "No QHM", 1 "Low-Rank QHM", 2 "Full-Rank QHM" (Sec. 3.2) */
  double  omega;                 /* QHM mixing coefficient in [0, 1]; ignored when qhm_mode == 0        */
  int32_t error_feedback;        /* 1: keep the residual E and project G + E (Alg. 1 error-feedback lines) */
  int32_t outer_nesterov;        /* with outer_momentum != 0: 1 Nesterov, 0 heavy ball                  */
  double  outer_lr;              /* eta_s; 1.0 with outer_momentum 0 is plain averaging (Alg. 1)        */
  double  outer_momentum;        /* mu; 0 keeps no momentum buffer                                      */
  int32_t power_iters;           /* block power iterations of the range finder, 0..8                    */
  int32_t orth_passes;           /* orthonormalisation of the refresh: 2 (default if 0): one shifted CholeskyQR pass after
                                    every product of the power iteration, shifted + plain at the end -- for sources whose
                                    r leading singular values span less than about three orders of magnitude;
                                    3: the robust variant, shifted + shifted after every product and shifted, shifted,
                                    plain at the end (conditioning up to about 1e6; about 1.5 times the refresh time).
                                    Beyond these limits, and for a source of rank below r, a non-positive pivot is
                                    latched (LORDO_ENUMERIC) */
  int32_t grad_dtype;            /* LORDO_BF16 or LORDO_F32: element type of every G                    */
  int32_t uplink_buffer;         /* 1: keep the r x q up-link buffer A = sum over the window of eta_t N_t (App. A.5.1);
                                    not with qhm_mode 2, whose update has no low-rank form              */
  int32_t rayleigh_ritz;         /* 1: every refresh ends with a Rayleigh-Ritz step, so that the columns of Q are the
                                    approximate left singular vectors of the source, largest singular value first, as
                                    the SVD projection of Sec. 2 orders them (0: an unordered orthonormal basis of the
                                    same subspace).  Needs every rank <= 1024 (LORDO_EINVAL otherwise); sets of ranks up to 128 take a
                                    much faster solver                                                  */
  int32_t param_dtype;           /* element type of every W: LORDO_F32 (0, the default) or LORDO_BF16 -- bf16 STORAGE of the
                                    weights: every update is formed in fp32 from the stored value and rounded to nearest-even
                                    once when it is written back; the anchor and the outer momentum stay fp32 (the anchor
                                    holds the stored, i.e. rounded, model).  Every update case, with or without error
                                    feedback; not with uplink_buffer, whose fused outer step writes fp32 (LORDO_EINVAL) */
  int32_t err_dtype;             /* storage type of the error-feedback residual E: LORDO_F32 (0, the default) or LORDO_BF16.
                                    bf16: E <- rne(s G + E - Q g), formed in fp32 from the stored value and rounded once;
                                    LORDO_STATE_ERR is still read and written as fp32 (converted).  Needs error_feedback,
                                    bf16 gradients and no right-projected matrix; lordo_refresh_subspace_local (whose
                                    source s G + E is formed inside the residual buffer) then returns LORDO_EINVAL */
  int32_t reserved;              /* must be 0                                                           */
  uint64_t seed;                 /* seed of the library's own Gaussian generator, used where the caller passes no
                                    random block: lordo_init_projection(Block = NULL) (Alg. 1 "Require": random Q_0) and
                                    lordo_refresh_subspace*(Omega = NULL).  Counter-based (Philox-4x32-10 + Box-Muller):
                                    element e of the block of matrix i in the k-th such call of the context is a function
                                    of (seed, i, k, e) alone, so two contexts initialised alike draw the same blocks */
} lordo_hparams;

/* Bytes of arena lordo_init needs for these shapes and hyper-parameters (host call). */
int lordo_workspace_bytes(const lordo_shape* shapes, int32_t n, const lordo_hparams* hp, size_t* out_bytes);

/* Create a context (the north-star call "lordo_init": matrix shapes, rank, hyper-parameters).
 *   arena        device, caller-allocated, 256-byte aligned, >= lordo_workspace_bytes; the library
 *                keeps Q, u, v, the anchor, the outer momentum and all scratch in it until destroy.
 *   W            host array of n device pointers to p x q weights of hp.param_dtype; read once: anchor <- W.
 * State after init: Q = first r columns of the identity (Alg. 2 "Require"), u = v = 0,
 * b = 0, t = 0 (Alg. 1 "Require").  Synchronises `stream` before returning. */
int lordo_init(lordo_ctx** out, const lordo_shape* shapes, int32_t n, const lordo_hparams* hp,
               void* arena, size_t arena_bytes, void* const* W, void* stream);

/* lordo_init for callers that cannot allocate device memory at all (code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc): the same context, but its workspace -- projection, moments, anchor, momentum and
 * all scratch that lordo_init places in the caller's arena -- lives in a fixed array inside the library,
 * LORDO_STATIC_WORKSPACE_BYTES per GPU, held from the first such call on a GPU until the process ends.  No device
 * memory is allocated or freed, here or in any later call on the context.
 *   shapes, n, hp, W, stream   as for lordo_init.
 * Returns LORDO_ENOMEM (with the sizes on stderr) when lordo_workspace_bytes(shapes, n, hp) exceeds
 * LORDO_STATIC_WORKSPACE_BYTES, and LORDO_ESTATE while another context created by this call is alive on the current
 * GPU: every such context of a GPU uses the same array, so only one may exist at a time (lordo_destroy releases it);
 * the array keeps the previous context's contents, which this call overwrites or clears as lordo_init does with an
 * uninitialised arena.  Calls on the one live context follow the stream-ordering rule above; issued from two host
 * threads or two streams without ordering they race on the array like any two calls on one context.
 * Every other entry point takes the context as if it came from lordo_init. */
#define LORDO_STATIC_WORKSPACE_BYTES (64u << 20)
int lordo_init_static(lordo_ctx** out, const lordo_shape* shapes, int32_t n, const lordo_hparams* hp,
                      void* const* W, void* stream);

/* Random initial projection of the global variant (Alg. 1 "Require": Q_0 random, against the identity
 * columns of Alg. 2 that lordo_init leaves): Q_0 = orthonormal basis of the caller's block, by the same
 * CholeskyQR as the refresh (columns signed so that the triangular factor has a positive diagonal).
 *   Block  host array of n device pointers, p x r fp32 each (e.g. Gaussian), read only, full column rank;
 *          NULL: the library draws Gaussian blocks from hp.seed.
 * Valid only before the first local step (LORDO_ESTATE afterwards: changing the basis of running moments
 * is what lordo_refresh_subspace does). */
int lordo_init_projection(lordo_ctx* ctx, const void* const* Block, void* stream);

/* One local step on every matrix (Sec. 2; Alg. 1 inner loop):
 *   t <- t+1;  A = grad_scale * G  (+ E with error feedback);  g = Q^T A;  [E <- A - Q g];
 *   u <- beta1 u + (1-beta1) g;  v <- beta2 v + (1-beta2) g*g;  u^ = u/c1, v^ = v/c2, c_i = 1-beta_i^t
 *   (1 if bias_correction == 0);  den = sqrt(v^) + eps;
 *   qhm_mode 0:  N = u^ / den;                             W <- W - lr * Q N
 *   qhm_mode 1:  N = (omega u^ + (1-omega) g) / den;       W <- W - lr * Q N
 *   qhm_mode 2:  N = u^ / den;  s_j = mean_i den_ij;       W <- W - lr * ((1-omega) grad_scale G diag(1/s) + omega Q N)
 *   W   host array of n device pointers, p x q of hp.param_dtype, updated in place.
 *   G   host array of n device pointers, p x q of hp.grad_dtype, read only.
 *   grad_scale  scalar the caller's gradient clipping produced (1 = none).
 * qhm_mode 2 and error feedback need q % 4 == 0 for every matrix, W aligned to 16 bytes and G to
 * 8 bytes (bf16) or 16 bytes (fp32); otherwise LORDO_EINVAL and nothing is enqueued. */
int lordo_local_step(lordo_ctx* ctx, void* const* W, const void* const* G,
                     double lr, double grad_scale, void* stream);

/* New projection for every matrix and rotation of both moments into it
 * (Sec. 2 ComputeProjection, here a Gaussian-start block power iteration:
 *  Y = orth(Src Omega); power_iters x { Z = orth(Src^T Y); Y = orth(Src Z) }; Q_new = Y, columns
 *  signed so that the triangular factor has a positive diagonal; then, if t > 0, Alg. 1 rotation:
 *  R = Q_new^T Q;  u <- R u;  v <- c2 | (R o R)(v/c2 - (u/c1)^2) + (R u/c1)^2 |;  finally Q <- Q_new).
 *   Src        host array of n device pointers, p x q each, element type src_dtype
 *              (a gradient, or an averaged pseudo-gradient); read only.  A NULL entry leaves that matrix
 *              out: its Q, u, v (and its value in lordo_get_mssv) stay as they are.
 *   Omega      host array of n device pointers, q x r fp32 Gaussian start blocks, read only (entries of
 *              matrices that are left out may be NULL); NULL: the library draws the blocks from hp.seed.
 * The storage behind LORDO_STATE_GLOW and LORDO_STATE_NUPD serves as scratch: both hold the values of the
 * last local step only until the next refresh.  With hp.uplink_buffer the call returns LORDO_ESTATE while
 * the buffer is non-empty (see lordo_export_uplink). */
int lordo_refresh_subspace(lordo_ctx* ctx, const void* const* Src, int32_t src_dtype,
                           const void* const* Omega, void* stream);

/* Refresh of the local variant (Alg. 2): the projection is computed from this step's clipped
 * gradient plus the error buffer, Q_new = ComputeProjection(grad_scale * G + E), with the same
 * range finder and moment rotation as lordo_refresh_subspace.  Needs hp.error_feedback = 1.
 * The sum is formed in place: after this call the error buffer holds grad_scale * G + E, and the
 * NEXT call on this context must be lordo_local_step with the same G array (same pointers; its
 * grad_scale then only scales the full-rank QHM term), which takes g = Q^T (buffer) and leaves
 * E = buffer - Q g, exactly the step of Alg. 2 that follows the refresh.  Until then
 * lordo_refresh_subspace*, and get/set of LORDO_STATE_ERR, return LORDO_ESTATE; so does a local step
 * with other gradient pointers.
 *   G      host array of n device pointers, p x q of hp.grad_dtype, read only.
 *   Omega  host array of n device pointers, q x r fp32 Gaussian start blocks, read only; NULL: drawn from hp.seed. */
int lordo_refresh_subspace_local(lordo_ctx* ctx, const void* const* G, double grad_scale,
                                 const void* const* Omega, void* stream);

/* This worker's pseudo-gradient (App. A.1): DeltaOut_i <- anchor_i - W_i, fp32 p x q (W of hp.param_dtype). */
int lordo_export_pseudograd(lordo_ctx* ctx, const void* const* W, void* const* DeltaOut, void* stream);

/* Outer step (Alg. 1 OuterOpt; App. A.2): with D = AvgDelta_i (the cross-worker mean, fp32 p x q)
 * or, if AvgDelta == NULL, this worker's own anchor - W:
 *   mu == 0:  W <- anchor - eta_s D
 *   mu != 0:  b <- mu b + D;  W <- anchor - eta_s (D + mu b) (Nesterov) or anchor - eta_s b (heavy ball)
 * then anchor <- W.  W is written (and read only when AvgDelta == NULL).  With AvgDelta == NULL the call needs at
 * least one local step since the last outer step (LORDO_ESTATE otherwise: there is no pseudo-gradient yet). */
int lordo_outer_step(lordo_ctx* ctx, void* const* W, const void* const* AvgDelta, void* stream);

/* Up-link time buffer (App. A.5.1, "Worker Communication"; memory-overhead table): with
 * hp.uplink_buffer = 1 every local step also does A <- A + lr * N (r x q per matrix, N the bracketed
 * low-rank update of that step), so that between two outer steps anchor - W = Q A and only A has to
 * be sent.  The buffer is in coordinates of the current Q: lordo_refresh_subspace* return
 * LORDO_ESTATE while it is non-empty (local steps taken since the last outer step); both outer-step
 * calls clear it.
 * lordo_export_uplink: AccOut_i <- A_i, plain row-major fp32 r x q (host array of n device pointers).
 * lordo_outer_step_lowrank: the outer step of lordo_outer_step with Delta_i = Q_i AvgAcc_i, AvgAcc the
 *   cross-worker mean of the exported buffers (fp32 r x q each; NULL: the buffer as it lies in the
 *   workspace -- this worker's own, or the mean if the packed payload was averaged in place), formed
 *   tile by tile inside the update -- no p x q pseudo-gradient is materialised.  Every worker must hold
 *   the same Q (the global variant).  Overwrites the planes behind LORDO_STATE_NUPD.
 * Both return LORDO_ESTATE without hp.uplink_buffer. */
int lordo_export_uplink(lordo_ctx* ctx, void* const* AccOut, void* stream);
int lordo_outer_step_lowrank(lordo_ctx* ctx, void* const* W, const void* const* AvgAcc, void* stream);

/* Packed synchronisation payload (Alg. 1, synchronisation of the optimizer states; App. A.5.1, "Worker
 * Communication"): everything a worker sends at a synchronisation -- first moments, second moments and,
 * with hp.uplink_buffer, the up-link buffers, of ALL matrices -- lies in one contiguous fp32 region of the
 * workspace, [u | v | A], so that a single in-place all-reduce(mean) over it replaces one collective per
 * matrix and tensor and no copy into a send buffer is needed.  The order of the elements inside the
 * region is internal (operand layout with zero padding) but depends on (shapes, hparams) alone: element k
 * means the same on every worker that was initialised alike, and padding is zero everywhere, so an
 * elementwise mean of the regions is the mean of every tensor.
 *   *dev_ptr        device pointer into the workspace (owned by the context, valid until lordo_destroy)
 *   *count          fp32 elements in the region
 *   *moments_count  (may be NULL) elements of the leading [u | v] part; the rest is A
 * The caller reads and writes the region on the stream it passes to the neighbouring library calls.  After
 * averaging it in place, lordo_outer_step_lowrank(ctx, W, NULL, stream) consumes the averaged A where it
 * lies.  Per-tensor access in plain row-major layout stays with lordo_get_state / lordo_set_state. */
int lordo_sync_payload(lordo_ctx* ctx, void** dev_ptr, size_t* count, size_t* moments_count);

/* Copy one state tensor of matrix `mat` to / from a plain row-major fp32 device buffer of the
 * shape listed at the selector.  set_state(Q) expects orthonormal columns and rebuilds the packed
 * operand copies; GLOW and NUPD cannot be set. */
int lordo_get_state(lordo_ctx* ctx, int32_t mat, int32_t which, void* dev_dst, void* stream);
int lordo_set_state(lordo_ctx* ctx, int32_t mat, int32_t which, const void* dev_src, void* stream);

/* Count t of local steps taken (drives the bias correction); host values. */
int lordo_get_step(lordo_ctx* ctx, int64_t* t);
int lordo_set_step(lordo_ctx* ctx, int64_t t);

/* Synchronise `stream` and return LORDO_ENUMERIC if a kernel latched a breakdown since the
 * last poll (the latch is cleared), else LORDO_OK. */
int lordo_poll_status(lordo_ctx* ctx, void* stream);

/* Similarity of consecutive subspaces (Sec. 5.1, Metrics): for every matrix the mean squared singular
 * value of R = Q_new^T Q_old of the last lordo_refresh_subspace, (1/r) sum sigma_i^2 = ||R||_F^2 / r
 * (1: same subspace, 0: orthogonal).  dev_out: device array of n floats.  LORDO_ESTATE before the
 * first refresh. */
int lordo_get_mssv(lordo_ctx* ctx, float* dev_out, void* stream);

/* Stable rank of the source of the last refresh (Sec. 5.1, Metrics): sr = ||Src||_F^2 / ||Src||_2^2 for every matrix,
 * the Frobenius norm summed over the source during the refresh, the spectral norm taken as the leading Ritz value
 * (exact up to the convergence of the range finder's first direction).  dev_out: device array of n floats.
 * LORDO_ESTATE without hp.rayleigh_ritz or before the first refresh. */
int lordo_get_stable_rank(lordo_ctx* ctx, float* dev_out, void* stream);

/* The r-th spectral gap sigma_r - sigma_{r+1} of a source (Sec. 5.1, Metrics), per matrix, as an estimate:
 * sigma_r is the smallest Ritz value of the last refresh; sigma_{r+1} is the largest Ritz value of two block power
 * iterations on the source deflated by the current basis, (I - Q Q^T) Src, i.e. an approximation from below of the
 * spectral norm of the deflated source -- which equals sigma_{r+1} when Q spans the leading subspace exactly and
 * exceeds it otherwise (directions the range finder has not resolved stay in the deflated source).
 * Src, src_dtype, Omega as for lordo_refresh_subspace; pass the source of the last refresh.
 * dev_out: device array of n floats.  Changes no state that survives a step (Q, moments, weights are left as they
 * are); uses the scratch of the refresh, including what LORDO_STATE_GLOW / NUPD show.
 * LORDO_ESTATE without hp.rayleigh_ritz, before the first refresh, or between lordo_refresh_subspace_local and its step. */
int lordo_spectral_gap(lordo_ctx* ctx, const void* const* Src, int32_t src_dtype, const void* const* Omega,
                       float* dev_out, void* stream);

/* Measurement aid: with profiling on, every kernel class below is bracketed by a pair of HIP events
 * on the caller's stream (a few microseconds of overhead per launch).  lordo_profile_read
 * synchronises `stream` and returns the summed event time and the number of spans of one class
 * since profiling was last enabled.  Enabling again, or disabling, discards the record. */
#define LORDO_K_DOWN    0   /* down-projection GEMM,   one span per lordo_local_step            */
#define LORDO_K_ADAM    1   /* fused low-rank Adam,    one span per lordo_local_step            */
#define LORDO_K_UP      2   /* up-projection + apply,  one span per lordo_local_step            */
#define LORDO_K_OUTER   3   /* outer-step kernel,      one span per lordo_outer_step            */
#define LORDO_K_EXPORT  4   /* pseudo-gradient kernel, one span per lordo_export_pseudograd     */
#define LORDO_K_REFRESH 5   /* every kernel of one lordo_refresh_subspace call, as one span     */
int lordo_profile_enable(lordo_ctx* ctx, int32_t on);
int lordo_profile_read(lordo_ctx* ctx, int32_t kernel_class, double* total_ms, int64_t* launches, void* stream);

const char* lordo_strerror(int code);

/* Frees host-side bookkeeping only (the arena is the caller's).  NULL is allowed. */
void lordo_destroy(lordo_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* LORDO_H */
