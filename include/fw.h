/*
 * fw.h -- C ABI of the MI355X (gfx950) feature-whitening hot path.
 *
 * Method: "Feature Whitening via Gradient Transformation for Improved Convergence"
 * (arXiv 2010.01546).  Per whitened layer the library
 *   (1) accumulates the block sums behind the input moments  mu_x, Phi_x, phi_x   (Sec. 2, Sec. 4.1),
 *   (2) transforms the weight gradient  G -> G Q,  Q = T^T T                      (Sec. 3.1),
 *   (3) runs the recursive condition-number-reduction update of T, Q, Q_s         (Sec. 4),
 *   (4) builds the EVD / ZCA whitening matrix as the reference construction       (Sec. 2, Sec. 3.2).
 *
 * Conventions shared by every entry point
 *   - Every data pointer is a DEVICE pointer owned by the caller unless the comment says "host".
 *     Parameter structs (fw_conv_desc, fw_cond_params, fw_evd_params, fw_cond_state) are HOST structs
 *     read during the call; the pointers inside fw_cond_state are device pointers.
 *   - Matrices are dense, row-major, leading dimension = number of columns, float32 unless stated.
 *     Device pointers must be 16-byte aligned (FW_ERR_ALIGNMENT otherwise).
 *   - A convolution layer is taken in unfolded form: the sample rows x are the B*P patches of the input
 *     (P = Ho*Wo output positions), M = Cin*kh*kw features in the order m = (c*kh + ky)*kw + kx (the order of a
 *     contiguous weight tensor [S, Cin, kh, kw] viewed as [S, M]) unless the layout says otherwise, zero padding
 *     counts as data.  N_rows = B*P.  Whatever order is chosen, G, T, Q and Phi_x of a layer must all use it.
 *   - The library allocates no device memory, keeps no device state between calls and never frees, and has no
 *     process-wide setting (host side, each calling thread keeps the launch geometry of the layers it saw most recently,
 *     a pure function of the descriptor; fw_cond_reduce_step_static alone owns a fixed device array, see there).
 *     Scratch comes from the caller through (ws, ws_bytes); fw_workspace_bytes gives the size an entry point needs.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Work is enqueued on it and the
 *     call returns without waiting, except fw_whiten_evd, which waits on its own convergence flag.
 *   - Errors are return codes.  Arguments are validated before anything is enqueued; on a non-OK return
 *     from validation no output has been touched.  Data-dependent events of the recursive step (empty
 *     coherence set, estimate below the target power) are not errors: they are reported in fw_cond_info.
 */
#ifndef FW_H
#define FW_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    FW_OK = 0,
    FW_ERR_INVALID_ARG = 1,   /* NULL pointer, non-positive size, parameter out of its range */
    FW_ERR_UNSUPPORTED = 2,   /* valid in principle but not built (e.g. a shape beyond a stated limit) */
    FW_ERR_ALIGNMENT = 3,     /* a device pointer is not 16-byte aligned */
    FW_ERR_WORKSPACE = 4,     /* ws is NULL or ws_bytes is below fw_workspace_bytes(...) */
    FW_ERR_HIP = 5,           /* a HIP runtime call failed (launch error, no device) */
    FW_ERR_NOT_CONVERGED = 6  /* fw_whiten_evd hit max_sweeps; outputs hold the last iterate's result */
} fw_status;

typedef enum { FW_F32 = 0, FW_BF16 = 1 } fw_dtype;

typedef enum {
    FW_LAYOUT_ROWS = 0,  /* X is the row matrix [N_rows, M] itself (fully connected layer, or pre-unfolded) */
    FW_LAYOUT_NCHW = 1,  /* activation tensor [B, Cin, H, W] */
    FW_LAYOUT_NHWC = 2,  /* activation tensor [B, H, W, Cin] */
    FW_LAYOUT_NHWC_KKC = 3 /* activation tensor [B, H, W, Cin], features ordered m = (ky*kw + kx)*Cin + c: the order of a
                              channels-last weight tensor [S, kh, kw, Cin] viewed as [S, M].  This is the order the kernels
                              work in; the other tensor layouts pay a permutation of A when the sums are written out. */
} fw_layout;

/* Which form fw_cov_accumulate takes where both the direct product of the unfolded patch rows and the shift form
 * (stride-1 windows: tap pairs with the same offset share one product) apply.  Both compute the same sums of Sec. 2;
 * AUTO picks by an estimate of the run time.  SHIFT and DIRECT are meant for tuning and for tests that must reach one
 * form at sizes where the estimate prefers the other; where the shift form does not apply the field changes nothing. */
typedef enum {
    FW_COV_FORM_AUTO = 0,     /* by estimate: for float32 input this includes FW_COV_FORM_SPLIT from the measured break-even
                                 on: at least 32768 rows for 512 <= M < 1024, 8192 for M < 2048, 1024 for M < 4096, 256 beyond */
    FW_COV_FORM_SHIFT = 1,    /* shift form wherever it applies (products in the input's own precision) */
    FW_COV_FORM_DIRECT = 2,   /* never the shift form (products in the input's own precision) */
    FW_COV_FORM_SPLIT = 3     /* float32 input only (ignored for bfloat16): every value is split into two bfloat16 numbers
                                 hi + lo (16 significant bits, residual <= 2^-17 |x| of either sign) and the sums are taken on
                                 the bfloat16 matrix cores as (hi+lo)(hi+lo) with float32 accumulation: several times faster; the
                                 residuals are zero-mean rounding errors whose sum over N rows grows like sqrt(N) */
} fw_cov_form;

/* Geometry of a layer input.  FW_LAYOUT_ROWS: B = N_rows, Cin = M, H = W = kh = kw = stride = 1, pad = 0.
 * `form` (a fw_cov_form) travels with the geometry, so that fw_workspace_bytes, fw_cov_plan_query and fw_cov_accumulate
 * given the same descriptor always agree on how the layer runs; a zero-initialised field means AUTO. */
typedef struct { int B, Cin, H, W, kh, kw, stride, pad, form; } fw_conv_desc;

/* Operations for fw_workspace_bytes. */
typedef enum {
    FW_OP_COV_ACCUMULATE = 0, FW_OP_GRAD_TRANSFORM = 1, FW_OP_COND_REDUCE_STEP = 2, FW_OP_WHITEN_EVD = 3, FW_OP_COND_STATE_REFRESH = 4,
    FW_OP_GRAD_TRANSFORM_TAPS = 5, FW_OP_SGD_UPDATE = 6, FW_OP_DIAGNOSTICS = 7, FW_OP_COND_PROBE = 8
} fw_op;

/* ------------------------------------------------------------------------------------------------------------
 * (1) Moment accumulation -- the sums inside eqs. (vmuxi), (vPhixi) of Sec. 2 and eq. (phixmi) of Sec. 4.1.
 *
 *   A[i][j] += sum_rows x_i x_j   for i >= j (lower triangle incl. diagonal; entries above it are not touched)
 *   s[i]    += sum_rows x_i
 * over the N_rows = B*P patch rows of X, formed on the fly from the activation tensor (never materialised).
 *   X      in   activation in layout `lay`, element type `dt` (float32, or bfloat16 as raw 16-bit patterns)
 *   d      host geometry
 *   A      i/o  [M, M] float32, accumulated in place (zero it before the first batch of a block)
 *   s      i/o  [M] float32, accumulated in place
 *   ws     scratch, fw_workspace_bytes(FW_OP_COV_ACCUMULATE, M, 0, d, dt) bytes
 * Products are accumulated in float32 on the matrix cores (bf16 inputs: bf16 x bf16 -> float32; float32 inputs: float32
 * products, or hi + lo bfloat16 pairs in the split form, see fw_cov_form).  When the rows are
 * split into ranges, the partial sums of the ranges are combined in float64 before they are added to A; a tile
 * covered by a single range is added to A directly in float32.  The result is deterministic run to run.
 * Limits: M <= 16384; activation below 2^31 elements.
 */
fw_status fw_cov_accumulate(const void* X, fw_dtype dt, fw_layout lay, const fw_conv_desc* d,
                            float* A, float* s, void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------------------------------------------------
 * (1') Block moments from the accumulated sums -- eqs. (vmuxi), (vPhixi), (vmuxnz), (vPhixnz), (phixmi), (blambday).
 *
 *   mhat = s/n;   mu(i) = alpha*mu(i-1) + (1-alpha)*mhat
 *   C    = A/n - mhat mu(i)^T - mu(i) mhat^T + mu(i) mu(i)^T        (the covariance centred on mu(i), expanded)
 *   Phi_x(i) = alpha*Phi_x(i-1) + (1-alpha)*C;   phi_x(i) = alpha*phi_x(i-1) + (1-alpha)*diag(A)/n
 *   lambda_bar = mean(phi_x(i));   first_block != 0 drops the recursive average (alpha is ignored).
 *   A, s     in   sums from fw_cov_accumulate (lower triangle of A is read)
 *   n        total number of rows accumulated into A and s
 *   mu       i/o  [M]     in: mu(i-1), out: mu(i)
 *   Phi_x    i/o  [M, M]  in: Phi_x(i-1), out: Phi_x(i), written as a full symmetric matrix
 *   phi_x    i/o  [M]
 *   lambda_bar out one float on the device
 * Evaluated in float64 per element, stored as float32.
 */
fw_status fw_cov_finalize(const float* A, const float* s, long long n, int M, float alpha, int first_block,
                          float* mu, float* Phi_x, float* phi_x, float* lambda_bar, void* stream);

/* ------------------------------------------------------------------------------------------------------------
 * (2) Gradient transformation -- eqs. (mod_weight_grad), (vQ) of Sec. 3.1:  G_out = G Q,  Q = T^T T.
 *
 *   G      in   [S, M] element type `dt`
 *   Q      in   [M, M] float32, symmetric (Q or its smoothed version Q_s, eq. (vQs)); may be NULL if T is given
 *   T      in   [M, M] float32 or NULL.  Used only when Q is NULL: Q = T^T T is then built in the workspace first (in
 *               float32 below FW_REFRESH_SPLIT_MIN_M features; from there on with the columns of T split into bfloat16
 *               hi + lo planes on the bfloat16 matrix cores, relative Frobenius error of Q a few 1e-6, about 15 times
 *               faster at M = 4608).
 *   G_out  out  [S, M] element type `dt`; must not overlap G
 *   ws     scratch, fw_workspace_bytes(FW_OP_GRAD_TRANSFORM, M, S, NULL, dt) bytes; required when Q is NULL (the first
 *               fw_workspace_bytes(FW_OP_GRAD_TRANSFORM, M, 0, NULL, FW_F32) bytes of it suffice for that), optional
 *               otherwise: with all of it a product with few output tiles (small S) cuts its contraction index into runs
 *               over more workgroups and adds the runs in a fixed order (same float32 arithmetic, another summation
 *               order); for dt = FW_BF16 with Q given it also selects the widened form below (several times faster); for
 *               dt = FW_F32 and a large enough product (M >= 1024, S >= 128, S M >= FW_GRAD_SPLIT_MIN_SM, or
 *               FW_GRAD_SPLIT_MIN_SM_WIDE from M = 2048 on: the measured break-even) it selects the split form: G and Q
 *               are split into bfloat16 hi + lo planes (16 significant bits each) and multiplied on the bfloat16 matrix
 *               cores as hi hi + hi lo + lo hi with float32 accumulation (relative Frobenius error a few 1e-6 instead of
 *               a few 1e-7; 1.5 to 2.6 times as fast)
 * dt = FW_F32: float32 matrix-core products.
 * dt = FW_BF16 with the workspace: G is widened to float32 in the workspace, the products are float32 on the matrix
 *   cores with Q as it is (past the size rule above, with M a multiple of 4: the split form), G_out is rounded to
 *   bfloat16 (nearest even).
 * dt = FW_BF16 without it: Q is rounded to bfloat16 on the fly, products are bf16 x bf16 accumulated in float32,
 *   G_out is rounded to bfloat16.  Q must be symmetric in every mode (its rows are read as its columns).
 */
#define FW_GRAD_SPLIT_MIN_SM 1500000
#define FW_GRAD_SPLIT_MIN_SM_WIDE 1100000
fw_status fw_grad_transform(const void* G, fw_dtype dt, int S, int M, const float* T, const float* Q,
                            void* G_out, void* ws, size_t ws_bytes, void* stream);

/* How fw_grad_transform would run the product G Q for a given shape, element type and workspace size (host arithmetic
 * only): whether it takes the split form, and the flops the matrix cores execute for it (split form: bfloat16 flops,
 * three terms per float32 multiplication, whole tiles; otherwise 2 S M^2 float32 flops). */
typedef struct { int split; double mfma_flops_issued; } fw_grad_plan;
fw_status fw_grad_plan_query(fw_dtype dt, int S, int M, size_t ws_bytes, fw_grad_plan* plan);

/* Per-tap form of eq. (mod_weight_grad): a layer of eq. (vzrp3) has one S x M weight matrix per spatial offset n, and
 * each of their gradients is multiplied by the same Q.  For a convolution whitened per input channel (M = Cin, the
 * whitening placed in front of the convolution, Sec. 6) the offsets are the kernel taps:
 *   G_out[s][:][t] = G[s][:][t] Q   for every tap t
 *   G, G_out   [S, M, taps] element type `dt` (the layout of a convolution weight [S, Cin, kh, kw], taps = kh kw);
 *              must not overlap.  A channels-last weight [S, kh, kw, Cin] is plain [S taps, M] rows: use fw_grad_transform.
 *   Q          [M, M] float32, symmetric
 *   ws         scratch, fw_workspace_bytes(FW_OP_GRAD_TRANSFORM_TAPS, M, S * taps, NULL, dt) bytes (the gradient as rows)
 * Products are float32 on the matrix cores for both element types; bfloat16 results are rounded to nearest even.
 * When M is a multiple of 4 and the S * taps rows meet fw_grad_transform's size rule for the split form, the product takes
 * that form (bfloat16 hi + lo planes, relative error a few 1e-6).
 */
fw_status fw_grad_transform_taps(const void* G, fw_dtype dt, int S, int M, int taps, const float* Q, void* G_out,
                                 void* ws, size_t ws_bytes, void* stream);

/* Weight update with the transformed gradient fused into the product -- eqs. (vtWrn_SGD), (mod_weight_grad); momentum
 * and weight decay as named in Sec. 6 (heavy-ball form; the decay acts on the stored parameter):
 *   d = G Q + weight_decay W;   V = momentum V + d  (when momentum > 0);   W -= lr (V, or d without momentum)
 *   G      in      [S, M] (taps = 1) or [S, M, taps], element type `dt`; not overlapping W or V
 *   W      in/out  stored weights W~, float32, same shape as G
 *   V      in/out  momentum buffer, float32, same shape, zero before the first update; may be NULL when momentum = 0
 *   ws     scratch, fw_workspace_bytes(FW_OP_SGD_UPDATE, M, S * taps, NULL, dt) bytes; not needed for FW_F32 with taps = 1.
 *          With it, M a multiple of 4 and S * taps rows that meet fw_grad_transform's size rule for the split form, the
 *          product takes that form (about 1.7 times faster at S = 512, M = 4608); its runs of the contraction index are
 *          then kept in the workspace and added by the pass that updates W and V.
 * Without the split form the transformed gradient is not written anywhere.
 */
typedef struct { float lr, momentum, weight_decay; } fw_sgd_params;
fw_status fw_sgd_update(const void* G, fw_dtype dt, int S, int M, int taps, const float* Q, const fw_sgd_params* p,
                        float* W, float* V, void* ws, size_t ws_bytes, void* stream);

/* Bias compensation when the tracked mean moves at a block boundary -- Sec. 3.1, eq. (vtb_corr):
 *   b[s] += scale * sum_{c,t} W[s][c][t] (mu_new[c] - mu_old[c])
 * so that sum W~ (x - mu) + b is the same before and after (new mean minus old mean: the sign that keeps that relation;
 * the printed equation has the two means swapped).
 *   b        in/out  [S] float32
 *   W        in      [S, M] (taps = 1) or [S, M, taps] float32
 *   mu_old, mu_new   [M] float32
 *   scale    the factor (1/R) sum_r of the equation for weights shared over the R output positions: 1
 */
fw_status fw_bias_compensate(float* b, const float* W, int S, int M, int taps, const float* mu_old, const float* mu_new,
                             float scale, void* stream);

/* ------------------------------------------------------------------------------------------------------------
 * (3) Recursive condition-number reduction -- Sec. 4 (eqs. (lambda)-(vQ_rec), (xim)-(tve)).
 */
typedef struct {
    float gamma;        /* leakage factor, 0 < gamma <= 1                      eq. (vT_rec) */
    float delta;        /* power-reduction target factor, > 0                  eq. (ge)     */
    float eps;          /* lower bound of the denominator, > 0                 eq. (ge)     */
    float c_rel;        /* relative coherence threshold                        Sec. 4.2     */
    float c_abs;        /* absolute coherence threshold                        Sec. 4.2     */
    float beta;         /* smoothing factor of Q_s, 0 <= beta < 1              eq. (vQs)    */
    int n_power_iters;  /* extra refinements v <- Phi_y v/|Phi_y v| of the estimate (0 = the paper's estimator) */
    int guard;          /* != 0: skip the shrink when it would amplify (g_e >= 1); the leak is still applied */
} fw_cond_params;

/* State of one layer; all pointers are device pointers to caller-owned [M, M] float32 matrices unless noted. */
typedef struct {
    int M;
    const float* Phi_x;     /* in:  covariance of the block, symmetric (from fw_cov_finalize)          */
    const float* lambda_bar;/* in:  one float on the device, average input power, eq. (blambday)       */
    float* T;               /* i/o: whitening matrix (non-symmetric in general)                         */
    float* Q;               /* i/o: T^T T, maintained by eq. (vQ_rec)                                   */
    float* Qs;              /* i/o: smoothed Q, eq. (vQs)                                               */
    float* Phi_y;           /* i/o: T Phi_x T^T, maintained by O(M^2) updates                           */
    float* Psi;             /* i/o: T Phi_x, needed for the update of Phi_y when gamma < 1; may be NULL if gamma == 1 */
    float* xi2;             /* i/o: [M] squared column norms of Phi_y, carried from step to step        */
} fw_cond_state;

/* Diagnostics of one step, written to device memory. */
typedef struct {
    float lambda_e, g_e, a_e, v_norm;  /* eq. (lambda), eq. (ge), eq. (xi) as applied (0 if skipped), |v~| */
    int m_prime, set_size;            /* eq. (mt), |set| of Sec. 4.2 */
    int applied;                      /* 1 if the shrink was applied, 0 if only the leak */
    int flags;                        /* bit 0: coherence set empty; bit 1: skipped by the guard; bit 2: non-finite value seen */
} fw_cond_info;

/* T = Q = Qs = I, Phi_y = Psi = Phi_x, xi2 = squared column norms of Phi_x  (eqs. (vT_init), Qs(-1) = I). */
fw_status fw_cond_state_init(const fw_cond_state* st, void* stream);

/* A new block brings a new Phi_x while T, Q, Qs carry over (Sec. 2: the moments are re-estimated block by block; Sec. 4:
 * the recursion works on the covariance of the transformed input).  Recomputes, for the T at hand,
 *   Psi = T Phi_x,   Phi_y = T Phi_x T^T (written exactly symmetric),   xi2 = squared column norms of Phi_y
 * by two M x M x M products on the matrix cores.  T, Q, Qs are not touched.
 *   ws   scratch of fw_workspace_bytes(FW_OP_COND_STATE_REFRESH, M, 0, NULL, FW_F32) bytes (about 16 M^2 bytes).
 *        With it the float32 operands are split into two bfloat16 numbers each (hi + lo, 16 significant bits) and the
 *        products run on the bfloat16 matrix cores as hi hi + hi lo + lo hi with float32 accumulation: relative
 *        Frobenius error of Psi and Phi_y a few 1e-6, several times faster.
 *        With ws NULL or smaller than that, or M < FW_REFRESH_SPLIT_MIN_M (where the split form would not be faster), the
 *        products run in plain float32 (error a few 1e-7); that needs st->Psi, or at least M^2 floats (rounded up to 256
 *        bytes) of ws to stand in for it (FW_ERR_WORKSPACE otherwise).
 */
#define FW_REFRESH_SPLIT_MIN_M 1536

/* How fw_cond_state_refresh would run for a given M and workspace size (host arithmetic only): which form the two
 * products take and the flops the matrix cores execute for them (split form: bfloat16 flops, three terms per float32
 * multiplication, whole tiles, lower triangle only for Phi_y; float32 form: 4 M^3). */
typedef struct { int split; double mfma_flops_issued; } fw_refresh_plan;
fw_status fw_cond_refresh_plan_query(int M, size_t ws_bytes, fw_refresh_plan* plan);
fw_status fw_cond_state_refresh(const fw_cond_state* st, void* ws, size_t ws_bytes, void* stream);

/* One step: estimate the high-power direction v of Phi_y (Sec. 4.2), lambda_e, g_e, a_e (eqs. (lambda), (ge), (xi)),
 * t = T^T v, then in one pass T <- gamma (T + a v t^T) + (1-gamma) I (eq. (vT_rec)), Q by eq. (vQ_rec),
 * Qs <- beta Qs + (1-beta) Q (eq. (vQs)), and Phi_y, Psi, xi2 brought up to date for the new T.
 *   info_dev  out  one fw_cond_info on the device (may be NULL)
 *   ws        scratch, fw_workspace_bytes(FW_OP_COND_REDUCE_STEP, M, 0, NULL, FW_F32) bytes
 * Phi_y is taken as symmetric (its rows are read where the paper names columns).  Ties of the arg-max go to the
 * lowest index.
 */
fw_status fw_cond_reduce_step(const fw_cond_state* st, const fw_cond_params* p, fw_cond_info* info_dev,
                              void* ws, size_t ws_bytes, void* stream);

/* The same step for callers that cannot allocate device memory or hand over a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc.  Identical arithmetic and kernels; the scratch is a fixed array
 * of 6 MiB in the library's device image (one copy per GPU, held until the process ends), so
 *   - M is limited to FW_COND_STATIC_MAX_M (FW_ERR_UNSUPPORTED beyond it, nothing enqueued),
 *   - the call allocates and frees nothing (its only set-up is one symbol-address lookup per device, on the first call
 *     made with that device current),
 *   - all calls on one GPU share the array: calls that overlap in time on one GPU (different streams, different
 *     threads) race on it and must be serialised by the caller.  Nothing in the array has to survive between calls and
 *     every entry is written before it is read, so a call is not affected by what the previous one left.
 * Other arguments, validation and error codes as fw_cond_reduce_step. */
#define FW_COND_STATIC_MAX_M 4608
fw_status fw_cond_reduce_step_static(const fw_cond_state* st, const fw_cond_params* p, fw_cond_info* info_dev, void* stream);

/* ------------------------------------------------------------------------------------------------------------
 * (4) EVD / ZCA reference -- eqs. (vPhix_evd), (vT_EVD), (vg) of Sec. 2; gain variant eqs. (hMs), (g_mod) of Sec. 3.2.
 */
typedef struct {
    float eps;        /* eq. (vg) */
    float g_max;      /* eq. (g_mod), gain_mode 1 only */
    float beta;       /* smoothing of Qs when Qs != NULL, eq. (vQs) */
    float tol;        /* rotation threshold of the Jacobi sweeps (relative); <= 0 selects the default 1e-12 */
    int gain_mode;    /* 0: g = 1/max(lambda, eps); 1: g = min(1/(M lambda_bar_m), g_max) on the signal subspace, 1 elsewhere */
    int max_sweeps;   /* <= 0 selects the default 30 */
} fw_evd_params;

/*   Phi_x   in   [M, M] symmetric
 *   T, Q    out  [M, M]: T = V diag(sqrt g) V^T, Q = V diag(g) V^T
 *   Qs      i/o  [M, M] or NULL: Qs <- beta Qs + (1-beta) Q
 *   lambda  out  [M] eigenvalues, decreasing
 *   ws      scratch, fw_workspace_bytes(FW_OP_WHITEN_EVD, M, 0, NULL, FW_F32) bytes
 * The decomposition is a one-sided Jacobi iteration carried out in float64 inside the workspace; the call blocks
 * once per sweep to read the rotation count.
 */
fw_status fw_whiten_evd(const float* Phi_x, int M, const fw_evd_params* p, float* T, float* Q, float* Qs,
                        float* lambda, void* ws, size_t ws_bytes, void* stream);

/* Monitoring figures of Sec. 6.
 *   Phi_y   in   [M, M] float32 with positive diagonal, or NULL:  out[0] = rho = M / sum_{m,m'} Phi_y[m'][m]^2 /
 *                (Phi_y[m][m] Phi_y[m'][m'])   (eq. (rho), summed over all pairs, m = m' included: the reading that has
 *                both stated extremes, 1 for a diagonal matrix and 1/M for fully correlated features)
 *   lambda  in   [M] float32 eigenvalues (any order), or NULL:  out[2] = Ms_hat = exp(-sum lb log lb), lb = lambda /
 *                sum(lambda), non-positive eigenvalues counted as zero (eq. (hMs), read as the exponential of the spectral
 *                entropy);  out[1] = kappa = Ms_hat / M
 *   out     out  device float32[3]; entries whose input is NULL are left alone
 *   ws      scratch, fw_workspace_bytes(FW_OP_DIAGNOSTICS, M, 0, NULL, FW_F32) bytes, needed when Phi_y is given
 */
fw_status fw_diagnostics(const float* Phi_y, const float* lambda, int M, float* out, void* ws, size_t ws_bytes, void* stream);

/* Condition-number probe.  Sec. 4 builds the recursion on one figure: the condition number of Phi_y (convergence time is
 * proportional to it, 1 means white).  This call estimates it without an eigen-decomposition: k steps of the Lanczos
 * iteration on Phi_y from the start vector b0 (fully re-orthogonalised, vectors and sums in float64, Phi_y read once per
 * step: k M^2 words of traffic), then the extreme eigenvalues of the k x k tridiagonal projection.  Those Ritz values lie
 * inside the spectrum, so the ratio never overestimates the condition number; the top converges within a few steps, the
 * bottom more slowly.
 *   Phi_y   in   [M, M] float32, symmetric
 *   b0      in   [M] float32 start vector, or NULL for the all-ones vector
 *   k       Krylov dimension, 1 .. FW_COND_PROBE_MAX_K; the iteration stops early when the space becomes invariant
 *   out     out  device float32[4]: largest Ritz value, smallest Ritz value, their ratio (inf when the smallest is <= 0),
 *                dimension reached
 *   ws      scratch, fw_workspace_bytes(FW_OP_COND_PROBE, M, k, NULL, FW_F32) bytes (the S argument carries k)
 * No host synchronisation. */
#define FW_COND_PROBE_MAX_K 32
fw_status fw_cond_probe(const float* Phi_y, int M, const float* b0, int k, float* out, void* ws, size_t ws_bytes, void* stream);

/* How fw_cov_accumulate would run a layer (host arithmetic only, no GPU call): for introspection and tests.
 *   shift              1: stride-1 window accumulated through shift correlations (tap pairs with the same offset share one
 *                      product), 0: direct products of the unfolded patch rows
 *   regions            shift form: image regions whose pixels serve the same set of taps (0 in the direct form)
 *   covered_pixels     shift form: pixels of all regions together (= B H W when every pixel lies under some window)
 *   differences        shift form: tap differences kept (13 for a 3x3 window)
 *   workgroups         workgroups of the contraction kernel
 *   ranges             pieces the reduction axis (patch rows / pixels) is cut into
 *   mfma_flops_issued  flops the matrix cores execute per call, padding included (the algorithmic count is
 *                      N_rows M (M + 1))
 */
typedef struct {
    int shift, regions, differences, workgroups, ranges;
    long long covered_pixels;
    double mfma_flops_issued;
    int split_bf16;           /* 1: float32 input taken in the split form (the other fields then describe the bfloat16 run on
                                 twice the channels, mfma_flops_issued counts bfloat16 flops) */
} fw_cov_plan;
fw_status fw_cov_plan_query(fw_dtype dt, fw_layout lay, const fw_conv_desc* d, fw_cov_plan* plan);

/* Measurement helper (not a step of the method): every compute unit runs nothing but dense bfloat16 matrix instructions
 * (v_mfma_f32_32x32x16_bf16 on register operands: pseudo-random values, or zeros when zero_operands != 0) for `iters` rounds
 * of 16 products per wavefront, 4096 wavefronts.  Timed by the caller, *flops_host / time is what the matrix cores
 * sustain under the chip's power limit: the ceiling against which the rates of the product kernels are read
 * (the published peak assumes a clock the chip does not hold under this load).
 *   sink        out  one float on the device (never actually written: it keeps the products alive)
 *   flops_host  out  HOST double: flops the launch executes; may be NULL
 */
fw_status fw_mfma_rate_probe(int zero_operands, int iters, float* sink, double* flops_host, void* stream);

/* Scratch bytes an entry point needs for the given sizes (0 if none).  `d` is needed for FW_OP_COV_ACCUMULATE only;
 * for the per-tap operations S is the number of gradient rows, S * taps; for FW_OP_COND_PROBE S is the Krylov dimension k. */
size_t fw_workspace_bytes(fw_op op, int M, int S, const fw_conv_desc* d, fw_dtype dt);

const char* fw_status_string(fw_status st);

/* Library version as major*10000 + minor*100 + patch. */
int fw_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FW_H */
