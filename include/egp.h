/*
 * egp.h -- C ABI of libegp: the hot path of exact Gaussian-process training on one MI355X (gfx950).
 *
 * The kernel matrix K(X,X) is touched only through products with it; its tiles are formed on the fly
 * in registers and never stored in device memory (paper, Method: "O(n) memory MVM-based inference" and
 * "Partitioned kernel MVMs"). That product drives a batched preconditioned conjugate-gradient solver
 * with a partial pivoted-Cholesky preconditioner (paper, Background: "Conjugate gradients"; Method:
 * "Preconditioning", "PCG Convergence Criteria").
 *
 * Conventions common to every entry point
 *   - "device" pointers are HIP device memory on the current device, 16-byte aligned, owned by the
 *     caller; the library never allocates or frees device memory and keeps no pointer after return.
 *   - "host" pointers are ordinary host memory, read or written during the call only.
 *   - X is row-major n x d fp32. V, B, U, out are row-major n x t fp32 (t contiguous).
 *   - ws is a device workspace of at least egp_*_ws_bytes(...) bytes (256-byte aligned); its content
 *     on entry is ignored and on return is unspecified.
 *   - stream is a hipStream_t passed as void* (NULL = the default stream). Work is enqueued on it;
 *     entry points that return host results synchronise on it before returning.
 *   - Return value: 0 on success, a negative egp_status_t otherwise; egp_last_error() then returns a
 *     thread-local, statically stored message. Nothing is written to outputs on EGP_ERR_ARG / EGP_ERR_WS.
 *   - Inputs are never modified.
 *   - Threads: the library keeps no state between calls except two process-wide defaults (egp_set_kmm_mode,
 *     egp_set_mbcg_shrink) and the profiling counters. Each call reads the defaults once, at its entry, and works on
 *     that copy to its end: a setter called from another thread while a call runs affects later calls only. Calls
 *     from different threads may run concurrently when their workspaces and outputs do not overlap. The *_ex entry
 *     points take the two options per call (egp_call_opts_t) and do not depend on the defaults at all.
 */
#ifndef EGP_H
#define EGP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  EGP_OK = 0,
  EGP_ERR_ARG = -1,       /* null / misaligned pointer, size out of range, bad enum, non-positive scale */
  EGP_ERR_WS = -2,        /* workspace too small */
  EGP_ERR_DEVICE = -3,    /* a HIP call failed; message holds hipGetErrorString */
  EGP_ERR_BREAKDOWN = -4  /* non-positive curvature d^T Khat d in CG, or non-finite values */
} egp_status_t;

/* Stationary kernels named by the paper (Background: RBF and Matern; Experiment details: Matern-3/2;
 * appendix: independent lengthscales). k(x,x') = outputscale * g(r), r^2 = sum_k ((x_k-x'_k)/l_k)^2,
 *   RBF       g = exp(-r^2/2)
 *   MATERN32  g = (1 + sqrt3 r) exp(-sqrt3 r)
 *   MATERN52  g = (1 + sqrt5 r + 5 r^2/3) exp(-sqrt5 r)
 *   MATERN12  g = exp(-r)   (the Matern family's nu = 1/2 member; its lengthscale derivative keeps a 1/r, taken as
 *                            0 for a point against itself)                                           */
typedef enum { EGP_RBF = 0, EGP_MATERN32 = 1, EGP_MATERN52 = 2, EGP_MATERN12 = 3 } egp_kernel_t;

#define EGP_D_MAX 31        /* largest input dimension of egp_kmm_grad (the materialised derivative product) and of
                               the bf16-split modes */
#define EGP_D_WIDE_MAX 399  /* largest input dimension of every other entry point (d > 31 runs variants that keep
                               the row operands in LDS) */
#define EGP_T_MAX 1024   /* largest number of right-hand-side columns */
#define EGP_RANK_MAX 1024 /* largest preconditioner rank and Lanczos cache rank */

typedef struct {
  int32_t kernel_type;        /* egp_kernel_t */
  int32_t d;                  /* 1..EGP_D_WIDE_MAX (1..EGP_D_MAX for egp_kmm_grad) */
  const float* lengthscales;  /* host, d values > 0 (a shared lengthscale is d equal values) */
  float outputscale;          /* s > 0 */
  float noise;                /* sigma^2 >= 0, the value added to the diagonal: Khat = K + noise*I
                                 (paper, Background, Notation) */
} egp_hyper_t;

/* Rank-k preconditioner P = L L^T + noise*I (paper, Method, "Preconditioning").
 * Buffers are the caller's; egp_piv_chol_precond fills them, egp_mbcg reads them. */
typedef struct {
  int32_t rank;      /* in: capacity of L / pivots / small; out: steps actually taken (<= capacity) */
  float* L;          /* device, [capacity][n]: column m of the factor is contiguous (row-major k x n) */
  int32_t* pivots;   /* host, capacity entries: original row indices in selection order */
  double* small;     /* host, capacity*capacity + 1 doubles: lower Cholesky factor (row-major rank x rank)
                        of noise*I + L^T L, followed at index capacity*capacity by log|P| */
  double* small_dev; /* device, capacity*capacity doubles: inverse of noise*I + L^T L (row-major
                        rank x rank), used by the solver to apply P^{-1}. fp64 because P^{-1} r subtracts
                        nearly equal vectors: the k x k algebra and its n-term sums run in fp64 */
} egp_precond_t;

/* Per-call options of the *_ex entry points. A field set to -1 takes the process-wide default of the matching
 * setter; opts = NULL takes both defaults (egp_x(...) is egp_x_ex(..., NULL)).
 *   kmm_mode     an egp_kmm_mode_t (see egp_set_kmm_mode)
 *   mbcg_shrink  0 or 1 (see egp_mbcg)
 * Other values return EGP_ERR_ARG. */
typedef struct {
  int32_t kmm_mode;
  int32_t mbcg_shrink;
} egp_call_opts_t;

/* out = Khat V = K(X,X) V + noise V, K never materialised (paper, Method, "Partitioned kernel MVMs":
 * row blocks of the kernel matrix are formed, multiplied and discarded; here a block lives in
 * registers). noise = 0 gives K V. t in 1..EGP_T_MAX. Asynchronous on `stream`. The same call gives the same
 * bits every time (fixed summation orders; sums that cross workgroups are exact integer adds). */
int egp_kmm(const float* X /*device n x d*/, int64_t n, const float* V /*device n x t*/, int32_t t,
            const egp_hyper_t* h /*host*/, float* out /*device n x t*/, void* ws, size_t ws_bytes,
            void* stream);
int egp_kmm_ex(const float* X, int64_t n, const float* V, int32_t t, const egp_hyper_t* h, float* out, void* ws,
               size_t ws_bytes, void* stream, const egp_call_opts_t* opts /*host, may be NULL*/);
size_t egp_kmm_ws_bytes(int64_t n, int32_t d, int32_t t);      /* covers every mode */

/* dout[k] = (dK/dl_k) V for k = 0..d-1, dout laid out [d][n][t]: the products the marginal-likelihood
 * gradient needs (paper, Eq. 2). dK/dl_k [i,j] = s h(r_ij) (x_ik-x_jk)^2 / l_k^3 with h = g for RBF,
 * 3 exp(-sqrt3 r) for MATERN32, (5/3)(1+sqrt5 r) exp(-sqrt5 r) for MATERN52. t in 1..EGP_T_MAX.
 * Asynchronous on `stream`. */
int egp_kmm_grad(const float* X, int64_t n, const float* V, int32_t t, const egp_hyper_t* h,
                 float* dout /*device d x n x t*/, void* ws, size_t ws_bytes, void* stream);
size_t egp_kmm_grad_ws_bytes(int64_t n, int32_t d, int32_t t);

/* Bilinear forms with the kernel derivatives, without the d x n x t intermediate of egp_kmm_grad:
 *   out[k] = sum_c w[c] A[:,c]^T (dK/dl_k) B[:,c]   for k = 0..d-1,
 *   out[d] = sum_c w[c] A[:,c]^T K B[:,c] / outputscale         (the outputscale derivative of K),
 * which is what every term of the marginal-likelihood gradient is (paper, Eq. 2: A = B = Khat^{-1} y for the
 * data term; A = Khat^{-1} z_c, B = P^{-1} z_c for the probe estimate of the trace).
 *   A, B  device n x t row-major, t in 1..36;  w host, t weights (NULL = all ones);  out host, d + 1 doubles.
 * Synchronises on `stream`. */
int egp_kmm_grad_bilinear(const float* X, int64_t n, const float* A, const float* B, int32_t t, const float* w,
                          const egp_hyper_t* h, double* out, void* ws, size_t ws_bytes, void* stream);
size_t egp_kmm_grad_bilinear_ws_bytes(int64_t n, int32_t d, int32_t t);

/* Partial pivoted Cholesky of the noise-free K from `rank` kernel rows computed on the fly (paper,
 * Method, "Preconditioning": a rank-k preconditioner needs only k kernel rows and is built once
 * before CG). Greedy diagonal pivoting, ties to the lowest index; stops early when the largest
 * remaining residual diagonal is <= tol_abs. Fills P (see egp_precond_t; P->rank must hold the
 * capacity = requested rank on entry, 1..min(n, EGP_RANK_MAX)). Synchronises on `stream`. The k x k factor and
 * inverse are fp64 work on the host; from rank 128 on it is spread over up to 16 host threads for the duration of
 * the call. */
int egp_piv_chol_precond(const float* X, int64_t n, const egp_hyper_t* h, float tol_abs,
                         egp_precond_t* P, void* ws, size_t ws_bytes, void* stream);
size_t egp_piv_chol_precond_ws_bytes(int64_t n, int32_t d, int32_t rank);

/* Batched preconditioned CG on Khat U = B for all t columns at once (paper, Background, "Conjugate
 * gradients" and the modified PCG it cites; Method: four vectors u, r, p, z per column).
 * Starts from U = 0. After every completed iteration the relative residuals ||r_c|| / ||b_c|| of the
 * recurrence residual are read back; the solve stops when their maximum is <= tol or after max_iter
 * iterations (not reaching tol is not an error). P = NULL runs plain CG.
 *   U          device n x t, the solutions
 *   cg_coef    host, [max_iter][2][t] doubles: alpha_j and beta_j per column (beta_j of the last
 *              iteration is 0); from these the caller builds the Lanczos tridiagonals
 *              T[j,j] = 1/alpha_j + beta_{j-1}/alpha_{j-1}, T[j,j+1] = sqrt(beta_j)/alpha_j.  May be NULL.
 *   gamma0     host, t doubles: b_c^T P^{-1} b_c (quadrature weights). May be NULL.
 *   iters_done host, one int32
 *   rel_resid  host, t floats, relative residuals after the last iteration
 *   resid_hist host, [max_iter][t] floats: relative residuals after every iteration. May be NULL.
 * t in 1..33. Synchronises on `stream`. With max_iter = 0 no iteration runs: U = 0 and rel_resid is 1 for every
 * column with b_c != 0.
 * Column shrinking (mbcg_shrink = 1 in egp_call_opts_t, or the process-wide default egp_set_mbcg_shrink(1); off
 * unless asked for): trailing columns that have met the tolerance leave the
 * iteration: after each iteration the active columns are [0, 1 + last column still above tol), so with B = [y | probes]
 * and y the slowest column the late iterations run on fewer columns (down to one). A column that has left keeps its
 * solution and residual of that moment; its alpha_j, beta_j in cg_coef are 0 from then on (its own iteration count
 * m_c is the number of non-zero alpha_j; beta_{m_c - 1} belongs to a step it did not take and is to be ignored).
 * Columns are independent in CG, so every column's iterates are the ones it has without the switch; only the extra
 * iterations that converged columns otherwise receive are skipped.
 * egp_mll and egp_train_adam honour the option as well, and there it changes the result: a probe's Lanczos
 * tridiagonal then has only as many steps as the probe needed to meet the tolerance, so the quadrature order of the
 * log-determinant estimate is truncated and the estimate is biased. At a loose tolerance the shift is large: with
 * tol = 1 (the paper's training tolerance) probes leave after a handful of steps, and on a 2^21-point Matern-3/2
 * problem the value moved by about 7 % (158.1e3 -> 147.7e3); at tight tolerances both settings agree. Use it for
 * solves; leave it off for likelihood values unless that bias is acceptable. */
int egp_mbcg(const float* X, int64_t n, const float* B, int32_t t, const egp_hyper_t* h,
             const egp_precond_t* P, int32_t max_iter, float tol, float* U, double* cg_coef,
             double* gamma0, int32_t* iters_done, float* rel_resid, float* resid_hist, void* ws,
             size_t ws_bytes, void* stream);
int egp_mbcg_ex(const float* X, int64_t n, const float* B, int32_t t, const egp_hyper_t* h, const egp_precond_t* P,
                int32_t max_iter, float tol, float* U, double* cg_coef, double* gamma0, int32_t* iters_done,
                float* rel_resid, float* resid_hist, void* ws, size_t ws_bytes, void* stream,
                const egp_call_opts_t* opts /*host, may be NULL*/);
size_t egp_mbcg_ws_bytes(int64_t n, int32_t d, int32_t t, int32_t rank, int32_t max_iter);

/* One evaluation of the log marginal likelihood and its gradient (paper, Eq. 1 and Eq. 2) by the
 * modified-PCG route the paper builds on: rank-`rank` pivoted-Cholesky preconditioner, one batched solve
 * on [y | tp probe vectors], stochastic Lanczos quadrature for log|Khat|, probe estimates of the trace
 * terms, derivative products through egp_kmm_grad's kernel. Zero prior mean.
 *   y    device, n floats
 *   W1   device, rank x tp Rademacher (+-1) draws (row-major); ignored when rank = 0
 *   W2   device, n x tp Rademacher draws; probe c is z_c = L W1[:,c] + sqrt(noise) W2[:,c] (covariance P);
 *        with rank = 0 the probes are W2 itself
 *   out  host: value, log-determinant estimate, y^T Khat^{-1} y, gradient w.r.t.
 *        (l_1..l_d, outputscale, noise) in grad[0..d+1], iterations used, rank used, worst residual
 * tp in 1..32, rank in 0..EGP_RANK_MAX (noise > 0 needed when rank > 0). Synchronises on `stream`. */
typedef struct {
  double mll, logdet, quad;
  double grad[EGP_D_WIDE_MAX + 2];
  int32_t iters, precond_rank;
  float rel_resid_max;
} egp_mll_result_t;
int egp_mll(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
            const egp_hyper_t* h, int32_t rank, int32_t max_iter, float tol, egp_mll_result_t* out,
            void* ws, size_t ws_bytes, void* stream);
int egp_mll_ex(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
               const egp_hyper_t* h, int32_t rank, int32_t max_iter, float tol, egp_mll_result_t* out,
               void* ws, size_t ws_bytes, void* stream, const egp_call_opts_t* opts /*host, may be NULL*/);
size_t egp_mll_ws_bytes(int64_t n, int32_t d, int32_t tp, int32_t rank, int32_t max_iter);

/* Hyper-parameter fitting: `steps` Adam ascent steps on the log marginal likelihood (paper, Experiment details:
 * Adam with step size 0.1, a few steps on the full data after pre-training on a subset — pre-training is this
 * same call on a subset; learned noise kept above a floor). Each step is one egp_mll evaluation with the given
 * probe draws (the same draws at every step). Parameters move in log-space: l_k, outputscale, and
 * noise - noise_floor stay positive. The objective is L / n.
 *   lengthscales  host, d floats: start values in, fitted values out
 *   outputscale, noise  host scalars: start values in, fitted values out
 *   last          host, optional: the evaluation at the final parameters
 *   mll_history   host, optional, steps + 1 doubles: L before each step and at the end
 * Workspace: egp_mll_ws_bytes. Synchronises on `stream`. */
typedef struct {
  int32_t steps;      /* >= 0 */
  float lr;           /* Adam step size (0.1 in the paper) */
  float beta1, beta2, eps;   /* 0.9, 0.999, 1e-8 */
  float noise_floor;  /* >= 0 (0.1 in the paper's largest runs) */
} egp_adam_t;
int egp_train_adam(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
                   int32_t kernel_type, int32_t d, float* lengthscales, float* outputscale, float* noise,
                   int32_t rank, int32_t max_iter, float tol, const egp_adam_t* opt, egp_mll_result_t* last,
                   double* mll_history, void* ws, size_t ws_bytes, void* stream);
int egp_train_adam_ex(const float* X, int64_t n, const float* y, const float* W1, const float* W2, int32_t tp,
                      int32_t kernel_type, int32_t d, float* lengthscales, float* outputscale, float* noise,
                      int32_t rank, int32_t max_iter, float tol, const egp_adam_t* opt, egp_mll_result_t* last,
                      double* mll_history, void* ws, size_t ws_bytes, void* stream,
                      const egp_call_opts_t* opts /*host, may be NULL*/);

/* Host-only helper of egp_mll, exported for testing: e1^T log(T) e1 of the symmetric positive definite
 * tridiagonal T with diagonal diag[0..m) and off-diagonal off[0..m-1). Returns 0, or EGP_ERR_BREAKDOWN
 * when T is not positive definite. */
int egp_tridiag_logquad(const double* diag, const double* off, int32_t m, double* out);

/* Prediction path (paper, Method "Predictions"; predictive mean and variance equations).
 *
 * egp_kmm_cross: out (nq x t) = K(Xq, X) V, the rectangular product between nq query points and the n
 * training points (no noise term). V is n x t row-major. Asynchronous.
 *
 * egp_lanczos: training-data-dependent variance cache. r Lanczos steps on Khat with full
 * re-orthogonalisation from the start vector b (e.g. y): Q (device, [r][n], orthonormal rows) and the
 * tridiagonal T = Q Khat Q^T as alpha[r] (diagonal) and beta[r-1] (off-diagonal) on the host. *steps <= r is
 * the number of vectors produced (fewer when the Krylov space is exhausted). r in 1..EGP_RANK_MAX.
 * Synchronises.
 *
 * egp_predict: mean (device, nq) = K(Xq, X) a with the cached solve a = Khat^{-1} y (device, n); when var is
 * not NULL, var (device, nq) = outputscale - g^T T^{-1} g with g = Q K(X, xq): the variance of the latent
 * function from the rank-r cache, O(n r) per query point and no solve. It is never below the exact variance
 * and reaches it as r grows. Synchronises.
 *
 * egp_block_lanczos: the same cache from a block of b start vectors (B0: device, n x b row-major, b in 1..32; e.g.
 * [y | random signs]). Builds an orthonormal basis Q (device, [b*blocks][n]) of span{B0, Khat B0, ..,
 * Khat^(blocks-1) B0} and the projected matrix T = Q Khat Q^T (host, (b*blocks)^2 doubles, row-major with leading
 * dimension b*blocks; rows and columns beyond *rows are zero). One fused multiply serves b basis vectors, which
 * makes the cache b times cheaper per vector than egp_lanczos. *rows = b * (blocks completed), fewer than
 * b*blocks when the Krylov space is exhausted. b*blocks in 1..EGP_RANK_MAX. Synchronises.
 *
 * egp_predict_dense: egp_predict with such a dense T (leading dimension ldt) in place of (alpha, beta). */
int egp_kmm_cross(const float* Xq, int64_t nq, const float* X, int64_t n, const float* V, int32_t t,
                  const egp_hyper_t* h, float* out, void* ws, size_t ws_bytes, void* stream);
size_t egp_kmm_cross_ws_bytes(int64_t nq, int64_t n, int32_t d, int32_t t);
int egp_lanczos(const float* X, int64_t n, const egp_hyper_t* h, const float* b, int32_t r, float* Q,
                double* alpha, double* beta, int32_t* steps, void* ws, size_t ws_bytes, void* stream);
size_t egp_lanczos_ws_bytes(int64_t n, int32_t d, int32_t r);
int egp_predict(const float* Xq, int64_t nq, const float* X, int64_t n, const egp_hyper_t* h, const float* a,
                const float* Q, int32_t r, const double* alpha, const double* beta, float* mean, float* var,
                void* ws, size_t ws_bytes, void* stream);
size_t egp_predict_ws_bytes(int64_t nq, int64_t n, int32_t d, int32_t r);
int egp_block_lanczos(const float* X, int64_t n, const egp_hyper_t* h, const float* B0, int32_t b, int32_t blocks,
                      float* Q, double* T, int32_t* rows, void* ws, size_t ws_bytes, void* stream);
size_t egp_block_lanczos_ws_bytes(int64_t n, int32_t d, int32_t b, int32_t blocks);
int egp_predict_dense(const float* Xq, int64_t nq, const float* X, int64_t n, const egp_hyper_t* h, const float* a,
                      const float* Q, int32_t r, const double* T, int32_t ldt, float* mean, float* var, void* ws,
                      size_t ws_bytes, void* stream);

/* Z = P^{-1} R with P = L L^T + noise*I through the Woodbury identity, R and Z device n x t.
 * Exposed so that probe vectors and trace terms can be formed outside the solver. Asynchronous. */
int egp_precond_apply(const egp_precond_t* P, int64_t n, float noise, const float* R, int32_t t,
                      float* Z, void* ws, size_t ws_bytes, void* stream);
size_t egp_precond_apply_ws_bytes(int64_t n, int32_t t, int32_t rank);

/* Arithmetic of the fused kernel: the process-wide default that a call takes when its options do not name a mode
 * (initially EGP_KMM_FP32). A call reads it once at its entry. Every mode gives bit-reproducible results.
 *   EGP_KMM_FP32        fp32 MFMA throughout: the reference mode, the one every reported fp32 figure uses. In a
 *                       square product (egp_kmm, the solver, Lanczos, the likelihood) with n >= 32257 the symmetry
 *                       of the kernel matrix is exploited (paper, Background: K is a covariance matrix): every tile
 *                       off the block diagonal is formed once and used for both the row-side and the column-side
 *                       output. The column-side sums travel between workgroups as 64-bit fixed-point atomic adds,
 *                       which commute exactly, so the order of the adds does not show in the result (one unit is
 *                       2^-61 of the column's sum of |V|: far below the fp32 rounding of the sums themselves). This covers
 *                       d <= 355, groups of 1, 16 or 17 columns (1: d <= 31) and, up to d = 31, of 32 or 33 columns
 *                       (33: d <= 11); every other shape forms every tile (the kernels of EGP_KMM_FP32_ONE_SIDED).
 *   EGP_KMM_SPLIT_BF16  the kernel entries and V are each split into a high and a low bf16 part and
 *                       contracted as k_hi v_hi + k_hi v_lo + k_lo v_hi on the bf16 MFMA with fp32 accumulation
 *                       (16 significant bits per factor); distances and the transform stay in fp32. Faster,
 *                       because the bf16 MFMA co-executes with the transform's VALU work on this chip; its
 *                       error and speed are reported separately from the fp32 figures.
 *   EGP_KMM_SPLIT_BF16_ALL  additionally the distance step: scaled points are carried as three bf16 parts
 *                       (24 significant bits, exact) and the six products above the fp32 rounding level are
 *                       accumulated in fp32 on the bf16 MFMA. Faster again; also reported separately.
 *   EGP_KMM_FP32_ONE_SIDED  fp32 arithmetic with every tile formed in every product (no use of the symmetry): the
 *                       same results as EGP_KMM_FP32 up to summation order, 1.1x to 1.7x slower on large square
 *                       products; kept for comparison and measurement.
 * Affects egp_kmm, egp_kmm_cross, egp_mbcg, egp_lanczos, egp_mll. Returns EGP_ERR_ARG for an unknown mode. */
typedef enum { EGP_KMM_FP32 = 0, EGP_KMM_SPLIT_BF16 = 1, EGP_KMM_SPLIT_BF16_ALL = 2, EGP_KMM_FP32_ONE_SIDED = 3 } egp_kmm_mode_t;
int egp_set_kmm_mode(int32_t mode);
int egp_get_kmm_mode(void);
int egp_set_mbcg_shrink(int32_t on);      /* process-wide default of column shrinking, see egp_mbcg; returns EGP_OK */
int egp_get_mbcg_shrink(void);

/* Host-only self-check of the launch planning, for tests; touches no GPU. The fused kernel cuts the column points
 * into splits whose partial sums sit in the workspace before a deterministic reduction. For a product with
 * n_rows x n_cols kernel entries and t right-hand sides in the current default mode, used[0] (host) receives the largest
 * split count any of its launches takes and sized[0] (host) the count the workspace of egp_kmm_ws_bytes /
 * egp_kmm_cross_ws_bytes holds; used <= sized always (a launch that would break this returns EGP_ERR_WS instead of
 * running). Returns 0, or EGP_ERR_ARG for sizes outside the library's limits or null outputs. */
int egp_kmm_plan_splits(int64_t n_rows, int64_t n_cols, int32_t d, int32_t t, int32_t* used, int32_t* sized);
/* The same for the mode named in opts (NULL or kmm_mode = -1: the process default), read once like in every call. */
int egp_kmm_plan_splits_ex(int64_t n_rows, int64_t n_cols, int32_t d, int32_t t, const egp_call_opts_t* opts,
                           int32_t* used, int32_t* sized);

/* In-stream timing of kernel groups with HIP events, for roofline reporting. While enabled, each launch
 * of a group is bracketed by an event pair on the stream it runs on. egp_profile_enable(1) clears the
 * counters; egp_profile_read waits for the recorded events, and returns the summed duration and the
 * number of brackets of one group. Groups: */
typedef enum {
  EGP_PROF_KMM = 0,      /* the fused kernel-matrix-multiply kernel alone */
  EGP_PROF_PACK = 1,     /* row preparation, right-hand-side packing, split reduction / epilogue */
  EGP_PROF_CG_VEC = 2,   /* CG vector kernels (dot, update, direction) of one iteration */
  EGP_PROF_PRECOND = 3,  /* one application of P^{-1} */
  EGP_PROF_PIVCHOL = 4,  /* all steps of one pivoted-Cholesky build */
  EGP_PROF_GRAD = 5      /* the fused derivative kernel alone */
} egp_prof_group_t;
int egp_profile_enable(int on);
int egp_profile_read(int32_t group, double* total_ms /*host*/, int64_t* launches /*host*/);

/* Measurement aid: dst[0..count) = src[0..count) with one plain copy kernel (count a multiple of 4).
 * Reads and writes exactly 4*count bytes each; used to calibrate hardware HBM-traffic counters. */
int egp_calib_copy(const float* src /*device*/, float* dst /*device*/, int64_t count, void* stream);

/* egp_kmm for callers that cannot allocate device memory or provide a workspace: code under HIP graph capture,
 * tight serving loops, harnesses that forbid hipMalloc. Same product, same kernels, same bits as egp_kmm in the
 * process-default mode; the workspace is a device array built into the library (EGP_NOALLOC_SCRATCH_BYTES per GPU the
 * library runs on, held until the process ends). The call allocates and frees nothing on the device.
 *   - sizes whose egp_kmm_ws_bytes(n, d, t) exceeds EGP_NOALLOC_SCRATCH_BYTES return EGP_ERR_ARG (for d = 11, t = 17
 *     that is n up to 146944; for d = 18, t = 17 up to 95744); use egp_kmm with a workspace beyond that;
 *   - every call on a GPU shares that GPU's array: calls that overlap in time on one GPU (different streams or
 *     threads) race; calls on one stream are ordered and safe. What the kernels need at zero is cleared by the call;
 *   - the first call on a device looks up the array's address (hipGetSymbolAddress); make one call outside a
 *     capture before capturing;
 *   - keep profiling (egp_profile_enable) off around it: event brackets are host-side allocations.
 * Asynchronous on `stream`. */
#define EGP_NOALLOC_SCRATCH_BYTES (128u << 20)
int egp_kmm_noalloc(const float* X /*device n x d*/, int64_t n, const float* V /*device n x t*/, int32_t t,
                    const egp_hyper_t* h /*host*/, float* out /*device n x t*/, void* stream);

/* Message of the last failing call on this thread ("" if none). */
const char* egp_last_error(void);

/* Library version, "major.minor". */
const char* egp_version(void);

#ifdef __cplusplus
}
#endif
#endif /* EGP_H */
