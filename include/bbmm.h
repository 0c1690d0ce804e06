/*
 * bbmm.h -- C ABI of the MI355X (gfx950) BBMM inference hot path.
 *
 * One call computes, for an exact Gaussian process with kernel matrix
 * K_hat = K_XX + sigma^2 I, the three quantities that dominate training
 * (paper Sec. 3, "Required operations"):
 *     K_hat^{-1} y,   log|K_hat|,   Tr(K_hat^{-1} dK_hat/dtheta),
 * through ONE run of preconditioned modified batched conjugate gradients
 * (mBCG, Alg. 2) on the right-hand-side block [y, z_1 .. z_t] (Eq. (3)),
 * with the rank-k pivoted-Cholesky preconditioner of Sec. 4.1 / App. C.
 *
 * Conventions
 *   - "device" pointers are HIP device memory on the context's GPU, "host"
 *     pointers are ordinary host memory.  All matrices are dense row-major.
 *   - The caller owns every buffer it passes; the library never frees them.
 *     bbmm_solve_logdet_grad uses them only until it returns; the stage-level
 *     entry points read the problem's device buffers (X, y, E1, E2, Uind,
 *     u0_init) again, so these must stay valid while the problem set by
 *     bbmm_setup is in use.
 *   - Work is queued on the context's HIP stream (bbmm_solve_logdet_grad and
 *     bbmm_sgpr_build also use a second stream of the context, joined back
 *     before they return).  A call
 *     that returns host values synchronises the stream once before it returns.
 *   - Precision: K_hat entries are fp32; inside the library every n x c block of
 *     the iteration, the pivoted-Cholesky factor and all sums are fp64.  float
 *     block arguments are converted on entry and rounded once on exit.
 *   - Every function returns an int status (BBMM_OK == 0).  No exceptions,
 *     no exit().  bbmm_last_error() gives a message for the last failure.
 *   - A context is not thread-safe; use one context per stream.
 *   - Hyperparameter order in every per-hyperparameter array:
 *         lengthscale(s) (1 or d entries), outputscale, noise (sigma^2);
 *     raw values, no log/softplus transform.
 *   - Limits: 1 <= t <= 31, 0 <= k <= 32, 1 <= d <= 64, max_iters <= 256;
 *     BBMM_MODE_SGPR: 1 <= m <= min(n, 4096), d <= 32.
 */
#ifndef BBMM_H
#define BBMM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct bbmm_ctx bbmm_ctx;

enum {
  BBMM_OK = 0,
  BBMM_EINVAL = 1,     /* bad shape, NULL pointer, limit exceeded, wrong call order */
  BBMM_ENOMEM = 2,     /* device allocation failed (e.g. materialised K_hat does not fit) */
  BBMM_ENOTPD = 3,     /* capacitance matrix (or K_UU + jitter I) not positive definite */
  BBMM_ENONFINITE = 4, /* a non-finite value reached a result */
  BBMM_EHIP = 5,       /* a HIP runtime call failed */
  BBMM_ENOCONV = 6     /* the tridiagonal eigen-solver did not reduce a matrix within its sweep budget */
};

enum { BBMM_KERNEL_RBF = 0, BBMM_KERNEL_MATERN52 = 1 };
enum { BBMM_MODE_MATERIALISED = 0, BBMM_MODE_ONTHEFLY = 1, BBMM_MODE_SGPR = 2 };

/*
 * Problem statement (Sec. 2 notation).
 *   kernel       RBF:       k = s exp(-|x-x'|^2 / (2 l^2))   (per-dimension l_d when ARD)
 *                MATERN52:  rho^2 = sum_d (x_d-x'_d)^2 / l_d^2,
 *                           k = s (1 + sqrt5 rho + 5 rho^2/3) exp(-sqrt5 rho)
 *   mode         how K_hat.M products are formed inside mBCG: from an fp32 K_hat
 *                stored in device memory (4 n^2 bytes, held by the context), or
 *                from X tile by tile without ever storing K_hat.
 *                BBMM_MODE_SGPR replaces the covariance itself by the subset-of-regressors
 *                form of Sec. 5 (sparse GP regression paragraph),
 *                    K_hat = K_XU K_UU^{-1} K_UX + sigma^2 I,
 *                with m inducing inputs Uind; K_UU gets jitter_rel * outputscale on its
 *                diagonal before it is factorised.  The library keeps the n x m root
 *                A = K_XU G^{-T} (K_UU = G G^T) in fp32 in both layouts (8 n m bytes) and
 *                forms products as A (A^T M).  Preconditioner, probes, mBCG, log-det and
 *                traces are those of the SoR matrix; the inducing inputs are fixed, not
 *                hyperparameters.  SGPR supports one shared lengthscale (n_lengthscale 1)
 *                or one per dimension, 1 <= m <= min(n, 4096), d <= 32.
 *   n, d         number of training points and input dimension
 *   t            number of probe vectors z_i (right-hand-side block has t+1 columns)
 *   k            rank of the pivoted-Cholesky preconditioner (0 = P = sigma^2 I)
 *   max_iters    mBCG iteration cap p
 *   tol          > 0: stop when |r_j|/|b| < tol for ALL columns; <= 0: run p iterations
 *   n_lengthscale 1 (isotropic) or d (ARD);  lengthscale: host array of that length
 *   X            device, n x d float
 *   y            device, n float
 *   E1           device, k x t float, entries +-1 (may be NULL when k == 0)
 *   E2           device, n x t float, entries +-1
 *                probes are z_i = L_k E1[:,i] + sigma E2[:,i]  (App. C, sampling from N(0,P))
 *   m, Uind, jitter_rel   BBMM_MODE_SGPR only (ignored otherwise): number of inducing inputs,
 *                device m x d float (coordinates of X), relative jitter >= 0
 *   pivots_in    host, k distinct row indices, or NULL.  NULL: the greedy rule of App. C (largest
 *                residual diagonal, lowest index on ties).  Otherwise the pivoted Cholesky takes
 *                these rows in this order.  The greedy order is not unique under rounding when
 *                residual diagonals tie (a stationary kernel's diagonal is constant; the inducing
 *                rows of an SoR matrix agree to ~1e-10), so a caller who needs the same
 *                preconditioner as another run or implementation passes that run's pivots.
 *   u0_init      device, n float, or NULL.  Alg. 1/2 take the current solution as input and start
 *                from r_0 = b - K_hat u_0; with u0_init the y column (column 0 of the block) starts
 *                from it, at the cost of one more product (e.g. the solve of the previous
 *                optimiser step).  The probe columns always start from zero: their Lanczos
 *                tridiagonals need r_0 = z_i.  Residuals stay relative to |b|.  Used by
 *                bbmm_solve_logdet_grad and bbmm_mbcg; the pointer must stay valid while the
 *                problem set by bbmm_setup is in use.
 */
typedef struct {
  int32_t kernel;
  int32_t mode;
  int64_t n, d, t, k, max_iters;
  double tol;
  int64_t n_lengthscale;
  const double* lengthscale;
  double outputscale;
  double noise;
  const float* X;
  const float* y;
  const float* E1;
  const float* E2;
  int64_t m;
  const float* Uind;
  double jitter_rel;
  const int64_t* pivots_in;
  const float* u0_init;
} bbmm_problem;

/*
 * Results.  Pointers are caller-allocated; optional ones may be NULL.
 *   u0             device, n float: K_hat^{-1} y after the last mBCG iteration (required)
 *   U              device, n x (t+1) float: all solves [u_0 .. u_t]           (optional)
 *   logdet         stochastic-Lanczos-quadrature estimate of log|K_hat| (Eq. (5),(7))
 *   logdet_precond log|P| from the matrix determinant lemma (App. C)
 *   yKinvy         y^T u_0
 *   nlml           1/2 (y^T u_0 + logdet + n log 2 pi)
 *   trace[h]       (1/t) sum_i u_i^T (dK_hat/dtheta_h) P^{-1} z_i      (Eq. (8))  host, H entries
 *   quad[h]        u_0^T (dK_hat/dtheta_h) u_0                                  host, H entries
 *   grad_nlml[h]   1/2 (trace[h] - quad[h])                                      host, H entries
 *                  H = n_lengthscale + 2
 *   iters_run      mBCG iterations executed
 *   rank           preconditioner rank actually built (< k only if the residual diagonal vanished)
 *   alpha, beta    host, max_iters x (t+1) doubles, row j = coefficients of iteration j (optional)
 *   resid          host, max_iters x (t+1): |r_j|/|b| per column                  (optional)
 *   pivots         host, k entries: pivot rows in the order chosen                (optional)
 *   slq_terms      host, t entries: (z_i^T P^{-1} z_i) e_1^T log(T_i) e_1         (optional)
 */
typedef struct {
  float* u0;
  float* U;
  double logdet;
  double logdet_precond;
  double yKinvy;
  double nlml;
  double* trace;
  double* quad;
  double* grad_nlml;
  int64_t iters_run;
  int64_t rank;
  double* alpha;
  double* beta;
  double* resid;
  int64_t* pivots;
  double* slq_terms;
} bbmm_result;

/* Create a context bound to GPU `device` and to `hip_stream` (a hipStream_t, NULL = default
 * stream).  Workspaces are allocated lazily and reused across calls. */
int bbmm_create(bbmm_ctx** out, int device, void* hip_stream);
int bbmm_destroy(bbmm_ctx* ctx);
const char* bbmm_last_error(const bbmm_ctx* ctx);

/* Tuning knobs for experiments (all have sensible defaults):
 *   "mat_wgs"    number of workgroups a materialised product is dealt out to (default: one per
 *                compute unit; for a block of at most 12 columns a whole number per column strip
 *                of K_hat close to that; clamped to [strips, 60 * strips], strips = column strips
 *                of K_hat)
 *   "otf_split"  number of row chunks an on-the-fly product is split into (with "otf_sym": number
 *                of workgroups of each of its two launches, default two per compute unit)
 *   "otf_sym"    1 (default): an on-the-fly product of at most 16 columns over at most 32 input
 *                dimensions and at least 12288 (padded) rows evaluates only the tiles on and above
 *                the diagonal and uses each for both of its contributions (K is symmetric);
 *                2: the same for any number of rows; 0: every tile is evaluated for the one
 *                contribution, as it is for wider blocks and inputs.  Same values, fp64 sums in
 *                another order
 *   "ur_blocks"  upper limit of the workgroups of the fused U/R update (default 128, at most 512)
 *   "khat_panel" layout of the materialised K_hat: column panels of that width (a multiple of
 *                256; default 1024), each panel row-major; 1 = plain row-major.  Takes effect at
 *                the next bbmm_build_khat
 *   "khat_sym"   1: BBMM_MODE_MATERIALISED keeps only the upper triangle of the symmetric K_hat
 *                (packed column panels of 1024: about half the memory and half the HBM bytes per
 *                product) and uses every tile for both of its contributions to K_hat M; the
 *                entries are the same fp32 values, the fp64 sums are formed in another order.
 *                0 (default): the whole matrix.  Takes effect at the next bbmm_build_khat (a
 *                change marks the stored matrix as not built); "khat_panel" is ignored while set;
 *                "mat_wgs" then counts the workgroups of each of its two launches.  A block of
 *                more than 16 columns takes one pass over the triangle per group of 16 columns
 *                (the whole-matrix product takes one pass for up to 32), so beyond 16 columns
 *                the whole matrix is the faster storage
 *   "zd_blocks"  workgroups per compute unit of the direction update (default 16, at most 64)
 *   "sgpr_wgs1", "sgpr_wgs2"  workgroups of the two streaming products of an SGPR product
 *                (A^T M, then A (.)); clamped like "mat_wgs"; takes effect at the next bbmm_sgpr_build
 *   "loop_graph" 1: the iteration loop of an mBCG run whose launch sequence equals that of an
 *                earlier run of this context (same sizes, mode, tuning values and buffers; the
 *                hyperparameters and the tolerance may differ, the loop's kernels read them from
 *                device memory) is replayed as one HIP graph, recorded at the second such run;
 *                0 (default): every kernel is launched on its own.  Same kernels, same results;
 *                it frees the calling thread earlier but the GPU time is the same (the chain of
 *                dependent kernels is bound by dispatch on the device).  Runs with "time_mm" set
 *                are never replayed
 *   "slq_eig"    how e_1^T log(T_i) e_1 of the log-det estimate is evaluated.  0 (default): by a
 *                trapezoid quadrature in ln s of int_0^inf [1/(1+s) - e_1^T (T_i + s I)^{-1} e_1] ds,
 *                the resolvent being a continued fraction (every node an independent chain of p
 *                divisions; exact to ~1e-15, no eigenvalues formed); 1: by the eigen-decomposition
 *                of T_i as App. B writes it (implicit-shift QR, one thread per probe: 0.7 ms at
 *                p = 50 against ~15 us).  The two agree to 1e-13 ... 2e-10 relative
 *   "eig_sweeps" trip budget of the tridiagonal eigen-solver per matrix row (sweeps and deflations;
 *                default 60, at most 1000; about two sweeps per eigenvalue are needed).  A matrix
 *                not reduced within it makes the call return BBMM_ENOCONV
 *   "time_mm"    1: record HIP events on the context's stream around every K_hat.M launch of
 *                the next mBCG runs (read back with bbmm_mm_timing); 0: off (default)
 * value <= 0 restores the default (for "khat_sym" and "otf_sym" the value is the setting itself).
 * Unknown key: BBMM_EINVAL. */
int bbmm_tune(bbmm_ctx* ctx, const char* key, int64_t value);

/* Duration of the K_hat.M launches of the last mBCG run, measured with HIP events on the
 * context's stream (needs bbmm_tune("time_mm", 1) before the run).  Only launches of iterations
 * that really executed are counted.  avg_ms, total_ms, launches: host (each optional). */
int bbmm_mm_timing(bbmm_ctx* ctx, double* avg_ms, double* total_ms, int64_t* launches);

/* How often this context has recorded the iteration loop of Alg. 2 as a HIP graph and how often
 * it has replayed one (see "loop_graph" above).  captures, replays: host, each optional. */
int bbmm_loop_graph_stats(bbmm_ctx* ctx, int64_t* captures, int64_t* replays);

/* The whole path (Sec. 3 + Sec. 4): preconditioner, probes, mBCG, log-det, traces. */
int bbmm_solve_logdet_grad(bbmm_ctx* ctx, const bbmm_problem* in, bbmm_result* out);

/* ------------------------------------------------------------------------
 * Stage-level entry points (same kernels as the full call; used for parity
 * tests and for profiling one stage in isolation).  bbmm_setup must be called
 * first; it validates the problem, sizes the workspaces and prepares the
 * scaled copies of X.  Stages that depend on earlier ones say so.
 * ---------------------------------------------------------------------- */
int bbmm_setup(bbmm_ctx* ctx, const bbmm_problem* in);

/* Materialise K_hat = K_XX + sigma^2 I in fp32 in the context (Sec. 2, notation). */
int bbmm_build_khat(bbmm_ctx* ctx);
/* Copy the block K_hat[row0:row0+nrows, col0:col0+ncols] to `out` (device, nrows x ncols). */
int bbmm_khat_block(bbmm_ctx* ctx, int64_t row0, int64_t nrows, int64_t col0, int64_t ncols,
                    float* out);

/* BBMM_MODE_SGPR: form the root A = K_XU G^{-T} of the subset-of-regressors matrix (Sec. 5) in
 * the context: K_UU and its Cholesky factor in fp64, A rounded once to fp32.  Must run before any
 * other SGPR stage. */
int bbmm_sgpr_build(bbmm_ctx* ctx);
/* Copy rows [row0, row0 + nrows) of the root A (n x m) to `out` (device, nrows x m float). */
int bbmm_sgpr_root_rows(bbmm_ctx* ctx, int64_t row0, int64_t nrows, float* out);

/* V = K_hat M, the product every mBCG iteration is built on (Sec. 3, "Runtime and space").
 * M, V: device n x c float, 1 <= c <= 32.  mode MATERIALISED needs bbmm_build_khat first, mode
 * SGPR bbmm_sgpr_build; an SGPR problem takes mode SGPR only, and no other problem does. */
int bbmm_kernel_mm(bbmm_ctx* ctx, int32_t mode, const float* M, int64_t c, float* V);

/* Rank-k pivoted Cholesky of K_XX (App. C; of the SoR matrix for an SGPR problem).  L: device n x k double, row-major (optional, NULL to
 * skip) -- the factor is built and kept in fp64, and this is that factor unrounded;
 * pivots: host k (optional), rank: host (optional). */
int bbmm_pivoted_cholesky(bbmm_ctx* ctx, double* L, int64_t* pivots, int64_t* rank);

/* Capacitance matrix C = sigma^2 I + L^T L, its Cholesky factor, and log|P| (App. C).
 * Needs bbmm_pivoted_cholesky.  logdet_precond: host. */
int bbmm_precond_setup(bbmm_ctx* ctx, double* logdet_precond);

/* Z = P^{-1} R by the Woodbury formula (App. C).  R, Z: device n x c float.
 * Needs bbmm_precond_setup. */
int bbmm_precond_solve(bbmm_ctx* ctx, const float* R, int64_t c, float* Z);

/* B = [y, L E1 + sigma E2] (Eq. (6); App. C).  B: device n x (t+1) float.
 * Needs bbmm_pivoted_cholesky. */
int bbmm_make_probes(bbmm_ctx* ctx, float* B);

/* mBCG (Alg. 2) on the block B (device n x c float) with the context's preconditioner.
 * U: device n x c float.  alpha/beta/resid: host max_iters x c doubles (optional).
 * Needs bbmm_precond_setup (and bbmm_build_khat for MATERIALISED). */
int bbmm_mbcg(bbmm_ctx* ctx, int32_t mode, const float* B, int64_t c, float* U,
              double* alpha, double* beta, double* resid, int64_t* iters_run);

/* Eigen-decomposition of `batch` symmetric tridiagonal matrices of size m <= 256
 * (App. B, log-det paragraph): diag is batch x m, off is batch x (m-1) (host).
 * eigvals: host batch x m (ascending not guaranteed), first_row: host batch x m,
 * first_row[b][i] = first component of the unit eigenvector of eigvals[b][i].
 * 1 <= batch <= 65535.  BBMM_ENOCONV when a matrix is not reduced within the sweep budget
 * ("eig_sweeps"); the outputs then hold the unfinished state and must not be used. */
int bbmm_tridiag_eig_batched(bbmm_ctx* ctx, const double* diag, const double* off, int64_t m,
                             int64_t batch, double* eigvals, double* first_row);

/* bbmm_tridiag_eig_batched for callers that cannot allocate device memory (code that must not
 * call hipMalloc: tight serving loops, harnesses that forbid it, code between the capture calls
 * of a HIP graph on another stream).  Same arguments, same kernel, same results; the device copies
 * of the batch live in a fixed work area inside the library (576 KB per GPU, held until the
 * process ends) instead of a buffer of the context, and the call makes no hipMalloc / hipFree.
 * Limit: batch * m <= 16384 (BBMM_EINVAL beyond it, with a message).  All calls on one GPU share
 * that work area -- from any context -- so calls that overlap in time on one GPU race; calls
 * issued one after the other (this entry point synchronises the context's stream before it
 * returns) are safe.  Nothing needs clearing between calls: every word read is written first. */
int bbmm_tridiag_eig_batched_noalloc(bbmm_ctx* ctx, const double* diag, const double* off, int64_t m,
                                     int64_t batch, double* eigvals, double* first_row);

/* log|K_hat| estimate from the coefficients of the LAST bbmm_mbcg run, whose block must have
 * been [y, z_1..z_t] (columns 1..t are used): log|P| + (1/t) sum_i rho0_i e_1^T log(T_i) e_1.
 * logdet: host; slq_terms: host t (optional). */
int bbmm_slq_logdet(bbmm_ctx* ctx, double* logdet, double* slq_terms);

/* The same estimate from coefficients the caller hands in (App. A, Observation: Lanczos
 * tridiagonals from the CG coefficients; App. B, log-det paragraph; Eq. (5),(7)):
 *   T_i[j][j] = 1/alpha_j + beta_(j-1)/alpha_(j-1),  T_i[j-1][j] = sqrt(beta_(j-1))/alpha_(j-1),
 *   logdet = logdet_precond + (1/t) sum_i rho0[i] e_1^T log(T_i) e_1.
 * alpha, beta: host p x t doubles, row j = iteration j, column i = probe i (probe columns only, no
 * y column); rho0: host t (z_i^T P^{-1} z_i); m_valid: host t, size of T_i (coefficients of
 * iterations >= m_valid[i] are ignored: a column frozen or stopped early), NULL = p for all;
 * 1 <= p <= 256, 1 <= t <= 31.  logdet: host; slq_terms: host t (either may be NULL, not both).
 * Needs no bbmm_setup.  BBMM_ENOCONV / BBMM_ENONFINITE as for bbmm_slq_logdet. */
int bbmm_slq_from_coeffs(bbmm_ctx* ctx, const double* alpha, const double* beta, const double* rho0,
                         const int64_t* m_valid, int64_t p, int64_t t, double logdet_precond,
                         double* logdet, double* slq_terms);

/* Derivative products (Eq. (8), App. B): with U = [u_0 .. u_t] (device n x (t+1)) and
 * W = [w_1 .. w_t] (device n x t, w_i = P^{-1} z_i):
 *   trace[h] = (1/t) sum_i u_i^T (dK_hat/dtheta_h) w_i,   quad[h] = u_0^T (dK_hat/dtheta_h) u_0.
 * trace, quad: host, n_lengthscale + 2 entries each. */
int bbmm_dk_traces(bbmm_ctx* ctx, const float* U, const float* W, double* trace, double* quad);

/* ------------------------------------------------------------------------
 * Predictive distribution at test inputs (Sec. 2, Eq. (1), zero prior mean).
 * Both need bbmm_setup (or a completed bbmm_solve_logdet_grad) for the same
 * training data and hyperparameters; Xstar is device memory, ns x d float,
 * in the coordinates of X.
 * For an SGPR problem every covariance is the subset-of-regressors one,
 * q(a, b) = k_{aU} K_UU^{-1} k_{Ub} (bbmm_sgpr_build must have run): mean = q_{x* X} u0,
 * var = q(x*, x*) - q_{x* X} K_hat^{-1} q_{X x*}.
 * ---------------------------------------------------------------------- */

/* mean[a] = k_{X x*_a}^T u0 with u0 = K_hat^{-1} y (device, n float; e.g. the u0 of
 * bbmm_solve_logdet_grad).  mean: device, ns float.  Kernel values in fp64 from X. */
int bbmm_predict_mean(bbmm_ctx* ctx, const float* Xstar, int64_t ns, const float* u0, float* mean);

/* var[a] = k(x*_a, x*_a) - k_{X x*_a}^T K_hat^{-1} k_{X x*_a} (latent function; add sigma^2 for
 * observations): one preconditioned mBCG run (Alg. 2) whose right-hand sides are the columns
 * k_{X x*_a}, with the context's preconditioner, iteration cap and tolerance.  1 <= ns <= 32 per
 * call.  var: device, ns float.  iters_run, max_resid (largest relative residual over the columns
 * at the last iteration): host, optional.  Needs bbmm_precond_setup (and bbmm_build_khat for
 * MATERIALISED); overwrites the solves and coefficient histories held in the context. */
int bbmm_predict_var(bbmm_ctx* ctx, int32_t mode, const float* Xstar, int64_t ns, float* var,
                     int64_t* iters_run, double* max_resid);

#ifdef __cplusplus
}
#endif
#endif /* BBMM_H */
