// Internal declarations shared by the kernel files and the host orchestrator.
// Not part of the public ABI (see include/bbmm.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#define BBMM_MAXC 32      // padded right-hand-side columns (ld of every n x c block is 16 or 32)
#define BBMM_MAXK 32      // preconditioner rank limit
#define BBMM_MAXD 64      // input dimension limit
#define BBMM_MAXP 256     // mBCG iteration limit
#define BBMM_VEC_THREADS 256

// Device-resident scalar state of one call.  Everything the iteration needs between
// kernels lives here so that the host never reads coefficients back inside the loop.
struct DevState {
  double rho[BBMM_MAXC];        // r^T P^{-1} r of the current residual, per column
  double rho0[BBMM_MAXC];       // b^T P^{-1} b (first rho), per column
  double bnorm[BBMM_MAXC];      // |b| per column
  double alpha_cur[BBMM_MAXC];
  double beta_cur[BBMM_MAXC];
  double dvtot[BBMM_MAXC];      // d^T K_hat d of the current iteration, per column
  double Qt[BBMM_MAXK * BBMM_MAXC];   // C^{-1} L^T R, [m][q]
  double G[BBMM_MAXK * BBMM_MAXK];    // lower Cholesky factor of C = sigma^2 I + L^T L, [a][b]
  double Ginv[BBMM_MAXK * BBMM_MAXK]; // G^{-1} (lower triangular, zero padded), [a][b]
  double logdetP;
  double pivdmax[BBMM_MAXK + 1];
  double slq_terms[BBMM_MAXC];
  double slq_mean;
  double dk_out[2 * (BBMM_MAXD + 3)];  // raw accumulators of the derivative pass
  double xmean[BBMM_MAXD];
  // scalars of the iteration loop (set once per mBCG run by launch_set_loop_scalars).  The loop's
  // kernels read them from here when they are handed a negative noise / diagonal term instead, so
  // that the launches of the loop do not depend on the hyperparameters and can be replayed as a graph.
  double loop_noise, loop_tol, loop_scaleV, loop_addD;
  int active[BBMM_MAXC];
  int m_valid[BBMM_MAXC];
  int piv[BBMM_MAXK + 1];
  int done;         // set when the tolerance test passed; later kernels of the loop exit at once
  int iters_run;
  int status;       // BBMM_* code raised on the device (0 = ok)
  int rank;         // preconditioner rank actually built
  unsigned counter[8][40];   // arrival tickets per kernel family: [0] final, [1 + g] group g
};

struct HypArgs {
  double inv_ls[BBMM_MAXD];   // 1 / l_d (isotropic: the same value d times)
  double xscale[BBMM_MAXD];   // factor applied to centred x_d in fp64; the product is rounded to fp32 once
  double outputscale;
  double noise;
  int kernel;
  int d;
};

// MmPiece / MmPlan (work of one workgroup of a streaming product) come from bbmm_plan.h.
#include "bbmm_plan.h"

// How the partial products in Vp are to be summed: `nsplit` slots for every row, or, when nseg is
// set, nseg[row / seg_cols] slots.
struct VpShape {
  int nsplit;
  const int* nseg;
  int seg_cols;
  int max_slots;   // host-side knowledge: the largest slot count of any row (0 = not known)
};

// ---- launchers implemented in kernels_vec.hip ---------------------------------------------
// n x c blocks (U, R, V, Z0, D4, Vp) and the factor L are fp64; kernel matrix and X copies are fp32.
void launch_fill_f64(hipStream_t s, double* p, size_t count, double v);
void launch_fill_bytes0(hipStream_t s, void* p, size_t bytes);
// several buffers zeroed by one launch: pointers and sizes in 4-byte words (all 4-byte aligned)
struct ZeroSegs {
  void* p[6];
  size_t words[6];
  int n;
};
void launch_fill_multi0(hipStream_t s, const ZeroSegs& z);
void launch_colmean(hipStream_t s, const float* X, int n, int d, DevState* st, double* partial,
                    double* gpartial);
void launch_prep_x(hipStream_t s, const float* X, int n, int d, int np, int KK, HypArgs hyp,
                   const DevState* st, float* Xa, float* Xb, float* Xs, float* X4, float* sq);
void launch_pack_d4(hipStream_t s, const float* M, int n, int c, int np, int ld, double* D4);
void launch_unpack_rows(hipStream_t s, const double* src, int ld, int n, int c, float* dst);
void launch_unpack_rows_f64(hipStream_t s, const double* src, int ld, int n, int c, double* dst);
void launch_pack_rows(hipStream_t s, const float* src, int n, int c, int ld, double* dst);
void launch_pack_cols_at(hipStream_t s, const float* src, int n, int c, int ld, int dstcol0, double* dst);
// tri: src is the packed upper triangle of a symmetric matrix (see launch_mm_sym)
void launch_copy_block(hipStream_t s, const float* src, size_t pw, size_t rows_p, int tri, int row0,
                       int nrows, int col0, int ncols, float* dst);
void launch_warm_rhs(hipStream_t s, const float* u_init, int n, int ld, double* D4);
void launch_warm_apply(hipStream_t s, const float* u_init, const double* V, int n, int ld, double* U,
                       double* R);
void launch_vreduce(hipStream_t s, const double* Vp, VpShape shape, int n, int np, int ld, double scaleV,
                    double addD, const double* D4, double* V);
// diag_in / row_in: NULL for a plain kernel matrix of X (constant diagonal, rows evaluated from X);
// otherwise the matrix diagonal (n) and, per step, the pivot's row at row_in[i * row_ld].
// forced / next_forced: -1 for the greedy rule; otherwise the pivot this step must take and the
// one the following step will take (a replayed pivot order).
void launch_pc_init(hipStream_t s, int n, HypArgs hyp, double* delta, DevState* st, double* arg_out,
                    int nblocks, const double* diag_in, int next_forced);
void launch_pc_step(hipStream_t s, const float* X, int n, int m, int kp, HypArgs hyp, double* delta,
                    double* L, DevState* st, const double* arg_in, double* arg_out, int nblocks,
                    const double* row_in, int row_ld, int forced, int next_forced);
void launch_pre_setup(hipStream_t s, const double* L, int n, int k, int kp, double noise, DevState* st,
                      double* partial, double* gpartial, int nblocks);
void launch_probes(hipStream_t s, const float* y, const float* E1, const float* E2, const double* L,
                   int n, int t, int kp, int ld, double noise, const DevState* st, double* R);
void launch_set_loop_scalars(hipStream_t s, DevState* st, double noise, double tol, double scaleV, double addD);
// launch_dv: addD < 0, launch_ur / launch_zd: noise < 0  =>  the scalars come from st->loop_*
void launch_dv(hipStream_t s, const double* Vp, VpShape shape, int n, int np, int ld, double scaleV,
               double addD, const double* D4, double* V, const DevState* st, double* partial_dv,
               int nblocks);
void launch_ur(hipStream_t s, int init, int n, int ld, int c, int kp, double noise, double tol,
               const double* D4, const double* V, double* U, double* R, const double* L, DevState* st,
               const double* partial_dv, int nb_dv, double* partial, int nb_ur, int iter,
               double* alpha_hist, double* beta_hist, double* resid_hist);
void launch_zd(hipStream_t s, int init, int n, int ld, int kp, double noise, const double* R,
               const double* L, double* D4, double* Z0, DevState* st, int nblocks);
void launch_psolve_apply(hipStream_t s, int n, int ld, int kp, double noise, const double* R,
                         const double* L, double* Z, DevState* st, int nblocks);
void launch_cross_block(hipStream_t s, const float* X, const float* Xs, int n, int ns, int ld, HypArgs hyp,
                        double* B);
void launch_cross_dot(hipStream_t s, const float* X, const float* Xs, int n, int ns, HypArgs hyp,
                      const double* V, int ldv, int percol, double prior, double sign, float* out);
// sweeps_per_row: trip budget of the tridiagonal eigen-solver per matrix row (sweeps and deflations;
// about two sweeps per eigenvalue are needed); a matrix that is not reduced within it is reported
// through st->status / status[] as BBMM_ENOCONV instead of being used.
// eig != 0: e_1^T log(T) e_1 through the eigen-decomposition of T (one thread per probe); 0: through
// a quadrature of the resolvent e_1^T (T + s I)^{-1} e_1 (all threads; no eigenvalues computed)
void launch_slq(hipStream_t s, const double* alpha_hist, const double* beta_hist, int t, int eig,
                int sweeps_per_row, DevState* st);
// alpha, beta: p x t row-major; rho0, m_valid: t entries; terms, status: t entries out
void launch_slq_coeffs(hipStream_t s, const double* alpha, const double* beta, const double* rho0,
                       const int* m_valid, int t, int eig, int sweeps_per_row, double* terms, int* status);
void launch_tridiag_eig(hipStream_t s, const double* diag, const double* off, int m, int batch,
                        int sweeps_per_row, double* eigvals, double* first_row, int* status);
void launch_noise_terms(hipStream_t s, const double* U, const double* Z0, const float* y, int n, int ld,
                        int t, int slot, DevState* st, double* partial, double* gpartial, int nblocks);

// ---- launchers implemented in kernels_sgpr.hip (subset-of-regressors covariance) ----------
void launch_sgpr_kuu(hipStream_t s, const float* Uind, int m, int mp, HypArgs hyp, double jitter,
                     double* KUU);
void launch_sgpr_chol(hipStream_t s, double* KUU, double* G, int mp, double tiny, DevState* st);
void launch_sgpr_trinv(hipStream_t s, const double* G, double* Ginv, int mp);
int launch_sgpr_kux(hipStream_t s, const float* X, const float* Uind, int n, int np, int m, int mp, int dp,
                    HypArgs hyp, double* Kux);
void launch_sgpr_root(hipStream_t s, const double* Ginv, double* GinvP, const double* Kux, int mp, int np,
                      float* AT);
void launch_root_transpose(hipStream_t s, const float* ATp, int mp, int np, float* A);
void launch_sgpr_qdiag(hipStream_t s, const float* A, int n, int mp, double* qdiag);
void launch_sgpr_mid(hipStream_t s, const double* Tp, VpShape shape, int mp, int ld, const DevState* st,
                     double* T4);
void launch_sgpr_mid_rows(hipStream_t s, const double* Tp, VpShape shape, int mp, int ld, double* T);
void launch_sgpr_pick(hipStream_t s, const float* A, int mp, const double* arg_in, int npart,
                      double* T4, int forced);

void launch_rows_to_d4(hipStream_t s, const double* src, int n, int np, int ld, double* D4);
void launch_sgpr_bsolve(hipStream_t s, const double* Ginv, const double* T, int mp, int ld, double* B);
void launch_sgpr_fsolve(hipStream_t s, const double* Ginv, const double* T, int mp, int ld, double* B);
void launch_colnorm2(hipStream_t s, const double* V, int mp, int ld, double* out);
void launch_coldot_var(hipStream_t s, const double* B, const double* U, int n, int ld, int ns,
                       const double* prior, float* var);
void launch_sgpr_sterm(hipStream_t s, const double* TU, const double* TW, int mp, int ld, int t,
                       double outputscale, int slot, DevState* st);
void launch_sgpr_dk_ops(hipStream_t s, const double* U, const double* Z0, const double* BU,
                        const double* BW, int n, int np, int m, int mp, int ld, int t, int NT, float* PR,
                        float* qr, float* PCx, float* qcx, float* PRu, float* qru, float* PCu);
int launch_dk_rect(hipStream_t s, int kernel, int dp, int NT, int ard, const float* Xr, const float* Xc,
                   const float* PR, const float* qr, const float* PC, const float* qc, int nrows_p,
                   int ncols, double* partial, int pstride);

// ---- launchers implemented in kernels_mm.hip ----------------------------------------------
// panel_width > 0: K_hat is written in column panels of that width (see launch_mm_mat); 0: row-major.
// tri: panel P keeps rows [0, (P+1) * panel_width) only and the panels are packed (see launch_mm_sym).
int launch_build_khat(hipStream_t s, int kernel, int KK, const float* Xa, const float* Xb,
                      const float* sq, int n, int np, int panel_width, int tri, double outputscale,
                      double noise, float* Khat);
// ---- launcher implemented in kernels_sym.hip ------------------------------------------------
// K_hat D from the upper triangle of K_hat stored in packed column panels of BBMM_SYM_PANEL columns
// (panel P: rows [0, min(np, (P+1) * BBMM_SYM_PANEL)), row-major, at float offset
// BBMM_SYM_PANEL^2 * P (P+1) / 2).  pieces: flat work list; first_dual / first_single: per workgroup
// of the launch over the rows above the diagonal blocks / inside them, the range of the list to run
// (wgs + 1 entries each).  slot_base[s]: first slot of output panel s that takes row-side sums.
#define BBMM_SYM_PANEL 1024
// cols: columns of the block really in use (a 16-column group with at most 12 of them takes a
// narrower MFMA on the column-side use).
int launch_mm_sym(hipStream_t s, const float* Ktri, const double* D4, double* Vp, int np, int ld, int cols,
                  const MmPiece* pieces, const int* first_dual, int wgs_dual, const int* first_single,
                  int wgs_single, const int* slot_base, const DevState* st);
// Streams the row-major fp32 matrix M (row stride = column count `np`, a multiple of 256) once and
// leaves partial sums of M^T D in Vp, D4 indexed by the rows of M.  For the symmetric K_hat that is
// K_hat D; the SGPR root uses it on both of its layouts.  plan: one entry per workgroup, laid out
// by the host (see make_plan).  panel_width > 0: M is stored in column panels of that width
// (a multiple of 256), each panel row-major with panel_rows rows; 0: plain row-major.
// cols: columns of the block really in use (0 = all ld of them): with at most 12 of 16 the product
// runs on the narrower fp64 MFMA and columns 12..15 of the result are written as zero.
int launch_mm_mat(hipStream_t s, const float* Khat, const double* D4, double* Vp, int np, int ld,
                  const MmPlan* plan, int wgs, const DevState* st, int panel_width, int panel_rows,
                  int cols);
#define BBMM_SGPR_PANEL 512   // column-panel width of the transposed SGPR root
// c: number of columns really used (<= ld); lets 17..20 columns run one MFMA group plus vector FMAs
int launch_mm_otf(hipStream_t s, int kernel, int KK, const float* Xa, const float* Xb, const float* sq,
                  const double* D4, double* Vp, int np, int ld, int c, int nsplit, const DevState* st);
// The same product with every pair of tiles (I, J), (J, I) evaluated once and used for both of its
// contributions; ld = 16 and KK <= 8 only (returns 1 otherwise).  Work lists as for launch_mm_sym, with
// panels of BBMM_OTF_PANEL columns.
#define BBMM_OTF_PANEL 512
int launch_mm_otf_tri(hipStream_t s, int kernel, int KK, const float* Xa, const float* Xb, const float* sq,
                      const double* D4, double* Vp, int np, int cols, const MmPiece* pieces,
                      const int* first_dual, int wgs_dual, const int* first_single, int wgs_single,
                      const int* slot_base, const DevState* st);
// derivative pass: one partial row (pstride doubles) per wave, then a fixed-order fp64 sum into
// st->dk_out.  Returns non-zero when the configuration is not supported.
int launch_dk(hipStream_t s, int kernel, int KK, int ard, int TS, const float* Xa, const float* Xb,
              const float* sq, const float* Xs, const float* X4, const float* SA, const float* SB,
              const float* u0, int np, int nsplit, double* partial, int pstride, int max_rows,
              DevState* st);
// dk_out[e] = fixed-order fp64 sum over the first `nrows` partial rows, e < nvalues
void launch_dk_finish(hipStream_t s, const double* partial, int nrows, int pstride, int nvalues,
                      DevState* st);
void launch_swizzle_cols(hipStream_t s, const double* src, int ld, int n, int np, int col0, int ncols,
                         int TS, int dstcol0, float scale, float* dst);
void launch_extract_col(hipStream_t s, const double* src, int ld, int n, int np, int col, float* dst);
