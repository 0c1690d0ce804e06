// Subset-of-regressors (SGPR) covariance for gfx950 (CDNA4): K_hat = Q + sigma^2 I with
// Q = K_XU K_UU^{-1} K_UX (Sec. 5, "Programmability", sparse GP regression paragraph).
//
// Once per call the library forms the root  A = K_XU G^{-T}  (n x m), K_UU + jitter I = G G^T,
// so that Q = A A^T exactly and no K_UU solve is left inside the iteration:
//   * k_kuu_f64, k_chol_panel / k_chol_update, k_trinv_diag / k_trinv_off: K_UU, its Cholesky
//     factor and G^{-1}, all fp64 (m x m is small);
//   * k_kux_f64: K_UX in fp64 from the raw inputs;
//   * k_sgpr_root: A^T = G^{-1} K_UX by fp64 MFMA, rounded ONCE to fp32 (rows of A have norm
//     sqrt(Q_ii) <= sqrt(s), so the rounding perturbs Q by ~1e-7 s, like an fp32 kernel matrix);
//   * k_root_transpose: A from A^T (both layouts are streamed once per iteration; A^T is kept in
//     column panels of 512 points so that its 1024 long rows do not cost a memory page each).
// Derivative terms (Eq. (4),(8) with the derivative of the SoR matrix): dQ = dK_XU Kinv K_UX +
// (its transpose) - K_XU Kinv dK_UU Kinv K_UX, so u^T dQ w needs b_u = Kinv K_UX u = G^{-T} A^T u
// and b_w likewise (m-vectors, k_sgpr_bsolve) and then two sums over pairs, (X, U) and (U, U),
// of the lengthscale derivative of the kernel against rank-one weights (k_dk_rect).
// Per iteration the product Q D = A (A^T D) is two launches of the materialised streaming
// product (k_mm_mat) on the two layouts, with k_sgpr_mid between them.  The pivoted Cholesky of Q
// (App. C: a row of an SoR matrix costs O(nm)) gets its diagonal from k_sgpr_qdiag and each
// pivot row from one more streaming product, prepared by k_sgpr_pick.
#include "bbmm_dev.h"
#include "bbmm_kfun.h"

#include <math.h>

namespace {

typedef double f64x4 __attribute__((ext_vector_type(4)));

// fp64 MFMA 16x16x4: A[m = lane%16][k = lane/16], B[k = lane/16][n = lane%16]; register r of the
// result holds D[m = 4*r + lane/16][n = lane%16].
__device__ inline f64x4 mfma16d(double a, double b, f64x4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

__device__ inline size_t d4_index(int i, int q, int ld) {
  return (size_t)(i >> 2) * (size_t)(4 * ld) + (size_t)q * 4 + (size_t)(i & 3);
}

__device__ inline int perm16(int q) { return (q & ~15) | ((q & 3) << 2) | ((q >> 2) & 3); }

// k(a, b) in fp64 from two raw input rows (Sec. 2 notation).
__device__ inline double kernel_f64(const float* __restrict__ pa, const float* __restrict__ pb,
                                    const HypArgs& hyp) {
  double rho2 = 0.0;
  for (int dim = 0; dim < hyp.d; ++dim) {
    double df = ((double)pa[dim] - (double)pb[dim]) * hyp.inv_ls[dim];
    rho2 += df * df;
  }
  if (hyp.kernel == 0) return hyp.outputscale * exp(-0.5 * rho2);
  double rho = sqrt(rho2);
  const double s5 = 2.23606797749978969;
  return hyp.outputscale * (1.0 + s5 * rho + (5.0 / 3.0) * rho2) * exp(-s5 * rho);
}

// ------------------------------------------------------------ K_UU, fp64 -----
// KUU (mp x mp): kernel values plus jitter on the diagonal; the padding is the identity, so the
// factor and its inverse are well defined on the whole padded matrix.
__global__ void k_kuu_f64(const float* __restrict__ Uind, int m, int mp, HypArgs hyp, double jitter,
                          double* __restrict__ KUU) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)mp * mp) return;
  int a = (int)(idx / mp), b = (int)(idx % mp);
  double v = 0.0;
  if (a < m && b < m) {
    v = kernel_f64(Uind + (size_t)a * hyp.d, Uind + (size_t)b * hyp.d, hyp);
    if (a == b) v += jitter;
  } else if (a == b) {
    v = 1.0;
  }
  KUU[idx] = v;
}

// ------------------------------------------------ blocked Cholesky, fp64 -----
// Right-looking, panels of CH_NB columns.  Panel kernel: every block factors the diagonal block
// in LDS (it is tiny) and solves its own 256 rows below it; block 0 stores the diagonal block.
// A is read, G (zero-filled beforehand) is written, so blocks never read what others write.
constexpr int CH_NB = 32;

__global__ __launch_bounds__(256) void k_chol_panel(const double* __restrict__ A,
                                                     double* __restrict__ G, int mp, int j0,
                                                     double tiny, DevState* st) {
  __shared__ double D[CH_NB][CH_NB + 1];
  int tid = threadIdx.x;
  for (int e = tid; e < CH_NB * CH_NB; e += 256) {
    int r = e / CH_NB, c = e % CH_NB;
    D[r][c] = A[(size_t)(j0 + r) * mp + j0 + c];
  }
  __syncthreads();
  for (int c = 0; c < CH_NB; ++c) {
    double piv = D[c][c];
    __syncthreads();
    if (!(piv > tiny)) {   // a pivot at rounding level: the matrix is numerically singular
      if (blockIdx.x == 0 && tid == 0) st->status = 3;   // BBMM_ENOTPD
      piv = 1.0;
    }
    double root = sqrt(piv);
    if (tid < CH_NB && tid >= c) D[tid][c] = (tid == c) ? root : D[tid][c] / root;
    __syncthreads();
    for (int e = tid; e < CH_NB * CH_NB; e += 256) {
      int r = e / CH_NB, cc = e % CH_NB;
      if (cc > c && r >= cc) D[r][cc] -= D[r][c] * D[cc][c];
    }
    __syncthreads();
  }
  if (blockIdx.x == 0)
    for (int e = tid; e < CH_NB * CH_NB; e += 256) {
      int r = e / CH_NB, c = e % CH_NB;
      if (c <= r) G[(size_t)(j0 + r) * mp + j0 + c] = D[r][c];
    }
  // rows below the diagonal block: x G11^T = A[i, panel]
  int i = j0 + CH_NB + blockIdx.x * 256 + tid;
  if (i >= mp) return;
  double x[CH_NB];
#pragma unroll
  for (int c = 0; c < CH_NB; ++c) x[c] = A[(size_t)i * mp + j0 + c];
#pragma unroll
  for (int c = 0; c < CH_NB; ++c) {
    double v = x[c];
#pragma unroll
    for (int k = 0; k < c; ++k) v -= x[k] * D[c][k];
    x[c] = v / D[c][c];
  }
#pragma unroll
  for (int c = 0; c < CH_NB; ++c) G[(size_t)i * mp + j0 + c] = x[c];
}

// Trailing update A[i][j] -= sum_k G[i][j0+k] G[j][j0+k] on the lower triangle behind the panel;
// one block per 32 x 32 tile (tiles above the diagonal return at once).
__global__ __launch_bounds__(256) void k_chol_update(double* __restrict__ A,
                                                      const double* __restrict__ G, int mp, int j0) {
  int ti = blockIdx.y, tj = blockIdx.x;
  if (tj > ti) return;
  __shared__ double Gi[CH_NB][CH_NB + 1], Gj[CH_NB][CH_NB + 1];
  int base = j0 + CH_NB;
  int tid = threadIdx.x;
  for (int e = tid; e < CH_NB * CH_NB; e += 256) {
    int r = e / CH_NB, k = e % CH_NB;
    Gi[r][k] = G[(size_t)(base + ti * CH_NB + r) * mp + j0 + k];
    Gj[r][k] = G[(size_t)(base + tj * CH_NB + r) * mp + j0 + k];
  }
  __syncthreads();
  int c = tid % CH_NB;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    int r = tid / CH_NB + 8 * u;
    double acc = 0.0;
#pragma unroll
    for (int k = 0; k < CH_NB; ++k) acc += Gi[r][k] * Gj[c][k];
    A[(size_t)(base + ti * CH_NB + r) * mp + base + tj * CH_NB + c] -= acc;
  }
}

// ---------------------------------------- inverse of the lower factor, fp64 --
// Diagonal blocks: X_II = G_II^{-1}; thread c solves G_II x = e_c in registers.
__global__ __launch_bounds__(CH_NB) void k_trinv_diag(const double* __restrict__ G,
                                                       double* __restrict__ X, int mp) {
  __shared__ double D[CH_NB][CH_NB + 1];
  int I = blockIdx.x, c = threadIdx.x;
  for (int r = 0; r < CH_NB; ++r) D[r][c] = G[(size_t)(I * CH_NB + r) * mp + I * CH_NB + c];
  __syncthreads();
  double x[CH_NB];
#pragma unroll
  for (int r = 0; r < CH_NB; ++r) {
    double v = (r == c) ? 1.0 : 0.0;
#pragma unroll
    for (int k = 0; k < r; ++k) v -= D[r][k] * x[k];
    x[r] = v / D[r][r];
  }
#pragma unroll
  for (int r = 0; r < CH_NB; ++r) X[(size_t)(I * CH_NB + r) * mp + I * CH_NB + c] = (r >= c) ? x[r] : 0.0;
}

// Blocks below the diagonal, one workgroup per block column J, top to bottom:
//   X_IJ = - X_II ( sum_{K = J}^{I-1} G_IK X_KJ ).
// The X_KJ blocks are the workgroup's own earlier results, read back from global memory after a
// barrier.
__global__ __launch_bounds__(256) void k_trinv_off(const double* __restrict__ G, double* X, int mp) {
  __shared__ double sG[CH_NB][CH_NB + 1], sX[CH_NB][CH_NB + 1];
  int J = blockIdx.x, nblk = mp / CH_NB;
  int tid = threadIdx.x, c = tid % CH_NB, r0 = tid / CH_NB;
  for (int I = J + 1; I < nblk; ++I) {
    double acc[4] = {0.0, 0.0, 0.0, 0.0};
    for (int K = J; K < I; ++K) {
      for (int e = tid; e < CH_NB * CH_NB; e += 256) {
        int r = e / CH_NB, k = e % CH_NB;
        sG[r][k] = G[(size_t)(I * CH_NB + r) * mp + K * CH_NB + k];
        sX[r][k] = X[(size_t)(K * CH_NB + r) * mp + J * CH_NB + k];
      }
      __syncthreads();
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        int r = r0 + 8 * u;
#pragma unroll
        for (int k = 0; k < CH_NB; ++k) acc[u] += sG[r][k] * sX[k][c];
      }
      __syncthreads();
    }
    // S -> sX, X_II -> sG, then X_IJ = -X_II S
#pragma unroll
    for (int u = 0; u < 4; ++u) sX[r0 + 8 * u][c] = acc[u];
    for (int e = tid; e < CH_NB * CH_NB; e += 256) {
      int r = e / CH_NB, k = e % CH_NB;
      sG[r][k] = X[(size_t)(I * CH_NB + r) * mp + I * CH_NB + k];
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int r = r0 + 8 * u;
      double v = 0.0;
#pragma unroll
      for (int k = 0; k < CH_NB; ++k) v += sG[r][k] * sX[k][c];
      X[(size_t)(I * CH_NB + r) * mp + J * CH_NB + c] = -v;
    }
    __threadfence_block();
    __syncthreads();
  }
}

// G^{-1} in the order the root kernel feeds its MFMAs: GinvP[row / 16][col / 4][(col % 4) * 16 + row % 16]
__global__ void k_pack_ginv(const double* __restrict__ Ginv, int mp, double* __restrict__ GinvP) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)mp * mp) return;
  int lane = (int)(idx & 63);
  size_t blk = idx >> 6;
  int ks = (int)(blk % (mp / 4)), rt = (int)(blk / (mp / 4));
  int row = rt * 16 + (lane & 15), col = ks * 4 + (lane >> 4);
  GinvP[idx] = Ginv[(size_t)row * mp + col];
}

// ---------------------------------------------------------- K_UX, fp64 -------
// K_UX in fp64: k(u_b, x_i), b < m, i < n; zero for padding points.  Stored in panels of 128
// points, and inside a panel in the order the root kernel feeds its MFMAs,
//   Kux[panel][b / 4][(i % 128) / 16][(b % 4) * 16 + i % 16],
// so that every MFMA operand of the root kernel is 512 contiguous bytes.  Thread = one point, a run of KUX_RUN inducing inputs (their
// coordinates are uniform across the wave).
constexpr int KUX_RUN = 16;

template <int DP>
__global__ __launch_bounds__(256) void k_kux_f64(const float* __restrict__ X,
                                                  const float* __restrict__ Uind, int n, int mp,
                                                  int m, HypArgs hyp, double* __restrict__ Kux) {
  int i = blockIdx.x * 256 + threadIdx.x;
  double* panel = Kux + (size_t)(i >> 7) * mp * 128 + ((i & 127) >> 4) * 64 + (i & 15);
  int b0 = blockIdx.y * KUX_RUN;
  double xi[DP];
#pragma unroll
  for (int dim = 0; dim < DP; ++dim)
    xi[dim] = (i < n && dim < hyp.d) ? (double)X[(size_t)i * hyp.d + dim] * hyp.inv_ls[dim] : 0.0;
  const double s5 = 2.23606797749978969;
  for (int b = b0; b < min(m, b0 + KUX_RUN); ++b) {
    double rho2 = 0.0;
#pragma unroll
    for (int dim = 0; dim < DP; ++dim) {
      double ub = (dim < hyp.d) ? (double)Uind[(size_t)b * hyp.d + dim] * hyp.inv_ls[dim] : 0.0;
      double df = xi[dim] - ub;
      rho2 += df * df;
    }
    double v;
    if (hyp.kernel == 0) {
      v = hyp.outputscale * exp(-0.5 * rho2);
    } else {
      double rho = sqrt(rho2);
      v = hyp.outputscale * (1.0 + s5 * rho + (5.0 / 3.0) * rho2) * exp(-s5 * rho);
    }
    panel[(size_t)(b >> 2) * 512 + (b & 3) * 16] = (i < n) ? v : 0.0;
  }
}

// ------------------------------------------------- root: A^T = G^{-1} K_UX ---
// fp64 MFMA product without LDS and without barriers.  Both operands lie in MFMA operand order in
// global memory (k_pack_ginv, k_kux_f64), so every operand is one 512-byte coalesced load.
// Workgroup: NW waves, 32 NW rows of A^T (inducing index a) x 128 points; wave w owns row tiles
// w and 2 NW - 1 - w (16 rows each) x 8 point tiles = 16 accumulators, reads its own G^{-1}
// operands, and shares the K_UX operands with the other waves through L1.  Operands are requested
// PF k steps ahead of their MFMAs.
//
// G^{-1} is lower triangular: a row block contracts over the columns up to its own end only, and
// inside the diagonal block row tile t needs the 16-column chunks 0..t only (pairing tiles w and
// 2 NW - 1 - w gives every wave the same share).  So work differs 4 : 1 between the last and the
// first row block, while the hardware deals consecutive workgroups round-robin to the 8 XCDs:
// with (row block, panel) = (id % nrb, id / nrb) one XCD gets all the longest workgroups (measured:
// compute units busy 55 % of the launch).  The flat id is decoded as XCD x = id % 8, sequence
// j = id / 8 on that XCD; every XCD takes the panels x, x + 8, ... and walks them once per row
// block, longest block first, so that at any time an XCD works on ONE row block and its slab of
// G^{-1} (at most 2 MB) stays in that XCD's L2.  (Walking all row blocks of a panel first instead
// keeps the K_UX panel hot but has every workgroup pull a different slab of the 8 MB G^{-1}
// through the fabric: 12.3 ms against 10.4.)
//
// History at n = 500,000, m = 1024: operands gathered straight from row-major global memory
// 35.8 ms (address units saturated: 16 cache lines per G^{-1} operand) -> LDS staging 19.1 ->
// XCD-balanced 14.0 -> operands pre-packed 12.6 -> zero tiles of the diagonal block skipped 12.3
// -> row-block-major order 10.7 -> no LDS, 8 waves per workgroup 10.4 ms (51 TFLOP/s fp64).
constexpr int RT_PTS = 128;

template <int PF, int NW>
__global__ __launch_bounds__(64 * NW, 2) void k_sgpr_root(const double* __restrict__ GinvP,
                                                                  const double* __restrict__ Kux,
                                                                  int mp, int np,
                                                                  float* __restrict__ AT) {
  constexpr int ROWS = 32 * NW;
  int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  int g = lane >> 4, jc = lane & 15;
  int nrb = mp / ROWS;
  int xcd = blockIdx.x & 7, seq = blockIdx.x >> 3;
  int ppx = (np / RT_PTS + 7) / 8;                 // panels per XCD
  int panel = (seq % ppx) * 8 + xcd;
  if (panel >= np / RT_PTS) return;
  int a_blk = (nrb - 1 - seq / ppx) * ROWS;
  int i0 = panel * RT_PTS;
  int nsteps = min(mp, a_blk + ROWS) / 4;          // k steps of 4
  int dstep = a_blk / 4;                           // first k step of the diagonal block
  int tile[2] = {wave, 2 * NW - 1 - wave};
  f64x4 acc[2][8];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) acc[rt][ct] = (f64x4){0.0, 0.0, 0.0, 0.0};
  const double* pa[2];
#pragma unroll
  for (int rt = 0; rt < 2; ++rt) pa[rt] = GinvP + ((size_t)(a_blk / 16 + tile[rt]) * (mp / 4)) * 64 + lane;
  const double* pb = Kux + (size_t)panel * mp * RT_PTS + lane;
  double av[PF][2], bv[PF][8];
#pragma unroll
  for (int p = 0; p < PF; ++p) {
    int ks = min(p, nsteps - 1);
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) av[p][rt] = pa[rt][(size_t)ks * 64];
#pragma unroll
    for (int ct = 0; ct < 8; ++ct) bv[p][ct] = pb[((size_t)ks * 8 + ct) * 64];
  }
  for (int ks0 = 0; ks0 < nsteps; ks0 += PF) {
#pragma unroll
    for (int p = 0; p < PF; ++p) {
      int ks = ks0 + p;
      double ac[2], bc[8];
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) ac[rt] = av[p][rt];
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) bc[ct] = bv[p][ct];
      int kn = min(ks + PF, nsteps - 1);
#pragma unroll
      for (int rt = 0; rt < 2; ++rt) av[p][rt] = pa[rt][(size_t)kn * 64];
#pragma unroll
      for (int ct = 0; ct < 8; ++ct) bv[p][ct] = pb[((size_t)kn * 8 + ct) * 64];
      int cd = (ks - dstep) >> 2;                  // chunk of 16 inside the diagonal block
      if (cd <= tile[0]) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) acc[0][ct] = mfma16d(ac[0], bc[ct], acc[0][ct]);
      }
      if (cd <= tile[1]) {
#pragma unroll
        for (int ct = 0; ct < 8; ++ct) acc[1][ct] = mfma16d(ac[1], bc[ct], acc[1][ct]);
      }
    }
  }
#pragma unroll
  for (int rt = 0; rt < 2; ++rt)
#pragma unroll
    for (int ct = 0; ct < 8; ++ct)
#pragma unroll
      for (int r = 0; r < 4; ++r)
        AT[((size_t)(i0 / BBMM_SGPR_PANEL) * mp + (size_t)(a_blk + tile[rt] * 16 + 4 * r + g)) * BBMM_SGPR_PANEL +
           (size_t)(i0 % BBMM_SGPR_PANEL + ct * 16 + jc)] = (float)acc[rt][ct][r];
}

// A (np x mp, row-major) from A^T stored in column panels of BBMM_SGPR_PANEL points.
__global__ __launch_bounds__(256) void k_root_transpose(const float* __restrict__ ATp, int mp,
                                                         float* __restrict__ A) {
  __shared__ float tile[64][65];
  int a0 = blockIdx.y * 64, i0 = blockIdx.x * 64;
  int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
  const float* src = ATp + (size_t)(i0 / BBMM_SGPR_PANEL) * mp * BBMM_SGPR_PANEL + i0 % BBMM_SGPR_PANEL;
  for (int r = ty; r < 64; r += 4) tile[r][tx] = src[(size_t)(a0 + r) * BBMM_SGPR_PANEL + tx];
  __syncthreads();
  for (int c = ty; c < 64; c += 4) A[(size_t)(i0 + c) * mp + a0 + tx] = tile[tx][c];
}

// qdiag[i] = sum_a A[i][a]^2 in fp64 (the diagonal of Q = A A^T as the iteration sees it);
// one wave per row.
__global__ __launch_bounds__(256) void k_sgpr_qdiag(const float* __restrict__ A, int n, int mp,
                                                     double* __restrict__ qdiag) {
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int i = blockIdx.x * 4 + wave;
  if (i >= n) return;
  const float* row = A + (size_t)i * mp;
  double acc = 0.0;
  for (int a = lane * 4; a < mp; a += 256) {
    float4 v = *(const float4*)(row + a);
    acc += (double)v.x * v.x + (double)v.y * v.y + (double)v.z * v.z + (double)v.w * v.w;
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
  if (lane == 0) qdiag[i] = acc;
}

// T4 (quad-swizzled, mp rows, ld columns) = sum over the partial results of A^T D left by the
// streaming product (slot-major, column q at position perm16(q); shape.nseg[a / seg_cols] slots
// for row a).
__global__ void k_sgpr_mid(const double* __restrict__ Tp, VpShape shape, int mp, int ld,
                           const DevState* __restrict__ st, double* __restrict__ T4) {
  if (st->done) return;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)mp * ld) return;
  int a = (int)(idx / ld), pq = (int)(idx % ld);
  int nslot = shape.nseg ? shape.nseg[a / shape.seg_cols] : shape.nsplit;
  size_t stride = (size_t)mp * ld;
  double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
  int sl = 0;
  for (; sl + 3 < nslot; sl += 4) {
    s0 += Tp[(size_t)sl * stride + idx];
    s1 += Tp[(size_t)(sl + 1) * stride + idx];
    s2 += Tp[(size_t)(sl + 2) * stride + idx];
    s3 += Tp[(size_t)(sl + 3) * stride + idx];
  }
  for (; sl < nslot; ++sl) s0 += Tp[(size_t)sl * stride + idx];
  // position pq of a row holds column perm16(pq) (the permutation is an involution)
  T4[d4_index(a, perm16(pq), ld)] = (s0 + s1) + (s2 + s3);
}

// Row-major copy of the same sums (mp x ld, column order restored), for the derivative terms.
__global__ void k_sgpr_mid_rows(const double* __restrict__ Tp, VpShape shape, int mp, int ld,
                                double* __restrict__ T) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)mp * ld) return;
  int a = (int)(idx / ld), pq = (int)(idx % ld);
  int nslot = shape.nseg ? shape.nseg[a / shape.seg_cols] : shape.nsplit;
  size_t stride = (size_t)mp * ld;
  double s = 0.0;
  for (int sl = 0; sl < nslot; ++sl) s += Tp[(size_t)sl * stride + idx];
  T[(size_t)a * ld + perm16(pq)] = s;
}

// Right-hand side of the product that yields row `piv` of Q: column 0 = row piv of A, the other
// columns zero.  The pivot is the argmax of the candidates left by the previous pivoted-Cholesky
// kernel (lowest index on ties), found again here by every block.
__global__ __launch_bounds__(256) void k_sgpr_pick(const float* __restrict__ A, int mp,
                                                    const double* __restrict__ arg_in, int npart,
                                                    double* __restrict__ T4, int forced) {
  __shared__ double sval[256];
  __shared__ int sidx[256];
  double v = -1.0e300;
  int ix = 0x7fffffff;
  for (int b = threadIdx.x; b < npart; b += 256) {
    double v2 = arg_in[2 * b];
    int i2 = (int)arg_in[2 * b + 1];
    if (v2 > v || (v2 == v && i2 < ix)) {
      v = v2;
      ix = i2;
    }
  }
  sval[threadIdx.x] = v;
  sidx[threadIdx.x] = ix;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      double v2 = sval[threadIdx.x + w];
      int i2 = sidx[threadIdx.x + w];
      if (v2 > sval[threadIdx.x] || (v2 == sval[threadIdx.x] && i2 < sidx[threadIdx.x])) {
        sval[threadIdx.x] = v2;
        sidx[threadIdx.x] = i2;
      }
    }
    __syncthreads();
  }
  int piv = (forced >= 0) ? forced : sidx[0];
  int a = blockIdx.x * 256 + threadIdx.x;
  if (a >= mp) return;
  // an empty candidate list (every diagonal entry already picked) leaves no valid pivot
  double val = (piv >= 0 && piv != 0x7fffffff) ? (double)A[(size_t)piv * mp + a] : 0.0;
  for (int q = 0; q < 16; ++q) T4[d4_index(a, q, 16)] = (q == 0) ? val : 0.0;
}


// ------------------------------------------------------- derivative terms ----
// padded row-major fp64 block (stride ld) -> quad-swizzled right-hand side, zero beyond row n
__global__ void k_rows_to_d4(const double* __restrict__ src, int n, int np, int ld,
                             double* __restrict__ D4) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)np * ld) return;
  int i = (int)(idx / ld), q = (int)(idx % ld);
  D4[d4_index(i, q, ld)] = (i < n) ? src[idx] : 0.0;
}

// forward: B = G^{-1} T,  B[a][q] = sum_{b <= a} Ginv[a][b] T[b][q]   (mp x ld, row-major)
__global__ void k_sgpr_fsolve(const double* __restrict__ Ginv, const double* __restrict__ T, int mp,
                              int ld, double* __restrict__ B) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)mp * ld) return;
  int q = (int)(idx % ld), a = (int)(idx / ld);
  double s0 = 0.0, s1 = 0.0;
  int b = 0;
  for (; b + 1 <= a; b += 2) {
    s0 += Ginv[(size_t)a * mp + b] * T[(size_t)b * ld + q];
    s1 += Ginv[(size_t)a * mp + b + 1] * T[(size_t)(b + 1) * ld + q];
  }
  if (b <= a) s0 += Ginv[(size_t)a * mp + b] * T[(size_t)b * ld + q];
  B[idx] = s0 + s1;
}

// out[q] = sum_a V[a][q]^2, q < ld (one block; V is mp x ld)
__global__ __launch_bounds__(256) void k_colnorm2(const double* __restrict__ V, int mp, int ld,
                                                   double* __restrict__ out) {
  __shared__ double red[256];
  int q = threadIdx.x % ld, part = threadIdx.x / ld, parts = 256 / ld;
  double acc = 0.0;
  for (int a = part; a < mp; a += parts) {
    double v = V[(size_t)a * ld + q];
    acc += v * v;
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  if (part == 0) {
    double s = 0.0;
    for (int pp = 0; pp < parts; ++pp) s += red[pp * ld + q];
    out[q] = s;
  }
}

// var[a] = prior[a] - sum_i B[i][a] U[i][a]  (one block per column a, fixed-order fp64 block sum)
__global__ __launch_bounds__(256) void k_coldot_var(const double* __restrict__ B,
                                                     const double* __restrict__ U, int n, int ld,
                                                     const double* __restrict__ prior,
                                                     float* __restrict__ var) {
  __shared__ double red[256];
  int a = blockIdx.x;
  double acc = 0.0;
  for (int i = threadIdx.x; i < n; i += 256) acc += B[(size_t)i * ld + a] * U[(size_t)i * ld + a];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) var[a] = (float)(prior[a] - red[0]);
}

// B = G^{-T} T:  B[a][q] = sum_{b >= a} Ginv[b][a] T[b][q]   (mp x ld, row-major)
__global__ void k_sgpr_bsolve(const double* __restrict__ Ginv, const double* __restrict__ T, int mp,
                              int ld, double* __restrict__ B) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)mp * ld) return;
  int a = (int)(idx % mp), q = (int)(idx / mp);
  double s0 = 0.0, s1 = 0.0;
  int b = a;
  for (; b + 1 < mp; b += 2) {
    s0 += Ginv[(size_t)b * mp + a] * T[(size_t)b * ld + q];
    s1 += Ginv[(size_t)(b + 1) * mp + a] * T[(size_t)(b + 1) * ld + q];
  }
  if (b < mp) s0 += Ginv[(size_t)b * mp + a] * T[(size_t)b * ld + q];
  B[(size_t)a * ld + q] = s0 + s1;
}

// Outputscale terms: dQ/ds = Q / s = A A^T / s (the jitter scales with s), so
//   trace = (1/(t s)) sum_i (A^T u_i).(A^T w_i),  quad = |A^T u_0|^2 / s.   One block.
__global__ __launch_bounds__(256) void k_sgpr_sterm(const double* __restrict__ TU,
                                                     const double* __restrict__ TW, int mp, int ld,
                                                     int t, double outputscale, int slot, DevState* st) {
  __shared__ double r1[256], r2[256];
  double tr = 0.0, qd = 0.0;
  for (int a = threadIdx.x; a < mp; a += 256) {
    const double* u = TU + (size_t)a * ld;
    const double* w = TW + (size_t)a * ld;
    for (int i = 1; i <= t; ++i) tr += u[i] * w[i];
    qd += u[0] * u[0];
  }
  r1[threadIdx.x] = tr;
  r2[threadIdx.x] = qd;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      r1[threadIdx.x] += r1[threadIdx.x + w];
      r2[threadIdx.x] += r2[threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    st->dk_out[2 * slot] = r1[0] / ((double)t * outputscale);
    st->dk_out[2 * slot + 1] = r2[0] / outputscale;
  }
}

// Rank-one weights of the two pair sums, as fp32 operand rows of NT entries (zero padded):
//   pairs (x_i, u_a):  S_ia = PR_i . PC_a,  PR_i = [u_i1..u_it, w_i1..w_it] / t,  PC_a = [bw_a1.., bu_a1..]
//                      q_ia = (2 u_i0) (bu_a0)
//   pairs (u_a, u_b):  PR_a = [-bu_a1..-bu_at, 0..] / t,  PC_b = [bw_b1..bw_bt, 0..],  q_ab = (-bu_a0)(bu_b0)
__global__ void k_sgpr_dk_ops_x(const double* __restrict__ U, const double* __restrict__ Z0, int n,
                                int np, int ld, int t, int NT, float* __restrict__ PR,
                                float* __restrict__ qr) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)np * NT) return;
  int i = (int)(idx / NT), c = (int)(idx % NT);
  double v = 0.0;
  if (i < n) {
    if (c < t) v = U[(size_t)i * ld + 1 + c] / (double)t;
    else if (c < 2 * t) v = Z0[(size_t)i * ld + 1 + (c - t)] / (double)t;
  }
  PR[idx] = (float)v;
  if (c == 0) qr[i] = (i < n) ? (float)(2.0 * U[(size_t)i * ld]) : 0.f;
}

__global__ void k_sgpr_dk_ops_u(const double* __restrict__ BU, const double* __restrict__ BW, int m,
                                int mp, int ld, int t, int NT, float* __restrict__ PCx,
                                float* __restrict__ qcx, float* __restrict__ PRu,
                                float* __restrict__ qru, float* __restrict__ PCu) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)mp * NT) return;
  int a = (int)(idx / NT), c = (int)(idx % NT);
  double pcx = 0.0, pru = 0.0, pcu = 0.0;
  if (a < m) {
    if (c < t) {
      pcx = BW[(size_t)a * ld + 1 + c];
      pru = -BU[(size_t)a * ld + 1 + c] / (double)t;
      pcu = BW[(size_t)a * ld + 1 + c];
    } else if (c < 2 * t) {
      pcx = BU[(size_t)a * ld + 1 + (c - t)];
    }
  }
  PCx[idx] = (float)pcx;
  PRu[idx] = (float)pru;
  PCu[idx] = (float)pcu;
  if (c == 0) {
    float b0 = (a < m) ? (float)BU[(size_t)a * ld] : 0.f;
    qcx[a] = b0;       // also the column factor of the (U, U) quad term
    qru[a] = -b0;
  }
}

// sum over pairs (row i, column a) of  g(rho_ia) * Delta_h^2 * S_ia  (and * q_ia), Delta in the
// scaled coordinates, per lengthscale slot h (one slot when isotropic: sum over the dimensions).
// Thread = one row against a chunk of DKR_COLS columns staged in LDS; fp32 inside the chunk,
// fp64 block sum; one partial row of `pstride` doubles per block: [2h] trace-type, [2h+1] quad-type.
constexpr int DKR_COLS = 128;

template <int DP, int NT, int ARD>
__global__ __launch_bounds__(256) void k_dk_rect(int kind, const float* __restrict__ Xr,
                                                  const float* __restrict__ Xc,
                                                  const float* __restrict__ PR,
                                                  const float* __restrict__ qr,
                                                  const float* __restrict__ PC,
                                                  const float* __restrict__ qc, int nrows_p,
                                                  int ncols, double* __restrict__ partial,
                                                  int pstride) {
  __shared__ float sc[DKR_COLS][DP];
  __shared__ float spc[DKR_COLS][NT];
  __shared__ float sqc[DKR_COLS];
  __shared__ double red[4][2 * (ARD ? DP : 1)];
  constexpr int NL = ARD ? DP : 1;
  int tid = threadIdx.x;
  int i = blockIdx.x * 256 + tid;
  int a0 = blockIdx.y * DKR_COLS;
  int na = min(DKR_COLS, ncols - a0);
  for (int e = tid; e < DKR_COLS * DP; e += 256) {
    int a = e / DP, dim = e % DP;
    sc[a][dim] = (a < na) ? Xc[(size_t)(a0 + a) * DP + dim] : 0.f;
  }
  for (int e = tid; e < DKR_COLS * NT; e += 256) {
    int a = e / NT, cidx = e % NT;
    spc[a][cidx] = (a < na) ? PC[(size_t)(a0 + a) * NT + cidx] : 0.f;
  }
  if (tid < DKR_COLS) sqc[tid] = (tid < na) ? qc[a0 + tid] : 0.f;
  float xi[DP], pr[NT];
  bool live = i < nrows_p;
#pragma unroll
  for (int dim = 0; dim < DP; ++dim) xi[dim] = live ? Xr[(size_t)i * DP + dim] : 0.f;
#pragma unroll
  for (int cidx = 0; cidx < NT; ++cidx) pr[cidx] = live ? PR[(size_t)i * NT + cidx] : 0.f;
  float qri = live ? qr[i] : 0.f;
  float atr[NL], aq[NL];
#pragma unroll
  for (int h = 0; h < NL; ++h) {
    atr[h] = 0.f;
    aq[h] = 0.f;
  }
  __syncthreads();
  for (int a = 0; a < na; ++a) {
    float d2[DP];
    float r2 = 0.f;
#pragma unroll
    for (int dim = 0; dim < DP; ++dim) {
      float df = xi[dim] - sc[a][dim];
      d2[dim] = df * df;
      r2 += d2[dim];
    }
    float e, gw;
    if (kind == 0) unit_kernel_and_weight<0>(r2, e, gw);
    else unit_kernel_and_weight<1>(r2, e, gw);
    float S = 0.f;
#pragma unroll
    for (int cidx = 0; cidx < NT; ++cidx) S = fmaf(pr[cidx], spc[a][cidx], S);
    float ws = gw * S, wq = gw * (qri * sqc[a]);
    if (ARD) {
#pragma unroll
      for (int h = 0; h < NL; ++h) {
        atr[h] = fmaf(ws, d2[h], atr[h]);
        aq[h] = fmaf(wq, d2[h], aq[h]);
      }
    } else {
      atr[0] = fmaf(ws, r2, atr[0]);
      aq[0] = fmaf(wq, r2, aq[0]);
    }
  }
  int lane = tid & 63, wave = tid >> 6;
#pragma unroll
  for (int h = 0; h < NL; ++h) {
    double v1 = (double)atr[h], v2 = (double)aq[h];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      v1 += __shfl_xor(v1, o, 64);
      v2 += __shfl_xor(v2, o, 64);
    }
    if (lane == 0) {
      red[wave][2 * h] = v1;
      red[wave][2 * h + 1] = v2;
    }
  }
  __syncthreads();
  double* pout = partial + (size_t)(blockIdx.y * gridDim.x + blockIdx.x) * pstride;
  if (tid < 2 * NL) pout[tid] = (red[0][tid] + red[1][tid]) + (red[2][tid] + red[3][tid]);
}

}  // namespace

// ------------------------------------------------------------------ launchers
void launch_sgpr_kuu(hipStream_t s, const float* Uind, int m, int mp, HypArgs hyp, double jitter,
                     double* KUU) {
  size_t total = (size_t)mp * mp;
  k_kuu_f64<<<(int)((total + 255) / 256), 256, 0, s>>>(Uind, m, mp, hyp, jitter, KUU);
}

// G = lower Cholesky factor of KUU (destroyed); G must be zero-filled by the caller.  A pivot
// <= tiny raises BBMM_ENOTPD in st->status.
void launch_sgpr_chol(hipStream_t s, double* KUU, double* G, int mp, double tiny, DevState* st) {
  for (int j0 = 0; j0 < mp; j0 += CH_NB) {
    int below = mp - j0 - CH_NB;
    int blocks = below > 0 ? (below + 255) / 256 : 1;
    k_chol_panel<<<blocks, 256, 0, s>>>(KUU, G, mp, j0, tiny, st);
    if (below > 0) {
      int T = below / CH_NB;
      k_chol_update<<<dim3(T, T), 256, 0, s>>>(KUU, G, mp, j0);
    }
  }
}

// Ginv = G^{-1} (lower triangular); Ginv must be zero-filled by the caller.
void launch_sgpr_trinv(hipStream_t s, const double* G, double* Ginv, int mp) {
  int nblk = mp / CH_NB;
  k_trinv_diag<<<nblk, CH_NB, 0, s>>>(G, Ginv, mp);
  if (nblk > 1) k_trinv_off<<<nblk - 1, 256, 0, s>>>(G, Ginv, mp);
}

// Kux: (np / 128) panels of mp x 128 doubles; rows m..mp-1 of every panel must be zero (the
// caller zero-fills the buffer when mp > m).
int launch_sgpr_kux(hipStream_t s, const float* X, const float* Uind, int n, int np, int m, int mp, int dp,
                    HypArgs hyp, double* Kux) {
  dim3 grid(np / 256, (m + KUX_RUN - 1) / KUX_RUN);
  switch (dp) {
    case 4: k_kux_f64<4><<<grid, 256, 0, s>>>(X, Uind, n, mp, m, hyp, Kux); break;
    case 8: k_kux_f64<8><<<grid, 256, 0, s>>>(X, Uind, n, mp, m, hyp, Kux); break;
    case 16: k_kux_f64<16><<<grid, 256, 0, s>>>(X, Uind, n, mp, m, hyp, Kux); break;
    case 32: k_kux_f64<32><<<grid, 256, 0, s>>>(X, Uind, n, mp, m, hyp, Kux); break;
    case 64: k_kux_f64<64><<<grid, 256, 0, s>>>(X, Uind, n, mp, m, hyp, Kux); break;
    default: return 1;
  }
  return 0;
}

// AT (mp x np, in column panels of BBMM_SGPR_PANEL points: ceil(np / panel) * mp * panel floats)
// = Ginv Kux in fp32; mp and np are multiples of 256.  GinvP: scratch of mp x mp
// doubles that receives G^{-1} in MFMA operand order.
void launch_sgpr_root(hipStream_t s, const double* Ginv, double* GinvP, const double* Kux, int mp, int np,
                      float* AT) {
  size_t total = (size_t)mp * mp;
  k_pack_ginv<<<(int)((total + 255) / 256), 256, 0, s>>>(Ginv, mp, GinvP);
  int panels = np / RT_PTS, nrb = mp / 256;        // 8 waves: 256 rows per workgroup
  int grid = ((panels + 7) / 8) * nrb * 8;
  k_sgpr_root<2, 8><<<grid, 512, 0, s>>>(GinvP, Kux, mp, np, AT);
}

void launch_root_transpose(hipStream_t s, const float* ATp, int mp, int np, float* A) {
  k_root_transpose<<<dim3(np / 64, mp / 64), 256, 0, s>>>(ATp, mp, A);
}

void launch_sgpr_qdiag(hipStream_t s, const float* A, int n, int mp, double* qdiag) {
  k_sgpr_qdiag<<<(n + 3) / 4, 256, 0, s>>>(A, n, mp, qdiag);
}

void launch_sgpr_mid(hipStream_t s, const double* Tp, VpShape shape, int mp, int ld, const DevState* st,
                     double* T4) {
  size_t total = (size_t)mp * ld;
  k_sgpr_mid<<<(int)((total + 255) / 256), 256, 0, s>>>(Tp, shape, mp, ld, st, T4);
}

void launch_sgpr_mid_rows(hipStream_t s, const double* Tp, VpShape shape, int mp, int ld, double* T) {
  size_t total = (size_t)mp * ld;
  k_sgpr_mid_rows<<<(int)((total + 255) / 256), 256, 0, s>>>(Tp, shape, mp, ld, T);
}

void launch_sgpr_pick(hipStream_t s, const float* A, int mp, const double* arg_in, int npart,
                      double* T4, int forced) {
  k_sgpr_pick<<<(mp + 255) / 256, 256, 0, s>>>(A, mp, arg_in, npart, T4, forced);
}

void launch_rows_to_d4(hipStream_t s, const double* src, int n, int np, int ld, double* D4) {
  size_t total = (size_t)np * ld;
  k_rows_to_d4<<<(int)((total + 255) / 256), 256, 0, s>>>(src, n, np, ld, D4);
}

void launch_sgpr_bsolve(hipStream_t s, const double* Ginv, const double* T, int mp, int ld, double* B) {
  size_t total = (size_t)mp * ld;
  k_sgpr_bsolve<<<(int)((total + 255) / 256), 256, 0, s>>>(Ginv, T, mp, ld, B);
}

void launch_sgpr_fsolve(hipStream_t s, const double* Ginv, const double* T, int mp, int ld, double* B) {
  size_t total = (size_t)mp * ld;
  k_sgpr_fsolve<<<(int)((total + 255) / 256), 256, 0, s>>>(Ginv, T, mp, ld, B);
}

void launch_colnorm2(hipStream_t s, const double* V, int mp, int ld, double* out) {
  k_colnorm2<<<1, 256, 0, s>>>(V, mp, ld, out);
}

void launch_coldot_var(hipStream_t s, const double* B, const double* U, int n, int ld, int ns,
                       const double* prior, float* var) {
  k_coldot_var<<<ns, 256, 0, s>>>(B, U, n, ld, prior, var);
}

void launch_sgpr_sterm(hipStream_t s, const double* TU, const double* TW, int mp, int ld, int t,
                       double outputscale, int slot, DevState* st) {
  k_sgpr_sterm<<<1, 256, 0, s>>>(TU, TW, mp, ld, t, outputscale, slot, st);
}

void launch_sgpr_dk_ops(hipStream_t s, const double* U, const double* Z0, const double* BU,
                        const double* BW, int n, int np, int m, int mp, int ld, int t, int NT, float* PR,
                        float* qr, float* PCx, float* qcx, float* PRu, float* qru, float* PCu) {
  size_t tx = (size_t)np * NT, tu = (size_t)mp * NT;
  k_sgpr_dk_ops_x<<<(int)((tx + 255) / 256), 256, 0, s>>>(U, Z0, n, np, ld, t, NT, PR, qr);
  k_sgpr_dk_ops_u<<<(int)((tu + 255) / 256), 256, 0, s>>>(BU, BW, m, mp, ld, t, NT, PCx, qcx, PRu, qru, PCu);
}

// One pair sum; returns the number of partial rows written (one per block), or -1 when the
// configuration is not supported.  nrows_p: padded row count (operand arrays hold that many rows).
int launch_dk_rect(hipStream_t s, int kernel, int dp, int NT, int ard, const float* Xr, const float* Xc,
                   const float* PR, const float* qr, const float* PC, const float* qc, int nrows_p,
                   int ncols, double* partial, int pstride) {
  dim3 grid((nrows_p + 255) / 256, (ncols + DKR_COLS - 1) / DKR_COLS);
#define RECT(D, N, A) \
  k_dk_rect<D, N, A><<<grid, 256, 0, s>>>(kernel, Xr, Xc, PR, qr, PC, qc, nrows_p, ncols, partial, pstride)
#define RECT_N(D, A)            \
  if (NT == 32) RECT(D, 32, A); \
  else if (NT == 64) RECT(D, 64, A); \
  else return -1
#define RECT_D(D)       \
  if (ard) {            \
    RECT_N(D, 1);       \
  } else {              \
    RECT_N(D, 0);       \
  }
  switch (dp) {
    case 4: RECT_D(4); break;
    case 8: RECT_D(8); break;
    case 16: RECT_D(16); break;
    case 32: RECT_D(32); break;
    default: return -1;
  }
#undef RECT_D
#undef RECT_N
#undef RECT
  return (int)(grid.x * grid.y);
}
