// O(n t) kernels of the BBMM path: input preparation, pivoted Cholesky (App. C),
// capacitance matrix / Woodbury solve (App. C), probe construction (App. C),
// the fused mBCG vector updates with all alpha/beta bookkeeping on the device
// (Alg. 2), and the batched tridiagonal eigen-solver for stochastic Lanczos
// quadrature (App. B).
//
// Reductions over rows use a deterministic two-stage scheme: every block writes
// fp64 partial sums, the block that finishes last adds them in a fixed order and
// does the small fp64 scalar algebra (alpha, beta, k x k solves), so no value is
// read back by the host inside the iteration.
#include "bbmm_dev.h"

#include <math.h>

#define VT BBMM_VEC_THREADS

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

// Returns true in every thread of exactly one block: the one that arrives last.
__device__ inline bool last_block_arrives(unsigned* counter) {
  __shared__ int is_last;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned ticket = atomicAdd(counter, 1u);
    is_last = (ticket == gridDim.x - 1);
  }
  __syncthreads();
  if (is_last) __threadfence();
  return is_last != 0;
}

__device__ inline bool finite_d(double x) { return x == x && fabs(x) < 1.0e300; }

// Column q of a product block sits at position perm16(q) of its row in the partial buffers:
// the fp64 MFMA accumulator holds rows 4*r + lane/16, so a lane's four values are the columns
// lane/16, 4 + lane/16, 8 + lane/16, 12 + lane/16, stored contiguously.
__device__ inline int perm16(int q) { return (q & ~15) | ((q & 3) << 2) | ((q >> 2) & 3); }

// Deterministic two-level sum of per-block partial vectors (the latency of a single block adding
// hundreds of partial rows one after the other would dominate these small kernels).
// Every block has written partial[blockIdx.x * stride + e], e < E.  Blocks are grouped by
// RGROUP: the last block of a group to arrive adds its group's rows into gpartial[group], the
// last group to finish adds the group rows into tot (LDS).  Returns true, in every thread, only
// in that final block.  counters: 1 + number of groups tickets, all zero on entry, reset on exit.
constexpr int RGROUP = 16;
__device__ inline bool reduce_blocks(const double* __restrict__ partial, double* __restrict__ gpartial,
                                     size_t stride, int E, unsigned* counters, double* tot) {
  __shared__ int flag;
  int nb = gridDim.x, ng = (nb + RGROUP - 1) / RGROUP;
  int grp = blockIdx.x / RGROUP;
  int gsize = min(RGROUP, nb - grp * RGROUP);
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) flag = (atomicAdd(&counters[1 + grp], 1u) == (unsigned)(gsize - 1));
  __syncthreads();
  if (!flag) return false;
  __threadfence();
  const double* base = partial + (size_t)grp * RGROUP * stride;
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    double v[RGROUP];
#pragma unroll
    for (int b = 0; b < RGROUP; ++b) v[b] = (b < gsize) ? base[(size_t)b * stride + e] : 0.0;
    double s = 0.0;
#pragma unroll
    for (int b = 0; b < RGROUP; ++b) s += v[b];
    gpartial[(size_t)grp * stride + e] = s;
  }
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) flag = (atomicAdd(&counters[0], 1u) == (unsigned)(ng - 1));
  __syncthreads();
  if (!flag) return false;
  __threadfence();
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    int g = 0;
    for (; g + 3 < ng; g += 4) {
      s0 += gpartial[(size_t)g * stride + e];
      s1 += gpartial[(size_t)(g + 1) * stride + e];
      s2 += gpartial[(size_t)(g + 2) * stride + e];
      s3 += gpartial[(size_t)(g + 3) * stride + e];
    }
    for (; g < ng; ++g) s0 += gpartial[(size_t)g * stride + e];
    tot[e] = (s0 + s1) + (s2 + s3);
  }
  __syncthreads();
  if ((int)threadIdx.x <= ng) counters[threadIdx.x] = 0u;
  return true;
}

// ------------------------------------------------------------------ fills ----
__global__ void k_fill_f64(double* p, size_t count, double v) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) p[i] = v;
}

__global__ void k_fill_u32(unsigned* p, size_t count) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < count; i += stride) p[i] = 0u;
}

// Zeroes up to six buffers in one launch (sizes in 4-byte words): a launch costs several
// microseconds whatever it does, which is what a call on a small problem consists of.
__global__ void k_fill_multi0(ZeroSegs z) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
#pragma unroll 1
  for (int k = 0; k < z.n; ++k) {
    unsigned* p = (unsigned*)z.p[k];
    for (size_t j = i; j < z.words[k]; j += stride) p[j] = 0u;
  }
}

// ------------------------------------------------------- input preparation ---
// Column means of X (fp64): per-block partial sums, last block finishes.
__global__ __launch_bounds__(VT) void k_colmean(const float* __restrict__ X, int n, int d,
                                                 DevState* st, double* partial, double* gpartial) {
  __shared__ double red[VT];
  __shared__ double tot[BBMM_MAXD];
  // thread -> (row slot, dim): consecutive threads read consecutive floats of X
  size_t total = (size_t)n * d;
  size_t start = (size_t)blockIdx.x * VT + threadIdx.x;
  size_t stride = (size_t)gridDim.x * VT;
  // stride is kept a multiple of d so that a thread always sees the same dimension
  int dim = (int)(start % d);
  double acc = 0.0;
  for (size_t e = start; e < total; e += stride) acc += (double)X[e];
  for (int dd = 0; dd < d; ++dd) {
    red[threadIdx.x] = (dim == dd) ? acc : 0.0;
    __syncthreads();
    for (int w = VT / 2; w > 0; w >>= 1) {
      if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
      __syncthreads();
    }
    if (threadIdx.x == 0) partial[(size_t)blockIdx.x * BBMM_MAXD + dd] = red[0];
    __syncthreads();
  }
  if (!reduce_blocks(partial, gpartial, BBMM_MAXD, d, st->counter[5], tot)) return;
  if ((int)threadIdx.x < d) st->xmean[threadIdx.x] = tot[threadIdx.x] / (double)n;
}

// Scaled, centred copies of X in the layouts the tile kernels read:
//   Xb[(b*KK + kk)*64 + l] = xs[16 b + l%16][4 kk + l/16]          (MFMA operand order)
//   Xa = -2 * Xb
//   Xs[i*dp + dim]  (row-major),  X4[(i/4)*4*dp + dim*4 + i%4]  (quad-swizzled)
//   sq[i] = sum_dim xs^2
// with xs[i][dim] = (X[i][dim] - mean[dim]) * xscale[dim], zero for padding rows / dims.
__global__ void k_prep_x(const float* __restrict__ X, int n, int d, int np, int KK, HypArgs hyp,
                         const DevState* __restrict__ st, float* __restrict__ Xa,
                         float* __restrict__ Xb, float* __restrict__ Xs, float* __restrict__ X4,
                         float* __restrict__ sq) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= np) return;
  int dp = 4 * KK;
  float acc = 0.f;
  int b = i >> 4, r16 = i & 15;
  for (int dim = 0; dim < dp; ++dim) {
    float v = 0.f;
    if (i < n && dim < d) v = (float)(((double)X[(size_t)i * d + dim] - st->xmean[dim]) * hyp.xscale[dim]);
    int kk = dim >> 2, g = dim & 3;
    size_t sw = ((size_t)b * KK + kk) * 64 + (size_t)(g * 16 + r16);
    Xb[sw] = v;
    Xa[sw] = -2.f * v;
    Xs[(size_t)i * dp + dim] = v;
    X4[(size_t)(i >> 2) * (size_t)(4 * dp) + (size_t)dim * 4 + (i & 3)] = v;
    acc = fmaf(v, v, acc);
  }
  sq[i] = acc;
}

// Row-major n x c (stride c) -> quad-swizzled D4 with np rows and ld columns, zero padded.
__global__ void k_pack_d4(const float* __restrict__ M, int n, int c, int np, int ld,
                          double* __restrict__ D4) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t total = (size_t)np * ld;
  if (idx >= total) return;
  int i = (int)(idx / ld), q = (int)(idx % ld);
  double v = (i < n && q < c) ? (double)M[(size_t)i * c + q] : 0.0;
  D4[d4_index(i, q, ld)] = v;
}

// padded row-major (stride ld) -> dense n x c
__global__ void k_unpack_rows(const double* __restrict__ src, int ld, int n, int c,
                              float* __restrict__ dst) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * c) return;
  int i = (int)(idx / c), q = (int)(idx % c);
  dst[idx] = (float)src[(size_t)i * ld + q];
}

// padded fp64 rows (stride ld) -> dense n x c fp64 (used for the Cholesky factor)
__global__ void k_unpack_rows_f64(const double* __restrict__ src, int ld, int n, int c,
                                  double* __restrict__ dst) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * c) return;
  int i = (int)(idx / c), q = (int)(idx % c);
  dst[idx] = src[(size_t)i * ld + q];
}

// dense n x c -> padded row-major (stride ld), padding columns zero
__global__ void k_pack_rows(const float* __restrict__ src, int n, int c, int ld,
                            double* __restrict__ dst) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * ld) return;
  int i = (int)(idx / ld), q = (int)(idx % ld);
  dst[idx] = (q < c) ? (double)src[(size_t)i * c + q] : 0.0;
}

// dense n x c written into columns dstcol0.. of a padded row-major block (other columns untouched)
__global__ void k_pack_cols_at(const float* __restrict__ src, int n, int c, int ld, int dstcol0,
                               double* __restrict__ dst) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * c) return;
  int i = (int)(idx / c), q = (int)(idx % c);
  dst[(size_t)i * ld + dstcol0 + q] = (double)src[idx];
}

// dst (nrows x ncols, dense) = src[row0:row0+nrows, col0:col0+ncols]; src is stored in column
// panels of width pw, each row-major with rows_p rows (pw = row length: plain row-major).
// tri: packed upper triangle of a symmetric matrix, panel P keeping rows [0, (P+1) pw) only; an
// element below that is read at its mirror position.
__global__ void k_copy_block(const float* __restrict__ src, size_t pw, size_t rows_p, int tri, int row0,
                             int nrows, int col0, int ncols, float* __restrict__ dst) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)nrows * ncols) return;
  int i = (int)(idx / ncols), j = (int)(idx % ncols);
  size_t row = (size_t)(row0 + i), col = (size_t)(col0 + j);
  if (tri) {
    if (row >= (col / pw + 1) * pw) {
      size_t t = row;
      row = col;
      col = t;
    }
    size_t P = col / pw;
    dst[idx] = src[pw * pw * (P * (P + 1) / 2) + row * pw + col % pw];
  } else {
    dst[idx] = src[(col / pw) * rows_p * pw + row * pw + col % pw];
  }
}

// V = scaleV * sum_s Vp[s] + addD * D  (no dot product; used by the stand-alone product call)
__global__ void k_vreduce(const double* __restrict__ Vp, VpShape shape, int n, int np, int ld,
                          double scaleV, double addD, const double* __restrict__ D4,
                          double* __restrict__ V) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * ld) return;
  int i = (int)(idx / ld), q = (int)(idx % ld);
  size_t pidx = (size_t)i * ld + perm16(q);
  int nsplit = shape.nseg ? shape.nseg[i / shape.seg_cols] : shape.nsplit;
  double s = 0.0;
  for (int sp = 0; sp < nsplit; ++sp) s += Vp[(size_t)sp * np * ld + pidx];
  V[idx] = scaleV * s + addD * D4[d4_index(i, q, ld)];
}

// Warm start of column 0 (Alg. 1/2 take the current solution as input): the quad-swizzled
// right-hand side gets u_init in column 0 (the rest of the block was zero-filled) ...
__global__ void k_warm_rhs(const float* __restrict__ u_init, int n, int ld, double* __restrict__ D4) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) D4[d4_index(i, 0, ld)] = (double)u_init[i];
}

// ... and with V = K_hat [u_init, 0, ..] the iteration starts from U[:,0] = u_init, R[:,0] = b - V[:,0].
__global__ void k_warm_apply(const float* __restrict__ u_init, const double* __restrict__ V, int n,
                             int ld, double* __restrict__ U, double* __restrict__ R) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n) return;
  U[(size_t)i * ld] = (double)u_init[i];
  R[(size_t)i * ld] -= V[(size_t)i * ld];
}

// ------------------------------------------------------- pivoted Cholesky ----
__device__ inline double kernel_value_f64(const float* __restrict__ X, int a, int b,
                                          const HypArgs& hyp) {
  double rho2 = 0.0;
  for (int dim = 0; dim < hyp.d; ++dim) {
    double df = ((double)X[(size_t)a * hyp.d + dim] - (double)X[(size_t)b * hyp.d + dim]) *
                hyp.inv_ls[dim];
    rho2 += df * df;
  }
  if (hyp.kernel == 0) return hyp.outputscale * exp(-0.5 * rho2);
  double rho = sqrt(rho2);
  const double s5 = 2.23606797749978969;
  return hyp.outputscale * (1.0 + s5 * rho + (5.0 / 3.0) * rho2) * exp(-s5 * rho);
}

// Block-level argmax of (value, lowest index on ties); result valid in thread 0.
__device__ inline void block_argmax(double v, int idx, double* sval, int* sidx, double* outv,
                                    int* outi) {
  sval[threadIdx.x] = v;
  sidx[threadIdx.x] = idx;
  __syncthreads();
  for (int w = blockDim.x / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      double v2 = sval[threadIdx.x + w];
      int i2 = sidx[threadIdx.x + w];
      double v1 = sval[threadIdx.x];
      int i1 = sidx[threadIdx.x];
      if (v2 > v1 || (v2 == v1 && i2 < i1)) {
        sval[threadIdx.x] = v2;
        sidx[threadIdx.x] = i2;
      }
    }
    __syncthreads();
  }
  *outv = sval[0];
  *outi = sidx[0];
  __syncthreads();
}

// Argmax across blocks without in-kernel communication (a device-wide fence costs tens of
// microseconds on a multi-die GPU): every block writes (value, index) to arg[2*b], arg[2*b+1];
// the NEXT kernel starts with every block reducing those pairs, which is cheap and gives all
// blocks the same pivot.  Two buffers alternate so that a step never overwrites what it reads.
__device__ inline void reduce_argmax(const double* __restrict__ arg, int npart, double* sval,
                                     int* sidx, double* outv, int* outi) {
  double v = -1.0e300;
  int ix = 0x7fffffff;
  for (int b = threadIdx.x; b < npart; b += blockDim.x) {
    double v2 = arg[2 * b];
    int i2 = (int)arg[2 * b + 1];
    if (v2 > v || (v2 == v && i2 < ix)) {
      v = v2;
      ix = i2;
    }
  }
  block_argmax(v, ix, sval, sidx, outv, outi);
}

// delta = diag(K_XX) = outputscale (stationary kernels), or the diagonal handed in (a covariance
// whose diagonal is not constant); block argmax candidates for pivot 0.
// next_forced >= 0: the caller replays a given pivot order; the thread that owns that row leaves
// its residual diagonal in st->pivdmax[0] for the first step (a step cannot read delta[] of a
// row that another block of the same launch is about to overwrite).
__global__ __launch_bounds__(VT) void k_pc_init(int n, HypArgs hyp, double* __restrict__ delta,
                                                 DevState* st, double* __restrict__ arg_out,
                                                 const double* __restrict__ diag_in, int next_forced) {
  __shared__ double sval[VT];
  __shared__ int sidx[VT];
  double bv = -1.0e300;
  int bi = 0x7fffffff;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    double v = diag_in ? diag_in[i] : hyp.outputscale;
    delta[i] = v;
    if (i == next_forced) st->pivdmax[0] = v;
    if (v > bv || (v == bv && i < bi)) {
      bv = v;
      bi = i;
    }
  }
  double ov;
  int oi;
  block_argmax(bv, bi, sval, sidx, &ov, &oi);
  if (threadIdx.x == 0) {
    arg_out[2 * blockIdx.x] = ov;
    arg_out[2 * blockIdx.x + 1] = (double)oi;
    if (blockIdx.x == 0) st->rank = 0;
  }
}

// Step m of the greedy factorisation: pivot m = argmax of the candidates left by the previous
// kernel, column m of L from row piv of K_XX, residual diagonal update, and the candidates for
// pivot m+1.  Picked rows carry delta = -1.  If the largest residual diagonal has vanished the
// step (and every later one, which sees the same candidates) does nothing.
// The pivot's row of the matrix is evaluated in fp64 from X, or read from row_in[i * row_ld]
// when the caller has formed it (a covariance that is not a plain kernel matrix of X).
__global__ __launch_bounds__(VT) void k_pc_step(const float* __restrict__ X, int n, int m, int kp,
                                                 HypArgs hyp, double* __restrict__ delta,
                                                 double* __restrict__ L, DevState* st,
                                                 const double* __restrict__ arg_in,
                                                 double* __restrict__ arg_out, double stop_thresh,
                                                 const double* __restrict__ row_in, int row_ld,
                                                 int forced, int next_forced) {
  __shared__ double sval[VT];
  __shared__ int sidx[VT];
  __shared__ double lpiv[BBMM_MAXK];
  double dpiv;
  int piv;
  reduce_argmax(arg_in, gridDim.x, sval, sidx, &dpiv, &piv);
  if (forced >= 0) {          // replayed pivot order: its residual diagonal was left by the previous kernel
    piv = forced;
    dpiv = st->pivdmax[m];
  }
  if (!(dpiv > stop_thresh)) {
    // keep the candidates alive for the remaining steps
    if (threadIdx.x == 0) {
      arg_out[2 * blockIdx.x] = arg_in[2 * blockIdx.x];
      arg_out[2 * blockIdx.x + 1] = arg_in[2 * blockIdx.x + 1];
    }
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    st->piv[m] = piv;
    st->pivdmax[m] = dpiv;
    st->rank = m + 1;
  }
  double root = sqrt(dpiv);
  if ((int)threadIdx.x < m) lpiv[threadIdx.x] = (double)L[(size_t)piv * kp + threadIdx.x];
  __syncthreads();
  double bv = -1.0e300;
  int bi = 0x7fffffff;
  for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n; i += gridDim.x * blockDim.x) {
    double di = delta[i];
    double lval;
    if (i == piv) {
      lval = root;
      di = -1.0;
    } else if (di < 0.0) {
      lval = 0.0;                  // already picked
    } else {
      double kv = row_in ? row_in[(size_t)i * row_ld] : kernel_value_f64(X, piv, i, hyp);
      for (int j = 0; j < m; ++j) kv -= lpiv[j] * (double)L[(size_t)i * kp + j];
      lval = kv / root;
      di = di - lval * lval;
      if (di < 0.0) di = 0.0;
    }
    L[(size_t)i * kp + m] = lval;
    delta[i] = di;
    if (i == next_forced) st->pivdmax[m + 1] = di;
    if (di >= 0.0 && (di > bv || (di == bv && i < bi))) {
      bv = di;
      bi = i;
    }
  }
  double ov;
  int oi;
  block_argmax(bv, bi, sval, sidx, &ov, &oi);
  if (threadIdx.x == 0) {
    arg_out[2 * blockIdx.x] = ov;
    arg_out[2 * blockIdx.x + 1] = (double)oi;
  }
}

// --------------------------------------------- predictions at test inputs ----
// k(x_j, x*_a) in fp64 from the raw inputs (Sec. 2, Eq. (1) needs the columns k_{X x*}).
__device__ inline double cross_value_f64(const float* __restrict__ X, int j,
                                         const float* __restrict__ Xs, int a, const HypArgs& hyp) {
  double rho2 = 0.0;
  for (int dim = 0; dim < hyp.d; ++dim) {
    double df = ((double)X[(size_t)j * hyp.d + dim] - (double)Xs[(size_t)a * hyp.d + dim]) *
                hyp.inv_ls[dim];
    rho2 += df * df;
  }
  if (hyp.kernel == 0) return hyp.outputscale * exp(-0.5 * rho2);
  double rho = sqrt(rho2);
  const double s5 = 2.23606797749978969;
  return hyp.outputscale * (1.0 + s5 * rho + (5.0 / 3.0) * rho2) * exp(-s5 * rho);
}

// B[j][a] = k(x_j, x*_a): the right-hand-side block of the variance solves (stride ld, zero padded)
__global__ void k_cross_block(const float* __restrict__ X, const float* __restrict__ Xs, int n,
                              int ns, int ld, HypArgs hyp, double* __restrict__ B) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * ld) return;
  int j = (int)(idx / ld), a = (int)(idx % ld);
  B[idx] = (a < ns) ? cross_value_f64(X, j, Xs, a, hyp) : 0.0;
}

// out[a] = prior + sign * sum_j k(x*_a, x_j) V[j][percol ? a : 0], one block per test point,
// fixed-order fp64 block sum.  Mean: V = K_hat^{-1} y, prior 0, sign +1.  Variance: V = the
// solves of the block above, prior k(x*, x*) = s (both kernels are stationary), sign -1.
__global__ __launch_bounds__(VT) void k_cross_dot(const float* __restrict__ X,
                                                   const float* __restrict__ Xs, int n,
                                                   HypArgs hyp, const double* __restrict__ V,
                                                   int ldv, int percol, double prior, double sign,
                                                   float* __restrict__ out) {
  __shared__ double red[VT];
  int a = blockIdx.x;
  int col = percol ? a : 0;
  double acc = 0.0;
  for (int j = threadIdx.x; j < n; j += VT)
    acc += cross_value_f64(X, j, Xs, a, hyp) * V[(size_t)j * ldv + col];
  red[threadIdx.x] = acc;
  __syncthreads();
  for (int w = VT / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) out[a] = (float)(prior + sign * red[0]);
}

// ---------------------------------------------- capacitance matrix, log|P| ---
// C = sigma^2 I + L^T L (k x k, fp64), Cholesky factor G, log|P| = log|C| + (n-k) log sigma^2.
__global__ __launch_bounds__(VT) void k_pre_setup(const double* __restrict__ L, int n, int kp,
                                                   double noise, DevState* st, double* partial,
                                                   double* gpartial) {
  int k = st->rank;
  int npairs = k * k;
  // each thread owns pairs e = tid, tid + VT, ... (at most 4 for k <= 32)
  double acc[4] = {0.0, 0.0, 0.0, 0.0};
  int rows_per_block = (n + gridDim.x - 1) / gridDim.x;
  int r0 = blockIdx.x * rows_per_block;
  int r1 = min(n, r0 + rows_per_block);
  for (int i = r0; i < r1; ++i) {
    const double* li = L + (size_t)i * kp;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      int e = threadIdx.x + u * VT;
      if (e < npairs) acc[u] += (double)li[e / k] * (double)li[e % k];
    }
  }
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    int e = threadIdx.x + u * VT;
    if (e < npairs) partial[(size_t)blockIdx.x * (BBMM_MAXK * BBMM_MAXK) + e] = acc[u];
  }
  __shared__ double C[BBMM_MAXK * BBMM_MAXK];
  __shared__ double tot[BBMM_MAXK * BBMM_MAXK];
  if (!reduce_blocks(partial, gpartial, BBMM_MAXK * BBMM_MAXK, npairs, st->counter[1], tot)) return;
  for (int e = threadIdx.x; e < npairs; e += VT) {
    int a = e / k, c = e % k;
    C[a * BBMM_MAXK + c] = tot[e] + (a == c ? noise : 0.0);
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    // in-place lower Cholesky factorisation of C in LDS
    double logdet = 0.0;
    int bad = 0;
    for (int a = 0; a < k; ++a) {
      for (int c = 0; c <= a; ++c) {
        double s = C[a * BBMM_MAXK + c];
        for (int j = 0; j < c; ++j) s -= C[a * BBMM_MAXK + j] * C[c * BBMM_MAXK + j];
        if (a == c) {
          if (!(s > 0.0) || !finite_d(s)) {
            bad = 1;
            s = 1.0;
          }
          double g = sqrt(s);
          C[a * BBMM_MAXK + a] = g;
          logdet += 2.0 * log(g);
        } else {
          C[a * BBMM_MAXK + c] = s / C[c * BBMM_MAXK + c];
        }
      }
    }
    st->logdetP = logdet + (double)(n - k) * log(noise);
    if (bad) st->status = 3;
  }
  __syncthreads();
  // G^{-1}, one column per thread by forward substitution on the unit vectors; the iteration
  // applies C^{-1} = G^{-T} G^{-1} as two small dense products instead of serial substitutions
  // (cond(G) = sqrt(cond(C)) <= sqrt(1 + |L|^2 / sigma^2): harmless in fp64).
  for (int e = threadIdx.x; e < BBMM_MAXK * BBMM_MAXK; e += VT) tot[e] = 0.0;
  __syncthreads();
  if ((int)threadIdx.x < k) {
    int j = threadIdx.x;
    tot[j * BBMM_MAXK + j] = 1.0 / C[j * BBMM_MAXK + j];
    for (int i = j + 1; i < k; ++i) {
      double sacc = 0.0;
      for (int a = j; a < i; ++a) sacc += C[i * BBMM_MAXK + a] * tot[a * BBMM_MAXK + j];
      tot[i * BBMM_MAXK + j] = -sacc / C[i * BBMM_MAXK + i];
    }
  }
  __syncthreads();
  for (int e = threadIdx.x; e < BBMM_MAXK * BBMM_MAXK; e += VT) {
    int a = e / BBMM_MAXK, c = e % BBMM_MAXK;
    bool low = a < k && c <= a;
    st->G[e] = low ? C[e] : 0.0;
    st->Ginv[e] = low ? tot[e] : 0.0;
  }
}

// -------------------------------------------------------------- probes -------
// R[:,0] = y,  R[:,1+i] = L E1[:,i] + sigma E2[:,i]   (row-major, stride ld, zero padded)
__global__ void k_probes(const float* __restrict__ y, const float* __restrict__ E1,
                         const float* __restrict__ E2, const double* __restrict__ L, int n, int t,
                         int kp, int ld, double sigma, const DevState* __restrict__ st,
                         double* __restrict__ R) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)n * ld) return;
  int i = (int)(idx / ld), q = (int)(idx % ld);
  int k = st->rank;
  double v = 0.0;
  if (q == 0) {
    v = (double)y[i];
  } else if (q <= t) {
    double s = sigma * (double)E2[(size_t)i * t + (q - 1)];
    for (int m = 0; m < k; ++m) s += (double)L[(size_t)i * kp + m] * (double)E1[(size_t)m * t + (q - 1)];
    v = s;
  }
  R[idx] = v;
}

// ------------------------------------------------ fused mBCG vector updates --
// All n x c blocks of the iteration (U, R, D, V, Z0) are kept in fp64: perturbations of
// relative size 2^-24 in the iterates are amplified by many orders of magnitude over a few
// tens of CG iterations on ill-conditioned kernel matrices, which would make a fixed-iteration
// comparison with an fp64 reference meaningless.  They are O(n c) and cost ~nothing next to
// the O(n^2) product.
//
// Reductions over rows are split over kernels instead of being finished inside one kernel:
// a kernel writes per-block fp64 partial sums, the NEXT kernel (or a one-block finishing kernel)
// adds them in a fixed order.  Kernel boundaries give the needed ordering for free, whereas a
// device-wide fence inside a kernel was measured at ~60 us here.
//
// (1) after the product: V = scaleV * sum_s Vp[s] + addD * D, and per-block partial d^T v.
//     RU rows per loop trip and thread; the first NL partial slots of each and its D entry are
//     requested before anything is added, so a trip costs one memory round trip.  <3, 8> is the
//     general form; <8, 2> serves products that leave at most two slots per row (the SGPR product:
//     one), where three rows per trip leave too few loads in flight to cover the latency.
template <int RU, int NL>
__global__ __launch_bounds__(VT) void k_dv(const double* __restrict__ Vp, VpShape shape, int n, int np,
                                            int ld, double scaleV, double addD,
                                            const double* __restrict__ D4, double* __restrict__ V,
                                            const DevState* __restrict__ st,
                                            double* __restrict__ partial_dv) {
  __shared__ double red[VT];
  if (st->done) return;
  if (addD < 0.0) {
    scaleV = st->loop_scaleV;
    addD = st->loop_addD;
  }
  int q = threadIdx.x % ld, rl = threadIdx.x / ld, rpp = VT / ld;
  int pq = perm16(q);
  double acc = 0.0;
  int stride = gridDim.x * rpp;
  size_t slot_stride = (size_t)np * ld;
  for (int ib = blockIdx.x * rpp + rl; ib < n; ib += RU * stride) {
    double pv[RU][NL], dd[RU];
    int ns[RU];
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      int i = ib + u * stride;
      bool ok = i < n;
      int ic = ok ? i : ib;
      ns[u] = ok ? (shape.nseg ? shape.nseg[ic / shape.seg_cols] : shape.nsplit) : 0;
      size_t pidx = (size_t)ic * ld + pq;
#pragma unroll
      for (int sp = 0; sp < NL; ++sp) pv[u][sp] = (sp < ns[u]) ? Vp[(size_t)sp * slot_stride + pidx] : 0.0;
      dd[u] = ok ? D4[d4_index(ic, q, ld)] : 0.0;
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      int i = ib + u * stride;
      if (i < n) {
        double sv;
        if (NL == 8)
          sv = ((pv[u][0] + pv[u][1]) + (pv[u][2] + pv[u][3])) + ((pv[u][4] + pv[u][5]) + (pv[u][6] + pv[u][7]));
        else
          sv = (NL > 1) ? pv[u][0] + pv[u][NL > 1 ? 1 : 0] : pv[u][0];
        size_t pidx = (size_t)i * ld + pq;
        // further slots eight at a time, all requested before any is added (the product from the
        // triangular storage leaves up to one slot per panel)
        for (int s0 = NL; s0 < ns[u]; s0 += 8) {
          double t[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) t[e] = (s0 + e < ns[u]) ? Vp[(size_t)(s0 + e) * slot_stride + pidx] : 0.0;
          sv += ((t[0] + t[1]) + (t[2] + t[3])) + ((t[4] + t[5]) + (t[6] + t[7]));
        }
        double v = scaleV * sv + addD * dd[u];
        V[(size_t)i * ld + q] = v;
        acc += dd[u] * v;
      }
    }
  }
  red[threadIdx.x] = acc;
  __syncthreads();
  if (rl == 0) {
    double s = 0.0;
    for (int r = 0; r < rpp; ++r) s += red[r * ld + q];
    partial_dv[(size_t)blockIdx.x * ld + q] = s;
  }
}

constexpr int UT = 1024;      // threads of the update kernel
static_assert(BBMM_MAXK * BBMM_MAXK == UT, "k_ur_fin loads one entry of G per thread");

// alpha_j for column q from the d^T v total, with the freeze guard (k_ur_main needs the value,
// k_ur_fin records it; both evaluate this on the state they read at their start).
__device__ inline double alpha_from(int active, double rho, double dv, int q, int c, int* ok_out) {
  int ok = active && finite_d(dv) && dv > 0.0 && q < c;
  *ok_out = ok;
  return ok ? rho / dv : 0.0;
}

// (2a) every block first adds the d^T v partials of k_dv (same order in every block), forms
//      alpha_j, then U += alpha D, R -= alpha V and its partial sums of |r|^2 and L^T R.
//      init != 0: no update, just the sums for R = B (gives Z_0, rho_0).  init == 2: the same
//      after a warm start, R = B - K_hat U_0: the norms |b| of the first pass are kept.
//      A wave takes 4 rows per step: lane l holds element (row l/16, column l%16 [+16]) of the
//      blocks, which is exactly the B operand of an fp64 MFMA whose A operand is the same four
//      rows of L, so L^T R costs one load of L per 16 columns of L instead of one per entry.
template <int KP, int NQ>
__global__ __launch_bounds__(UT) void k_ur_main(int init, int n, int c,
                                                 const double* __restrict__ D4,
                                                 const double* __restrict__ V,
                                                 double* __restrict__ U, double* __restrict__ R,
                                                 const double* __restrict__ L, DevState* st,
                                                 const double* __restrict__ partial_dv, int nb_dv,
                                                 double* __restrict__ partial) {
  constexpr int LD = 16 * NQ;
  constexpr int MB = (KP + 15) / 16;
  constexpr int NW = UT / 64;
  __shared__ double stage[NW][256];
  __shared__ double dvtot[BBMM_MAXC];
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int q = lane & 15, g = lane >> 4;
  // state reads are requested together with the first partial sums (one memory round trip)
  int done = st->done;
  double alpha[NQ], s_rho[NQ];
  int s_active[NQ];
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    alpha[qb] = 0.0;
    s_rho[qb] = st->rho[qb * 16 + q];
    s_active[qb] = st->active[qb * 16 + q];
  }
  if (!init) {
    // thread (row group rl, column cq): rows rl, rl + rpp, ... of the partials
    int cq = threadIdx.x % LD, rl = threadIdx.x / LD;
    constexpr int rpp = UT / LD;
    // all rows of a thread are requested before the first is added (one memory round trip)
    double sv = 0.0;
    for (int b0 = rl; b0 < nb_dv; b0 += 8 * rpp) {
      double v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        int b = b0 + u * rpp;
        v[u] = (b < nb_dv) ? partial_dv[(size_t)b * LD + cq] : 0.0;
      }
      sv += ((v[0] + v[1]) + (v[2] + v[3])) + ((v[4] + v[5]) + (v[6] + v[7]));
    }
    // a wave holds 64 / LD row groups of the same columns
    sv += __shfl_xor(sv, 32, 64);
    if (LD == 16) sv += __shfl_xor(sv, 16, 64);
    if (lane < LD) stage[wave][lane] = sv;
    __syncthreads();
    if ((int)threadIdx.x < LD) {
      double t = 0.0;
#pragma unroll
      for (int w = 0; w < NW; ++w) t += stage[w][threadIdx.x];
      dvtot[threadIdx.x] = t;
      if (blockIdx.x == 0) st->dvtot[threadIdx.x] = t;
    }
    __syncthreads();
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
      int ok;
      alpha[qb] = alpha_from(s_active[qb], s_rho[qb], dvtot[qb * 16 + q], qb * 16 + q, c, &ok);
    }
  }
  if (done) return;                                   // block-uniform
  double rr[NQ];
  f64x4 acc[MB > 0 ? MB : 1][NQ];
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    rr[qb] = 0.0;
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) acc[mb][qb] = (f64x4){0.0, 0.0, 0.0, 0.0};
  }
  // RU row quads per loop trip, all their loads requested before the first use
  constexpr int RU = (NQ == 1) ? 4 : 2;
  int gw = blockIdx.x * NW + wave, nw = gridDim.x * NW;
  for (int ib = 4 * gw; ib < n; ib += 4 * nw * RU) {   // wave-uniform bounds: MFMA needs all lanes
    double dd[RU][NQ], uu[RU][NQ], vv[RU][NQ], rv[RU][NQ], la[RU][MB > 0 ? MB : 1];
    bool ok[RU];
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      int i = ib + u * 4 * nw + g;
      ok[u] = i < n;
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        int col = qb * 16 + q;
        size_t idx = (size_t)i * LD + col;
        dd[u][qb] = uu[u][qb] = vv[u][qb] = rv[u][qb] = 0.0;
        if (ok[u]) {
          rv[u][qb] = R[idx];
          if (!init) {
            dd[u][qb] = D4[d4_index(i, col, LD)];
            uu[u][qb] = U[idx];
            vv[u][qb] = V[idx];
          }
        }
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb) {
        int m = mb * 16 + q;
        la[u][mb] = (ok[u] && m < KP) ? L[(size_t)i * KP + m] : 0.0;
      }
    }
#pragma unroll
    for (int u = 0; u < RU; ++u) {
      int i = ib + u * 4 * nw + g;
      double rd[NQ];
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) {
        size_t idx = (size_t)i * LD + qb * 16 + q;
        double v = rv[u][qb];
        if (!init && ok[u]) {
          U[idx] = uu[u][qb] + alpha[qb] * dd[u][qb];
          v = v - alpha[qb] * vv[u][qb];
          R[idx] = v;
        }
        rd[qb] = v;
        rr[qb] += v * v;
      }
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) acc[mb][qb] = mfma16d(la[u][mb], rd[qb], acc[mb][qb]);
    }
  }
  // ---- block reduction over the waves, 256 values (16 rows of L^T R x 16 columns) per round ----
  size_t pstride = (size_t)(KP + 1) * LD;
  double* pout = partial + (size_t)blockIdx.x * pstride;
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    double v = rr[qb];
    v += __shfl_xor(v, 16, 64);
    v += __shfl_xor(v, 32, 64);
    if (g == 0) stage[wave][qb * 16 + q] = v;
  }
  __syncthreads();
  if ((int)threadIdx.x < LD) {
    double t = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) t += stage[w][threadIdx.x];
    pout[threadIdx.x] = t;
  }
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
      __syncthreads();
#pragma unroll
      for (int r = 0; r < 4; ++r) stage[wave][(4 * r + g) * 16 + q] = acc[mb][qb][r];
      __syncthreads();
      if ((int)threadIdx.x < 256) {
        int m = mb * 16 + (int)threadIdx.x / 16, qq = qb * 16 + (int)threadIdx.x % 16;
        if (m < KP) {
          double t = 0.0;
#pragma unroll
          for (int w = 0; w < NW; ++w) t += stage[w][threadIdx.x];
          pout[(size_t)(1 + m) * LD + qq] = t;
        }
      }
    }
}

// (2b) one block: totals of |r|^2 and L^T R, the k x k solves (one wave per column, lanes =
//      rows of the triangular systems), rho' = (|r|^2 - (L^T r)^T C^{-1} (L^T r)) / sigma^2
//      (= r^T P^{-1} r by the Woodbury formula), alpha/beta bookkeeping, residual history, stop flag.
template <int KP>
__global__ __launch_bounds__(UT) void k_ur_fin(int init, int ld, int c, double noise, double tol,
                                                DevState* st, const double* __restrict__ partial,
                                                int nb, int iter, double* alpha_hist,
                                                double* beta_hist, double* resid_hist) {
  __shared__ double tot[(BBMM_MAXK + 1) * BBMM_MAXC];
  __shared__ double psum[(BBMM_MAXK + 1) * BBMM_MAXC];   // parts x E, parts * E <= this size
  __shared__ double Gs[BBMM_MAXK * BBMM_MAXK];
  __shared__ double quad_s[BBMM_MAXC];
  __shared__ double rel_s[BBMM_MAXC];
  // Everything this block needs from the state is requested first, together with the partial
  // sums, so that the kernel pays one memory round trip instead of one per dependent read.
  int done = st->done;
  if (noise < 0.0) {
    noise = st->loop_noise;
    tol = st->loop_tol;
  }
  int tq = (int)threadIdx.x < ld ? (int)threadIdx.x : 0;
  double s_rho = st->rho[tq], s_bnorm = st->bnorm[tq], s_dv = st->dvtot[tq];
  int s_active = st->active[tq], s_mvalid = st->m_valid[tq];
  double g_mine = st->Ginv[threadIdx.x];   // BBMM_MAXK * BBMM_MAXK == UT entries
  size_t pstride = (size_t)(KP + 1) * ld;
  int E = (KP + 1) * ld;
  // totals over the nb partial rows: `parts` thread groups take every parts-th row
  int parts = (E <= UT / 4) ? 4 : ((E <= UT / 2) ? 2 : 1);
  int per = UT / parts;
  int part = threadIdx.x / per, te = threadIdx.x % per;
  for (int e = te; e < E; e += per) {
    // 32 loads are issued before the first is consumed: the sum is latency-, not bandwidth-bound
    // (a round trip to memory written by other compute units costs ~2.4 us here)
    double tsum = 0.0;
    int b = part;
    for (; b + 31 * parts < nb; b += 32 * parts) {
      double v[32];
#pragma unroll
      for (int u = 0; u < 32; ++u) v[u] = partial[(size_t)(b + u * parts) * pstride + e];
#pragma unroll
      for (int w = 16; w > 0; w >>= 1)
#pragma unroll
        for (int u = 0; u < w; ++u) v[u] += v[u + w];
      tsum += v[0];
    }
    for (; b < nb; b += parts) tsum += partial[(size_t)b * pstride + e];
    psum[part * E + e] = tsum;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < E; e += UT) {
    double t = psum[e];
    for (int pp = 1; pp < parts; ++pp) t += psum[pp * E + e];
    tot[e] = t;
  }
  if (done) return;                     // block-uniform
  Gs[threadIdx.x] = g_mine;             // G^{-1}, zero outside the leading k x k lower triangle
  __syncthreads();
  // C^{-1} (L^T r) for all columns at once: w = G^{-1} y, quad = w^T w, x = G^{-T} w; thread
  // (m, qq) owns one entry; sums run over the compiled rank limit (padding is zero)
  {
    int m = threadIdx.x / ld, qq = threadIdx.x % ld;
    double wv = 0.0;
    if (m < KP) {
#pragma unroll
      for (int a = 0; a < KP; ++a) wv += Gs[m * BBMM_MAXK + a] * tot[(size_t)(1 + a) * ld + qq];
      psum[m * ld + qq] = wv;
    }
    __syncthreads();
    if (m < KP) {
      double xv = 0.0;
#pragma unroll
      for (int a = 0; a < KP; ++a) xv += Gs[a * BBMM_MAXK + m] * psum[a * ld + qq];
      st->Qt[m * BBMM_MAXC + qq] = xv;
    }
    if ((int)threadIdx.x < ld) {
      double sq = 0.0;
#pragma unroll
      for (int a = 0; a < KP; ++a) {
        double wa = psum[a * ld + threadIdx.x];
        sq += wa * wa;
      }
      quad_s[threadIdx.x] = sq;
    }
  }
  __syncthreads();
  if ((int)threadIdx.x < ld) {
    int qq = threadIdx.x;
    double rrq = tot[qq];
    double rho_new = (rrq - quad_s[qq]) / noise;
    if (init) {
      int ok = finite_d(rho_new) && rho_new > 0.0 && qq < c;
      st->rho[qq] = rho_new;
      st->rho0[qq] = rho_new;
      if (init != 2) st->bnorm[qq] = sqrt(rrq);   // init == 2: warm start, |b| is already there
      st->active[qq] = ok;
      st->m_valid[qq] = 0;
      st->beta_cur[qq] = 0.0;
      st->alpha_cur[qq] = 0.0;
    } else {
      int ok;
      double alpha = alpha_from(s_active, s_rho, s_dv, qq, c, &ok);
      st->alpha_cur[qq] = alpha;
      st->m_valid[qq] = s_mvalid + ok;
      alpha_hist[(size_t)iter * BBMM_MAXC + qq] = alpha;
      int ok2 = ok && finite_d(rho_new) && rho_new > 0.0;
      double beta = ok2 ? rho_new / s_rho : 0.0;
      st->active[qq] = ok2;
      st->beta_cur[qq] = beta;
      if (ok2) st->rho[qq] = rho_new;
      beta_hist[(size_t)iter * BBMM_MAXC + qq] = beta;
      double bn = s_bnorm;
      double rel = sqrt(rrq) / (bn > 0.0 ? bn : 1.0);
      resid_hist[(size_t)iter * BBMM_MAXC + qq] = rel;
      rel_s[qq] = rel;
    }
  }
  __syncthreads();
  if (threadIdx.x == 0 && !init) {
    st->iters_run = iter + 1;
    if (tol > 0.0) {
      int all = 1;
      for (int qq = 0; qq < c; ++qq)
        if (!(rel_s[qq] < tol)) all = 0;
      if (all) st->done = 1;
    }
  }
}

// (3) z = P^{-1} r by the Woodbury formula, z = (r - L (C^{-1} L^T r)) / sigma^2 with C^{-1} L^T r
//     left in st->Qt by k_ur_fin, then D <- z + beta D (MODE 0), or Z0 = D = z at the start
//     (MODE 1), or just Z = z for the stand-alone preconditioner solve (MODE 2).
//     A wave takes 16 rows per step: L Qt is KP / 4 fp64 MFMAs whose result register r holds
//     row 4 r + lane / 16, column lane % 16 -- rows in which R and the quad-swizzled D are
//     contiguous across the wave.
template <int KP, int NQ, int MODE>
__global__ __launch_bounds__(VT) void k_zd(int n, double noise, const double* __restrict__ R,
                                            const double* __restrict__ L, double* __restrict__ D4,
                                            double* __restrict__ Z, const DevState* __restrict__ st) {
  constexpr int LD = 16 * NQ;
  constexpr int KS = KP / 4;
  if (MODE != 2 && st->done) return;
  if (noise < 0.0) noise = st->loop_noise;
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int q = lane & 15, g = lane >> 4;
  double beta[NQ];
  double qtb[KS > 0 ? KS : 1][NQ];
#pragma unroll
  for (int qb = 0; qb < NQ; ++qb) {
    beta[qb] = (MODE == 0) ? st->beta_cur[qb * 16 + q] : 0.0;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) qtb[kk][qb] = st->Qt[(4 * kk + g) * BBMM_MAXC + qb * 16 + q];
  }
  double inv_noise = 1.0 / noise;
  constexpr int NW = VT / 64;
  int gw = blockIdx.x * NW + wave, nw = gridDim.x * NW;
  for (int i0 = 16 * gw; i0 < n; i0 += 16 * nw) {   // wave-uniform bounds: MFMA needs all lanes
    f64x4 acc[NQ];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) acc[qb] = (f64x4){0.0, 0.0, 0.0, 0.0};
    int arow = i0 + q;
#pragma unroll
    for (int kk = 0; kk < KS; ++kk) {
      double la = (arow < n) ? L[(size_t)arow * KP + 4 * kk + g] : 0.0;
#pragma unroll
      for (int qb = 0; qb < NQ; ++qb) acc[qb] = mfma16d(la, qtb[kk][qb], acc[qb]);
    }
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int i = i0 + 4 * r + g;
      if (i < n) {
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) {
          int col = qb * 16 + q;
          size_t idx = (size_t)i * LD + col;
          double z = (R[idx] - acc[qb][r]) * inv_noise;
          if (MODE == 2) {
            Z[idx] = z;
          } else {
            size_t di = d4_index(i, col, LD);
            if (MODE == 1) {
              Z[idx] = z;
              D4[di] = z;
            } else {
              D4[di] = z + beta[qb] * D4[di];
            }
          }
        }
      }
    }
  }
}

// ---------------------------------------- tridiagonal eigen-solver and SLQ ---
// Eigenvalues of a symmetric tridiagonal matrix (diagonal a[0..m-1], off-diagonal
// b[0..m-2]) together with the FIRST component of every unit eigenvector, which is all
// that e_1^T f(T) e_1 = sum_i w_i^2 f(lambda_i) needs.  Implicit-shift QR sweeps with the
// Wilkinson shift; each Givens rotation of a sweep is also applied to the row vector
// w (initially e_1), so w ends up as the first row of the eigenvector matrix.
// Serial, O(m^2); arrays live in LDS.  b needs m entries (b[m-1] is scratch).
// One thread runs this, so its cost is its instruction count plus every wait for an LDS value:
// the top of the unreduced block is therefore not searched for before each sweep but kept from
// sweep to sweep, and a sweep tests the off-diagonal entries it rewrites as it goes (all of the
// block's but the last, which the deflation test at the top covers).
// Returns true when every eigenvalue has deflated within `sweeps_per_row` * m trips (sweeps and
// deflations); false means a[] still holds an unreduced block and must not be used.
__device__ bool tridiag_eig_first_row(double* a, double* b, double* w, int m, int sweeps_per_row) {
  for (int i = 0; i < m; ++i) w[i] = (i == 0) ? 1.0 : 0.0;
  if (m <= 1) return true;
  b[m - 1] = 0.0;
  const double eps = 2.220446049250313e-16;
  int hi = m - 1;
  int lo = -1;                          // top of the unreduced block that ends at hi; -1: not known
  int budget = sweeps_per_row * m;
  while (hi > 0 && budget-- > 0) {
    // deflate converged eigenvalues at the bottom
    double bb = b[hi - 1], ah = a[hi], ahm = a[hi - 1];
    if (fabs(bb) <= eps * (fabs(ahm) + fabs(ah))) {
      b[hi - 1] = 0.0;
      --hi;
      continue;
    }
    if (lo < 0 || lo >= hi) {
      // the block above the one just finished: search for its top
      lo = hi - 1;
      while (lo > 0 && fabs(b[lo - 1]) > eps * (fabs(a[lo - 1]) + fabs(a[lo]))) --lo;
      if (lo > 0) b[lo - 1] = 0.0;
    }
    // Wilkinson shift from the trailing 2 x 2 block
    double dlt = 0.5 * (ahm - ah);
    double denom = dlt + (dlt >= 0.0 ? 1.0 : -1.0) * sqrt(dlt * dlt + bb * bb);
    double mu = (denom != 0.0) ? ah - bb * bb / denom : ah;
    // chase the bulge from lo to hi.  The values that one rotation hands to the next (the entries
    // a[i], b[i], w[i] that it has just changed, and the bulge x, z) travel in registers; the LDS
    // arrays are only read at entries no rotation of this sweep has touched yet (one step ahead of
    // their use) and written with final values, so no step waits for a store of the step before.
    double x = a[lo] - mu;
    double z = b[lo];
    double ai = a[lo], bi = b[lo], wi = w[lo];
    double an = a[lo + 1], bn = b[lo + 1], wn = w[lo + 1];
    double ap = 0.0;                    // a[i - 1] as the rotation before left it
    int split = -1;
    for (int i = lo; i < hi; ++i) {
      double aj = an, bj = bn, wj = wn;
      if (i + 2 <= hi) {
        an = a[i + 2];
        bn = b[i + 2];
        wn = w[i + 2];
      }
      // rotation (c, s) that zeroes z against x:  [c s; -s c]^T applied to rows/cols i, i+1
      // (1 / r from the hardware's reciprocal square root and two Newton steps: a third of the
      // instructions of sqrt and a division)
      double h = fma(x, x, z * z);
      bool nz = h > 1e-290;
      double y = __builtin_amdgcn_rsq(nz ? h : 1.0);
#pragma unroll
      for (int it = 0; it < 2; ++it) {
        double hy = h * y;
        y = fma(0.5 * y, fma(-hy, y, 1.0), y);
      }
      double rinv = nz ? y : 0.0;
      double r = h * rinv;
      double c = nz ? x * rinv : 1.0;
      double s = z * rinv;
      double cs2 = 2.0 * c * s * bi;
      double anew = c * c * ai + cs2 + s * s * aj;
      a[i] = anew;
      if (i > lo) {
        // b[i - 1] = r is final now, and so are its two neighbours on the diagonal
        bool negligible = r <= eps * (fabs(ap) + fabs(anew));
        b[i - 1] = negligible ? 0.0 : r;
        if (negligible) split = i;
      }
      ap = anew;
      w[i] = c * wi + s * wj;
      x = (c * c - s * s) * bi + c * s * (aj - ai);
      ai = s * s * ai - cs2 + c * c * aj;
      wi = -s * wi + c * wj;
      z = s * bj;                       // (unused after the last rotation: b[hi] is not in the block)
      bi = c * bj;
    }
    a[hi] = ai;
    w[hi] = wi;
    b[hi - 1] = x;
    if (split >= 0) lo = split;
  }
  return hi == 0;
}

// (z^T P^{-1} z) e_1^T log(T) e_1 for one probe column: T of size m from that column's CG
// coefficients (Observation in App. A; coefficient j of the column at alpha[j * stride]), its
// eigenvalues and first eigenvector row (App. B, log-det paragraph).  *status receives 0, or the
// BBMM_* code of what went wrong (eigen-solver out of budget: 6; non-positive eigenvalue with
// weight, or a non-finite term: 4).  a, b, w: LDS arrays of BBMM_MAXP doubles.
__device__ double slq_term(const double* __restrict__ alpha, const double* __restrict__ beta, size_t stride,
                           int m, double rho0, int sweeps_per_row, double* a, double* b, double* w,
                           int* status) {
  if (m > BBMM_MAXP) m = BBMM_MAXP;
  for (int j = 0; j < m; ++j) {
    double al = alpha[(size_t)j * stride];
    double dg = 1.0 / al;
    if (j > 0) {
      double alp = alpha[(size_t)(j - 1) * stride];
      double bep = beta[(size_t)(j - 1) * stride];
      dg += bep / alp;
      b[j - 1] = sqrt(bep) / alp;
    }
    a[j] = dg;
  }
  bool conv = tridiag_eig_first_row(a, b, w, m, sweeps_per_row);
  double g = 0.0;
  int bad = 0;
  for (int j = 0; j < m; ++j) {
    if (!(a[j] > 0.0)) {
      if (w[j] * w[j] > 1e-20) bad = 1;
      continue;
    }
    g += w[j] * w[j] * log(a[j]);
  }
  double term = rho0 * g;
  if (!finite_d(term)) bad = 1;
  *status = !conv ? 6 : (bad ? 4 : 0);
  return term;
}

// The same quantity without an eigen-decomposition.  log(x) = int_0^inf [1/(1+s) - 1/(x+s)] ds, so
//   e_1^T log(T) e_1 = int_0^inf [1/(1+s) - r(s)] ds,   r(s) = e_1^T (T + s I)^{-1} e_1,
// and with s = e^u the integrand decays like e^{-|u|} on both sides and is analytic for
// |Im u| < pi: the trapezoid rule with step h converges like exp(-2 pi^2 / h) (h = 1/2: 7e-18).
// r(s) is the continued fraction delta_m = a_m + s, delta_j = a_j + s - b_j^2 / delta_{j+1},
// r = 1 / delta_1 (all delta > 0: T + s I is positive definite), and
//   1/(1+s) - r(s) = (a_1 - 1 - b_1^2 / delta_2) / ((1+s) delta_1)
// has no cancellation in s.  Every node is one thread's chain of m divisions, the nodes of all
// probes run side by side: microseconds where the serial QR sweeps of one thread per probe take
// most of a millisecond at m = 50 (a rotation is ~25 dependent fp64 instructions).  The range of u
// needs bounds of the spectrum: Gershgorin from above, and from below the largest G 2^-i (i < 64)
// under which no eigenvalue lies, by Sturm counts taken side by side as well.  The eigenvalues
// never appear, so clusters of near-duplicate Ritz values need no care.
// Agreement with the eigen-decomposition route: 1e-13 ... 2e-10 relative (condition 2e8).
constexpr int SLQ_THREADS = 256;
constexpr double SLQ_H = 0.5;        // trapezoid step in u = ln s
constexpr double SLQ_PAD = 37.0;     // e^-37 = 9e-17: what is cut off at either end
static_assert(SLQ_THREADS <= BBMM_MAXP, "the reduction buffer of the quadrature is an LDS array of BBMM_MAXP doubles");

// All SLQ_THREADS threads of the block call this; the result is valid in thread 0.
// a, b2: LDS, BBMM_MAXP doubles each; red: LDS, SLQ_THREADS doubles; cnt: LDS, 65 ints.
__device__ double slq_term_quadrature(const double* __restrict__ alpha, const double* __restrict__ beta,
                                      size_t stride, int m, double rho0, double* a, double* b2, double* red,
                                      int* cnt, int* status) {
  int tid = threadIdx.x;
  if (m > BBMM_MAXP) m = BBMM_MAXP;
  if (m <= 0) {
    if (tid == 0) *status = 0;
    return 0.0;
  }
  // T from the coefficients (Observation in App. A); only b^2 is needed
  for (int j = tid; j < m; j += SLQ_THREADS) {
    double al = alpha[(size_t)j * stride];
    double dg = 1.0 / al;
    if (j > 0) {
      double alp = alpha[(size_t)(j - 1) * stride];
      double bep = beta[(size_t)(j - 1) * stride];
      dg += bep / alp;
      b2[j - 1] = bep / (alp * alp);
    }
    a[j] = dg;
  }
  __syncthreads();
  // Gershgorin bound of the largest eigenvalue
  double gmax = 0.0;
  for (int j = tid; j < m; j += SLQ_THREADS) {
    double r = a[j] + (j + 1 < m ? sqrt(b2[j]) : 0.0) + (j > 0 ? sqrt(b2[j - 1]) : 0.0);
    gmax = fmax(gmax, finite_d(r) ? r : 1.0e300);
  }
  red[tid] = gmax;
  __syncthreads();
  for (int w = SLQ_THREADS / 2; w > 0; w >>= 1) {
    if (tid < w) red[tid] = fmax(red[tid], red[tid + w]);
    __syncthreads();
  }
  double G = red[0];
  __syncthreads();
  // Sturm counts: thread i < 64 counts the eigenvalues below G 2^-i, thread 64 those below 0
  if (tid <= 64) {
    double x = (tid < 64) ? ldexp(G, -tid) : 0.0;
    double q = a[0] - x;
    int c = q < 0.0;
    for (int j = 1; j < m; ++j) {
      if (q == 0.0) q = 1.0e-300;
      q = a[j] - x - b2[j - 1] / q;
      c += q < 0.0;
    }
    cnt[tid] = (q == q) ? c : m;          // a NaN anywhere: treated as "eigenvalues below"
  }
  __syncthreads();
  int ilo = -1;
  for (int i = 0; i < 64; ++i)
    if (cnt[i] == 0) {
      ilo = i;
      break;
    }
  bool pd = ilo >= 0 && cnt[64] == 0 && G > 0.0 && G < 1.0e300;
  if (!pd) {
    // not positive definite (or conditioned beyond 2^63): no logarithm to report
    if (tid == 0) *status = 4;
    return 0.0;
  }
  double xlo = ldexp(G, -ilo);
  double ulo = log(fmin(1.0, xlo)) - SLQ_PAD, uhi = log(fmax(1.0, G)) + SLQ_PAD;
  int N = (int)ceil((uhi - ulo) / SLQ_H) + 1;
  double acc = 0.0;
  for (int k = tid; k < N; k += SLQ_THREADS) {
    double sft = exp(ulo + SLQ_H * (double)k);
    double d = a[m - 1] + sft, below = 0.0;      // below: b_1^2 / delta_2
    for (int j = m - 2; j >= 0; --j) {
      below = b2[j] / d;
      d = a[j] + sft - below;
    }
    acc += sft * (a[0] - 1.0 - below) / ((1.0 + sft) * d);
  }
  red[tid] = acc;
  __syncthreads();
  for (int w = SLQ_THREADS / 2; w > 0; w >>= 1) {
    if (tid < w) red[tid] += red[tid + w];
    __syncthreads();
  }
  double term = rho0 * (SLQ_H * red[0]);
  if (tid == 0) *status = finite_d(term) ? 0 : 4;
  return term;
}

// One block per probe column: T from the CG coefficients (Observation in App. A),
// e_1^T log(T) e_1, times rho0.  Thread 0 of the last block to arrive forms the mean.
// EIG: by the eigen-decomposition of T (App. B) in thread 0; else by the quadrature above.
template <bool EIG>
__global__ __launch_bounds__(SLQ_THREADS) void k_slq(const double* __restrict__ alpha_hist,
                                                      const double* __restrict__ beta_hist, int t,
                                                      int sweeps_per_row, DevState* st) {
  __shared__ double a[BBMM_MAXP], b[BBMM_MAXP], w[BBMM_MAXP];
  __shared__ int cnt[65];
  int col = blockIdx.x + 1;
  int bad = 0;
  double term = 0.0;
  if (EIG) {
    if (threadIdx.x == 0)
      term = slq_term(alpha_hist + col, beta_hist + col, BBMM_MAXC, st->m_valid[col], st->rho0[col],
                      sweeps_per_row, a, b, w, &bad);
  } else {
    __shared__ int status_s;
    term = slq_term_quadrature(alpha_hist + col, beta_hist + col, BBMM_MAXC, st->m_valid[col], st->rho0[col],
                               a, b, w, cnt, &status_s);
    if (threadIdx.x == 0) bad = status_s;
  }
  if (threadIdx.x == 0) {
    st->slq_terms[blockIdx.x] = term;
    if (bad) st->status = bad;
  }
  if (!last_block_arrives(&st->counter[4][0])) return;
  if (threadIdx.x == 0) {
    double s = 0.0;
    for (int i = 0; i < t; ++i) s += st->slq_terms[i];
    st->slq_mean = s / (double)t;
    st->counter[4][0] = 0u;
  }
}

// The same term from coefficient arrays handed in by the caller: alpha, beta are p x t row-major
// (row j = iteration j), rho0 and m_valid have t entries; one block per probe column.
template <bool EIG>
__global__ __launch_bounds__(SLQ_THREADS) void k_slq_coeffs(const double* __restrict__ alpha,
                                                             const double* __restrict__ beta,
                                                             const double* __restrict__ rho0,
                                                             const int* __restrict__ m_valid, int t,
                                                             int sweeps_per_row, double* __restrict__ terms,
                                                             int* __restrict__ status) {
  __shared__ double a[BBMM_MAXP], b[BBMM_MAXP], w[BBMM_MAXP];
  __shared__ int cnt[65];
  int i = blockIdx.x;
  int bad = 0;
  double term = 0.0;
  if (EIG) {
    if (threadIdx.x == 0)
      term = slq_term(alpha + i, beta + i, (size_t)t, m_valid[i], rho0[i], sweeps_per_row, a, b, w, &bad);
  } else {
    __shared__ int status_s;
    term = slq_term_quadrature(alpha + i, beta + i, (size_t)t, m_valid[i], rho0[i], a, b, w, cnt, &status_s);
    if (threadIdx.x == 0) bad = status_s;
  }
  if (threadIdx.x == 0) {
    terms[i] = term;
    status[i] = bad;
  }
}

// Stand-alone batched eigen-solve (host arrays copied to the device by the caller).
// status[b] = 0, or 6 when matrix b did not deflate within the budget.
__global__ __launch_bounds__(64) void k_tridiag_eig(const double* __restrict__ diag,
                                                     const double* __restrict__ off, int m,
                                                     int sweeps_per_row,
                                                     double* __restrict__ eigvals,
                                                     double* __restrict__ first_row,
                                                     int* __restrict__ status) {
  __shared__ double a[BBMM_MAXP], b[BBMM_MAXP], w[BBMM_MAXP];
  if (threadIdx.x != 0) return;
  size_t bi = blockIdx.x;
  for (int j = 0; j < m; ++j) a[j] = diag[bi * m + j];
  for (int j = 0; j + 1 < m; ++j) b[j] = off[bi * (m - 1) + j];
  bool conv = tridiag_eig_first_row(a, b, w, m, sweeps_per_row);
  for (int j = 0; j < m; ++j) {
    eigvals[bi * m + j] = a[j];
    first_row[bi * m + j] = w[j];
  }
  status[bi] = conv ? 0 : 6;
}

// Noise-derivative terms (dK_hat/dsigma^2 = I): (1/t) sum_i u_i^T w_i and u_0^T u_0, plus y^T u_0.
// dk_out[2*slot], dk_out[2*slot+1] receive (trace, quad), dk_out[2*slot+2] = y^T u_0.
__global__ __launch_bounds__(VT) void k_noise_terms(const double* __restrict__ U,
                                                     const double* __restrict__ Z0,
                                                     const float* __restrict__ y, int n, int ld,
                                                     int t, int slot, DevState* st, double* partial,
                                                     double* gpartial) {
  __shared__ double r1[VT], r2[VT], r3[VT];
  __shared__ double tot[4];
  double tr = 0.0, qd = 0.0, yu = 0.0;
  int q = threadIdx.x % ld, rl = threadIdx.x / ld, rpp = VT / ld;
  for (int i = blockIdx.x * rpp + rl; i < n; i += gridDim.x * rpp) {
    double u = U[(size_t)i * ld + q];
    if (q == 0) {
      qd += u * u;
      yu += u * (double)y[i];
    } else if (q <= t) {
      tr += u * Z0[(size_t)i * ld + q];
    }
  }
  r1[threadIdx.x] = tr;
  r2[threadIdx.x] = qd;
  r3[threadIdx.x] = yu;
  __syncthreads();
  for (int w = VT / 2; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) {
      r1[threadIdx.x] += r1[threadIdx.x + w];
      r2[threadIdx.x] += r2[threadIdx.x + w];
      r3[threadIdx.x] += r3[threadIdx.x + w];
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    partial[(size_t)blockIdx.x * 4] = r1[0];
    partial[(size_t)blockIdx.x * 4 + 1] = r2[0];
    partial[(size_t)blockIdx.x * 4 + 2] = r3[0];
  }
  if (!reduce_blocks(partial, gpartial, 4, 3, st->counter[6], tot)) return;
  if (threadIdx.x == 0) {
    st->dk_out[2 * slot] = tot[0] / (double)t;
    st->dk_out[2 * slot + 1] = tot[1];
    st->dk_out[2 * slot + 2] = tot[2];
  }
}

inline int blocks_for(size_t count, int threads) { return (int)((count + threads - 1) / threads); }

}  // namespace

// ------------------------------------------------------------------ launchers
void launch_fill_f64(hipStream_t s, double* p, size_t count, double v) {
  if (!count) return;
  int nb = (int)((count + 255) / 256);
  if (nb > 4096) nb = 4096;
  k_fill_f64<<<nb, 256, 0, s>>>(p, count, v);
}

void launch_fill_bytes0(hipStream_t s, void* p, size_t bytes) {
  size_t count = bytes / 4;
  if (!count) return;
  int nb = (int)((count + 255) / 256);
  if (nb > 4096) nb = 4096;
  k_fill_u32<<<nb, 256, 0, s>>>((unsigned*)p, count);
}

void launch_fill_multi0(hipStream_t s, const ZeroSegs& z) {
  size_t most = 0;
  for (int k = 0; k < z.n; ++k) most = z.words[k] > most ? z.words[k] : most;
  if (!most) return;
  int nb = (int)((most + 255) / 256);
  if (nb > 4096) nb = 4096;
  k_fill_multi0<<<nb, 256, 0, s>>>(z);
}

void launch_colmean(hipStream_t s, const float* X, int n, int d, DevState* st, double* partial,
                    double* gpartial) {
  // grid stride must be a multiple of d: use nb blocks with nb * 256 % d == 0
  int nb = 64;
  while (((size_t)nb * VT) % d != 0) ++nb;      // d <= 64, terminates within d steps
  k_colmean<<<nb, VT, 0, s>>>(X, n, d, st, partial, gpartial);
}

void launch_prep_x(hipStream_t s, const float* X, int n, int d, int np, int KK, HypArgs hyp,
                   const DevState* st, float* Xa, float* Xb, float* Xs, float* X4, float* sq) {
  k_prep_x<<<blocks_for(np, 256), 256, 0, s>>>(X, n, d, np, KK, hyp, st, Xa, Xb, Xs, X4, sq);
}

void launch_pack_d4(hipStream_t s, const float* M, int n, int c, int np, int ld, double* D4) {
  k_pack_d4<<<blocks_for((size_t)np * ld, 256), 256, 0, s>>>(M, n, c, np, ld, D4);
}

void launch_unpack_rows(hipStream_t s, const double* src, int ld, int n, int c, float* dst) {
  k_unpack_rows<<<blocks_for((size_t)n * c, 256), 256, 0, s>>>(src, ld, n, c, dst);
}

void launch_unpack_rows_f64(hipStream_t s, const double* src, int ld, int n, int c, double* dst) {
  k_unpack_rows_f64<<<blocks_for((size_t)n * c, 256), 256, 0, s>>>(src, ld, n, c, dst);
}

void launch_pack_rows(hipStream_t s, const float* src, int n, int c, int ld, double* dst) {
  k_pack_rows<<<blocks_for((size_t)n * ld, 256), 256, 0, s>>>(src, n, c, ld, dst);
}

void launch_pack_cols_at(hipStream_t s, const float* src, int n, int c, int ld, int dstcol0, double* dst) {
  k_pack_cols_at<<<blocks_for((size_t)n * c, 256), 256, 0, s>>>(src, n, c, ld, dstcol0, dst);
}

void launch_copy_block(hipStream_t s, const float* src, size_t pw, size_t rows_p, int tri, int row0,
                       int nrows, int col0, int ncols, float* dst) {
  k_copy_block<<<blocks_for((size_t)nrows * ncols, 256), 256, 0, s>>>(src, pw, rows_p, tri, row0, nrows,
                                                                      col0, ncols, dst);
}

void launch_vreduce(hipStream_t s, const double* Vp, VpShape shape, int n, int np, int ld, double scaleV,
                    double addD, const double* D4, double* V) {
  k_vreduce<<<blocks_for((size_t)n * ld, 256), 256, 0, s>>>(Vp, shape, n, np, ld, scaleV, addD, D4, V);
}

void launch_warm_rhs(hipStream_t s, const float* u_init, int n, int ld, double* D4) {
  k_warm_rhs<<<(n + 255) / 256, 256, 0, s>>>(u_init, n, ld, D4);
}

void launch_warm_apply(hipStream_t s, const float* u_init, const double* V, int n, int ld, double* U,
                       double* R) {
  k_warm_apply<<<(n + 255) / 256, 256, 0, s>>>(u_init, V, n, ld, U, R);
}

void launch_pc_init(hipStream_t s, int n, HypArgs hyp, double* delta, DevState* st, double* arg_out,
                    int nblocks, const double* diag_in, int next_forced) {
  k_pc_init<<<nblocks, VT, 0, s>>>(n, hyp, delta, st, arg_out, diag_in, next_forced);
}

void launch_pc_step(hipStream_t s, const float* X, int n, int m, int kp, HypArgs hyp, double* delta,
                    double* L, DevState* st, const double* arg_in, double* arg_out, int nblocks,
                    const double* row_in, int row_ld, int forced, int next_forced) {
  double thresh = 1e-12 * hyp.outputscale;
  k_pc_step<<<nblocks, VT, 0, s>>>(X, n, m, kp, hyp, delta, L, st, arg_in, arg_out, thresh, row_in, row_ld,
                                   forced, next_forced);
}

void launch_pre_setup(hipStream_t s, const double* L, int n, int k, int kp, double noise, DevState* st,
                      double* partial, double* gpartial, int nblocks) {
  (void)k;
  k_pre_setup<<<nblocks, VT, 0, s>>>(L, n, kp, noise, st, partial, gpartial);
}

void launch_probes(hipStream_t s, const float* y, const float* E1, const float* E2, const double* L,
                   int n, int t, int kp, int ld, double noise, const DevState* st, double* R) {
  k_probes<<<blocks_for((size_t)n * ld, 256), 256, 0, s>>>(y, E1, E2, L, n, t, kp, ld, sqrt(noise), st, R);
}

__global__ void k_set_loop_scalars(DevState* st, double noise, double tol, double scaleV, double addD) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    st->loop_noise = noise;
    st->loop_tol = tol;
    st->loop_scaleV = scaleV;
    st->loop_addD = addD;
  }
}

void launch_set_loop_scalars(hipStream_t s, DevState* st, double noise, double tol, double scaleV, double addD) {
  k_set_loop_scalars<<<1, 64, 0, s>>>(st, noise, tol, scaleV, addD);
}

void launch_dv(hipStream_t s, const double* Vp, VpShape shape, int n, int np, int ld, double scaleV,
               double addD, const double* D4, double* V, const DevState* st, double* partial_dv,
               int nblocks) {
  if (shape.max_slots > 0 && shape.max_slots <= 2)
    k_dv<8, 2><<<nblocks, VT, 0, s>>>(Vp, shape, n, np, ld, scaleV, addD, D4, V, st, partial_dv);
  else
    k_dv<3, 8><<<nblocks, VT, 0, s>>>(Vp, shape, n, np, ld, scaleV, addD, D4, V, st, partial_dv);
}

#define DISPATCH_KP_T(KERNEL, kp, grid, threads, ...)                        \
  switch (kp) {                                                             \
    case 0: KERNEL<0><<<grid, threads, 0, s>>>(__VA_ARGS__); break;         \
    case 8: KERNEL<8><<<grid, threads, 0, s>>>(__VA_ARGS__); break;         \
    case 16: KERNEL<16><<<grid, threads, 0, s>>>(__VA_ARGS__); break;       \
    case 24: KERNEL<24><<<grid, threads, 0, s>>>(__VA_ARGS__); break;       \
    default: KERNEL<32><<<grid, threads, 0, s>>>(__VA_ARGS__); break;       \
  }
// kernels templated on the rank limit and on the block width in units of 16 columns
#define DISPATCH_KP_NQ(KERNEL, kp, nq, grid, threads, ...)                        \
  switch (kp) {                                                                  \
    case 0:                                                                      \
      if (nq == 1) KERNEL(0, 1)<<<grid, threads, 0, s>>>(__VA_ARGS__);           \
      else KERNEL(0, 2)<<<grid, threads, 0, s>>>(__VA_ARGS__);                   \
      break;                                                                     \
    case 8:                                                                      \
      if (nq == 1) KERNEL(8, 1)<<<grid, threads, 0, s>>>(__VA_ARGS__);           \
      else KERNEL(8, 2)<<<grid, threads, 0, s>>>(__VA_ARGS__);                   \
      break;                                                                     \
    case 16:                                                                     \
      if (nq == 1) KERNEL(16, 1)<<<grid, threads, 0, s>>>(__VA_ARGS__);          \
      else KERNEL(16, 2)<<<grid, threads, 0, s>>>(__VA_ARGS__);                  \
      break;                                                                     \
    case 24:                                                                     \
      if (nq == 1) KERNEL(24, 1)<<<grid, threads, 0, s>>>(__VA_ARGS__);          \
      else KERNEL(24, 2)<<<grid, threads, 0, s>>>(__VA_ARGS__);                  \
      break;                                                                     \
    default:                                                                     \
      if (nq == 1) KERNEL(32, 1)<<<grid, threads, 0, s>>>(__VA_ARGS__);          \
      else KERNEL(32, 2)<<<grid, threads, 0, s>>>(__VA_ARGS__);                  \
      break;                                                                     \
  }

// U, R update + partial sums (nb_ur blocks of 1024 threads), then the one-block finish.
void launch_ur(hipStream_t s, int init, int n, int ld, int c, int kp, double noise, double tol,
               const double* D4, const double* V, double* U, double* R, const double* L, DevState* st,
               const double* partial_dv, int nb_dv, double* partial, int nb_ur, int iter,
               double* alpha_hist, double* beta_hist, double* resid_hist) {
  int nq = ld / 16;
#define UR_MAIN(KP, NQ) k_ur_main<KP, NQ>
  DISPATCH_KP_NQ(UR_MAIN, kp, nq, nb_ur, UT, init, n, c, D4, V, U, R, L, st, partial_dv, nb_dv, partial);
#undef UR_MAIN
  DISPATCH_KP_T(k_ur_fin, kp, 1, UT, init, ld, c, noise, tol, st, partial, nb_ur, iter, alpha_hist,
                beta_hist, resid_hist);
}

void launch_zd(hipStream_t s, int init, int n, int ld, int kp, double noise, const double* R,
               const double* L, double* D4, double* Z0, DevState* st, int nblocks) {
  int nq = ld / 16;
  if (init) {
#define ZD_INIT(KP, NQ) k_zd<KP, NQ, 1>
    DISPATCH_KP_NQ(ZD_INIT, kp, nq, nblocks, VT, n, noise, R, L, D4, Z0, st);
#undef ZD_INIT
  } else {
#define ZD_ITER(KP, NQ) k_zd<KP, NQ, 0>
    DISPATCH_KP_NQ(ZD_ITER, kp, nq, nblocks, VT, n, noise, R, L, D4, Z0, st);
#undef ZD_ITER
  }
}

void launch_psolve_apply(hipStream_t s, int n, int ld, int kp, double noise, const double* R,
                         const double* L, double* Z, DevState* st, int nblocks) {
  int nq = ld / 16;
#define ZD_APPLY(KP, NQ) k_zd<KP, NQ, 2>
  DISPATCH_KP_NQ(ZD_APPLY, kp, nq, nblocks, VT, n, noise, R, L, (double*)nullptr, Z, st);
#undef ZD_APPLY
}

void launch_cross_block(hipStream_t s, const float* X, const float* Xs, int n, int ns, int ld, HypArgs hyp,
                        double* B) {
  k_cross_block<<<blocks_for((size_t)n * ld, 256), 256, 0, s>>>(X, Xs, n, ns, ld, hyp, B);
}

void launch_cross_dot(hipStream_t s, const float* X, const float* Xs, int n, int ns, HypArgs hyp,
                      const double* V, int ldv, int percol, double prior, double sign, float* out) {
  k_cross_dot<<<ns, VT, 0, s>>>(X, Xs, n, hyp, V, ldv, percol, prior, sign, out);
}

void launch_slq(hipStream_t s, const double* alpha_hist, const double* beta_hist, int t, int eig,
                int sweeps_per_row, DevState* st) {
  if (eig) k_slq<true><<<t, SLQ_THREADS, 0, s>>>(alpha_hist, beta_hist, t, sweeps_per_row, st);
  else k_slq<false><<<t, SLQ_THREADS, 0, s>>>(alpha_hist, beta_hist, t, sweeps_per_row, st);
}

void launch_slq_coeffs(hipStream_t s, const double* alpha, const double* beta, const double* rho0,
                       const int* m_valid, int t, int eig, int sweeps_per_row, double* terms, int* status) {
  if (eig) k_slq_coeffs<true><<<t, SLQ_THREADS, 0, s>>>(alpha, beta, rho0, m_valid, t, sweeps_per_row, terms, status);
  else k_slq_coeffs<false><<<t, SLQ_THREADS, 0, s>>>(alpha, beta, rho0, m_valid, t, sweeps_per_row, terms, status);
}

void launch_tridiag_eig(hipStream_t s, const double* diag, const double* off, int m, int batch,
                        int sweeps_per_row, double* eigvals, double* first_row, int* status) {
  k_tridiag_eig<<<batch, 64, 0, s>>>(diag, off, m, sweeps_per_row, eigvals, first_row, status);
}

void launch_noise_terms(hipStream_t s, const double* U, const double* Z0, const float* y, int n, int ld,
                        int t, int slot, DevState* st, double* partial, double* gpartial, int nblocks) {
  k_noise_terms<<<nblocks, VT, 0, s>>>(U, Z0, y, n, ld, t, slot, st, partial, gpartial);
}
