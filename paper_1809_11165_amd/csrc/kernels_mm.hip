// Kernel-matrix tile kernels for gfx950 (CDNA4): the O(n^2) part of BBMM.
//
//   * k_mm_mat   V = K_hat D from a materialised fp32 K_hat streamed once from HBM
//   * k_mm_otf   the same product with K_hat tiles rebuilt from X on the fly
//   * k_build_khat  materialises K_hat
//   * k_dk       derivative pass: sums of (dK/dtheta)_ij S_ij over all pairs
//
// All four work on 16 x 16 tiles held in the accumulator layout of
// v_mfma_f32_16x16x4_f32: lane l, register r  <->  tile element (row 4*(l/16)+r, col l%16).
// Squared distances come from the MFMA contraction  -2 x_i . x_j  plus |x_i|^2 + |x_j|^2
// on inputs that were centred and divided by the lengthscales beforehand; the kernel
// function is applied in registers; the tile is then used directly as the B operand
// of a second MFMA whose A operand is the right-hand-side block stored "quad-swizzled"
// (4 consecutive rows interleaved), so that both operands are single coalesced loads.
// Because K_hat is symmetric, a tile computed at (rows I, cols J) is used to accumulate
// the output rows J (contraction over I), which is what lets lanes own output columns.
#include "bbmm_dev.h"
#include "bbmm_kfun.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));

namespace {

__device__ inline f32x4 mfma16(float a, float b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
}

// fp64 MFMA 16x16x4: A[m = lane%16][k = lane/16], B[k = lane/16][n = lane%16] as for fp32, but the
// accumulator holds D[m = 4*r + lane/16][n = lane%16] in register r.  The product with the
// right-hand-side block is done in fp64 (kernel values converted on the fly) because the CG
// recurrences amplify fp32-level errors of this product beyond any useful parity bound.
__device__ inline f64x4 mfma16d(double a, double b, f64x4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// fp64 MFMA 4x4x4 (16 cycles, the same flop rate as the 16x16x4 one): the four diagonal 4 x 4 blocks
// of what that instruction would compute, C[i = lane/16][j = lane%4] of block p = (lane/4)%4
//   += sum_k A(lane 16 k + 4 p + i) * B(lane 16 k + 4 p + j)      (one register each; measured).
// With the B operand of the product unchanged and D[row][rhs 4q + lane%4] as A operand, three of
// them (q = 0, 1, 2) give right-hand-side columns 0..11 in 48 cycles instead of 64; the lane then
// holds out[column lane%16][rhs 4q + lane/16], i.e. element q of the 16x16 accumulator's four.
__device__ inline double mfma4d(double a, double b, double c) {
  return __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, c, 0, 0, 0);
}

// r2 tile: |xs_i - xs_j|^2 for a 16 x 16 tile.  The expansion |x|^2 + |x'|^2 - 2 x.x' can come out
// a rounding error below zero for near-identical points: the absolute value is taken (as good a
// guess as a clamp at zero for what is rounding noise either way, and free: an operand modifier
// of the instruction that consumes it).
template <int KK>
__device__ inline f32x4 tile_r2(const float (&a)[KK], const float (&b)[KK], f32x4 sqi, float sqj) {
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) acc = mfma16(a[kk], b[kk], acc);
  f32x4 r2;
#pragma unroll
  for (int r = 0; r < 4; ++r) r2[r] = __builtin_fabsf(acc[r] + (sqi[r] + sqj));
  return r2;
}

// exact zero distance on the diagonal of a diagonal tile
__device__ inline f32x4 fix_diag(f32x4 r2, int lane) {
  int jc = lane & 15, ib = (lane >> 4) * 4;
#pragma unroll
  for (int r = 0; r < 4; ++r)
    if (ib + r == jc) r2[r] = 0.f;
  return r2;
}

// The same on a condition that is uniform over the wave and true for one tile in thousands: kept
// as a real branch (the empty volatile statement cannot be executed speculatively); turned into
// selects it costs two vector instructions per value in every tile.
__device__ __forceinline__ f32x4 fix_diag_if(bool diag_tile, f32x4 r2, int lane) {
  if (diag_tile) {
    asm volatile("");
    r2 = fix_diag(r2, lane);
  }
  return r2;
}

// --------------------------------------------------------- materialise K_hat --
// One wave: column block jb (16 columns) x 4 row blocks, each tile kept for its transposed position
// (K is symmetric), so the wave owns 16 rows x 64 adjacent columns of K_hat.  The four tiles pass
// through a 16 x 64 LDS area of the wave and come back one row per 16 lanes: every store
// instruction then writes 4 rows x 256 contiguous bytes (straight from the accumulator layout it
// would write 16 rows x 64 bytes, which the memory system takes at 2.5 TB/s only).
constexpr int BK_TLD = 68;   // floats per row of the wave's area (64 + 4: both accesses conflict-free)

template <int KIND, int KK>
__global__ __launch_bounds__(256) void k_build_khat(const float* __restrict__ Xa,
                                                     const float* __restrict__ Xb,
                                                     const float* __restrict__ sq, int n, int np,
                                                     int pw, int tri, float outputscale,
                                                     float noise, float* __restrict__ Khat) {
  __shared__ __align__(16) float T[4][16 * BK_TLD];
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int jb = blockIdx.y * 4 + wave;
  int jc = lane & 15, g = lane >> 4;
  // triangular storage: panel P keeps rows [0, (P+1) pw) only (pw is a multiple of 64, so the four
  // row blocks of this wave lie in one panel)
  int col0 = blockIdx.x * 64;
  if (tri && jb * 16 >= (col0 / pw + 1) * pw) return;
  float* Tw = T[wave];
  float b[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) b[kk] = Xb[((size_t)jb * KK + kk) * 64 + lane];
  float sqj = sq[jb * 16 + jc];
  int j = jb * 16 + jc;
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    int ib = blockIdx.x * 4 + u;
    float a[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) a[kk] = Xa[((size_t)ib * KK + kk) * 64 + lane];
    f32x4 sqi = *(const f32x4*)(sq + ib * 16 + g * 4);
    f32x4 r2 = tile_r2<KK>(a, b, sqi, sqj);
    r2 = fix_diag_if(ib == jb, r2, lane);
    f32x4 out;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int i = ib * 16 + g * 4 + r;
      float v = outputscale * unit_kernel<KIND>(r2[r]);
      if (i == j) v += noise;
      if (i >= n || j >= n) v = 0.f;
      out[r] = v;
    }
    // K_hat[row j][columns 16 u + 4 g .. + 3 of the wave's 64]
    *(f32x4*)(Tw + jc * BK_TLD + 16 * u + 4 * g) = out;
  }
  __builtin_amdgcn_wave_barrier();   // (a wave's LDS operations execute in order)
  // column panels of width pw, each row-major (pw == np: plain row-major); the panels of the
  // triangular storage follow each other without the rows they leave out
  size_t P = (size_t)(col0 / pw);
  size_t poff = tri ? (size_t)pw * pw * (P * (P + 1) / 2) : P * np * pw;
  float* dst = Khat + poff + (size_t)(col0 % pw) + (size_t)(4 * jc);
#pragma unroll
  for (int s4 = 0; s4 < 4; ++s4) {
    int row = 4 * s4 + g;
    f32x4 v = *(const f32x4*)(Tw + row * BK_TLD + 4 * jc);
    __builtin_nontemporal_store(v, (f32x4*)(dst + (size_t)(jb * 16 + row) * pw));
  }
}

// ------------------------------------------------ product from a stored K_hat --
// Wave: 64*NC output columns, a chunk of K_hat rows.  Per 16-row step each lane loads
// 4 rows x 4 consecutive columns per column group (row 4*(l/16)+r, columns 4*(l%16)..+3):
// element (r, cc) of that load, converted to fp64, is the B operand of one fp64 MFMA whose A
// operand is the quad-swizzled fp64 right-hand side.  Result partials go to Vp[split]; a lane's
// four accumulator values (block columns l/16, 4+l/16, 8+l/16, 12+l/16) are stored contiguously.
//
// The loads run one 16-row step ahead of the arithmetic: as soon as the MFMAs of one load's
// registers are issued, the same registers receive the load for the next step, so every wave
// keeps 16*NC KB in flight while its MFMAs run.
// NARROW (NQ = 1, at most 12 columns of the block in use): the product runs on the fp64 4x4x4 MFMA
// (see mfma4d): three right-hand-side operands D[row][4q + lane%4], q = 0..2, per row quad, three
// scalar accumulators per 4 matrix columns, 48 matrix-pipe cycles per element instead of 64.
template <int NQ, bool NARROW>
__device__ __forceinline__ void mm_mat_load_d(const double* __restrict__ D4, int j0, int jc, int g,
                                              f64x4 (&dop)[NARROW ? 3 : NQ]) {
  constexpr int LD = 16 * NQ;
  if (NARROW) {
#pragma unroll
    for (int q = 0; q < 3; ++q)
      dop[q] = *(const f64x4*)(D4 + ((size_t)(j0 / 4 + g) * LD + (size_t)(4 * q + (jc & 3))) * 4);
  } else {
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
      dop[nq] = *(const f64x4*)(D4 + ((size_t)(j0 / 4 + g) * LD + (size_t)(nq * 16 + jc)) * 4);
  }
}

// One 16-row step.  kv / dop hold this step's operands on entry and the next step's on exit
// (MORE); the right-hand-side operand of the next step is requested first because memory
// results return in issue order.
template <int NQ, int NC, bool MORE, bool NARROW>
__device__ __forceinline__ void mm_mat_step(const float* __restrict__ knext,
                                            const double* __restrict__ D4, int jnext, int ldk, int jc,
                                            int g, f32x4 (&kv)[NC][4], f64x4 (&dop)[NARROW ? 3 : NQ],
                                            f64x4 (&acc)[NC][4][NQ], double (&accn)[NC][4][3]) {
  constexpr int ND = NARROW ? 3 : NQ;
  f64x4 dcur[ND];
#pragma unroll
  for (int nq = 0; nq < ND; ++nq) dcur[nq] = dop[nq];
  if (MORE) mm_mat_load_d<NQ, NARROW>(D4, jnext, jc, g, dop);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int nc = 0; nc < NC; ++nc) {
      double kd[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) kd[cc] = (double)kv[nc][r][cc];
      // the registers are free once converted: refill them before the MFMAs are issued
      if (MORE) kv[nc][r] = __builtin_nontemporal_load((const f32x4*)(knext + (size_t)r * ldk + nc * 64));
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        if (NARROW) {
#pragma unroll
          for (int q = 0; q < 3; ++q) accn[nc][cc][q] = mfma4d(dcur[q][r], kd[cc], accn[nc][cc][q]);
        } else {
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) acc[nc][cc][nq] = mfma16d(dcur[nq][r], kd[cc], acc[nc][cc][nq]);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    }
}

// Workgroup = 4 waves on 256*NC adjacent columns (one strip); it runs the pieces of its plan
// entry one after the other.  All workgroups get the same number of 16-row steps (+-1), so the
// launch ends without a tail however strips and compute units divide.
//
// Matrix layout: element (row, col) lies at  (col / pw) * panel_stride + row * ldk + col % pw.
// Plain row-major: pw >= np, ldk = np.  Column panels of width pw (a multiple of 256), each
// panel row-major with ldk = pw: a matrix with few, very long rows (the transposed SGPR root:
// 1024 x 500,000) then keeps the 16 rows of a step within 16 * pw * 4 bytes instead of one
// memory page per row.
template <int NQ, int NC, bool NARROW>
__global__ __launch_bounds__(256, 2) void k_mm_mat(const float* __restrict__ Khat,
                                                    const double* __restrict__ D4,
                                                    double* __restrict__ Vp, int np, int pw,
                                                    size_t panel_stride, int ldk,
                                                    const MmPlan* __restrict__ plan,
                                                    const DevState* __restrict__ st) {
  static_assert(!NARROW || NQ == 1, "the narrow product covers one group of 12 columns");
  if (st->done) return;
  constexpr int LD = 16 * NQ;
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int jc = lane & 15, g = lane >> 4;
#pragma unroll 1
  for (int pc = 0; pc < BBMM_MM_PIECES; ++pc) {
    MmPiece P = plan[blockIdx.x].piece[pc];
    int j_begin = P.row_begin, j_end = P.row_end;
    int col0 = (P.strip * 4 + wave) * (64 * NC);
    if (j_begin >= j_end || col0 >= np) continue;
    f64x4 acc[NC][4][NQ];
    double accn[NC][4][3];
#pragma unroll
    for (int nc = 0; nc < NC; ++nc)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) acc[nc][cc][nq] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int q = 0; q < 3; ++q) accn[nc][cc][q] = 0.0;
      }

    const float* kp = Khat + (size_t)(col0 / pw) * panel_stride + (size_t)(j_begin + g * 4) * ldk +
                      (size_t)(col0 % pw + 4 * jc);
    f32x4 kv[NC][4];
    f64x4 dop[NARROW ? 3 : NQ];
    mm_mat_load_d<NQ, NARROW>(D4, j_begin, jc, g, dop);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int nc = 0; nc < NC; ++nc)
        kv[nc][r] = __builtin_nontemporal_load((const f32x4*)(kp + (size_t)r * ldk + nc * 64));
    int j0 = j_begin;
    for (; j0 + 16 < j_end; j0 += 16) {
      kp += (size_t)16 * ldk;
      mm_mat_step<NQ, NC, true, NARROW>(kp, D4, j0 + 16, ldk, jc, g, kv, dop, acc, accn);
    }
    mm_mat_step<NQ, NC, false, NARROW>(kp, D4, j0, ldk, jc, g, kv, dop, acc, accn);

    double* vout = Vp + (size_t)P.slot * np * LD;
#pragma unroll
    for (int nc = 0; nc < NC; ++nc)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc)
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
          *(f64x4*)(vout + (size_t)(col0 + nc * 64 + 4 * jc + cc) * LD + nq * 16 + g * 4) =
              NARROW ? (f64x4){accn[nc][cc][0], accn[nc][cc][1], accn[nc][cc][2], 0.0} : acc[nc][cc][nq];
  }
}

// ------------------------------------------------------- product on the fly ---
// Wave: NJ column blocks (16*NJ output rows of V), a chunk of row blocks to contract over.
// Distances by fp32 MFMA, kernel function in registers, product with the block by fp64 MFMA.
// Writes partial sums of (K/s) D; the caller scales by s and adds sigma^2 D.
//
// NQ groups of 16 right-hand-side columns go through the fp64 MFMA.  NX further columns
// (16*NQ .. 16*NQ+NX-1) are accumulated with plain fp64 FMAs instead: on this chip an fp64 MFMA
// runs at the rate of the fp64 vector unit, so a 17th column costs 4 FMAs per tile and lane this
// way against a whole second MFMA group (4 x 64 cycles) of which 15/16 would be padding.  A lane
// then holds the sum over its own 4 rows of each tile; the four lane groups are added at the end
// and stored where the MFMA path would have put them.
//
// NARROW (NQ = 1, NX = 0, at most 12 columns in use): the product runs on the 4x4x4 MFMA.
template <int KIND, int KK, int NQ, int NJ, int NX, bool NARROW = false>
__global__ __launch_bounds__(256) void k_mm_otf(const float* __restrict__ Xa,
                                                 const float* __restrict__ Xb,
                                                 const float* __restrict__ sq,
                                                 const double* __restrict__ D4,
                                                 double* __restrict__ Vp, int np, int nsplit,
                                                 int blocks_per_split,
                                                 const DevState* __restrict__ st) {
  if (st->done) return;
  static_assert(NX >= 0 && NX <= 4, "at most 4 columns on the vector unit");
  static_assert(!NARROW || (NQ == 1 && NX == 0), "the narrow product covers one group of 12 columns");
  constexpr int LD = 16 * (NQ + (NX > 0 ? 1 : 0));
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int nblk = np >> 4;
  int split = blockIdx.x % nsplit;
  int sstrip = blockIdx.x / nsplit;
  int jb0 = (sstrip * 4 + wave) * NJ;
  if (jb0 >= nblk) return;
  int jc = lane & 15, g = lane >> 4;
  float b[NJ][KK];
  float sqj[NJ];
  f64x4 acc[NJ][NQ];
  double accn[NJ][3];
  double accx[NJ][NX > 0 ? NX : 1];
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) b[jb][kk] = Xb[((size_t)(jb0 + jb) * KK + kk) * 64 + lane];
    sqj[jb] = sq[(jb0 + jb) * 16 + jc];
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) acc[jb][nq] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int q = 0; q < 3; ++q) accn[jb][q] = 0.0;
#pragma unroll
    for (int x = 0; x < NX; ++x) accx[jb][x] = 0.0;
  }
  int ib_begin = split * blocks_per_split;
  int ib_end = min(nblk, ib_begin + blocks_per_split);
  for (int ib = ib_begin; ib < ib_end; ++ib) {
    float a[KK];
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) a[kk] = Xa[((size_t)ib * KK + kk) * 64 + lane];
    f32x4 sqi = *(const f32x4*)(sq + ib * 16 + g * 4);
    f64x4 dop[NARROW ? 3 : NQ];
    f64x4 dx[NX > 0 ? NX : 1];
    if (NARROW) {
#pragma unroll
      for (int q = 0; q < 3; ++q)
        dop[q] = *(const f64x4*)(D4 + ((size_t)(ib * 4 + g) * LD + (size_t)(4 * q + (jc & 3))) * 4);
    } else {
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq)
        dop[nq] = *(const f64x4*)(D4 + ((size_t)(ib * 4 + g) * LD + (size_t)(nq * 16 + jc)) * 4);
    }
#pragma unroll
    for (int x = 0; x < NX; ++x)   // rows 4g..4g+3 of column 16 NQ + x (the same for all jc)
      dx[x] = *(const f64x4*)(D4 + ((size_t)(ib * 4 + g) * LD + (size_t)(NQ * 16 + x)) * 4);
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb) {
      f32x4 r2 = tile_r2<KK>(a, b[jb], sqi, sqj[jb]);
      r2 = fix_diag_if(ib == jb0 + jb, r2, lane);
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        double e = (double)unit_kernel<KIND>(r2[r]);
        if (NARROW) {
#pragma unroll
          for (int q = 0; q < 3; ++q) accn[jb][q] = mfma4d(dop[q][r], e, accn[jb][q]);
        } else {
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) acc[jb][nq] = mfma16d(dop[nq][r], e, acc[jb][nq]);
        }
#pragma unroll
        for (int x = 0; x < NX; ++x) accx[jb][x] = fma(e, dx[x][r], accx[jb][x]);
      }
    }
  }
  double* vout = Vp + (size_t)split * np * LD;
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
      *(f64x4*)(vout + (size_t)((jb0 + jb) * 16 + jc) * LD + nq * 16 + g * 4) =
          NARROW ? (f64x4){accn[jb][0], accn[jb][1], accn[jb][2], 0.0} : acc[jb][nq];
    if (NX > 0) {
      // column 16 NQ + x belongs at position 4 x of the last group (the order the MFMA path
      // stores its columns in): lane group g writes positions 4g..4g+3, i.e. column g and zeros
      double mine = 0.0;
#pragma unroll
      for (int x = 0; x < NX; ++x) {
        double v = accx[jb][x];
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        if (g == x) mine = v;
      }
      *(f64x4*)(vout + (size_t)((jb0 + jb) * 16 + jc) * LD + NQ * 16 + g * 4) =
          (f64x4){mine, 0.0, 0.0, 0.0};
    }
  }
}

// ------------------------------------- product on the fly, each tile pair once --
// K is symmetric, so tile (I, J) is tile (J, I) transposed: only the strips' tiles on and above the
// diagonal are evaluated, and a tile above it serves both  out[J] += T^T D[I]  (as in k_mm_otf) and
// out[I] += T D[J].  Work division as for the stored triangle (launch_mm_sym), with panels of
// BBMM_OTF_PANEL = 512 columns (4 waves x 8 column blocks): a piece is a run of 16-row blocks of one
// panel, either above its diagonal block (DUAL: both uses) or inside it (the whole square block is
// evaluated, column-side use only).  The second use needs the tile with rows across lane%16: the
// wave writes its four values per lane to a private LDS tile [column][row] (one 16-byte write) and
// reads K[row lane%16][column 4 (lane/16) + s], s = 0..3, back; the A operand D[J] (one f64x4 per
// column block and lane) is loaded once per piece.  The row-side sums of a row block (16 x 16 per
// wave, over its 128 columns) are staged in LDS; every OT_GROUP row blocks the four waves' parts are
// added in a fixed order and written to the slot  slot_base[s] + P - s - 1  of output panel s.
// NARROW: at most 12 columns in use, column-side use on the 4x4x4 MFMA (see mfma4d).
constexpr int OT_NJ = 8;
constexpr int OT_GROUP = 4;
constexpr int OT_PLD = 18;      // doubles per staged row (16 + 2: conflict-free 32-byte stores)
constexpr int OT_TLD = 20;      // floats per column of the transposition tile (16 + 4)
static_assert(BBMM_OTF_PANEL == 4 * OT_NJ * 16, "a workgroup of four waves covers one panel");
typedef double f64x4s __attribute__((ext_vector_type(4), aligned(16)));   // as laid out in LDS

template <int KIND, int KK, bool NARROW, bool DUAL>
__global__ __launch_bounds__(256, 2) void k_mm_otf_tri(const float* __restrict__ Xa,
                                                        const float* __restrict__ Xb,
                                                        const float* __restrict__ sq,
                                                        const double* __restrict__ D4,
                                                        double* __restrict__ Vp, int np,
                                                        const MmPiece* __restrict__ pieces,
                                                        const int* __restrict__ first,
                                                        const int* __restrict__ slot_base,
                                                        const DevState* __restrict__ st) {
  if (st->done) return;
  constexpr int LD = 16;
  __shared__ __align__(16) float T[DUAL ? 4 : 1][DUAL ? 16 * OT_TLD : 4];
  __shared__ __align__(16) double S[DUAL ? 4 : 1][DUAL ? 16 * OT_GROUP * OT_PLD : 2];
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int jc = lane & 15, g = lane >> 4;
  float* Tw = T[DUAL ? wave : 0];
  double* Sw = S[DUAL ? wave : 0];
  int pb = first[blockIdx.x], pe = first[blockIdx.x + 1];
#pragma unroll 1
  for (int pc = pb; pc < pe; ++pc) {
    MmPiece P = pieces[pc];
    int jb0 = (P.strip * 4 + wave) * OT_NJ;
    bool active = jb0 * 16 < np;
    int ib_begin = P.row_begin >> 4, ib_end = P.row_end >> 4;
    if (ib_begin >= ib_end) continue;
    float b[OT_NJ][KK];
    float sqj[OT_NJ];
    f64x4 acc[OT_NJ];
    double accn[OT_NJ][3];
    f64x4 dJ[OT_NJ];
#pragma unroll
    for (int jb = 0; jb < OT_NJ; ++jb) {
      acc[jb] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
      for (int q = 0; q < 3; ++q) accn[jb][q] = 0.0;
      if (active) {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) b[jb][kk] = Xb[((size_t)(jb0 + jb) * KK + kk) * 64 + lane];
        sqj[jb] = sq[(jb0 + jb) * 16 + jc];
        // columns 16 (jb0+jb) + 4 g + s, s = 0..3, right-hand side jc
        if (DUAL) dJ[jb] = *(const f64x4*)(D4 + ((size_t)((jb0 + jb) * 4 + g) * LD + (size_t)jc) * 4);
      }
    }
    if (DUAL && !active) {
      // a wave whose columns lie beyond the matrix stages nothing in this piece: its area must read
      // as zero in the flushes (the barrier that ended the previous flush has passed)
      for (int i = lane; i < 16 * OT_GROUP * OT_PLD; i += 64) Sw[i] = 0.0;
    }
#pragma unroll 1
    for (int ig = ib_begin; ig < ib_end; ig += OT_GROUP) {
      int ng = min(OT_GROUP, ib_end - ig);
      if (active) {
#pragma unroll 1
        for (int qi = 0; qi < ng; ++qi) {
          int ib = ig + qi;
          float a[KK];
#pragma unroll
          for (int kk = 0; kk < KK; ++kk) a[kk] = Xa[((size_t)ib * KK + kk) * 64 + lane];
          f32x4 sqi = *(const f32x4*)(sq + ib * 16 + g * 4);
          f64x4 dop[NARROW ? 3 : 1];
          if (NARROW) {
#pragma unroll
            for (int q = 0; q < 3; ++q)
              dop[q] = *(const f64x4*)(D4 + ((size_t)(ib * 4 + g) * LD + (size_t)(4 * q + (jc & 3))) * 4);
          } else {
            dop[0] = *(const f64x4*)(D4 + ((size_t)(ib * 4 + g) * LD + (size_t)jc) * 4);
          }
          f64x4 acc2[2];
          acc2[0] = (f64x4){0.0, 0.0, 0.0, 0.0};
          acc2[1] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
          for (int jb = 0; jb < OT_NJ; ++jb) {
            f32x4 r2 = tile_r2<KK>(a, b[jb], sqi, sqj[jb]);
            if (!DUAL) r2 = fix_diag_if(ib == jb0 + jb, r2, lane);
            f32x4 e;
#pragma unroll
            for (int r = 0; r < 4; ++r) e[r] = unit_kernel<KIND>(r2[r]);
#pragma unroll
            for (int r = 0; r < 4; ++r) {
              double ed = (double)e[r];
              if (NARROW) {
#pragma unroll
                for (int q = 0; q < 3; ++q) accn[jb][q] = mfma4d(dop[q][r], ed, accn[jb][q]);
              } else {
                acc[jb] = mfma16d(dop[0][r], ed, acc[jb]);
              }
            }
            if (DUAL) {
              *(f32x4*)(Tw + jc * OT_TLD + 4 * g) = e;          // [column jc][rows 4g .. 4g+3]
              __builtin_amdgcn_wave_barrier();
              float kt[4];
#pragma unroll
              for (int s = 0; s < 4; ++s) kt[s] = Tw[(4 * g + s) * OT_TLD + jc];   // K[row jc][column 4g+s]
              __builtin_amdgcn_wave_barrier();
#pragma unroll
              for (int s = 0; s < 4; ++s) acc2[s & 1] = mfma16d(dJ[jb][s], (double)kt[s], acc2[s & 1]);
            }
          }
          if (DUAL) *(f64x4s*)(Sw + (qi * 16 + jc) * OT_PLD + 4 * g) = acc2[0] + acc2[1];
        }
      }
      if (DUAL) {
        __syncthreads();
        int rl = threadIdx.x >> 1, half = threadIdx.x & 1;
        if (rl < ng * 16) {
          int row = ig * 16 + rl;
          const double* sp = &S[0][0] + rl * OT_PLD + 8 * half;
          f64x4 lo = *(const f64x4s*)sp, hi = *(const f64x4s*)(sp + 4);
#pragma unroll
          for (int w = 1; w < 4; ++w) {
            lo += *(const f64x4s*)(sp + w * (16 * OT_GROUP * OT_PLD));
            hi += *(const f64x4s*)(sp + w * (16 * OT_GROUP * OT_PLD) + 4);
          }
          int so = row / BBMM_OTF_PANEL;
          int slot = slot_base[so] + (P.strip - so - 1);
          double* dst = Vp + ((size_t)slot * np + (size_t)row) * LD + 8 * half;
          *(f64x4*)dst = lo;
          *(f64x4*)(dst + 4) = hi;
        }
        __syncthreads();
      }
    }
    if (active) {
      double* vout = Vp + (size_t)P.slot * np * LD;
#pragma unroll
      for (int jb = 0; jb < OT_NJ; ++jb)
        *(f64x4*)(vout + (size_t)((jb0 + jb) * 16 + jc) * LD + g * 4) =
            NARROW ? (f64x4){accn[jb][0], accn[jb][1], accn[jb][2], 0.0} : acc[jb];
    }
  }
}

// ------------------------------------------------------------ derivative pass --
// For every pair (i, j):  S_ij = sum_c SA[i][c] SB[j][c]  (the probe outer products, divided by t
// and symmetrised by the caller) and Q_ij = u0_i u0_j.  Accumulates
//     sum_ij E_ij S_ij,  sum_ij E_ij Q_ij                         (outputscale)
//   isotropic:  sum_ij g_ij r2_ij S_ij,  sum_ij g_ij r2_ij Q_ij   (lengthscale)
//   ARD:        per dimension  sum_ij T_ij (xs_id - xs_jd)^2,  T = g o S (and g o Q), evaluated per
//               tile as  sum_j [ xs_jd^2 c_j + Y2_jd - 2 xs_jd Y_jd ],  c_j = sum_i T_ij,
//               Y_jd = sum_i T_ij xs_id,  Y2_jd = sum_i T_ij xs_id^2  (two MFMA contractions).
// Every summand is symmetric in (i, j), so only tiles with row block <= column block are
// evaluated: weight 1 above the diagonal, 1/2 on it, and the total is doubled at the end.
// Partial results: one row of `pstride` doubles per wave: [2*h] trace-type, [2*h+1] quad-type,
// h = lengthscale slots (1 or 4*KK) then the outputscale slot.
constexpr int DK_NJ = 4;
constexpr int DK_TSMAX = 16;

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

template <int KK, int ARD>
struct DkAcc {
  static constexpr int MB = (4 * KK + 15) / 16;
  float es_tr = 0.f, es_q = 0.f, el_tr = 0.f, el_q = 0.f;
  f32x4 ytr[DK_NJ][ARD ? MB : 1], yq[DK_NJ][ARD ? MB : 1], y2tr[DK_NJ][ARD ? MB : 1],
      y2q[DK_NJ][ARD ? MB : 1];
  float ctr[DK_NJ], cq[DK_NJ];
};

// One row block ib against the wave's DK_NJ column blocks.  NEAR: the row block lies inside the
// wave's own column range, so the tile weights (1, 1/2, 0) differ per column block.
template <int KIND, int KK, int ARD, bool NEAR>
__device__ __forceinline__ void dk_step(int ib, int jb0, int lane, int TS, const float* __restrict__ Xa,
                                        const float* __restrict__ sq, const float* __restrict__ X4,
                                        const float* __restrict__ SA, const float* __restrict__ u0,
                                        const float* __restrict__ sb_lds, const float (&b)[DK_NJ][KK],
                                        const float (&sqj)[DK_NJ], const float (&u0j)[DK_NJ],
                                        DkAcc<KK, ARD>& A) {
  constexpr int DP = 4 * KK;
  constexpr int MB = (DP + 15) / 16;
  constexpr int NJ = DK_NJ;
  int jc = lane & 15, g = lane >> 4;
  float a[KK];
#pragma unroll
  for (int kk = 0; kk < KK; ++kk) a[kk] = Xa[((size_t)ib * KK + kk) * 64 + lane];
  f32x4 sqi = *(const f32x4*)(sq + ib * 16 + g * 4);
  f32x4 u0i = *(const f32x4*)(u0 + ib * 16 + g * 4);
  f32x4 xop[ARD ? MB : 1], xop2[ARD ? MB : 1];
  if (ARD) {
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
      int dim = mb * 16 + jc;
      xop[mb] = (dim < DP) ? *(const f32x4*)(X4 + ((size_t)(ib * 4 + g) * DP + dim) * 4)
                           : (f32x4){0.f, 0.f, 0.f, 0.f};
      xop2[mb] = xop[mb] * xop[mb];
    }
  }
  // S tiles for all column blocks: contraction over the probe index, TS chunks of 4
  f32x4 S[NJ];
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) S[jb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const float* sap = SA + (size_t)ib * TS * 64 + lane;
  float sa_next = sap[0];
  for (int kk = 0; kk < TS; ++kk) {
    float sa = sa_next;
    if (kk + 1 < TS) sa_next = sap[(kk + 1) * 64];
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb) S[jb] = mfma16(sa, sb_lds[(jb * TS + kk) * 64 + lane], S[jb]);
  }
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
    float wt = 1.f;
    if (NEAR) {
      int jbg = jb0 + jb;
      wt = (ib < jbg) ? 1.f : ((ib == jbg) ? 0.5f : 0.f);
    }
    f32x4 r2 = tile_r2<KK>(a, b[jb], sqi, sqj[jb]);
    if (NEAR) r2 = fix_diag_if(ib == jb0 + jb, r2, lane);
    f32x4 ts, tq;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      float e, gw;
      unit_kernel_and_weight<KIND>(r2[r], e, gw);
      if (NEAR) {
        e *= wt;
        gw *= wt;
      }
      float q = u0i[r] * u0j[jb];
      A.es_tr = fmaf(e, S[jb][r], A.es_tr);
      A.es_q = fmaf(e, q, A.es_q);
      if (ARD) {
        ts[r] = gw * S[jb][r];
        tq[r] = gw * q;
        A.ctr[jb] += ts[r];
        A.cq[jb] += tq[r];
      } else {
        float w = gw * r2[r];
        A.el_tr = fmaf(w, S[jb][r], A.el_tr);
        A.el_q = fmaf(w, q, A.el_q);
      }
    }
    if (ARD) {
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          A.ytr[jb][mb] = mfma16(xop[mb][r], ts[r], A.ytr[jb][mb]);
          A.yq[jb][mb] = mfma16(xop[mb][r], tq[r], A.yq[jb][mb]);
          A.y2tr[jb][mb] = mfma16(xop2[mb][r], ts[r], A.y2tr[jb][mb]);
          A.y2q[jb][mb] = mfma16(xop2[mb][r], tq[r], A.y2q[jb][mb]);
        }
    }
  }
}

template <int KIND, int KK, int ARD>
__global__ __launch_bounds__(256) void k_dk(const float* __restrict__ Xa,
                                             const float* __restrict__ Xb,
                                             const float* __restrict__ sq,
                                             const float* __restrict__ Xs,
                                             const float* __restrict__ X4,
                                             const float* __restrict__ SA,
                                             const float* __restrict__ SB, int TS,
                                             const float* __restrict__ u0, int np, int nsplit,
                                             int blocks_per_split, double* __restrict__ partial,
                                             int pstride) {
  extern __shared__ float dk_lds[];   // [wave][NJ][TS][64]: the wave's SB operands
  constexpr int DP = 4 * KK;
  constexpr int MB = (DP + 15) / 16;
  constexpr int NJ = DK_NJ;
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int nblk = np >> 4;
  int split = blockIdx.x % nsplit;
  int sstrip = blockIdx.x / nsplit;
  int jb0 = (sstrip * 4 + wave) * NJ;
  size_t wave_id = (size_t)blockIdx.x * 4 + wave;
  double* pout = partial + wave_id * pstride;
  // row blocks of this chunk that lie on or above the diagonal of the wave's column blocks
  int ib_begin = split * blocks_per_split;
  int ib_end = min(min(nblk, ib_begin + blocks_per_split), jb0 + NJ);
  if (jb0 >= nblk || ib_begin >= ib_end) {
    for (int e = lane; e < pstride; e += 64) pout[e] = 0.0;
    return;
  }
  int jc = lane & 15, g = lane >> 4;
  float* sb_lds = dk_lds + (size_t)wave * NJ * TS * 64;
  float b[NJ][KK], sqj[NJ], u0j[NJ];
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) b[jb][kk] = Xb[((size_t)(jb0 + jb) * KK + kk) * 64 + lane];
    for (int kk = 0; kk < TS; ++kk)
      sb_lds[(jb * TS + kk) * 64 + lane] = SB[((size_t)(jb0 + jb) * TS + kk) * 64 + lane];
    sqj[jb] = sq[(jb0 + jb) * 16 + jc];
    u0j[jb] = u0[(jb0 + jb) * 16 + jc];
  }
  DkAcc<KK, ARD> A;
#pragma unroll
  for (int jb = 0; jb < NJ; ++jb) {
    A.ctr[jb] = 0.f;
    A.cq[jb] = 0.f;
#pragma unroll
    for (int mb = 0; mb < (ARD ? MB : 1); ++mb) {
      A.ytr[jb][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
      A.yq[jb][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
      A.y2tr[jb][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
      A.y2q[jb][mb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    }
  }
  int ib = ib_begin;
  int far_end = min(ib_end, jb0);
  for (; ib < far_end; ++ib)
    dk_step<KIND, KK, ARD, false>(ib, jb0, lane, TS, Xa, sq, X4, SA, u0, sb_lds, b, sqj, u0j, A);
  for (; ib < ib_end; ++ib)
    dk_step<KIND, KK, ARD, true>(ib, jb0, lane, TS, Xa, sq, X4, SA, u0, sb_lds, b, sqj, u0j, A);

  // ---- wave-level epilogue (the factor 2 restores the tiles below the diagonal) -------
  int nls = ARD ? DP : 1;
  if (ARD) {
    float dtr[MB][4], dq[MB][4];
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        dtr[mb][rr] = 0.f;
        dq[mb][rr] = 0.f;
      }
#pragma unroll
    for (int jb = 0; jb < NJ; ++jb) {
      float c1 = A.ctr[jb], c2 = A.cq[jb];
      c1 += __shfl_xor(c1, 16, 64);
      c1 += __shfl_xor(c1, 32, 64);
      c2 += __shfl_xor(c2, 16, 64);
      c2 += __shfl_xor(c2, 32, 64);
      int j = (jb0 + jb) * 16 + jc;
#pragma unroll
      for (int mb = 0; mb < MB; ++mb)
#pragma unroll
        for (int rr = 0; rr < 4; ++rr) {
          int dim = mb * 16 + g * 4 + rr;
          float xj = (dim < DP) ? Xs[(size_t)j * DP + dim] : 0.f;
          dtr[mb][rr] += A.y2tr[jb][mb][rr] + xj * (xj * c1 - 2.f * A.ytr[jb][mb][rr]);
          dq[mb][rr] += A.y2q[jb][mb][rr] + xj * (xj * c2 - 2.f * A.yq[jb][mb][rr]);
        }
    }
    // sum over the 16 columns held by lanes with the same l/16
#pragma unroll
    for (int mb = 0; mb < MB; ++mb)
#pragma unroll
      for (int rr = 0; rr < 4; ++rr) {
        float v1 = dtr[mb][rr], v2 = dq[mb][rr];
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) {
          v1 += __shfl_xor(v1, o, 64);
          v2 += __shfl_xor(v2, o, 64);
        }
        int dim = mb * 16 + g * 4 + rr;
        if (jc == 0 && dim < DP) {
          pout[2 * dim] = 2.0 * (double)v1;
          pout[2 * dim + 1] = 2.0 * (double)v2;
        }
      }
  } else {
    float v1 = wave_sum(A.el_tr), v2 = wave_sum(A.el_q);
    if (lane == 0) {
      pout[0] = 2.0 * (double)v1;
      pout[1] = 2.0 * (double)v2;
    }
  }
  float s1 = wave_sum(A.es_tr), s2 = wave_sum(A.es_q);
  if (lane == 0) {
    pout[2 * nls] = 2.0 * (double)s1;
    pout[2 * nls + 1] = 2.0 * (double)s2;
  }
}

// dk_out[e] = sum over waves of partial[w][e], fixed order, fp64; one block per value e.
__global__ __launch_bounds__(256) void k_dk_finish(const double* __restrict__ partial, int nrows,
                                                    int pstride, DevState* st) {
  __shared__ double red[256];
  int e = blockIdx.x;
  double s = 0.0;
  for (int w = threadIdx.x; w < nrows; w += 256) s += partial[(size_t)w * pstride + e];
  red[threadIdx.x] = s;
  __syncthreads();
  for (int w = 128; w > 0; w >>= 1) {
    if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) st->dk_out[e] = red[0];
}

// Columns [col0, col0+ncols) of a row-major block (stride ld), times `scale`, into MFMA
// operand order at operand columns dstcol0..: dst[((i/16)*TS + c/4)*64 + (c%4)*16 + i%16].
__global__ void k_swizzle_cols(const double* __restrict__ src, int ld, int n, int np, int col0,
                               int ncols, int TS, int dstcol0, float scale,
                               float* __restrict__ dst) {
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (size_t)np * ncols) return;
  int i = (int)(idx / ncols), cc = (int)(idx % ncols);
  float v = (i < n) ? (float)(src[(size_t)i * ld + col0 + cc] * (double)scale) : 0.f;
  int c = dstcol0 + cc;
  dst[((size_t)(i >> 4) * TS + (c >> 2)) * 64 + (size_t)((c & 3) * 16 + (i & 15))] = v;
}

__global__ void k_extract_col(const double* __restrict__ src, int ld, int n, int np, int col,
                              float* __restrict__ dst) {
  int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= np) return;
  dst[i] = (i < n) ? (float)src[(size_t)i * ld + col] : 0.f;
}

}  // namespace

// ------------------------------------------------------------------ launchers
#define FOR_KK(MACRO)                  \
  switch (KK) {                        \
    case 1: MACRO(1); break;           \
    case 2: MACRO(2); break;           \
    case 4: MACRO(4); break;           \
    case 8: MACRO(8); break;           \
    case 16: MACRO(16); break;         \
    default: return 1;                 \
  }

int launch_build_khat(hipStream_t s, int kernel, int KK, const float* Xa, const float* Xb,
                      const float* sq, int n, int np, int panel_width, int tri, double outputscale,
                      double noise, float* Khat) {
  int pw = panel_width > 0 ? panel_width : np;
  if (tri && (panel_width <= 0 || panel_width % 64 != 0)) return 1;
  dim3 grid(np / 64, np / 64);
#define BUILD(K)                                                                                  \
  if (kernel == 0)                                                                                \
    k_build_khat<0, K><<<grid, 256, 0, s>>>(Xa, Xb, sq, n, np, pw, tri, (float)outputscale, (float)noise, Khat); \
  else                                                                                            \
    k_build_khat<1, K><<<grid, 256, 0, s>>>(Xa, Xb, sq, n, np, pw, tri, (float)outputscale, (float)noise, Khat)
  FOR_KK(BUILD)
#undef BUILD
  return 0;
}

int launch_mm_mat(hipStream_t s, const float* Khat, const double* D4, double* Vp, int np, int ld,
                  const MmPlan* plan, int wgs, const DevState* st, int panel_width, int panel_rows,
                  int cols) {
  // panel_width 0: plain row-major with row stride np
  int pw = panel_width > 0 ? panel_width : np;
  int ldk = panel_width > 0 ? panel_width : np;
  size_t panel_stride = panel_width > 0 ? (size_t)panel_rows * panel_width : 0;
  if (pw % 256 != 0) return 1;
  if (ld == 16 && cols > 0 && cols <= 12)
    k_mm_mat<1, 4, true><<<wgs, 256, 0, s>>>(Khat, D4, Vp, np, pw, panel_stride, ldk, plan, st);
  else if (ld == 16)
    k_mm_mat<1, 4, false><<<wgs, 256, 0, s>>>(Khat, D4, Vp, np, pw, panel_stride, ldk, plan, st);
  else if (ld == 32)
    k_mm_mat<2, 2, false><<<wgs, 256, 0, s>>>(Khat, D4, Vp, np, pw, panel_stride, ldk, plan, st);
  else
    return 1;
  return 0;
}

int launch_mm_otf(hipStream_t s, int kernel, int KK, const float* Xa, const float* Xb, const float* sq,
                  const double* D4, double* Vp, int np, int ld, int c, int nsplit, const DevState* st) {
  constexpr int NJ = 8;
  int nblk = np / 16;
  int blocks_per_split = (nblk + nsplit - 1) / nsplit;
  int sstrips = (nblk + 4 * NJ - 1) / (4 * NJ);
  int grid = sstrips * nsplit;
  // MFMA column groups and columns left to the vector unit: 17..20 columns = one group + 1, 2 or 4
  int nq = ld / 16, nx = 0;
  if (ld == 32 && c > 16 && c <= 20) {
    nq = 1;
    nx = (c == 17) ? 1 : ((c == 18) ? 2 : 4);
  }
  if (ld != 16 && ld != 32) return 1;
#define OTF_LAUNCH(KIND, K, Q, X) \
  k_mm_otf<KIND, K, Q, NJ, X><<<grid, 256, 0, s>>>(Xa, Xb, sq, D4, Vp, np, nsplit, blocks_per_split, st)
#define OTF_KIND(KIND, K)                             \
  if (nq == 2) OTF_LAUNCH(KIND, K, 2, 0);             \
  else if (nx == 0 && c <= 12)                        \
    k_mm_otf<KIND, K, 1, NJ, 0, true><<<grid, 256, 0, s>>>(Xa, Xb, sq, D4, Vp, np, nsplit, blocks_per_split, st); \
  else if (nx == 0) OTF_LAUNCH(KIND, K, 1, 0);        \
  else if (nx == 1) OTF_LAUNCH(KIND, K, 1, 1);        \
  else if (nx == 2) OTF_LAUNCH(KIND, K, 1, 2);        \
  else OTF_LAUNCH(KIND, K, 1, 4)
#define OTF(K)                  \
  if (kernel == 0) {            \
    OTF_KIND(0, K);             \
  } else {                      \
    OTF_KIND(1, K);             \
  }
  FOR_KK(OTF)
#undef OTF
#undef OTF_KIND
#undef OTF_LAUNCH
  return 0;
}

// On-the-fly product with each tile pair evaluated once (ld = 16 and KK <= 8 only): one launch over
// the pieces above the diagonal blocks, one over the pieces inside them.
int launch_mm_otf_tri(hipStream_t s, int kernel, int KK, const float* Xa, const float* Xb, const float* sq,
                      const double* D4, double* Vp, int np, int cols, const MmPiece* pieces,
                      const int* first_dual, int wgs_dual, const int* first_single, int wgs_single,
                      const int* slot_base, const DevState* st) {
  bool narrow = cols <= 12;
#define TRI_LAUNCH(KIND, K, NARROW)                                                                       \
  do {                                                                                                    \
    if (wgs_dual > 0)                                                                                     \
      k_mm_otf_tri<KIND, K, NARROW, true><<<wgs_dual, 256, 0, s>>>(Xa, Xb, sq, D4, Vp, np, pieces,        \
                                                                   first_dual, slot_base, st);            \
    k_mm_otf_tri<KIND, K, NARROW, false><<<wgs_single, 256, 0, s>>>(Xa, Xb, sq, D4, Vp, np, pieces,       \
                                                                    first_single, slot_base, st);         \
  } while (0)
#define TRI(K)                                   \
  if (kernel == 0) {                             \
    if (narrow) TRI_LAUNCH(0, K, true);          \
    else TRI_LAUNCH(0, K, false);                \
  } else {                                       \
    if (narrow) TRI_LAUNCH(1, K, true);          \
    else TRI_LAUNCH(1, K, false);                \
  }
  // up to 32 input dimensions: beyond that the two-use form does not fit the register file
  switch (KK) {
    case 1: TRI(1); break;
    case 2: TRI(2); break;
    case 4: TRI(4); break;
    case 8: TRI(8); break;
    default: return 1;
  }
#undef TRI
#undef TRI_LAUNCH
  return 0;
}

int launch_dk(hipStream_t s, int kernel, int KK, int ard, int TS, const float* Xa, const float* Xb,
              const float* sq, const float* Xs, const float* X4, const float* SA, const float* SB,
              const float* u0, int np, int nsplit, double* partial, int pstride, int max_rows,
              DevState* st) {
  int nblk = np / 16;
  int blocks_per_split = (nblk + nsplit - 1) / nsplit;
  int sstrips = (nblk + 4 * DK_NJ - 1) / (4 * DK_NJ);
  int grid = sstrips * nsplit;
  int nrows = grid * 4;
  if (nrows > max_rows || TS < 1 || TS > DK_TSMAX) return 1;
  size_t lds = (size_t)4 * DK_NJ * TS * 64 * sizeof(float);
#define DK(K)                                                                                        \
  if (kernel == 0 && !ard)                                                                           \
    k_dk<0, K, 0><<<grid, 256, lds, s>>>(Xa, Xb, sq, Xs, X4, SA, SB, TS, u0, np, nsplit, blocks_per_split, partial, pstride); \
  else if (kernel == 0 && ard)                                                                       \
    k_dk<0, K, 1><<<grid, 256, lds, s>>>(Xa, Xb, sq, Xs, X4, SA, SB, TS, u0, np, nsplit, blocks_per_split, partial, pstride); \
  else if (kernel == 1 && !ard)                                                                      \
    k_dk<1, K, 0><<<grid, 256, lds, s>>>(Xa, Xb, sq, Xs, X4, SA, SB, TS, u0, np, nsplit, blocks_per_split, partial, pstride); \
  else                                                                                               \
    k_dk<1, K, 1><<<grid, 256, lds, s>>>(Xa, Xb, sq, Xs, X4, SA, SB, TS, u0, np, nsplit, blocks_per_split, partial, pstride)
  FOR_KK(DK)
#undef DK
  int nls = ard ? 4 * KK : 1;
  k_dk_finish<<<2 * (nls + 1), 256, 0, s>>>(partial, nrows, pstride, st);
  return 0;
}

void launch_dk_finish(hipStream_t s, const double* partial, int nrows, int pstride, int nvalues,
                      DevState* st) {
  k_dk_finish<<<nvalues, 256, 0, s>>>(partial, nrows, pstride, st);
}

void launch_swizzle_cols(hipStream_t s, const double* src, int ld, int n, int np, int col0, int ncols,
                         int TS, int dstcol0, float scale, float* dst) {
  size_t total = (size_t)np * ncols;
  k_swizzle_cols<<<(int)((total + 255) / 256), 256, 0, s>>>(src, ld, n, np, col0, ncols, TS, dstcol0,
                                                            scale, dst);
}

void launch_extract_col(hipStream_t s, const double* src, int ld, int n, int np, int col, float* dst) {
  k_extract_col<<<(np + 255) / 256, 256, 0, s>>>(src, ld, n, np, col, dst);
}
