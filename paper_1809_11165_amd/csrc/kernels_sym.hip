// Product V = K_hat D from ONE triangle of the materialised fp32 K_hat (gfx950 / CDNA4).
//
// K_hat is symmetric, so its upper triangle holds everything: stored in column panels of
// BBMM_SYM_PANEL columns, panel P keeping rows [0, (P+1) * BBMM_SYM_PANEL) (the square block on the
// diagonal is stored whole), the product streams half the bytes of the full matrix.  A tile T at
// (rows I, columns J) above the diagonal blocks is then used twice,
//     out[J] += T^T D[I]      (contraction over the tile's rows, as in k_mm_mat)
//     out[I] += T   D[J]      (contraction over its columns),
// both on the fp64 matrix pipe (v_mfma_f64_16x16x4; the first use takes the 4x4x4 form when at most
// 12 columns of the block are in use).  The second use needs the tile in the transposed lane layout;
// every wave passes its 16 x 64 tile through a private LDS area for that (no barrier: a wave's LDS
// operations execute in order), one tile ahead of its use.  The first kind of partial sum stays in
// registers for a whole piece of work; the second kind is finished after every 16-row step, staged
// in LDS per wave, and every SYM_GROUP steps the four waves' parts are added in a fixed order and
// written to a partial-result slot (two barriers per group).  The matrix-pipe work is that of the
// full-matrix product, which is what bounds this kernel: HBM traffic is halved, arithmetic is not.
#include "bbmm_dev.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x4s __attribute__((ext_vector_type(4), aligned(16)));   // as laid out in LDS

namespace {

// A[m = lane%16][k = lane/16], B[k = lane/16][n = lane%16]; register r of the result holds
// C[m = 4*r + lane/16][n = lane%16].
__device__ inline f64x4 mfma16d(double a, double b, f64x4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

// The fp64 4x4x4 MFMA (16 cycles, the same flop rate) computes the four diagonal 4 x 4 blocks of what
// the 16x16x4 instruction would: C[i = lane/16][j = lane%4] of block p = (lane/4)%4
//   += sum_k A(lane 16 k + 4 p + i) * B(lane 16 k + 4 p + j)      (one register each; measured).
// With the B operand as above (k <-> rows 4k+r, lane%16 <-> columns 4 (lane%16) + cc) and the A
// operand D[row 4k+r][rhs 4q + lane%4], three of them (q = 0, 1, 2) give right-hand-side columns
// 0..11 of the same 64 matrix columns in 48 cycles instead of 64: lane (jc, g) then holds
// out[column 4jc+cc][rhs 4q+g], which is element q of the 16x16 accumulator's four.
__device__ inline double mfma4d(double a, double b, double c) {
  return __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, c, 0, 0, 0);
}

// Column-side use of one row quad of a tile: 16-wide (all 16 right-hand-side columns of the group)
// or NARROW (columns 0..11 only, accumulated in accn[cc][q], q = rhs / 4).
// dcur[q][r]: 16-wide: q = 0 only, D[row 4g+r][rhs jc]; NARROW: D[row 4g+r][rhs 4q + jc%4].
template <bool NARROW>
__device__ __forceinline__ void sym_col_mma(const f64x4 (&dcur)[3], int r, const double (&kd)[4], f64x4 (&acc)[4],
                                            double (&accn)[4][3]) {
#pragma unroll
  for (int cc = 0; cc < 4; ++cc) {
    if (NARROW) {
#pragma unroll
      for (int q = 0; q < 3; ++q) accn[cc][q] = mfma4d(dcur[q][r], kd[cc], accn[cc][q]);
    } else {
      acc[cc] = mfma16d(dcur[0][r], kd[cc], acc[cc]);
    }
  }
}

template <bool NARROW>
__device__ __forceinline__ void sym_load_drows(const double* __restrict__ Dq, int j, int LD, int jc, int g,
                                               f64x4 (&d)[3]) {
  if (NARROW) {
#pragma unroll
    for (int q = 0; q < 3; ++q)
      d[q] = *(const f64x4*)(Dq + ((size_t)(j / 4 + g) * LD + (size_t)(4 * q + (jc & 3))) * 4);
  } else {
    d[0] = *(const f64x4*)(Dq + ((size_t)(j / 4 + g) * LD + (size_t)jc) * 4);
  }
}

constexpr int SYM_NC = 4;                    // 64-column groups per wave
constexpr int SYM_W = BBMM_SYM_PANEL;        // columns per workgroup = panel width of the storage
constexpr int SYM_TLD = 68;                  // floats per row of a wave's transposition area (64 + 4:
                                             // the transposed 16-byte reads then hit all banks once)
constexpr int SYM_GROUP = 8;                 // 16-row steps between two flushes of the row-side sums
constexpr int SYM_PLD = 18;                  // doubles per staged row (16 + 2: conflict-free stores)
static_assert(SYM_W == 256 * SYM_NC, "a workgroup of four waves covers one panel");

__device__ __forceinline__ size_t sym_panel_offset(int P) {
  return (size_t)SYM_W * SYM_W * ((size_t)P * (size_t)(P + 1) / 2);
}

// Passes one 16 x 64 tile through the wave's LDS area: written as loaded (rows 4g+r, columns 4jc..),
// read back transposed for the row-side use.  Split in four parts so that a step can place one part
// after each group of MFMAs.  On this chip a few LDS reads and memory loads issue for free beside the
// fp64 MFMAs, VALU instructions do not (each adds its ~5 cycles), and an LDS *write* holds the matrix
// pipe up for ~11 cycles per dword (measured: 45 cycles per ds_write_b128 per wave, wherever it is
// placed), which makes the transposition the largest cost of this kernel after the MFMAs.
__device__ __forceinline__ void sym_lds_part(int part, float* __restrict__ Tw, int jc, int g,
                                             const f32x4 (&kvt)[4], f32x4 (&kt)[4]) {
  if (part < 2) {
#pragma unroll
    for (int r = 2 * part; r < 2 * part + 2; ++r) *(f32x4*)(Tw + (4 * g + r) * SYM_TLD + 4 * jc) = kvt[r];
    if (part == 1) __builtin_amdgcn_wave_barrier();
  } else {
#pragma unroll
    for (int s = 2 * part - 4; s < 2 * part - 2; ++s) kt[s] = *(const f32x4*)(Tw + jc * SYM_TLD + 16 * s + 4 * g);
    if (part == 3) __builtin_amdgcn_wave_barrier();
  }
}

// One 16-row step that uses every tile twice.  kv / dI / kt hold this step's operands on entry and
// the next step's on exit (knext / jnext point at the same step again after the last one, so the
// loads need no branch).  Lane (jc = lane%16, g = lane/16):
//   kv[nc][r]   rows 4g+r, columns 64 nc + 4 jc .. +3 of the wave's 16 x 256 slab
//   dI[q][r]    A operand of the first use: D[row 4g+r of the step][rhs jc] (q = 0), or, NARROW,
//               D[row 4g+r of the step][rhs 4q + jc%4], q = 0..2
//   dJ[nc][s]   D[column 64 nc + 16 s + 4 g + cc of the wave][rhs jc]  (A operand of the second use)
//   kt[s][cc]   K[row jc of the step][column 64 nc + 16 s + 4 g + cc]  (from LDS, B operand); on
//               entry that of tile 0, requested for tile nc+1 during the second use of tile nc
// out2: lane holds out[row jc of the step][rhs 4 i + g], i = 0..3, summed over the wave's columns.
template <bool NARROW>
__device__ __forceinline__ void sym_step_dual(const float* __restrict__ knext, const double* __restrict__ Dq,
                                              int jnext, int LD, int jc, int g, float* __restrict__ Tw,
                                              f32x4 (&kv)[SYM_NC][4], f64x4 (&dI)[3], f32x4 (&kt)[4],
                                              const f64x4 (&dJ)[SYM_NC][4], f64x4 (&acc1)[SYM_NC][4],
                                              double (&acc1n)[SYM_NC][4][3], f64x4& out2) {
  f64x4 dcur[3];
#pragma unroll
  for (int q = 0; q < (NARROW ? 3 : 1); ++q) dcur[q] = dI[q];
  sym_load_drows<NARROW>(Dq, jnext, LD, jc, g, dI);
  f64x4 acc2[4];
#pragma unroll
  for (int cc = 0; cc < 4; ++cc) acc2[cc] = (f64x4){0.0, 0.0, 0.0, 0.0};
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int nc = 0; nc < SYM_NC; ++nc) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      double kd[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) kd[cc] = (double)kv[nc][r][cc];
      kv[nc][r] = __builtin_nontemporal_load((const f32x4*)(knext + (size_t)r * SYM_W + nc * 64));
      sym_col_mma<NARROW>(dcur, r, kd, acc1[nc], acc1n[nc]);
      __builtin_amdgcn_sched_barrier(0);
    }
    // the tile that follows: nc + 1 of this step, or tile 0 of the next (already reloaded above)
    f32x4 ktn[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      double kd[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) kd[cc] = (double)kt[s][cc];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) acc2[cc] = mfma16d(dJ[nc][s][cc], kd[cc], acc2[cc]);
      sym_lds_part(s, Tw, jc, g, kv[(nc + 1) % SYM_NC], ktn);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) kt[s] = ktn[s];
  }
  out2 = (acc2[0] + acc2[1]) + (acc2[2] + acc2[3]);
}

// One 16-row step inside a diagonal block: the first use only.
template <bool NARROW>
__device__ __forceinline__ void sym_step_single(const float* __restrict__ knext, const double* __restrict__ Dq,
                                                int jnext, int LD, int jc, int g, f32x4 (&kv)[SYM_NC][4],
                                                f64x4 (&dI)[3], f64x4 (&acc1)[SYM_NC][4],
                                                double (&acc1n)[SYM_NC][4][3]) {
  f64x4 dcur[3];
#pragma unroll
  for (int q = 0; q < (NARROW ? 3 : 1); ++q) dcur[q] = dI[q];
  sym_load_drows<NARROW>(Dq, jnext, LD, jc, g, dI);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int nc = 0; nc < SYM_NC; ++nc) {
      double kd[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) kd[cc] = (double)kv[nc][r][cc];
      kv[nc][r] = __builtin_nontemporal_load((const f32x4*)(knext + (size_t)r * SYM_W + nc * 64));
      sym_col_mma<NARROW>(dcur, r, kd, acc1[nc], acc1n[nc]);
      __builtin_amdgcn_sched_barrier(0);
    }
}

// Workgroup = 4 waves on the 1024 columns of one panel; it runs pieces first[b] .. first[b+1]-1 of
// the work list, each a run of rows of one panel.  A piece above its panel's diagonal block uses
// every tile twice; a piece inside the block (stored whole) makes the column-side use only.
// DUAL = false: a launch over pieces of the second kind only.  DUAL = true: pieces of the first
// kind and then, in the NARROW form when first_diag is given, the workgroup's share of the second
// kind too (one launch for the whole product; the 16-wide form has no registers to spare for both
// loops, and the second kind then runs as its own, lighter launch).  Partial results: the
// column-side sum of a piece goes to slot `piece.slot` of its panel's rows of the output; the
// row-side sums of panel P for output rows of panel s < P go to slot slot_base[s] + P - s - 1.
//
// Dq / Vq point at the 16-column group of the right-hand side / output that this launch handles;
// LD (16 or 32) is the padded width of both.
template <bool DUAL, bool NARROW>
__global__ __launch_bounds__(256, DUAL ? 1 : 2) void k_mm_sym(const float* __restrict__ Kt, const double* __restrict__ Dq,
                                                double* __restrict__ Vq, int np, int LD,
                                                const MmPiece* __restrict__ pieces,
                                                const int* __restrict__ first,
                                                const int* __restrict__ first_diag,
                                                const int* __restrict__ slot_base,
                                                const DevState* __restrict__ st) {
  if (st->done) return;
  __shared__ __align__(16) float T[DUAL ? 4 : 1][DUAL ? 16 * SYM_TLD : 4];
  __shared__ __align__(16) double S[DUAL ? 4 : 1][DUAL ? 16 * SYM_GROUP * SYM_PLD : 2];
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int jc = lane & 15, g = lane >> 4;
  float* Tw = T[DUAL ? wave : 0];
  double* Sw = S[DUAL ? wave : 0];

  // DUAL: the workgroup's pieces above the diagonal blocks, then (first_diag given) its share of
  // the pieces inside them
  int pb = first[blockIdx.x], pe = first[blockIdx.x + 1];
  int db = 0, de = 0;
  if (DUAL && NARROW && first_diag) {   // (the 16-wide form has no registers to spare for both loops)
    db = first_diag[blockIdx.x];
    de = first_diag[blockIdx.x + 1];
  }
  int npieces = (pe - pb) + (de - db);
#pragma unroll 1
  for (int pi = 0; pi < npieces; ++pi) {
    const bool dual_piece = DUAL && (!NARROW || pi < pe - pb);
    int pc = dual_piece || !DUAL ? pb + pi : db + (pi - (pe - pb));
    MmPiece P = pieces[pc];
    int colw = P.strip * SYM_W + wave * (64 * SYM_NC);
    bool active = colw < np;
    int nsteps = (P.row_end - P.row_begin) >> 4;
    if (nsteps <= 0) continue;
    const float* kp = Kt + sym_panel_offset(P.strip) + (size_t)(P.row_begin + g * 4) * SYM_W +
                      (size_t)(wave * (64 * SYM_NC) + 4 * jc);
    f64x4 acc1[SYM_NC][4];
    double acc1n[SYM_NC][4][3];
#pragma unroll
    for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        acc1[nc][cc] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int q = 0; q < 3; ++q) acc1n[nc][cc][q] = 0.0;
      }
    f32x4 kv[SYM_NC][4];
    f64x4 dI[3];
#pragma unroll
    for (int q = 0; q < 3; ++q) dI[q] = (f64x4){0.0, 0.0, 0.0, 0.0};
    if (active) {
      sym_load_drows<NARROW>(Dq, P.row_begin, LD, jc, g, dI);
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int nc = 0; nc < SYM_NC; ++nc)
          kv[nc][r] = __builtin_nontemporal_load((const f32x4*)(kp + (size_t)r * SYM_W + nc * 64));
    }
    int j0 = P.row_begin;
    if (!dual_piece) {
      if (active) {
#pragma unroll 1
        for (int q = 0; q < nsteps; ++q, j0 += 16) {
          bool more = q + 1 < nsteps;
          if (more) kp += (size_t)16 * SYM_W;
          sym_step_single<NARROW>(kp, Dq, more ? j0 + 16 : j0, LD, jc, g, kv, dI, acc1, acc1n);
        }
      }
    } else {
      f64x4 dJ[SYM_NC][4];
      f32x4 kt[4];
      if (active) {
#pragma unroll
        for (int part = 0; part < 4; ++part) sym_lds_part(part, Tw, jc, g, kv[0], kt);
      }
      if (!active) {
        // a wave whose columns lie beyond the matrix (last, narrower panel) stages nothing in this
        // piece: its area must read as zero in the flushes (the barrier that ended the previous
        // flush has passed, so nobody reads the old content any more)
        for (int i = lane; i < 16 * SYM_GROUP * SYM_PLD; i += 64) Sw[i] = 0.0;
      }
      if (active) {
#pragma unroll
        for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
          for (int s = 0; s < 4; ++s)
            dJ[nc][s] = *(const f64x4*)(Dq + ((size_t)((colw + nc * 64) / 4 + 4 * s + g) * LD + (size_t)jc) * 4);
      }
#pragma unroll 1
      for (int q0 = 0; q0 < nsteps; q0 += SYM_GROUP) {
        int ng = min(SYM_GROUP, nsteps - q0);
        int jg = j0;
        if (active) {
#pragma unroll 1
          for (int q = 0; q < ng; ++q, j0 += 16) {
            bool more = q0 + q + 1 < nsteps;
            if (more) kp += (size_t)16 * SYM_W;
            f64x4 out2;
            sym_step_dual<NARROW>(kp, Dq, more ? j0 + 16 : j0, LD, jc, g, Tw, kv, dI, kt, dJ, acc1, acc1n, out2);
            *(f64x4s*)(Sw + (q * 16 + jc) * SYM_PLD + 4 * g) = out2;
          }
        } else {
          j0 += 16 * ng;
        }
        __syncthreads();
        {
          int rl = threadIdx.x >> 1, half = threadIdx.x & 1;
          if (rl < ng * 16) {
            int row = jg + rl;
            const double* sp = &S[0][0] + rl * SYM_PLD + 8 * half;
            f64x4 lo = *(const f64x4s*)sp, hi = *(const f64x4s*)(sp + 4);
#pragma unroll
            for (int w = 1; w < 4; ++w) {
              lo += *(const f64x4s*)(sp + w * (16 * SYM_GROUP * SYM_PLD));
              hi += *(const f64x4s*)(sp + w * (16 * SYM_GROUP * SYM_PLD) + 4);
            }
            int so = row / SYM_W;
            int slot = slot_base[so] + (P.strip - so - 1);
            double* dst = Vq + ((size_t)slot * np + (size_t)row) * LD + 8 * half;
            *(f64x4*)dst = lo;
            *(f64x4*)(dst + 4) = hi;
          }
        }
        __syncthreads();
      }
    }
    if (active) {
      double* vout = Vq + (size_t)P.slot * np * LD;
#pragma unroll
      for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
          *(f64x4*)(vout + (size_t)(colw + nc * 64 + 4 * jc + cc) * LD + g * 4) =
              NARROW ? (f64x4){acc1n[nc][cc][0], acc1n[nc][cc][1], acc1n[nc][cc][2], 0.0} : acc1[nc][cc];
    }
  }
}

}  // namespace

// K_hat D from the triangular storage: per group of 16 right-hand-side columns one launch over
// the pieces above the diagonal blocks and one over the pieces inside them.
int launch_mm_sym(hipStream_t s, const float* Ktri, const double* D4, double* Vp, int np, int ld, int cols,
                  const MmPiece* pieces, const int* first_dual, int wgs_dual, const int* first_single,
                  int wgs_single, const int* slot_base, const DevState* st) {
  if (ld != 16 && ld != 32) return 1;
  for (int nq = 0; nq < ld / 16; ++nq) {
    // a group of which at most 12 columns are in use takes the narrower column-side instruction
    bool narrow = cols - 16 * nq <= 12;
    const double* Dq = D4 + 64 * nq;
    double* Vq = Vp + 16 * nq;
    // with the same number of workgroups in both lists one launch runs both kinds of piece
    bool merged = narrow && wgs_dual > 0 && wgs_dual == wgs_single;
    const int* fd = merged ? first_single : nullptr;
    if (wgs_dual > 0) {
      if (narrow)
        k_mm_sym<true, true><<<wgs_dual, 256, 0, s>>>(Ktri, Dq, Vq, np, ld, pieces, first_dual, fd, slot_base, st);
      else
        k_mm_sym<true, false><<<wgs_dual, 256, 0, s>>>(Ktri, Dq, Vq, np, ld, pieces, first_dual, fd, slot_base, st);
    }
    if (merged) continue;
    if (narrow)
      k_mm_sym<false, true><<<wgs_single, 256, 0, s>>>(Ktri, Dq, Vq, np, ld, pieces, first_single, nullptr,
                                                       slot_base, st);
    else
      k_mm_sym<false, false><<<wgs_single, 256, 0, s>>>(Ktri, Dq, Vq, np, ld, pieces, first_single, nullptr,
                                                        slot_base, st);
  }
  return 0;
}
