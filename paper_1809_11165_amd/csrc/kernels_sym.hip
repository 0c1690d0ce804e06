// Product V = K_hat D from ONE triangle of the materialised fp32 K_hat (gfx950 / CDNA4).
//
// K_hat is symmetric, so its upper triangle holds everything: stored in column panels of
// BBMM_SYM_PANEL columns, panel P keeping rows [0, (P+1) * BBMM_SYM_PANEL) (the square block on the
// diagonal is stored whole), the product streams half the bytes of the full matrix.  A tile T at
// (rows I, columns J) above the diagonal blocks is then used twice,
//     out[J] += T^T D[I]      (contraction over the tile's rows, as in k_mm_mat)
//     out[I] += T   D[J]      (contraction over its columns),
// both with v_mfma_f64_16x16x4_f64.  The two uses need the tile in two lane layouts (one the
// transpose of the other); the tiles are loaded straight into LDS and read from there in both.  The
// first kind of partial sum stays in registers for a whole piece of work; the second kind is
// finished after every 16-row step, staged in LDS per wave, and every SYM_GROUP steps the four
// waves' parts are added in a fixed order and written to a partial-result slot (two barriers per
// group).  The number of fp64 MFMAs is that of the full-matrix product, which is what bounds this
// kernel: HBM traffic is halved, arithmetic is not.
#include "bbmm_dev.h"

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef double f64x4 __attribute__((ext_vector_type(4)));
typedef double f64x4s __attribute__((ext_vector_type(4), aligned(16)));   // as laid out in LDS
typedef double f64x2 __attribute__((ext_vector_type(2)));

namespace {

// A[m = lane%16][k = lane/16], B[k = lane/16][n = lane%16]; register r of the result holds
// C[m = 4*r + lane/16][n = lane%16].
__device__ inline f64x4 mfma16d(double a, double b, f64x4 c) {
  return __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, c, 0, 0, 0);
}

constexpr int SYM_NC = 4;                    // 64-column groups per wave
constexpr int SYM_W = BBMM_SYM_PANEL;        // columns per workgroup = panel width of the storage
constexpr int SYM_GROUP = 8;                 // 16-row steps between two flushes of the row-side sums
constexpr int SYM_PLD = 18;                  // doubles per staged row (16 + 2: conflict-free stores)
static_assert(SYM_W == 256 * SYM_NC, "a workgroup of four waves covers one panel");

__device__ __forceinline__ size_t sym_panel_offset(int P) {
  return (size_t)SYM_W * SYM_W * ((size_t)P * (size_t)(P + 1) / 2);
}

// ---- tiles through LDS without passing registers -------------------------------------------
// On this chip LDS reads and memory loads issue for free beside the fp64 MFMAs, VALU instructions
// do not (each adds its ~5 cycles), and an LDS *write* from registers holds the matrix pipe up for
// ~11 cycles per dword (measured: 45 cycles per ds_write_b128 per wave, wherever it is placed).  So
// the tiles are loaded straight into LDS (global_load_lds_dwordx4: lane l of the instruction
// deposits its 16 bytes at M0 + 16 l) and both lane layouts are then read from there.
//
// A 16 x 64 tile is 256 chunks of 16 bytes, chunk (row rho, column group kappa) = columns
// 4 kappa .. 4 kappa + 3 of row rho.  It sits in a 4 KB slot at chunk position
//     pos(rho, kappa) = 16 rho + (kappa + rho) % 16,
// a row-major image with row rho rotated by rho chunks: the column-side read (16 lanes: one row,
// kappa = 0..15) and the row-side read (16 lanes: rho = 0..15, one kappa) both touch every group of
// four banks exactly once.  Load instruction i = 0..3 fills positions 64 i .. 64 i + 63, i.e. rows
// 4i .. 4i+3, each as one contiguous 256-byte piece of memory.
//
// The compiler knows nothing about these loads, so all waiting is written out: memory operations
// complete in issue order and the vmcnt argument below is the number of loads issued after the one
// waited for.
typedef __attribute__((address_space(3))) float lds_float;

__device__ __forceinline__ void sym_dma_tile(const float* gbase, unsigned slot_bytes, const unsigned (&voff)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voff[i]), "s"(gbase), "s"(slot_bytes + 1024u * i) : "memory", "m0");
}

// The 16 rows of D of one step (2 KB in the quad-swizzled layout: lane (jc, g) owns the 32 bytes
// D[rows 4g .. 4g+3][rhs jc]) go the same way, 16 bytes per lane and instruction, and every lane
// reads its own two pieces back.  (Loading them into registers by an asm statement instead would
// let the compiler copy those registers before the data has arrived.)
__device__ __forceinline__ void sym_dma_drows(const double* dbase, unsigned dbuf_bytes, const unsigned (&voffd)[2]) {
#pragma unroll
  for (int h = 0; h < 2; ++h)
    asm volatile("s_mov_b32 m0, %2\n\tglobal_load_lds_dwordx4 %0, %1"
                 :: "v"(voffd[h]), "s"(dbase), "s"(dbuf_bytes + 1024u * h) : "memory", "m0");
}

template <int N>
__device__ __forceinline__ void sym_wait_vm() {
  asm volatile("s_waitcnt vmcnt(%0)" :: "n"(N) : "memory");
}

__device__ __forceinline__ void sym_wait_lds() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// One 16-row step that uses every tile twice.  Slot nc of the wave's ring holds tile nc of this
// step on entry and of the next step on exit (gnext / dnext point at the same step again after
// the last one, so the loads need no branch).  Lane (jc = lane%16, g = lane/16):
//   a1[.][r]    K[row 4g+r of the step][columns 4 jc .. +3 of the tile]        (column-side use)
//   a2[.][s]    K[row jc of the step][columns 16 s + 4 g .. +3 of the tile]    (row-side use)
//   dn          D[rows 4g .. 4g+3 of the step][rhs jc]     (A operand of the column-side use; the next
//               step's rows are requested during tile 0 and read from their LDS buffer during tile 3)
//   dJ[nc][s]   D[column 64 nc + 16 s + 4 g + cc of the wave][rhs jc]    (A operand, row-side)
// a1 / a2 are double-buffered: while tile nc is multiplied, tile nc+1 (tile 0 of the next step
// after tile 3) is read from its slot; set 0 holds tile 0 on entry and on exit.
// Loads per step, in issue order: tile 0 (4), D of the next step (2), tiles 1, 2, 3 (4 each).
// out2: lane holds out[row jc of the step][rhs 4 i + g], i = 0..3, summed over the wave's columns.
__device__ __forceinline__ void sym_step_dual(const float* gnext, const double* dnext, int jc, int g,
                                              const float* __restrict__ ring, unsigned ring_bytes,
                                              const f64x2* __restrict__ dbuf, unsigned dbuf_bytes,
                                              const unsigned (&voff)[4], const unsigned (&voffd)[2],
                                              const int (&rd1)[4], const int (&rd2)[4],
                                              f32x4 (&a1)[2][4], f32x4 (&a2)[2][4], f64x4& dn,
                                              const f64x4 (&dJ)[SYM_NC][4], f64x4 (&acc1)[SYM_NC][4],
                                              f64x4& out2) {
  f64x4 dcur = dn;
  f64x4 acc2[4];
#pragma unroll
  for (int cc = 0; cc < 4; ++cc) acc2[cc] = (f64x4){0.0, 0.0, 0.0, 0.0};
#pragma unroll
  for (int nc = 0; nc < SYM_NC; ++nc) {
    const int cur = nc & 1, nxt = cur ^ 1, nn = (nc + 1) % SYM_NC;
    // the reads of this tile (issued one tile ago) are complete: its slot can take the next step's
    sym_wait_lds();
    sym_dma_tile(gnext + nc * 64, ring_bytes + 4096u * nc, voff);
    if (nc == 0) sym_dma_drows(dnext, dbuf_bytes, voffd);   // read into dn (below) during tile 3
    // the tile that follows was requested 14 loads ago (one step back, or during tile 0 for the
    // next step's tile 0); the D rows came right after that tile 0, 12 loads ago
    if (nc == SYM_NC - 1) sym_wait_vm<12>(); else sym_wait_vm<14>();
    const float* slot = ring + 1024 * nn;
#pragma unroll
    for (int r = 0; r < 4; ++r) a1[nxt][r] = *(const f32x4*)(slot + rd1[r]);
#pragma unroll
    for (int s = 0; s < 4; ++s) a2[nxt][s] = *(const f32x4*)(slot + rd2[s]);
    if (nc == SYM_NC - 1) {
      f64x2 lo = dbuf[0], hi = dbuf[64];      // the lane's own two pieces
      dn = (f64x4){lo[0], lo[1], hi[0], hi[1]};
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      double kd[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) kd[cc] = (double)a1[cur][r][cc];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) acc1[nc][cc] = mfma16d(dcur[r], kd[cc], acc1[nc][cc]);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      double kd[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) kd[cc] = (double)a2[cur][s][cc];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) acc2[cc] = mfma16d(dJ[nc][s][cc], kd[cc], acc2[cc]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  out2 = (acc2[0] + acc2[1]) + (acc2[2] + acc2[3]);
}

// One 16-row step inside a diagonal block: the first use only.
__device__ __forceinline__ void sym_step_single(const float* __restrict__ knext, const double* __restrict__ Dq,
                                                int jnext, int LD, int jc, int g, f32x4 (&kv)[SYM_NC][4],
                                                f64x4& dI, f64x4 (&acc1)[SYM_NC][4]) {
  f64x4 dcur = dI;
  dI = *(const f64x4*)(Dq + ((size_t)(jnext / 4 + g) * LD + (size_t)jc) * 4);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int nc = 0; nc < SYM_NC; ++nc) {
      double kd[4];
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) kd[cc] = (double)kv[nc][r][cc];
      kv[nc][r] = __builtin_nontemporal_load((const f32x4*)(knext + (size_t)r * SYM_W + nc * 64));
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) acc1[nc][cc] = mfma16d(dcur[r], kd[cc], acc1[nc][cc]);
      __builtin_amdgcn_sched_barrier(0);
    }
}

// Pieces inside the diagonal blocks (stored whole): the column-side use only, as in k_mm_mat.
// Workgroup = 4 waves on the 1024 columns of one panel; it runs pieces first[b] .. first[b+1]-1 of
// the work list; the sum of a piece goes to slot `piece.slot` of its panel's rows of the output.
//
// Dq / Vq point at the 16-column group of the right-hand side / output that this launch handles;
// LD (16 or 32) is the padded width of both.
__global__ __launch_bounds__(256, 2) void k_mm_sym_diag(const float* __restrict__ Kt,
                                                         const double* __restrict__ Dq,
                                                         double* __restrict__ Vq, int np, int LD,
                                                         const MmPiece* __restrict__ pieces,
                                                         const int* __restrict__ first,
                                                         const DevState* __restrict__ st) {
  if (st->done) return;
  int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int jc = lane & 15, g = lane >> 4;
  int pb = first[blockIdx.x], pe = first[blockIdx.x + 1];
#pragma unroll 1
  for (int pc = pb; pc < pe; ++pc) {
    MmPiece P = pieces[pc];
    int colw = P.strip * SYM_W + wave * (64 * SYM_NC);
    int nsteps = (P.row_end - P.row_begin) >> 4;
    if (nsteps <= 0 || colw >= np) continue;
    const float* kp = Kt + sym_panel_offset(P.strip) + (size_t)(P.row_begin + g * 4) * SYM_W +
                      (size_t)(wave * (64 * SYM_NC) + 4 * jc);
    f64x4 acc1[SYM_NC][4];
#pragma unroll
    for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) acc1[nc][cc] = (f64x4){0.0, 0.0, 0.0, 0.0};
    f32x4 kv[SYM_NC][4];
    f64x4 dI = *(const f64x4*)(Dq + ((size_t)(P.row_begin / 4 + g) * LD + (size_t)jc) * 4);
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int nc = 0; nc < SYM_NC; ++nc)
        kv[nc][r] = __builtin_nontemporal_load((const f32x4*)(kp + (size_t)r * SYM_W + nc * 64));
    int j0 = P.row_begin;
#pragma unroll 1
    for (int q = 0; q < nsteps; ++q, j0 += 16) {
      bool more = q + 1 < nsteps;
      if (more) kp += (size_t)16 * SYM_W;
      sym_step_single(kp, Dq, more ? j0 + 16 : j0, LD, jc, g, kv, dI, acc1);
    }
    double* vout = Vq + (size_t)P.slot * np * LD;
#pragma unroll
    for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc)
        *(f64x4*)(vout + (size_t)(colw + nc * 64 + 4 * jc + cc) * LD + g * 4) = acc1[nc][cc];
  }
}

// Pieces above the diagonal blocks: every tile is used twice.  Same work division; in addition the
// row-side sums of panel P for output rows of panel s < P go to slot slot_base[s] + P - s - 1.
// LDS: per wave a ring of four 4 KB tile slots (slot nc = tile nc of the current or next step) and
// the staging area of the row-side sums.
__global__ __launch_bounds__(256, 1) void k_mm_sym_dual(const float* __restrict__ Kt,
                                                         const double* __restrict__ Dq,
                                                         double* __restrict__ Vq, int np, int LD,
                                                         const MmPiece* __restrict__ pieces,
                                                         const int* __restrict__ first,
                                                         const int* __restrict__ slot_base,
                                                         const DevState* __restrict__ st) {
  if (st->done) return;
  __shared__ __align__(16) float ringmem[4][SYM_NC * 1024];
  __shared__ __align__(16) double dmem[4][256];
  __shared__ __align__(16) double S[4][16 * SYM_GROUP * SYM_PLD];
  int lane = threadIdx.x & 63;
  int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int jc = lane & 15, g = lane >> 4;
  const float* ring = ringmem[wave];
  unsigned ring_bytes = (unsigned)(size_t)(lds_float*)ringmem[wave];
  const f64x2* dbuf = (const f64x2*)dmem[wave] + lane;
  unsigned dbuf_bytes = (unsigned)(size_t)(lds_float*)(float*)dmem[wave];
  double* Sw = S[wave];
  unsigned voff[4], voffd[2];
  int rd1[4], rd2[4];
  voffd[0] = (unsigned)((g * LD + jc) * 4) * 8u;
  voffd[1] = voffd[0] + 16u;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int rho = 4 * i + g;                                   // lane's row in load instruction i
    voff[i] = (unsigned)(rho * SYM_W + 4 * ((jc - rho) & 15)) * 4u;
    int r1 = 4 * g + i;                                    // column-side read r = i
    rd1[i] = 4 * (16 * r1 + ((jc + r1) & 15));
    rd2[i] = 4 * (16 * jc + ((4 * i + g + jc) & 15));      // row-side read s = i
  }

  int pb = first[blockIdx.x], pe = first[blockIdx.x + 1];
#pragma unroll 1
  for (int pc = pb; pc < pe; ++pc) {
    MmPiece P = pieces[pc];
    int colw = P.strip * SYM_W + wave * (64 * SYM_NC);
    bool active = colw < np;
    int nsteps = (P.row_end - P.row_begin) >> 4;
    if (nsteps <= 0) continue;
    // first tile of the wave's slab at the piece's first row (uniform over the wave)
    const float* gp = Kt + sym_panel_offset(P.strip) + (size_t)P.row_begin * SYM_W + (size_t)(wave * (64 * SYM_NC));
    f64x4 acc1[SYM_NC][4];
#pragma unroll
    for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) acc1[nc][cc] = (f64x4){0.0, 0.0, 0.0, 0.0};
    f64x4 dJ[SYM_NC][4];
    f32x4 a1[2][4], a2[2][4];
    f64x4 dn = (f64x4){0.0, 0.0, 0.0, 0.0};
    if (!active) {
      // a wave whose columns lie beyond the matrix (last, narrower panel) stages nothing in this
      // piece: its area must read as zero in the flushes (the barrier that ended the previous
      // flush has passed, so nobody reads the old content any more)
      for (int i = lane; i < 16 * SYM_GROUP * SYM_PLD; i += 64) Sw[i] = 0.0;
    } else {
      // the first step's tiles and D rows, in the issue order of a step
      sym_dma_tile(gp, ring_bytes, voff);
      sym_dma_drows(Dq + (size_t)(P.row_begin / 4) * LD * 4, dbuf_bytes, voffd);
#pragma unroll
      for (int nc = 1; nc < SYM_NC; ++nc) sym_dma_tile(gp + nc * 64, ring_bytes + 4096u * nc, voff);
#pragma unroll
      for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
        for (int s = 0; s < 4; ++s)
          dJ[nc][s] = *(const f64x4*)(Dq + ((size_t)((colw + nc * 64) / 4 + 4 * s + g) * LD + (size_t)jc) * 4);
      // These are the only loads of the piece that the compiler sees, and it waits for them where
      // they are first used; it cannot count the loads issued above and inside the steps, so a wait
      // placed inside the loop would stand for "everything".  Using the values here puts that wait
      // (for everything, once per piece) in front of the loop instead.
#pragma unroll
      for (int nc = 0; nc < SYM_NC; ++nc)
        asm volatile("" :: "v"(dJ[nc][0]), "v"(dJ[nc][1]), "v"(dJ[nc][2]), "v"(dJ[nc][3]));
      sym_wait_vm<14>();
#pragma unroll
      for (int r = 0; r < 4; ++r) a1[0][r] = *(const f32x4*)(ring + rd1[r]);
#pragma unroll
      for (int s = 0; s < 4; ++s) a2[0][s] = *(const f32x4*)(ring + rd2[s]);
      f64x2 lo = dbuf[0], hi = dbuf[64];
      dn = (f64x4){lo[0], lo[1], hi[0], hi[1]};
    }
    int j0 = P.row_begin;
#pragma unroll 1
    for (int q0 = 0; q0 < nsteps; q0 += SYM_GROUP) {
      int ng = min(SYM_GROUP, nsteps - q0);
      int jg = j0;
      int so0 = __builtin_amdgcn_readfirstlane(jg / SYM_W);
      int sb0 = slot_base[so0], sb1 = slot_base[min(so0 + 1, P.strip - 1)];
      if (active) {
#pragma unroll 1
        for (int q = 0; q < ng; ++q, j0 += 16) {
          bool more = q0 + q + 1 < nsteps;
          if (more) gp += (size_t)16 * SYM_W;
          f64x4 out2;
          sym_step_dual(gp, Dq + (size_t)((more ? j0 + 16 : j0) / 4) * LD * 4, jc, g, ring, ring_bytes, dbuf,
                        dbuf_bytes, voff, voffd, rd1, rd2, a1, a2, dn, dJ, acc1, out2);
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
          // a group of rows touches at most two output panels; their slot numbers come by scalar
          // loads (a vector load here would make the compiler wait for every load in flight)
          int so = row / SYM_W;
          int slot = (so == so0 ? sb0 : sb1) + (P.strip - so - 1);
          double* dst = Vq + ((size_t)slot * np + (size_t)row) * LD + 8 * half;
          *(f64x4*)dst = lo;
          *(f64x4*)(dst + 4) = hi;
        }
      }
      __syncthreads();
    }
    if (active) {
      // loads of the (repeated) last step are still on their way to the ring: let them land
      // before the next piece refills it
      sym_wait_vm<0>();
      sym_wait_lds();
      double* vout = Vq + (size_t)P.slot * np * LD;
#pragma unroll
      for (int nc = 0; nc < SYM_NC; ++nc)
#pragma unroll
        for (int cc = 0; cc < 4; ++cc)
          *(f64x4*)(vout + (size_t)(colw + nc * 64 + 4 * jc + cc) * LD + g * 4) = acc1[nc][cc];
    }
  }
}

}  // namespace

// K_hat D from the triangular storage: per group of 16 right-hand-side columns one launch over
// the pieces above the diagonal blocks and one over the pieces inside them.
int launch_mm_sym(hipStream_t s, const float* Ktri, const double* D4, double* Vp, int np, int ld,
                  const MmPiece* pieces, const int* first_dual, int wgs_dual, const int* first_single,
                  int wgs_single, const int* slot_base, const DevState* st) {
  if (ld != 16 && ld != 32) return 1;
  for (int nq = 0; nq < ld / 16; ++nq) {
    if (wgs_dual > 0)
      k_mm_sym_dual<<<wgs_dual, 256, 0, s>>>(Ktri, D4 + 64 * nq, Vp + 16 * nq, np, ld, pieces, first_dual,
                                             slot_base, st);
    k_mm_sym_diag<<<wgs_single, 256, 0, s>>>(Ktri, D4 + 64 * nq, Vp + 16 * nq, np, ld, pieces, first_single, st);
  }
  return 0;
}
