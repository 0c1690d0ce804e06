// Issue-rate probe for gfx950: time per wave instruction with one wave per SIMD, for the
// instruction mixes of the product kernels (fp64 MFMA alone and interleaved with conversions,
// integer VALU work, LDS reads, LDS writes and global loads).  Not part of the library.
//
//   hipcc -O3 --offload-arch=gfx950 -Xclang -target-feature -Xclang -packed-fp32-ops \
//         paper_1809_11165_amd/csrc/probes/issue_rates.hip -o issue_rates && ./issue_rates
//
// Every access stays inside the 32 KB of LDS and the two small device buffers allocated in main();
// loads issued by the asm statements are drained by the s_waitcnt before the end of the kernel.
// Findings on MI355X that the kernels in this directory rely on: v_mfma_f64_16x16x4 takes 64
// cycles, v_mfma_f64_4x4x4 16 (the same flop rate); a VALU instruction between fp64 MFMAs adds its
// own ~5 cycles (no overlap); LDS reads and global loads add nothing; an LDS write adds ~11 cycles
// per dword (45 per ds_write_b128), wherever it is placed.  At the density of one 8-byte LDS read per
// 4x4x4 MFMA (16 cycles) the reads are no longer free: ~3 cycles each.  v_exp_f32 and v_sqrt_f32
// take 9.3 cycles per wave (other vector instructions 5.6), ~10 between MFMAs; fp64 MFMAs that
// accumulate onto one register issue back to back at the full rate (no wait for the result of the
// one before); v_mfma_f32_16x16x4 takes 32 cycles.
#include <hip/hip_runtime.h>
#include <cstdio>
typedef double f64x4 __attribute__((ext_vector_type(4)));
#define REP 64
template <int MODE>
__global__ __launch_bounds__(256) void k(double* out, const float* in, int iters) {
  int lane = threadIdx.x;
  typedef float f32x4 __attribute__((ext_vector_type(4)));
  __shared__ float lds[8192];   // 32 KB: 256 lanes x 16 B x 4 offsets (+4096 B steps) fit
  f32x4 q0 = {0, 0, 0, 0}, q1 = q0, q2 = q0, q3 = q0;
  for (int i = lane; i < 8192; i += 256) lds[i] = 0.f;
  __syncthreads();
  float f[8];
  for (int i = 0; i < 8; ++i) f[i] = in[lane + 64 * i];
  double acc0 = 0, acc1 = 0, acc2 = 0, acc3 = 0;
  f64x4 m0 = {0, 0, 0, 0}, m1 = m0, m2 = m0, m3 = m0;
  double a = in[lane], b = in[lane + 1];
  unsigned u[4] = {__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3])};
  long long t0 = clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < REP; ++r) {
      if (MODE == 0) {   // 4 cvt f64<-f32
        double d0, d1, d2, d3;
        asm volatile("v_cvt_f64_f32 %0, %4\n v_cvt_f64_f32 %1, %5\n v_cvt_f64_f32 %2, %6\n v_cvt_f64_f32 %3, %7"
                     : "=v"(d0), "=v"(d1), "=v"(d2), "=v"(d3) : "v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
        acc0 += 0; asm volatile("" ::"v"(d0), "v"(d1), "v"(d2), "v"(d3));
      } else if (MODE == 1) {   // 4 independent v_fma_f64
        asm volatile("v_fma_f64 %0, %4, %5, %0\n v_fma_f64 %1, %4, %5, %1\n v_fma_f64 %2, %4, %5, %2\n v_fma_f64 %3, %4, %5, %3"
                     : "+v"(acc0), "+v"(acc1), "+v"(acc2), "+v"(acc3) : "v"(a), "v"(b));
      } else if (MODE == 2) {   // 4 integer shifts
        asm volatile("v_lshrrev_b32 %0, 3, %0\n v_lshrrev_b32 %1, 3, %1\n v_lshrrev_b32 %2, 3, %2\n v_lshrrev_b32 %3, 3, %3"
                     : "+v"(u[0]), "+v"(u[1]), "+v"(u[2]), "+v"(u[3]));
      } else if (MODE == 3) {   // 4 mfma f64 16x16x4 on independent accumulators
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
      } else if (MODE == 4) {   // 4 mfma f64 4x4x4 (4 blocks)
        acc0 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc0, 0, 0, 0);
        acc1 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc1, 0, 0, 0);
        acc2 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc2, 0, 0, 0);
        acc3 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc3, 0, 0, 0);
      } else if (MODE == 5) {   // 4 mfma + 4 cvt interleaved (as in the product kernels)
        double d0, d1, d2, d3;
        asm volatile("v_cvt_f64_f32 %0, %4\n v_cvt_f64_f32 %1, %5\n v_cvt_f64_f32 %2, %6\n v_cvt_f64_f32 %3, %7"
                     : "=v"(d0), "=v"(d1), "=v"(d2), "=v"(d3) : "v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d0, m0, 0, 0, 0);
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d1, m1, 0, 0, 0);
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d2, m2, 0, 0, 0);
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d3, m3, 0, 0, 0);
      } else if (MODE == 6) {   // 4 mfma + 16 integer ops interleaved
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        asm volatile("v_lshrrev_b32 %0, 3, %0\n v_lshrrev_b32 %1, 3, %1\n v_lshrrev_b32 %2, 3, %2\n v_lshrrev_b32 %3, 3, %3"
                     : "+v"(u[0]), "+v"(u[1]), "+v"(u[2]), "+v"(u[3]));
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        asm volatile("v_lshrrev_b32 %0, 3, %0\n v_lshrrev_b32 %1, 3, %1\n v_lshrrev_b32 %2, 3, %2\n v_lshrrev_b32 %3, 3, %3"
                     : "+v"(u[0]), "+v"(u[1]), "+v"(u[2]), "+v"(u[3]));
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        asm volatile("v_lshrrev_b32 %0, 3, %0\n v_lshrrev_b32 %1, 3, %1\n v_lshrrev_b32 %2, 3, %2\n v_lshrrev_b32 %3, 3, %3"
                     : "+v"(u[0]), "+v"(u[1]), "+v"(u[2]), "+v"(u[3]));
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
        asm volatile("v_lshrrev_b32 %0, 3, %0\n v_lshrrev_b32 %1, 3, %1\n v_lshrrev_b32 %2, 3, %2\n v_lshrrev_b32 %3, 3, %3"
                     : "+v"(u[0]), "+v"(u[1]), "+v"(u[2]), "+v"(u[3]));
      } else if (MODE == 7) {   // 4 cvt f32<-f64 style: v_cvt_f32_f64 ... not needed; 4 v_fma_f32
        asm volatile("v_fma_f32 %0, %4, %5, %0\n v_fma_f32 %1, %4, %5, %1\n v_fma_f32 %2, %4, %5, %2\n v_fma_f32 %3, %4, %5, %3"
                     : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]) : "v"(f[4]), "v"(f[5]));
      } else if (MODE == 8) {   // 4 mfma + 4 ds_read_b128, no waits inside
        unsigned ad = 16 * lane;
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        asm volatile("ds_read_b128 %0, %1" : "=v"(q0) : "v"(ad));
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        asm volatile("ds_read_b128 %0, %1 offset:4096" : "=v"(q1) : "v"(ad));
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(q2) : "v"(ad));
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
        asm volatile("ds_read_b128 %0, %1 offset:12288" : "=v"(q3) : "v"(ad));
      } else if (MODE == 9) {   // 4 mfma + 1 global_load_dwordx4 (cached), no waits inside
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(q0) : "v"(in + 4 * (lane & 63)));
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
      } else if (MODE == 10) {   // 4 mfma + 4 ds_write_b128, no waits inside
        unsigned ad = 16 * lane;
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        asm volatile("ds_write_b128 %0, %1" : : "v"(ad), "v"(q0));
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        asm volatile("ds_write_b128 %0, %1 offset:4096" : : "v"(ad), "v"(q0));
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        asm volatile("ds_write_b128 %0, %1 offset:8192" : : "v"(ad), "v"(q0));
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
        asm volatile("ds_write_b128 %0, %1 offset:12288" : : "v"(ad), "v"(q0));
      } else if (MODE == 12) {   // 4 ds_write_b128 back to back, then 4 mfma
        unsigned ad = 16 * lane;
        asm volatile("ds_write_b128 %0, %1\n ds_write_b128 %0, %1 offset:4096\n ds_write_b128 %0, %1 offset:8192\n ds_write_b128 %0, %1 offset:12288" : : "v"(ad), "v"(q0));
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
      } else if (MODE == 13) {   // 4 cvt, 4 ds_write_b128, 4 mfma
        unsigned ad = 16 * lane;
        double d0, d1, d2, d3;
        asm volatile("v_cvt_f64_f32 %0, %4\n v_cvt_f64_f32 %1, %5\n v_cvt_f64_f32 %2, %6\n v_cvt_f64_f32 %3, %7"
                     : "=v"(d0), "=v"(d1), "=v"(d2), "=v"(d3) : "v"(f[0]), "v"(f[1]), "v"(f[2]), "v"(f[3]));
        asm volatile("ds_write_b128 %0, %1\n ds_write_b128 %0, %1 offset:4096\n ds_write_b128 %0, %1 offset:8192\n ds_write_b128 %0, %1 offset:12288" : : "v"(ad), "v"(q0));
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d0, m0, 0, 0, 0);
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d1, m1, 0, 0, 0);
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d2, m2, 0, 0, 0);
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, d3, m3, 0, 0, 0);
      } else if (MODE == 14) {   // 4 mfma interleaved with 4 ds_write_b32
        unsigned ad = 4 * lane;
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        asm volatile("ds_write_b32 %0, %1" : : "v"(ad), "v"(f[0]));
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        asm volatile("ds_write_b32 %0, %1 offset:4096" : : "v"(ad), "v"(f[0]));
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        asm volatile("ds_write_b32 %0, %1 offset:8192" : : "v"(ad), "v"(f[0]));
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
        asm volatile("ds_write_b32 %0, %1 offset:12288" : : "v"(ad), "v"(f[0]));
      } else if (MODE == 15) {   // 16 mfma, then 4 ds_write_b128 back to back
        unsigned ad = 16 * lane;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
          m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
          m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
          m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
        }
        asm volatile("ds_write_b128 %0, %1\n ds_write_b128 %0, %1 offset:4096\n ds_write_b128 %0, %1 offset:8192\n ds_write_b128 %0, %1 offset:12288" : : "v"(ad), "v"(q0));
      } else if (MODE == 17) {   // 4 mfma4 + 4 ds_read_b64 (broadcast over lane/4%4, as the row-side A operand would be)
        unsigned ad = ((lane >> 4) * 4 * 13 + (lane & 3)) * 8;
        double x0, x1, x2, x3;
        asm volatile("ds_read_b64 %0, %1" : "=v"(x0) : "v"(ad));
        acc0 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc0, 0, 0, 0);
        asm volatile("ds_read_b64 %0, %1 offset:32" : "=v"(x1) : "v"(ad));
        acc1 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc1, 0, 0, 0);
        asm volatile("ds_read_b64 %0, %1 offset:64" : "=v"(x2) : "v"(ad));
        acc2 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc2, 0, 0, 0);
        asm volatile("ds_read_b64 %0, %1 offset:104" : "=v"(x3) : "v"(ad));
        acc3 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc3, 0, 0, 0);
        asm volatile("" :: "v"(x0), "v"(x1), "v"(x2), "v"(x3));
      } else if (MODE == 18) {   // as 17 plus 1 ds_read_b128 (the transposed tile reads) per 4 mfma4
        unsigned ad = ((lane >> 4) * 4 * 13 + (lane & 3)) * 8;
        unsigned ad2 = 16 * lane;
        double x0, x1, x2, x3;
        asm volatile("ds_read_b64 %0, %1" : "=v"(x0) : "v"(ad));
        acc0 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc0, 0, 0, 0);
        asm volatile("ds_read_b64 %0, %1 offset:32" : "=v"(x1) : "v"(ad));
        acc1 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc1, 0, 0, 0);
        asm volatile("ds_read_b64 %0, %1 offset:64" : "=v"(x2) : "v"(ad));
        acc2 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc2, 0, 0, 0);
        asm volatile("ds_read_b64 %0, %1 offset:104" : "=v"(x3) : "v"(ad));
        acc3 = __builtin_amdgcn_mfma_f64_4x4x4f64(a, b, acc3, 0, 0, 0);
        asm volatile("ds_read_b128 %0, %1 offset:8192" : "=v"(q1) : "v"(ad2));
        asm volatile("" :: "v"(x0), "v"(x1), "v"(x2), "v"(x3));
      } else if (MODE == 11) {   // 4 mfma + 4 global_load_dwordx4 (cached), no waits inside
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(q0) : "v"(in + 4 * (lane & 63)));
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(q1) : "v"(in + 4 * (lane & 63)));
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(q2) : "v"(in + 4 * (lane & 63)));
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
        asm volatile("global_load_dwordx4 %0, %1, off" : "=v"(q3) : "v"(in + 4 * (lane & 63)));
      } else if (MODE == 19) {   // 4 independent v_exp_f32 (the transcendental unit)
        asm volatile("v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3"
                     : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
      } else if (MODE == 20) {   // 4 independent v_sqrt_f32
        asm volatile("v_sqrt_f32 %0, %0\n v_sqrt_f32 %1, %1\n v_sqrt_f32 %2, %2\n v_sqrt_f32 %3, %3"
                     : "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]));
      } else if (MODE == 21) {   // 4 mfma f64 16x16x4 + 4 v_exp_f32 interleaved
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        asm volatile("v_exp_f32 %0, %0" : "+v"(f[0]));
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        asm volatile("v_exp_f32 %0, %0" : "+v"(f[1]));
        m2 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m2, 0, 0, 0);
        asm volatile("v_exp_f32 %0, %0" : "+v"(f[2]));
        m3 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m3, 0, 0, 0);
        asm volatile("v_exp_f32 %0, %0" : "+v"(f[3]));
      } else if (MODE == 22) {   // 4 mfma f64 16x16x4 on ONE accumulator (each waits for the one before)
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
      } else if (MODE == 23) {   // ... on TWO accumulators in turn
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
        m0 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m0, 0, 0, 0);
        m1 = __builtin_amdgcn_mfma_f64_16x16x4f64(a, b, m1, 0, 0, 0);
      } else if (MODE == 24) {   // 4 mfma f32 16x16x4 on independent accumulators
        typedef float f32x4b __attribute__((ext_vector_type(4)));
        float af = f[4], bf = f[5];
        q0 = __builtin_amdgcn_mfma_f32_16x16x4f32(af, bf, q0, 0, 0, 0);
        q1 = __builtin_amdgcn_mfma_f32_16x16x4f32(af, bf, q1, 0, 0, 0);
        q2 = __builtin_amdgcn_mfma_f32_16x16x4f32(af, bf, q2, 0, 0, 0);
        q3 = __builtin_amdgcn_mfma_f32_16x16x4f32(af, bf, q3, 0, 0, 0);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  long long t1 = clock64();
  double s = acc0 + acc1 + acc2 + acc3 + m0[0] + m1[1] + m2[2] + m3[3] + u[0] + u[1] + u[2] + u[3] + f[0] + f[1] + f[2] + f[3] + q0[0] + q1[1] + q2[2] + q3[3];
  out[blockIdx.x * 256 + threadIdx.x] = s;
  if (threadIdx.x == 0 && blockIdx.x == 0) out[1 << 20] = (double)(t1 - t0);
}
template <int MODE>
void run(const char* name, double* out, float* in, int per_rep) {
  int iters = 200;
  hipEvent_t e0, e1;
  hipEventCreate(&e0); hipEventCreate(&e1);
  k<MODE><<<256, 256>>>(out, in, 10);
  hipDeviceSynchronize();
  hipEventRecord(e0);
  k<MODE><<<256, 256>>>(out, in, iters);
  hipEventRecord(e1);
  hipDeviceSynchronize();
  float ms; hipEventElapsedTime(&ms, e0, e1);
  double n_inst = (double)iters * REP * per_rep;
  // 1 wave per SIMD; cycles at 2.4 GHz nominal
  printf("%-40s %8.3f ms  %.2f ns per wave-instruction  (%.1f cycles at 2.4 GHz)\n", name, ms, ms * 1e6 / n_inst, ms * 1e6 / n_inst * 2.4);
  fflush(stdout);
}
int main() {
  double* out; float* in;
  hipMalloc(&out, ((1 << 20) + 8) * sizeof(double));
  hipMalloc(&in, 4096 * sizeof(float));
  hipMemset(in, 0, 4096 * sizeof(float));
  run<0>("v_cvt_f64_f32 x4", out, in, 4);
  run<1>("v_fma_f64 x4", out, in, 4);
  run<2>("v_lshrrev_b32 x4", out, in, 4);
  run<7>("v_fma_f32 x4", out, in, 4);
  run<3>("mfma_f64_16x16x4 x4", out, in, 4);
  run<4>("mfma_f64_4x4x4 x4", out, in, 4);
  run<5>("4 mfma16 + 4 cvt (per group of 8)", out, in, 8);
  run<6>("4 mfma16 + 16 int (per group of 20)", out, in, 20);
  run<8>("4 mfma16 + 4 ds_read_b128 (per group of 8)", out, in, 8);
  run<9>("4 mfma16 + 1 global_load_x4 (per group of 5)", out, in, 5);
  run<11>("4 mfma16 + 4 global_load_x4 (per group of 8)", out, in, 8);
  run<10>("4 mfma16 + 4 ds_write_b128 (per group of 8)", out, in, 8);
  run<12>("4 ds_write_b128 bunched + 4 mfma (group of 8)", out, in, 8);
  run<13>("4 cvt + 4 ds_write_b128 + 4 mfma (group of 12)", out, in, 12);
  run<14>("4 mfma + 4 ds_write_b32 interleaved (group of 8)", out, in, 8);
  run<15>("16 mfma + 4 ds_write_b128 bunched (group of 20)", out, in, 20);
  run<17>("4 mfma4 + 4 ds_read_b64 broadcast (group of 8)", out, in, 8);
  run<18>("4 mfma4 + 4 ds_read_b64 + 1 ds_read_b128 (group of 9)", out, in, 9);
  run<19>("v_exp_f32 x4", out, in, 4);
  run<20>("v_sqrt_f32 x4", out, in, 4);
  run<21>("4 mfma16 + 4 v_exp_f32 (per group of 8)", out, in, 8);
  run<22>("mfma_f64_16x16x4 x4 on one accumulator", out, in, 4);
  run<23>("mfma_f64_16x16x4 x4 on two accumulators in turn", out, in, 4);
  run<24>("mfma_f32_16x16x4 x4", out, in, 4);
  run<4>("mfma_f64_4x4x4 x4 again", out, in, 4);
  run<3>("mfma_f64_16x16x4 x4 again", out, in, 4);
  hipError_t e = hipGetLastError();
  printf("status %s\n", hipGetErrorString(e));
  return 0;
}
