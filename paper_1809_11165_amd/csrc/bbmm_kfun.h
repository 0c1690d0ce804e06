// Kernel functions on fp32 tiles / pairs, shared by the tile kernels.  Inputs are squared
// distances of coordinates that were centred and scaled beforehand (HypArgs::xscale).
#pragma once

#include <hip/hip_runtime.h>

// Matern-5/2 with inputs scaled by sqrt(5) log2(e) / l: the scaled distance a = sqrt(r2) is the
// exponent itself, k/s = (1 + sqrt5 rho + 5/3 rho^2) e^(-sqrt5 rho) = (1 + kMatK1 a + kMatK2 a^2) 2^(-a),
// kMatK1 = ln 2, kMatK2 = (ln 2)^2 / 3.  (No constant multiplies the distance any more, so no rounded
// constant can bias the exponent: the scale factor is applied to the coordinates in fp64.)
constexpr float kMatK1 = 0.69314718055994530942f;
constexpr float kMatK2 = 0.16015100463940046f;

// Unit-outputscale kernel value from the scaled squared distance.
//   RBF:      inputs were scaled by sqrt(log2(e)/2)/l, so k/s = 2^(-r2)
//   Matern52: inputs were scaled by sqrt(5) log2(e)/l, a = sqrt(r2), k/s = (1 + K1 a + K2 a^2) 2^(-a)
template <int KIND>
__device__ __forceinline__ float unit_kernel(float r2) {
  if (KIND == 0) {
    return __builtin_amdgcn_exp2f(-r2);
  } else {
    float a = __builtin_amdgcn_sqrtf(r2);
    float e = __builtin_amdgcn_exp2f(-a);
    float poly = fmaf(a, fmaf(a, kMatK2, kMatK1), 1.f);
    return poly * e;
  }
}

// Kernel value and the radial weight g of the lengthscale derivative
//   dk/dl_d = s * g * (Delta_d / l_d)^2 / l_d,   g = k/s (RBF),  g = (5/3)(1 + sqrt5 rho) e^(-sqrt5 rho)
//   = (5/3)(1 + K1 a) 2^(-a) (Matern52)
template <int KIND>
__device__ __forceinline__ void unit_kernel_and_weight(float r2, float& e_out, float& g_out) {
  if (KIND == 0) {
    float e = __builtin_amdgcn_exp2f(-r2);
    e_out = e;
    g_out = e;
  } else {
    float a = __builtin_amdgcn_sqrtf(r2);
    float e = __builtin_amdgcn_exp2f(-a);
    e_out = fmaf(a, fmaf(a, kMatK2, kMatK1), 1.f) * e;
    g_out = fmaf(a, (5.f / 3.f) * kMatK1, 5.f / 3.f) * e;
  }
}

