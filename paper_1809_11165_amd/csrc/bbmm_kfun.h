// Kernel functions on fp32 tiles / pairs, shared by the tile kernels.  Inputs are squared
// distances of coordinates that were centred and scaled beforehand (HypArgs::xscale).
#pragma once

#include <hip/hip_runtime.h>

constexpr float kSqrt5 = 2.2360679774997896964f;
constexpr float kLog2e = 1.4426950408889634074f;
// sqrt(5) * log2(e) as the nearest float, and ln(2) times what that rounding drops: the exponent
// is evaluated with the float, the dropped part re-enters as the factor (1 - kMatExpFix * rho),
// so the value carries no bias that grows with rho.
constexpr float kMatExpC = 3.225964069366455f;
constexpr float kMatExpFix = 7.8230743523e-8f;

// Unit-outputscale kernel value from the scaled squared distance.
//   RBF:      inputs were scaled by sqrt(log2(e)/2)/l, so k/s = 2^(-r2)
//   Matern52: inputs were scaled by 1/l, rho = sqrt(r2), k/s = (1 + sqrt5 rho + 5/3 rho^2) e^(-sqrt5 rho)
template <int KIND>
__device__ __forceinline__ float unit_kernel(float r2) {
  if (KIND == 0) {
    return __builtin_amdgcn_exp2f(-r2);
  } else {
    float rho = __builtin_amdgcn_sqrtf(r2);
    float e = __builtin_amdgcn_exp2f(-kMatExpC * rho);
    float poly = fmaf(rho, fmaf(rho, 5.f / 3.f, kSqrt5), 1.f);
    float v = poly * e;
    return fmaf(-kMatExpFix * rho, v, v);
  }
}

// Kernel value and the radial weight g of the lengthscale derivative
//   dk/dl_d = s * g * (Delta_d / l_d)^2 / l_d,   g = k/s (RBF),  g = (5/3)(1 + sqrt5 rho) e^(-sqrt5 rho) (Matern52)
template <int KIND>
__device__ __forceinline__ void unit_kernel_and_weight(float r2, float& e_out, float& g_out) {
  if (KIND == 0) {
    float e = __builtin_amdgcn_exp2f(-r2);
    e_out = e;
    g_out = e;
  } else {
    float rho = __builtin_amdgcn_sqrtf(r2);
    float e = __builtin_amdgcn_exp2f(-kMatExpC * rho);
    e = fmaf(-kMatExpFix * rho, e, e);
    e_out = fmaf(rho, fmaf(rho, 5.f / 3.f, kSqrt5), 1.f) * e;
    g_out = (5.f / 3.f) * fmaf(rho, kSqrt5, 1.f) * e;
  }
}

