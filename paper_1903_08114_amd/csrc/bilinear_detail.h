// Shared by the two bilinear-form kernels (kmm_bilinear.hip for d <= 31, kmm_bilinear_wide.hip beyond).
#pragma once

#include "egp_internal.h"

namespace egp {
namespace bilinear_detail {

typedef float f4 __attribute__((ext_vector_type(4)));

constexpr float kLn2 = 0.6931471805599453f;

// h(r) and g(r) up to the constant factors the host applies (see kmm_grad.hip): returns h', sets g'
template <int KIND>
__device__ __forceinline__ float hg(float acc, float* g) {
  if constexpr (KIND == EGP_RBF) {
    const float e = __builtin_amdgcn_exp2f(-acc);
    *g = e;
    return e;
  } else if constexpr (KIND == EGP_MATERN32) {
    const float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
    const float e = __builtin_amdgcn_exp2f(-a);
    *g = __builtin_fmaf(a, kLn2, 1.0f) * e;
    return e;
  } else if constexpr (KIND == EGP_MATERN12) {
    // g = exp(-r), h = exp(-r) / r: the 1/r does not cancel here. A point against itself (acc = 0) has a zero
    // squared difference in every feature; its weight is set to 0 so that 0 * inf cannot arise.
    const float m = __builtin_fabsf(acc);
    const float e = __builtin_amdgcn_exp2f(-__builtin_amdgcn_sqrtf(m));
    *g = e;
    return m > 0.f ? e * __builtin_amdgcn_rsqf(m) : 0.f;
  } else {
    const float a = __builtin_amdgcn_sqrtf(__builtin_fabsf(acc));
    const float e = __builtin_amdgcn_exp2f(-a);
    const float lin = __builtin_fmaf(a, kLn2, 1.0f);
    *g = __builtin_fmaf(a * a, kLn2 * kLn2 / 3.0f, lin) * e;
    return lin * e;
  }
}

// d > 31, defined in kmm_bilinear_wide.hip
size_t bilinear_wide_ws_bytes(int64_t n, int d, int t);
int bilinear_wide_core(const Prepared& P, const egp_hyper_t* h, const float* A, const float* B, int t,
                       const float* wcol, double* out, void* ws2, hipStream_t stream);

}  // namespace bilinear_detail
}  // namespace egp
