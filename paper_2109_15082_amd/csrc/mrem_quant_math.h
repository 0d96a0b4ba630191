// The ratio that decides a quantizer code (Section 3.1, Eq. 1): v = (a - z) / s, taken as
// IEEE fp32 operations.  Kept in a header of its own, free of HIP types, so that the same
// source also builds for the host, where a test compares the FMA form with the division.
#pragma once

#include <math.h>

#if defined(__HIPCC__)
#include <hip/hip_runtime.h>
#define MREM_HD __host__ __device__ __forceinline__
#else
#define MREM_HD inline
#endif

namespace mrem {

// single IEEE operations that the compiler may not contract into a fused one
MREM_HD float fp_sub(float a, float b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __fsub_rn(a, b);
#else
  volatile float r = a - b;
  return r;
#endif
}
MREM_HD float fp_mul(float a, float b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __fmul_rn(a, b);
#else
  volatile float r = a * b;
  return r;
#endif
}
MREM_HD float fp_div(float a, float b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __fdiv_rn(a, b);
#else
  volatile float r = a / b;
  return r;
#endif
}
MREM_HD float fp_fma(float a, float b, float c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __fmaf_rn(a, b, c);
#else
  return fmaf(a, b, c);
#endif
}

// v = (a - z) / s as two IEEE fp32 operations
MREM_HD float quant_ratio_div(float a, float z, float s) { return fp_div(fp_sub(a, z), s); }

// The same quotient without the division sequence: with rs the correctly rounded reciprocal of s,
// t = fl(n * rs), then t + fl(n - s * t) * rs with fused multiply-adds: the residual n - s * t is
// exact and the last operation rounds the true quotient (the residual-correction step of FMA
// division); activations and step sizes are far from the overflow and underflow ranges where that
// needs care.  One step size serves millions of elements, so the reciprocal is taken once per thread.
MREM_HD float quant_ratio_fma(float a, float z, float s, float rs) {
  const float n = fp_sub(a, z);
  const float t = fp_mul(n, rs);
  return fp_fma(fp_fma(-s, t, n), rs, t);
}
MREM_HD float quant_reciprocal(float s) { return fp_div(1.0f, s); }

}  // namespace mrem
