// Host build of the quantizer-ratio arithmetic of the HIP kernels (csrc/mrem_quant_math.h), for
// tests/test_quant_math_cpu.py: the FMA form against the IEEE division, array at a time.
#include "../paper_2109_15082_amd/csrc/mrem_quant_math.h"

extern "C" void mrem_host_ratio_fma(const float* a, const float* z, const float* s, float* out, long n) {
  for (long i = 0; i < n; ++i) out[i] = mrem::quant_ratio_fma(a[i], z[i], s[i], mrem::quant_reciprocal(s[i]));
}
extern "C" void mrem_host_ratio_div(const float* a, const float* z, const float* s, float* out, long n) {
  for (long i = 0; i < n; ++i) out[i] = mrem::quant_ratio_div(a[i], z[i], s[i]);
}
