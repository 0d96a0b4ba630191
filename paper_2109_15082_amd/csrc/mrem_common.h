// Device-side helpers shared by the gfx950 kernels of the MREM module step.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "mrem_quant_math.h"

namespace mrem {

typedef __bf16 bf16_t;

constexpr int kWave = 64;  // CDNA wavefront width

// ---- storage type access: everything computes in fp32 ------------------------
__device__ __forceinline__ float ldf(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const bf16_t* p, size_t i) { return static_cast<float>(p[i]); }
__device__ __forceinline__ void stf(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void stf(bf16_t* p, size_t i, float v) { p[i] = static_cast<bf16_t>(v); }

// value after a round trip through the storage type (round-to-nearest-even)
template <class T>
__device__ __forceinline__ float round_to(float v);
template <>
__device__ __forceinline__ float round_to<float>(float v) { return v; }
template <>
__device__ __forceinline__ float round_to<bf16_t>(float v) { return static_cast<float>(static_cast<bf16_t>(v)); }

// ---- the quantizer of Eq. 1 (Section 3.1) -----------------------------------
// v = (a - z) / s as two IEEE fp32 operations; code = nearest-even(clamp(v));
// inside = [qn <= v <= qp] is the straight-through mask (Section 3.1.1).
struct QuantParam {
  float s, z, qn, qp;
  int on;    // 0: quantizer disabled (identity)
  float rs;  // correctly rounded 1 / s (only for q_ratio_fma)
};

__device__ __forceinline__ float q_ratio(float a, const QuantParam& q) { return quant_ratio_div(a, q.z, q.s); }
// the FMA form of the same quotient (mrem_quant_math.h), with q.rs = quant_reciprocal(q.s)
__device__ __forceinline__ float q_ratio_fma(float a, const QuantParam& q) { return quant_ratio_fma(a, q.z, q.s, q.rs); }
// fp32 storage (the check mode) divides; bf16 storage uses the FMA form
template <class T>
__device__ __forceinline__ float q_ratio_t(float a, const QuantParam& q) {
  if constexpr (sizeof(T) == 4) return q_ratio(a, q);
  else return q_ratio_fma(a, q);
}
__device__ __forceinline__ float q_code(float v, const QuantParam& q) { return rintf(fminf(fmaxf(v, q.qn), q.qp)); }
__device__ __forceinline__ bool q_inside(float v, const QuantParam& q) { return v >= q.qn && v <= q.qp; }

// ---- reductions --------------------------------------------------------------
// Sum over the 64 lanes with data-parallel-primitive moves (no trip through the LDS crossbar): four steps inside
// each row of 16 lanes (neighbour, pair, mirrored half row, mirrored row) leave every lane with its row's sum; two
// row broadcasts carry the sums of rows 0 and 2 into rows 1 and 3 and that of rows 0..1 into rows 2..3, so the last
// lane holds the total, which is read back as a wavefront-uniform value.  Fixed order: deterministic.
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_term(float v) {
  // lanes of rows outside ROW_MASK receive 0
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xF, false));
}
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_term<0xB1, 0xF>(v);   // quad_perm [1,0,3,2]
  v += dpp_term<0x4E, 0xF>(v);   // quad_perm [2,3,0,1]
  v += dpp_term<0x141, 0xF>(v);  // row_half_mirror
  v += dpp_term<0x140, 0xF>(v);  // row_mirror
  v += dpp_term<0x142, 0xA>(v);  // row_bcast15 into rows 1 and 3
  v += dpp_term<0x143, 0xC>(v);  // row_bcast31 into rows 2 and 3
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}
__device__ __forceinline__ float wave_min(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v = fminf(v, __shfl_xor(v, o, kWave));
  return v;
}

// Sum over a block of up to 1024 threads (blockDim.x multiple of 64). Result valid
// in every thread.  `scratch` is 17 floats of LDS.  Fixed order: deterministic.
__device__ __forceinline__ float block_sum(float v, float* scratch) {
  v = wave_sum(v);
  const int w = threadIdx.x / kWave, nw = blockDim.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) scratch[w] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int i = 0; i < nw; ++i) t += scratch[i];
    scratch[16] = t;
  }
  __syncthreads();
  return scratch[16];
}
__device__ __forceinline__ float block_max(float v, float* scratch) {
  v = wave_max(v);
  const int w = threadIdx.x / kWave, nw = blockDim.x / kWave;
  __syncthreads();
  if ((threadIdx.x & (kWave - 1)) == 0) scratch[w] = v;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = scratch[0];
    for (int i = 1; i < nw; ++i) t = fmaxf(t, scratch[i]);
    scratch[16] = t;
  }
  __syncthreads();
  return scratch[16];
}

__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.0f + erff(u * 0.70710678118654752440f)) + u * __expf(-0.5f * u * u) * 0.39894228040143267794f;
}

// erf(x) = 1 - 1 / (1 + a1 x + ... + a6 x^6)^16 for x >= 0 (Abramowitz & Stegun 7.1.28; absolute
// error below 3e-7 in exact arithmetic, about 2e-6 in fp32): a fraction of the instructions of
// erff, and far inside what survives the rounding of GELU outputs to bf16.
__device__ __forceinline__ float erf_rational(float x) {
  const float ax = fabsf(x);
  float p = 0.0000430638f;
  p = fmaf(p, ax, 0.0002765672f);
  p = fmaf(p, ax, 0.0001520143f);
  p = fmaf(p, ax, 0.0092705272f);
  p = fmaf(p, ax, 0.0422820123f);
  p = fmaf(p, ax, 0.0705230784f);
  p = fmaf(p, ax, 1.0f);
  p *= p; p *= p; p *= p; p *= p;
  return copysignf(1.0f - __builtin_amdgcn_rcpf(p), x);
}
// GELU and its derivative for values stored as T: fp32 storage (the check mode) uses erff
template <class T>
__device__ __forceinline__ float gelu_t(float u) {
  if constexpr (sizeof(T) == 4) return gelu_f(u);
  else return 0.5f * u * (1.0f + erf_rational(u * 0.70710678118654752440f));
}
template <class T>
__device__ __forceinline__ float gelu_grad_t(float u) {
  if constexpr (sizeof(T) == 4) return gelu_grad_f(u);
  else return 0.5f * (1.0f + erf_rational(u * 0.70710678118654752440f)) + u * __expf(-0.5f * u * u) * 0.39894228040143267794f;
}

}  // namespace mrem
