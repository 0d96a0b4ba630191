// Device-side helpers shared by the gfx950 kernels of the MREM module step.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

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
  int on;  // 0: quantizer disabled (identity)
};

__device__ __forceinline__ float q_ratio(float a, const QuantParam& q) { return __fdiv_rn(__fsub_rn(a, q.z), q.s); }
__device__ __forceinline__ float q_code(float v, const QuantParam& q) { return rintf(fminf(fmaxf(v, q.qn), q.qp)); }
__device__ __forceinline__ bool q_inside(float v, const QuantParam& q) { return v >= q.qn && v <= q.qp; }

// ---- reductions --------------------------------------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
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

// Cross-block reduction without atomics on the data: every block stores its
// partial(s), then calls this.  It returns true (uniformly) in the block that
// arrives last; that block then sums the partials in index order, which makes the
// result independent of scheduling.  The counter must be 0 on entry of the grid
// and is reset by the last block.
__device__ __forceinline__ bool last_block_arrives(unsigned* counter, unsigned nblocks) {
  __shared__ int is_last_;
  __threadfence();
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned t = atomicAdd(counter, 1u);
    is_last_ = (t == nblocks - 1u);
    if (is_last_) *counter = 0u;
  }
  __syncthreads();
  if (is_last_) __threadfence();
  return is_last_ != 0;
}

__device__ __forceinline__ float gelu_f(float u) { return 0.5f * u * (1.0f + erff(u * 0.70710678118654752440f)); }
__device__ __forceinline__ float gelu_grad_f(float u) {
  return 0.5f * (1.0f + erff(u * 0.70710678118654752440f)) + u * __expf(-0.5f * u * u) * 0.39894228040143267794f;
}

}  // namespace mrem
