// Softmax attention of one encoder layer on quantizer codes (Section 3.1: both
// operands of Q*K^T and of P*V are quantized; the softmax probabilities use the
// unsigned grid), forward and straight-through backward.
//
// This file holds the scalar-ALU version: one wavefront per query row (forward,
// and the row part of backward) or per key row (column part of backward).  The
// operands are the integer-valued code tensors produced by qkv_quantize, so all
// dot products of codes are exact in fp32.
#include "mrem_common.h"
#include "mrem_kernels.h"

namespace mrem {

constexpr int kMaxKeysPerLane = 8;  // seq <= 512
constexpr int kMaxHeadDim = 128;

__device__ __forceinline__ void ld8(const float* p, float* o) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void ld8(const bf16_t* p, float* o) {
  const uint4 r = *reinterpret_cast<const uint4*>(p);
  o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
  o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
  o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
  o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
}

struct AttnScales {
  float qk;      // s_q * s_k / sqrt(d)
  float sp, sv;  // steps of P and V (1 when that quantizer is off)
  float sq, sk;
  int p_on;
  float p_qp;
};
__device__ __forceinline__ AttnScales load_scales(const AttnQ& a, int d) {
  AttnScales s;
  s.sq = a.q.on ? *a.q.s : 1.f;
  s.sk = a.k.on ? *a.k.s : 1.f;
  s.sp = a.p.on ? *a.p.s : 1.f;
  s.sv = a.v.on ? *a.v.s : 1.f;
  s.qk = s.sq * s.sk / sqrtf((float)d);
  s.p_on = a.p.on;
  s.p_qp = a.p.qp;
  return s;
}

// Softmax probabilities of query row i against all keys; lane l owns keys l, l+64, ...
// qrow: the query's codes in LDS.  Returns through p[].
template <class T>
__device__ __forceinline__ void prob_row(const T* __restrict__ kbase, int ld, const float* qrow, int S, int len, int d, float qk,
                                         float* p) {
  const int lane = threadIdx.x & 63;
  float mx = -INFINITY;
#pragma unroll
  for (int jj = 0; jj < kMaxKeysPerLane; ++jj) {
    const int j = lane + 64 * jj;
    float a = -INFINITY;
    if (j < S && j < len) {
      float dot = 0.f;
      for (int e = 0; e < d; e += 8) {
        float kv[8];
        ld8(kbase + (size_t)j * ld + e, kv);
#pragma unroll
        for (int t = 0; t < 8; ++t) dot += qrow[e + t] * kv[t];
      }
      a = dot * qk;
    }
    p[jj] = a;
    mx = fmaxf(mx, a);
  }
  mx = wave_max(mx);
  float sum = 0.f;
#pragma unroll
  for (int jj = 0; jj < kMaxKeysPerLane; ++jj) {
    const float e = (p[jj] == -INFINITY) ? 0.f : expf(p[jj] - mx);
    p[jj] = e;
    sum += e;
  }
  sum = wave_sum(sum);
#pragma unroll
  for (int jj = 0; jj < kMaxKeysPerLane; ++jj) p[jj] = p[jj] / sum;
}

// value of the (possibly quantized) probability as it enters P*V, in units of sp
template <class T>
__device__ __forceinline__ float prob_operand(float p, const AttnScales& sc) {
  if (sc.p_on) return rintf(fminf(fmaxf(__fdiv_rn(p, sc.sp), 0.f), sc.p_qp));
  return round_to<T>(p);
}

template <class T>
__global__ void attn_fwd_k(const T* __restrict__ codes, T* __restrict__ ctx, T* __restrict__ ctx_codes, AttnQ aq,
                           const int32_t* __restrict__ seqlens, int S, int H, int d, float* __restrict__ pmax_rows) {
  __shared__ float qrow[4][kMaxHeadDim];
  __shared__ float prow[4][kMaxKeysPerLane * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x * 4 + wave, h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  const bool active = i < S;
  const int len = seqlens ? seqlens[b] : S;
  const int ld = 3 * H;
  const T* base = codes + (size_t)b * S * ld;
  const AttnScales sc = load_scales(aq, d);
  if (active)
    for (int e = lane; e < d; e += 64) qrow[wave][e] = ldf(base, (size_t)i * ld + h * d + e);
  __syncthreads();
  float p[kMaxKeysPerLane];
  if (active) {
    prob_row<T>(base + H + h * d, ld, qrow[wave], S, len, d, sc.qk, p);
    float pm = 0.f;
#pragma unroll
    for (int jj = 0; jj < kMaxKeysPerLane; ++jj) {
      const int j = lane + 64 * jj;
      pm = fmaxf(pm, p[jj]);
      if (j < S) prow[wave][j] = prob_operand<T>(p[jj], sc);
    }
    if (pmax_rows) {
      pm = wave_max(pm);
      if (lane == 0) pmax_rows[((size_t)b * nh + h) * S + i] = pm;
    }
  }
  __syncthreads();
  if (active) {
    const QuantParam qc = {aq.c.on ? *aq.c.s : 1.f, 0.f, aq.c.qn, aq.c.qp, aq.c.on};
    for (int e = lane; e < d; e += 64) {
      const T* vcol = base + 2 * H + h * d + e;
      float acc = 0.f;
      for (int j = 0; j < len; ++j) acc += prow[wave][j] * ldf(vcol, (size_t)j * ld);
      const float out = acc * sc.sp * sc.sv;
      const size_t o = ((size_t)b * S + i) * H + h * d + e;
      stf(ctx, o, out);
      if (ctx_codes) {
        const float r = round_to<T>(out);
        stf(ctx_codes, o, qc.on ? q_code(q_ratio(r, qc), qc) : r);
      }
    }
  }
}

void attn_fwd(int dt, const void* codes, void* ctx, void* ctx_codes, const AttnQ& aq, const int32_t* seqlens, int B, int S,
              int nh, int d, float* pmax_rows, hipStream_t st) {
  dim3 g((S + 3) / 4, nh, B);
  const int H = nh * d;
  if (dt == DT_BF16)
    hipLaunchKernelGGL(attn_fwd_k<bf16_t>, g, dim3(256), 0, st, (const bf16_t*)codes, (bf16_t*)ctx, (bf16_t*)ctx_codes, aq, seqlens, S,
                       H, d, pmax_rows);
  else
    hipLaunchKernelGGL(attn_fwd_k<float>, g, dim3(256), 0, st, (const float*)codes, (float*)ctx, (float*)ctx_codes, aq, seqlens, S, H, d,
                       pmax_rows);
}

// Row part of backward: recomputes the probabilities, pushes d(context) through
// P*V, the probability quantizer and the softmax, writes dA and P^ rows to
// scratch and the gradient of the quantized queries.
template <class T>
__global__ void attn_bwd_rows_k(const T* __restrict__ codes, const T* __restrict__ dctx, T* __restrict__ d_qkvh, AttnQ aq,
                                const int32_t* __restrict__ seqlens, int S, int H, int d, float* __restrict__ scratch_da,
                                float* __restrict__ scratch_ph, float* __restrict__ ds_rows) {
  __shared__ float qrow[4][kMaxHeadDim];
  __shared__ float crow[4][kMaxHeadDim];
  __shared__ float arow[4][kMaxKeysPerLane * 64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int i = blockIdx.x * 4 + wave, h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  const bool active = i < S;
  const int len = seqlens ? seqlens[b] : S;
  const int ld = 3 * H;
  const T* base = codes + (size_t)b * S * ld;
  const AttnScales sc = load_scales(aq, d);
  if (active)
    for (int e = lane; e < d; e += 64) {
      qrow[wave][e] = ldf(base, (size_t)i * ld + h * d + e);
      crow[wave][e] = ldf(dctx, ((size_t)b * S + i) * H + h * d + e);
    }
  __syncthreads();
  float p[kMaxKeysPerLane], dp[kMaxKeysPerLane];
  const size_t srow = (((size_t)b * nh + h) * S + i) * S;
  if (active) {
    prob_row<T>(base + H + h * d, ld, qrow[wave], S, len, d, sc.qk, p);
    float dsp = 0.f, rowdot = 0.f;
#pragma unroll
    for (int jj = 0; jj < kMaxKeysPerLane; ++jj) {
      const int j = lane + 64 * jj;
      dp[jj] = 0.f;
      if (j < S) {
        float dot = 0.f;
        const T* vrow = base + (size_t)j * ld + 2 * H + h * d;
        for (int e = 0; e < d; e += 8) {
          float vv[8];
          ld8(vrow + e, vv);
#pragma unroll
          for (int t = 0; t < 8; ++t) dot += crow[wave][e + t] * vv[t];
        }
        const float dph = dot * sc.sv;  // gradient w.r.t. the quantized probability
        float ph;
        if (sc.p_on) {
          const float v = __fdiv_rn(p[jj], sc.sp);
          const bool in = (v >= 0.f) && (v <= sc.p_qp);
          const float c = rintf(fminf(fmaxf(v, 0.f), sc.p_qp));
          dsp += dph * (c - (in ? v : 0.f));
          dp[jj] = in ? dph : 0.f;
          ph = c * sc.sp;
        } else {
          dp[jj] = dph;
          ph = round_to<T>(p[jj]);
        }
        scratch_ph[srow + j] = ph;
        rowdot += dp[jj] * p[jj];
      }
    }
    rowdot = wave_sum(rowdot);
    dsp = wave_sum(dsp);
    if (lane == 0) ds_rows[((size_t)b * nh + h) * S + i] = dsp;
#pragma unroll
    for (int jj = 0; jj < kMaxKeysPerLane; ++jj) {
      const int j = lane + 64 * jj;
      if (j < S) {
        const float da = p[jj] * (dp[jj] - rowdot);
        arow[wave][j] = da;
        scratch_da[srow + j] = da;
      }
    }
  }
  __syncthreads();
  if (active) {
    const float f = sc.sk / sqrtf((float)d);
    for (int e = lane; e < d; e += 64) {
      const T* kcol = base + H + h * d + e;
      float acc = 0.f;
      for (int j = 0; j < len; ++j) acc += arow[wave][j] * ldf(kcol, (size_t)j * ld);
      stf(d_qkvh, ((size_t)b * S + i) * ld + h * d + e, acc * f);
    }
  }
}

// Column part: gradients of the quantized keys and values of key row j.
template <class T>
__global__ void attn_bwd_cols_k(const T* __restrict__ codes, const T* __restrict__ dctx, T* __restrict__ d_qkvh, AttnQ aq, int S,
                                int H, int d, const float* __restrict__ scratch_da, const float* __restrict__ scratch_ph) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int j = blockIdx.x * 4 + wave, h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  if (j >= S) return;
  const int ld = 3 * H;
  const T* base = codes + (size_t)b * S * ld;
  const AttnScales sc = load_scales(aq, d);
  const size_t sbase = ((size_t)b * nh + h) * S * S;
  const float f = sc.sq / sqrtf((float)d);
  for (int e = lane; e < d; e += 64) {
    float dv = 0.f, dk = 0.f;
    for (int i = 0; i < S; ++i) {
      const float ph = scratch_ph[sbase + (size_t)i * S + j];
      const float da = scratch_da[sbase + (size_t)i * S + j];
      dv += ph * ldf(dctx, ((size_t)b * S + i) * H + h * d + e);
      dk += da * ldf(base, (size_t)i * ld + h * d + e);
    }
    stf(d_qkvh, ((size_t)b * S + j) * ld + H + h * d + e, dk * f);
    stf(d_qkvh, ((size_t)b * S + j) * ld + 2 * H + h * d + e, dv);
  }
}

void attn_bwd(int dt, const void* codes, const void* dctx, void* d_qkvh, const AttnQ& aq, const int32_t* seqlens, int B, int S,
              int nh, int d, float* scratch_da, float* scratch_ph, float* ds_rows, hipStream_t st) {
  dim3 g((S + 3) / 4, nh, B);
  const int H = nh * d;
  if (dt == DT_BF16) {
    hipLaunchKernelGGL(attn_bwd_rows_k<bf16_t>, g, dim3(256), 0, st, (const bf16_t*)codes, (const bf16_t*)dctx, (bf16_t*)d_qkvh, aq,
                       seqlens, S, H, d, scratch_da, scratch_ph, ds_rows);
    hipLaunchKernelGGL(attn_bwd_cols_k<bf16_t>, g, dim3(256), 0, st, (const bf16_t*)codes, (const bf16_t*)dctx, (bf16_t*)d_qkvh, aq, S,
                       H, d, scratch_da, scratch_ph);
  } else {
    hipLaunchKernelGGL(attn_bwd_rows_k<float>, g, dim3(256), 0, st, (const float*)codes, (const float*)dctx, (float*)d_qkvh, aq, seqlens,
                       S, H, d, scratch_da, scratch_ph, ds_rows);
    hipLaunchKernelGGL(attn_bwd_cols_k<float>, g, dim3(256), 0, st, (const float*)codes, (const float*)dctx, (float*)d_qkvh, aq, S, H, d,
                       scratch_da, scratch_ph);
  }
}

}  // namespace mrem
