// C[M,N] = A[M,K] * B[N,K]^T with a fused epilogue: the products of the four linear
// layers of an encoder layer in the quantized module (integer codes as operands,
// step sizes applied to the accumulator -- Section 3.1, Eq. 1), of the
// full-precision module, and of the backward pass (input and weight gradients).
#include "mrem_common.h"
#include "mrem_kernels.h"

#include <vector>

namespace mrem {

// ---- optional timing of every product launch with HIP events (measurement aid) ----
namespace {
struct GemmRecord {
  hipEvent_t e0, e1;
  double flops;
};
bool g_prof_on = false;
std::vector<GemmRecord> g_prof;
}  // namespace

void gemm_profile_begin() {
  for (auto& r : g_prof) { hipEventDestroy(r.e0); hipEventDestroy(r.e1); }
  g_prof.clear();
  g_prof_on = true;
}
int gemm_profile_end(double* ms, double* flops, int64_t* launches) {
  g_prof_on = false;
  double t = 0.0, f = 0.0;
  int rc = 0;
  for (auto& r : g_prof) {
    float e = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&e, r.e0, r.e1) != hipSuccess) rc = -1;
    t += e;
    f += r.flops;
    hipEventDestroy(r.e0);
    hipEventDestroy(r.e1);
  }
  *ms = t;
  *flops = f;
  *launches = (int64_t)g_prof.size();
  g_prof.clear();
  return rc;
}

struct EpiVals {
  float alpha, beta;
};

template <class TO>
__device__ __forceinline__ void epilogue_store(TO* C, int ldc, int m, int n, float acc, const Epilogue& e, const EpiVals& ev) {
  float v = acc * (ev.alpha * (e.col_scale ? e.col_scale[n] : 1.f));
  if (e.beta) v += ev.beta * ((e.col_vec ? e.col_vec[n] : 0.f) + (e.row_vec ? e.row_vec[m] : 0.f));
  if (e.bias) v += e.bias[n];
  if (e.gelu) v = gelu_f(round_to<TO>(v));
  stf(C, (size_t)m * ldc + n, v);
}

// ------------------------------------------------------------------------------
// generic scalar-ALU kernel: any M, N, K; fp32 or bf16 operands; used by the fp32
// check mode and for shapes the MFMA kernel does not take
// ------------------------------------------------------------------------------
template <class TA, class TO>
__global__ void gemm_nt_simt_k(const TA* __restrict__ A, int lda, const TA* __restrict__ B, int ldb, TO* __restrict__ C, int ldc, int M,
                               int N, int K, Epilogue e) {
  __shared__ float As[16][64 + 4];
  __shared__ float Bs[16][64 + 4];
  const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.f;
  for (int k0 = 0; k0 < K; k0 += 16) {
    // 64 rows x 16 k per operand = 1024 elements, 4 per thread
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const int idx = threadIdx.x + 256 * t;
      const int r = idx >> 4, kk = idx & 15;
      const int k = k0 + kk;
      As[kk][r] = (m0 + r < M && k < K) ? ldf(A, (size_t)(m0 + r) * lda + k) : 0.f;
      Bs[kk][r] = (n0 + r < N && k < K) ? ldf(B, (size_t)(n0 + r) * ldb + k) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < 16; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] += a[i] * b[j];
    }
    __syncthreads();
  }
  EpiVals ev;
  ev.alpha = e.alpha ? *e.alpha : 1.f;
  ev.beta = e.beta ? *e.beta : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) epilogue_store(C, ldc, m, n, acc[i][j], e, ev);
    }
}

static void gemm_nt_launch(int dt, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                           const Epilogue& e, hipStream_t st);

void gemm_nt(int dt, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
             hipStream_t st) {
  if (!g_prof_on) {
    gemm_nt_launch(dt, A, lda, B, ldb, C, ldc, M, N, K, e, st);
    return;
  }
  GemmRecord r;
  r.flops = 2.0 * (double)M * (double)N * (double)K;
  hipEventCreate(&r.e0);
  hipEventCreate(&r.e1);
  hipEventRecord(r.e0, st);
  gemm_nt_launch(dt, A, lda, B, ldb, C, ldc, M, N, K, e, st);
  hipEventRecord(r.e1, st);
  g_prof.push_back(r);
}

static void gemm_nt_launch(int dt, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                           const Epilogue& e, hipStream_t st) {
  dim3 g((N + 63) / 64, (M + 63) / 64);
  if (dt == DT_BF16) {
    if (e.out_f32)
      hipLaunchKernelGGL((gemm_nt_simt_k<bf16_t, float>), g, dim3(256), 0, st, (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (float*)C, ldc,
                         M, N, K, e);
    else
      hipLaunchKernelGGL((gemm_nt_simt_k<bf16_t, bf16_t>), g, dim3(256), 0, st, (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (bf16_t*)C,
                         ldc, M, N, K, e);
  } else {
    hipLaunchKernelGGL((gemm_nt_simt_k<float, float>), g, dim3(256), 0, st, (const float*)A, lda, (const float*)B, ldb, (float*)C, ldc, M,
                       N, K, e);
  }
}

}  // namespace mrem
