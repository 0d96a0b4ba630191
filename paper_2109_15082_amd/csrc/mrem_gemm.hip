// C[M,N] = A[M,K] * B[N,K]^T with a fused epilogue: the products of the four linear
// layers of an encoder layer in the quantized module (integer codes as operands,
// step sizes applied to the accumulator -- Section 3.1, Eq. 1), of the
// full-precision module, and of the backward pass (input and weight gradients).
#include "mrem_common.h"
#include "mrem_kernels.h"

#include <hip/hip_ext.h>

#include <atomic>
#include <string>
#include <cstdlib>
#include <type_traits>

#include <vector>

namespace mrem {

// ---- optional timing of every product launch with HIP events (measurement aid) ----
// The records live in a GemmProfile that the caller (a context) owns.  Return codes of event calls are
// not looked at here: the runtime keeps the last error, and every entry point of the library ends by
// reading it (hipGetLastError).
thread_local LaunchEvents tl_launch_events;

void gemm_profile_begin(GemmProfile* p) {
  for (auto& r : p->recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
  p->recs.clear();
  p->stats.clear();
  p->on = true;
}
int gemm_profile_end(GemmProfile* p, double ms[2], double flops[2], int64_t launches[2]) {
  p->on = false;
  ms[0] = ms[1] = flops[0] = flops[1] = 0.0;
  launches[0] = launches[1] = 0;
  int rc = 0;
  for (auto& r : p->recs) {
    float e = 0.f;
    if (hipEventSynchronize(r.e1) != hipSuccess || hipEventElapsedTime(&e, r.e0, r.e1) != hipSuccess) rc = -1;
    if (r.cls < 2) {
      ms[r.cls] += e;
      flops[r.cls] += r.flops;
      launches[r.cls] += 1;
    } else {
      KernelStat* ks = nullptr;
      for (auto& k : p->stats)
        if (k.label == r.label || std::string(k.label) == r.label) ks = &k;
      if (!ks) { p->stats.push_back(KernelStat{r.label, 0.0, 0.0, 0}); ks = &p->stats.back(); }
      ks->ms += e;
      ks->bytes += r.flops;
      ks->launches += 1;
    }
    (void)hipEventDestroy(r.e0);
    (void)hipEventDestroy(r.e1);
  }
  p->recs.clear();
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
  if (e.gelu) v = gelu_t<TO>(round_to<TO>(v));
  stf(C, (size_t)m * ldc + n, v);
}

// ------------------------------------------------------------------------------
// generic scalar-ALU kernel: any M, N, K; fp32 or bf16 operands; used by the fp32
// check mode and for shapes the MFMA kernel does not take
// ------------------------------------------------------------------------------
template <class TA, class TO>
__global__ void gemm_nt_simt_k(const TA* __restrict__ A, int lda, const TA* __restrict__ B, int ldb, TO* __restrict__ C, int ldc, int M,
                               int N, int K, Epilogue e, int a_t = 0, int b_t = 0) {
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
      As[kk][r] = (m0 + r < M && k < K) ? ldf(A, a_t ? (size_t)k * lda + m0 + r : (size_t)(m0 + r) * lda + k) : 0.f;
      Bs[kk][r] = (n0 + r < N && k < K) ? ldf(B, b_t ? (size_t)k * ldb + n0 + r : (size_t)(n0 + r) * ldb + k) : 0.f;
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
  ev.beta = (e.beta ? *e.beta : 0.f) + e.beta_alpha * ev.alpha;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) epilogue_store(C, ldc, m, n, acc[i][j], e, ev);
    }
}


// ------------------------------------------------------------------------------
// MFMA products (v_mfma_f32_32x32x16_bf16 with fp32 accumulation, v_mfma_i32_32x32x32_i8 with exact
// int32 accumulation): kernel gemm_dl_k in mrem_gemm_dl.h.  Integer codes (|q| <= 255) are exact in
// bf16 and their products and partial sums are exact in fp32 while they stay below 2^24 (always for
// 4-bit weights: K * 255 * 7 < 2^24 up to K = 9398; with 8-bit weights only up to K = 518, beyond
// that a product on bf16 codes rounds like any fp32 sum); the int8 mode is exact for every supported K.
// Requires M and N multiples of 128, K a multiple of 64 (128 int8 codes) and 16-byte aligned rows.
// ------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x16_t __attribute__((ext_vector_type(16)));
typedef short s16x4_t __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;  // k-granularity of the MFMA kernels, in 2-byte elements

}  // namespace mrem
#include "mrem_gemm_dl.h"
namespace mrem {

static bool mfma_ok(const void* A, int lda, const void* B, int ldb, int M, int N, int K) {
  return M % 128 == 0 && N % 128 == 0 && K % kBK == 0 && lda % 8 == 0 && ldb % 8 == 0 &&
         (reinterpret_cast<uintptr_t>(A) & 15) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0;
}

static void gemm_launch(int dt, int a_t, int b_t, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                        const Epilogue& e, hipStream_t st);

void gemm(int dt, int a_t, int b_t, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
          const Epilogue& e, hipStream_t st, GemmProfile* prof) {
  if (!prof || !prof->on) {
    gemm_launch(dt, a_t, b_t, A, lda, B, ldb, C, ldc, M, N, K, e, st);
    return;
  }
  GemmRecord r;
  r.flops = 2.0 * (double)M * (double)N * (double)K;
  (void)hipEventCreate(&r.e0);
  (void)hipEventCreate(&r.e1);
  tl_launch_events.e0 = r.e0;
  tl_launch_events.e1 = r.e1;
  gemm_launch(dt, a_t, b_t, A, lda, B, ldb, C, ldc, M, N, K, e, st);
  tl_launch_events = LaunchEvents();
  prof->recs.push_back(r);
}

bool gemm_i8_ok(const void* A, int lda, const void* B, int ldb, int M, int N, int K) {
  return M % 128 == 0 && N % 128 == 0 && K % 128 == 0 && lda % 16 == 0 && ldb % 16 == 0 &&
         (reinterpret_cast<uintptr_t>(A) & 15) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0;
}
// int8 mode: two int8 codes travel as one 16-bit element, so leading dimensions and the contraction
// length are halved.
// Which tile serves a product (measured on the module step, two streams sharing the device):
//   256 x 256 (8 wavefronts of 64 x 128, two stages of 128-byte rows, one block per compute unit) when the
//     output has at least 192 such tiles -- the query/key/value and first feed-forward projections and
//     the input gradient of the second one at 4096 tokens: half the operand bytes per flop of the small tile;
//   128 x 128 with 8 wavefronts (two groups of 4; each group multiplies every other 16-deep k-substep of a
//     stage and the groups' partial sums meet in LDS before the epilogue), four stages of 128-byte rows, one
//     block per compute unit, when the output has at most 256 such tiles -- one tile per compute unit, so the
//     second wavefront on each SIMD is what overlaps fragment reads, barriers and MFMA issue;
//   128 x 128 with 4 wavefronts of 64 x 64, four stages of 64-byte rows, two blocks per compute unit, otherwise:
//     the second block fills the barrier and epilogue gaps of the first.
//   Four stages hide the latency of operands that the previous kernel has just written or that come from HBM.
template <bool AT, bool BT, class TO, bool I8>
static void launch_dl_tiles(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                            hipStream_t st, int splits) {
  if (splits == 1 && M % 256 == 0 && N % 256 == 0 && (M / 256) * (N / 256) >= 192)
    return launch_dl<256, 256, 4, 2, AT, BT, 2, 128, TO, I8, 1>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
  if ((M / 128) * (N / 128) <= 256)
    return launch_dl<128, 128, 2, 2, AT, BT, 4, 128, TO, I8, 1, 2>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  return launch_dl<128, 128, 2, 2, AT, BT, 4, 64, TO, I8, 2>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
}
static void gemm_i8_launch(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                           hipStream_t st) {
  launch_dl_tiles<false, false, bf16_t, true>(A, lda / 2, B, ldb / 2, C, ldc, M, N, K / 2, e, st, 1);
}
void gemm_i8(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e, hipStream_t st,
             GemmProfile* prof) {
  if (!prof || !prof->on) {
    gemm_i8_launch(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    return;
  }
  GemmRecord r;
  r.flops = 2.0 * (double)M * (double)N * (double)K;
  (void)hipEventCreate(&r.e0);
  (void)hipEventCreate(&r.e1);
  tl_launch_events.e0 = r.e0;
  tl_launch_events.e1 = r.e1;
  gemm_i8_launch(A, lda, B, ldb, C, ldc, M, N, K, e, st);
  tl_launch_events = LaunchEvents();
  r.cls = 1;
  prof->recs.push_back(r);
}

void gemm_nt(int dt, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
             hipStream_t st, GemmProfile* prof) {
  gemm(dt, 0, 0, A, lda, B, ldb, C, ldc, M, N, K, e, st, prof);
}

// Tiles for at most half of the compute units and a long contraction (weight gradients of the
// square projections): two k-slices.  (Larger weight gradients run beside the rest of the backward
// pass, where a second slice only adds atomic traffic.)  Two atomic adds onto a zeroed fp32 value
// commute exactly, so the result does not depend on which slice arrives first.
static int f32_k_slices(int M, int N, int K) {
  const int tiles = (M / 128) * (N / 128);
  return (tiles <= 128 && K >= 2048 && (K / kBK) % 2 == 0) ? 2 : 1;
}
int gemm_f32_k_slices(int dt, int M, int N, int K) {
  return (dt == DT_BF16 && M % 128 == 0 && N % 128 == 0 && K % kBK == 0) ? f32_k_slices(M, N, K) : 1;
}

template <bool AT, bool BT>
static void launch_mfma_modes(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                              hipStream_t st) {
  if (e.out_f32) {
    const int splits = e.gelu ? 1 : f32_k_slices(M, N, K);
    if (splits > 1 && !e.c_zeroed) fill_f32((float*)C, 0.f, (int64_t)M * ldc, st);
    launch_dl_tiles<AT, BT, float, false>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  } else {
    launch_dl_tiles<AT, BT, bf16_t, false>(A, lda, B, ldb, C, ldc, M, N, K, e, st, 1);
  }
}

static void gemm_launch(int dt, int a_t, int b_t, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
                        const Epilogue& e, hipStream_t st) {
  if (dt == DT_BF16 && mfma_ok(A, lda, B, ldb, M, N, K)) {
    if (!a_t && !b_t) {
      launch_mfma_modes<false, false>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    } else if (!a_t && b_t) {
      launch_mfma_modes<false, true>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    } else if (a_t && b_t) {
      launch_mfma_modes<true, true>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    } else {
      launch_mfma_modes<true, false>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    }
    return;
  }
  dim3 g((N + 63) / 64, (M + 63) / 64);
  const hipEvent_t t0 = tl_launch_events.e0, t1 = tl_launch_events.e1;  // the fallback kernels are timed by recorded events
  if (t0) (void)hipEventRecord(t0, st);
  if (dt == DT_BF16) {
    if (e.out_f32)
      hipLaunchKernelGGL((gemm_nt_simt_k<bf16_t, float>), g, dim3(256), 0, st, (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (float*)C, ldc,
                         M, N, K, e, a_t, b_t);
    else
      hipLaunchKernelGGL((gemm_nt_simt_k<bf16_t, bf16_t>), g, dim3(256), 0, st, (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (bf16_t*)C,
                         ldc, M, N, K, e, a_t, b_t);
  } else {
    hipLaunchKernelGGL((gemm_nt_simt_k<float, float>), g, dim3(256), 0, st, (const float*)A, lda, (const float*)B, ldb, (float*)C, ldc, M,
                       N, K, e, a_t, b_t);
  }
  if (t1) (void)hipEventRecord(t1, st);
}

}  // namespace mrem
