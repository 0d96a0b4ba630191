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


// ------------------------------------------------------------------------------
// bf16 MFMA kernel (v_mfma_f32_32x32x16_bf16, fp32 accumulate)
//
// Block tile BM x BN x 64, 256 threads = 4 wavefronts in a 2 x 2 grid, each owning a
// (BM/2) x (BN/2) sub-tile made of 32 x 32 MFMA tiles.  Operand tiles are staged
// global -> registers -> LDS (two LDS stages, one barrier per k-step); LDS rows are
// padded to 144 bytes so that the 16-byte fragment reads of 16 consecutive rows hit
// distinct banks.  Integer codes (|q| <= 255) are exact in bf16 and their products
// and partial sums are exact in fp32 up to 2^24, so the quantized forward products
// are exact integers before the epilogue applies the step sizes.
// Requires M % BM == 0, N % BN == 0, K % 64 == 0 and 16-byte aligned rows.
// ------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));

constexpr int kBK = 64;
constexpr int kLdsStride = kBK + 8;  // elements per LDS row (144 bytes)

template <int BM, int BN, class TO>
__global__ __launch_bounds__(256) void gemm_nt_mfma_k(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B, int ldb,
                                                      TO* __restrict__ C, int ldc, int M, int N, int K, Epilogue e, int tiles_m,
                                                      int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int WM = BM / 2, WN = BN / 2;   // wavefront sub-tile
  constexpr int MT = WM / 32, NT = WN / 32; // MFMA tiles per wavefront
  constexpr int A_ELEMS = BM * kLdsStride, B_ELEMS = BN * kLdsStride;
  constexpr int STAGE = A_ELEMS + B_ELEMS;
  constexpr int A_CH = BM * 8 / 256, B_CH = BN * 8 / 256;  // 16-byte chunks per thread per k-step

  // Tile order: consecutive block ids land on different XCDs (8 of them, each with its
  // own L2), so give each XCD a contiguous range of tiles, walked in groups of 8 tile
  // rows so that concurrently running blocks share operand panels in that L2.
  const int nblocks = tiles_m * tiles_n;
  int pid = blockIdx.x;
  if ((nblocks & 7) == 0) pid = (pid & 7) * (nblocks >> 3) + (pid >> 3);
  constexpr int GROUP = 8;
  const int group_sz = GROUP * tiles_n;
  const int g = pid / group_sz;
  const int first_m = g * GROUP;
  const int gm = (tiles_m - first_m) < GROUP ? (tiles_m - first_m) : GROUP;
  const int tm = first_m + (pid % group_sz) % gm;
  const int tn = (pid % group_sz) / gm;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16_t acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  u32x4_t ra[A_CH], rb[B_CH];
  const bf16_t* Ag = A + (size_t)m0 * lda;
  const bf16_t* Bg = B + (size_t)n0 * ldb;
  const int ld_row = tid >> 3, ld_ch = tid & 7;  // this thread's chunk in rows ld_row + 32*i
  const bf16_t* Agt = Ag + (size_t)ld_row * lda + ld_ch * 8;
  const bf16_t* Bgt = Bg + (size_t)ld_row * ldb + ld_ch * 8;
  const int lds_off = ld_row * kLdsStride + ld_ch * 8;

#define MREM_LOAD_GLOBAL(k0)                                                                           \
  {                                                                                                    \
    _Pragma("unroll") for (int i = 0; i < A_CH; ++i)                                                   \
        ra[i] = *reinterpret_cast<const u32x4_t*>(Agt + (size_t)(32 * i) * lda + (k0));                  \
    _Pragma("unroll") for (int i = 0; i < B_CH; ++i)                                                   \
        rb[i] = *reinterpret_cast<const u32x4_t*>(Bgt + (size_t)(32 * i) * ldb + (k0));                  \
  }
#define MREM_STORE_LDS(stage)                                                                          \
  {                                                                                                    \
    bf16_t* As_ = smem + (stage) * STAGE + lds_off;                                                    \
    bf16_t* Bs_ = As_ + A_ELEMS;                                                                       \
    _Pragma("unroll") for (int i = 0; i < A_CH; ++i)                                                   \
        *reinterpret_cast<u32x4_t*>(As_ + 32 * i * kLdsStride) = ra[i];                                  \
    _Pragma("unroll") for (int i = 0; i < B_CH; ++i)                                                   \
        *reinterpret_cast<u32x4_t*>(Bs_ + 32 * i * kLdsStride) = rb[i];                                  \
  }

  const int KT = K / kBK;
  MREM_LOAD_GLOBAL(0)
  MREM_STORE_LDS(0)
  __syncthreads();
  const int frag_row = lane & 31, frag_ch = lane >> 5;
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) MREM_LOAD_GLOBAL((kt + 1) * kBK)
    const bf16_t* As = smem + cur * STAGE + (wm * WM + frag_row) * kLdsStride + frag_ch * 8;
    const bf16_t* Bs = smem + cur * STAGE + A_ELEMS + (wn * WN + frag_row) * kLdsStride + frag_ch * 8;
#pragma unroll
    for (int kk = 0; kk < kBK / 16; ++kk) {
      bf16x8_t af[MT], bfr[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) af[i] = *reinterpret_cast<const bf16x8_t*>(As + i * 32 * kLdsStride + kk * 16);
#pragma unroll
      for (int j = 0; j < NT; ++j) bfr[j] = *reinterpret_cast<const bf16x8_t*>(Bs + j * 32 * kLdsStride + kk * 16);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) MREM_STORE_LDS(cur ^ 1)
    __syncthreads();
  }
#undef MREM_LOAD_GLOBAL
#undef MREM_STORE_LDS

  // epilogue: out = acc * (alpha * col_scale[n]) + beta * (col_vec[n] + row_vec[m]) + bias[n]
  const float alpha = e.alpha ? *e.alpha : 1.f;
  const float beta = e.beta ? *e.beta : 0.f;
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int n = n0 + wn * WN + j * 32 + (lane & 31);
    const float cs = alpha * (e.col_scale ? e.col_scale[n] : 1.f);
    float cb = e.bias ? e.bias[n] : 0.f;
    if (e.beta && e.col_vec) cb += beta * e.col_vec[n];
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int mb = m0 + wm * WM + i * 32 + 4 * (lane >> 5);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = mb + 8 * (r >> 2) + (r & 3);
        float v = acc[i][j][r] * cs + cb;
        if (e.beta && e.row_vec) v += beta * e.row_vec[m];
        if (e.gelu) v = gelu_f(round_to<TO>(v));
        stf(C, (size_t)m * ldc + n, v);
      }
    }
  }
}

template <int BM, int BN, class TO>
static void launch_mfma(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                        hipStream_t st) {
  constexpr size_t lds = 2 * (size_t)(BM + BN) * kLdsStride * sizeof(bf16_t);
  static bool configured = false;
  if (!configured) {
    hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_mfma_k<BM, BN, TO>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured = true;
  }
  const int tiles_m = M / BM, tiles_n = N / BN;
  hipLaunchKernelGGL((gemm_nt_mfma_k<BM, BN, TO>), dim3(tiles_m * tiles_n), dim3(256), lds, st, (const bf16_t*)A, lda, (const bf16_t*)B, ldb,
                     (TO*)C, ldc, M, N, K, e, tiles_m, tiles_n);
}

static bool mfma_ok(const void* A, int lda, const void* B, int ldb, int M, int N, int K) {
  return M % 128 == 0 && N % 128 == 0 && K % kBK == 0 && lda % 8 == 0 && ldb % 8 == 0 &&
         (reinterpret_cast<uintptr_t>(A) & 15) == 0 && (reinterpret_cast<uintptr_t>(B) & 15) == 0;
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
  if (dt == DT_BF16 && mfma_ok(A, lda, B, ldb, M, N, K)) {
    if (e.out_f32) launch_mfma<128, 128, float>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    else launch_mfma<128, 128, bf16_t>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    return;
  }
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
