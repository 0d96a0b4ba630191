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
// bf16 MFMA kernel (v_mfma_f32_32x32x16_bf16, fp32 accumulate)
//
// Block tile BM x BN x 64, 256 threads = 4 wavefronts in a 2 x 2 grid, each owning a
// (BM/2) x (BN/2) sub-tile made of 32 x 32 MFMA tiles.  Operand tiles are staged
// global -> registers -> LDS (two LDS stages, one barrier per k-step); LDS rows are
// padded to 144 bytes so that the 16-byte fragment reads of 16 consecutive rows hit
// distinct banks.  Integer codes (|q| <= 255) are exact in bf16 and their products
// and partial sums are exact in fp32 while they stay below 2^24 (always for 4-bit weights:
// K * 255 * 7 < 2^24 up to K = 9398; with 8-bit weights only while K * 255 * 127 < 2^24,
// K <= 518, beyond that the bf16 fallback rounds like any fp32 sum; the int8 mode below
// accumulates in int32 and is exact for every supported K).
// Requires M % BM == 0, N % BN == 0, K % 64 == 0 and 16-byte aligned rows.
// ------------------------------------------------------------------------------
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x4_t __attribute__((ext_vector_type(4)));
typedef int i32x16_t __attribute__((ext_vector_type(16)));

constexpr int kBK = 64;
constexpr int kRegBK = 64;  // k-step of the register-staged kernel

typedef short s16x4_t __attribute__((ext_vector_type(4)));

// One operand of the product as the register-staged kernel sees it.
//   TR = false: the matrix is stored [rows][k] (k contiguous); LDS tile [ROWS][64 + 8].
//   TR = true : the matrix is stored [k][rows] (the contraction index is the slow one, as for
//               both operands of a weight-gradient product and for the weight in an
//               input-gradient product); LDS tile [64][ROWS + 16], and MFMA fragments are
//               gathered with the transposing LDS read (ds_read_b64_tr_b16): in a group of 16
//               lanes, lane s supplies the 8-byte chunk of row s/4, columns 4*(s%4)..+3, and
//               receives column s of the four rows.
template <bool TR, int ROWS, int NTHREADS, int BK>
struct OperandTile {
  static constexpr int PITCH = TR ? ROWS + 16 : BK + 8;
  static constexpr int ELEMS = TR ? BK * PITCH : ROWS * PITCH;
  static constexpr int CPR = BK / 8;                   // 16-byte chunks per row of a k-contiguous tile
  static constexpr int NCH = ROWS * CPR / NTHREADS;    // 16-byte chunks per thread per k-step
  // chunk q of the tile: (tile row, first element) in the matrix, and offset in LDS
  static __device__ __forceinline__ size_t gofs(int q, int ld, int tile0, int k0) {
    if (TR) { const int row = q / (ROWS / 8), ch = q % (ROWS / 8); return (size_t)(k0 + row) * ld + tile0 + ch * 8; }
    const int row = q / CPR, ch = q % CPR;
    return (size_t)(tile0 + row) * ld + k0 + ch * 8;
  }
  static __device__ __forceinline__ int lofs(int q) {
    if (TR) { const int row = q / (ROWS / 8), ch = q % (ROWS / 8); return row * PITCH + ch * 8; }
    return (q / CPR) * PITCH + (q % CPR) * 8;
  }
  // fragment of 32 tile rows starting at row0 for k-substep kk (16 of the 64 k values)
  static __device__ __forceinline__ bf16x8_t frag(const bf16_t* tile, int row0, int kk, int lane) {
    if (TR) {
      const int g = lane >> 4, s = lane & 15;
      const bf16_t* p = tile + (16 * kk + 8 * (g >> 1) + (s >> 2)) * PITCH + row0 + 16 * (g & 1) + 4 * (s & 3);
      union { bf16x8_t v; s16x4_t h[2]; } u;
      u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p));
      u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p + 4 * PITCH));
      return u.v;
    }
    return *reinterpret_cast<const bf16x8_t*>(tile + (row0 + (lane & 31)) * PITCH + kk * 16 + (lane >> 5) * 8);
  }
};

// I8: the operands are int8 codes seen as pairs (the caller passes K, lda and ldb in units of two
// bytes): data movement and fragment addresses are those of the bf16 case, the product runs on
// the 32x32x32 int8 instruction with exact int32 accumulation.  Not for transposed operands.
// Two blocks per compute unit are part of the design (LDS: 2 x 74 KB); the launch bound makes the
// compiler keep the register budget that goes with it (256 per lane, accumulators included).
template <int BM, int BN, int WAVES_M, int WAVES_N, bool AT, bool BT, int BK, class TO, bool I8 = false>
__global__ __launch_bounds__(64 * WAVES_M * WAVES_N, 2) void gemm_mfma_k(const bf16_t* __restrict__ A, int lda, const bf16_t* __restrict__ B,
                                                                      int ldb, TO* __restrict__ C, int ldc, int M, int N, int K, Epilogue e,
                                                                      int tiles_m, int tiles_n) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);
  constexpr int NTHREADS = 64 * WAVES_M * WAVES_N;
  constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // wavefront sub-tile
  constexpr int MT = WM / 32, NT = WN / 32;            // MFMA tiles per wavefront
  typedef OperandTile<AT, BM, NTHREADS, BK> OpA;
  typedef OperandTile<BT, BN, NTHREADS, BK> OpB;
  constexpr int STAGE = OpA::ELEMS + OpB::ELEMS;

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
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;

  static_assert(!I8 || (!AT && !BT), "int8 operands are read along k only");
  typedef typename std::conditional<I8, i32x16_t, f32x16_t>::type acc_t;
  acc_t acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  // gridDim.y > 1: split-K, each y-slice accumulates its share of the k-steps into fp32 C with atomic adds
  const int KT = K / BK / (int)gridDim.y;
  const int kbase = (int)blockIdx.y * KT * BK;

  u32x4_t ra[OpA::NCH], rb[OpB::NCH];
#define MREM_LOAD_GLOBAL(k0)                                                                                       \
  {                                                                                                                \
    _Pragma("unroll") for (int i = 0; i < OpA::NCH; ++i)                                                           \
        ra[i] = *reinterpret_cast<const u32x4_t*>(A + OpA::gofs(tid + NTHREADS * i, lda, m0, kbase + (k0)));       \
    _Pragma("unroll") for (int i = 0; i < OpB::NCH; ++i)                                                           \
        rb[i] = *reinterpret_cast<const u32x4_t*>(B + OpB::gofs(tid + NTHREADS * i, ldb, n0, kbase + (k0)));       \
  }
#define MREM_STORE_LDS(stage)                                                                                      \
  {                                                                                                                \
    bf16_t* As_ = smem + (stage) * STAGE;                                                                          \
    bf16_t* Bs_ = As_ + OpA::ELEMS;                                                                                \
    _Pragma("unroll") for (int i = 0; i < OpA::NCH; ++i)                                                           \
        *reinterpret_cast<u32x4_t*>(As_ + OpA::lofs(tid + NTHREADS * i)) = ra[i];                                  \
    _Pragma("unroll") for (int i = 0; i < OpB::NCH; ++i)                                                           \
        *reinterpret_cast<u32x4_t*>(Bs_ + OpB::lofs(tid + NTHREADS * i)) = rb[i];                                  \
  }

  MREM_LOAD_GLOBAL(0)
  MREM_STORE_LDS(0)
  __syncthreads();
  for (int kt = 0; kt < KT; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < KT) MREM_LOAD_GLOBAL((kt + 1) * BK)
    const bf16_t* As = smem + cur * STAGE;
    const bf16_t* Bs = As + OpA::ELEMS;
    __builtin_amdgcn_s_setprio(1);  // the wavefront that multiplies goes first: the other one of the SIMD is fetching
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8_t af[MT], bfr[NT];
#pragma unroll
      for (int i = 0; i < MT; ++i) af[i] = OpA::frag(As, wm * WM + i * 32, kk, lane);
#pragma unroll
      for (int j = 0; j < NT; ++j) bfr[j] = OpB::frag(Bs, wn * WN + j * 32, kk, lane);
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j) {
          if constexpr (I8) {
            union { bf16x8_t h; i32x4_t w; } ua, ub;
            ua.h = af[i];
            ub.h = bfr[j];
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ua.w, ub.w, acc[i][j], 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
          }
        }
    }
    __builtin_amdgcn_s_setprio(0);
    if (kt + 1 < KT) MREM_STORE_LDS(cur ^ 1)
    __syncthreads();
  }
#undef MREM_LOAD_GLOBAL
#undef MREM_STORE_LDS

  // epilogue: out = acc * (alpha * col_scale[n]) + beta * (col_vec[n] + row_vec[m]) + bias[n]
  // The rare terms (row vector, GELU) are decided once per block, not once per element.
  const float alpha = e.alpha ? *e.alpha : 1.f;
  const float beta = (e.beta ? *e.beta : 0.f) + e.beta_alpha * alpha;
  const bool split = gridDim.y > 1, lead = blockIdx.y == 0;  // the additive terms go in once, with slice 0
  auto write_out = [&](auto with_row, auto with_gelu, auto with_split) {
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int n = n0 + wn * WN + j * 32 + (lane & 31);
      const float cs = alpha * (e.col_scale ? e.col_scale[n] : 1.f);
      float cb = (e.bias && lead) ? e.bias[n] : 0.f;
      if (e.beta && e.col_vec && lead) cb += beta * e.col_vec[n];
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int mb = m0 + wm * WM + i * 32 + 4 * (lane >> 5);
        TO* __restrict__ out = C + (size_t)mb * ldc + n;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int dm = 8 * (r >> 2) + (r & 3);
          float v = (float)acc[i][j][r] * cs + cb;
          if constexpr (decltype(with_row)::value) v += beta * e.row_vec[mb + dm];
          if constexpr (decltype(with_split)::value) {
            atomicAdd(reinterpret_cast<float*>(out) + (size_t)dm * ldc, v);
          } else {
            if constexpr (decltype(with_gelu)::value) v = gelu_t<TO>(round_to<TO>(v));
            stf(out, (size_t)dm * ldc, v);
          }
        }
      }
    }
  };
  const bool row_term = e.beta && e.row_vec && lead;
  if constexpr (sizeof(TO) == 4) {
    if (split) {  // k-slices: fp32 output only, never with GELU (the launcher sees to both)
      if (row_term) write_out(std::true_type{}, std::false_type{}, std::true_type{});
      else write_out(std::false_type{}, std::false_type{}, std::true_type{});
      return;
    }
  }
  if (e.gelu) {
    if (row_term) write_out(std::true_type{}, std::true_type{}, std::false_type{});
    else write_out(std::false_type{}, std::true_type{}, std::false_type{});
  } else {
    if (row_term) write_out(std::true_type{}, std::false_type{}, std::false_type{});
    else write_out(std::false_type{}, std::false_type{}, std::false_type{});
  }
}

}  // namespace mrem
#include "mrem_gemm_dl.h"
namespace mrem {

template <int BM, int BN, int WAVES_M, int WAVES_N, bool AT, bool BT, int BK, class TO, bool I8 = false>
static void launch_mfma(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                        hipStream_t st, int k_splits = 1) {
  constexpr int NTHREADS = 64 * WAVES_M * WAVES_N;
  constexpr size_t lds = 2 * (size_t)(OperandTile<AT, BM, NTHREADS, BK>::ELEMS + OperandTile<BT, BN, NTHREADS, BK>::ELEMS) * sizeof(bf16_t);
  // the attribute belongs to the (kernel, device) pair: set again when the current device changes
  static std::atomic<int> configured_dev{-1};
  int dev = -1;
  (void)hipGetDevice(&dev);
  if (dev != configured_dev.load()) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_mfma_k<BM, BN, WAVES_M, WAVES_N, AT, BT, BK, TO, I8>),
                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured_dev.store(dev);
  }
  const int tiles_m = M / BM, tiles_n = N / BN;
  if (tl_launch_events.e0) {
    hipExtLaunchKernelGGL((gemm_mfma_k<BM, BN, WAVES_M, WAVES_N, AT, BT, BK, TO, I8>), dim3(tiles_m * tiles_n, k_splits), dim3(NTHREADS),
                          lds, st, tl_launch_events.e0, tl_launch_events.e1, 0, (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (TO*)C, ldc, M, N, K, e,
                          tiles_m, tiles_n);
    return;
  }
  hipLaunchKernelGGL((gemm_mfma_k<BM, BN, WAVES_M, WAVES_N, AT, BT, BK, TO, I8>), dim3(tiles_m * tiles_n, k_splits), dim3(NTHREADS), lds, st,
                     (const bf16_t*)A, lda, (const bf16_t*)B, ldb, (TO*)C, ldc, M, N, K, e, tiles_m, tiles_n);
}

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
// The register-staged kernel in its int8 mode: two int8 codes travel as one 16-bit element, so
// leading dimensions and the contraction length are halved.
static int gemm_policy() {
  static int pol = -1;
  if (pol < 0) { const char* v = getenv("MREM_GEMM_POLICY"); pol = v ? atoi(v) : 15; }
  return pol;
}
// experimental dispatch: policy = 10 * big + small
template <bool AT, bool BT, class TO, bool I8>
static void launch_dl_policy(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                             hipStream_t st, int splits) {
  const int pol = gemm_policy(), small = pol % 10, big = pol / 10;
  if (big && splits == 1 && M % 256 == 0 && N % 256 == 0 && (M / 256) * (N / 256) >= 192) {
    if (big == 1) return launch_dl<256, 256, 4, 2, AT, BT, 2, 128, TO, I8, 1>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    if (big == 2) return launch_dl<256, 128, 2, 2, AT, BT, 3, 64, TO, I8, 2>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    if (big == 3) return launch_dl<256, 256, 4, 2, AT, BT, 4, 64, TO, I8, 1>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    if (big == 4) return launch_dl<128, 256, 2, 2, AT, BT, 3, 64, TO, I8, 2>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
  }
  if (small == 1) return launch_dl<128, 128, 2, 2, AT, BT, 2, 128, TO, I8, 2>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  if (small == 3) return launch_dl<128, 128, 2, 2, AT, BT, 4, 128, TO, I8, 1>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  if (small == 4) return launch_dl<128, 128, 2, 2, AT, BT, 3, 128, TO, I8, 1>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  if (small == 6) return launch_dl<128, 128, 2, 2, AT, BT, 3, 64, TO, I8, 3>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  if (small == 7) return launch_dl<128, 128, 2, 2, AT, BT, 3, 64, TO, I8, 2>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  return launch_dl<128, 128, 2, 2, AT, BT, 4, 64, TO, I8, 2>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
}
static void gemm_i8_launch(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e,
                           hipStream_t st) {
  if (gemm_policy() == 0) { launch_mfma<128, 128, 2, 2, false, false, kRegBK, bf16_t, true>(A, lda / 2, B, ldb / 2, C, ldc, M, N, K / 2, e, st); return; }
  launch_dl_policy<false, false, bf16_t, true>(A, lda / 2, B, ldb / 2, C, ldc, M, N, K / 2, e, st, 1);
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
    if (gemm_policy() == 0) launch_mfma<128, 128, 2, 2, AT, BT, kRegBK, float>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
    else launch_dl_policy<AT, BT, float, false>(A, lda, B, ldb, C, ldc, M, N, K, e, st, splits);
  } else {
    if (gemm_policy() == 0) launch_mfma<128, 128, 2, 2, AT, BT, kRegBK, bf16_t>(A, lda, B, ldb, C, ldc, M, N, K, e, st);
    else launch_dl_policy<AT, BT, bf16_t, false>(A, lda, B, ldb, C, ldc, M, N, K, e, st, 1);
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
