// Host-side launchers of the gfx950 kernels.  Tensors whose element type depends
// on the activation storage type are passed as void* together with `dt`
// (0 = bfloat16, 1 = fp32).  Every launcher only enqueues work on `st`.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stddef.h>
#include <stdint.h>

#include <vector>

namespace mrem {

enum { DT_BF16 = 0, DT_F32 = 1 };
inline size_t dt_size(int dt) { return dt == DT_BF16 ? 2 : 4; }

// One quantizer as the kernels see it: step and offset live in device memory
// (they are trained), the integer range is a launch constant.
struct QArg {
  const float* s = nullptr;  // device scalar
  const float* z = nullptr;  // device scalar or null (0)
  float qn = 0.f, qp = 0.f;
  int on = 0;
};

// out[m,n] = acc * (alpha * col_scale[n]) + (beta + beta_alpha * alpha) * (col_vec[n] + row_vec[m]) + bias[n]
// alpha/beta are device scalars (null: alpha = 1, beta = 0); vectors may be null.  beta_alpha
// undoes a constant subtracted from the codes of A (unsigned codes stored as int8).
// gelu: out = round(gelu(round(out))) in the storage type.  out_f32: C is fp32.
struct Epilogue {
  const float* alpha = nullptr;
  const float* col_scale = nullptr;
  const float* beta = nullptr;
  const float* col_vec = nullptr;
  const float* row_vec = nullptr;
  const float* bias = nullptr;
  int gelu = 0;
  int out_f32 = 0;
  int c_zeroed = 0;  // the caller has already zeroed an fp32 C (a split contraction adds into it)
  float beta_alpha = 0.f;
};

// Timing of product launches with the pair of HIP events that a launch itself carries (measurement aid).
// A context owns one; products launched with a profile whose `on` is set are recorded in it.
struct GemmRecord {
  hipEvent_t e0, e1;
  double flops;             // 2 M N K of a product; algorithmic bytes of a bandwidth-bound kernel
  int cls = 0;              // 0: product on bf16 (or fp32) operands, 1: product on int8 operands, 2: bandwidth-bound kernel
  const char* label = "";   // cls 2: which kernel (a string literal)
};
struct KernelStat {
  const char* label;
  double ms, bytes;
  int64_t launches;
};
struct GemmProfile {
  bool on = false;
  std::vector<GemmRecord> recs;
  std::vector<KernelStat> stats;  // per label, filled by gemm_profile_end from the cls-2 records
};
// While a timed launch is being issued on this thread: the event pair that the launch itself carries (the
// runtime stamps them with the kernel's own begin and end, so no packet is added to the queue and the
// elapsed time is the kernel's duration).  Launch sites that can be timed go through MREM_LAUNCH.
struct LaunchEvents {
  hipEvent_t e0 = nullptr, e1 = nullptr;
};
extern thread_local LaunchEvents tl_launch_events;
#define MREM_LAUNCH(kern, grid, block, lds, st, ...)                                                                        \
  do {                                                                                                                      \
    if (::mrem::tl_launch_events.e0)                                                                                        \
      hipExtLaunchKernelGGL(kern, grid, block, lds, st, ::mrem::tl_launch_events.e0, ::mrem::tl_launch_events.e1, 0, __VA_ARGS__); \
    else                                                                                                                    \
      hipLaunchKernelGGL(kern, grid, block, lds, st, __VA_ARGS__);                                                          \
  } while (0)
void gemm_profile_begin(GemmProfile* p);
int gemm_profile_end(GemmProfile* p, double ms[2], double flops[2], int64_t launches[2]);  // [0] bf16 operands, [1] int8 operands

// C[M,N] = op(A) * op(B)^T.  a_t = 0: A is stored [M,K] (K contiguous); a_t = 1: A is stored
// [K,M] (the contraction index is the slow one).  Same for B with N.  lda/ldb: row pitch.
void gemm(int dt, int a_t, int b_t, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
          const Epilogue& e, hipStream_t st, GemmProfile* prof = nullptr);
// C[M,N] (bf16) = A[M,K] * B[N,K]^T on int8 codes with exact int32 accumulation; needs
// gemm_i8_ok(...).  Same epilogue.
bool gemm_i8_ok(const void* A, int lda, const void* B, int ldb, int M, int N, int K);
void gemm_i8(const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K, const Epilogue& e, hipStream_t st,
             GemmProfile* prof = nullptr);
// C[M,N] = A[M,K] * B[N,K]^T  (both operands contiguous along K)
void gemm_nt(int dt, const void* A, int lda, const void* B, int ldb, void* C, int ldc, int M, int N, int K,
             const Epilogue& e, hipStream_t st, GemmProfile* prof = nullptr);

// ---- weights ------------------------------------------------------------------
// per_channel = 0: one step scale[0] for the whole tensor
void weight_quantize_i8(const float* w, float* scale, int8_t* codes, int64_t N, int64_t K, int bits, int per_channel, int init_scale,
                        hipStream_t st);
void weight_step_init(const float* w, float* scale, int64_t N, int64_t K, int bits, hipStream_t st);
// scale[0..N) := max_n scale[n]  (one step for the whole matrix, kept as N equal entries)
void tie_steps_max(float* scale, int64_t N, hipStream_t st);
// Per matrix w[N,K] with steps sw[N]: codes[N,K] (integer-valued, storage type), what[N,K] =
// round(s*q) (may be null), zcorr[N] = s[n] * sum_k q[n,k].  bits = 0: codes = what = round(w),
// zcorr[n] = sum_k round(w[n,k]).  All matrices of the list go into one launch (kMaxMatrixJobs per launch).
constexpr int kMaxMatrixJobs = 24;
struct WeightJob {
  const float* w;
  const float* sw;
  void* codes;     // may be null when only the int8 codes are wanted
  void* what;
  float* zcorr;
  int8_t* codes8;  // may be null
  int N, K;
};
void weight_prepare(int dt, const WeightJob* jobs, int njobs, int bits, hipStream_t st);
void convert_f32(int dt, const float* src, void* dst, int64_t n, hipStream_t st);

// ---- elementwise / normalisation ------------------------------------------------
// codes8 (may be null): the same codes as int8, for the int8 products of the forward pass
void act_quantize(int dt, const void* a, void* codes, int64_t n, QArg q, hipStream_t st, int8_t* codes8 = nullptr);
// Eq. 4 in the same pass: mixed = round(wa * a + wb * b) is stored and quantized
void mix_quantize(int dt, const void* a, const void* b, float wa, float wb, void* mixed, void* codes, int64_t n, QArg q, hipStream_t st,
                  int8_t* codes8 = nullptr);
// codes8 (may be null): codes - shift8 as int8 (the unsigned grid of the GELU output, recentred)
void gelu_quantize(int dt, const void* u, void* codes, int64_t n, QArg q, hipStream_t st, int8_t* codes8 = nullptr, float shift8 = 0.f);
// bf16/fp32 integer codes -> int8 (codes - shift); for producers without an int8 output of their own
void codes_to_i8(int dt, const void* codes, int8_t* codes8, int64_t n, float shift, hipStream_t st);
// Grid of the column-walking backward kernels over a [T, C] tensor: gx column blocks, gy row
// slabs (gy <= kColMaxParts, gx * gy <= 2048).
constexpr int kColMaxParts = 512;
struct ColGrid { int gx, gy; };
ColGrid col_grid(int T_, int C);
// du[T,C] = dgh * inside(g) * gelu'(u); partials[gx*gy]: step-size gradient terms;
// colparts[gy][C] (may be null): column sums of du per row slab (bias gradient)
ColGrid gelu_quant_bwd(int dt, const void* dgh, const void* u, void* du, int T_, int C, QArg q, float* partials, float* colparts,
                       hipStream_t st);
// d_out = d_q * inside(a) (d_out may be null); partials[grid]: step-size gradient terms
int quant_bwd(int dt, const void* d_q, const void* a, void* d_out, int64_t n, QArg q, float* partials, hipStream_t st);
// partial sums of d_q * (code - v*inside) only (layer-0 input quantizer)
int quant_bwd_reduce(int dt, const void* d_q, const void* a, int64_t n, QArg q, float* partials, hipStream_t st);

// y = LN(x + r) * gamma + beta ; optional codes of y ; mean/rstd saved
void ln_fwd(int dt, const void* x, const void* r, const float* gamma, const float* beta, void* y, void* ycodes, QArg q,
            float* mu, float* rstd, int T, int H, float eps, hipStream_t st, int8_t* ycodes8 = nullptr);
// dy = d_a + d_q * inside(a_q) + 2 * loss_scale * (a_q - loss_ref)   (each of d_a, d_q, loss_ref may be null; the
// last term is the gradient of the squared-error term of Eq. 3, and the sum of (a_q - loss_ref)^2 is returned in
// the partials).
// dr = LN backward of dy through LN(x + r); partials[nparts][3H+2]: dgamma, dbeta, colsum(dr), ds, squared error
int ln_bwd(int dt, const void* d_a, const void* d_q, const void* a_q, QArg q, const void* x,
           const void* r, const float* mu, const float* rstd, const float* gamma, void* dr, float* partials, int T,
           int H, hipStream_t st, const void* loss_ref = nullptr, float loss_scale = 0.f);
int ln_bwd_parts(int T);


// out[c] = scale * sum_p partials[p*width + begin + c], c < len.  Jobs are collected on the
// host while the first-stage kernels are enqueued and finished by reduce_jobs afterwards.
struct ReduceJob {
  const float* partials = nullptr;
  float* out = nullptr;
  int nparts = 0, width = 0, begin = 0, len = 0;
  float scale = 1.f;
};
constexpr int kMaxReduceJobs = 64;
void reduce_jobs(const ReduceJob* jobs, int njobs, hipStream_t st);
// nonfinite_flag (device, may be null): set to 1 when the total is not finite
void loss_total(float* loss_out, int n_layers, int* nonfinite_flag, hipStream_t st);
void fill_f32(float* p, float v, int64_t n, hipStream_t st);
// zeroes up to kMaxFillRegions regions in one launch
constexpr int kMaxFillRegions = 64;
struct FillRegion { float* p; int64_t n; };
void zero_regions(const FillRegion* regions, int count, hipStream_t st);
// 2 if a product with fp32 output of this shape is accumulated into its (zeroed) output in two
// k-slices, 1 if it is written
int gemm_f32_k_slices(int dt, int M, int N, int K);
void axpby(int dt, const void* a, const void* b, float wa, float wb, void* out, int64_t n, hipStream_t st);
// dy = 2 * scale * (yq - yfp) over n values (multiple of 8); partials[returned count]: sums of (yq - yfp)^2
int mse_grad(int dt, const void* yq, const void* yfp, void* dy, int64_t n, float scale, float* partials, hipStream_t st);

// ---- attention -----------------------------------------------------------------
struct AttnQ {
  QArg q, k, p, v, c;
};
// three column sections of qkv[T,3H] with their own quantizers -> integer codes
void qkv_quantize(int dt, const void* qkv, void* codes, int T_, int H, QArg q, QArg k, QArg v, hipStream_t st);
// d_qkv = d_qkvh * inside ; partials[gx*gy][3]: step-size gradient terms of q, k, v;
// colparts[gy][3H] (may be null): column sums of d_qkv per row slab (bias gradient)
ColGrid qkv_quant_bwd(int dt, const void* d_qkvh, const void* qkv, void* d_qkv, int T_, int H, QArg q, QArg k, QArg v, float* partials,
                      float* colparts, hipStream_t st);
// codes [T,3H] (or raw values when the quantizers are off); ctx [T,H] stored context,
// ctx_codes [T,H] its codes under quantizer c (null: skip); pmax_rows [B*nh*S] row
// maxima of the probabilities (null: skip); seqlens may be null
void attn_fwd(int dt, const void* codes, void* ctx, void* ctx_codes, const AttnQ& aq, const int32_t* seqlens, int B, int S, int nh,
              int d, float* pmax_rows, hipStream_t st);
// dctx [T,H]: gradient w.r.t. the (unquantized) context; writes d_qkvh [T,3H], the
// gradient w.r.t. the quantized q, k, v; scratch_da, scratch_ph: [B*nh*S*S] fp32;
// ds_rows [B*nh*S]: per-row step-size gradient terms of the probability quantizer
void attn_bwd(int dt, const void* codes, const void* dctx, void* d_qkvh, const AttnQ& aq, const int32_t* seqlens, int B, int S, int nh,
              int d, float* scratch_da, float* scratch_ph, float* ds_rows, hipStream_t st);

// Matrix-core versions (bf16, head dimension 64, 64 <= S <= 384).  The forward saves the
// row maximum and row sum of the softmax (stat_m, stat_l: [B*nh*S], may be null); the
// backward needs them, two bf16 scratch tiles of B*nh*s_pad^2 elements (s_pad = S rounded
// up to 32) and returns the number of partial sums written to ds_parts.
bool attn_mfma_ok(int dt, int S, int d);
void attn_fwd_mfma(const void* codes, void* ctx, void* ctx_codes, const AttnQ& aq, const int32_t* seqlens, int B, int S, int nh,
                   float* pmax_rows, float* stat_m, float* stat_l, hipStream_t st, int8_t* ctx_codes8 = nullptr);
int attn_bwd_mfma(const void* codes, const void* dctx, void* d_qkvh, const AttnQ& aq, const int32_t* seqlens, int B, int S, int nh,
                  const float* stat_m, const float* stat_l, void* pt_scratch, void* dat_scratch, float* ds_parts, hipStream_t st);

// ---- calibration reductions -------------------------------------------------------
// partials[grid][3]: max|a|, min(f(a)), max(f(a)) over a strided [rows, cols] view; f = gelu if gelu != 0
int absminmax(int dt, const void* a, int rows, int cols, int ld, int gelu, float* partials, hipStream_t st);
// mode 0: s = max|a| / qp ; mode 1: s = max / qp (z = 0) ; mode 2: z = min, s = (max - z) / qp
void calib_finalize(const float* partials, int nparts, int mode, float qp, float* s_out, float* z_out, hipStream_t st);

// ---- update ----------------------------------------------------------------------
struct AdamArg {
  float lr, beta1, beta2, eps, wd, bc1, bc2;  // bc = 1 - beta^t
  float floor;                                // lower bound applied when clamp != 0
};
// one block per row n of w[N,K]: straight-through mask on dw_hat (in grads), row
// reduction for the step gradient, AdamW on w[n,:] and on sw[n].  z_in/db (may be null):
// offset of an asymmetric input quantizer and the bias gradient, dw_hat[n,:] += z * db[n].
// All matrices of the list go into one launch (kMaxMatrixJobs per launch).
struct AdamJob {
  float *w, *sw, *g_w, *g_sw, *m_w, *v_w, *m_sw, *v_sw;
  const float* z_in;
  const float* db;
  int N, K;
};
// tied != 0 (one step per matrix): the row kernels only leave their step gradients in g_sw; a second
// launch sums them per matrix in a fixed order, updates the one step and writes it, its moments and its
// gradient to all N entries.
void adam_matrix(const AdamJob* jobs, int njobs, int bits, AdamArg a, int write_grads, int tied, hipStream_t st);
// AdamW without decay on segments [off, off + n) of the parameter vector (all vectors share one
// layout); clamp != 0 applies the lower bound a.floor afterwards (step sizes).  One launch per
// kMaxVecJobs segments.
constexpr int kMaxVecJobs = 64;
struct VecJob {
  int64_t off;
  int64_t n;
  int clamp;
};
void adam_vector(float* p, const float* g, float* m, float* v, const VecJob* jobs, int njobs, AdamArg a, hipStream_t st);

}  // namespace mrem
