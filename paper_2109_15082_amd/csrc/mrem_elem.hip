// Bandwidth-bound kernels of the MREM module step: quantizers (Section 3.1, Eq. 1,
// with the straight-through backward of Section 3.1.1), residual + LayerNorm,
// GELU, the per-layer squared-error term of Eq. 3 (inside the backward kernel of the
// second LayerNorm), calibration reductions and the AdamW update.
#include "mrem_common.h"
#include "mrem_kernels.h"

#include <float.h>

namespace mrem {

// ------------------------------------------------------------------------------
// 8-element (16 or 32 byte) vector access
// ------------------------------------------------------------------------------
__device__ __forceinline__ void load8(const float* p, float* o) {
  const float4 a = *reinterpret_cast<const float4*>(p);
  const float4 b = *reinterpret_cast<const float4*>(p + 4);
  o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w; o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16_t* p, float* o) {
  const uint4 r = *reinterpret_cast<const uint4*>(p);
  o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xffff0000u);
  o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xffff0000u);
  o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xffff0000u);
  o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xffff0000u);
}
__device__ __forceinline__ void store8(float* p, const float* v) {
  *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
  *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ uint32_t pack2(float lo, float hi) {
  union { bf16_t h[2]; uint32_t u; } c;
  c.h[0] = static_cast<bf16_t>(lo);
  c.h[1] = static_cast<bf16_t>(hi);
  return c.u;
}
__device__ __forceinline__ void store8(bf16_t* p, const float* v) {
  uint4 r;
  r.x = pack2(v[0], v[1]); r.y = pack2(v[2], v[3]); r.z = pack2(v[4], v[5]); r.w = pack2(v[6], v[7]);
  *reinterpret_cast<uint4*>(p) = r;
}

// eight stored values kept as loaded (4 registers for bf16, 8 for fp32) until they are needed
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2e_t __attribute__((ext_vector_type(2)));
typedef float f32x4v_t __attribute__((ext_vector_type(4)));
template <class T>
struct Raw8;
template <>
struct Raw8<bf16_t> {
  u32x4_t r;
  __device__ __forceinline__ void load(const bf16_t* p) { r = *reinterpret_cast<const u32x4_t*>(p); }
  __device__ __forceinline__ float get(int j) const {
    const unsigned w = r[j >> 1];
    return __uint_as_float((j & 1) ? (w & 0xffff0000u) : (w << 16));
  }
};
template <>
struct Raw8<float> {
  f32x4v_t a, b;
  __device__ __forceinline__ void load(const float* p) {
    a = *reinterpret_cast<const f32x4v_t*>(p);
    b = *reinterpret_cast<const f32x4v_t*>(p + 4);
  }
  __device__ __forceinline__ float get(int j) const { return j < 4 ? a[j] : b[j - 4]; }
};

// eight integer-valued codes (minus shift) as int8, one 8-byte store
__device__ __forceinline__ void store8_i8(int8_t* p, const float* v, float shift) {
  unsigned lo = 0u, hi = 0u;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    lo |= ((unsigned)(int)(v[j] - shift) & 0xffu) << (8 * j);
    hi |= ((unsigned)(int)(v[4 + j] - shift) & 0xffu) << (8 * j);
  }
  u32x2e_t r = {lo, hi};
  *reinterpret_cast<u32x2e_t*>(p) = r;
}

__device__ __forceinline__ QuantParam load_q(const QArg& a) {
  QuantParam q;
  q.on = a.on;
  q.s = a.on ? *a.s : 1.f;
  q.z = (a.on && a.z) ? *a.z : 0.f;
  q.qn = a.qn;
  q.qp = a.qp;
  q.rs = quant_reciprocal(q.s);
  return q;
}

static inline int ew_grid(int64_t n) {
  int64_t g = (n / 8 + 255) / 256;
  if (g < 1) g = 1;
  if (g > 2048) g = 2048;
  return (int)g;
}

#define MREM_DISPATCH(dt, ...)                      \
  do {                                              \
    if ((dt) == DT_BF16) { typedef bf16_t T; __VA_ARGS__; } \
    else { typedef float T; __VA_ARGS__; }          \
  } while (0)

// ------------------------------------------------------------------------------
// activation quantizer forward: integer-valued codes in the storage type
// ------------------------------------------------------------------------------
template <class T>
__global__ void act_quantize_k(const T* __restrict__ a, T* __restrict__ codes, int64_t nchunks, QArg qa, int8_t* __restrict__ codes8) {
  const QuantParam q = load_q(qa);
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunks; c += (int64_t)gridDim.x * blockDim.x) {
    float v[8];
    load8(a + c * 8, v);
    if (q.on) {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = q_code(q_ratio_t<T>(v[j], q), q);
    }
    store8(codes + c * 8, v);
    if (codes8) store8_i8(codes8 + c * 8, v, 0.f);
  }
}
void act_quantize(int dt, const void* a, void* codes, int64_t n, QArg q, hipStream_t st, int8_t* codes8) {
  MREM_DISPATCH(dt, MREM_LAUNCH(act_quantize_k<T>, dim3(ew_grid(n)), dim3(256), 0, st, (const T*)a, (T*)codes, n / 8, q, codes8));
}
// Eq. 4 folded into the input quantizer of a module's first layer: mixed = wa * a + wb * b is stored (the
// layer's residual path and its backward pass read it) and quantized in the same pass.
template <class T>
__global__ void mix_quantize_k(const T* __restrict__ a, const T* __restrict__ b, float wa, float wb, T* __restrict__ mixed,
                               T* __restrict__ codes, int64_t nchunks, QArg qa, int8_t* __restrict__ codes8) {
  const QuantParam q = load_q(qa);
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunks; c += (int64_t)gridDim.x * blockDim.x) {
    float x[8], y[8], v[8];
    load8(a + c * 8, x);
    load8(b + c * 8, y);
#pragma unroll
    for (int j = 0; j < 8; ++j) v[j] = round_to<T>(wa * x[j] + wb * y[j]);
    store8(mixed + c * 8, v);
    if (q.on) {
#pragma unroll
      for (int j = 0; j < 8; ++j) v[j] = q_code(q_ratio_t<T>(v[j], q), q);
    }
    store8(codes + c * 8, v);
    if (codes8) store8_i8(codes8 + c * 8, v, 0.f);
  }
}
void mix_quantize(int dt, const void* a, const void* b, float wa, float wb, void* mixed, void* codes, int64_t n, QArg q, hipStream_t st,
                  int8_t* codes8) {
  MREM_DISPATCH(dt, MREM_LAUNCH(mix_quantize_k<T>, dim3(ew_grid(n)), dim3(256), 0, st, (const T*)a, (const T*)b, wa, wb, (T*)mixed,
                                       (T*)codes, n / 8, q, codes8));
}
template <class T>
__global__ void codes_to_i8_k(const T* __restrict__ codes, int8_t* __restrict__ codes8, int64_t nchunks, float shift) {
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunks; c += (int64_t)gridDim.x * blockDim.x) {
    float v[8];
    load8(codes + c * 8, v);
    store8_i8(codes8 + c * 8, v, shift);
  }
}
void codes_to_i8(int dt, const void* codes, int8_t* codes8, int64_t n, float shift, hipStream_t st) {
  MREM_DISPATCH(dt, MREM_LAUNCH(codes_to_i8_k<T>, dim3(ew_grid(n)), dim3(256), 0, st, (const T*)codes, codes8, n / 8, shift));
}

// Three column sections of qkv[T,3H] with their own quantizers.  A thread owns one 8-element
// column chunk (so its quantizer is fixed) and walks down the rows, four rows in flight; a block
// of 128 threads covers 2 KiB of a row.
constexpr int kQkvThreads = 128, kQkvRows = 4;
struct QkvGrid { int gx, gy; };
static inline QkvGrid qkv_grid(int T_, int H) {
  QkvGrid g;
  g.gx = (3 * H / 8 + kQkvThreads - 1) / kQkvThreads;
  const int groups = (T_ + kQkvRows - 1) / kQkvRows;
  const int cap = 2048 / g.gx > 0 ? 2048 / g.gx : 1;  // the reductions downstream hold at most 2048 blocks
  const int iters = (groups + cap - 1) / cap;          // every block walks the same number of row groups
  g.gy = iters > 0 ? (groups + iters - 1) / iters : 1;
  if (g.gy < 1) g.gy = 1;
  return g;
}
__device__ __forceinline__ QuantParam pick_q(int sec, const QuantParam& a, const QuantParam& b, const QuantParam& c) {
  return sec == 0 ? a : (sec == 1 ? b : c);
}

template <class T>
__global__ __launch_bounds__(kQkvThreads) void qkv_quantize_k(const T* __restrict__ a, T* __restrict__ codes, int T_, int H8, QArg q0,
                                                               QArg q1, QArg q2) {
  const int cc = blockIdx.x * kQkvThreads + threadIdx.x, row_chunks = 3 * H8;
  if (cc >= row_chunks) return;
  const QuantParam q = pick_q(cc / H8, load_q(q0), load_q(q1), load_q(q2));
  for (int r0 = blockIdx.y * kQkvRows; r0 < T_; r0 += gridDim.y * kQkvRows) {
    float v[kQkvRows][8];
#pragma unroll
    for (int i = 0; i < kQkvRows; ++i)
      if (r0 + i < T_) load8(a + ((size_t)(r0 + i) * row_chunks + cc) * 8, v[i]);
#pragma unroll
    for (int i = 0; i < kQkvRows; ++i) {
      if (r0 + i >= T_) break;
      if (q.on) {
#pragma unroll
        for (int j = 0; j < 8; ++j) v[i][j] = q_code(q_ratio_t<T>(v[i][j], q), q);
      }
      store8(codes + ((size_t)(r0 + i) * row_chunks + cc) * 8, v[i]);
    }
  }
}
void qkv_quantize(int dt, const void* qkv, void* codes, int T_, int H, QArg q, QArg k, QArg v, hipStream_t st) {
  const QkvGrid g = qkv_grid(T_, H);
  MREM_DISPATCH(dt, MREM_LAUNCH(qkv_quantize_k<T>, dim3(g.gx, g.gy), dim3(kQkvThreads), 0, st, (const T*)qkv, (T*)codes, T_,
                                       H / 8, q, k, v));
}

// Column-walking backward kernels: a thread owns one 8-element column chunk and walks down its
// share of the rows, kColRows rows in flight, so the column sums of what it writes (the bias
// gradient of the projection in front) stay in its registers.  Grid y splits the rows into
// at most kColMaxParts slabs; block (x, y) writes row y of colparts[gy][C] for its columns.
constexpr int kColRows = 8;
ColGrid col_grid(int T_, int C) {
  ColGrid g;
  g.gx = (C / 8 + kQkvThreads - 1) / kQkvThreads;
  const int groups = (T_ + kColRows - 1) / kColRows;
  int cap = 2048 / g.gx;  // the reductions downstream hold at most 2048 blocks
  if (cap > kColMaxParts) cap = kColMaxParts;
  if (cap < 1) cap = 1;
  const int iters = (groups + cap - 1) / cap;  // every block walks the same number of row groups
  g.gy = iters > 0 ? (groups + iters - 1) / iters : 1;
  if (g.gy < 1) g.gy = 1;
  return g;
}

// d_out = d_q * inside ; partial[block][sec] += d_q * (code - v * inside) ; colparts: column sums of d_out
template <class T>
__global__ __launch_bounds__(kQkvThreads) void qkv_quant_bwd_k(const T* __restrict__ dq, const T* __restrict__ a, T* __restrict__ dout,
                                                                int T_, int H8, QArg q0, QArg q1, QArg q2, float* __restrict__ partials,
                                                                float* __restrict__ colparts) {
  __shared__ float red[17];
  const int cc = blockIdx.x * kQkvThreads + threadIdx.x, row_chunks = 3 * H8;
  const bool live = cc < row_chunks;
  const int sec = live ? cc / H8 : 0;
  const QuantParam q = pick_q(sec, load_q(q0), load_q(q1), load_q(q2));
  float acc = 0.f, col[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (live) {
    for (int r0 = blockIdx.y * kColRows; r0 < T_; r0 += gridDim.y * kColRows) {
      Raw8<T> graw[kColRows], xraw[kColRows];
#pragma unroll
      for (int i = 0; i < kColRows; ++i) {
        if (r0 + i < T_) {
          const size_t o = ((size_t)(r0 + i) * row_chunks + cc) * 8;
          graw[i].load(dq + o);
          if (q.on) xraw[i].load(a + o);
        }
      }
#pragma unroll
      for (int i = 0; i < kColRows; ++i) {
        if (r0 + i >= T_) break;
        float g[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          g[j] = graw[i].get(j);
          if (q.on) {
            const float v = q_ratio_t<T>(xraw[i].get(j), q);
            const bool in = q_inside(v, q);
            acc += g[j] * (q_code(v, q) - (in ? v : 0.f));
            g[j] = in ? g[j] : 0.f;
          }
          col[j] += round_to<T>(g[j]);
        }
        if (dout) store8(dout + ((size_t)(r0 + i) * row_chunks + cc) * 8, g);
      }
    }
    if (colparts) store8(colparts + ((size_t)blockIdx.y * row_chunks + cc) * 8, col);
  }
  const int block = blockIdx.y * gridDim.x + blockIdx.x;
  for (int s = 0; s < 3; ++s) {
    const float t = block_sum((live && sec == s) ? acc : 0.f, red);
    if (threadIdx.x == 0) partials[block * 3 + s] = t;
  }
}
ColGrid qkv_quant_bwd(int dt, const void* d_qkvh, const void* qkv, void* d_qkv, int T_, int H, QArg q, QArg k, QArg v,
                      float* partials, float* colparts, hipStream_t st) {
  const ColGrid g = col_grid(T_, 3 * H);
  MREM_DISPATCH(dt, MREM_LAUNCH(qkv_quant_bwd_k<T>, dim3(g.gx, g.gy), dim3(kQkvThreads), 0, st, (const T*)d_qkvh, (const T*)qkv,
                                       (T*)d_qkv, T_, H / 8, q, k, v, partials, colparts));
  return g;
}

// generic single-quantizer backward (d_out may be null: reduction only)
template <class T>
__global__ void quant_bwd_k(const T* __restrict__ dq, const T* __restrict__ a, T* __restrict__ dout, int64_t nchunks, QArg qa,
                            float* __restrict__ partials) {
  __shared__ float red[17];
  const QuantParam q = load_q(qa);
  float acc = 0.f;
  // two chunks per thread and round, both fetched before the first is used
  const int64_t stride = (int64_t)gridDim.x * blockDim.x;
  for (int64_t c0 = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c0 < nchunks; c0 += 2 * stride) {
    const int64_t c1 = c0 + stride;
    const bool two = c1 < nchunks;
    Raw8<T> graw[2], xraw[2];
    graw[0].load(dq + c0 * 8);
    if (q.on) xraw[0].load(a + c0 * 8);
    if (two) {
      graw[1].load(dq + c1 * 8);
      if (q.on) xraw[1].load(a + c1 * 8);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (i == 1 && !two) break;
      float g[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        g[j] = graw[i].get(j);
        if (q.on) {
          const float v = q_ratio_t<T>(xraw[i].get(j), q);
          const bool in = q_inside(v, q);
          acc += g[j] * (q_code(v, q) - (in ? v : 0.f));
          g[j] = in ? g[j] : 0.f;
        }
      }
      if (dout) store8(dout + (i ? c1 : c0) * 8, g);
    }
  }
  const float t = block_sum(acc, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = t;
}
int quant_bwd(int dt, const void* d_q, const void* a, void* d_out, int64_t n, QArg q, float* partials, hipStream_t st) {
  const int g = ew_grid((n + 1) / 2);
  MREM_DISPATCH(dt, MREM_LAUNCH(quant_bwd_k<T>, dim3(g), dim3(256), 0, st, (const T*)d_q, (const T*)a, (T*)d_out,
                                       n / 8, q, partials));
  return g;
}
int quant_bwd_reduce(int dt, const void* d_q, const void* a, int64_t n, QArg q, float* partials, hipStream_t st) {
  return quant_bwd(dt, d_q, a, nullptr, n, q, partials, st);
}

// ------------------------------------------------------------------------------
// GELU + quantizer of its output (unsigned grid with offset)
// ------------------------------------------------------------------------------
template <class T>
__global__ void gelu_quantize_k(const T* __restrict__ u, T* __restrict__ codes, int64_t nchunks, QArg qa, int8_t* __restrict__ codes8,
                                float shift8) {
  const QuantParam q = load_q(qa);
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunks; c += (int64_t)gridDim.x * blockDim.x) {
    float v[8];
    load8(u + c * 8, v);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float g = gelu_t<T>(v[j]);
      v[j] = q.on ? q_code(q_ratio_t<T>(g, q), q) : g;
    }
    store8(codes + c * 8, v);
    if (codes8) store8_i8(codes8 + c * 8, v, shift8);
  }
}
void gelu_quantize(int dt, const void* u, void* codes, int64_t n, QArg q, hipStream_t st, int8_t* codes8, float shift8) {
  MREM_DISPATCH(dt, MREM_LAUNCH(gelu_quantize_k<T>, dim3(ew_grid(n)), dim3(256), 0, st, (const T*)u, (T*)codes, n / 8, q, codes8,
                                       shift8));
}

// du = dgh * inside * gelu'(u) ; partials[block]: step-size gradient terms ; colparts: column sums of du
template <class T>
__global__ __launch_bounds__(kQkvThreads) void gelu_quant_bwd_k(const T* __restrict__ dgh, const T* __restrict__ u, T* __restrict__ du,
                                                                 int T_, int C8, QArg qa, float* __restrict__ partials,
                                                                 float* __restrict__ colparts) {
  __shared__ float red[17];
  const int cc = blockIdx.x * kQkvThreads + threadIdx.x;
  const bool live = cc < C8;
  const QuantParam q = load_q(qa);
  float acc = 0.f, col[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  if (live) {
    for (int r0 = blockIdx.y * kColRows; r0 < T_; r0 += gridDim.y * kColRows) {
      Raw8<T> graw[kColRows], xraw[kColRows];
#pragma unroll
      for (int i = 0; i < kColRows; ++i) {
        if (r0 + i < T_) {
          const size_t o = ((size_t)(r0 + i) * C8 + cc) * 8;
          graw[i].load(dgh + o);
          xraw[i].load(u + o);
        }
      }
#pragma unroll
      for (int i = 0; i < kColRows; ++i) {
        if (r0 + i >= T_) break;
        float g[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float x = xraw[i].get(j);
          float dg = graw[i].get(j);
          if (q.on) {
            const float v = q_ratio_t<T>(gelu_t<T>(x), q);
            const bool in = q_inside(v, q);
            acc += dg * (q_code(v, q) - (in ? v : 0.f));
            dg = in ? dg : 0.f;
          }
          g[j] = dg * gelu_grad_t<T>(x);
          col[j] += round_to<T>(g[j]);
        }
        store8(du + ((size_t)(r0 + i) * C8 + cc) * 8, g);
      }
    }
    if (colparts) store8(colparts + ((size_t)blockIdx.y * C8 + cc) * 8, col);
  }
  const float t = block_sum(acc, red);
  if (threadIdx.x == 0) partials[blockIdx.y * gridDim.x + blockIdx.x] = t;
}
ColGrid gelu_quant_bwd(int dt, const void* dgh, const void* u, void* du, int T_, int C, QArg q, float* partials, float* colparts,
                       hipStream_t st) {
  const ColGrid g = col_grid(T_, C);
  MREM_DISPATCH(dt, MREM_LAUNCH(gelu_quant_bwd_k<T>, dim3(g.gx, g.gy), dim3(kQkvThreads), 0, st, (const T*)dgh, (const T*)u, (T*)du,
                                       T_, C / 8, q, partials, colparts));
  return g;
}

// ------------------------------------------------------------------------------
// residual + LayerNorm: one wavefront per token row, 8-element chunks per lane
// ------------------------------------------------------------------------------
// hidden <= 64 lanes * 8 values * 4 chunks = 2048 (checked when the context is created)

// NCH: 8-element chunks per lane (hidden <= 512 * NCH)
template <class T, int NCH>
__global__ __launch_bounds__(256) void ln_fwd_k(const T* __restrict__ x, const T* __restrict__ r, const float* __restrict__ gamma,
                         const float* __restrict__ beta, T* __restrict__ y, T* __restrict__ ycodes, QArg qa,
                         float* __restrict__ mu_out, float* __restrict__ rstd_out, int T_, int H, float eps,
                         int8_t* __restrict__ ycodes8) {
  const QuantParam q = load_q(qa);
  const int lane = threadIdx.x & 63;
  const int row = blockIdx.x * (blockDim.x / 64) + threadIdx.x / 64;
  if (row >= T_) return;
  const int nch = H / 8;
  float v[NCH][8];
  float sum = 0.f;
  Raw8<T> ra[NCH], rb[NCH];
  Raw8<float> rg[NCH], rbeta[NCH];
  // every load of the row goes out before the first value is used: the gain and shift vectors (cache hits) arrive
  // under the two reductions instead of after them
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      ra[i].load(x + (size_t)row * H + c * 8);
      rb[i].load(r + (size_t)row * H + c * 8);
    }
  }
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      rg[i].load(gamma + c * 8);
      rbeta[i].load(beta + c * 8);
    }
  }
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { v[i][j] = ra[i].get(j) + rb[i].get(j); sum += v[i][j]; }
    }
  }
  const float mean = wave_sum(sum) / (float)H;
  float sq = 0.f;
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
#pragma unroll
      for (int j = 0; j < 8; ++j) { const float t = v[i][j] - mean; sq += t * t; }
    }
  }
  const float var = wave_sum(sq) / (float)H;
  const float rstd = 1.0f / sqrtf(var + eps);
  if (lane == 0) { mu_out[row] = mean; rstd_out[row] = rstd; }
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
    const int c = lane + 64 * i;
    if (c < nch) {
      float o[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) o[j] = (v[i][j] - mean) * rstd * rg[i].get(j) + rbeta[i].get(j);
      store8(y + (size_t)row * H + c * 8, o);
      if (ycodes) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const float s = round_to<T>(o[j]);
          o[j] = q.on ? q_code(q_ratio_t<T>(s, q), q) : s;
        }
        store8(ycodes + (size_t)row * H + c * 8, o);
        if (ycodes8) store8_i8(ycodes8 + (size_t)row * H + c * 8, o, 0.f);
      }
    }
  }
}
void ln_fwd(int dt, const void* x, const void* r, const float* gamma, const float* beta, void* y, void* ycodes, QArg q,
            float* mu, float* rstd, int T_, int H, float eps, hipStream_t st, int8_t* ycodes8) {
#define MREM_LN_FWD(NCH)                                                                                                      \
  MREM_DISPATCH(dt, MREM_LAUNCH((ln_fwd_k<T, NCH>), dim3((T_ + 3) / 4), dim3(256), 0, st, (const T*)x, (const T*)r, gamma, beta, \
                                (T*)y, (T*)ycodes, q, mu, rstd, T_, H, eps, ycodes8))
  if (H <= 512) MREM_LN_FWD(1);
  else if (H <= 1024) MREM_LN_FWD(2);
  else MREM_LN_FWD(4);
#undef MREM_LN_FWD
}

constexpr int kLnBwdWaves = 4;       // wavefronts per block (256 threads: such a block still fits beside another stream's product block)
constexpr int kLnBwdRowsPerWave = 2;  // token rows per wavefront, both in flight when registers allow
constexpr int kLnBwdRows = kLnBwdWaves * kLnBwdRowsPerWave;  // token rows per block
int ln_bwd_parts(int T_) { return (T_ + kLnBwdRows - 1) / kLnBwdRows; }

// One wavefront per token row, kLnBwdRowsPerWave rows per wavefront with the column sums
// (gamma, beta and residual-bias gradients) accumulated in registers; the wavefronts of a block
// then meet in LDS (upper half onto lower half, then the lower half) and the block writes one partial row
// [3H + 2] (the last two values are the step-size gradient of the quantizer in front of the next layer
// and the squared-error sum of this layer's term of Eq. 3).
// NCH: 8-element chunks per lane (hidden <= 512 * NCH)
// HAS_A, HAS_Q, HAS_L: which of the optional inputs exist (gradient from above d_a, gradient d_q through the
// quantizer of a_q, full-precision output loss_ref for the layer's loss term): decided per instantiation, so the
// per-element code has no tests on them.
template <class T, int NCH, bool HAS_A, bool HAS_Q, bool HAS_L>
__global__ __launch_bounds__(64 * kLnBwdWaves) void ln_bwd_k(const T* __restrict__ d_a, const T* __restrict__ d_q,
                                                             const T* __restrict__ a_q, QArg qa, const T* __restrict__ x, const T* __restrict__ r,
                                                             const float* __restrict__ mu, const float* __restrict__ rstd_in,
                                                             const float* __restrict__ gamma, T* __restrict__ dr, float* __restrict__ partials,
                                                             int T_, int H, const T* __restrict__ loss_ref, float loss_scale) {
  extern __shared__ float red[];  // [kLnBwdWaves/2][3*H] + 2 * kLnBwdWaves
  constexpr int HALF = kLnBwdWaves / 2;
  const QuantParam q = load_q(qa);
  const int lane = threadIdx.x & 63, wave = threadIdx.x / 64;
  const int nch = H / 8;
  float acc_g[NCH][8], acc_b[NCH][8], acc_d[NCH][8], gam[NCH][8];
#pragma unroll
  for (int i = 0; i < NCH; ++i) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc_g[i][j] = acc_b[i][j] = acc_d[i][j] = gam[i][j] = 0.f;
    if (lane + 64 * i < nch) load8(gamma + (lane + 64 * i) * 8, gam[i]);
  }
  float ds_acc = 0.f, loss_acc = 0.f;

  constexpr int INF = NCH * sizeof(T) <= 4 ? 2 : 1;  // rows in flight: two when their loaded values fit the registers
  const int row_base = blockIdx.x * kLnBwdRows + wave * kLnBwdRowsPerWave;
#pragma unroll 1
  for (int pair = 0; pair < kLnBwdRowsPerWave; pair += INF) {
    float dy[INF][NCH][8], xh[INF][NCH][8], mean[INF], rstd[INF];
    // issue the loads of the rows in flight, then do the arithmetic
    Raw8<T> t_a[INF][NCH], t_b[INF][NCH], t_q[INF][NCH], t_v[INF][NCH], t_x[INF][NCH], t_r[INF][NCH];
#pragma unroll
    for (int k = 0; k < INF; ++k) {
      const int row = row_base + pair + k;
      const bool live = row < T_;
      mean[k] = live ? mu[row] : 0.f;
      rstd[k] = live ? rstd_in[row] : 0.f;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (live && c < nch) {
          const size_t off = (size_t)row * H + c * 8;
          if constexpr (HAS_A) t_a[k][i].load(d_a + off);
          if constexpr (HAS_L) t_b[k][i].load(loss_ref + off);
          if constexpr (HAS_Q) t_q[k][i].load(d_q + off);
          if ((HAS_Q && q.on) || HAS_L) t_v[k][i].load(a_q + off);
          t_x[k][i].load(x + off);
          t_r[k][i].load(r + off);
        }
      }
    }
#pragma unroll
    for (int k = 0; k < INF; ++k) {
      const int row = row_base + pair + k;
      if (row >= T_) continue;
      float s1 = 0.f, s2 = 0.f;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            float d = 0.f;
            if constexpr (HAS_A) d += t_a[k][i].get(j);
            if constexpr (HAS_L) {
              // Eq. 3 term of this layer: a_q holds the quantized module's output, loss_ref the full-precision one
              const float diff = t_v[k][i].get(j) - t_b[k][i].get(j);
              loss_acc += diff * diff;
              d += 2.0f * diff * loss_scale;
            }
            if constexpr (HAS_Q) {
              float t = t_q[k][i].get(j);
              if (q.on) {
                const float v = q_ratio_t<T>(t_v[k][i].get(j), q);
                const bool in = q_inside(v, q);
                ds_acc += t * (q_code(v, q) - (in ? v : 0.f));
                t = in ? t : 0.f;
              }
              d += t;
            }
            const float xhat = (t_x[k][i].get(j) + t_r[k][i].get(j) - mean[k]) * rstd[k];
            xh[k][i][j] = xhat;
            acc_g[i][j] += d * xhat;
            acc_b[i][j] += d;
            d *= gam[i][j];  // now d(xhat)
            dy[k][i][j] = d;
            s1 += d;
            s2 += d * xhat;
          }
        }
      }
      const float m1 = wave_sum(s1) / (float)H, m2 = wave_sum(s2) / (float)H;
#pragma unroll
      for (int i = 0; i < NCH; ++i) {
        const int c = lane + 64 * i;
        if (c < nch) {
          float o[8];
#pragma unroll
          for (int j = 0; j < 8; ++j) {
            o[j] = rstd[k] * (dy[k][i][j] - m1 - xh[k][i][j] * m2);
            acc_d[i][j] += round_to<T>(o[j]);
          }
          store8(dr + (size_t)row * H + c * 8, o);
        }
      }
    }
  }
  // the wavefronts meet in LDS: the upper half adds onto the lower half, whose sum in wavefront
  // order is the block's partial row
  ds_acc = wave_sum(ds_acc);
  loss_acc = wave_sum(loss_acc);
  float* mine = red + (size_t)(wave % HALF) * 3 * H;
  float* dsv = red + (size_t)HALF * 3 * H;
  if (lane == 0) { dsv[wave] = ds_acc; dsv[kLnBwdWaves + wave] = loss_acc; }
  if (wave >= HALF) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        store8(mine + c * 8, acc_g[i]);
        store8(mine + H + c * 8, acc_b[i]);
        store8(mine + 2 * H + c * 8, acc_d[i]);
      }
    }
  }
  __syncthreads();
  if (wave < HALF) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int c = lane + 64 * i;
      if (c < nch) {
        float t[8];
        load8(mine + c * 8, t);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc_g[i][j] += t[j];
        load8(mine + H + c * 8, t);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc_b[i][j] += t[j];
        load8(mine + 2 * H + c * 8, t);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc_d[i][j] += t[j];
        store8(mine + c * 8, acc_g[i]);
        store8(mine + H + c * 8, acc_b[i]);
        store8(mine + 2 * H + c * 8, acc_d[i]);
      }
    }
  }
  __syncthreads();
  const int width = 3 * H + 2;
  float* out = partials + (size_t)blockIdx.x * width;
  for (int c = threadIdx.x; c < 3 * H; c += blockDim.x) {
    float t = red[c];
#pragma unroll
    for (int w = 1; w < HALF; ++w) t += red[(size_t)w * 3 * H + c];
    out[c] = t;
  }
  if (threadIdx.x == 0) {
    float t = 0.f, tl = 0.f;
    for (int w = 0; w < kLnBwdWaves; ++w) { t += dsv[w]; tl += dsv[kLnBwdWaves + w]; }
    out[3 * H] = t;
    out[3 * H + 1] = tl;
  }
}
int ln_bwd(int dt, const void* d_a, const void* d_q, const void* a_q, QArg q, const void* x, const void* r,
           const float* mu, const float* rstd, const float* gamma, void* dr, float* partials, int T_, int H, hipStream_t st,
           const void* loss_ref, float loss_scale) {
  const int g = ln_bwd_parts(T_);
  const size_t lds = ((size_t)(kLnBwdWaves / 2) * 3 * H + 2 * kLnBwdWaves) * sizeof(float);
#define MREM_LN_BWD_V(NCH, A, Q, L)                                                                                                 \
  MREM_DISPATCH(dt, if (lds > 48 * 1024) (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&ln_bwd_k<T, NCH, A, Q, L>),              \
                                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);                \
                    MREM_LAUNCH((ln_bwd_k<T, NCH, A, Q, L>), dim3(g), dim3(64 * kLnBwdWaves), lds, st, (const T*)d_a, (const T*)d_q,    \
                                       (const T*)a_q, q, (const T*)x, (const T*)r, mu, rstd, gamma, (T*)dr, partials, T_, H,              \
                                       (const T*)loss_ref, loss_scale))
#define MREM_LN_BWD(NCH)                                                 \
  do {                                                                   \
    const int v = (d_a ? 1 : 0) | (d_q ? 2 : 0) | (loss_ref ? 4 : 0);    \
    switch (v) {                                                         \
      case 0: MREM_LN_BWD_V(NCH, false, false, false); break;            \
      case 1: MREM_LN_BWD_V(NCH, true, false, false); break;             \
      case 2: MREM_LN_BWD_V(NCH, false, true, false); break;             \
      case 3: MREM_LN_BWD_V(NCH, true, true, false); break;              \
      case 4: MREM_LN_BWD_V(NCH, false, false, true); break;             \
      case 5: MREM_LN_BWD_V(NCH, true, false, true); break;              \
      case 6: MREM_LN_BWD_V(NCH, false, true, true); break;              \
      default: MREM_LN_BWD_V(NCH, true, true, true); break;              \
    }                                                                    \
  } while (0)
  if (H <= 512) MREM_LN_BWD(1);
  else if (H <= 1024) MREM_LN_BWD(2);
  else MREM_LN_BWD(4);
#undef MREM_LN_BWD
#undef MREM_LN_BWD_V
  return g;
}

// ------------------------------------------------------------------------------
// second stage of the two-stage reductions (fixed order => run-to-run identical).
// All first-stage kernels of a backward pass leave their partial sums in the workspace;
// one launch of this kernel then finishes up to kMaxReduceJobs of them.
// ------------------------------------------------------------------------------
struct ReduceJobTable {
  ReduceJob j[kMaxReduceJobs];
  int unit_start[kMaxReduceJobs + 1];  // prefix sums of work units (16 columns each; 1 for a scalar)
  int n;
};
__global__ __launch_bounds__(256) void reduce_jobs_k(ReduceJobTable t) {
  // 256 threads = 16 columns x 16 groups of partial rows; the group sums are added in group
  // order, so the result does not depend on scheduling.
  __shared__ float red[16][17];
  __shared__ float sred[17];
  int ji = 0;
  while (ji + 1 < t.n && (int)blockIdx.x >= t.unit_start[ji + 1]) ++ji;
  const ReduceJob jb = t.j[ji];
  const int unit = blockIdx.x - t.unit_start[ji];
  if (jb.len == 1) {
    float v = 0.f;
    for (int p = threadIdx.x; p < jb.nparts; p += blockDim.x) v += jb.partials[(size_t)p * jb.width + jb.begin];
    v = block_sum(v, sred);
    if (threadIdx.x == 0) jb.out[0] = v * jb.scale;
    return;
  }
  const int col = threadIdx.x & 15, grp = threadIdx.x >> 4;
  const int c = unit * 16 + col;
  float t0 = 0.f, t1 = 0.f;
  if (c < jb.len) {
    const float* src = jb.partials + jb.begin + c;
    int p = grp;
    for (; p + 16 < jb.nparts; p += 32) {
      t0 += src[(size_t)p * jb.width];
      t1 += src[(size_t)(p + 16) * jb.width];
    }
    for (; p < jb.nparts; p += 16) t0 += src[(size_t)p * jb.width];
  }
  red[grp][col] = t0 + t1;
  __syncthreads();
  if (grp == 0 && c < jb.len) {
    float v = 0.f;
#pragma unroll
    for (int g = 0; g < 16; ++g) v += red[g][col];
    jb.out[c] = v * jb.scale;
  }
}
void reduce_jobs(const ReduceJob* jobs, int njobs, hipStream_t st) {
  for (int first = 0; first < njobs; first += kMaxReduceJobs) {
    ReduceJobTable t;
    t.n = njobs - first < kMaxReduceJobs ? njobs - first : kMaxReduceJobs;
    int units = 0;
    for (int i = 0; i < t.n; ++i) {
      t.j[i] = jobs[first + i];
      t.unit_start[i] = units;
      units += t.j[i].len == 1 ? 1 : (t.j[i].len + 15) / 16;
    }
    t.unit_start[t.n] = units;
    MREM_LAUNCH(reduce_jobs_k, dim3(units), dim3(256), 0, st, t);
  }
}

__global__ void loss_total_k(float* loss_out, int n_layers, int* nonfinite_flag) {
  if (threadIdx.x == 0 && blockIdx.x == 0) {
    float t = 0.f;
    for (int l = 0; l < n_layers; ++l) t += loss_out[1 + l];
    loss_out[0] = t;
    // a NaN or infinity anywhere in the layer outputs reaches its layer's squared-error sum
    if (nonfinite_flag && !(fabsf(t) <= FLT_MAX)) *nonfinite_flag = 1;
  }
}
void loss_total(float* loss_out, int n_layers, int* nonfinite_flag, hipStream_t st) {
  MREM_LAUNCH(loss_total_k, dim3(1), dim3(64), 0, st, loss_out, n_layers, nonfinite_flag);
}

__global__ void fill_k(float* p, float v, int64_t n) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
void fill_f32(float* p, float v, int64_t n, hipStream_t st) {
  int g = (int)((n + 255) / 256);
  if (g > 4096) g = 4096;
  if (g < 1) g = 1;
  MREM_LAUNCH(fill_k, dim3(g), dim3(256), 0, st, p, v, n);
}
typedef float f32x4_t __attribute__((ext_vector_type(4)));
struct FillTable {
  FillRegion r[kMaxFillRegions];
};
__global__ void zero_regions_k(FillTable t) {
  const FillRegion rg = t.r[blockIdx.y];
  f32x4_t* p4 = reinterpret_cast<f32x4_t*>(rg.p);  // regions start 16-byte aligned (checked on the host)
  const int64_t n4 = rg.n / 4;
  const f32x4_t z = {0.f, 0.f, 0.f, 0.f};
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n4; i += (int64_t)gridDim.x * blockDim.x) p4[i] = z;
  if (blockIdx.x == 0 && threadIdx.x < (rg.n & 3)) rg.p[n4 * 4 + threadIdx.x] = 0.f;
}
void zero_regions(const FillRegion* regions, int count, hipStream_t st) {
  for (int c0 = 0; c0 < count; c0 += kMaxFillRegions) {
    FillTable t;
    const int nr = count - c0 < kMaxFillRegions ? count - c0 : kMaxFillRegions;
    int64_t longest = 1;
    for (int k = 0; k < nr; ++k) {
      t.r[k] = regions[c0 + k];
      if ((reinterpret_cast<uintptr_t>(t.r[k].p) & 15) != 0) {  // unaligned start: plain fill
        fill_f32(t.r[k].p, 0.f, t.r[k].n, st);
        t.r[k].n = 0;
      }
      if (t.r[k].n > longest) longest = t.r[k].n;
    }
    int gx = (int)((longest / 4 + 255) / 256);
    if (gx > 2048) gx = 2048;
    if (gx < 1) gx = 1;
    MREM_LAUNCH(zero_regions_k, dim3(gx, nr), dim3(256), 0, st, t);
  }
}

// Squared distance of two stored tensors and its gradient (the reconstruction objective of a single matrix
// product, Section 3.2, Eq. 2): dy = 2 * scale * (yq - yfp), partials[block] = sum (yq - yfp)^2
template <class T>
__global__ void mse_grad_k(const T* __restrict__ yq, const T* __restrict__ yfp, T* __restrict__ dy, int64_t nchunks, float scale,
                           float* __restrict__ partials) {
  __shared__ float red[17];
  float acc = 0.f;
  for (int64_t c = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; c < nchunks; c += (int64_t)gridDim.x * blockDim.x) {
    float a[8], b[8];
    load8(yq + c * 8, a);
    load8(yfp + c * 8, b);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const float d = a[j] - b[j];
      acc += d * d;
      a[j] = 2.0f * d * scale;
    }
    store8(dy + c * 8, a);
  }
  acc = block_sum(acc, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = acc;
}
int mse_grad(int dt, const void* yq, const void* yfp, void* dy, int64_t n, float scale, float* partials, hipStream_t st) {
  const int g = ew_grid(n);
  MREM_DISPATCH(dt, MREM_LAUNCH(mse_grad_k<T>, dim3(g), dim3(256), 0, st, (const T*)yq, (const T*)yfp, (T*)dy, n / 8, scale, partials));
  return g;
}

// Eq. 4: out = wa * a + wb * b
template <class T>
__global__ void axpby_k(const T* __restrict__ a, const T* __restrict__ b, float wa, float wb, T* __restrict__ out, int64_t n) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    stf(out, i, wa * ldf(a, i) + wb * ldf(b, i));
}
void axpby(int dt, const void* a, const void* b, float wa, float wb, void* out, int64_t n, hipStream_t st) {
  int g = (int)((n + 255) / 256);
  if (g > 4096) g = 4096;
  if (g < 1) g = 1;
  MREM_DISPATCH(dt, MREM_LAUNCH(axpby_k<T>, dim3(g), dim3(256), 0, st, (const T*)a, (const T*)b, wa, wb, (T*)out, n));
}

template <class T>
__global__ void convert_k(const float* __restrict__ src, T* __restrict__ dst, int64_t n) {
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) stf(dst, i, src[i]);
}
void convert_f32(int dt, const float* src, void* dst, int64_t n, hipStream_t st) {
  int g = (int)((n + 255) / 256);
  if (g > 8192) g = 8192;
  if (g < 1) g = 1;
  MREM_DISPATCH(dt, MREM_LAUNCH(convert_k<T>, dim3(g), dim3(256), 0, st, src, (T*)dst, n));
}

// ------------------------------------------------------------------------------
// weight quantizer (Eq. 1 per output channel)
// ------------------------------------------------------------------------------
__device__ __forceinline__ float row_step_init(const float* __restrict__ wr, int64_t K, float qp, float* red) {
  float m = 0.f;
  for (int64_t k = threadIdx.x; k < K; k += blockDim.x) m = fmaxf(m, fabsf(wr[k]));
  m = block_max(m, red);
  float s = __fdiv_rn(m, qp);
  if (!(s > 0.f)) s = FLT_MIN;
  return s;
}

__global__ void weight_quantize_i8_k(const float* __restrict__ w, float* __restrict__ scale, int8_t* __restrict__ codes, int64_t K,
                                     float qp, int init_scale) {
  __shared__ float red[17];
  const int64_t n = blockIdx.x;
  const float* wr = w + n * K;
  float s;
  if (init_scale) {
    s = row_step_init(wr, K, qp, red);
    if (threadIdx.x == 0) scale[n] = s;
  } else {
    s = scale[n];
  }
  for (int64_t k = threadIdx.x; k < K; k += blockDim.x) {
    const float v = __fdiv_rn(wr[k], s);
    codes[n * K + k] = (int8_t)(int)rintf(fminf(fmaxf(v, -qp), qp));
  }
}
// one step for the whole tensor: a single block finds max |w| (initial step), every block then uses scale[0]
__global__ void tensor_step_init_k(const float* __restrict__ w, float* __restrict__ scale, int64_t n, float qp) {
  __shared__ float red[17];
  float m = 0.f;
  for (int64_t i = threadIdx.x; i < n; i += blockDim.x) m = fmaxf(m, fabsf(w[i]));
  m = block_max(m, red);
  float s = __fdiv_rn(m, qp);
  if (!(s > 0.f)) s = FLT_MIN;
  if (threadIdx.x == 0) scale[0] = s;
}
__global__ void tensor_quantize_i8_k(const float* __restrict__ w, const float* __restrict__ scale, int8_t* __restrict__ codes, int64_t n,
                                     float qp) {
  const float s = scale[0];
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
    codes[i] = (int8_t)(int)rintf(fminf(fmaxf(__fdiv_rn(w[i], s), -qp), qp));
}
void weight_quantize_i8(const float* w, float* scale, int8_t* codes, int64_t N, int64_t K, int bits, int per_channel, int init_scale,
                        hipStream_t st) {
  const float qp = (float)((1 << (bits - 1)) - 1);
  if (per_channel) {
    MREM_LAUNCH(weight_quantize_i8_k, dim3((unsigned)N), dim3(256), 0, st, w, scale, codes, K, qp, init_scale);
    return;
  }
  const int64_t n = N * K;
  if (init_scale) MREM_LAUNCH(tensor_step_init_k, dim3(1), dim3(1024), 0, st, w, scale, n, qp);
  int g = (int)((n + 255) / 256);
  if (g > 8192) g = 8192;
  MREM_LAUNCH(tensor_quantize_i8_k, dim3(g), dim3(256), 0, st, w, (const float*)scale, codes, n, qp);
}

__global__ void weight_step_init_k(const float* __restrict__ w, float* __restrict__ scale, int64_t K, float qp) {
  __shared__ float red[17];
  const float s = row_step_init(w + (int64_t)blockIdx.x * K, K, qp, red);
  if (threadIdx.x == 0) scale[blockIdx.x] = s;
}
void weight_step_init(const float* w, float* scale, int64_t N, int64_t K, int bits, hipStream_t st) {
  const float qp = (float)((1 << (bits - 1)) - 1);
  MREM_LAUNCH(weight_step_init_k, dim3((unsigned)N), dim3(256), 0, st, w, scale, K, qp);
}

__global__ void tie_steps_max_k(float* __restrict__ scale, int64_t N) {
  __shared__ float red[17];
  float m = 0.f;
  for (int64_t i = threadIdx.x; i < N; i += blockDim.x) m = fmaxf(m, scale[i]);
  m = block_max(m, red);
  for (int64_t i = threadIdx.x; i < N; i += blockDim.x) scale[i] = m;
}
void tie_steps_max(float* scale, int64_t N, hipStream_t st) { MREM_LAUNCH(tie_steps_max_k, dim3(1), dim3(256), 0, st, scale, N); }

// codes (integer-valued, storage type), dequantized weights s*code (same layout), and
// zcorr[n] = s[n] * sum_k code (sum_k of the stored weight when the quantizers are off); one block per output channel, all matrices of a table in one launch
struct WeightJobTable {
  WeightJob job[kMaxMatrixJobs];
  int first_row[kMaxMatrixJobs + 1];
  int njobs;
};
template <class T>
__global__ __launch_bounds__(128) void weight_codes_k(WeightJobTable tab, float qp, int on) {
  __shared__ float red[17];
  int ji = 0;
  while (ji + 1 < tab.njobs && (int)blockIdx.x >= tab.first_row[ji + 1]) ++ji;
  const WeightJob& jb = tab.job[ji];
  const int n = blockIdx.x - tab.first_row[ji], K = jb.K;
  const float* __restrict__ w = jb.w;
  T* __restrict__ codes = reinterpret_cast<T*>(jb.codes);
  T* __restrict__ what = reinterpret_cast<T*>(jb.what);
  const float s = on ? jb.sw[n] : 1.f;
  float acc = 0.f;
  const size_t row = (size_t)n * K;
  for (int k = threadIdx.x * 8; k < K; k += blockDim.x * 8) {
    float x[8], c[8];
    load8(w + row + k, x);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      c[j] = x[j];
      if (on) { c[j] = rintf(fminf(fmaxf(__fdiv_rn(x[j], s), -qp), qp)); acc += c[j]; x[j] = s * c[j]; }
      else acc += round_to<T>(x[j]);  // quantizers off: the stored weights themselves are the operand
    }
    if (codes) store8(codes + row + k, c);
    if (jb.codes8) store8_i8(jb.codes8 + row + k, c, 0.f);
    if (what) store8(what + row + k, x);
  }
  acc = block_sum(acc, red);
  // s * sum_k code (s = 1 with the weight quantizers off): what the offset z of an asymmetric input
  // quantizer multiplies in the product's epilogue, x^ = s_a q + z (Section 3.1)
  if (threadIdx.x == 0) jb.zcorr[n] = s * acc;
}
void weight_prepare(int dt, const WeightJob* jobs, int njobs, int bits, hipStream_t st) {
  const int on = bits > 0;
  const float qp = on ? (float)((1 << (bits - 1)) - 1) : 0.f;
  for (int j0 = 0; j0 < njobs; j0 += kMaxMatrixJobs) {
    WeightJobTable tab;
    tab.njobs = njobs - j0 < kMaxMatrixJobs ? njobs - j0 : kMaxMatrixJobs;
    int rows = 0;
    for (int j = 0; j < tab.njobs; ++j) { tab.job[j] = jobs[j0 + j]; tab.first_row[j] = rows; rows += jobs[j0 + j].N; }
    tab.first_row[tab.njobs] = rows;
    if (rows == 0) continue;
    MREM_DISPATCH(dt, MREM_LAUNCH(weight_codes_k<T>, dim3(rows), dim3(128), 0, st, tab, qp, on));
  }
}

// ------------------------------------------------------------------------------
// calibration reductions
// ------------------------------------------------------------------------------
template <class T>
__global__ void absminmax_k(const T* __restrict__ a, int rows, int cols, int ld, int gelu, float* __restrict__ partials) {
  __shared__ float red[17];
  float amax = 0.f, mn = FLT_MAX, mx = -FLT_MAX;
  const int64_t n = (int64_t)rows * cols;
  for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) {
    const int64_t r = i / cols, c = i - r * cols;
    float v = ldf(a, (size_t)(r * ld + c));
    if (gelu) v = gelu_t<T>(v);
    amax = fmaxf(amax, fabsf(v));
    mn = fminf(mn, v);
    mx = fmaxf(mx, v);
  }
  amax = block_max(amax, red);
  mx = block_max(mx, red);
  mn = -block_max(-mn, red);
  if (threadIdx.x == 0) {
    partials[blockIdx.x * 3 + 0] = amax;
    partials[blockIdx.x * 3 + 1] = mn;
    partials[blockIdx.x * 3 + 2] = mx;
  }
}
int absminmax(int dt, const void* a, int rows, int cols, int ld, int gelu, float* partials, hipStream_t st) {
  int64_t n = (int64_t)rows * cols;
  int g = (int)((n + 255) / 256);
  if (g > 1024) g = 1024;
  if (g < 1) g = 1;
  MREM_DISPATCH(dt, MREM_LAUNCH(absminmax_k<T>, dim3(g), dim3(256), 0, st, (const T*)a, rows, cols, ld, gelu, partials));
  return g;
}
__global__ void calib_finalize_k(const float* __restrict__ partials, int nparts, int mode, float qp, float* s_out, float* z_out) {
  __shared__ float red[17];
  float amax = 0.f, mn = FLT_MAX, mx = -FLT_MAX;
  for (int p = threadIdx.x; p < nparts; p += blockDim.x) {
    amax = fmaxf(amax, partials[p * 3]);
    mn = fminf(mn, partials[p * 3 + 1]);
    mx = fmaxf(mx, partials[p * 3 + 2]);
  }
  amax = block_max(amax, red);
  mx = block_max(mx, red);
  mn = -block_max(-mn, red);
  if (threadIdx.x == 0) {
    float s, z = 0.f;
    if (mode == 0) s = __fdiv_rn(amax, qp);
    else if (mode == 1) s = __fdiv_rn(mx, qp);
    else { z = mn; s = __fdiv_rn(__fsub_rn(mx, z), qp); }
    if (!(s > 0.f)) s = FLT_MIN;
    *s_out = s;
    *z_out = z;
  }
}
void calib_finalize(const float* partials, int nparts, int mode, float qp, float* s_out, float* z_out, hipStream_t st) {
  MREM_LAUNCH(calib_finalize_k, dim3(1), dim3(256), 0, st, partials, nparts, mode, qp, s_out, z_out);
}

// ------------------------------------------------------------------------------
// AdamW (decoupled weight decay, bias-corrected), Section 5.1.2
// ------------------------------------------------------------------------------
__device__ __forceinline__ float adam_one(float p, float g, float& m, float& v, const AdamArg& a) {
  m = a.beta1 * m + (1.f - a.beta1) * g;
  v = a.beta2 * v + (1.f - a.beta2) * g * g;
  const float mhat = m / a.bc1, vhat = v / a.bc2;
  return p - a.lr * (mhat / (sqrtf(vhat) + a.eps) + a.wd * p);
}

// One block per output channel.  g_w holds d(loss)/d(w_hat) on entry; the
// straight-through mask and the step-size gradient (row reduction) are formed
// here, from the weights and the step before their update.

struct AdamJobTable {
  AdamJob job[kMaxMatrixJobs];
  int first_row[kMaxMatrixJobs + 1];
  int njobs;
};
__global__ __launch_bounds__(256) void adam_matrix_k(AdamJobTable tab, float qp, int on, AdamArg a, int write_grads, int tied) {
  __shared__ float red[17];
  int ji = 0;
  while (ji + 1 < tab.njobs && (int)blockIdx.x >= tab.first_row[ji + 1]) ++ji;
  const AdamJob& jb = tab.job[ji];
  const int n = blockIdx.x - tab.first_row[ji], K = jb.K;
  float* __restrict__ w = jb.w;
  float* __restrict__ g_w = jb.g_w;
  float* __restrict__ m_w = jb.m_w;
  float* __restrict__ v_w = jb.v_w;
  const float s = on ? jb.sw[n] : 1.f;
  // offset term of an asymmetric input quantizer: d(loss)/d(w_hat[n,:]) += z * sum_t dy[t,n]
  const float zterm = jb.z_in ? (*jb.z_in) * jb.db[n] : 0.f;
  const bool store_g = write_grads && (on || jb.z_in);
  float acc = 0.f;
  const size_t row = (size_t)n * K;
  for (int k = threadIdx.x * 4; k < K; k += blockDim.x * 4) {
    const size_t i = row + k;
    f32x4_t x = *reinterpret_cast<const f32x4_t*>(w + i);
    f32x4_t g = *reinterpret_cast<const f32x4_t*>(g_w + i);
    f32x4_t m = *reinterpret_cast<const f32x4_t*>(m_w + i);
    f32x4_t vv = *reinterpret_cast<const f32x4_t*>(v_w + i);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float gj = g[j] + zterm;
      g[j] = gj;
      if (on) {
        const float v = __fdiv_rn(x[j], s);
        const bool in = (v >= -qp) && (v <= qp);
        const float c = rintf(fminf(fmaxf(v, -qp), qp));
        acc += gj * (c - (in ? v : 0.f));
        gj = in ? gj : 0.f;
        g[j] = gj;
      }
      float mj = m[j], vj = vv[j];
      x[j] = adam_one(x[j], gj, mj, vj, a);
      m[j] = mj;
      vv[j] = vj;
    }
    *reinterpret_cast<f32x4_t*>(w + i) = x;
    *reinterpret_cast<f32x4_t*>(m_w + i) = m;
    *reinterpret_cast<f32x4_t*>(v_w + i) = vv;
    if (store_g) *reinterpret_cast<f32x4_t*>(g_w + i) = g;
  }
  if (on) {
    acc = block_sum(acc, red);
    if (threadIdx.x == 0 && tied) {
      jb.g_sw[n] = acc;  // summed over the rows and applied by adam_tied_steps_k
    } else if (threadIdx.x == 0) {
      if (write_grads) jb.g_sw[n] = acc;
      AdamArg as = a;
      as.wd = 0.f;
      float m = jb.m_sw[n], vv = jb.v_sw[n];
      const float ns = adam_one(s, acc, m, vv, as);
      jb.sw[n] = fmaxf(ns, a.floor);
      jb.m_sw[n] = m;
      jb.v_sw[n] = vv;
    }
  } else if (write_grads && threadIdx.x == 0) {
    jb.g_sw[n] = 0.f;
  }
}
// one block per matrix: fixed-order sum of the rows' step gradients, AdamW on the one step, broadcast
__global__ __launch_bounds__(256) void adam_tied_steps_k(AdamJobTable tab, AdamArg a) {
  __shared__ float red[17];
  const AdamJob& jb = tab.job[blockIdx.x];
  float t = 0.f;
  for (int i = threadIdx.x; i < jb.N; i += blockDim.x) t += jb.g_sw[i];
  const float g = block_sum(t, red);
  AdamArg as = a;
  as.wd = 0.f;
  float m = jb.m_sw[0], vv = jb.v_sw[0];
  const float ns = fmaxf(adam_one(jb.sw[0], g, m, vv, as), a.floor);
  __syncthreads();  // every thread has read entry 0 before anyone overwrites it
  for (int i = threadIdx.x; i < jb.N; i += blockDim.x) {
    jb.sw[i] = ns;
    jb.m_sw[i] = m;
    jb.v_sw[i] = vv;
    jb.g_sw[i] = g;
  }
}
void adam_matrix(const AdamJob* jobs, int njobs, int bits, AdamArg a, int write_grads, int tied, hipStream_t st) {
  const int on = bits > 0;
  const float qp = on ? (float)((1 << (bits - 1)) - 1) : 0.f;
  for (int j0 = 0; j0 < njobs; j0 += kMaxMatrixJobs) {
    AdamJobTable tab;
    tab.njobs = njobs - j0 < kMaxMatrixJobs ? njobs - j0 : kMaxMatrixJobs;
    int rows = 0;
    for (int j = 0; j < tab.njobs; ++j) { tab.job[j] = jobs[j0 + j]; tab.first_row[j] = rows; rows += jobs[j0 + j].N; }
    tab.first_row[tab.njobs] = rows;
    if (rows == 0) continue;
    MREM_LAUNCH(adam_matrix_k, dim3(rows), dim3(256), 0, st, tab, qp, on, a, write_grads, (on && tied) ? 1 : 0);
    if (on && tied) MREM_LAUNCH(adam_tied_steps_k, dim3(tab.njobs), dim3(256), 0, st, tab, a);
  }
}

struct VecJobTable {
  VecJob job[kMaxVecJobs];
};
__global__ void adam_vector_k(float* __restrict__ p, const float* __restrict__ g, float* __restrict__ m, float* __restrict__ v,
                              VecJobTable tab, AdamArg a) {
  const VecJob jb = tab.job[blockIdx.y];
  for (int64_t k = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; k < jb.n; k += (int64_t)gridDim.x * blockDim.x) {
    const int64_t i = jb.off + k;
    float mm = m[i], vv = v[i];
    float np_ = adam_one(p[i], g[i], mm, vv, a);
    if (jb.clamp) np_ = fmaxf(np_, a.floor);
    p[i] = np_;
    m[i] = mm;
    v[i] = vv;
  }
}
void adam_vector(float* p, const float* g, float* m, float* v, const VecJob* jobs, int njobs, AdamArg a, hipStream_t st) {
  for (int j0 = 0; j0 < njobs; j0 += kMaxVecJobs) {
    VecJobTable tab;
    const int nj = njobs - j0 < kMaxVecJobs ? njobs - j0 : kMaxVecJobs;
    int64_t longest = 1;
    for (int j = 0; j < nj; ++j) { tab.job[j] = jobs[j0 + j]; if (jobs[j0 + j].n > longest) longest = jobs[j0 + j].n; }
    int gx = (int)((longest + 255) / 256);
    if (gx > 1024) gx = 1024;
    MREM_LAUNCH(adam_vector_k, dim3(gx, nj), dim3(256), 0, st, p, g, m, v, tab, a);
  }
}

}  // namespace mrem
