// Softmax attention on the matrix cores (v_mfma_f32_32x32x16_bf16) for head
// dimension 64, bf16 storage and 64 <= seq <= 384: forward, and the backward pass
// split into a query-major and a key-major kernel.  Operands are quantizer codes
// (Section 3.1: Q, K, V and the softmax probabilities are quantized before their
// products), so Q*K^T and P*V are exact integer products in fp32.
//
// Layout trick used throughout: the score tile is computed transposed,
// D[key][query] = K_tile * Q_tile^T, so that in the 32x32 accumulator layout a lane
// owns ONE query (lane % 32) and 16 of the 32 keys of the tile; the other 16 keys sit
// in lane ^ 32.  Row-wise softmax statistics then need a single cross-lane exchange,
// and the accumulator registers already have the layout of the B operand of the next
// product (contraction over keys), with the key order fixed by `key_of`.
//
// All tiles (K, V, Q, dC) sit row-major in LDS as they do in memory; where a product
// needs an operand with the contraction index along the rows, the fragment is gathered
// with the transposing LDS read (ds_read_tr16_b64), see `ld_frag_tr`.
#include "mrem_common.h"
#include "mrem_kernels.h"

namespace mrem {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));

constexpr int kD = 64;            // head dimension handled here
constexpr int kRowStride = 72;    // elements per row of a row-major LDS tile (144 bytes)

// key (row of the transposed score tile) held in accumulator register i of a lane in half h
__device__ __forceinline__ int key_of(int t, int i, int h) { return 32 * t + 8 * (i >> 2) + 4 * h + (i & 3); }

struct FwdScales {
  float qk, sp, sv, p_qp;
  int p_on;
  float rsp;  // correctly rounded 1 / sp
};
// x / d from rd = fl(1 / d): t = fl(x * rd), then t + fl(x - d * t) * rd with fused multiply-adds.
// The residual is exact and, rd being correctly rounded, the result is the correctly rounded
// quotient (the residual-correction step of FMA division), so this matches an IEEE division while
// one reciprocal serves a whole row (softmax sums) or tensor (step sizes).
__device__ __forceinline__ float div_by(float x, float d, float rd) {
  const float t = __fmul_rn(x, rd);
  return __fmaf_rn(__fmaf_rn(-d, t, x), rd, t);
}
__device__ __forceinline__ FwdScales load_fwd_scales(const AttnQ& a) {
  FwdScales s;
  const float sq = a.q.on ? *a.q.s : 1.f, sk = a.k.on ? *a.k.s : 1.f;
  s.sp = a.p.on ? *a.p.s : 1.f;
  s.sv = a.v.on ? *a.v.s : 1.f;
  s.qk = sq * sk / sqrtf((float)kD);
  s.p_on = a.p.on;
  s.p_qp = a.p.qp;
  s.rsp = __fdiv_rn(1.0f, s.sp);
  return s;
}

// stage rows [0, S) of a [S, 64] slice (row stride ld elements) row-major into LDS, zero rows up to s_pad
__device__ __forceinline__ void stage_rows(const bf16_t* __restrict__ src, int ld, int S, int s_pad, bf16_t* dst) {
  for (int q = threadIdx.x; q < s_pad * 8; q += blockDim.x) {
    const int row = q >> 3, ch = q & 7;
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (row < S) v = *reinterpret_cast<const u32x4_t*>(src + (size_t)row * ld + ch * 8);
    *reinterpret_cast<u32x4_t*>(dst + row * kRowStride + ch * 8) = v;
  }
}
__device__ __forceinline__ bf16x8_t ld_frag(const bf16_t* p) { return *reinterpret_cast<const bf16x8_t*>(p); }

// MFMA operand fragment gathered down the rows of a row-major LDS tile (pitch kRowStride) with the
// transposing LDS read (ds_read_b64_tr_b16): lane l receives, for column c0 + l%32, rows
// r_first + 0..3 and r_second + 0..3 (the caller picks the two row bases for its half l/32).  In a
// group of 16 lanes, lane s supplies the 8-byte chunk of row s/4, columns 4*(s%4)..+3, and receives
// column s of the four rows.  Lets K, V, Q and dC stay row-major in LDS (16-byte conflict-free stores)
// where the products contract over their row index.
typedef short s16x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ bf16x8_t ld_frag_tr(const bf16_t* tile, int c0, int r_first, int r_second, int lane) {
  const int g = lane >> 4, s = lane & 15;
  const bf16_t* p = tile + (s >> 2) * kRowStride + c0 + 16 * (g & 1) + 4 * (s & 3);
  union { bf16x8_t v; s16x4_t h[2]; } u;
  u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p + r_first * kRowStride));
  u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4_t*)(p + r_second * kRowStride));
  return u.v;
}

__device__ __forceinline__ void store4(bf16_t* p, float a, float b, float c, float d) {
  bf16x4_t v = {static_cast<bf16_t>(a), static_cast<bf16_t>(b), static_cast<bf16_t>(c), static_cast<bf16_t>(d)};
  *reinterpret_cast<bf16x4_t*>(p) = v;
}

// ------------------------------------------------------------------------------
// forward: one block = up to 128 queries of one (batch, head); one wavefront = 32 queries
// ------------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(256) void attn_fwd_mfma_k(const bf16_t* __restrict__ codes, bf16_t* __restrict__ ctx,
                                                       bf16_t* __restrict__ ctx_codes, AttnQ aq, const int32_t* __restrict__ seqlens,
                                                       int S, int H, int nt, float* __restrict__ pmax_rows, float* __restrict__ stat_m,
                                                       float* __restrict__ stat_l, int8_t* __restrict__ ctx_codes8) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int s_pad = 32 * nt;
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem_raw);  // [s_pad][72]
  bf16_t* Vs = Ks + s_pad * kRowStride;              // [s_pad][72]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  const int ld = 3 * H;
  const bf16_t* base = codes + (size_t)b * S * ld + h * kD;
  const int len = seqlens ? seqlens[b] : S;
  const FwdScales sc = load_fwd_scales(aq);

  stage_rows(base + H, ld, S, s_pad, Ks);
  stage_rows(base + 2 * H, ld, S, s_pad, Vs);
  __syncthreads();

  const int q0 = blockIdx.x * 128 + wave * 32;
  if (q0 >= S) return;
  const int q = q0 + (lane & 31);
  const int qc = q < S ? q : S - 1;
  bf16x8_t qf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) qf[kk] = ld_frag(base + (size_t)qc * ld + (kk * 2 + half) * 8);

  f32x16_t sacc[NT];
  float mx = -INFINITY;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (t < nt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[t][r] = 0.f;
      const bf16_t* kp = Ks + (32 * t + (lane & 31)) * kRowStride + half * 8;
#pragma unroll
      for (int kk = 0; kk < 4; ++kk) sacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(kp + kk * 16), qf[kk], sacc[t], 0, 0, 0);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float a = key_of(t, r, half) < len ? __fmul_rn(sacc[t][r], sc.qk) : -INFINITY;
        sacc[t][r] = a;
        mx = fmaxf(mx, a);
      }
    }
  }
  mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
  float sum = 0.f;
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (t < nt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = sacc[t][r] == -INFINITY ? 0.f : __expf(__fsub_rn(sacc[t][r], mx));
        sacc[t][r] = e;
        sum += e;
      }
    }
  }
  sum += __shfl_xor(sum, 32, 64);
  const size_t stat_idx = ((size_t)b * nh + h) * S + q;
  if (half == 0 && q < S) {
    if (stat_m) { stat_m[stat_idx] = mx; stat_l[stat_idx] = sum; }
    if (pmax_rows) pmax_rows[stat_idx] = 1.0f / sum;  // the largest exponential of a row is exp(0) = 1
  }

  f32x16_t oacc[2];
#pragma unroll
  for (int et = 0; et < 2; ++et)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[et][r] = 0.f;
  const float rsum = __fdiv_rn(1.0f, sum);
#pragma unroll
  for (int t = 0; t < NT; ++t) {
    if (t < nt) {
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        bf16x8_t pf;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const float p = div_by(sacc[t][8 * s + i], sum, rsum);
          const float c = sc.p_on ? rintf(fminf(fmaxf(div_by(p, sc.sp, sc.rsp), 0.f), sc.p_qp)) : p;
          pf[i] = static_cast<bf16_t>(c);
        }
        // V^T fragments: keys in the order the accumulator registers of the score tile hold them
        const int k0 = 32 * t + 16 * s + 4 * half;
        oacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_tr(Vs, 0, k0, k0 + 8, lane), pf, oacc[0], 0, 0, 0);
        oacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_tr(Vs, 32, k0, k0 + 8, lane), pf, oacc[1], 0, 0, 0);
      }
    }
  }
  if (q < S) {
    const float os = sc.sp * sc.sv;
    QuantParam qc5 = {aq.c.on ? *aq.c.s : 1.f, 0.f, aq.c.qn, aq.c.qp, aq.c.on, 0.f};
    qc5.rs = quant_reciprocal(qc5.s);
    const size_t orow = ((size_t)b * S + q) * H + h * kD;
#pragma unroll
    for (int et = 0; et < 2; ++et)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        float o[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) o[i] = oacc[et][4 * g + i] * os;
        const int e = 32 * et + 8 * g + 4 * half;
        store4(ctx + orow + e, o[0], o[1], o[2], o[3]);
        if (ctx_codes) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            const float r = round_to<bf16_t>(o[i]);
            o[i] = qc5.on ? q_code(q_ratio_fma(r, qc5), qc5) : r;
          }
          store4(ctx_codes + orow + e, o[0], o[1], o[2], o[3]);
          if (ctx_codes8) {
            const unsigned pk = ((unsigned)(int)o[0] & 0xffu) | (((unsigned)(int)o[1] & 0xffu) << 8) | (((unsigned)(int)o[2] & 0xffu) << 16) |
                                (((unsigned)(int)o[3] & 0xffu) << 24);
            *reinterpret_cast<unsigned*>(ctx_codes8 + orow + e) = pk;
          }
        }
      }
  }
}

// ------------------------------------------------------------------------------
// backward, query-major part: for 32 queries per wavefront recomputes P from the saved
// row statistics, forms dP^ = dC * V^T, applies the straight-through rule of the
// probability quantizer, the softmax backward, and dQ^ = dA * K^.  Writes the transposed
// tiles P^T[key][query] and dA^T[key][query] (bf16) for the key-major kernel.
// NT > 0: rows of at most NT key tiles, kept in registers; NT = 0: any length, tiles formed twice.
// ------------------------------------------------------------------------------
template <int NT>
__global__ __launch_bounds__(256) void attn_bwd_q_mfma_k(const bf16_t* __restrict__ codes, const bf16_t* __restrict__ dctx,
                                                         bf16_t* __restrict__ d_qkvh, AttnQ aq, const int32_t* __restrict__ seqlens, int S,
                                                         int H, int nt, const float* __restrict__ stat_m, const float* __restrict__ stat_l,
                                                         bf16_t* __restrict__ pt_out, bf16_t* __restrict__ dat_out,
                                                         float* __restrict__ ds_parts) {
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  const int s_pad = 32 * nt;
  bf16_t* Ks = reinterpret_cast<bf16_t*>(smem_raw);  // [s_pad][72]
  bf16_t* Vs = Ks + s_pad * kRowStride;              // [s_pad][72]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  const int ld = 3 * H;
  const bf16_t* base = codes + (size_t)b * S * ld + h * kD;
  const int len = seqlens ? seqlens[b] : S;
  const FwdScales sc = load_fwd_scales(aq);
  const float sk = aq.k.on ? *aq.k.s : 1.f;

  stage_rows(base + H, ld, S, s_pad, Ks);
  stage_rows(base + 2 * H, ld, S, s_pad, Vs);
  __syncthreads();

  const int q0 = blockIdx.x * 128 + wave * 32;
  const int part_idx = (((b * nh + h) * gridDim.x) + blockIdx.x) * 4 + wave;
  if (q0 >= s_pad) {
    ds_parts[part_idx] = 0.f;
    return;
  }
  const int q = q0 + (lane & 31);
  const bool qvalid = q < S;
  const int qc = qvalid ? q : S - 1;
  bf16x8_t qf[4], cf[4];
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) {
    qf[kk] = ld_frag(base + (size_t)qc * ld + (kk * 2 + half) * 8);
    cf[kk] = ld_frag(dctx + ((size_t)b * S + qc) * H + h * kD + (kk * 2 + half) * 8);
  }
  const size_t stat_idx = ((size_t)b * nh + h) * S + qc;
  const float mx = stat_m[stat_idx], inv_l = stat_l[stat_idx];  // row maximum and row sum of the forward
  const float rl = __fdiv_rn(1.0f, inv_l);

  float rowdot = 0.f, dsp = 0.f;
  f32x16_t dqacc[2];
#pragma unroll
  for (int et = 0; et < 2; ++et)
#pragma unroll
    for (int r = 0; r < 16; ++r) dqacc[et][r] = 0.f;
  const size_t tbase = ((size_t)b * nh + h) * s_pad * s_pad;

  // one tile of 32 keys: P (recomputed with the rounding steps of the forward) and dP after the
  // straight-through rule of the probability quantizer; adds the tile's terms to dsp when asked
  auto probs = [&](int t, float* p_out, float* dp_out, bool add_dsp) {
    f32x16_t sacc, dacc;
#pragma unroll
    for (int r = 0; r < 16; ++r) sacc[r] = dacc[r] = 0.f;
    const bf16_t* kp = Ks + (32 * t + (lane & 31)) * kRowStride + half * 8;
    const bf16_t* vp = Vs + (32 * t + (lane & 31)) * kRowStride + half * 8;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      sacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(kp + kk * 16), qf[kk], sacc, 0, 0, 0);
      dacc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag(vp + kk * 16), cf[kk], dacc, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = key_of(t, r, half);
      const float p = j < len ? div_by(__expf(__fsub_rn(__fmul_rn(sacc[r], sc.qk), mx)), inv_l, rl) : 0.f;
      const float dph = dacc[r] * sc.sv;
      float dp = dph;
      if (sc.p_on) {
        const float v = div_by(p, sc.sp, sc.rsp);
        const bool in = v <= sc.p_qp;
        if (add_dsp) dsp += dph * (rintf(fminf(v, sc.p_qp)) - (in ? v : 0.f));
        dp = in ? dph : 0.f;
      }
      p_out[r] = p;
      dp_out[r] = dp;
    }
  };
  // the same tile once rowdot = sum_j dP[q][j] * P[q][j] is known: dA = P * (dP - rowdot), the
  // transposed tiles for the key-major kernel, and the tile's share of dQ^ = dA * K^
  auto consume = [&](int t, const float* p_in, const float* dp_in) {
    float da[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const float p = p_in[r];
      const float c = sc.p_on ? rintf(fminf(div_by(p, sc.sp, sc.rsp), sc.p_qp)) : p;
      da[r] = p * (dp_in[r] - rowdot);
      const int j = key_of(t, r, half);
      const size_t o = tbase + (size_t)j * s_pad + q;
      pt_out[o] = static_cast<bf16_t>(qvalid ? c : 0.f);
      dat_out[o] = static_cast<bf16_t>(qvalid ? da[r] : 0.f);
    }
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      bf16x8_t af;
#pragma unroll
      for (int i = 0; i < 8; ++i) af[i] = static_cast<bf16_t>(da[8 * s + i]);
      const int k0 = 32 * t + 16 * s + 4 * half;
      dqacc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_tr(Ks, 0, k0, k0 + 8, lane), af, dqacc[0], 0, 0, 0);
      dqacc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ld_frag_tr(Ks, 32, k0, k0 + 8, lane), af, dqacc[1], 0, 0, 0);
    }
  };
  if constexpr (NT > 0) {
    // at most NT key tiles: P and dP of the whole row stay in registers between the two passes
    float pk[NT][16], dpk[NT][16];
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      if (t < nt) {
        probs(t, pk[t], dpk[t], true);
#pragma unroll
        for (int r = 0; r < 16; ++r) rowdot += dpk[t][r] * pk[t][r];
      }
    }
    rowdot += __shfl_xor(rowdot, 32, 64);
#pragma unroll
    for (int t = 0; t < NT; ++t)
      if (t < nt) consume(t, pk[t], dpk[t]);
  } else {
    // longer rows: the tiles are formed twice, first for rowdot (and dsp), then to be consumed
    float pt[16], dpt[16];
#pragma unroll 1
    for (int t = 0; t < nt; ++t) {
      probs(t, pt, dpt, true);
#pragma unroll
      for (int r = 0; r < 16; ++r) rowdot += dpt[r] * pt[r];
    }
    rowdot += __shfl_xor(rowdot, 32, 64);
#pragma unroll 1
    for (int t = 0; t < nt; ++t) {
      probs(t, pt, dpt, false);
      consume(t, pt, dpt);
    }
  }
  // step-size gradient terms of the probability quantizer (padded query rows excluded)
  dsp = wave_sum(qvalid ? dsp : 0.f);
  if (lane == 0) ds_parts[part_idx] = dsp;
  if (qvalid) {
    const float f = sk / sqrtf((float)kD);
    const size_t orow = ((size_t)b * S + q) * ld + h * kD;
#pragma unroll
    for (int et = 0; et < 2; ++et)
#pragma unroll
      for (int g = 0; g < 4; ++g)
        store4(d_qkvh + orow + 32 * et + 8 * g + 4 * half, dqacc[et][4 * g] * f, dqacc[et][4 * g + 1] * f, dqacc[et][4 * g + 2] * f,
               dqacc[et][4 * g + 3] * f);
  }
}

// ------------------------------------------------------------------------------
// backward, key-major part: dV^[j] = sum_q P^[q][j] dC[q], dK^[j] = sum_q dA[q][j] Q^[q] / sqrt(d).
// One wavefront = 32 keys; queries are streamed in chunks of 128 through LDS (row-major, read transposed).
// ------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void attn_bwd_k_mfma_k(const bf16_t* __restrict__ codes, const bf16_t* __restrict__ dctx,
                                                         bf16_t* __restrict__ d_qkvh, AttnQ aq, int S, int H, int nt,
                                                         const bf16_t* __restrict__ pt_in, const bf16_t* __restrict__ dat_in) {
  __shared__ __attribute__((aligned(16))) bf16_t Qs[128 * kRowStride];  // one chunk of queries, row-major
  __shared__ __attribute__((aligned(16))) bf16_t Cs[128 * kRowStride];  // the same rows of dC
  const int s_pad = 32 * nt;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, half = lane >> 5;
  const int h = blockIdx.y, b = blockIdx.z, nh = gridDim.y;
  const int ld = 3 * H;
  const bf16_t* base = codes + (size_t)b * S * ld + h * kD;
  const bf16_t* cbase = dctx + (size_t)b * S * H + h * kD;
  const int jt = blockIdx.x * 4 + wave;  // key tile of this wavefront
  const bool active = jt < nt;
  const size_t tbase = ((size_t)b * nh + h) * s_pad * s_pad;
  const int jrow = 32 * jt + (lane & 31);

  f32x16_t vacc[2], kacc[2];
#pragma unroll
  for (int et = 0; et < 2; ++et)
#pragma unroll
    for (int r = 0; r < 16; ++r) vacc[et][r] = kacc[et][r] = 0.f;

  for (int c0 = 0; c0 < s_pad; c0 += 128) {
    const int cn = (s_pad - c0) < 128 ? (s_pad - c0) : 128;
    __syncthreads();
    stage_rows(base + (size_t)c0 * ld, ld, S - c0, cn, Qs);
    stage_rows(cbase + (size_t)c0 * H, H, S - c0, cn, Cs);
    __syncthreads();
    if (active) {
      const bf16_t* prow = pt_in + tbase + (size_t)jrow * s_pad + c0 + 8 * half;
      const bf16_t* arow = dat_in + tbase + (size_t)jrow * s_pad + c0 + 8 * half;
      for (int s = 0; s < cn / 16; ++s) {
        const bf16x8_t pf = ld_frag(prow + 16 * s);
        const bf16x8_t af = ld_frag(arow + 16 * s);
        const int q0 = 16 * s + 8 * half;  // queries of this lane's k-slots, in natural order
#pragma unroll
        for (int et = 0; et < 2; ++et) {
          vacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf, ld_frag_tr(Cs, 32 * et, q0, q0 + 4, lane), vacc[et], 0, 0, 0);
          kacc[et] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af, ld_frag_tr(Qs, 32 * et, q0, q0 + 4, lane), kacc[et], 0, 0, 0);
        }
      }
    }
  }
  if (!active) return;
  const float sp = aq.p.on ? *aq.p.s : 1.f;
  const float fq = (aq.q.on ? *aq.q.s : 1.f) / sqrtf((float)kD);
#pragma unroll
  for (int et = 0; et < 2; ++et)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int j = 32 * jt + 8 * (r >> 2) + 4 * half + (r & 3);
      if (j < S) {
        const size_t o = ((size_t)b * S + j) * ld + h * kD + 32 * et + (lane & 31);
        d_qkvh[o + H] = static_cast<bf16_t>(kacc[et][r] * fq);
        d_qkvh[o + 2 * H] = static_cast<bf16_t>(vacc[et][r] * sp);
      }
    }
}

// ------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------
bool attn_mfma_ok(int dt, int S, int d) { return dt == DT_BF16 && d == kD && S >= 64 && S <= 384; }

template <int NT>
static void fwd_launch(const void* codes, void* ctx, void* ctx_codes, const AttnQ& aq, const int32_t* seqlens, int B, int S, int nh,
                       float* pmax_rows, float* stat_m, float* stat_l, hipStream_t st, int8_t* ctx_codes8) {
  const int nt = (S + 31) / 32, s_pad = 32 * nt;
  const size_t lds = (size_t)2 * s_pad * kRowStride * sizeof(bf16_t);
  // the attribute belongs to the (kernel, device) pair: set again when the current device changes
  static size_t configured = 0;
  static int configured_dev = -1;
  int dev = -1;
  (void)hipGetDevice(&dev);
  if (dev != configured_dev) { configured = 0; configured_dev = dev; }
  if (lds > configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_fwd_mfma_k<NT>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured = lds;
  }
  dim3 g((S + 127) / 128, nh, B);
  hipLaunchKernelGGL(attn_fwd_mfma_k<NT>, g, dim3(256), lds, st, (const bf16_t*)codes, (bf16_t*)ctx, (bf16_t*)ctx_codes, aq, seqlens, S,
                     nh * kD, nt, pmax_rows, stat_m, stat_l, ctx_codes8);
}
void attn_fwd_mfma(const void* codes, void* ctx, void* ctx_codes, const AttnQ& aq, const int32_t* seqlens, int B, int S, int nh,
                   float* pmax_rows, float* stat_m, float* stat_l, hipStream_t st, int8_t* ctx_codes8) {
  if (S <= 128) fwd_launch<4>(codes, ctx, ctx_codes, aq, seqlens, B, S, nh, pmax_rows, stat_m, stat_l, st, ctx_codes8);
  else fwd_launch<12>(codes, ctx, ctx_codes, aq, seqlens, B, S, nh, pmax_rows, stat_m, stat_l, st, ctx_codes8);
}

// returns the number of partial sums written to ds_parts
int attn_bwd_mfma(const void* codes, const void* dctx, void* d_qkvh, const AttnQ& aq, const int32_t* seqlens, int B, int S, int nh,
                  const float* stat_m, const float* stat_l, void* pt_scratch, void* dat_scratch, float* ds_parts, hipStream_t st) {
  const int nt = (S + 31) / 32, s_pad = 32 * nt;
  const size_t lds = (size_t)2 * s_pad * kRowStride * sizeof(bf16_t);
  // the attribute belongs to the (kernel, device) pair: set again when the current device changes
  static size_t configured = 0;
  static int configured_dev = -1;
  int dev = -1;
  (void)hipGetDevice(&dev);
  if (dev != configured_dev) { configured = 0; configured_dev = dev; }
  if (lds > configured) {
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_q_mfma_k<4>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bwd_q_mfma_k<0>), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    configured = lds;
  }
  dim3 gq((s_pad + 127) / 128, nh, B);
  if (nt <= 4)
    hipLaunchKernelGGL(attn_bwd_q_mfma_k<4>, gq, dim3(256), lds, st, (const bf16_t*)codes, (const bf16_t*)dctx, (bf16_t*)d_qkvh, aq,
                       seqlens, S, nh * kD, nt, stat_m, stat_l, (bf16_t*)pt_scratch, (bf16_t*)dat_scratch, ds_parts);
  else
    hipLaunchKernelGGL(attn_bwd_q_mfma_k<0>, gq, dim3(256), lds, st, (const bf16_t*)codes, (const bf16_t*)dctx, (bf16_t*)d_qkvh, aq,
                       seqlens, S, nh * kD, nt, stat_m, stat_l, (bf16_t*)pt_scratch, (bf16_t*)dat_scratch, ds_parts);
  dim3 gk((nt + 3) / 4, nh, B);
  hipLaunchKernelGGL(attn_bwd_k_mfma_k, gk, dim3(256), 0, st, (const bf16_t*)codes, (const bf16_t*)dctx, (bf16_t*)d_qkvh, aq, S, nh * kD, nt,
                     (const bf16_t*)pt_scratch, (const bf16_t*)dat_scratch);
  return (int)(gq.x * nh * B * 4);
}

}  // namespace mrem
