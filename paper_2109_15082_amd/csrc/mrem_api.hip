// C ABI of the MREM module step (Algorithm 2) and the host-side orchestration of
// its kernels.  Host code only enqueues kernels on the caller's stream; all
// arithmetic of the method runs on the device.
#include "../../include/mrem.h"
#include "mrem_kernels.h"

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <string>
#include <vector>

using namespace mrem;

static thread_local std::string g_err;

struct mrem_ctx {
  mrem_config cfg;
  int dt, L, H, F, nh, d;
  int64_t foff[MREM_F_COUNT], fsize[MREM_F_COUNT];
  int64_t layer_stride;
  int64_t tc_off[4], tc_layer_stride;  // teacher cache, in elements
  int wN[4], wK[4];                    // the four linear layers [N,K]
  std::string err;
  // side stream for the teacher's forward pass of a step (created on the first step, on the
  // device that is current then; default priority) and the two events of its fork and join
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  hipEvent_t ev_codes = nullptr;     // the side stream has prepared the weights of the layers above the first
  std::vector<hipEvent_t> ev_layer;  // "the backward pass of layer l is enqueued", one per layer
  std::vector<hipEvent_t> ev_ready;  // [4 * l + i]: the output gradient of linear layer i of layer l is written
  std::vector<hipEvent_t> ev_done;   // [4 * l + i]: its weight-gradient product has read it
  int side_device = -1;
  GemmProfile prof;                // per-launch timing of the matrix products (measurement aid)
  int32_t* nonfinite_flag = nullptr;  // device, caller-owned, optional
};

static mrem_status fail(const mrem_ctx* ctx, mrem_status st, const std::string& msg) {
  g_err = msg;
  if (ctx) const_cast<mrem_ctx*>(ctx)->err = msg;
  return st;
}

static bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

extern "C" const char* mrem_last_error(const mrem_ctx* ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

extern "C" mrem_status mrem_create(const mrem_config* cfg, mrem_ctx** out) {
  if (!cfg || !out) return fail(nullptr, MREM_EINVAL, "mrem_create: null argument");
  const mrem_config& c = *cfg;
  if (c.n_layers < 1 || c.n_layers > 32) return fail(nullptr, MREM_ESHAPE, "n_layers must be in 1..32");
  if (c.hidden < 8 || c.hidden % 8 || c.hidden > 2048) return fail(nullptr, MREM_ESHAPE, "hidden must be a multiple of 8, <= 2048");
  if (c.ffn < 8 || c.ffn % 8) return fail(nullptr, MREM_ESHAPE, "ffn must be a multiple of 8");
  if (c.n_heads < 1 || c.hidden % c.n_heads) return fail(nullptr, MREM_ESHAPE, "hidden must be divisible by n_heads");
  const int d = c.hidden / c.n_heads;
  if (d % 8 || d > 128) return fail(nullptr, MREM_ESHAPE, "head dimension must be a multiple of 8, <= 128");
  if (c.max_seq < 1 || c.max_seq > 512) return fail(nullptr, MREM_ESHAPE, "max_seq must be in 1..512");
  if (c.max_batch < 1) return fail(nullptr, MREM_ESHAPE, "max_batch must be >= 1");
  if (!(c.w_bits == 0 || (c.w_bits >= 2 && c.w_bits <= 8))) return fail(nullptr, MREM_EINVAL, "w_bits must be 0 or 2..8");
  if (!(c.a_bits == 0 || (c.a_bits >= 2 && c.a_bits <= 8))) return fail(nullptr, MREM_EINVAL, "a_bits must be 0 or 2..8");
  if (c.act_dtype != MREM_BF16 && c.act_dtype != MREM_FP32) return fail(nullptr, MREM_EINVAL, "act_dtype must be MREM_BF16 or MREM_FP32");
  if (c.per_channel != 0 && c.per_channel != 1) return fail(nullptr, MREM_EINVAL, "per_channel must be 0 or 1");
  mrem_ctx* x = new mrem_ctx();
  x->cfg = c;
  x->dt = c.act_dtype == MREM_BF16 ? DT_BF16 : DT_F32;
  x->L = c.n_layers; x->H = c.hidden; x->F = c.ffn; x->nh = c.n_heads; x->d = d;
  const int64_t H = x->H, F = x->F;
  const int64_t sizes[MREM_F_COUNT] = {3 * H * H, H * H, F * H, H * F, 3 * H, H, H, H, F, H, H, H, 3 * H, H, F, H, 8, 8};
  int64_t off = 0;
  for (int f = 0; f < MREM_F_COUNT; ++f) { x->foff[f] = off; x->fsize[f] = sizes[f]; off += sizes[f]; }
  x->layer_stride = off;
  x->wN[0] = 3 * H; x->wK[0] = H; x->wN[1] = H; x->wK[1] = H; x->wN[2] = F; x->wK[2] = H; x->wN[3] = H; x->wK[3] = F;
  int64_t t = 0;
  for (int i = 0; i < 4; ++i) { x->tc_off[i] = t; t += (int64_t)x->wN[i] * x->wK[i]; }
  x->tc_layer_stride = t;
  *out = x;
  return MREM_OK;
}

// Releases the side stream and its events (null handles are skipped, so it also cleans up after
// a creation that failed half way).
static void release_side(mrem_ctx* ctx) {
  if (ctx->side) (void)hipStreamSynchronize(ctx->side);
  for (hipEvent_t* e : {&ctx->ev_fork, &ctx->ev_join, &ctx->ev_codes}) {
    if (*e) (void)hipEventDestroy(*e);
    *e = nullptr;
  }
  for (std::vector<hipEvent_t>* evs : {&ctx->ev_layer, &ctx->ev_ready, &ctx->ev_done}) {
    for (hipEvent_t e : *evs)
      if (e) (void)hipEventDestroy(e);
    evs->clear();
  }
  if (ctx->side) (void)hipStreamDestroy(ctx->side);
  ctx->side = nullptr;
  ctx->side_device = -1;
}
// All or nothing: on failure nothing is left behind and the next call tries again.
static bool create_side(mrem_ctx* ctx, int dev) {
  bool ok = hipStreamCreateWithFlags(&ctx->side, hipStreamNonBlocking) == hipSuccess &&
            hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming) == hipSuccess &&
            hipEventCreateWithFlags(&ctx->ev_codes, hipEventDisableTiming) == hipSuccess;
  ctx->ev_layer.assign((size_t)ctx->L, nullptr);
  ctx->ev_ready.assign((size_t)ctx->L * 4, nullptr);
  ctx->ev_done.assign((size_t)ctx->L * 4, nullptr);
  for (std::vector<hipEvent_t>* evs : {&ctx->ev_layer, &ctx->ev_ready, &ctx->ev_done})
    for (hipEvent_t& e : *evs) ok = ok && hipEventCreateWithFlags(&e, hipEventDisableTiming) == hipSuccess;
  if (!ok) {
    release_side(ctx);
    (void)hipGetLastError();  // the failure is reported by the caller's return value
    return false;
  }
  ctx->side_device = dev;
  return true;
}

extern "C" void mrem_destroy(mrem_ctx* ctx) {
  if (!ctx) return;
  release_side(ctx);
  delete ctx;
}
extern "C" int64_t mrem_param_count(const mrem_ctx* ctx) { return ctx ? ctx->layer_stride * ctx->L : -1; }
extern "C" int64_t mrem_teacher_count(const mrem_ctx* ctx) { return mrem_param_count(ctx); }
extern "C" int64_t mrem_param_offset(const mrem_ctx* ctx, int32_t layer, int32_t field) {
  if (!ctx || layer < 0 || layer >= ctx->L || field < 0 || field >= MREM_F_COUNT) return -1;
  return ctx->layer_stride * layer + ctx->foff[field];
}
extern "C" int64_t mrem_param_size(const mrem_ctx* ctx, int32_t field) {
  if (!ctx || field < 0 || field >= MREM_F_COUNT) return -1;
  return ctx->fsize[field];
}
extern "C" size_t mrem_teacher_cache_bytes(const mrem_ctx* ctx) {
  return ctx ? (size_t)(ctx->tc_layer_stride * ctx->L) * dt_size(ctx->dt) : 0;
}

// ------------------------------------------------------------------------------
// workspace plan
// ------------------------------------------------------------------------------
namespace {

struct Bump {
  size_t off = 0;
  size_t take(size_t bytes) {
    const size_t o = off;
    off += (bytes + 255) & ~size_t(255);
    return o;
  }
};

struct LayerWs {
  size_t wcodes[4], what[4], zcorr[4];
  size_t wcodes8[4], xcodes8, ctxcodes8, x1codes8, gcodes8;  // int8 copies of the codes the forward products read
  size_t xcodes, qkv, qkvcodes, ctx, ctxcodes, o, x1, x1codes, u, gcodes, y, mu1, rstd1, mu2, rstd2, stat_m, stat_l;
};

struct Plan {
  LayerWs lw[32];
  // teacher scratch
  size_t t_qkv, t_ctx, t_o, t_x1, t_g, t_y, t_mu, t_rstd;
  // backward scratch
  size_t dr2, dr1, dxh, dx1h, dch, dc, dgh, du, dqkvh, dqkv, s_da, s_ph, partials, partials_per_layer, grads, pmax, xmix;
  size_t total;
};

// The forward products of the quantized module run on int8 codes (exact int32 accumulation) when
// the storage type is bf16 and both bit widths are between 1 and 8; the token count must also
// fit the tiles, which is decided per call.
bool i8_config(const mrem_ctx* c) {
  return c->dt == DT_BF16 && c->cfg.a_bits >= 1 && c->cfg.a_bits <= 8 && c->cfg.w_bits >= 1 && c->cfg.w_bits <= 8 && c->H % 128 == 0 &&
         c->F % 128 == 0;
}

Plan make_plan(const mrem_ctx* c, int B, int S) {
  Plan p;
  Bump b;
  const size_t T = (size_t)B * S, H = c->H, F = c->F, es = dt_size(c->dt);
  for (int l = 0; l < c->L; ++l) {
    LayerWs& w = p.lw[l];
    for (int i = 0; i < 4; ++i) {
      const size_t n = (size_t)c->wN[i] * c->wK[i];
      w.wcodes[i] = b.take(n * es);
      w.what[i] = b.take(n * es);
      w.zcorr[i] = b.take((size_t)c->wN[i] * 4);
      w.wcodes8[i] = b.take(i8_config(c) ? n : 0);
    }
    w.xcodes8 = b.take(i8_config(c) ? T * H : 0); w.ctxcodes8 = b.take(i8_config(c) ? T * H : 0);
    w.x1codes8 = b.take(i8_config(c) ? T * H : 0); w.gcodes8 = b.take(i8_config(c) ? T * F : 0);
    w.xcodes = b.take(T * H * es); w.qkv = b.take(T * 3 * H * es); w.qkvcodes = b.take(T * 3 * H * es);
    w.ctx = b.take(T * H * es); w.ctxcodes = b.take(T * H * es); w.o = b.take(T * H * es);
    w.x1 = b.take(T * H * es); w.x1codes = b.take(T * H * es); w.u = b.take(T * F * es); w.gcodes = b.take(T * F * es);
    w.y = b.take(T * H * es);
    w.mu1 = b.take(T * 4); w.rstd1 = b.take(T * 4); w.mu2 = b.take(T * 4); w.rstd2 = b.take(T * 4);
    w.stat_m = b.take((size_t)B * c->nh * S * 4); w.stat_l = b.take((size_t)B * c->nh * S * 4);
  }
  p.t_qkv = b.take(T * 3 * H * es); p.t_ctx = b.take(T * H * es); p.t_o = b.take(T * H * es); p.t_x1 = b.take(T * H * es);
  p.t_g = b.take(T * F * es); p.t_y = b.take(T * H * es); p.t_mu = b.take(T * 4); p.t_rstd = b.take(T * 4);
  p.dr2 = b.take(T * H * es); p.dr1 = b.take(T * H * es); p.dxh = b.take(T * H * es);
  p.dx1h = b.take(T * H * es); p.dch = b.take(T * H * es); p.dc = b.take(T * H * es);
  p.dgh = b.take(T * F * es); p.du = b.take(T * F * es); p.dqkvh = b.take(T * 3 * H * es); p.dqkv = b.take(T * 3 * H * es);
  const size_t s_pad = ((size_t)S + 31) / 32 * 32;
  const size_t pp = (size_t)B * c->nh * s_pad * s_pad;
  p.s_da = b.take(pp * 4); p.s_ph = b.take(pp * 4);
  p.pmax = b.take((size_t)B * c->nh * S * 4);
  // first-stage partial sums of one layer's backward pass (all of them stay until the single
  // second-stage launch at the end of the backward pass): two LayerNorms, two bias column sums,
  // the elementwise kernels (at most 2048 blocks, up to 3 values each) and the attention rows
  size_t np = 2 * (size_t)ln_bwd_parts((int)T) * (3 * H + 2) + (size_t)kColMaxParts * (F + 3 * H) + 8 * 2048 + (size_t)B * c->nh * S;
  np = (np + 63) & ~size_t(63);
  p.partials_per_layer = np;
  p.partials = b.take(np * 4 * c->L);
  p.grads = b.take((size_t)mrem_param_count(c) * 4);
  p.xmix = b.take(T * H * es);  // Eq. 4: the mixed module input, when a step is given a lambda > 0
  p.total = b.off;
  return p;
}

struct Run {
  const mrem_ctx* c;
  Plan p;
  char* ws;
  hipStream_t st;
  int B, S, T;
  const int32_t* seqlens;
  GemmProfile* prof = nullptr;
  template <class X = void> X* at(size_t off) const { return reinterpret_cast<X*>(ws + off); }
  bool i8() const { return i8_config(c) && T % 128 == 0; }
  int8_t* at8(size_t off) const { return i8() ? reinterpret_cast<int8_t*>(ws + off) : nullptr; }
};

// One launch of a bandwidth-bound kernel; while a context's timing is on, the launch carries an event pair and
// is recorded with its algorithmic bytes (what the kernel must read and write at least) under `label`.
template <class F>
void timed(const Run& r, const char* label, double bytes, F&& launch) {
  if (!r.prof || !r.prof->on) { launch(); return; }
  GemmRecord rec;
  rec.flops = bytes; rec.cls = 2; rec.label = label;
  (void)hipEventCreate(&rec.e0);
  (void)hipEventCreate(&rec.e1);
  tl_launch_events.e0 = rec.e0;
  tl_launch_events.e1 = rec.e1;
  launch();
  tl_launch_events = LaunchEvents();
  r.prof->recs.push_back(rec);
}

// Second-stage reductions of a backward pass, collected while the first-stage kernels are enqueued.
struct Reductions {
  std::vector<ReduceJob> jobs;
  float* next = nullptr;  // bump pointer into the partials area
  float* take(size_t n) { float* p = next; next += (n + 63) & ~size_t(63); return p; }
  void add(const float* partials, int nparts, int width, int begin, int len, float* out, float scale = 1.f) {
    ReduceJob j;
    j.partials = partials; j.nparts = nparts; j.width = width; j.begin = begin; j.len = len; j.out = out; j.scale = scale;
    jobs.push_back(j);
  }
};

QArg make_q(const mrem_ctx* c, const float* params, int layer, int idx) {
  QArg q;
  q.on = c->cfg.a_bits > 0;
  if (!q.on) return q;
  const float* base = params + c->layer_stride * layer;
  q.s = base + c->foff[MREM_F_S_A] + idx;
  const bool uns = (idx == 3 || idx == 7);
  q.z = (idx == 7) ? base + c->foff[MREM_F_Z_A] + idx : nullptr;
  if (uns) { q.qn = 0.f; q.qp = (float)((1 << c->cfg.a_bits) - 1); }
  else { q.qp = (float)((1 << (c->cfg.a_bits - 1)) - 1); q.qn = -q.qp; }
  return q;
}

AttnQ make_attn_q(const mrem_ctx* c, const float* params, int layer, bool quant) {
  AttnQ a;
  if (!quant) return a;
  a.q = make_q(c, params, layer, 1); a.k = make_q(c, params, layer, 2); a.p = make_q(c, params, layer, 3);
  a.v = make_q(c, params, layer, 4); a.c = make_q(c, params, layer, 5);
  return a;
}

const int kWField[4] = {MREM_F_W_QKV, MREM_F_W_O, MREM_F_W_1, MREM_F_W_2};
const int kBField[4] = {MREM_F_B_QKV, MREM_F_B_O, MREM_F_B_1, MREM_F_B_2};
const int kSField[4] = {MREM_F_SW_QKV, MREM_F_SW_O, MREM_F_SW_1, MREM_F_SW_2};
const int kInQuant[4] = {0, 5, 6, 7};  // activation quantizer feeding each linear layer

// quantized linear layer i of layer l: out = codes_in * wcodes^T with the steps in the epilogue
void student_linear(const Run& r, const float* params, int l, int i, const void* in_codes, const int8_t* in_codes8, void* out) {
  const mrem_ctx* c = r.c;
  const float* base = params + c->layer_stride * l;
  Epilogue e;
  const QArg q = make_q(c, params, l, kInQuant[i]);
  if (q.on) e.alpha = q.s;
  if (c->cfg.w_bits > 0) e.col_scale = base + c->foff[kSField[i]];
  if (q.on && q.z) { e.beta = q.z; e.col_vec = r.at<float>(r.p.lw[l].zcorr[i]); }
  e.bias = base + c->foff[kBField[i]];
  if (r.i8() && in_codes8) {
    // unsigned codes (GELU output) are stored recentred by half their range; the epilogue adds that back
    if (q.z) e.beta_alpha = 0.5f * (q.qp + 1.f);
    gemm_i8(in_codes8, c->wK[i], r.at8(r.p.lw[l].wcodes8[i]), c->wK[i], out, c->wN[i], r.T, c->wN[i], c->wK[i], e, r.st, r.prof);
    return;
  }
  gemm_nt(c->dt, in_codes, c->wK[i], r.at(r.p.lw[l].wcodes[i]), c->wK[i], out, c->wN[i], r.T, c->wN[i], c->wK[i], e, r.st, r.prof);
}

// (layers [l0, l1); l1 < 0: to the last layer)
void prepare_weights(const Run& r, const float* params, int l0 = 0, int l1 = -1) {
  const mrem_ctx* c = r.c;
  if (l1 < 0) l1 = c->L;
  if (l0 >= l1) return;
  std::vector<WeightJob> jobs;
  jobs.reserve((size_t)(l1 - l0) * 4);
  for (int l = l0; l < l1; ++l) {
    const float* base = params + c->layer_stride * l;
    for (int i = 0; i < 4; ++i) {
      WeightJob j;
      j.w = base + c->foff[kWField[i]]; j.sw = base + c->foff[kSField[i]];
      j.codes8 = r.at8(r.p.lw[l].wcodes8[i]);
      j.codes = j.codes8 ? nullptr : r.at(r.p.lw[l].wcodes[i]);  // the forward reads one or the other
      j.what = r.at(r.p.lw[l].what[i]); j.zcorr = r.at<float>(r.p.lw[l].zcorr[i]);
      j.N = c->wN[i]; j.K = c->wK[i];
      jobs.push_back(j);
    }
  }
  double nw = 0;
  for (const WeightJob& j : jobs) nw += (double)j.N * j.K;
  // fp32 master in; codes (int8, or the storage type) and the dequantized copy out
  timed(r, "weight_codes_k", nw * (4 + (r.i8() ? 1 : dt_size(c->dt)) + dt_size(c->dt)),
        [&] { weight_prepare(c->dt, jobs.data(), (int)jobs.size(), c->cfg.w_bits, r.st); });
}

// Layers [l0, l1) of the quantized module (l1 < 0: to the last layer).
// mix_fp != null (with 0 < lambda <= 1): the module input is lambda * mix_fp + (1 - lambda) * x_in (Eq. 4), formed and
// stored in x_q (a workspace buffer) by the kernel that quantizes the first layer's input.
void student_forward(const Run& r, const float* params, const void* x_q, void* per_layer_q, int l0 = 0, int l1 = -1,
                     const void* mix_fp = nullptr, const void* mix_in = nullptr, float lambda = 0.f) {
  const mrem_ctx* c = r.c;
  const size_t es = dt_size(c->dt);
  const int H = c->H, F = c->F, T = r.T;
  const size_t slice = (size_t)T * H * es;
  if (l1 < 0) l1 = c->L;
  for (int l = l0; l < l1; ++l) {
    const LayerWs& w = r.p.lw[l];
    const float* base = params + c->layer_stride * l;
    const void* x = l == 0 ? x_q : (const char*)per_layer_q + slice * (l - 1);
    void* f = (char*)per_layer_q + slice * l;
    // every code tensor that feeds a linear layer is also written as int8 when the int8 products are in use
    // (the input codes of layers 1.. come from the second LayerNorm of the layer before)
    if (l == 0 && mix_fp)
      mix_quantize(c->dt, mix_fp, mix_in, lambda, 1.f - lambda, const_cast<void*>(x), r.at(w.xcodes), (int64_t)T * H, make_q(c, params, l, 0), r.st,
                   r.at8(w.xcodes8));
    else if (l == 0)
      timed(r, "act_quantize_k", (double)T * H * (2 * es + (r.i8() ? 1 : 0)),
            [&] { act_quantize(c->dt, x, r.at(w.xcodes), (int64_t)T * H, make_q(c, params, l, 0), r.st, r.at8(w.xcodes8)); });
    student_linear(r, params, l, 0, r.at(w.xcodes), r.at8(w.xcodes8), r.at(w.qkv));
    const AttnQ aq = make_attn_q(c, params, l, true);
    timed(r, "qkv_quantize_k", (double)T * 3 * H * 2 * es, [&] { qkv_quantize(c->dt, r.at(w.qkv), r.at(w.qkvcodes), T, H, aq.q, aq.k, aq.v, r.st); });
    if (attn_mfma_ok(c->dt, r.S, c->d)) {
      attn_fwd_mfma(r.at(w.qkvcodes), r.at(w.ctx), r.at(w.ctxcodes), aq, r.seqlens, r.B, r.S, c->nh, nullptr, r.at<float>(w.stat_m),
                    r.at<float>(w.stat_l), r.st, r.at8(w.ctxcodes8));
    } else {
      attn_fwd(c->dt, r.at(w.qkvcodes), r.at(w.ctx), r.at(w.ctxcodes), aq, r.seqlens, r.B, r.S, c->nh, c->d, nullptr, r.st);
      if (r.i8()) codes_to_i8(c->dt, r.at(w.ctxcodes), r.at8(w.ctxcodes8), (int64_t)T * H, 0.f, r.st);
    }
    student_linear(r, params, l, 1, r.at(w.ctxcodes), r.at8(w.ctxcodes8), r.at(w.o));
    const double ln_q_bytes = (double)T * H * (4 * es + (r.i8() ? 1 : 0));  // x, r in; y and its codes (and int8 codes) out
    timed(r, "ln_fwd_k", ln_q_bytes, [&] {
      ln_fwd(c->dt, x, r.at(w.o), base + c->foff[MREM_F_LN1_G], base + c->foff[MREM_F_LN1_B], r.at(w.x1), r.at(w.x1codes),
             make_q(c, params, l, 6), r.at<float>(w.mu1), r.at<float>(w.rstd1), T, H, c->cfg.ln_eps, r.st, r.at8(w.x1codes8));
    });
    student_linear(r, params, l, 2, r.at(w.x1codes), r.at8(w.x1codes8), r.at(w.u));
    {
      const QArg qg = make_q(c, params, l, 7);
      timed(r, "gelu_quantize_k", (double)T * F * (2 * es + (r.i8() ? 1 : 0)),
            [&] { gelu_quantize(c->dt, r.at(w.u), r.at(w.gcodes), (int64_t)T * F, qg, r.st, r.at8(w.gcodes8), 0.5f * (qg.qp + 1.f)); });
    }
    student_linear(r, params, l, 3, r.at(w.gcodes), r.at8(w.gcodes8), r.at(w.y));
    if (l + 1 < c->L) {
      // the layer output and, in the same pass, its codes under the next layer's input quantizer
      const LayerWs& wn = r.p.lw[l + 1];
      timed(r, "ln_fwd_k", ln_q_bytes, [&] {
        ln_fwd(c->dt, r.at(w.x1), r.at(w.y), base + c->foff[MREM_F_LN2_G], base + c->foff[MREM_F_LN2_B], f, r.at(wn.xcodes),
               make_q(c, params, l + 1, 0), r.at<float>(w.mu2), r.at<float>(w.rstd2), T, H, c->cfg.ln_eps, r.st, r.at8(wn.xcodes8));
      });
    } else {
      timed(r, "ln_fwd_k", (double)T * H * 3 * es, [&] {
        ln_fwd(c->dt, r.at(w.x1), r.at(w.y), base + c->foff[MREM_F_LN2_G], base + c->foff[MREM_F_LN2_B], f, nullptr, QArg(),
               r.at<float>(w.mu2), r.at<float>(w.rstd2), T, H, c->cfg.ln_eps, r.st);
      });
    }
  }
}

// Full-precision module.  With calib_params != null the clipping ranges of the
// eight activation quantizers of every layer are derived on the way.
// Layers [l0, l1) (l1 < 0: to the last layer).
void teacher_forward(const Run& r, const float* teacher, const void* cache, const void* x_fp, void* per_layer_fp, float* calib_params,
                     int l0 = 0, int l1 = -1) {
  const mrem_ctx* c = r.c;
  const size_t es = dt_size(c->dt);
  const int H = c->H, F = c->F, T = r.T;
  const size_t slice = (size_t)T * H * es;
  const float qp_s = (float)((1 << (c->cfg.a_bits > 0 ? c->cfg.a_bits - 1 : 1)) - 1);
  const float qp_u = (float)((1 << (c->cfg.a_bits > 0 ? c->cfg.a_bits : 1)) - 1);
  float* parts = r.at<float>(r.p.partials);
  auto calib = [&](int l, int idx, const void* a, int dt, int rows, int cols, int ld, int gelu, int mode) {
    float* base = calib_params + c->layer_stride * l;
    const int n = absminmax(dt, a, rows, cols, ld, gelu, parts, r.st);
    calib_finalize(parts, n, mode, mode == 0 ? qp_s : qp_u, base + c->foff[MREM_F_S_A] + idx, base + c->foff[MREM_F_Z_A] + idx, r.st);
  };
  if (l1 < 0) l1 = c->L;
  for (int l = l0; l < l1; ++l) {
    const float* base = teacher + c->layer_stride * l;
    const char* wc = (const char*)cache + (size_t)c->tc_layer_stride * l * es;
    auto W = [&](int i) { return (const void*)(wc + (size_t)c->tc_off[i] * es); };
    const void* x = l == 0 ? x_fp : (const char*)per_layer_fp + slice * (l - 1);
    void* f = (char*)per_layer_fp + slice * l;
    Epilogue e;
    if (calib_params) calib(l, 0, x, c->dt, T, H, H, 0, 0);
    e.bias = base + c->foff[MREM_F_B_QKV];
    gemm_nt(c->dt, x, H, W(0), H, r.at(r.p.t_qkv), 3 * H, T, 3 * H, H, e, r.st, r.prof);
    if (calib_params) {
      const char* q = r.at<char>(r.p.t_qkv);
      calib(l, 1, q, c->dt, T, H, 3 * H, 0, 0);
      calib(l, 2, q + (size_t)H * es, c->dt, T, H, 3 * H, 0, 0);
      calib(l, 4, q + (size_t)2 * H * es, c->dt, T, H, 3 * H, 0, 0);
    }
    if (attn_mfma_ok(c->dt, r.S, c->d))
      attn_fwd_mfma(r.at(r.p.t_qkv), r.at(r.p.t_ctx), nullptr, AttnQ(), r.seqlens, r.B, r.S, c->nh,
                    calib_params ? r.at<float>(r.p.pmax) : nullptr, nullptr, nullptr, r.st);
    else
      attn_fwd(c->dt, r.at(r.p.t_qkv), r.at(r.p.t_ctx), nullptr, AttnQ(), r.seqlens, r.B, r.S, c->nh, c->d,
               calib_params ? r.at<float>(r.p.pmax) : nullptr, r.st);
    if (calib_params) {
      calib(l, 3, r.at(r.p.pmax), DT_F32, 1, r.B * c->nh * r.S, r.B * c->nh * r.S, 0, 1);
      calib(l, 5, r.at(r.p.t_ctx), c->dt, T, H, H, 0, 0);
    }
    e.bias = base + c->foff[MREM_F_B_O];
    gemm_nt(c->dt, r.at(r.p.t_ctx), H, W(1), H, r.at(r.p.t_o), H, T, H, H, e, r.st, r.prof);
    timed(r, "ln_fwd_k", (double)T * H * 3 * es, [&] {
      ln_fwd(c->dt, x, r.at(r.p.t_o), base + c->foff[MREM_F_LN1_G], base + c->foff[MREM_F_LN1_B], r.at(r.p.t_x1), nullptr, QArg(),
             r.at<float>(r.p.t_mu), r.at<float>(r.p.t_rstd), T, H, c->cfg.ln_eps, r.st);
    });
    if (calib_params) calib(l, 6, r.at(r.p.t_x1), c->dt, T, H, H, 0, 0);
    e.bias = base + c->foff[MREM_F_B_1];
    if (calib_params) {
      // pre-activation first, so that the range of gelu(u) can be measured on unrounded values
      gemm_nt(c->dt, r.at(r.p.t_x1), H, W(2), H, r.at(r.p.t_g), F, T, F, H, e, r.st, r.prof);
      calib(l, 7, r.at(r.p.t_g), c->dt, T, F, F, 1, 2);
      gelu_quantize(c->dt, r.at(r.p.t_g), r.at(r.p.t_g), (int64_t)T * F, QArg(), r.st);
    } else {
      e.gelu = 1;
      gemm_nt(c->dt, r.at(r.p.t_x1), H, W(2), H, r.at(r.p.t_g), F, T, F, H, e, r.st, r.prof);
      e.gelu = 0;
    }
    e.bias = base + c->foff[MREM_F_B_2];
    gemm_nt(c->dt, r.at(r.p.t_g), F, W(3), F, r.at(r.p.t_y), H, T, H, F, e, r.st, r.prof);
    timed(r, "ln_fwd_k", (double)T * H * 3 * es, [&] {
      ln_fwd(c->dt, r.at(r.p.t_x1), r.at(r.p.t_y), base + c->foff[MREM_F_LN2_G], base + c->foff[MREM_F_LN2_B], f, nullptr, QArg(),
             r.at<float>(r.p.t_mu), r.at<float>(r.p.t_rstd), T, H, c->cfg.ln_eps, r.st);
    });
  }
}

// weight-gradient product of linear layer i: grads[w] = (dY^T * codes_in) * s_a (+ z * db);
// dy is [T, N_out], codes_in is [T, K_in]: the token index is the contraction index of both
void wgrad(const Run& r, const float* params, float* grads, int l, int i, const void* dy, const void* codes_in) {
  const mrem_ctx* c = r.c;
  float* g = grads + c->layer_stride * l;
  Epilogue e;
  const QArg q = make_q(c, params, l, kInQuant[i]);
  if (q.on) e.alpha = q.s;  // the offset term z * db[n] of an asymmetric input quantizer is added by the update kernel
  e.out_f32 = 1;
  e.c_zeroed = 1;  // the step starts by zeroing the gradients that are formed in k-slices
  gemm(c->dt, 1, 1, dy, c->wN[i], codes_in, c->wK[i], g + c->foff[kWField[i]], c->wK[i], c->wN[i], c->wK[i], r.T, e, r.st, r.prof);
}
// input-gradient product: d(in^) = dY * W^ with the dequantized weights [N_out, K_in]
void dgrad(const Run& r, int l, int i, const void* dy, void* out) {
  const mrem_ctx* c = r.c;
  Epilogue e;
  gemm(c->dt, 0, 1, dy, c->wN[i], r.at(r.p.lw[l].what[i]), c->wK[i], out, c->wK[i], r.T, c->wK[i], c->wN[i], e, r.st, r.prof);
}

// Zeroes what the backward pass adds into (weight gradients formed in two k-slices) or never
// writes (the slots of the fixed quantizer offsets; the vectors of a layer are one region).
void zero_gradient_slots(const Run& r, float* grads) {
  const mrem_ctx* c = r.c;
  std::vector<FillRegion> regions;
  for (int l = 0; l < c->L; ++l) {
    float* g = grads + c->layer_stride * l;
    regions.push_back(FillRegion{g + c->foff[MREM_F_B_QKV], c->layer_stride - c->foff[MREM_F_B_QKV]});
    for (int i = 0; i < 4; ++i)
      if (gemm_f32_k_slices(c->dt, c->wN[i], c->wK[i], r.T) > 1)
        regions.push_back(FillRegion{g + c->foff[kWField[i]], (int64_t)c->wN[i] * c->wK[i]});
  }
  zero_regions(regions.data(), (int)regions.size(), r.st);
}

// What the backward pass needs to update the weight matrices of a layer as soon as that layer's
// gradients are complete (Algorithm 2, last line), on `side` if there is one.
struct Update {
  float* params;
  float* m;
  float* v;
  AdamArg a;
  int write_grads;
  hipStream_t side;            // nullptr: everything on the caller's stream
  const hipEvent_t* ev_layer;  // one per layer when side != nullptr
  const hipEvent_t* ev_ready;  // four per layer
  const hipEvent_t* ev_done;   // four per layer
  hipEvent_t ev_join;
};
void update_matrices(const Run& r, const Update& u, float* grads, int l, hipStream_t st);

void student_backward(const Run& r, const float* params, const void* x_q, const void* per_layer_fp, const void* per_layer_q,
                      float* grads, float* loss_out, const Update& up) {
  const mrem_ctx* c = r.c;
  const size_t es = dt_size(c->dt);
  const int H = c->H, F = c->F, T = r.T, L = c->L;
  const size_t slice = (size_t)T * H * es;
  const int64_t numel = (int64_t)T * H;
  Reductions red;
  for (int l = L - 1; l >= 0; --l) {
    const size_t first_job = red.jobs.size();
    const LayerWs& w = r.p.lw[l];
    const float* base = params + c->layer_stride * l;
    float* g = grads + c->layer_stride * l;
    const void* x = l == 0 ? x_q : (const char*)per_layer_q + slice * (l - 1);
    const void* fq = (const char*)per_layer_q + slice * l;
    const void* ffp = (const char*)per_layer_fp + slice * l;
    const bool in_loss = (c->cfg.loss_layer_mask >> l) & 1u;
    red.next = r.at<float>(r.p.partials) + r.p.partials_per_layer * l;
    // The weight-gradient products feed nothing but the update, so with a side stream they run
    // there, beside the input-gradient products and the bandwidth-bound kernels of this stream.
    // The output-gradient buffers are shared by all layers: before this stream overwrites one, it
    // waits until the product of the layer above has read it.
    auto issue_wgrad = [&](int i, const void* dy, const void* codes) {
      if (!up.side) { wgrad(r, params, grads, l, i, dy, codes); return; }
      (void)hipEventRecord(up.ev_ready[4 * l + i], r.st);
      (void)hipStreamWaitEvent(up.side, up.ev_ready[4 * l + i], 0);
      Run rs = r;
      rs.st = up.side;
      wgrad(rs, params, grads, l, i, dy, codes);
      (void)hipEventRecord(up.ev_done[4 * l + i], up.side);
    };
    auto before_overwrite = [&](int i) {
      if (up.side && l < L - 1) (void)hipStreamWaitEvent(r.st, up.ev_done[4 * (l + 1) + i], 0);
    };
    // second LayerNorm: dy = [dr1 + dxh*mask of the layer above] + gradient of this layer's Eq. 3 term,
    // which the same kernel forms from the two layer outputs (it also returns the squared-error sum)
    {
      const bool top = (l == L - 1);
      const QArg q_above = top ? QArg() : make_q(c, params, l + 1, 0);
      const float scale = c->cfg.loss_mean ? 1.0f / (float)numel : 1.0f;
      const int wd = 3 * H + 2;
      float* parts = red.take((size_t)ln_bwd_parts(T) * wd);
      before_overwrite(3);
      int n = 0;
      // in: layer output, the two LayerNorm inputs, the full-precision output (loss), above the top layer also the two
      // gradients from above; out: the gradient of the LayerNorm input
      timed(r, "ln_bwd_k", (double)T * H * es * ((top ? 4 : 6) + (in_loss ? 1 : 0)), [&] {
        n = ln_bwd(c->dt, top ? nullptr : r.at(r.p.dr1), top ? nullptr : r.at(r.p.dxh), fq, q_above, r.at(w.x1), r.at(w.y),
                   r.at<float>(w.mu2), r.at<float>(w.rstd2), base + c->foff[MREM_F_LN2_G], r.at(r.p.dr2), parts, T, H, r.st,
                   in_loss ? ffp : nullptr, scale);
      });
      red.add(parts, n, wd, 0, H, g + c->foff[MREM_F_LN2_G]);
      red.add(parts, n, wd, H, H, g + c->foff[MREM_F_LN2_B]);
      red.add(parts, n, wd, 2 * H, H, g + c->foff[MREM_F_B_2]);
      if (!top) red.add(parts, n, wd, 3 * H, 1, grads + c->layer_stride * (l + 1) + c->foff[MREM_F_S_A] + 0);
      // a layer outside the loss mask contributes an exact zero (its partial sums are zero)
      red.add(parts, n, wd, 3 * H + 1, 1, loss_out + 1 + l, in_loss ? scale : 0.f);
    }
    // second feed-forward projection
    issue_wgrad(3, r.at(r.p.dr2), r.at(w.gcodes));
    dgrad(r, l, 3, r.at(r.p.dr2), r.at(r.p.dgh));
    // GELU and its output quantizer
    {
      // the kernel also leaves the column sums of du per row slab: the bias gradient of the first projection
      float* parts = red.take(2048);
      float* cols = red.take((size_t)kColMaxParts * F);
      before_overwrite(2);
      ColGrid cg{};
      timed(r, "gelu_quant_bwd_k", (double)T * F * 3 * es,
            [&] { cg = gelu_quant_bwd(c->dt, r.at(r.p.dgh), r.at(w.u), r.at(r.p.du), T, F, make_q(c, params, l, 7), parts, cols, r.st); });
      red.add(parts, cg.gx * cg.gy, 1, 0, 1, g + c->foff[MREM_F_S_A] + 7);
      red.add(cols, cg.gy, F, 0, F, g + c->foff[MREM_F_B_1]);
    }
    // first feed-forward projection
    issue_wgrad(2, r.at(r.p.du), r.at(w.x1codes));
    dgrad(r, l, 2, r.at(r.p.du), r.at(r.p.dx1h));
    // first LayerNorm: dy = dr2 (residual) + dx1h through the FFN-input quantizer
    {
      float* parts = red.take((size_t)ln_bwd_parts(T) * (3 * H + 2));
      before_overwrite(1);
      int n = 0;
      timed(r, "ln_bwd_k", (double)T * H * es * 6, [&] {
        n = ln_bwd(c->dt, r.at(r.p.dr2), r.at(r.p.dx1h), r.at(w.x1), make_q(c, params, l, 6), x, r.at(w.o),
                   r.at<float>(w.mu1), r.at<float>(w.rstd1), base + c->foff[MREM_F_LN1_G], r.at(r.p.dr1), parts, T, H, r.st);
      });
      const int wd = 3 * H + 2;
      red.add(parts, n, wd, 0, H, g + c->foff[MREM_F_LN1_G]);
      red.add(parts, n, wd, H, H, g + c->foff[MREM_F_LN1_B]);
      red.add(parts, n, wd, 2 * H, H, g + c->foff[MREM_F_B_O]);
      red.add(parts, n, wd, 3 * H, 1, g + c->foff[MREM_F_S_A] + 6);
    }
    // attention output projection
    issue_wgrad(1, r.at(r.p.dr1), r.at(w.ctxcodes));
    dgrad(r, l, 1, r.at(r.p.dr1), r.at(r.p.dch));
    {
      float* parts = red.take(2048);
      int n = 0;
      timed(r, "quant_bwd_k", (double)numel * 3 * es,
            [&] { n = quant_bwd(c->dt, r.at(r.p.dch), r.at(w.ctx), r.at(r.p.dc), numel, make_q(c, params, l, 5), parts, r.st); });
      red.add(parts, n, 1, 0, 1, g + c->foff[MREM_F_S_A] + 5);
    }
    // attention
    const AttnQ aq = make_attn_q(c, params, l, true);
    {
      int n = r.B * c->nh * r.S;
      float* parts = red.take((size_t)n);
      if (attn_mfma_ok(c->dt, r.S, c->d))
        n = attn_bwd_mfma(r.at(w.qkvcodes), r.at(r.p.dc), r.at(r.p.dqkvh), aq, r.seqlens, r.B, r.S, c->nh, r.at<float>(w.stat_m),
                          r.at<float>(w.stat_l), r.at(r.p.s_ph), r.at(r.p.s_da), parts, r.st);
      else
        attn_bwd(c->dt, r.at(w.qkvcodes), r.at(r.p.dc), r.at(r.p.dqkvh), aq, r.seqlens, r.B, r.S, c->nh, c->d, r.at<float>(r.p.s_da),
                 r.at<float>(r.p.s_ph), parts, r.st);
      red.add(parts, n, 1, 0, 1, g + c->foff[MREM_F_S_A] + 3);
    }
    {
      // the kernel also leaves the column sums of dqkv per row slab: the bias gradient of the projection
      float* parts = red.take(2048 * 3);
      float* cols = red.take((size_t)kColMaxParts * 3 * H);
      before_overwrite(0);
      ColGrid cg{};
      timed(r, "qkv_quant_bwd_k", (double)T * 3 * H * 3 * es,
            [&] { cg = qkv_quant_bwd(c->dt, r.at(r.p.dqkvh), r.at(w.qkv), r.at(r.p.dqkv), T, H, aq.q, aq.k, aq.v, parts, cols, r.st); });
      const int n = cg.gx * cg.gy;
      red.add(parts, n, 3, 0, 1, g + c->foff[MREM_F_S_A] + 1);
      red.add(parts, n, 3, 1, 1, g + c->foff[MREM_F_S_A] + 2);
      red.add(parts, n, 3, 2, 1, g + c->foff[MREM_F_S_A] + 4);
      red.add(cols, cg.gy, 3 * H, 0, 3 * H, g + c->foff[MREM_F_B_QKV]);
    }
    // query/key/value projection
    issue_wgrad(0, r.at(r.p.dqkv), r.at(w.xcodes));
    dgrad(r, l, 0, r.at(r.p.dqkv), r.at(r.p.dxh));
    if (l == 0) {
      // nothing flows out of the module (Section 4.2); only the input quantizer's step needs dxh
      float* parts = red.take(2048);
      const int n = quant_bwd_reduce(c->dt, r.at(r.p.dxh), x, numel, make_q(c, params, 0, 0), parts, r.st);
      red.add(parts, n, 1, 0, 1, g + c->foff[MREM_F_S_A] + 0);
    }
    // This layer's gradients are complete and nothing below reads its matrices or their steps
    // again (the input gradients used the dequantized copies): its second-stage reductions and
    // the update of its four matrices, which is bound by memory traffic, run beside the
    // matrix products of the layers below.
    hipStream_t us = r.st;
    if (up.side) {
      us = up.side;
      (void)hipEventRecord(up.ev_layer[l], r.st);
      (void)hipStreamWaitEvent(us, up.ev_layer[l], 0);
    }
    reduce_jobs(red.jobs.data() + first_job, (int)(red.jobs.size() - first_job), us);
    update_matrices(r, up, grads, l, us);
  }
  if (up.side) {
    (void)hipEventRecord(up.ev_join, up.side);
    (void)hipStreamWaitEvent(r.st, up.ev_join, 0);
  }
  loss_total(loss_out, L, c->nonfinite_flag, r.st);
}

AdamArg adam_arg(const mrem_ctx* c, int64_t step, float lr) {
  AdamArg a;
  a.lr = lr; a.beta1 = c->cfg.beta1; a.beta2 = c->cfg.beta2; a.eps = c->cfg.adam_eps; a.wd = c->cfg.weight_decay;
  a.bc1 = (float)(1.0 - std::pow((double)c->cfg.beta1, (double)step));
  a.bc2 = (float)(1.0 - std::pow((double)c->cfg.beta2, (double)step));
  a.floor = c->cfg.step_floor;
  return a;
}
// AdamW on the four weight matrices of layer l and their steps (they read the bias gradient and the
// activation offset of their layer, so the layer's reductions come first on the same stream)
void update_matrices(const Run& r, const Update& u, float* grads, int l, hipStream_t st) {
  const mrem_ctx* c = r.c;
  AdamJob jobs[4];
  const int64_t o = c->layer_stride * l;
  for (int i = 0; i < 4; ++i) {
    const int64_t ow = o + c->foff[kWField[i]], os = o + c->foff[kSField[i]];
    // the second feed-forward projection reads the GELU output through an asymmetric quantizer with offset z
    const bool zterm = (i == 3 && c->cfg.a_bits > 0);
    AdamJob& j = jobs[i];
    j.w = u.params + ow; j.sw = u.params + os; j.g_w = grads + ow; j.g_sw = grads + os;
    j.m_w = u.m + ow; j.v_w = u.v + ow; j.m_sw = u.m + os; j.v_sw = u.v + os;
    j.z_in = zterm ? u.params + o + c->foff[MREM_F_Z_A] + 7 : nullptr;
    j.db = zterm ? grads + o + c->foff[MREM_F_B_2] : nullptr;
    j.N = c->wN[i]; j.K = c->wK[i];
  }
  double nw = 0;
  for (int i = 0; i < 4; ++i) nw += (double)c->wN[i] * c->wK[i];
  Run rs = r;
  rs.st = st;
  // parameter, gradient and both moments in; parameter and both moments out (the masked gradient too when it is exported)
  timed(rs, "adam_matrix_k", nw * (28 + (u.write_grads ? 4 : 0)),
        [&] { adam_matrix(jobs, 4, c->cfg.w_bits, u.a, u.write_grads, c->cfg.per_channel ? 0 : 1, st); });
}
// AdamW (no decay) on everything that is not a matrix: biases, LayerNorm parameters, activation steps
void update_vectors(const Run& r, const Update& u, float* grads) {
  const mrem_ctx* c = r.c;
  AdamArg nodecay = u.a;
  nodecay.wd = 0.f;
  std::vector<VecJob> vjobs;
  for (int l = 0; l < c->L; ++l) {
    const int64_t o = c->layer_stride * l;
    vjobs.push_back(VecJob{o + c->foff[MREM_F_B_QKV], c->foff[MREM_F_SW_QKV] - c->foff[MREM_F_B_QKV], 0});
    if (c->cfg.a_bits > 0) vjobs.push_back(VecJob{o + c->foff[MREM_F_S_A], 8, 1});
  }
  adam_vector(u.params, grads, u.m, u.v, vjobs.data(), (int)vjobs.size(), nodecay, r.st);
}

mrem_status check_common(const mrem_ctx* ctx, int32_t batch, int32_t seq, const void* workspace, size_t workspace_bytes, const char* who,
                         Plan* plan) {
  if (!ctx) return fail(nullptr, MREM_EINVAL, std::string(who) + ": null context");
  if (batch < 1 || batch > ctx->cfg.max_batch) return fail(ctx, MREM_ESHAPE, std::string(who) + ": batch outside 1..max_batch");
  if (seq < 1 || seq > ctx->cfg.max_seq) return fail(ctx, MREM_ESHAPE, std::string(who) + ": seq outside 1..max_seq");
  if (!workspace || !aligned16(workspace)) return fail(ctx, MREM_EINVAL, std::string(who) + ": workspace null or misaligned");
  *plan = make_plan(ctx, batch, seq);
  if (workspace_bytes < plan->total) return fail(ctx, MREM_EWORKSPACE, std::string(who) + ": workspace too small");
  return MREM_OK;
}

mrem_status finish(const mrem_ctx* ctx, const char* who) {
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(ctx, MREM_EHIP, std::string(who) + ": " + hipGetErrorString(e));
  return MREM_OK;
}

#define REQUIRE_PTR(p, who)                                                                  \
  do {                                                                                       \
    if (!(p) || !aligned16(p)) return fail(ctx, MREM_EINVAL, std::string(who) + ": " #p " is null or not 16-byte aligned"); \
  } while (0)

}  // namespace

extern "C" size_t mrem_workspace_bytes(const mrem_ctx* ctx, int32_t batch, int32_t seq) {
  if (!ctx || batch < 1 || seq < 1) return 0;
  return make_plan(ctx, batch, seq).total;
}

extern "C" int64_t mrem_workspace_offset(const mrem_ctx* ctx, int32_t batch, int32_t seq, int32_t layer, int32_t item) {
  if (!ctx || batch < 1 || seq < 1 || layer < 0 || layer >= ctx->L) return -1;
  const Plan p = make_plan(ctx, batch, seq);
  const LayerWs& w = p.lw[layer];
  const bool i8 = i8_config(ctx) && (batch * seq) % 128 == 0;
  if (item >= MREM_WS_WCODES8 && item < MREM_WS_WCODES8 + 4) return i8 ? (int64_t)w.wcodes8[item - MREM_WS_WCODES8] : -1;
  if (item >= MREM_WS_WCODES && item < MREM_WS_WCODES + 4) return i8 ? -1 : (int64_t)w.wcodes[item - MREM_WS_WCODES];
  if (item == MREM_WS_QKV) return (int64_t)w.qkv;
  if (item == MREM_WS_XCODES8) return i8 ? (int64_t)w.xcodes8 : -1;
  return -1;
}

extern "C" mrem_status mrem_quantize(const float* w, int64_t N, int64_t K, int32_t bits, int32_t per_channel, int32_t init_scale,
                                     float* scale, int8_t* codes, void* hip_stream) {
  const mrem_ctx* ctx = nullptr;
  REQUIRE_PTR(w, "mrem_quantize");
  REQUIRE_PTR(scale, "mrem_quantize");
  REQUIRE_PTR(codes, "mrem_quantize");
  if (bits < 2 || bits > 8) return fail(nullptr, MREM_EINVAL, "mrem_quantize: bits must be in 2..8");
  if (N < 1 || K < 1 || N > 0x7fffffff) return fail(nullptr, MREM_ESHAPE, "mrem_quantize: N and K must be >= 1 (N < 2^31)");
  if (per_channel != 0 && per_channel != 1) return fail(nullptr, MREM_EINVAL, "mrem_quantize: per_channel must be 0 or 1");
  weight_quantize_i8(w, scale, codes, N, K, bits, per_channel, init_scale, (hipStream_t)hip_stream);
  return finish(nullptr, "mrem_quantize");
}

extern "C" mrem_status mrem_module_init_steps(mrem_ctx* ctx, float* params, void* hip_stream) {
  if (!ctx) return fail(nullptr, MREM_EINVAL, "mrem_module_init_steps: null context");
  REQUIRE_PTR(params, "mrem_module_init_steps");
  if (ctx->cfg.w_bits == 0) return fail(ctx, MREM_EINVAL, "mrem_module_init_steps: weight quantizers are off (w_bits = 0)");
  for (int l = 0; l < ctx->L; ++l)
    for (int i = 0; i < 4; ++i) {
      float* sw = params + ctx->layer_stride * l + ctx->foff[kSField[i]];
      weight_step_init(params + ctx->layer_stride * l + ctx->foff[kWField[i]], sw, ctx->wN[i], ctx->wK[i], ctx->cfg.w_bits,
                       (hipStream_t)hip_stream);
      // one step per matrix: max|W| / Qp is the largest of the rows' quotients (the division is monotone)
      if (!ctx->cfg.per_channel) tie_steps_max(sw, ctx->wN[i], (hipStream_t)hip_stream);
    }
  return finish(ctx, "mrem_module_init_steps");
}

extern "C" mrem_status mrem_teacher_prepare(mrem_ctx* ctx, const float* teacher, void* cache, void* hip_stream) {
  if (!ctx) return fail(nullptr, MREM_EINVAL, "mrem_teacher_prepare: null context");
  REQUIRE_PTR(teacher, "mrem_teacher_prepare");
  REQUIRE_PTR(cache, "mrem_teacher_prepare");
  const size_t es = dt_size(ctx->dt);
  for (int l = 0; l < ctx->L; ++l)
    for (int i = 0; i < 4; ++i)
      convert_f32(ctx->dt, teacher + ctx->layer_stride * l + ctx->foff[kWField[i]],
                  (char*)cache + ((size_t)ctx->tc_layer_stride * l + ctx->tc_off[i]) * es, (int64_t)ctx->wN[i] * ctx->wK[i],
                  (hipStream_t)hip_stream);
  return finish(ctx, "mrem_teacher_prepare");
}

extern "C" mrem_status mrem_module_calibrate(mrem_ctx* ctx, float* params, const float* teacher, const void* teacher_cache, const void* x_fp,
                                             const int32_t* seqlens, int32_t batch, int32_t seq, void* workspace, size_t workspace_bytes,
                                             void* hip_stream) {
  Plan plan;
  mrem_status s = check_common(ctx, batch, seq, workspace, workspace_bytes, "mrem_module_calibrate", &plan);
  if (s != MREM_OK) return s;
  REQUIRE_PTR(params, "mrem_module_calibrate");
  REQUIRE_PTR(teacher, "mrem_module_calibrate");
  REQUIRE_PTR(teacher_cache, "mrem_module_calibrate");
  REQUIRE_PTR(x_fp, "mrem_module_calibrate");
  if (ctx->cfg.a_bits == 0) return fail(ctx, MREM_EINVAL, "mrem_module_calibrate: activation quantizers are off (a_bits = 0)");
  Run r{ctx, plan, (char*)workspace, (hipStream_t)hip_stream, batch, seq, batch * seq, seqlens, &ctx->prof};
  // Layer by layer with two alternating output buffers: only the ranges are wanted, not the per-layer outputs.
  {
    mrem_ctx one = *ctx;
    one.L = 1;
    const size_t es = dt_size(ctx->dt);
    void* bufs[2] = {r.at(r.p.dr1), r.at(r.p.dr2)};
    const void* x = x_fp;
    for (int l = 0; l < ctx->L; ++l) {
      Run rl = r;
      rl.c = &one;
      teacher_forward(rl, teacher + ctx->layer_stride * l, (const char*)teacher_cache + (size_t)ctx->tc_layer_stride * l * es, x,
                      bufs[l & 1], params + ctx->layer_stride * l);
      x = bufs[l & 1];
    }
  }
  return finish(ctx, "mrem_module_calibrate");
}

namespace {
mrem_status forward_impl(mrem_ctx* ctx, const float* params, const float* teacher, const void* teacher_cache, const void* x_fp,
                         const void* x_q, const int32_t* seqlens, int32_t batch, int32_t seq, void* per_layer_fp, void* per_layer_q,
                         void* workspace, size_t workspace_bytes, void* hip_stream, const char* who) {
  Plan plan;
  mrem_status s = check_common(ctx, batch, seq, workspace, workspace_bytes, who, &plan);
  if (s != MREM_OK) return s;
  if (!per_layer_fp && !per_layer_q) return fail(ctx, MREM_EINVAL, std::string(who) + ": both outputs are null");
  Run r{ctx, plan, (char*)workspace, (hipStream_t)hip_stream, batch, seq, batch * seq, seqlens, &ctx->prof};
  if (per_layer_fp) {
    REQUIRE_PTR(teacher, who);
    REQUIRE_PTR(teacher_cache, who);
    REQUIRE_PTR(x_fp, who);
    if (!aligned16(per_layer_fp)) return fail(ctx, MREM_EINVAL, std::string(who) + ": per_layer_fp misaligned");
  }
  if (per_layer_q) {
    REQUIRE_PTR(params, who);
    REQUIRE_PTR(x_q, who);
    if (!aligned16(per_layer_q)) return fail(ctx, MREM_EINVAL, std::string(who) + ": per_layer_q misaligned");
  }
  if (per_layer_fp) teacher_forward(r, teacher, teacher_cache, x_fp, per_layer_fp, nullptr);
  if (per_layer_q) {
    prepare_weights(r, params);
    student_forward(r, params, x_q, per_layer_q);
  }
  return finish(ctx, who);
}
}  // namespace

extern "C" mrem_status mrem_module_forward(mrem_ctx* ctx, const float* params, const float* teacher, const void* teacher_cache,
                                           const void* x_fp, const void* x_q, const int32_t* seqlens, int32_t batch, int32_t seq,
                                           void* per_layer_fp, void* per_layer_q, void* workspace, size_t workspace_bytes, void* hip_stream) {
  return forward_impl(ctx, params, teacher, teacher_cache, x_fp, x_q, seqlens, batch, seq, per_layer_fp, per_layer_q, workspace,
                      workspace_bytes, hip_stream, "mrem_module_forward");
}

// ------------------------------------------------------------------------------
// The forward passes for callers that cannot allocate: the workspace is a static device array.
// ------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char scratch[MREM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
// Device address of `scratch` on each device (every device holds its own copy of the array at its
// own address; the array's name itself is only a host-side handle).  Looked up once per device,
// with that device current.
void* g_scratch_ptr[kMaxDevices] = {};
}  // namespace

extern "C" size_t mrem_static_scratch_bytes(void) { return MREM_STATIC_SCRATCH_BYTES; }

extern "C" mrem_status mrem_module_forward_static(mrem_ctx* ctx, const float* params, const float* teacher, const void* teacher_cache,
                                                  const void* x_fp, const void* x_q, const int32_t* seqlens, int32_t batch,
                                                  int32_t seq, void* per_layer_fp, void* per_layer_q, void* hip_stream) {
  const char* who = "mrem_module_forward_static";
  if (!ctx) return fail(nullptr, MREM_EINVAL, std::string(who) + ": null context");
  if (batch < 1 || seq < 1) return fail(ctx, MREM_ESHAPE, std::string(who) + ": batch and seq must be >= 1");
  const size_t need = make_plan(ctx, batch, seq).total;
  if (need > (size_t)MREM_STATIC_SCRATCH_BYTES)
    return fail(ctx, MREM_EWORKSPACE, std::string(who) + ": this module at this batch and seq needs " + std::to_string(need) +
                                          " bytes of scratch, the static array holds " + std::to_string((size_t)MREM_STATIC_SCRATCH_BYTES) +
                                          "; use mrem_module_forward with a caller-owned workspace");
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return fail(ctx, MREM_EHIP, std::string(who) + ": no current device");
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) return fail(ctx, MREM_EHIP, std::string(who) + ": hipGetSymbolAddress: " + hipGetErrorString(e));
    g_scratch_ptr[dev] = p;
  }
  // Nothing in the forward passes reads scratch memory that the same call has not written, so the
  // contents a previous call left behind need no clearing.
  return forward_impl(ctx, params, teacher, teacher_cache, x_fp, x_q, seqlens, batch, seq, per_layer_fp, per_layer_q,
                      g_scratch_ptr[dev], MREM_STATIC_SCRATCH_BYTES, hip_stream, who);
}

extern "C" mrem_status mrem_module_step(mrem_ctx* ctx, float* params, float* adam_m, float* adam_v, int64_t step_index, float lr,
                                        float lambda, const float* teacher, const void* teacher_cache, const void* x_fp, const void* x_q,
                                        const int32_t* seqlens, int32_t batch, int32_t seq, float* loss_out, void* per_layer_fp,
                                        void* per_layer_q, float* grads_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  Plan plan;
  mrem_status s = check_common(ctx, batch, seq, workspace, workspace_bytes, "mrem_module_step", &plan);
  if (s != MREM_OK) return s;
  REQUIRE_PTR(params, "mrem_module_step");
  REQUIRE_PTR(adam_m, "mrem_module_step");
  REQUIRE_PTR(adam_v, "mrem_module_step");
  REQUIRE_PTR(teacher, "mrem_module_step");
  REQUIRE_PTR(teacher_cache, "mrem_module_step");
  REQUIRE_PTR(x_fp, "mrem_module_step");
  REQUIRE_PTR(x_q, "mrem_module_step");
  REQUIRE_PTR(loss_out, "mrem_module_step");
  REQUIRE_PTR(per_layer_fp, "mrem_module_step");
  REQUIRE_PTR(per_layer_q, "mrem_module_step");
  if (grads_out && !aligned16(grads_out)) return fail(ctx, MREM_EINVAL, "mrem_module_step: grads_out misaligned");
  if (step_index < 1) return fail(ctx, MREM_EINVAL, "mrem_module_step: step_index is 1-based");
  if (!(lambda >= 0.f && lambda <= 1.f)) return fail(ctx, MREM_EINVAL, "mrem_module_step: lambda must be in [0,1]");
  Run r{ctx, plan, (char*)workspace, (hipStream_t)hip_stream, batch, seq, batch * seq, seqlens, &ctx->prof};
  float* grads = grads_out ? grads_out : r.at<float>(r.p.grads);
  // The teacher's forward pass shares nothing with the quantized forward pass (its own scratch, its
  // own outputs), so it runs on a side stream, forked from the caller's stream and joined before
  // the loss: kernels of the two passes fill each other's tails.
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return fail(ctx, MREM_EHIP, "mrem_module_step: no current device");
  if (!ctx->side && !create_side(ctx, dev))
    return fail(ctx, MREM_EHIP, "mrem_module_step: cannot create the side stream and its events");
  if (dev != ctx->side_device) return fail(ctx, MREM_EINVAL, "mrem_module_step: the context was first used on another device");
  const bool fork = !ctx->prof.on;  // per-launch timing wants every product alone on the device
  // Eq. 4: with lambda > 0 the quantized module reads lambda * x_fp + (1 - lambda) * x_q, formed by its first kernel
  const bool mix = lambda > 0.f && x_fp != x_q;
  const void* x_in = mix ? r.at(r.p.xmix) : x_q;
  const void* mix_fp = mix ? x_fp : nullptr;
  // Before the passes: the gradient slots that are added into or never written are zeroed.
  if (fork) {
    Run rt = r;
    rt.st = ctx->side;
    (void)hipEventRecord(ctx->ev_fork, r.st);
    (void)hipStreamWaitEvent(ctx->side, ctx->ev_fork, 0);
    zero_gradient_slots(r, grads);
    // Only the first layer's weights are prepared on this stream; those of the layers above are prepared on the side
    // stream ahead of the teacher's pass (which has slack before the loss needs it), so the quantized pass starts after
    // one layer's worth of that work instead of the whole module's.
    prepare_weights(r, params, 0, 1);
    if (ctx->L > 1) {
      prepare_weights(rt, params, 1, ctx->L);
      (void)hipEventRecord(ctx->ev_codes, ctx->side);
    }
    // the two passes are enqueued layer by layer in turn, so that both streams have work from the
    // start also when the caller's queue was empty
    for (int l = 0; l < ctx->L; ++l) {
      teacher_forward(rt, teacher, teacher_cache, x_fp, per_layer_fp, nullptr, l, l + 1);
      if (l == 1) (void)hipStreamWaitEvent(r.st, ctx->ev_codes, 0);
      student_forward(r, params, x_in, per_layer_q, l, l + 1, mix_fp, x_q, lambda);
    }
    (void)hipEventRecord(ctx->ev_join, ctx->side);
  } else {
    teacher_forward(r, teacher, teacher_cache, x_fp, per_layer_fp, nullptr);
    zero_gradient_slots(r, grads);
    prepare_weights(r, params);
    student_forward(r, params, x_in, per_layer_q, 0, -1, mix_fp, x_q, lambda);
  }
  if (fork) (void)hipStreamWaitEvent(r.st, ctx->ev_join, 0);
  const Update up{params, adam_m, adam_v, adam_arg(ctx, step_index, lr), grads_out != nullptr, fork ? ctx->side : nullptr,
                  ctx->ev_layer.data(), ctx->ev_ready.data(), ctx->ev_done.data(), ctx->ev_join};
  student_backward(r, params, x_in, per_layer_fp, per_layer_q, grads, loss_out, up);
  update_vectors(r, up, grads);
  return finish(ctx, "mrem_module_step");
}

// ------------------------------------------------------------------------------
// REM: the reconstruction step of ONE matrix product (Section 3.2, Eq. 2)
// ------------------------------------------------------------------------------
namespace {
struct RemPlan {
  size_t wt, wcodes, what, zcorr, xcodes, dy, dxh, partials, grads, total;
  int64_t n_vec;  // length of the flat vector [w | s_w | s_a, padded]
};
RemPlan rem_plan(int dt, int64_t T, int64_t N, int64_t K) {
  RemPlan p;
  Bump b;
  const size_t es = dt_size(dt);
  p.n_vec = ((N * K + N + 1 + 3) / 4) * 4;
  p.wt = b.take((size_t)N * K * es); p.wcodes = b.take((size_t)N * K * es); p.what = b.take((size_t)N * K * es);
  p.zcorr = b.take((size_t)N * 4);
  p.xcodes = b.take((size_t)T * K * es); p.dy = b.take((size_t)T * N * es); p.dxh = b.take((size_t)T * K * es);
  p.partials = b.take(2 * 2048 * 4);
  p.grads = b.take((size_t)p.n_vec * 4);
  p.total = b.off;
  return p;
}
}  // namespace

extern "C" int64_t mrem_rem_vector_count(int64_t N, int64_t K) { return (N < 1 || K < 1) ? -1 : ((N * K + N + 1 + 3) / 4) * 4; }
extern "C" size_t mrem_rem_workspace_bytes(const mrem_ctx* ctx, int64_t T, int64_t N, int64_t K) {
  if (!ctx || T < 1 || N < 1 || K < 1) return 0;
  return rem_plan(ctx->dt, T, N, K).total;
}

extern "C" mrem_status mrem_rem_step(mrem_ctx* ctx, int64_t T, int64_t N, int64_t K, float* vec, float* adam_m, float* adam_v,
                                     int64_t step_index, float lr, const float* w_fp, const void* a_fp, const void* a_q, float* loss_out,
                                     void* y_fp, void* y_q, float* grads_out, void* workspace, size_t workspace_bytes, void* hip_stream) {
  const char* who = "mrem_rem_step";
  if (!ctx) return fail(nullptr, MREM_EINVAL, std::string(who) + ": null context");
  if (T < 1 || N < 1 || K < 1 || T % 8 || N % 8 || K % 8 || T * std::max(N, K) > 0x7fffffff || N * K > 0x7fffffff)
    return fail(ctx, MREM_ESHAPE, std::string(who) + ": T, N, K must be positive multiples of 8 (products below 2^31)");
  if (ctx->cfg.w_bits == 0 || ctx->cfg.a_bits == 0) return fail(ctx, MREM_EINVAL, std::string(who) + ": both quantizer families must be on");
  if (step_index < 1) return fail(ctx, MREM_EINVAL, std::string(who) + ": step_index is 1-based");
  REQUIRE_PTR(vec, who); REQUIRE_PTR(adam_m, who); REQUIRE_PTR(adam_v, who); REQUIRE_PTR(w_fp, who); REQUIRE_PTR(a_fp, who);
  REQUIRE_PTR(a_q, who); REQUIRE_PTR(loss_out, who); REQUIRE_PTR(y_fp, who); REQUIRE_PTR(y_q, who); REQUIRE_PTR(workspace, who);
  if (grads_out && !aligned16(grads_out)) return fail(ctx, MREM_EINVAL, std::string(who) + ": grads_out misaligned");
  const RemPlan p = rem_plan(ctx->dt, T, N, K);
  if (workspace_bytes < p.total) return fail(ctx, MREM_EWORKSPACE, std::string(who) + ": workspace too small");
  const int dt = ctx->dt;
  hipStream_t st = (hipStream_t)hip_stream;
  char* ws = (char*)workspace;
  float* w = vec;
  float* sw = vec + N * K;
  float* sa = vec + N * K + N;
  float* grads = grads_out ? grads_out : reinterpret_cast<float*>(ws + p.grads);
  float* parts = reinterpret_cast<float*>(ws + p.partials);
  GemmProfile* prof = &ctx->prof;
  // full-precision product  y = a W^T  on the original weights
  convert_f32(dt, w_fp, ws + p.wt, N * K, st);
  gemm_nt(dt, a_fp, (int)K, ws + p.wt, (int)K, y_fp, (int)N, (int)T, (int)N, (int)K, Epilogue(), st, prof);
  // quantized product  y^ = Q(a) Q(w)^T: codes of both operands, the two steps in the epilogue
  WeightJob wj;
  wj.w = w; wj.sw = sw; wj.codes = ws + p.wcodes; wj.what = ws + p.what; wj.zcorr = reinterpret_cast<float*>(ws + p.zcorr); wj.codes8 = nullptr;
  wj.N = (int)N; wj.K = (int)K;
  weight_prepare(dt, &wj, 1, ctx->cfg.w_bits, st);
  QArg qa;
  qa.on = 1; qa.s = sa; qa.qp = (float)((1 << (ctx->cfg.a_bits - 1)) - 1); qa.qn = -qa.qp;
  act_quantize(dt, a_q, ws + p.xcodes, T * K, qa, st);
  Epilogue e;
  e.alpha = sa; e.col_scale = sw;
  gemm_nt(dt, ws + p.xcodes, (int)K, ws + p.wcodes, (int)K, y_q, (int)N, (int)T, (int)N, (int)K, e, st, prof);
  // Eq. 2 and its gradient with respect to y^
  const float scale = ctx->cfg.loss_mean ? 1.0f / (float)((double)T * (double)N) : 1.0f;
  const int nl = mse_grad(dt, y_q, y_fp, ws + p.dy, T * N, scale, parts, st);
  // straight-through backward: d w^ = dy^T a^ (the update kernel applies the mask and forms ds_w), d a^ = dy W^ for ds_a
  Epilogue ew;
  ew.alpha = sa; ew.out_f32 = 1;
  gemm(dt, 1, 1, ws + p.dy, (int)N, ws + p.xcodes, (int)K, grads, (int)K, (int)N, (int)K, (int)T, ew, st, prof);
  gemm(dt, 0, 1, ws + p.dy, (int)N, ws + p.what, (int)K, ws + p.dxh, (int)K, (int)T, (int)K, (int)N, Epilogue(), st, prof);
  const int ns = quant_bwd_reduce(dt, ws + p.dxh, a_q, T * K, qa, parts + 2048, st);
  ReduceJob jobs[2];
  jobs[0].partials = parts; jobs[0].nparts = nl; jobs[0].width = 1; jobs[0].begin = 0; jobs[0].len = 1; jobs[0].out = loss_out; jobs[0].scale = scale;
  jobs[1].partials = parts + 2048; jobs[1].nparts = ns; jobs[1].width = 1; jobs[1].begin = 0; jobs[1].len = 1; jobs[1].out = grads + N * K + N;
  reduce_jobs(jobs, 2, st);
  // AdamW on w (decay) and s_w, then on s_a (no decay, floor)
  const AdamArg a = adam_arg(ctx, step_index, lr);
  AdamJob aj;
  aj.w = w; aj.sw = sw; aj.g_w = grads; aj.g_sw = grads + N * K; aj.m_w = adam_m; aj.v_w = adam_v; aj.m_sw = adam_m + N * K; aj.v_sw = adam_v + N * K;
  aj.z_in = nullptr; aj.db = nullptr; aj.N = (int)N; aj.K = (int)K;
  adam_matrix(&aj, 1, ctx->cfg.w_bits, a, grads_out != nullptr, ctx->cfg.per_channel ? 0 : 1, st);
  AdamArg nodecay = a;
  nodecay.wd = 0.f;
  const VecJob vj{N * K + N, 1, 1};
  adam_vector(vec, grads, adam_m, adam_v, &vj, 1, nodecay, st);
  return finish(ctx, who);
}

extern "C" mrem_status mrem_mix_inputs(mrem_ctx* ctx, const void* x_fp, const void* x_q, float lambda, void* out, int64_t n,
                                       void* hip_stream) {
  if (!ctx) return fail(nullptr, MREM_EINVAL, "mrem_mix_inputs: null context");
  REQUIRE_PTR(x_fp, "mrem_mix_inputs");
  REQUIRE_PTR(x_q, "mrem_mix_inputs");
  REQUIRE_PTR(out, "mrem_mix_inputs");
  if (n < 1) return fail(ctx, MREM_ESHAPE, "mrem_mix_inputs: n must be >= 1");
  if (!(lambda >= 0.f && lambda <= 1.f)) return fail(ctx, MREM_EINVAL, "mrem_mix_inputs: lambda must be in [0,1]");
  axpby(ctx->dt, x_fp, x_q, lambda, 1.f - lambda, out, n, (hipStream_t)hip_stream);
  return finish(ctx, "mrem_mix_inputs");
}

extern "C" mrem_status mrem_profile_gemm_begin(mrem_ctx* ctx) {
  if (!ctx) return fail(nullptr, MREM_EINVAL, "mrem_profile_gemm_begin: null context");
  gemm_profile_begin(&ctx->prof);
  return MREM_OK;
}
extern "C" mrem_status mrem_profile_gemm_end(mrem_ctx* ctx, double* ms, double* flops, int64_t* launches) {
  if (!ctx || !ms || !flops || !launches) return fail(ctx, MREM_EINVAL, "mrem_profile_gemm_end: null argument");
  return gemm_profile_end(&ctx->prof, ms, flops, launches) == 0 ? MREM_OK : fail(ctx, MREM_EHIP, "mrem_profile_gemm_end: event query failed");
}

extern "C" int32_t mrem_profile_kernel_count(const mrem_ctx* ctx) { return ctx ? (int32_t)ctx->prof.stats.size() : -1; }
extern "C" mrem_status mrem_profile_kernel_get(const mrem_ctx* ctx, int32_t i, char* name, int32_t name_bytes, double* ms, double* bytes,
                                               int64_t* launches) {
  if (!ctx || !name || name_bytes < 1 || !ms || !bytes || !launches) return fail(ctx, MREM_EINVAL, "mrem_profile_kernel_get: null argument");
  if (i < 0 || i >= (int32_t)ctx->prof.stats.size()) return fail(ctx, MREM_EINVAL, "mrem_profile_kernel_get: no such entry");
  const KernelStat& k = ctx->prof.stats[(size_t)i];
  snprintf(name, (size_t)name_bytes, "%s", k.label);
  *ms = k.ms; *bytes = k.bytes; *launches = k.launches;
  return MREM_OK;
}

extern "C" mrem_status mrem_set_nonfinite_flag(mrem_ctx* ctx, int32_t* device_flag) {
  if (!ctx) return fail(nullptr, MREM_EINVAL, "mrem_set_nonfinite_flag: null context");
  if (device_flag && (reinterpret_cast<uintptr_t>(device_flag) & 3u)) return fail(ctx, MREM_EINVAL, "mrem_set_nonfinite_flag: misaligned flag");
  ctx->nonfinite_flag = device_flag;
  return MREM_OK;
}
extern "C" mrem_status mrem_check_nonfinite(mrem_ctx* ctx, void* hip_stream) {
  if (!ctx) return fail(nullptr, MREM_EINVAL, "mrem_check_nonfinite: null context");
  if (!ctx->nonfinite_flag) return fail(ctx, MREM_EINVAL, "mrem_check_nonfinite: no flag has been set");
  int32_t host = 0;
  if (hipStreamSynchronize((hipStream_t)hip_stream) != hipSuccess ||
      hipMemcpy(&host, ctx->nonfinite_flag, sizeof(host), hipMemcpyDeviceToHost) != hipSuccess)
    return fail(ctx, MREM_EHIP, "mrem_check_nonfinite: cannot read the flag");
  if (host) return fail(ctx, MREM_ENONFINITE, "a step since the flag was last cleared produced a non-finite loss");
  return MREM_OK;
}

// ------------------------------------------------------------------------------
// schedules (host arithmetic) and the input queue of Algorithm 1
// ------------------------------------------------------------------------------
extern "C" double mrem_schedule_lr(double lr0, int64_t t, int64_t total) {
  if (total < 1 || t < 0) return 0.0;
  return lr0 * (1.0 - (double)t / (double)total);
}
extern "C" double mrem_schedule_lambda(int64_t t, int64_t tf_steps) {
  if (tf_steps < 1 || t < 0) return 0.0;
  const double l = 1.0 - (double)t / (double)tf_steps;
  return l > 0.0 ? l : 0.0;
}

struct mrem_queue {
  int depth;            // readable entries
  size_t half_bytes, len_bytes;
  char* mem;            // device, caller-owned: (depth + 1) slots of [fp half | q half | lengths]
  int64_t published;    // entries handed over so far
  size_t slot_bytes() const { return 2 * half_bytes + len_bytes; }
};
static size_t round256(size_t b) { return (b + 255) & ~size_t(255); }
extern "C" size_t mrem_queue_bytes(int32_t depth, size_t half_bytes, size_t lengths_bytes) {
  if (depth < 1) return 0;
  return (size_t)(depth + 1) * (2 * round256(half_bytes) + round256(lengths_bytes));
}
extern "C" mrem_status mrem_queue_create(int32_t depth, size_t half_bytes, size_t lengths_bytes, void* device_mem, mrem_queue** out) {
  if (!out || !device_mem || !aligned16(device_mem)) return fail(nullptr, MREM_EINVAL, "mrem_queue_create: null or misaligned argument");
  if (depth < 1 || half_bytes < 1) return fail(nullptr, MREM_ESHAPE, "mrem_queue_create: depth and half_bytes must be >= 1");
  mrem_queue* q = new mrem_queue();
  q->depth = depth; q->half_bytes = round256(half_bytes); q->len_bytes = round256(lengths_bytes); q->mem = (char*)device_mem; q->published = 0;
  *out = q;
  return MREM_OK;
}
extern "C" void mrem_queue_destroy(mrem_queue* q) { delete q; }
extern "C" int32_t mrem_queue_size(const mrem_queue* q) { return q ? (int32_t)(q->published < q->depth ? q->published : q->depth) : -1; }
extern "C" mrem_status mrem_queue_write_slot(mrem_queue* q, void** fp, void** qd, void** lengths) {
  if (!q || !fp || !qd) return fail(nullptr, MREM_EINVAL, "mrem_queue_write_slot: null argument");
  char* slot = q->mem + (size_t)(q->published % (q->depth + 1)) * q->slot_bytes();
  *fp = slot; *qd = slot + q->half_bytes;
  if (lengths) *lengths = q->len_bytes ? slot + 2 * q->half_bytes : nullptr;
  return MREM_OK;
}
extern "C" mrem_status mrem_queue_push(mrem_queue* q, const void* fp, const void* qd, const void* lengths, size_t half_bytes,
                                       size_t lengths_bytes, void* hip_stream) {
  if (!q || !fp || !qd) return fail(nullptr, MREM_EINVAL, "mrem_queue_push: null argument");
  if (half_bytes > q->half_bytes || lengths_bytes > q->len_bytes) return fail(nullptr, MREM_ESHAPE, "mrem_queue_push: entry larger than a slot");
  void *dfp, *dq, *dl;
  (void)mrem_queue_write_slot(q, &dfp, &dq, &dl);
  hipStream_t st = (hipStream_t)hip_stream;
  bool ok = hipMemcpyAsync(dfp, fp, half_bytes, hipMemcpyDeviceToDevice, st) == hipSuccess &&
            hipMemcpyAsync(dq, qd, half_bytes, hipMemcpyDeviceToDevice, st) == hipSuccess;
  if (lengths && lengths_bytes) ok = ok && hipMemcpyAsync(dl, lengths, lengths_bytes, hipMemcpyDeviceToDevice, st) == hipSuccess;
  return ok ? MREM_OK : fail(nullptr, MREM_EHIP, "mrem_queue_push: copy failed");
}
extern "C" mrem_status mrem_queue_publish(mrem_queue* q) {
  if (!q) return fail(nullptr, MREM_EINVAL, "mrem_queue_publish: null queue");
  q->published += 1;
  return MREM_OK;
}
extern "C" mrem_status mrem_queue_entry(const mrem_queue* q, int32_t age, void** fp, void** qd, void** lengths) {
  if (!q || !fp || !qd) return fail(nullptr, MREM_EINVAL, "mrem_queue_entry: null argument");
  if (age < 0 || age >= mrem_queue_size(q)) return fail(nullptr, MREM_EINVAL, "mrem_queue_entry: no entry of that age");
  char* slot = q->mem + (size_t)((q->published - 1 - age) % (q->depth + 1)) * q->slot_bytes();
  *fp = slot; *qd = slot + q->half_bytes;
  if (lengths) *lengths = q->len_bytes ? slot + 2 * q->half_bytes : nullptr;
  return MREM_OK;
}
