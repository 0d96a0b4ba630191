/*
 * mrem.h -- C ABI of the MI355X (gfx950) implementation of one module-wise
 * reconstruction (MREM) training step.
 *
 * Paper: "Towards Efficient Post-training Quantization of Pre-trained Language
 * Models".  A module is a contiguous block of BERT encoder layers (Section 4.1).
 * One step (Algorithm 2) runs the full-precision module and its fake-quantized
 * copy forward, forms the module objective (Eq. 3), back-propagates through the
 * quantized copy with straight-through gradients (Section 3.1.1) and updates the
 * module's parameters and quantizer step sizes.
 *
 * General rules of this ABI
 *  - Every pointer marked "device" is HIP device memory owned by the caller.  The
 *    library never allocates, frees or retains device memory.  "host" pointers are
 *    ordinary host memory.
 *  - Boundary notes: quantizer placement (all six products of a layer) and the plain chain-rule step gradient
 *    are fixed, not options; lr and lambda are arguments of the step, their schedules are mrem_schedule_*.
 *  - All work is enqueued on the caller's hipStream_t (passed as void*, NULL = the
 *    default stream) or ordered with it: mrem_module_step runs the full-precision
 *    forward pass, the weight-gradient products and the update of each layer's
 *    weight matrices on a side stream that the context owns (default priority,
 *    created on the first step), forked from the caller's stream by events and
 *    joined to it before the loss and before the call's last kernels; to the caller
 *    the call behaves like work on its own stream.  Calls return without
 *    synchronising.
 *  - Arguments are validated on the host before anything is enqueued; a call that
 *    returns an error has had no effect on device memory.
 *  - Return value: MREM_OK or a negative mrem_status.  mrem_last_error() gives a
 *    human-readable message for the last failing call on that context (or for
 *    context-free calls, of the calling thread).
 *  - Matrices are row-major and contiguous.  Activations are [batch*seq, hidden]
 *    with the token index slowest.  Linear weights are [out_features, in_features].
 *  - Device pointers must be 16-byte aligned.
 *  - Calls on one context that overlap in time (different streams) race on the
 *    workspace; give each concurrent caller its own workspace.
 */
#ifndef MREM_H_
#define MREM_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mrem_ctx mrem_ctx; /* opaque, host memory only */

typedef enum {
  MREM_OK = 0,
  MREM_EINVAL = -1,     /* null pointer, bad enum, misaligned pointer */
  MREM_ESHAPE = -2,     /* sizes the kernels do not support */
  MREM_EWORKSPACE = -3, /* workspace smaller than mrem_workspace_bytes() */
  MREM_ENONFINITE = -4, /* mrem_check_nonfinite: a step produced a NaN or an infinite loss */
  MREM_EHIP = -5        /* a HIP runtime call failed */
} mrem_status;

typedef enum {
  MREM_BF16 = 0, /* activations and matmul operands stored as bfloat16, fp32 accumulation */
  MREM_FP32 = 1  /* check mode: everything fp32 */
} mrem_dtype;

/* Shape and hyper-parameters of one module.  (Section 4.1 for the partition into
 * modules; Section 3.1 for the bit-widths; Section 5.1.2 for the optimiser.) */
typedef struct {
  int32_t n_layers;  /* encoder layers in the module, 1..32 */
  int32_t hidden;    /* model width H, multiple of 8 */
  int32_t n_heads;   /* attention heads, H / n_heads in {32, 64, 128} */
  int32_t ffn;       /* feed-forward width F, multiple of 8 */
  int32_t max_seq;   /* largest seq passed to any call, <= 512 */
  int32_t max_batch; /* largest batch passed to any call */
  int32_t w_bits;    /* 2..8; 0 = weight quantizers off */
  int32_t a_bits;    /* 2..8; 0 = activation quantizers off */
  int32_t act_dtype; /* mrem_dtype */
  uint32_t loss_layer_mask; /* bit l set: layer l enters the sum of Eq. 3 */
  int32_t loss_mean; /* 1: each layer's term is the mean of squared differences; 0: the raw sum */
  float ln_eps;      /* LayerNorm epsilon (BERT: 1e-12) */
  float beta1, beta2, adam_eps, weight_decay; /* AdamW; decay applies to the four linear weights only */
  float step_floor;  /* step sizes are kept >= this after every update */
  int32_t per_channel; /* 1: one weight step per output channel; 0: one per weight matrix (Section 3.1's
                          default granularity): the step fields keep their [out_features] layout, all entries
                          of a matrix hold the same value and receive the same gradient (the sum over rows) */
} mrem_config;

/* Fields of one layer inside the flat fp32 parameter vector, in storage order;
 * layer l starts at l * (sum of all field sizes).  The teacher vector, the Adam
 * moment vectors and the gradient vector all use this same layout (the teacher's
 * step-size fields are ignored, so a copy of the initial student vector is a
 * valid teacher vector). */
typedef enum {
  MREM_F_W_QKV = 0, /* [3H,H] rows: query, key, value projections stacked */
  MREM_F_W_O,       /* [H,H]  attention output projection */
  MREM_F_W_1,       /* [F,H]  first feed-forward projection */
  MREM_F_W_2,       /* [H,F]  second feed-forward projection */
  MREM_F_B_QKV,     /* [3H] */
  MREM_F_B_O,       /* [H] */
  MREM_F_LN1_G,     /* [H] LayerNorm after attention: gain */
  MREM_F_LN1_B,     /* [H] shift */
  MREM_F_B_1,       /* [F] */
  MREM_F_B_2,       /* [H] */
  MREM_F_LN2_G,     /* [H] LayerNorm after the feed-forward network */
  MREM_F_LN2_B,     /* [H] */
  MREM_F_SW_QKV,    /* [3H] weight step sizes, one per output channel */
  MREM_F_SW_O,      /* [H] */
  MREM_F_SW_1,      /* [F] */
  MREM_F_SW_2,      /* [H] */
  MREM_F_S_A,       /* [8] activation step sizes: layer input, Q, K, softmax P, V, context, FFN input, GELU output */
  MREM_F_Z_A,       /* [8] fixed offsets of the two unsigned quantizers (P: 0, GELU output: its minimum); others 0 */
  MREM_F_COUNT
} mrem_field;

mrem_status mrem_create(const mrem_config* cfg /*host*/, mrem_ctx** out /*host*/);
void mrem_destroy(mrem_ctx* ctx);
const char* mrem_last_error(const mrem_ctx* ctx /* may be NULL */);

/* Layout queries (host only, no GPU work). Offsets and counts are in floats. */
int64_t mrem_param_count(const mrem_ctx* ctx);   /* student vector length */
int64_t mrem_teacher_count(const mrem_ctx* ctx); /* teacher vector length */
int64_t mrem_param_offset(const mrem_ctx* ctx, int32_t layer, int32_t field);
int64_t mrem_param_size(const mrem_ctx* ctx, int32_t field);
size_t mrem_workspace_bytes(const mrem_ctx* ctx, int32_t batch, int32_t seq);
/* bytes of the teacher cache written by mrem_teacher_prepare */
size_t mrem_teacher_cache_bytes(const mrem_ctx* ctx);

/*
 * Inspection aid (tests): where the forward pass of the quantized module leaves some of its
 * intermediate tensors inside the workspace.  Byte offset from the workspace pointer for the
 * given batch and seq, or -1 if that tensor does not exist in this configuration.  The contents
 * are those of the last mrem_module_forward / mrem_module_step on that workspace.
 *   MREM_WS_WCODES8 + i  int8 [N,K] codes of linear weight i (0 query/key/value, 1 attention output,
 *                        2 first, 3 second feed-forward projection): Eq. 1 applied to the current
 *                        parameters; present when the forward products run on int8 codes
 *                        (bf16 storage, both bit widths on, hidden and ffn multiples of 128, batch*seq
 *                        a multiple of 128)
 *   MREM_WS_WCODES + i   the same codes as integer values of the activation type; present otherwise
 *   MREM_WS_QKV          act_dtype [batch*seq, 3*hidden]: output of the query/key/value projection
 *   MREM_WS_XCODES8      int8 [batch*seq, hidden]: codes of the layer input (when int8 products are in use)
 */
typedef enum {
  MREM_WS_WCODES8 = 0, /* .. 3 */
  MREM_WS_WCODES = 4,  /* .. 7 */
  MREM_WS_QKV = 8,
  MREM_WS_XCODES8 = 9
} mrem_ws_item;
int64_t mrem_workspace_offset(const mrem_ctx* ctx, int32_t batch, int32_t seq, int32_t layer, int32_t item);

/*
 * mrem_quantize -- the uniform quantizer of Section 3.1, Eq. 1:
 *   codes[n,k] = nearest_even( clamp( w[n,k] / s, -Qp, Qp ) ),  Qp = 2^(bits-1) - 1,
 * with the quotient formed as one IEEE fp32 division; s = scale[n] with per_channel = 1 (one step per
 * output channel, the granularity of the module step) or s = scale[0] with per_channel = 0 (one step
 * for the whole tensor, Section 3.1's default granularity).
 *   w      device fp32 [N,K]             (in)
 *   scale  device fp32 [N] or [1]        (in; out if init_scale != 0)
 *   codes  device int8 [N,K]             (out)
 * init_scale != 0 first sets the step(s) to max |w| / Qp over the channel or the tensor (one fp32
 * division; all zeros give the smallest positive normal float).  bits in 2..8.
 * Errors: MREM_EINVAL (null/misaligned pointer, bits, per_channel), MREM_ESHAPE (N or K < 1).
 */
mrem_status mrem_quantize(const float* w, int64_t N, int64_t K, int32_t bits, int32_t per_channel, int32_t init_scale,
                          float* scale, int8_t* codes, void* hip_stream);

/*
 * mrem_module_init_steps -- initial weight step sizes of every layer of a student
 * vector: for each of the four linear weights, step[n] = max_k |w[n,k]| / Qp with
 * Qp = 2^(w_bits-1) - 1 (so that the largest weight of a channel maps to the last
 * level of the integer set of Eq. 1).  Writes only the four SW fields of params.
 * Error if w_bits = 0.
 */
mrem_status mrem_module_init_steps(mrem_ctx* ctx, float* params, void* hip_stream);

/*
 * mrem_teacher_prepare -- converts the teacher's fp32 parameter vector into the
 * operand format of the forward kernels (the full-precision module of Algorithm 2
 * is frozen, so this runs once).  teacher: device fp32 [mrem_teacher_count].
 * cache: device, mrem_teacher_cache_bytes() bytes, written.
 */
mrem_status mrem_teacher_prepare(mrem_ctx* ctx, const float* teacher, void* cache, void* hip_stream);

/*
 * mrem_module_calibrate -- initial clipping ranges of the activation quantizers
 * from the full-precision module's activations on one batch (Section 5.1.2 uses a
 * learned-step quantizer whose step is initialised from the data): for the six
 * symmetric quantizers s = max|a| / Qp, for the softmax probabilities z = 0 and
 * s = max(P) / (2^b - 1), for the GELU output z = min(g), s = (max(g) - z) / (2^b - 1).
 * Writes the S_A and Z_A fields of every layer of params; nothing else is touched.
 *   x_fp     device act_dtype [batch, seq, hidden]
 *   seqlens  device int32 [batch] valid keys per sequence, each in 1..seq, or NULL (no
 *            padding).  The values live on the device and are not checked: a sequence
 *            without a valid key has no softmax and yields NaN in its rows.
 */
mrem_status mrem_module_calibrate(mrem_ctx* ctx, float* params, const float* teacher, const void* teacher_cache,
                                  const void* x_fp, const int32_t* seqlens, int32_t batch, int32_t seq,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * mrem_module_forward -- the two forward passes of Algorithm 2: the full-precision
 * module on x_fp and the quantized module on x_q (Section 3.1: both operands of
 * every matrix multiplication are quantized; LayerNorm, residuals and biases are not).
 *   params         device fp32 [mrem_param_count]  (in)
 *   teacher        device fp32 [mrem_teacher_count] (in: biases and LayerNorm parameters)
 *   teacher_cache  device, from mrem_teacher_prepare (in: matrices)
 *   x_fp, x_q      device act_dtype [batch, seq, hidden]; may alias
 *   seqlens        device int32 [batch], each in 1..seq, or NULL (as for mrem_module_calibrate)
 *   per_layer_fp, per_layer_q  device act_dtype [n_layers, batch, seq, hidden] (out):
 *                  the layer outputs f_l and f^_l of Eq. 3; the last slice is the
 *                  module output handed to the next module.  Either may be NULL to
 *                  skip that pass.
 */
mrem_status mrem_module_forward(mrem_ctx* ctx, const float* params, const float* teacher, const void* teacher_cache,
                                const void* x_fp, const void* x_q, const int32_t* seqlens, int32_t batch,
                                int32_t seq, void* per_layer_fp, void* per_layer_q, void* workspace,
                                size_t workspace_bytes, void* hip_stream);

/*
 * mrem_module_forward_static -- mrem_module_forward for callers that cannot allocate device
 * memory and have no workspace to pass: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments without the workspace pair, same kernels,
 * same results; the scratch memory is a static device array of MREM_STATIC_SCRATCH_BYTES that
 * the library's code object carries (each GPU the library runs on holds its copy until the
 * process ends).  The call allocates and frees nothing, on the device or through any library.
 * Error MREM_EWORKSPACE if mrem_workspace_bytes(ctx, batch, seq) exceeds
 * MREM_STATIC_SCRATCH_BYTES (nothing is enqueued).  All calls on one GPU share that GPU's
 * array: calls that overlap in time on one GPU (different streams or threads) race on it.
 */
#define MREM_STATIC_SCRATCH_BYTES (64u << 20)
size_t mrem_static_scratch_bytes(void); /* MREM_STATIC_SCRATCH_BYTES of the loaded library */
mrem_status mrem_module_forward_static(mrem_ctx* ctx, const float* params, const float* teacher, const void* teacher_cache,
                                       const void* x_fp, const void* x_q, const int32_t* seqlens, int32_t batch,
                                       int32_t seq, void* per_layer_fp, void* per_layer_q, void* hip_stream);

/*
 * mrem_module_step -- one full iteration of Algorithm 2: the input mixing of Eq. 4, both forward
 * passes, the loss of Eq. 3, the straight-through backward pass
 * confined to the module (Section 4.2), and one AdamW update with rate lr of every
 * trainable parameter and every step size.
 *   params, adam_m, adam_v   device fp32 [mrem_param_count]  (in/out)
 *   step_index               1-based count of this update (bias correction)
 *   lr                       learning rate of this step (mrem_schedule_lr gives the linear decay)
 *   lambda                   in [0,1], Eq. 4: the quantized module reads lambda * x_fp + (1 - lambda) * x_q
 *                            (annealed teacher forcing, Section 4.2.1; mrem_schedule_lambda); formed and stored
 *                            by the kernel that quantizes the first layer's input.  0: x_q as it is
 *   loss_out                 device fp32 [1 + n_layers] (out): total, then per layer
 *   per_layer_fp, per_layer_q  device act_dtype [n_layers, batch, seq, hidden] (out, required)
 *   grads_out                device fp32 [mrem_param_count] or NULL (out): the gradients
 *                            that were applied (Z_A slots are written as 0)
 * A context must be used from the device that was current at its first step.
 */
mrem_status mrem_module_step(mrem_ctx* ctx, float* params, float* adam_m, float* adam_v, int64_t step_index,
                             float lr, float lambda, const float* teacher, const void* teacher_cache, const void* x_fp,
                             const void* x_q, const int32_t* seqlens, int32_t batch, int32_t seq,
                             float* loss_out, void* per_layer_fp, void* per_layer_q, float* grads_out,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * mrem_rem_step -- reconstruction error minimisation of ONE matrix product (Section 3.2, Eq. 2; the baseline
 * that module-wise reconstruction generalises): with a^ = Q(a_q) (symmetric, one step s_a) and w^ = Q(w) (one
 * step per output channel, or one per matrix with per_channel = 0),
 *   y = a_fp w_fp^T,  y^ = a^ w^^T,  loss = mean (or sum, loss_mean = 0) of (y^ - y)^2,
 * straight-through gradients for w, s_w and s_a, one AdamW update (decay on w only; steps kept >= step_floor).
 * Bit widths, activation type and optimiser constants are the context's; no bias, as in Eq. 2.
 *   vec, adam_m, adam_v  device fp32 [mrem_rem_vector_count(N, K)] (in/out): w [N,K], then s_w [N], then s_a [1], zero padding
 *   w_fp     device fp32 [N,K]        the frozen original weights
 *   a_fp,a_q device act_dtype [T,K]   inputs of the full-precision and of the quantized product (may alias)
 *   loss_out device fp32 [1]; y_fp, y_q device act_dtype [T,N] (out); grads_out device fp32 like vec, or NULL
 * T, N, K positive multiples of 8.  Workspace: mrem_rem_workspace_bytes(ctx, T, N, K).
 */
int64_t mrem_rem_vector_count(int64_t N, int64_t K);
size_t mrem_rem_workspace_bytes(const mrem_ctx* ctx, int64_t T, int64_t N, int64_t K);
mrem_status mrem_rem_step(mrem_ctx* ctx, int64_t T, int64_t N, int64_t K, float* vec, float* adam_m, float* adam_v, int64_t step_index,
                          float lr, const float* w_fp, const void* a_fp, const void* a_q, float* loss_out, void* y_fp, void* y_q,
                          float* grads_out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * mrem_mix_inputs -- annealed teacher forcing, Eq. 4: out = lambda * x_fp + (1 - lambda) * x_q,
 * elementwise over n values of act_dtype (device). out may alias x_q.
 */
mrem_status mrem_mix_inputs(mrem_ctx* ctx, const void* x_fp, const void* x_q, float lambda, void* out, int64_t n,
                            void* hip_stream);

/*
 * Non-finite detection.  mrem_set_nonfinite_flag gives the context a device int32 (caller-owned, cleared
 * by the caller; NULL switches the check off): every mrem_module_step on the context then sets it to 1
 * when its total loss is a NaN or infinite -- a non-finite value anywhere in a layer output reaches that
 * layer's term of Eq. 3.  The flag is sticky and costs nothing on the host.  mrem_check_nonfinite waits for
 * the stream, reads the flag and returns MREM_ENONFINITE if it is set (MREM_EINVAL if no flag was given).
 */
mrem_status mrem_set_nonfinite_flag(mrem_ctx* ctx, int32_t* device_flag);
mrem_status mrem_check_nonfinite(mrem_ctx* ctx, void* hip_stream);

/*
 * Schedules (host arithmetic only).  Section 5.1.2: linearly decayed rate lr0 * (1 - t / total),
 * t = 0 .. total-1.  Section 4.2.1: lambda_t = max(1 - t / tf_steps, 0); 0 when tf_steps < 1.
 */
double mrem_schedule_lr(double lr0, int64_t t, int64_t total);
double mrem_schedule_lambda(int64_t t, int64_t tf_steps);

/*
 * Input queue of Algorithm 1 (Section 4.2): the last `depth` pairs (f, f^) of module outputs, first in
 * first out, with the sequence lengths of their batch, in device memory that the caller owns
 * (mrem_queue_bytes).  The ring has depth + 1 slots: one is being written during a step while the
 * depth published ones stay readable, so a reader of the oldest entry never sees a slot that its
 * producer is overwriting.  Which entry a consumer samples is the caller's draw (an age, 0 = newest).
 *   mrem_queue_push      copies one entry (device to device, on the stream) into the write slot
 *   mrem_queue_write_slot  pointers of the write slot, for a producer that writes in place
 *   mrem_queue_publish   hands the written slot over (host bookkeeping; call once the step's work is enqueued
 *                        and ordered before the consumers' reads)
 *   mrem_queue_entry     pointers of the entry of the given age, 0 <= age < mrem_queue_size
 * The handle is host memory; calls on one queue from several threads need the caller's lock.
 */
typedef struct mrem_queue mrem_queue;
size_t mrem_queue_bytes(int32_t depth, size_t half_bytes, size_t lengths_bytes);
mrem_status mrem_queue_create(int32_t depth, size_t half_bytes, size_t lengths_bytes, void* device_mem, mrem_queue** out);
void mrem_queue_destroy(mrem_queue* q);
int32_t mrem_queue_size(const mrem_queue* q);
mrem_status mrem_queue_write_slot(mrem_queue* q, void** fp, void** qd, void** lengths);
mrem_status mrem_queue_push(mrem_queue* q, const void* fp, const void* qd, const void* lengths /* may be NULL */, size_t half_bytes,
                            size_t lengths_bytes, void* hip_stream);
mrem_status mrem_queue_publish(mrem_queue* q);
mrem_status mrem_queue_entry(const mrem_queue* q, int32_t age, void** fp, void** qd, void** lengths /* may be NULL */);

/*
 * Measurement aid (not part of the method): between mrem_profile_gemm_begin(ctx) and
 * mrem_profile_gemm_end(ctx, ...) every matrix-product kernel launch of that context carries a pair of HIP
 * events (kernel begin, kernel end), and its mrem_module_step keeps all its work on the caller's stream so
 * that every product runs alone.  _end waits for the events and returns, for products on bf16 operands in
 * element [0] and for products on int8 operands in element [1] of each host array: the summed kernel time
 * in milliseconds, the summed 2*M*N*K of those launches and their number.  The state lives in the context.
 */
mrem_status mrem_profile_gemm_begin(mrem_ctx* ctx);
mrem_status mrem_profile_gemm_end(mrem_ctx* ctx, double ms[2] /*host*/, double flops[2] /*host*/, int64_t launches[2] /*host*/);
/*
 * The same timed interval also records the bandwidth-bound kernels (LayerNorm, quantizer, GELU, weight-code and
 * update kernels), each launch with its algorithmic bytes: what it must read and write at least.  After
 * mrem_profile_gemm_end: mrem_profile_kernel_count entries, each a kernel name (copied into name[name_bytes]),
 * the summed kernel time in milliseconds, the summed algorithmic bytes and the number of launches.
 */
int32_t mrem_profile_kernel_count(const mrem_ctx* ctx);
mrem_status mrem_profile_kernel_get(const mrem_ctx* ctx, int32_t i, char* name /*host*/, int32_t name_bytes, double* ms /*host*/,
                                    double* bytes /*host*/, int64_t* launches /*host*/);

#ifdef __cplusplus
}
#endif
#endif /* MREM_H_ */
