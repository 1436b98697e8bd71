/*
 * qc.h - C ABI of the MI355X (gfx950) implementation of the quantised + cached
 * DiT sampler step of "Q&C: When Quantization Meets Cache in Efficient Image
 * Generation" (arXiv 2503.02508).
 *
 * Conventions (all entry points)
 *   - return value: QC_OK (0) or a negative qc_status; qc_last_error() gives a
 *     thread-local text for the last failure.  No exceptions, no aborts.
 *   - "dev" pointers are device (HBM) pointers owned by the caller and only
 *     borrowed for the call; "host" pointers are ordinary host memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Unless stated otherwise a call only enqueues work on that stream.
 *   - tensors are row-major and dense.  Activation codes are int8 holding the
 *     paper's unsigned code minus 128 (Eq. 1: q in [0, 255]); a zero point is
 *     passed in the paper's unsigned convention (0..255) and shifted inside.
 *   - weight matrices are [N, K] (one row per output channel).  4-bit weights
 *     are packed two per byte along K: element 2j in bits 0-3, element 2j+1 in
 *     bits 4-7, two's complement.
 *   - the library never allocates device memory: everything a context needs
 *     lives in one caller-provided arena.
 *   - argument checks run before any device call.
 *   - a context is not thread-safe: calls on one context must not overlap, and
 *     work enqueued through one context on different streams must be ordered by
 *     the caller (the context owns one workspace).  The denoiser entry points
 *     may run parts of a call on internal streams of the context; these fork
 *     from and join back into `stream`, so the caller only ever orders against
 *     `stream`.  Different contexts are independent.
 */
#ifndef QC_H_
#define QC_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum qc_status {
  QC_OK = 0,
  QC_ERR_NULL = -1,        /* a required pointer is NULL                      */
  QC_ERR_SHAPE = -2,       /* zero / negative / inconsistent dimension         */
  QC_ERR_ALIGN = -3,       /* pointer or leading dimension not 16-byte aligned */
  QC_ERR_RANGE = -4,       /* scale <= 0 or not finite, zero point outside 0..255, index out of range */
  QC_ERR_STATE = -5,       /* e.g. cached block before anything was stored     */
  QC_ERR_WORKSPACE = -6,   /* arena too small                                  */
  QC_ERR_UNSUPPORTED = -7, /* shape the kernels do not cover                   */
  QC_ERR_HIP = -8          /* a HIP runtime call failed                        */
} qc_status;

enum { QC_FULL = 0, QC_CACHED = 1 };                 /* block / step mode          */
enum { QC_CACHE_ATTN = 0, QC_CACHE_MLP = 1 };        /* which cached module output */
enum { QC_SITE_ADA = 0, QC_SITE_QKV = 1, QC_SITE_PROJ = 2, QC_SITE_FC1 = 3, QC_SITE_FC2 = 4, QC_NUM_SITES = 5 };
enum {                                               /* qc_workspace_ptr selectors */
  QC_WS_TOKENS = 0,   /* float (bfloat16 under QC_STREAM_BF16) [B, T, D]  residual stream of the last denoiser call */
  QC_WS_QACT_LN = 1,  /* int8   [B*T, D]   codes produced by the last LN+modulate+quantise */
  QC_WS_QACT_ATTN = 2,/* int8   [B*T, D]   codes of the last attention output              */
  QC_WS_QACT_MLP = 3, /* int8   [B*T, R]   codes of the last GELU output                    */
  QC_WS_QKV = 4,      /* float  [B*T, 3D]  last QKV projection (only with qc_keep_qkv_f32)          */
  QC_WS_MOD = 5,      /* float  [L, R, 6D] adaLN modulation of every block; R = max(512, max_batch) rows,
                         row = step slot of the prepared window * batch + batch element           */
  QC_WS_COND = 6,     /* float  [R, D]     conditioning vectors c, same rows                        */
  QC_WS_EPS = 7,      /* float  [B, C, H, W] last noise estimate                            */
  QC_WS_QKV_HEADS = 8 /* float  the copy of the last QKV projection the attention kernel reads: Q [B, H, T, d], then
                         K [B, H, T, d], then V transposed [B, H, dp, Tp] (d = D / H, dp = d rounded up to 16, Tp = T
                         rounded up to 64; the keys of each group of 32 interleaved in units of 4: key t sits at
                         (t & ~31) | (((u & 3) << 1 | u >> 2) << 2) | (t & 3), u = (t >> 2) & 7); B = max_batch   */
};

/* The network: a class-conditional DiT (the architecture the paper evaluates,
 * Experimental Settings) with `depth` adaLN-Zero blocks. */
typedef struct qc_model_desc {
  int32_t depth, hidden, heads, mlp_dim;
  int32_t patch, latent_c, latent_h, latent_w;
  int32_t num_classes;     /* label table has num_classes + 1 rows; the last is the null label */
  int32_t freq_dim;        /* width of the sinusoidal timestep embedding (256)                 */
  int32_t weight_bits;     /* 8 or 4 (Tables 1 and 2: W8A8, W4A8)                              */
  int32_t cache_interval;  /* N of the cache rule: step i is recomputed iff i mod N == 0       */
} qc_model_desc;

typedef struct qc_block_weights_f32 {   /* dev pointers, fp32, [N, K] / [N] */
  const float *ada_w, *ada_b;     /* [6D, D], [6D]  adaLN projection */
  const float *qkv_w, *qkv_b;     /* [3D, D], [3D]                   */
  const float *proj_w, *proj_b;   /* [D, D],  [D]                    */
  const float *fc1_w, *fc1_b;     /* [R, D],  [R]                    */
  const float *fc2_w, *fc2_b;     /* [D, R],  [D]                    */
} qc_block_weights_f32;

typedef struct qc_weights_f32 {
  const float *patch_w, *patch_b;   /* dev [D, C*p*p] (features ordered c, ph, pw), [D] */
  const float *pos;                 /* dev [T, D]                                      */
  const float *t_w1, *t_b1;         /* dev [D, freq_dim], [D]                           */
  const float *t_w2, *t_b2;         /* dev [D, D], [D]                                  */
  const float *label_table;         /* dev [num_classes + 1, D]                         */
  const float *fada_w, *fada_b;     /* dev [2D, D], [2D]  final-layer adaLN (shift, scale) */
  const float *flin_w, *flin_b;     /* dev [p*p*2C, D], [p*p*2C] (features ordered ph, pw, c) */
  const qc_block_weights_f32 *blocks; /* HOST array of `depth` entries holding dev pointers */
} qc_weights_f32;

typedef struct qc_ctx qc_ctx;

const char *qc_last_error(void);

/* ---------------------------------------------------------------- context */

/* Bytes of device arena a context needs for effective batches up to max_batch
 * (the effective batch is twice the number of latents under guidance). */
int qc_arena_bytes(const qc_model_desc *desc, int max_batch, size_t *bytes_out);

/* Creates a context inside `arena` (dev, 256-byte aligned, arena_bytes >=
 * qc_arena_bytes).  The arena stays owned by the caller and must outlive the
 * context.  Holds: quantised weights, per-site activation parameters, the
 * attention / MLP output cache (two fp32 [B, T, D] tensors per block) and
 * workspace. */
int qc_create(const qc_model_desc *desc, void *arena, size_t arena_bytes, int max_batch, qc_ctx **out);
int qc_destroy(qc_ctx *ctx);

/* Quantises the five linears of every block on the device ("channel-wise"
 * weights, Comparison on Performance section: one symmetric scale per output
 * row, s_w = max|row| / qmax, codes clip(round(w / s_w), -qmax, qmax), qmax =
 * 127 or 7; an all-zero row gets s_w = 1), stores row sums of the codes, and
 * copies the floating-point embedders / final layer into the arena. */
int qc_load_weights_f32(qc_ctx *ctx, const qc_weights_f32 *w, void *stream);

/* Static activation quantiser parameters of one site (Eq. 1-3; "tensor-wise"
 * activations).  scale > 0 finite, zero_point in 0..255.  Synchronous. */
int qc_set_act_qparams(qc_ctx *ctx, int block, int site, float scale, int zero_point);
int qc_get_act_qparams(const qc_ctx *ctx, int block, int site, float *scale, int *zero_point);

/* Derives every site's (s, z) from calibration data (Eq. 2-3): runs the
 * un-quantised fp32 network (weights w, the same structure that was given to
 * qc_load_weights_f32) on n inputs, one at a time, takes the global min l and
 * max u of each site's input, widens [l, u] to contain 0, s = (u - l) / 255,
 * z = round(-l / s), and installs them as with qc_set_act_qparams.
 * x: dev [n, C, H, W]; t, y: HOST [n].  Synchronous. */
int qc_calibrate_minmax(qc_ctx *ctx, const qc_weights_f32 *w, const float *x, const int32_t *t, const int32_t *y, int n,
                        void *stream);

/* ------------------------------------------------------- single operations */

/* Eq. 1 with b = 8: q[i] = clip(round(x[i] / scale) + zero_point, 0, 255) - 128,
 * round-half-to-even, x / scale an IEEE fp32 division.  x, q: dev, n elements. */
int qc_quantize_act(const float *x, int8_t *q, size_t n, float scale, int zero_point, void *stream);

/* Channel-wise weight quantiser (as in qc_load_weights_f32) for one matrix.
 * w: dev fp32 [N, K]; qw: dev int8 [N, K] or packed [N, K/2] for bits = 4;
 * w_scale: dev [N]; wsum: dev [N] (sum over k of the codes).  K % 16 == 0. */
int qc_quantize_weight(const float *w, int N, int K, int bits, void *qw, float *w_scale, int32_t *wsum, void *stream);

/* Quantised linear layer on codes (Eq. 1 applied to both operands, weights
 * channel-wise, activations tensor-wise):
 *   acc[m, n] = sum_k qx[m, k] * qw[n, k]                       (int32, exact)
 *   y[m, n]   = x_scale * w_scale[n] * (acc[m, n] - (x_zp - 128) * wsum[n]) + bias[n]
 * qx: dev int8 [M, K]; qw: dev [N, K] int8 (weight_bits 8) or [N, K/2] packed
 * (weight_bits 4); wsum, w_scale, bias: dev [N] (bias may be NULL); y: dev fp32
 * [M, N]; acc_or_null: dev int32 [M, N] receiving the raw accumulators, or
 * NULL.  K % 16 == 0; pointers 16-byte aligned. */
int qc_w8a8_linear(const int8_t *qx, const void *qw, const int32_t *wsum, const float *w_scale, const float *bias,
                   float x_scale, int x_zp, int M, int N, int K, int weight_bits,
                   float *y, int32_t *acc_or_null, void *stream);

/* Variance compensation, Eq. 10, channel-wise: x <- mu + K_t * (x - mu) on
 * x: dev [B, C, H, W] in place; K_t: dev [C]; mu_or_null: dev [C], or NULL to
 * use the spatial mean of each (sample, channel) plane (then the plane mean is
 * preserved and its variance scales by K_t^2, Eq. 9). */
int qc_vc_correct(float *x, const float *K_t, const float *mu_or_null, int B, int C, int H, int W, void *stream);

/* VC factors of one timestep ("Variance Align for Exposure Bias" section, the
 * argmin objective that follows Eq. 10): for every channel c the K that
 * minimises  sum ((x~ - x') / x')^2 + sum (x~ - x')^2,  x~ = mu + K (x^ - mu),
 * over all elements of channel c in the batch; mu is the spatial mean of the
 * x^ plane the element lies in.  The exact minimiser is computed,
 * K = sum d (x' - mu) w / sum d^2 w,  d = x^ - mu,  w = 1 + 1 / (x'^2 + eps)
 * (the closed form printed after the objective is this one for mu = 0, eps = 0);
 * a channel with d == 0 everywhere gets K = 1.  fp64 accumulation.
 * x_hat (accelerated sampler's sample, before VC), x_ref (full-precision
 * sampler's sample at the same step): dev fp32 [B, C, H, W], read only;
 * work: dev, B*C*2 doubles of scratch owned by the caller; K_t: dev fp32 [C],
 * written.  eps >= 0. */
int qc_vc_fit(const float *x_hat, const float *x_ref, int B, int C, int H, int W, float eps, double *work, float *K_t,
              void *stream);

/* qc_vc_fit for callers that cannot allocate device memory for `work` (code under HIP graph capture, serving loops
 * and harnesses that forbid allocation): the per-plane partial sums live in a fixed device array inside the library,
 * QC_VC_FIT_STATIC_MAX_PLANES planes (B * C) at most, 256 KiB per GPU the library runs on, held until the process
 * ends.  Same arguments, kernels and results as qc_vc_fit without `work`; B * C beyond the limit is QC_ERR_WORKSPACE.
 * The call allocates nothing.  Every call on a GPU uses that GPU's one array (each plane's slot is overwritten by
 * every call, nothing has to be cleared in between): calls that overlap on one GPU - different streams or host
 * threads - race and must be serialised by the caller. */
#define QC_VC_FIT_STATIC_MAX_PLANES 16384
int qc_vc_fit_static(const float *x_hat, const float *x_ref, int B, int C, int H, int W, float eps, float *K_t, void *stream);

/* Deterministic DDIM schedule on the 1000-step linear-beta (1e-4..2e-2)
 * training schedule: t[i] = (steps-1-i) * floor(1000/steps), abar_t[i],
 * abar_prev[i] (= 1 on the last step).  HOST arrays of `steps` entries. */
int qc_ddim_schedule(int steps, int32_t *t, double *abar_t, double *abar_prev);

/* ------------------------------------------------------------- DiT pieces */

/* One adaLN-Zero block on x: dev [B, T, D] in place, conditioning c: dev
 * [B, D].  QC_FULL: adaLN projection, LN+modulate+quantise, QKV, attention,
 * projection, MLP, all five linears quantised; stores the attention and MLP
 * module outputs (before the gate) in the cache.  QC_CACHED ("reuse for the
 * following N-1 steps", Quantization and Cache section): recomputes only the
 * two gates from c and adds gate * cached output twice.  QC_ERR_STATE when
 * nothing was stored for this block at this batch size. */
int qc_dit_block(qc_ctx *ctx, int block, int mode, float *x, const float *c, int B, void *stream);

/* Copy a module output into / add a gated cached module output from the cache.
 * src, x: dev [B, T, D]; gate: dev [B, ld_gate] rows, first D entries used. */
int qc_cache_store(qc_ctx *ctx, int block, int which, const float *src, int B, void *stream);
int qc_cache_reuse(qc_ctx *ctx, int block, int which, float *x, const float *gate, int ld_gate, int B, void *stream);
/* Device address of a cached tensor ([max_batch, T, D], first B rows valid), in
 * the format set by qc_set_cache_format: fp32 or bfloat16. */
int qc_cache_ptr(qc_ctx *ctx, int block, int which, void **ptr_out);

/* Storage format of the cached module outputs.  QC_CACHE_FP32 (default) keeps
 * them as the refresh step computed them.  QC_CACHE_BF16 stores the bfloat16
 * rounding (nearest even) of those fp32 values: a cached step then streams
 * half the bytes and adds gate * (rounded output); the refresh step itself is
 * unchanged, it uses the exact outputs.  Not in the paper: a precision choice
 * of this implementation, off by default.  Switching format discards what the
 * cache holds. */
enum { QC_CACHE_FP32 = 0, QC_CACHE_BF16 = 1 };
int qc_set_cache_format(qc_ctx *ctx, int format);
/* Storage format of the residual stream inside the network-level calls (qc_denoise, qc_sample_step, qc_sample):
 * the token tensor [B, T, D] that the patch embedding writes and every block reads and updates.  QC_STREAM_FP32
 * (default) keeps float32.  QC_STREAM_BF16 stores the bfloat16 rounding (nearest even) of every float32 value
 * written to it - the embedding's output and the stream after every gated add - so that the LayerNorm kernels,
 * the proj / fc2 epilogues and the cached-block kernel move half the bytes of it; all other tensors keep their
 * formats.  Not in the paper: a precision choice of this implementation, off by default; qc_dit_block, whose
 * stream is the caller's float32 tensor, is not affected.  Set it between sampling runs, not inside one. */
enum { QC_STREAM_FP32 = 0, QC_STREAM_BF16 = 1 };
int qc_set_stream_format(qc_ctx *ctx, int format);
/* Device address of an internal buffer, see QC_WS_*; for inspection by tests. */
int qc_workspace_ptr(qc_ctx *ctx, int which, void **ptr_out, size_t *bytes_out);

/* Per-(step, block, module) cache schedule, a generalisation of the interval
 * rule of the "Quantization and Cache" section to learned layer-caching
 * policies (the kind the ablation compares against): mask is a HOST array
 * [steps][depth][2] of 0/1, module 0 = attention, 1 = MLP; 1 recomputes the
 * module at that step and stores its output, 0 reuses the stored output (gates
 * always follow the current conditioning).  Row 0 must be all ones.  It
 * replaces `step_index mod N` in qc_sample_step (force_mode -1), qc_sample and
 * qc_vc_fit_sampler, which then accept at most `steps` steps; the array is
 * copied.  mask = NULL restores the interval rule. */
int qc_set_cache_mask(qc_ctx *ctx, const unsigned char *mask, int steps);

/* Inspection aid: when on, full blocks also write the QKV projection row-major into the
 * QC_WS_QKV buffer (the attention kernel itself reads head-major copies of the same fp32 values).
 * Only the general GEMM kernel writes that copy: while it is on, large QKV launches do not take the
 * large-M kernel (same values, slower); QC_WS_QKV_HEADS can be read without it. */
int qc_keep_qkv_f32(qc_ctx *ctx, int on);

/* Class labels live in device memory, so the entry points that take them (qc_denoise, qc_sample_step,
 * qc_sample, qc_vc_fit_sampler) cannot validate them on the host: the conditioning kernel clamps a label outside
 * [0, num_classes] into that range (Experimental Settings: num_classes real classes plus the null label
 * num_classes) and raises a flag on the device.  qc_check waits for `stream`, returns QC_ERR_RANGE if the flag was
 * raised since the last call (and clears it), QC_OK otherwise. */
int qc_check(qc_ctx *ctx, void *stream);

/* Noise estimate of the whole network at timestep t.  x: dev [n_labels, C, H, W],
 * labels: dev int32 [n_labels].  The effective batch B is n_labels, or
 * 2 * n_labels for guidance: then sample b + n_labels is latent b again with
 * the null label.  eps_out: dev [B, C, H, W] (first C of the 2C output
 * channels).  mode QC_FULL recomputes all blocks and refreshes the cache,
 * QC_CACHED reuses it (QC_ERR_STATE unless the cache holds this batch size). */
int qc_denoise(qc_ctx *ctx, const float *x, int t, const int32_t *labels, int n_labels, int B, int mode,
               float *eps_out, void *stream);

/* One sampler step on x: dev [B, C, H, W] in place: denoiser (full iff
 * step_index mod N == 0 unless force_mode is QC_FULL / QC_CACHED; pass -1 for
 * the rule), guidance when cfg_scale > 0 (the library runs the 2B batch
 * [labels ; null] and combines eps_u + w (eps_c - eps_u)), DDIM (eta = 0)
 * update with the given abar values, then VC (Eq. 10) with K_t: dev [C] unless
 * K_t is NULL. */
int qc_sample_step(qc_ctx *ctx, float *x, const int32_t *labels, int B, int step_index, int t,
                   double abar_t, double abar_prev, float cfg_scale, const float *K_t, int force_mode, void *stream);

/* The whole sampling loop: `steps` calls of qc_sample_step with the schedule
 * of qc_ddim_schedule; K: dev [steps, C] or NULL. */
int qc_sample(qc_ctx *ctx, float *x, const int32_t *labels, int B, int steps, float cfg_scale, const float *K,
              void *stream);

/* ------------------------------------------------------------- profiling */

/* Noise prediction of the UN-quantised network (fp32 weights and activations,
 * no cache): the reference that the VC factors are fitted against and the
 * network the activation ranges are calibrated on.  Set-up-grade kernels, one
 * sample at a time.  w: the fp32 weights (device pointers, as for
 * qc_load_weights_f32, which must have run: the embedders and the final layer
 * are taken from the context); x: dev [n_labels, C, H, W]; labels: dev
 * [n_labels]; B = n_labels, or 2*n_labels for [labels ; null label] on the
 * same latents; eps_out: dev [B, C, H, W]. */
int qc_denoise_f32(qc_ctx *ctx, const qc_weights_f32 *w, const float *x, int t, const int32_t *labels, int n_labels, int B,
                   float *eps_out, void *stream);

/* Fits K[steps, C] along a sampling trajectory ("Variance Align for Exposure
 * Bias" section): the un-quantised, un-cached sampler (x_ref) and the
 * quantised sampler under the cache rule (x_hat) run side by side from the
 * same initial latents and labels on the schedule of qc_ddim_schedule; at
 * every step the accelerated sample before VC is fitted against the reference
 * sample (qc_vc_fit with vc_eps), the fitted K_i is applied to it (Eq. 10) and
 * both go on.  x_hat, x_ref: dev [B, C, H, W], both holding the initial
 * latents on entry (distinct buffers), the two final samples on return;
 * labels: dev [B]; cfg_scale as in qc_sample_step; K_out: dev fp32
 * [steps, C], written.  Requires activation parameters for every site. */
int qc_vc_fit_sampler(qc_ctx *ctx, const qc_weights_f32 *w, float *x_hat, float *x_ref, const int32_t *labels, int B, int steps,
                      float cfg_scale, float vc_eps, float *K_out, void *stream);

/* Kernel classes of the per-launch timing below. */
enum {
  QC_K_ADALN = 0,          /* batched adaLN projection GEMM (all blocks, M = batch)      */
  QC_K_LN_QUANT = 1,       /* LayerNorm + modulate + quantise (two per block)            */
  QC_K_GEMM_QKV = 2,       /* QKV GEMM + dequantise                                       */
  QC_K_ATTENTION = 3,      /* softmax(QK^T)V + quantise                                   */
  QC_K_GEMM_PROJ = 4,      /* projection GEMM + cache store + gated residual             */
  QC_K_GEMM_FC1 = 5,       /* fc1 GEMM + GELU + requantise                                */
  QC_K_GEMM_FC2 = 6,       /* fc2 GEMM + cache store + gated residual                    */
  QC_K_CACHED_BLOCKS = 7,  /* all blocks of a cached step                                 */
  QC_K_DDIM_VC = 8,        /* guidance + solver update + VC                               */
  QC_K_COUNT = 9
};

/* Between qc_profile_begin and qc_profile_end every launch of the classes above
 * on this context is bracketed by two HIP events on the launch stream.
 * qc_profile_end synchronises the stream and returns, per class, the number of
 * launches and the sum of their durations in milliseconds (HOST arrays of
 * n_classes >= QC_K_COUNT entries).  The events serialise nothing but add a
 * little launch overhead: time whole-job throughput with profiling off. */
int qc_profile_begin(qc_ctx *ctx);
int qc_profile_end(qc_ctx *ctx, int n_classes, int32_t *launches, float *total_ms, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QC_H_ */
