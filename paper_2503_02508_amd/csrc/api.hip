// Host layer of the C ABI: argument checks, arena layout, and the sequence of
// kernel launches that makes up a DiT block, a denoiser call and a sampler step.
// Every check runs before the first device call, so error paths work without a GPU.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "qc_internal.h"

namespace qc {

constexpr int MAX_LANES = 4;
// rows of the conditioning tables: the conditioning of several sampler steps is prepared in one go
constexpr int WINDOW_ROWS = 512;

// a contiguous range of the (effective) batch handled by one stream; `lane` picks its private scratch
struct Sub {
  int b0, nb, lane;
  int r0;   // first row of this range in the conditioning tables (cond, fmod, mod, silu_q): step slot * batch + b0
};

static thread_local char g_err[512] = "";

void set_error(const char *fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

#define QC_FAIL(code, ...)      \
  do {                          \
    qc::set_error(__VA_ARGS__); \
    return (code);              \
  } while (0)

#define QC_HIP(expr)                                                                          \
  do {                                                                                        \
    hipError_t e_ = (expr);                                                                   \
    if (e_ != hipSuccess) QC_FAIL(QC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));        \
  } while (0)

static inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// bump allocator over the arena (base may be null when only sizing)
struct Bump {
  char *base;
  size_t off = 0;
  explicit Bump(char *b) : base(b) {}
  template <typename T>
  T *take(size_t count) {
    off = (off + 255) & ~size_t(255);
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

struct BlockQ {
  LinearQ lin[QC_NUM_SITES];
};

}  // namespace qc

using namespace qc;

struct qc_ctx {
  qc_model_desc d;
  int max_batch;
  int T, D, R, H, hd, L, C, F;   // F = patch feature count
  char *arena;
  size_t arena_bytes;
  std::vector<BlockQ> blk;
  // adaLN weights of all blocks are contiguous so that one batched launch covers them
  size_t ada_w_stride_bytes;
  float *patch_w, *patch_b, *pos, *t_w1, *t_b1, *t_w2, *t_b2, *label_table, *fada_w, *fada_b, *flin_w, *flin_b;
  std::vector<QParam> host_qp;
  std::vector<char> qp_set;
  QParam *dev_qp;   // [L][5]
  float *cache;     // [L][2][max_batch*T*D]
  std::vector<int> cache_batch;   // [L][2]: batch size held, 0 = nothing stored
  bool cache_bf16 = false;        // cached tensors stored as bfloat16 instead of fp32 (qc_set_cache_format)
  std::vector<unsigned char> cache_mask;   // optional [steps][L][2] schedule (1 = recompute); empty = interval rule
  int mask_steps = 0;
  // workspace
  float *emb, *h1, *te, *cond, *mod, *fmod, *tokens, *qkv, *eps;
  float *eps_ref;      // noise prediction of the un-quantised reference forward (VC fitting)
  double *vcfit_work;  // per-plane partial sums of the VC fit [max_batch * C][2]
  int8_t *silu_q, *qa_ln, *qa_attn, *qa_mlp;
  float *qkv_hm;              // float32 Q, K [B,H,T,hd] and V^T [B,H,DP,Tp] (head-major) for the attention kernel
  long long qkv_part_stride;  // elements per Q / K array
  size_t qkv_hm_bytes;
  int *dev_flags;             // [0]: bit 0 = a class label outside [0, num_classes] was met (and clamped)
  int DP, Tp;
  int win_rows;               // row capacity of cond / fmod / mod / silu_q (per block for the last two)
  bool keep_qkv_f32 = false;
  bool stream_bf16 = false;   // the network-level calls keep the residual stream (tokens) as bfloat16
  // calibration scratch (one sample)
  float *cal_h, *cal_o, *cal_a, *cal_u, *cal_mod;
  int *cal_slots, *cal_label;
  bool weights_loaded;
  // a denoiser call may run its batch as up to MAX_LANES independent sub-batches on internal streams
  hipStream_t lane_stream[4] = {nullptr, nullptr, nullptr, nullptr};
  hipEvent_t ev_fork = nullptr, ev_join[4] = {nullptr, nullptr, nullptr, nullptr};
  // optional per-kernel-class timing with HIP events (qc_profile_begin / qc_profile_end)
  bool prof_on = false;
  std::vector<hipEvent_t> prof_pool;
  size_t prof_used = 0;
  std::vector<int> prof_cls;
};

// Brackets one launch with two events while profiling is on.
struct ProfScope {
  qc_ctx *c;
  hipStream_t st;
  bool on;
  ProfScope(qc_ctx *ctx, int cls, hipStream_t s) : c(ctx), st(s), on(ctx->prof_on) {
    if (!on) return;
    while (c->prof_pool.size() < c->prof_used + 2) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
      c->prof_pool.push_back(e);
    }
    c->prof_cls.push_back(cls);
    (void)hipEventRecord(c->prof_pool[c->prof_used], st);
  }
  ~ProfScope() {
    if (!on) return;
    (void)hipEventRecord(c->prof_pool[c->prof_used + 1], st);
    c->prof_used += 2;
  }
};
#define QC_PROF(cls) ProfScope prof_scope_(ctx, (cls), st)

static size_t weight_bytes(const qc_model_desc &d, size_t N, size_t K) { return d.weight_bits == 4 ? N * K / 2 : N * K; }

static int check_desc(const qc_model_desc *d) {
  if (!d) QC_FAIL(QC_ERR_NULL, "model description is NULL");
  if (d->depth < 1 || d->hidden < 1 || d->heads < 1 || d->mlp_dim < 1 || d->patch < 1 || d->latent_c < 1 ||
      d->latent_h < 1 || d->latent_w < 1 || d->num_classes < 1 || d->freq_dim < 2)
    QC_FAIL(QC_ERR_SHAPE, "model description has a non-positive dimension");
  if (d->hidden % d->heads) QC_FAIL(QC_ERR_SHAPE, "hidden (%d) is not a multiple of heads (%d)", d->hidden, d->heads);
  if (d->latent_h % d->patch || d->latent_w % d->patch)
    QC_FAIL(QC_ERR_SHAPE, "latent %dx%d is not a multiple of the patch size %d", d->latent_h, d->latent_w, d->patch);
  if (d->freq_dim % 2) QC_FAIL(QC_ERR_SHAPE, "freq_dim must be even");
  if (d->weight_bits != 8 && d->weight_bits != 4) QC_FAIL(QC_ERR_UNSUPPORTED, "weight_bits must be 8 or 4");
  if (d->cache_interval < 1) QC_FAIL(QC_ERR_RANGE, "cache_interval must be >= 1");
  const int hd = d->hidden / d->heads;
  if (d->hidden % 16 || d->mlp_dim % 16) QC_FAIL(QC_ERR_UNSUPPORTED, "hidden and mlp_dim must be multiples of 16");
  if (d->hidden > 2048) QC_FAIL(QC_ERR_UNSUPPORTED, "hidden > 2048 is not covered by the row kernels");
  if (hd % 4 || hd > 80) QC_FAIL(QC_ERR_UNSUPPORTED, "head dim must be a multiple of 4 and at most 80");
  if (d->latent_c * d->patch * d->patch > 256) QC_FAIL(QC_ERR_UNSUPPORTED, "patch feature count above 256");
  return QC_OK;
}

// Lays the context out in the arena; with ctx == nullptr only measures.
static size_t layout(const qc_model_desc &d, int max_batch, char *base, qc_ctx *c) {
  Bump a(base);
  const size_t D = d.hidden, R = d.mlp_dim, L = d.depth, C = d.latent_c;
  const size_t T = (size_t)(d.latent_h / d.patch) * (d.latent_w / d.patch);
  const size_t F = C * d.patch * d.patch, O = (size_t)d.patch * d.patch * 2 * C;
  const size_t B = max_batch, M = B * T;
  // batched adaLN weights
  const size_t ada_bytes = (weight_bytes(d, 6 * D, D) + 255) & ~size_t(255);
  char *ada_q = a.take<char>(ada_bytes * L);
  float *ada_scale = a.take<float>(6 * D * L);
  int32_t *ada_wsum = a.take<int32_t>(6 * D * L);
  float *ada_bias = a.take<float>(6 * D * L);
  if (c) {
    c->ada_w_stride_bytes = ada_bytes;
    c->blk.resize(L);
  }
  const size_t Ns[QC_NUM_SITES] = {6 * D, 3 * D, D, R, D};
  const size_t Ks[QC_NUM_SITES] = {D, D, D, D, R};
  for (size_t l = 0; l < L; ++l) {
    for (int s = 0; s < QC_NUM_SITES; ++s) {
      LinearQ q;
      q.N = (int)Ns[s];
      q.K = (int)Ks[s];
      if (s == QC_SITE_ADA) {
        q.q = ada_q ? ada_q + l * ada_bytes : nullptr;
        q.scale = ada_scale ? ada_scale + l * 6 * D : nullptr;
        q.wsum = ada_wsum ? ada_wsum + l * 6 * D : nullptr;
        q.bias = ada_bias ? ada_bias + l * 6 * D : nullptr;
      } else {
        q.q = a.take<char>(weight_bytes(d, Ns[s], Ks[s]));
        // second copy in MFMA fragment order for the large-M GEMM (shapes its loop covers)
        if (Ns[s] % 32 == 0 && Ks[s] % 128 == 0) q.qt = a.take<char>(weight_bytes(d, Ns[s], Ks[s]));
        q.scale = a.take<float>(Ns[s]);
        q.wsum = a.take<int32_t>(Ns[s]);
        q.bias = a.take<float>(Ns[s]);
      }
      if (c) c->blk[l].lin[s] = q;
    }
  }
  float *patch_w = a.take<float>(D * F), *patch_b = a.take<float>(D), *pos = a.take<float>(T * D);
  float *t_w1 = a.take<float>(D * d.freq_dim), *t_b1 = a.take<float>(D), *t_w2 = a.take<float>(D * D), *t_b2 = a.take<float>(D);
  float *label_table = a.take<float>((size_t)(d.num_classes + 1) * D);
  float *fada_w = a.take<float>(2 * D * D), *fada_b = a.take<float>(2 * D);
  float *flin_w = a.take<float>(O * D), *flin_b = a.take<float>(O);
  QParam *dev_qp = a.take<QParam>(L * QC_NUM_SITES);
  float *cache = a.take<float>(L * 2 * M * D);
  const size_t WR = B > (size_t)WINDOW_ROWS ? B : (size_t)WINDOW_ROWS;
  float *emb = a.take<float>(WR * d.freq_dim), *h1 = a.take<float>(WR * D), *te = a.take<float>(WR * D);
  float *cond = a.take<float>(WR * D), *mod = a.take<float>(L * WR * 6 * D), *fmod = a.take<float>(WR * 2 * D);
  float *tokens = a.take<float>(M * D), *qkv = a.take<float>(M * 3 * D), *eps = a.take<float>(B * C * d.latent_h * d.latent_w);
  int8_t *silu_q = a.take<int8_t>(L * WR * D), *qa_ln = a.take<int8_t>(M * D), *qa_attn = a.take<int8_t>(M * D);
  int8_t *qa_mlp = a.take<int8_t>(M * R);
  const size_t hd = D / d.heads, DP = (hd + 15) / 16 * 16, Tp = (T + 63) / 64 * 64;
  const size_t part = B * d.heads * T * hd, vpart = B * d.heads * DP * Tp;
  float *qkv_hm = a.take<float>(2 * part + vpart);
  float *cal_h = a.take<float>(T * D), *cal_o = a.take<float>(T * D), *cal_a = a.take<float>(T * D);
  float *cal_u = a.take<float>(T * R), *cal_mod = a.take<float>(6 * D);
  int *cal_slots = a.take<int>(L * QC_NUM_SITES * 2), *cal_label = a.take<int>(4);
  float *eps_ref = a.take<float>(B * C * d.latent_h * d.latent_w);
  double *vcfit_work = a.take<double>(B * C * 2);
  int *dev_flags = a.take<int>(64);
  if (c) {
    c->patch_w = patch_w; c->patch_b = patch_b; c->pos = pos; c->t_w1 = t_w1; c->t_b1 = t_b1; c->t_w2 = t_w2; c->t_b2 = t_b2;
    c->label_table = label_table; c->fada_w = fada_w; c->fada_b = fada_b; c->flin_w = flin_w; c->flin_b = flin_b;
    c->dev_qp = dev_qp; c->cache = cache; c->emb = emb; c->h1 = h1; c->te = te; c->cond = cond; c->mod = mod; c->fmod = fmod;
    c->tokens = tokens; c->qkv = qkv; c->eps = eps; c->silu_q = silu_q; c->qa_ln = qa_ln; c->qa_attn = qa_attn;
    c->qa_mlp = qa_mlp; c->cal_h = cal_h; c->cal_o = cal_o; c->cal_a = cal_a; c->cal_u = cal_u; c->cal_mod = cal_mod;
    c->cal_slots = cal_slots; c->cal_label = cal_label; c->eps_ref = eps_ref; c->vcfit_work = vcfit_work; c->dev_flags = dev_flags;
    c->qkv_hm = qkv_hm; c->qkv_part_stride = (long long)part;
    c->qkv_hm_bytes = (2 * part + vpart) * sizeof(float); c->DP = (int)DP; c->Tp = (int)Tp;
    c->win_rows = (int)WR;
  }
  return (a.off + 255) & ~size_t(255);
}

extern "C" {

const char *qc_last_error(void) { return g_err; }

int qc_arena_bytes(const qc_model_desc *desc, int max_batch, size_t *bytes_out) {
  if (!bytes_out) QC_FAIL(QC_ERR_NULL, "bytes_out is NULL");
  int rc = check_desc(desc);
  if (rc) return rc;
  if (max_batch < 1) QC_FAIL(QC_ERR_SHAPE, "max_batch must be >= 1");
  *bytes_out = layout(*desc, max_batch, nullptr, nullptr);
  return QC_OK;
}

int qc_create(const qc_model_desc *desc, void *arena, size_t arena_bytes, int max_batch, qc_ctx **out) {
  if (!out) QC_FAIL(QC_ERR_NULL, "out is NULL");
  *out = nullptr;
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!arena) QC_FAIL(QC_ERR_NULL, "arena is NULL");
  if (max_batch < 1) QC_FAIL(QC_ERR_SHAPE, "max_batch must be >= 1");
  if (reinterpret_cast<uintptr_t>(arena) & 255u) QC_FAIL(QC_ERR_ALIGN, "arena must be 256-byte aligned");
  const size_t need = layout(*desc, max_batch, nullptr, nullptr);
  if (arena_bytes < need) QC_FAIL(QC_ERR_WORKSPACE, "arena holds %zu bytes, %zu needed", arena_bytes, need);
  qc_ctx *c = new (std::nothrow) qc_ctx();
  if (!c) QC_FAIL(QC_ERR_WORKSPACE, "out of host memory");
  c->d = *desc;
  c->max_batch = max_batch;
  c->D = desc->hidden; c->R = desc->mlp_dim; c->H = desc->heads; c->hd = desc->hidden / desc->heads; c->L = desc->depth;
  c->C = desc->latent_c; c->F = desc->latent_c * desc->patch * desc->patch;
  c->T = (desc->latent_h / desc->patch) * (desc->latent_w / desc->patch);
  c->arena = static_cast<char *>(arena);
  c->arena_bytes = arena_bytes;
  layout(*desc, max_batch, c->arena, c);
  c->host_qp.assign((size_t)c->L * QC_NUM_SITES, QParam{1.0f, 0});
  c->qp_set.assign((size_t)c->L * QC_NUM_SITES, 0);
  c->cache_batch.assign((size_t)c->L * 2, 0);
  c->weights_loaded = false;
  *out = c;
  return QC_OK;
}

int qc_destroy(qc_ctx *ctx) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  for (hipEvent_t e : ctx->prof_pool) (void)hipEventDestroy(e);
  for (int i = 0; i < MAX_LANES; ++i) {
    if (ctx->lane_stream[i]) (void)hipStreamDestroy(ctx->lane_stream[i]);
    if (ctx->ev_join[i]) (void)hipEventDestroy(ctx->ev_join[i]);
  }
  if (ctx->ev_fork) (void)hipEventDestroy(ctx->ev_fork);
  delete ctx;
  return QC_OK;
}

static int check_weights(const qc_ctx *ctx, const qc_weights_f32 *w) {
  if (!w) QC_FAIL(QC_ERR_NULL, "weights are NULL");
  const void *g[] = {w->patch_w, w->patch_b, w->pos, w->t_w1, w->t_b1, w->t_w2, w->t_b2, w->label_table,
                     w->fada_w, w->fada_b, w->flin_w, w->flin_b, w->blocks};
  for (const void *p : g)
    if (!p) QC_FAIL(QC_ERR_NULL, "a weight pointer is NULL");
  for (int l = 0; l < ctx->L; ++l) {
    const qc_block_weights_f32 &b = w->blocks[l];
    const void *q[] = {b.ada_w, b.ada_b, b.qkv_w, b.qkv_b, b.proj_w, b.proj_b, b.fc1_w, b.fc1_b, b.fc2_w, b.fc2_b};
    for (const void *p : q) {
      if (!p) QC_FAIL(QC_ERR_NULL, "a weight pointer of block %d is NULL", l);
      if (!aligned16(p)) QC_FAIL(QC_ERR_ALIGN, "a weight pointer of block %d is not 16-byte aligned", l);
    }
  }
  return QC_OK;
}

int qc_load_weights_f32(qc_ctx *ctx, const qc_weights_f32 *w, void *stream) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  int rc = check_weights(ctx, w);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t D = ctx->D, T = ctx->T, O = (size_t)ctx->d.patch * ctx->d.patch * 2 * ctx->C;
  struct { float *dst; const float *src; size_t n; } cp[] = {
      {ctx->patch_w, w->patch_w, D * ctx->F}, {ctx->patch_b, w->patch_b, D}, {ctx->pos, w->pos, T * D},
      {ctx->t_w1, w->t_w1, D * ctx->d.freq_dim}, {ctx->t_b1, w->t_b1, D}, {ctx->t_w2, w->t_w2, D * D}, {ctx->t_b2, w->t_b2, D},
      {ctx->label_table, w->label_table, (size_t)(ctx->d.num_classes + 1) * D}, {ctx->fada_w, w->fada_w, 2 * D * D},
      {ctx->fada_b, w->fada_b, 2 * D}, {ctx->flin_w, w->flin_w, O * D}, {ctx->flin_b, w->flin_b, O}};
  for (auto &c : cp) QC_HIP(hipMemcpyAsync(c.dst, c.src, c.n * sizeof(float), hipMemcpyDeviceToDevice, st));
  // padding features / keys of the fp16 attention operands are never written afterwards and must read as zero
  QC_HIP(hipMemsetAsync(ctx->qkv_hm, 0, ctx->qkv_hm_bytes, st));
  QC_HIP(hipMemsetAsync(ctx->dev_flags, 0, 64 * sizeof(int), st));
  for (int l = 0; l < ctx->L; ++l) {
    const qc_block_weights_f32 &b = w->blocks[l];
    const float *ws[QC_NUM_SITES] = {b.ada_w, b.qkv_w, b.proj_w, b.fc1_w, b.fc2_w};
    const float *bs[QC_NUM_SITES] = {b.ada_b, b.qkv_b, b.proj_b, b.fc1_b, b.fc2_b};
    for (int s = 0; s < QC_NUM_SITES; ++s) {
      LinearQ &q = ctx->blk[l].lin[s];
      QC_HIP(launch_quantize_weight(ws[s], q.N, q.K, ctx->d.weight_bits, q.q, q.scale, q.wsum, st));
      if (q.qt) QC_HIP(launch_tile_weight(q.q, q.qt, q.N, q.K, ctx->d.weight_bits, st));
      QC_HIP(hipMemcpyAsync(q.bias, bs[s], (size_t)q.N * sizeof(float), hipMemcpyDeviceToDevice, st));
    }
  }
  ctx->weights_loaded = true;
  return QC_OK;
}

static int check_site(const qc_ctx *ctx, int block, int site) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (block < 0 || block >= ctx->L) QC_FAIL(QC_ERR_RANGE, "block %d outside 0..%d", block, ctx->L - 1);
  if (site < 0 || site >= QC_NUM_SITES) QC_FAIL(QC_ERR_RANGE, "site %d outside 0..%d", site, QC_NUM_SITES - 1);
  return QC_OK;
}

static int check_qparam(float scale, int zp) {
  if (!(scale > 0.0f) || !std::isfinite(scale)) QC_FAIL(QC_ERR_RANGE, "scale must be positive and finite");
  if (zp < 0 || zp > 255) QC_FAIL(QC_ERR_RANGE, "zero point %d outside 0..255", zp);
  return QC_OK;
}

int qc_set_act_qparams(qc_ctx *ctx, int block, int site, float scale, int zero_point) {
  int rc = check_site(ctx, block, site);
  if (rc) return rc;
  rc = check_qparam(scale, zero_point);
  if (rc) return rc;
  const size_t i = (size_t)block * QC_NUM_SITES + site;
  ctx->host_qp[i] = QParam{scale, zero_point - 128};
  ctx->qp_set[i] = 1;
  QC_HIP(hipMemcpy(ctx->dev_qp + i, &ctx->host_qp[i], sizeof(QParam), hipMemcpyHostToDevice));
  return QC_OK;
}

int qc_get_act_qparams(const qc_ctx *ctx, int block, int site, float *scale, int *zero_point) {
  int rc = check_site(ctx, block, site);
  if (rc) return rc;
  if (!scale || !zero_point) QC_FAIL(QC_ERR_NULL, "output pointer is NULL");
  const size_t i = (size_t)block * QC_NUM_SITES + site;
  if (!ctx->qp_set[i]) QC_FAIL(QC_ERR_STATE, "activation parameters of block %d site %d were never set", block, site);
  *scale = ctx->host_qp[i].s;
  *zero_point = ctx->host_qp[i].z + 128;
  return QC_OK;
}

// ------------------------------------------------------------ single ops
int qc_quantize_act(const float *x, int8_t *q, size_t n, float scale, int zero_point, void *stream) {
  int rc = check_qparam(scale, zero_point);
  if (rc) return rc;
  if (n == 0) return QC_OK;   // an empty tensor may come with a null pointer
  if (!x || !q) QC_FAIL(QC_ERR_NULL, "x or q is NULL");
  if (!aligned16(x) || (reinterpret_cast<uintptr_t>(q) & 3u)) QC_FAIL(QC_ERR_ALIGN, "x must be 16-byte and q 4-byte aligned");
  QC_HIP(launch_quantize_act(x, q, n, scale, zero_point - 128, static_cast<hipStream_t>(stream)));
  return QC_OK;
}

int qc_quantize_weight(const float *w, int N, int K, int bits, void *qw, float *w_scale, int32_t *wsum, void *stream) {
  if (!w || !qw || !w_scale || !wsum) QC_FAIL(QC_ERR_NULL, "a pointer is NULL");
  if (N < 1 || K < 1) QC_FAIL(QC_ERR_SHAPE, "N and K must be positive");
  if (K % 16) QC_FAIL(QC_ERR_SHAPE, "K (%d) must be a multiple of 16", K);
  if (bits != 8 && bits != 4) QC_FAIL(QC_ERR_UNSUPPORTED, "bits must be 8 or 4");
  if (!aligned16(w) || !aligned16(qw)) QC_FAIL(QC_ERR_ALIGN, "w and qw must be 16-byte aligned");
  QC_HIP(launch_quantize_weight(w, N, K, bits, qw, w_scale, wsum, static_cast<hipStream_t>(stream)));
  return QC_OK;
}

int qc_w8a8_linear(const int8_t *qx, const void *qw, const int32_t *wsum, const float *w_scale, const float *bias,
                   float x_scale, int x_zp, int M, int N, int K, int weight_bits, float *y, int32_t *acc_or_null,
                   void *stream) {
  if (!qx || !qw || !wsum || !w_scale || !y) QC_FAIL(QC_ERR_NULL, "a required pointer is NULL");
  if (M < 0 || N < 0 || K < 1) QC_FAIL(QC_ERR_SHAPE, "M, N must be non-negative and K positive");
  if (K % 16) QC_FAIL(QC_ERR_SHAPE, "K (%d) must be a multiple of 16", K);
  if (weight_bits != 8 && weight_bits != 4) QC_FAIL(QC_ERR_UNSUPPORTED, "weight_bits must be 8 or 4");
  int rc = check_qparam(x_scale, x_zp);
  if (rc) return rc;
  if (!aligned16(qx) || !aligned16(qw)) QC_FAIL(QC_ERR_ALIGN, "qx and qw must be 16-byte aligned");
  if (M == 0 || N == 0) return QC_OK;
  GemmArgs a{};
  a.A = qx; a.W = qw; a.w_scale = w_scale; a.wsum = wsum; a.bias = bias;
  a.M = M; a.N = N; a.K = K; a.lda = K; a.w4 = weight_bits == 4;
  a.a_scale = x_scale; a.a_zp = x_zp - 128;
  a.y = y; a.ldy = N; a.acc_out = acc_or_null;
  QC_HIP(launch_gemm(a, EPI_F32, 1, static_cast<hipStream_t>(stream), QC_SITE_QKV));
  return QC_OK;
}

int qc_vc_correct(float *x, const float *K_t, const float *mu_or_null, int B, int C, int H, int W, void *stream) {
  if (!x || !K_t) QC_FAIL(QC_ERR_NULL, "x or K_t is NULL");
  if (B < 0 || C < 1 || H < 1 || W < 1) QC_FAIL(QC_ERR_SHAPE, "bad shape");
  if (B == 0) return QC_OK;
  QC_HIP(launch_vc(x, K_t, mu_or_null, B, C, H * W, static_cast<hipStream_t>(stream)));
  return QC_OK;
}

int qc_ddim_schedule(int steps, int32_t *t, double *abar_t, double *abar_prev) {
  if (!t || !abar_t || !abar_prev) QC_FAIL(QC_ERR_NULL, "an output array is NULL");
  if (steps < 1 || steps > 1000) QC_FAIL(QC_ERR_RANGE, "steps must be in 1..1000");
  double abar[1000];
  double prod = 1.0;
  for (int i = 0; i < 1000; ++i) {
    const double beta = 1e-4 + (2e-2 - 1e-4) * (double)i / 999.0;
    prod *= 1.0 - beta;
    abar[i] = prod;
  }
  const int stride = 1000 / steps;
  for (int i = 0; i < steps; ++i) {
    t[i] = (steps - 1 - i) * stride;
    abar_t[i] = abar[t[i]];
  }
  for (int i = 0; i < steps; ++i) abar_prev[i] = i + 1 < steps ? abar_t[i + 1] : 1.0;
  return QC_OK;
}

// ------------------------------------------------------------- DiT pieces
static int check_ready(const qc_ctx *ctx, int B) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (B < 1 || B > ctx->max_batch) QC_FAIL(QC_ERR_SHAPE, "batch %d outside 1..%d", B, ctx->max_batch);
  if (!ctx->weights_loaded) QC_FAIL(QC_ERR_STATE, "weights were not loaded");
  for (char s : ctx->qp_set)
    if (!s) QC_FAIL(QC_ERR_STATE, "activation parameters are not set for every site");
  return QC_OK;
}

// element `elem` of the cached tensor (block, which); the arena region is sized for fp32 and holds either format
static void *cache_at(const qc_ctx *ctx, int block, int which, size_t elem = 0) {
  const size_t e = ((size_t)block * 2 + which) * (size_t)ctx->max_batch * ctx->T * ctx->D + elem;
  return reinterpret_cast<char *>(ctx->cache) + e * (ctx->cache_bf16 ? 2 : 4);
}

// adaLN projection of blocks [l0, l0+nl) for `rows` rows of the conditioning tables starting at row r0:
// mod[l, r, :] = Lin_q(codes of SiLU(c[r])); gates only on request.
static int run_adaln(qc_ctx *ctx, int l0, int nl, int r0, int rows, bool gates_only, hipStream_t st) {
  const size_t D = ctx->D, WR = ctx->win_rows;
  GemmArgs a{};
  const LinearQ &q = ctx->blk[l0].lin[QC_SITE_ADA];
  a.A = ctx->silu_q + ((size_t)l0 * WR + r0) * D;
  a.W = q.q; a.w_scale = q.scale; a.wsum = q.wsum; a.bias = q.bias;
  a.M = rows; a.N = (int)(6 * D); a.K = (int)D; a.lda = (int)D; a.w4 = ctx->d.weight_bits == 4;
  a.a_qp = ctx->dev_qp + (size_t)l0 * QC_NUM_SITES + QC_SITE_ADA;
  a.zs_A = (long long)(WR * D); a.zs_W = (long long)ctx->ada_w_stride_bytes; a.zs_vecN = (long long)(6 * D);
  a.zs_out = (long long)(WR * 6 * D); a.zs_qp = QC_NUM_SITES;
  a.sel_D = (gates_only && D % 128 == 0) ? (int)D : 0;
  a.y = ctx->mod + ((size_t)l0 * WR + r0) * 6 * D; a.ldy = (int)(6 * D);
  QC_PROF(QC_K_ADALN);
  QC_HIP(launch_gemm(a, EPI_F32, nl, st, QC_SITE_ADA));
  return QC_OK;
}

// One full block on the rows of sub-batch sb; x points at the first of those rows.
static int run_block_full(qc_ctx *ctx, int l, void *x, int xb, const Sub &sb, hipStream_t st, bool attn_full = true,
                          bool mlp_full = true) {
  const int D = ctx->D, R = ctx->R, T = ctx->T, B = sb.nb, M = B * T;
  const size_t row0 = (size_t)sb.b0 * T;
  const float *mod = ctx->mod + ((size_t)l * ctx->win_rows + sb.r0) * 6 * D;
  const QParam *qp = ctx->dev_qp + (size_t)l * QC_NUM_SITES;
  const bool w4 = ctx->d.weight_bits == 4;
  const BlockQ &bq = ctx->blk[l];
  int8_t *qa_ln = ctx->qa_ln + row0 * D, *qa_attn = ctx->qa_attn + row0 * D, *qa_mlp = ctx->qa_mlp + row0 * R;
  float *q32 = ctx->qkv_hm + (size_t)sb.b0 * ctx->H * T * ctx->hd;
  float *k32 = q32 + ctx->qkv_part_stride;
  float *vt32 = ctx->qkv_hm + 2 * ctx->qkv_part_stride + (size_t)sb.b0 * ctx->H * ctx->DP * ctx->Tp;
  auto base = [&](const LinearQ &q, const int8_t *A, int K, int site) {
    GemmArgs a{};
    a.A = A; a.W = q.q; a.Wt = q.qt; a.w_scale = q.scale; a.wsum = q.wsum; a.bias = q.bias;
    a.M = M; a.N = q.N; a.K = K; a.lda = K; a.w4 = w4; a.a_qp = qp + site;
    return a;
  };
  if (!attn_full) {
    QC_HIP(launch_cache_reuse(x, xb, cache_at(ctx, l, QC_CACHE_ATTN, row0 * D), mod + 2 * D, 6 * D, B, T, D, ctx->cache_bf16, st));
  } else {
  {
    QC_PROF(QC_K_LN_QUANT);
    QC_HIP(launch_ln_mod_quant(x, xb, mod, mod + D, 6 * D, M, D, T, qp + QC_SITE_QKV, qa_ln, nullptr, st));
  }
  {
    GemmArgs a = base(bq.lin[QC_SITE_QKV], qa_ln, D, QC_SITE_QKV);
    a.q32 = q32; a.k32 = k32; a.vt32 = vt32;
    a.heads = ctx->H; a.hd = ctx->hd; a.DP = ctx->DP; a.Tp = ctx->Tp; a.rows_per_batch = T;
    if (ctx->keep_qkv_f32) { a.y = ctx->qkv + row0 * 3 * D; a.ldy = 3 * D; }      // row-major copy for inspection
    QC_PROF(QC_K_GEMM_QKV);
    QC_HIP(launch_gemm(a, EPI_QKV, 1, st, QC_SITE_QKV));
  }
  {
    QC_PROF(QC_K_ATTENTION);
    QC_HIP(launch_attention_f16(q32, k32, vt32, B, T, ctx->Tp, ctx->H, ctx->hd, ctx->DP, qp + QC_SITE_PROJ, qa_attn, st));
  }
  {
    GemmArgs a = base(bq.lin[QC_SITE_PROJ], qa_attn, D, QC_SITE_PROJ);
    a.cache_out = cache_at(ctx, l, QC_CACHE_ATTN, row0 * D); a.cache_bf16 = ctx->cache_bf16; a.x = x; a.x_bf16 = xb; a.gate = mod + 2 * D; a.ld_gate = 6 * D;
    a.rows_per_batch = T;
    QC_PROF(QC_K_GEMM_PROJ);
    QC_HIP(launch_gemm(a, EPI_RESID, 1, st, QC_SITE_PROJ));
  }
  }
  if (!mlp_full) {
    QC_HIP(launch_cache_reuse(x, xb, cache_at(ctx, l, QC_CACHE_MLP, row0 * D), mod + 5 * D, 6 * D, B, T, D, ctx->cache_bf16, st));
    return QC_OK;
  }
  {
    QC_PROF(QC_K_LN_QUANT);
    QC_HIP(launch_ln_mod_quant(x, xb, mod + 3 * D, mod + 4 * D, 6 * D, M, D, T, qp + QC_SITE_FC1, qa_ln, nullptr, st));
  }
  {
    GemmArgs a = base(bq.lin[QC_SITE_FC1], qa_ln, D, QC_SITE_FC1);
    a.q_out = qa_mlp; a.ldq = R; a.o_qp = qp + QC_SITE_FC2;
    QC_PROF(QC_K_GEMM_FC1);
    QC_HIP(launch_gemm(a, EPI_GELU_Q, 1, st, QC_SITE_FC1));
  }
  {
    GemmArgs a = base(bq.lin[QC_SITE_FC2], qa_mlp, R, QC_SITE_FC2);
    a.cache_out = cache_at(ctx, l, QC_CACHE_MLP, row0 * D); a.cache_bf16 = ctx->cache_bf16; a.x = x; a.x_bf16 = xb; a.gate = mod + 5 * D; a.ld_gate = 6 * D;
    a.rows_per_batch = T;
    QC_PROF(QC_K_GEMM_FC2);
    QC_HIP(launch_gemm(a, EPI_RESID, 1, st, QC_SITE_FC2));
  }
  return QC_OK;
}

int qc_dit_block(qc_ctx *ctx, int block, int mode, float *x, const float *c, int B, void *stream) {
  int rc = check_ready(ctx, B);
  if (rc) return rc;
  if (block < 0 || block >= ctx->L) QC_FAIL(QC_ERR_RANGE, "block %d outside 0..%d", block, ctx->L - 1);
  if (mode != QC_FULL && mode != QC_CACHED) QC_FAIL(QC_ERR_RANGE, "mode must be QC_FULL or QC_CACHED");
  if (!x || !c) QC_FAIL(QC_ERR_NULL, "x or c is NULL");
  if (!aligned16(x) || !aligned16(c)) QC_FAIL(QC_ERR_ALIGN, "x and c must be 16-byte aligned");
  if (mode == QC_CACHED && (ctx->cache_batch[(size_t)block * 2] != B || ctx->cache_batch[(size_t)block * 2 + 1] != B))
    QC_FAIL(QC_ERR_STATE, "block %d has no cached outputs for batch %d", block, B);
  hipStream_t st = static_cast<hipStream_t>(stream);
  const size_t D = ctx->D;
  QC_HIP(launch_silu_quant(c, B, (int)D, 1, ctx->dev_qp + (size_t)block * QC_NUM_SITES + QC_SITE_ADA, QC_NUM_SITES,
                           ctx->silu_q + (size_t)block * ctx->win_rows * D, (size_t)ctx->win_rows * D, st));
  const Sub whole{0, B, 0, 0};
  rc = run_adaln(ctx, block, 1, 0, B, mode == QC_CACHED, st);
  if (rc) return rc;
  if (mode == QC_FULL) {
    rc = run_block_full(ctx, block, x, 0, whole, st);
    ctx->cache_batch[(size_t)block * 2] = ctx->cache_batch[(size_t)block * 2 + 1] = B;
    return rc;
  }
  const float *mod = ctx->mod + (size_t)block * ctx->win_rows * 6 * D;
  QC_HIP(launch_cache_reuse(x, 0, cache_at(ctx, block, QC_CACHE_ATTN), mod + 2 * D, (int)(6 * D), B, ctx->T, (int)D, ctx->cache_bf16, st));
  QC_HIP(launch_cache_reuse(x, 0, cache_at(ctx, block, QC_CACHE_MLP), mod + 5 * D, (int)(6 * D), B, ctx->T, (int)D, ctx->cache_bf16, st));
  return QC_OK;
}

static int check_cache_args(const qc_ctx *ctx, int block, int which, int B) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (block < 0 || block >= ctx->L) QC_FAIL(QC_ERR_RANGE, "block %d outside 0..%d", block, ctx->L - 1);
  if (which != QC_CACHE_ATTN && which != QC_CACHE_MLP) QC_FAIL(QC_ERR_RANGE, "which must be QC_CACHE_ATTN or QC_CACHE_MLP");
  if (B < 1 || B > ctx->max_batch) QC_FAIL(QC_ERR_SHAPE, "batch %d outside 1..%d", B, ctx->max_batch);
  return QC_OK;
}

int qc_cache_store(qc_ctx *ctx, int block, int which, const float *src, int B, void *stream) {
  int rc = check_cache_args(ctx, block, which, B);
  if (rc) return rc;
  if (!src) QC_FAIL(QC_ERR_NULL, "src is NULL");
  if (!aligned16(src)) QC_FAIL(QC_ERR_ALIGN, "src must be 16-byte aligned");
  QC_HIP(launch_cache_store(src, cache_at(ctx, block, which), (size_t)B * ctx->T * ctx->D, ctx->cache_bf16, static_cast<hipStream_t>(stream)));
  ctx->cache_batch[(size_t)block * 2 + which] = B;
  return QC_OK;
}

int qc_cache_reuse(qc_ctx *ctx, int block, int which, float *x, const float *gate, int ld_gate, int B, void *stream) {
  int rc = check_cache_args(ctx, block, which, B);
  if (rc) return rc;
  if (!x || !gate) QC_FAIL(QC_ERR_NULL, "x or gate is NULL");
  if (ld_gate < ctx->D || ld_gate % 4) QC_FAIL(QC_ERR_SHAPE, "ld_gate must be >= hidden and a multiple of 4");
  if (!aligned16(x) || !aligned16(gate)) QC_FAIL(QC_ERR_ALIGN, "x and gate must be 16-byte aligned");
  if (ctx->cache_batch[(size_t)block * 2 + which] != B)
    QC_FAIL(QC_ERR_STATE, "block %d holds no cached tensor %d for batch %d", block, which, B);
  QC_HIP(launch_cache_reuse(x, 0, cache_at(ctx, block, which), gate, ld_gate, B, ctx->T, ctx->D, ctx->cache_bf16, static_cast<hipStream_t>(stream)));
  return QC_OK;
}

int qc_cache_ptr(qc_ctx *ctx, int block, int which, void **ptr_out) {
  int rc = check_cache_args(ctx, block, which, 1);
  if (rc) return rc;
  if (!ptr_out) QC_FAIL(QC_ERR_NULL, "ptr_out is NULL");
  *ptr_out = cache_at(ctx, block, which);
  return QC_OK;
}

int qc_workspace_ptr(qc_ctx *ctx, int which, void **ptr_out, size_t *bytes_out) {
  if (!ctx || !ptr_out) QC_FAIL(QC_ERR_NULL, "ctx or ptr_out is NULL");
  const size_t B = ctx->max_batch, M = B * ctx->T, D = ctx->D;
  void *p = nullptr;
  size_t n = 0;
  switch (which) {
    case QC_WS_TOKENS: p = ctx->tokens; n = M * D * (ctx->stream_bf16 ? 2 : 4); break;
    case QC_WS_QACT_LN: p = ctx->qa_ln; n = M * D; break;
    case QC_WS_QACT_ATTN: p = ctx->qa_attn; n = M * D; break;
    case QC_WS_QACT_MLP: p = ctx->qa_mlp; n = M * ctx->R; break;
    case QC_WS_QKV: p = ctx->qkv; n = M * 3 * D * 4; break;
    case QC_WS_MOD: p = ctx->mod; n = (size_t)ctx->L * ctx->win_rows * 6 * D * 4; break;
    case QC_WS_COND: p = ctx->cond; n = (size_t)ctx->win_rows * D * 4; break;
    case QC_WS_EPS: p = ctx->eps; n = B * ctx->C * ctx->d.latent_h * ctx->d.latent_w * 4; break;
    case QC_WS_QKV_HEADS: p = ctx->qkv_hm; n = ctx->qkv_hm_bytes; break;
    default: QC_FAIL(QC_ERR_RANGE, "unknown workspace selector %d", which);
  }
  *ptr_out = p;
  if (bytes_out) *bytes_out = n;
  return QC_OK;
}

int qc_set_cache_format(qc_ctx *ctx, int format) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (format != QC_CACHE_FP32 && format != QC_CACHE_BF16) QC_FAIL(QC_ERR_RANGE, "format must be QC_CACHE_FP32 or QC_CACHE_BF16");
  ctx->cache_bf16 = format == QC_CACHE_BF16;
  for (int &v : ctx->cache_batch) v = 0;      // what the cache holds is in the other format: nothing is stored
  return QC_OK;
}

int qc_set_stream_format(qc_ctx *ctx, int format) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (format != QC_STREAM_FP32 && format != QC_STREAM_BF16) QC_FAIL(QC_ERR_RANGE, "format must be QC_STREAM_FP32 or QC_STREAM_BF16");
  ctx->stream_bf16 = format == QC_STREAM_BF16;
  return QC_OK;
}

int qc_set_cache_mask(qc_ctx *ctx, const unsigned char *mask, int steps) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (!mask) {
    ctx->cache_mask.clear();
    ctx->mask_steps = 0;
    return QC_OK;
  }
  if (steps < 1) QC_FAIL(QC_ERR_SHAPE, "steps must be >= 1");
  const size_t row = (size_t)ctx->L * 2;
  for (size_t i = 0; i < row; ++i)
    if (!mask[i]) QC_FAIL(QC_ERR_RANGE, "step 0 must recompute every module (block %zu, module %zu is marked as reused)", i / 2, i % 2);
  for (size_t i = 0; i < row * steps; ++i)
    if (mask[i] > 1) QC_FAIL(QC_ERR_RANGE, "schedule entries must be 0 or 1");
  ctx->cache_mask.assign(mask, mask + row * steps);
  ctx->mask_steps = steps;
  return QC_OK;
}

// Waits for the stream, then reports and clears what the kernels flagged on the device.
static int report_flags(qc_ctx *ctx, hipStream_t st) {
  int f = 0;
  QC_HIP(hipMemcpyAsync(&f, ctx->dev_flags, sizeof(int), hipMemcpyDeviceToHost, st));
  QC_HIP(hipStreamSynchronize(st));
  if (f) {
    QC_HIP(hipMemsetAsync(ctx->dev_flags, 0, sizeof(int), st));
    QC_HIP(hipStreamSynchronize(st));
  }
  if (f & 1) QC_FAIL(QC_ERR_RANGE, "a class label outside [0, %d] was passed (the null label is %d); it was clamped", ctx->d.num_classes, ctx->d.num_classes);
  return QC_OK;
}

int qc_check(qc_ctx *ctx, void *stream) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (!ctx->weights_loaded) return QC_OK;
  return report_flags(ctx, static_cast<hipStream_t>(stream));
}

int qc_keep_qkv_f32(qc_ctx *ctx, int on) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  ctx->keep_qkv_f32 = on != 0;
  return QC_OK;
}

// Conditioning vectors for nw timesteps and one set of labels: c[w * B + b, :] = tMLP(sinusoid(t[w])) + E[y_b]
// (null label for b >= n_labels), rows 0 .. nw*B of the table.
static int run_cond(qc_ctx *ctx, const int32_t *t, int nw, const int32_t *labels, int n_labels, int B, hipStream_t st) {
  const int D = ctx->D, fd = ctx->d.freq_dim;
  bool affine = true;
  for (int w = 2; w < nw; ++w) affine = affine && (t[w] - t[w - 1] == t[1] - t[0]);
  if (affine) {
    QC_HIP(launch_time_embed(t[0], nw > 1 ? t[1] - t[0] : 0, nw, fd, ctx->emb, st));
  } else {
    for (int w = 0; w < nw; ++w) QC_HIP(launch_time_embed(t[w], 0, 1, fd, ctx->emb + (size_t)w * fd, st));
  }
  QC_HIP(launch_small_linear(ctx->emb, fd, ctx->t_w1, ctx->t_b1, ctx->h1, D, nw, D, fd, 0, 1, st));
  QC_HIP(launch_small_linear(ctx->h1, D, ctx->t_w2, ctx->t_b2, ctx->te, D, nw, D, D, 0, 0, st));
  QC_HIP(launch_cond_finish(ctx->te, ctx->label_table, labels, n_labels, ctx->d.num_classes, nw * B, B, D, ctx->cond, ctx->dev_flags, st));
  return QC_OK;
}

// Everything of the network that depends only on (timestep, label), for nw sampler steps at once: the
// conditioning vectors, the final layer's modulation and the adaLN projections of every block.  One
// int8 GEMM with nw * B rows replaces nw weight-bandwidth-bound launches with B rows each, and the
// steps themselves start at the patch embedding.  Step w of the window owns rows w*B .. (w+1)*B.
static int prepare_window(qc_ctx *ctx, const int32_t *t, int nw, const int32_t *labels, int n_labels, int B, bool gates_only,
                          hipStream_t st) {
  const int D = ctx->D, L = ctx->L, rows = nw * B;
  if (rows > ctx->win_rows) QC_FAIL(QC_ERR_WORKSPACE, "conditioning window of %d rows exceeds %d", rows, ctx->win_rows);
  int rc = run_cond(ctx, t, nw, labels, n_labels, B, st);
  if (rc) return rc;
  QC_HIP(launch_silu_quant(ctx->cond, rows, D, L, ctx->dev_qp + QC_SITE_ADA, QC_NUM_SITES, ctx->silu_q,
                           (size_t)ctx->win_rows * D, st));
  QC_HIP(launch_small_linear(ctx->cond, D, ctx->fada_w, ctx->fada_b, ctx->fmod, 2 * D, rows, 2 * D, D, 1, 0, st));
  return run_adaln(ctx, 0, L, 0, rows, gates_only, st);
}

// The x-dependent part of the network on one sub-batch (rows b0 .. b0+nb of the effective batch) in three
// pieces, so that the caller can interleave the launches of several sub-batches: the patch embedding ...
// The token tensor of the network-level calls: float32, or bfloat16 in the reduced-precision variant (the same
// buffer, half used); element offset -> address.
static void *tokens_at(qc_ctx *ctx, size_t elem) {
  return reinterpret_cast<char *>(ctx->tokens) + elem * (ctx->stream_bf16 ? 2 : 4);
}

static int denoise_head(qc_ctx *ctx, const float *x, int n_labels, const Sub &sb, hipStream_t st) {
  const int D = ctx->D;
  QC_HIP(launch_embed(x, ctx->patch_w, ctx->patch_b, ctx->pos, tokens_at(ctx, (size_t)sb.b0 * ctx->T * D), ctx->stream_bf16,
                      sb.nb, n_labels, ctx->C, ctx->d.latent_h, ctx->d.latent_w, ctx->d.patch, D, sb.b0, st));
  return QC_OK;
}

// ... all blocks of a cached step in one launch, and the final layer.
static int denoise_tail(qc_ctx *ctx, const Sub &sb, int mode, float *eps_out, hipStream_t st) {
  const int D = ctx->D, L = ctx->L, B = sb.nb;
  const size_t lat = (size_t)ctx->C * ctx->d.latent_h * ctx->d.latent_w;
  void *tokens = tokens_at(ctx, (size_t)sb.b0 * ctx->T * D);
  const int xb = ctx->stream_bf16;
  if (mode == QC_CACHED) {
    const size_t slot = (size_t)ctx->max_batch * ctx->T * D;
    QC_PROF(QC_K_CACHED_BLOCKS);
    QC_HIP(launch_cached_blocks(tokens, xb, cache_at(ctx, 0, 0, (size_t)sb.b0 * ctx->T * D), 2 * slot, slot, ctx->mod + (size_t)sb.r0 * 6 * D,
                                (size_t)ctx->win_rows * 6 * D, 6 * D, L, B, ctx->T, D, ctx->cache_bf16, st));
  }
  QC_HIP(launch_final(tokens, xb, ctx->fmod + (size_t)sb.r0 * 2 * D, ctx->flin_w, ctx->flin_b, eps_out + (size_t)sb.b0 * lat, B,
                      ctx->C, ctx->d.latent_h, ctx->d.latent_w, ctx->d.patch, D, st));
  return QC_OK;
}

// Small batches leave most of the chip idle inside every kernel (a launch has fewer workgroups than
// compute units, and every dependent kernel pays a few microseconds of dispatch latency), and latents
// are independent, so the batch may be cut into sub-batches that run the network concurrently: the first
// on the caller's stream, the others on internal streams, their launches interleaved block by block.
static int choose_lanes(qc_ctx *ctx, int B) {
  int n = (long long)B * ctx->T <= 4096 ? 2 : 1;
  if (n > MAX_LANES) n = MAX_LANES;
  if (n > B) n = B;
  return n < 1 ? 1 : n;
}

// One denoiser evaluation whose conditioning sits in slot `w` of the prepared window.  sched (optional,
// [L][2], 1 = recompute) decides per (block, module) instead of `mode`.
static int denoise_impl(qc_ctx *ctx, const float *x, int n_labels, int B, int mode, int w, float *eps_out, hipStream_t st,
                        const unsigned char *sched = nullptr) {
  bool mixed = false;
  if (sched) {
    int n_full = 0;
    for (int i = 0; i < 2 * ctx->L; ++i) n_full += sched[i] ? 1 : 0;
    for (int i = 0; i < 2 * ctx->L; ++i)
      if (!sched[i] && ctx->cache_batch[i] != B)
        QC_FAIL(QC_ERR_STATE, "block %d reuses cached tensor %d but the cache does not hold batch %d", i / 2, i % 2, B);
    if (n_full == 2 * ctx->L) mode = QC_FULL;
    else if (n_full == 0) mode = QC_CACHED;
    else mixed = true;
  }
  const int lanes = choose_lanes(ctx, B);
  Sub sub[MAX_LANES];
  hipStream_t ls[MAX_LANES];
  for (int i = 0, b0 = 0; i < lanes; ++i) {
    sub[i] = Sub{b0, B / lanes + (i < B % lanes ? 1 : 0), i, w * B + b0};
    b0 += sub[i].nb;
  }
  ls[0] = st;
  if (lanes > 1) {
    if (!ctx->ev_fork) QC_HIP(hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming));
    QC_HIP(hipEventRecord(ctx->ev_fork, st));
    for (int i = 1; i < lanes; ++i) {
      if (!ctx->lane_stream[i]) QC_HIP(hipStreamCreateWithFlags(&ctx->lane_stream[i], hipStreamNonBlocking));
      if (!ctx->ev_join[i]) QC_HIP(hipEventCreateWithFlags(&ctx->ev_join[i], hipEventDisableTiming));
      ls[i] = ctx->lane_stream[i];
      QC_HIP(hipStreamWaitEvent(ls[i], ctx->ev_fork, 0));
    }
  }
  int rc = QC_OK;
  for (int i = 0; i < lanes && !rc; ++i) rc = denoise_head(ctx, x, n_labels, sub[i], ls[i]);
  if (mode == QC_FULL || mixed)
    for (int l = 0; l < ctx->L && !rc; ++l)
      for (int i = 0; i < lanes && !rc; ++i)
        rc = run_block_full(ctx, l, tokens_at(ctx, (size_t)sub[i].b0 * ctx->T * ctx->D), ctx->stream_bf16, sub[i], ls[i],
                            mixed ? sched[2 * l] != 0 : true, mixed ? sched[2 * l + 1] != 0 : true);
  for (int i = 0; i < lanes && !rc; ++i) rc = denoise_tail(ctx, sub[i], mixed ? QC_FULL : mode, eps_out, ls[i]);
  // join even after an error so that the internal streams never run past the caller's stream unobserved
  for (int i = 1; i < lanes; ++i) {
    QC_HIP(hipEventRecord(ctx->ev_join[i], ls[i]));
    QC_HIP(hipStreamWaitEvent(st, ctx->ev_join[i], 0));
  }
  if (rc == QC_OK && mixed) {
    for (int i = 0; i < 2 * ctx->L; ++i)
      if (sched[i]) ctx->cache_batch[i] = B;
  } else if (rc == QC_OK && mode == QC_FULL) {
    for (int &v : ctx->cache_batch) v = B;
  }
  return rc;
}

static int check_denoise(qc_ctx *ctx, const float *x, const int32_t *labels, int n_labels, int B, int mode) {
  int rc = check_ready(ctx, B);
  if (rc) return rc;
  if (!x || !labels) QC_FAIL(QC_ERR_NULL, "x or labels is NULL");
  if (n_labels < 1 || (B != n_labels && B != 2 * n_labels))
    QC_FAIL(QC_ERR_SHAPE, "effective batch %d must be n_labels (%d) or twice that", B, n_labels);
  if (mode != QC_FULL && mode != QC_CACHED) QC_FAIL(QC_ERR_RANGE, "mode must be QC_FULL or QC_CACHED");
  if (mode == QC_CACHED)
    for (int v : ctx->cache_batch)
      if (v != B) QC_FAIL(QC_ERR_STATE, "cached step requested but the cache does not hold batch %d", B);
  return QC_OK;
}

int qc_denoise(qc_ctx *ctx, const float *x, int t, const int32_t *labels, int n_labels, int B, int mode, float *eps_out,
               void *stream) {
  int rc = check_denoise(ctx, x, labels, n_labels, B, mode);
  if (rc) return rc;
  if (!eps_out) QC_FAIL(QC_ERR_NULL, "eps_out is NULL");
  if (t < 0) QC_FAIL(QC_ERR_RANGE, "timestep must be non-negative");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int32_t t32 = t;
  rc = prepare_window(ctx, &t32, 1, labels, n_labels, B, mode == QC_CACHED, st);
  if (rc) return rc;
  return denoise_impl(ctx, x, n_labels, B, mode, 0, eps_out, st);
}

static int step_mode(const qc_ctx *ctx, int step_index, int force_mode) {
  return force_mode >= 0 ? force_mode : (step_index % ctx->d.cache_interval == 0 ? QC_FULL : QC_CACHED);
}

// Row of the installed per-(step, block, module) schedule for this step, or null when the interval rule (or a
// forced mode) decides.
static const unsigned char *step_sched(const qc_ctx *ctx, int step_index, int force_mode) {
  if (force_mode >= 0 || ctx->cache_mask.empty()) return nullptr;
  return ctx->cache_mask.data() + (size_t)step_index * ctx->L * 2;
}

// One sampler step whose conditioning sits in slot w of the prepared window: denoiser, CFG, DDIM update, VC.
static int sample_step_prepared(qc_ctx *ctx, float *x, int B, int mode, int w, double abar_t, double abar_prev, float cfg_scale,
                                const float *K_t, hipStream_t st, const unsigned char *sched = nullptr) {
  const int Beff = cfg_scale > 0.0f ? 2 * B : B;
  int rc = denoise_impl(ctx, x, B, Beff, mode, w, ctx->eps, st, sched);
  if (rc) return rc;
  const double cx = std::sqrt(abar_prev / abar_t);
  const double ce = std::sqrt(1.0 - abar_prev) - cx * std::sqrt(1.0 - abar_t);
  QC_PROF(QC_K_DDIM_VC);
  QC_HIP(launch_ddim_vc(x, ctx->eps, B, ctx->C, ctx->d.latent_h * ctx->d.latent_w, cx, ce, cfg_scale, K_t, st));
  return QC_OK;
}

int qc_sample_step(qc_ctx *ctx, float *x, const int32_t *labels, int B, int step_index, int t, double abar_t,
                   double abar_prev, float cfg_scale, const float *K_t, int force_mode, void *stream) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  if (step_index < 0 || t < 0) QC_FAIL(QC_ERR_RANGE, "step index and timestep must be non-negative");
  if (!(abar_t > 0.0 && abar_t <= 1.0) || !(abar_prev > 0.0 && abar_prev <= 1.0)) QC_FAIL(QC_ERR_RANGE, "abar values must be in (0, 1]");
  if (force_mode != -1 && force_mode != QC_FULL && force_mode != QC_CACHED) QC_FAIL(QC_ERR_RANGE, "force_mode must be -1, QC_FULL or QC_CACHED");
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int Beff = cfg_scale > 0.0f ? 2 * B : B;
  if (force_mode < 0 && !ctx->cache_mask.empty() && step_index >= ctx->mask_steps)
    QC_FAIL(QC_ERR_RANGE, "step %d is outside the installed cache schedule of %d steps", step_index, ctx->mask_steps);
  const unsigned char *sched = step_sched(ctx, step_index, force_mode);
  const int mode = sched ? QC_FULL : step_mode(ctx, step_index, force_mode);   // with a schedule the per-module check is in the denoiser
  int rc = check_denoise(ctx, x, labels, B, Beff, mode);
  if (rc) return rc;
  const int32_t t32 = t;
  rc = prepare_window(ctx, &t32, 1, labels, B, Beff, !sched && mode == QC_CACHED, st);
  if (rc) return rc;
  return sample_step_prepared(ctx, x, B, mode, 0, abar_t, abar_prev, cfg_scale, K_t, st, sched);
}

int qc_sample(qc_ctx *ctx, float *x, const int32_t *labels, int B, int steps, float cfg_scale, const float *K, void *stream) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  std::vector<int32_t> t(steps > 0 ? steps : 1);
  std::vector<double> at(t.size()), ap(t.size());
  int rc = qc_ddim_schedule(steps, t.data(), at.data(), ap.data());
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int Beff = cfg_scale > 0.0f ? 2 * B : B;
  rc = check_denoise(ctx, x, labels, B, Beff, QC_FULL);
  if (rc) return rc;
  if (!ctx->cache_mask.empty() && steps > ctx->mask_steps)
    QC_FAIL(QC_ERR_RANGE, "%d steps requested but the installed cache schedule has %d", steps, ctx->mask_steps);
  // the whole schedule is known: conditioning and adaLN projections are prepared a window of steps at a time
  const int W = std::max(1, std::min(steps, ctx->win_rows / Beff));
  for (int i0 = 0; i0 < steps; i0 += W) {
    const int nw = std::min(W, steps - i0);
    rc = prepare_window(ctx, t.data() + i0, nw, labels, B, Beff, false, st);
    if (rc) return rc;
    for (int i = i0; i < i0 + nw; ++i) {
      rc = sample_step_prepared(ctx, x, B, step_mode(ctx, i, -1), i - i0, at[i], ap[i], cfg_scale,
                                K ? K + (size_t)i * ctx->C : nullptr, st, step_sched(ctx, i, -1));
      if (rc) return rc;
    }
  }
  return QC_OK;
}

// ---------------------------------------------------------------- profiling
int qc_profile_begin(qc_ctx *ctx) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  ctx->prof_on = true;
  ctx->prof_used = 0;
  ctx->prof_cls.clear();
  return QC_OK;
}

int qc_profile_end(qc_ctx *ctx, int n_classes, int32_t *launches, float *total_ms, void *stream) {
  if (!ctx || !launches || !total_ms) QC_FAIL(QC_ERR_NULL, "a pointer is NULL");
  if (n_classes < QC_K_COUNT) QC_FAIL(QC_ERR_SHAPE, "n_classes must be at least %d", QC_K_COUNT);
  ctx->prof_on = false;
  QC_HIP(hipStreamSynchronize(static_cast<hipStream_t>(stream)));
  for (int i = 0; i < n_classes; ++i) { launches[i] = 0; total_ms[i] = 0.0f; }
  for (size_t i = 0; i < ctx->prof_cls.size(); ++i) {
    float ms = 0.0f;
    QC_HIP(hipEventElapsedTime(&ms, ctx->prof_pool[2 * i], ctx->prof_pool[2 * i + 1]));
    launches[ctx->prof_cls[i]] += 1;
    total_ms[ctx->prof_cls[i]] += ms;
  }
  ctx->prof_used = 0;
  ctx->prof_cls.clear();
  return QC_OK;
}

// ------------------------------------------------------------ calibration
static inline float ord2f(int i) {
  i ^= (i >> 31) & 0x7FFFFFFF;
  float f;
  std::memcpy(&f, &i, 4);
  return f;
}

}  // extern "C"

// Un-quantised fp32 forward of one sample through all blocks (the network the quantiser parameters are
// calibrated on and the reference the VC factors are fitted against): tokens must hold the embedded sample,
// cond the sample's conditioning vector.  With slots != null the min / max of the five quantiser sites of
// every block are folded into slots[l][site][2].
static int fp32_blocks_one(qc_ctx *ctx, const qc_weights_f32 *w, const float *cond, int *slots, hipStream_t st) {
  const int D = ctx->D, R = ctx->R, T = ctx->T, L = ctx->L;
  for (int l = 0; l < L; ++l) {
    const qc_block_weights_f32 &b = w->blocks[l];
    int *slot = slots ? slots + (size_t)l * QC_NUM_SITES * 2 : nullptr;
    float *mod = ctx->cal_mod;
    if (slot) QC_HIP(launch_minmax_silu(cond, D, slot + 2 * QC_SITE_ADA, st));
    QC_HIP(launch_small_linear(cond, D, b.ada_w, b.ada_b, mod, 6 * D, 1, 6 * D, D, 1, 0, st));
    QC_HIP(launch_ln_mod_quant(ctx->tokens, 0, mod, mod + D, 6 * D, T, D, T, nullptr, nullptr, ctx->cal_h, st));
    if (slot) QC_HIP(launch_minmax(ctx->cal_h, (size_t)T * D, slot + 2 * QC_SITE_QKV, st));
    QC_HIP(launch_linear_f32(ctx->cal_h, b.qkv_w, b.qkv_b, ctx->qkv, T, 3 * D, D, 0, st));
    QC_HIP(launch_attention(ctx->qkv, 1, T, ctx->H, ctx->hd, nullptr, nullptr, ctx->cal_o, st));
    if (slot) QC_HIP(launch_minmax(ctx->cal_o, (size_t)T * D, slot + 2 * QC_SITE_PROJ, st));
    QC_HIP(launch_linear_f32(ctx->cal_o, b.proj_w, b.proj_b, ctx->cal_a, T, D, D, 0, st));
    QC_HIP(launch_cache_reuse(ctx->tokens, 0, ctx->cal_a, mod + 2 * D, 6 * D, 1, T, D, false, st));
    QC_HIP(launch_ln_mod_quant(ctx->tokens, 0, mod + 3 * D, mod + 4 * D, 6 * D, T, D, T, nullptr, nullptr, ctx->cal_h, st));
    if (slot) QC_HIP(launch_minmax(ctx->cal_h, (size_t)T * D, slot + 2 * QC_SITE_FC1, st));
    QC_HIP(launch_linear_f32(ctx->cal_h, b.fc1_w, b.fc1_b, ctx->cal_u, T, R, D, 2, st));
    if (slot) QC_HIP(launch_minmax(ctx->cal_u, (size_t)T * R, slot + 2 * QC_SITE_FC2, st));
    QC_HIP(launch_linear_f32(ctx->cal_u, b.fc2_w, b.fc2_b, ctx->cal_a, T, D, R, 0, st));
    QC_HIP(launch_cache_reuse(ctx->tokens, 0, ctx->cal_a, mod + 5 * D, 6 * D, 1, T, D, false, st));
  }
  return QC_OK;
}

// eps[B] of the un-quantised network; x holds n_src latents, batch element b reads latent b % n_src
// (guidance runs the same latents with the labels and with the null label).
static int denoise_f32_impl(qc_ctx *ctx, const qc_weights_f32 *w, const float *x, int n_src, int t, const int32_t *labels,
                            int n_labels, int B, float *eps_out, hipStream_t st) {
  const int D = ctx->D;
  const size_t lat = (size_t)ctx->C * ctx->d.latent_h * ctx->d.latent_w;
  const int32_t t32 = t;
  int rc = run_cond(ctx, &t32, 1, labels, n_labels, B, st);
  if (rc) return rc;
  QC_HIP(launch_small_linear(ctx->cond, D, ctx->fada_w, ctx->fada_b, ctx->fmod, 2 * D, B, 2 * D, D, 1, 0, st));
  for (int b = 0; b < B; ++b) {
    QC_HIP(launch_embed(x, ctx->patch_w, ctx->patch_b, ctx->pos, ctx->tokens, 0, 1, n_src, ctx->C, ctx->d.latent_h, ctx->d.latent_w,
                        ctx->d.patch, D, b, st));
    rc = fp32_blocks_one(ctx, w, ctx->cond + (size_t)b * D, nullptr, st);
    if (rc) return rc;
    QC_HIP(launch_final(ctx->tokens, 0, ctx->fmod + (size_t)b * 2 * D, ctx->flin_w, ctx->flin_b, eps_out + b * lat, 1, ctx->C,
                        ctx->d.latent_h, ctx->d.latent_w, ctx->d.patch, D, st));
  }
  return QC_OK;
}

extern "C" {

int qc_calibrate_minmax(qc_ctx *ctx, const qc_weights_f32 *w, const float *x, const int32_t *t, const int32_t *y, int n,
                        void *stream) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  int rc = check_weights(ctx, w);
  if (rc) return rc;
  if (!x || !t || !y) QC_FAIL(QC_ERR_NULL, "x, t or y is NULL");
  if (n < 1) QC_FAIL(QC_ERR_SHAPE, "n must be >= 1");
  if (!ctx->weights_loaded) QC_FAIL(QC_ERR_STATE, "weights were not loaded");
  for (int i = 0; i < n; ++i) {
    if (t[i] < 0) QC_FAIL(QC_ERR_RANGE, "timestep must be non-negative");
    if (y[i] < 0 || y[i] > ctx->d.num_classes) QC_FAIL(QC_ERR_RANGE, "label %d outside 0..%d", y[i], ctx->d.num_classes);
  }
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int D = ctx->D, L = ctx->L;
  const size_t nslots = (size_t)L * QC_NUM_SITES;
  std::vector<int> init(nslots * 2);
  for (size_t i = 0; i < nslots; ++i) {
    init[2 * i] = 0x7FFFFFFF;
    init[2 * i + 1] = (int)0x80000000;
  }
  QC_HIP(hipMemcpyAsync(ctx->cal_slots, init.data(), init.size() * sizeof(int), hipMemcpyHostToDevice, st));
  QC_HIP(hipStreamSynchronize(st));
  const size_t lat = (size_t)ctx->C * ctx->d.latent_h * ctx->d.latent_w;
  for (int i = 0; i < n; ++i) {
    QC_HIP(hipMemcpyAsync(ctx->cal_label, &y[i], sizeof(int), hipMemcpyHostToDevice, st));
    QC_HIP(hipStreamSynchronize(st));
    rc = run_cond(ctx, &t[i], 1, ctx->cal_label, 1, 1, st);
    if (rc) return rc;
    QC_HIP(launch_embed(x + i * lat, ctx->patch_w, ctx->patch_b, ctx->pos, ctx->tokens, 0, 1, 1, ctx->C, ctx->d.latent_h,
                        ctx->d.latent_w, ctx->d.patch, D, 0, st));
    rc = fp32_blocks_one(ctx, w, ctx->cond, ctx->cal_slots, st);
    if (rc) return rc;
  }
  std::vector<int> got(nslots * 2);
  QC_HIP(hipMemcpyAsync(got.data(), ctx->cal_slots, got.size() * sizeof(int), hipMemcpyDeviceToHost, st));
  QC_HIP(hipStreamSynchronize(st));
  for (size_t i = 0; i < nslots; ++i) {
    // Eq. 2-3 in fp32: range widened to contain 0, s = (u - l) / 255, z = round(-l / s)
    float lo = std::fmin(ord2f(got[2 * i]), 0.0f), hi = std::fmax(ord2f(got[2 * i + 1]), 0.0f);
    float s = 1.0f;
    int z = 0;
    if (hi > lo) {
      s = (hi - lo) / 255.0f;
      float zf = std::nearbyintf(-lo / s);
      z = (int)std::fmin(std::fmax(zf, 0.0f), 255.0f);
    }
    rc = qc_set_act_qparams(ctx, (int)(i / QC_NUM_SITES), (int)(i % QC_NUM_SITES), s, z);
    if (rc) return rc;
  }
  return QC_OK;
}

int qc_vc_fit(const float *x_hat, const float *x_ref, int B, int C, int H, int W, float eps, double *work, float *K_t, void *stream) {
  if (!x_hat || !x_ref || !work || !K_t) QC_FAIL(QC_ERR_NULL, "a pointer is NULL");
  if (B < 1 || C < 1 || H < 1 || W < 1) QC_FAIL(QC_ERR_SHAPE, "B, C, H, W must be positive");
  if (!(eps >= 0.0f)) QC_FAIL(QC_ERR_RANGE, "eps must be >= 0");
  if (reinterpret_cast<uintptr_t>(work) & 7u) QC_FAIL(QC_ERR_ALIGN, "work must be 8-byte aligned");
  hipStream_t st = static_cast<hipStream_t>(stream);
  QC_HIP(launch_vc_fit(x_hat, x_ref, B, C, H * W, eps, work, K_t, st));
  return QC_OK;
}

}  // extern "C"

// Partial sums of qc_vc_fit_static: one copy per GPU, addressed through the pointer hipGetSymbolAddress returns for the
// current device (the array's name is only a host-side handle).
static __device__ __align__(256) double vc_fit_scratch[2 * QC_VC_FIT_STATIC_MAX_PLANES];
static std::mutex vc_fit_scratch_mutex;
static double *vc_fit_scratch_ptr[64] = {};      // per device, filled on the first call there

static int vc_fit_scratch_for_current_device(double **out) {
  int dev = 0;
  QC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= 64) QC_FAIL(QC_ERR_UNSUPPORTED, "device index %d outside 0..63", dev);
  std::lock_guard<std::mutex> lock(vc_fit_scratch_mutex);
  if (!vc_fit_scratch_ptr[dev]) {
    double *p = nullptr;
    QC_HIP(hipGetSymbolAddress((void **)&p, HIP_SYMBOL(vc_fit_scratch)));
    if (!p) QC_FAIL(QC_ERR_HIP, "hipGetSymbolAddress returned a null address");
    vc_fit_scratch_ptr[dev] = p;
  }
  *out = vc_fit_scratch_ptr[dev];
  return QC_OK;
}

extern "C" {

int qc_vc_fit_static(const float *x_hat, const float *x_ref, int B, int C, int H, int W, float eps, float *K_t, void *stream) {
  if (!x_hat || !x_ref || !K_t) QC_FAIL(QC_ERR_NULL, "a pointer is NULL");
  if (B < 1 || C < 1 || H < 1 || W < 1) QC_FAIL(QC_ERR_SHAPE, "B, C, H, W must be positive");
  if (!(eps >= 0.0f)) QC_FAIL(QC_ERR_RANGE, "eps must be >= 0");
  if ((long long)B * C > QC_VC_FIT_STATIC_MAX_PLANES)
    QC_FAIL(QC_ERR_WORKSPACE, "B * C = %lld planes exceed the %d the library's fixed scratch holds", (long long)B * C,
            QC_VC_FIT_STATIC_MAX_PLANES);
  double *work = nullptr;
  int rc = vc_fit_scratch_for_current_device(&work);
  if (rc) return rc;
  QC_HIP(launch_vc_fit(x_hat, x_ref, B, C, H * W, eps, work, K_t, static_cast<hipStream_t>(stream)));
  return QC_OK;
}

int qc_denoise_f32(qc_ctx *ctx, const qc_weights_f32 *w, const float *x, int t, const int32_t *labels, int n_labels, int B,
                   float *eps_out, void *stream) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  int rc = check_weights(ctx, w);
  if (rc) return rc;
  if (!x || !labels || !eps_out) QC_FAIL(QC_ERR_NULL, "x, labels or eps_out is NULL");
  if (!ctx->weights_loaded) QC_FAIL(QC_ERR_STATE, "weights were not loaded");
  if (B < 1 || B > ctx->max_batch) QC_FAIL(QC_ERR_SHAPE, "batch %d outside 1..%d", B, ctx->max_batch);
  if (n_labels < 1 || (B != n_labels && B != 2 * n_labels))
    QC_FAIL(QC_ERR_SHAPE, "effective batch %d must be n_labels (%d) or twice that", B, n_labels);
  if (t < 0) QC_FAIL(QC_ERR_RANGE, "timestep must be non-negative");
  return denoise_f32_impl(ctx, w, x, n_labels, t, labels, n_labels, B, eps_out, static_cast<hipStream_t>(stream));
}

int qc_vc_fit_sampler(qc_ctx *ctx, const qc_weights_f32 *w, float *x_hat, float *x_ref, const int32_t *labels, int B, int steps,
                      float cfg_scale, float vc_eps, float *K_out, void *stream) {
  if (!ctx) QC_FAIL(QC_ERR_NULL, "ctx is NULL");
  int rc = check_weights(ctx, w);
  if (rc) return rc;
  if (!x_hat || !x_ref || !K_out) QC_FAIL(QC_ERR_NULL, "x_hat, x_ref or K_out is NULL");
  if (x_hat == x_ref) QC_FAIL(QC_ERR_SHAPE, "x_hat and x_ref must be different buffers");
  if (!(vc_eps >= 0.0f)) QC_FAIL(QC_ERR_RANGE, "vc_eps must be >= 0");
  std::vector<int32_t> t(steps > 0 ? steps : 1);
  std::vector<double> at(t.size()), ap(t.size());
  rc = qc_ddim_schedule(steps, t.data(), at.data(), ap.data());
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(stream);
  const int Beff = cfg_scale > 0.0f ? 2 * B : B;
  rc = check_denoise(ctx, x_hat, labels, B, Beff, QC_FULL);
  if (rc) return rc;
  if (!ctx->cache_mask.empty() && steps > ctx->mask_steps)
    QC_FAIL(QC_ERR_RANGE, "%d steps requested but the installed cache schedule has %d", steps, ctx->mask_steps);
  const int HW = ctx->d.latent_h * ctx->d.latent_w, C = ctx->C;
  for (int i = 0; i < steps; ++i) {
    const double cx = std::sqrt(ap[i] / at[i]);
    const double ce = std::sqrt(1.0 - ap[i]) - cx * std::sqrt(1.0 - at[i]);
    // reference: un-quantised network, every step in full, no VC
    rc = denoise_f32_impl(ctx, w, x_ref, B, t[i], labels, B, Beff, ctx->eps_ref, st);
    if (rc) return rc;
    QC_HIP(launch_ddim_vc(x_ref, ctx->eps_ref, B, C, HW, cx, ce, cfg_scale, nullptr, st));
    // accelerated: quantised network under the cache rule, VC with the factor fitted at this very step
    const int mode = step_mode(ctx, i, -1);
    const unsigned char *sched = step_sched(ctx, i, -1);
    rc = prepare_window(ctx, &t[i], 1, labels, B, Beff, !sched && mode == QC_CACHED, st);
    if (rc) return rc;
    rc = denoise_impl(ctx, x_hat, B, Beff, mode, 0, ctx->eps, st, sched);
    if (rc) return rc;
    QC_HIP(launch_ddim_vc(x_hat, ctx->eps, B, C, HW, cx, ce, cfg_scale, nullptr, st));
    float *K_i = K_out + (size_t)i * C;
    QC_HIP(launch_vc_fit(x_hat, x_ref, B, C, HW, vc_eps, ctx->vcfit_work, K_i, st));
    QC_HIP(launch_vc(x_hat, K_i, nullptr, B, C, HW, st));
  }
  return QC_OK;
}

}  // extern "C"
