// Internal declarations shared by the host layer and the kernel launchers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <vector>
#include "qc.h"

namespace qc {

// Activation quantiser parameters as the kernels use them: zero point already
// shifted to the signed code range (paper's z minus 128).
struct QParam {
  float s;
  int z;
};

// One quantised weight matrix in the arena.
struct LinearQ {
  void *q = nullptr;         // int8 [N, K] or packed nibbles [N, K/2]
  void *qt = nullptr;        // the same codes in MFMA fragment order for the large-M kernel, or null
  float *scale = nullptr;    // [N]
  int32_t *wsum = nullptr;   // [N]
  float *bias = nullptr;     // [N]
  int N = 0, K = 0;
};

void set_error(const char *fmt, ...);

// ---- epilogues of the int8 GEMM
enum Epi { EPI_F32 = 0, EPI_GELU_Q = 1, EPI_RESID = 2, EPI_QKV = 3 };

struct GemmArgs {
  const int8_t *A;           // [M, lda] signed codes
  const void *W;             // [N, K] int8 or [N, K/2] packed
  const void *Wt;            // the same codes in MFMA fragment order (launch_tile_weight), or null
  const float *w_scale;
  const int32_t *wsum;
  const float *bias;         // may be null
  int M, N, K, lda;
  int w4;                    // weights are packed nibbles
  // activation parameters of the input: either by value or from device memory
  float a_scale;
  int a_zp;                  // signed
  const QParam *a_qp;        // if non-null overrides a_scale / a_zp
  // batching over blockIdx.z (element strides; 0 = shared)
  long long zs_A, zs_W, zs_vecN, zs_out;   // zs_W in bytes, the others in elements
  int zs_qp;
  // subset of output rows: when sel_D > 0 the launch covers 2*sel_D outputs,
  // logical column j maps to j + 2*sel_D for j < sel_D and j + 4*sel_D otherwise
  // (the two gate chunks of an adaLN projection).
  int sel_D;
  int xcd_m;                 // XCD grid rows (set by the launcher)
  int group_m;               // large-M kernel: tile rows per group of its tile order (set by the launcher)
  // EPI_F32
  float *y;
  int ldy;
  int32_t *acc_out;          // optional raw accumulators [M, N]
  // EPI_GELU_Q
  int8_t *q_out;
  int ldq;
  const QParam *o_qp;        // output quantiser
  // EPI_RESID
  void *cache_out;           // [M, N] fp32, or bfloat16 when cache_bf16 is set
  int cache_bf16;
  void *x;                   // [M, N] residual stream (fp32, or bfloat16 when x_bf16 is set), updated in place
  int x_bf16;
  const float *gate;         // [B, ld_gate]
  int ld_gate;
  int rows_per_batch;        // T
  // EPI_QKV: the float32 Q | K | V columns go out in the attention kernel's head-major layouts: Q and K
  // [B, H, T, hd]; V transposed and key-permuted [B, H, DP, Tp] (DP = hd rounded up to 16, Tp = T rounded up to 64);
  // y, when set, also receives them row-major
  float *q32, *k32, *vt32;
  int heads, hd, DP, Tp;
};

// position of key t inside V^T rows: within each group of 32 keys the units of 4 keys are interleaved so that
// the 8 keys a lane of the P^T operand owns (4g..4g+3 and 16+4g..16+4g+3) are contiguous
__host__ __device__ inline int vt_pos(int t) {
  const int u = (t >> 2) & 7;
  return (t & ~31) | ((((u & 3) << 1) | (u >> 2)) << 2) | (t & 3);
}

// ---- storage formats.  The cached tensors and, in the reduced-precision variant, the residual stream are stored as
// fp32 or as bfloat16 (round to nearest even of the fp32 value); element i of a tensor sits at index i of either format.
__host__ __device__ inline unsigned short bf16_bits(float v) {
  unsigned u = __builtin_bit_cast(unsigned, v);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (unsigned short)(u >> 16);
}
__host__ __device__ inline float bf16_value(unsigned short h) { return __builtin_bit_cast(float, (unsigned)h << 16); }
// element / four elements of the residual stream (bf != 0: bfloat16); i4 counts groups of four elements
__device__ __forceinline__ float stream_load(const void *x, size_t i, int bf) {
  return bf ? bf16_value(((const unsigned short *)x)[i]) : ((const float *)x)[i];
}
__device__ __forceinline__ void stream_store(void *x, size_t i, float v, int bf) {
  if (bf) ((unsigned short *)x)[i] = bf16_bits(v);
  else ((float *)x)[i] = v;
}
__device__ __forceinline__ float4 stream_load4(const void *x, size_t i4, int bf) {
  if (bf) {
    const uint2 r = ((const uint2 *)x)[i4];
    return make_float4(__builtin_bit_cast(float, r.x << 16), __builtin_bit_cast(float, r.x & 0xFFFF0000u),
                       __builtin_bit_cast(float, r.y << 16), __builtin_bit_cast(float, r.y & 0xFFFF0000u));
  }
  return ((const float4 *)x)[i4];
}
__device__ __forceinline__ void stream_store4(void *x, size_t i4, float4 v, int bf) {
  if (bf) {
    uint2 r;
    r.x = (unsigned)bf16_bits(v.x) | ((unsigned)bf16_bits(v.y) << 16);
    r.y = (unsigned)bf16_bits(v.z) | ((unsigned)bf16_bits(v.w) << 16);
    ((uint2 *)x)[i4] = r;
  } else {
    ((float4 *)x)[i4] = v;
  }
}

hipError_t launch_gemm(const GemmArgs &a, int epi, int nz, hipStream_t st, int site);
// row-major codes [N, K] (or packed [N, K/2]) -> fragment order; N % 32 == 0, K % 32 == 0
hipError_t launch_tile_weight(const void *q, void *qt, int N, int K, int bits, hipStream_t st);

// ---- elementwise / row kernels
hipError_t launch_quantize_act(const float *x, int8_t *q, size_t n, float s, int z_signed, hipStream_t st);
hipError_t launch_quantize_weight(const float *w, int N, int K, int bits, void *qw, float *scale, int32_t *wsum,
                                  hipStream_t st);
// x_bf16 / tok_bf16 below: the residual stream argument is bfloat16 instead of fp32
hipError_t launch_ln_mod_quant(const void *x, int x_bf16, const float *shift, const float *scale, int ld_mod, int M, int D, int T,
                               const QParam *qp, int8_t *q, float *f32_out, hipStream_t st);
hipError_t launch_small_linear(const float *x, int ldx, const float *W, const float *b, float *y, int ldy, int B, int N,
                               int K, int act_in, int act_out, hipStream_t st);
hipError_t launch_time_embed(int t_first, int t_step, int W, int dim, float *out, hipStream_t st);
hipError_t launch_cond_finish(const float *te, const float *table, const int32_t *labels, int n_labels, int null_label,
                              int rows, int B, int D, float *c, int *flags, hipStream_t st);
hipError_t launch_silu_quant(const float *c, int B, int D, int L, const QParam *qp, int qp_stride, int8_t *q,
                             size_t l_stride, hipStream_t st);
hipError_t launch_embed(const float *x, const float *pw, const float *pb, const float *pos, void *tok, int tok_bf16, int B,
                        int n_src, int C, int H, int W, int p, int D, int b_off, hipStream_t st);
hipError_t launch_final(const void *tok, int tok_bf16, const float *fmod, const float *fw, const float *fb, float *eps, int B,
                        int C, int H, int W, int p, int D, hipStream_t st);
hipError_t launch_cache_store(const float *src, void *dst, size_t n, bool bf16, hipStream_t st);
hipError_t launch_cache_reuse(void *x, int x_bf16, const void *cached, const float *gate, int ld_gate, int B, int T, int D,
                              bool bf16, hipStream_t st);
hipError_t launch_cached_blocks(void *x, int x_bf16, const void *cache, size_t cache_block_stride, size_t cache_which_stride,
                                const float *mod, size_t mod_block_stride, int ld_mod, int L, int B, int T, int D, bool bf16,
                                hipStream_t st);
hipError_t launch_ddim_vc(float *x, const float *eps, int B, int C, int HW, double cx, double ce, float cfg_scale,
                          const float *K_t, hipStream_t st);
hipError_t launch_vc(float *x, const float *K_t, const float *mu, int B, int C, int HW, hipStream_t st);
hipError_t launch_vc_fit(const float *x_hat, const float *x_ref, int B, int C, int HW, float eps, double *work, float *K_t,
                         hipStream_t st);
hipError_t launch_attention(const float *qkv, int B, int T, int H, int hd, const QParam *qp, int8_t *q_out, float *f32_out,
                            hipStream_t st);
hipError_t launch_attention_f16(const float *q32, const float *k32, const float *vt32, int B, int T, int Tp, int H, int hd,
                                int DPv, const QParam *qp, int8_t *q_out, hipStream_t st);
// calibration helpers
hipError_t launch_linear_f32(const float *x, const float *W, const float *b, float *y, int M, int N, int K, int act_out,
                             hipStream_t st);
hipError_t launch_minmax(const float *x, size_t n, int *slot, hipStream_t st);
hipError_t launch_minmax_silu(const float *x, size_t n, int *slot, hipStream_t st);
hipError_t launch_fill_i32(int *p, size_t n, int v, hipStream_t st);

}  // namespace qc
