// Bandwidth-bound kernels of the sampler step: activation / weight quantisers,
// LayerNorm + adaLN modulation + quantise, conditioning, patch embedding, final
// layer, cache store / reuse, DDIM update + variance compensation.
// One wavefront is 64 lanes; row reductions use cross-lane shuffles only.
#include "qc_internal.h"

namespace qc {

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ int wave_sum_i(int v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float silu_f(float x) { return x / (1.0f + expf(-x)); }
__device__ __forceinline__ float gelu_f(float v) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  return 0.5f * v * (1.0f + tanhf(k0 * (v + k1 * v * v * v)));
}
// Eq. 1 on signed codes: clip(round(v / s) + z, -128, 127), z already shifted.
__device__ __forceinline__ int quant_code(float v, float s, int z) {
  float r = rintf(v / s) + (float)z;
  return (int)fminf(fmaxf(r, -128.0f), 127.0f);
}
__device__ __forceinline__ unsigned pack4(int a, int b, int c, int d) {
  return (unsigned)(a & 0xFF) | ((unsigned)(b & 0xFF) << 8) | ((unsigned)(c & 0xFF) << 16) | ((unsigned)(d & 0xFF) << 24);
}

// ------------------------------------------------------------ quantize_act
__global__ __launch_bounds__(256) void quantize_act_kernel(const float *__restrict__ x, int8_t *__restrict__ q, size_t n,
                                                           float s, int z) {
  const size_t n4 = n >> 2;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    float4 v = ((const float4 *)x)[i];
    ((unsigned *)q)[i] = pack4(quant_code(v.x, s, z), quant_code(v.y, s, z), quant_code(v.z, s, z), quant_code(v.w, s, z));
  }
  if (blockIdx.x == 0) {
    size_t i = (n4 << 2) + threadIdx.x;
    if (i < n) q[i] = (int8_t)quant_code(x[i], s, z);
  }
}

hipError_t launch_quantize_act(const float *x, int8_t *q, size_t n, float s, int z, hipStream_t st) {
  if (n == 0) return hipSuccess;
  size_t blocks = ((n >> 2) + 255) / 256;
  if (blocks < 1) blocks = 1;
  if (blocks > 65536) blocks = 65536;
  hipLaunchKernelGGL(quantize_act_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, q, n, s, z);
  return hipGetLastError();
}

// ---------------------------------------------------------- quantize_weight
// One wavefront per output row: max |w|, scale, codes, row sum.
__global__ __launch_bounds__(256) void quantize_weight_kernel(const float *__restrict__ w, int N, int K, int bits,
                                                              unsigned char *__restrict__ qw, float *__restrict__ scale,
                                                              int32_t *__restrict__ wsum) {
  const int lane = threadIdx.x & 63;
  const int n = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (n >= N) return;
  const float *row = w + (size_t)n * K;
  float amax = 0.0f;
  for (int k = lane; k < K; k += 64) amax = fmaxf(amax, fabsf(row[k]));
  amax = wave_max(amax);
  const float qmax = (float)((1 << (bits - 1)) - 1);
  const float s = amax > 0.0f ? amax / qmax : 1.0f;
  int sum = 0;
  for (int k = 2 * lane; k < K; k += 128) {
    float2 v = *(const float2 *)(row + k);
    int q0 = (int)fminf(fmaxf(rintf(v.x / s), -qmax), qmax);
    int q1 = (int)fminf(fmaxf(rintf(v.y / s), -qmax), qmax);
    sum += q0 + q1;
    if (bits == 4) {
      qw[(size_t)n * (K >> 1) + (k >> 1)] = (unsigned char)((q0 & 0xF) | ((q1 & 0xF) << 4));
    } else {
      *(unsigned short *)(qw + (size_t)n * K + k) = (unsigned short)((q0 & 0xFF) | ((q1 & 0xFF) << 8));
    }
  }
  sum = wave_sum_i(sum);
  if (lane == 0) {
    scale[n] = s;
    wsum[n] = sum;
  }
}

hipError_t launch_quantize_weight(const float *w, int N, int K, int bits, void *qw, float *scale, int32_t *wsum,
                                  hipStream_t st) {
  hipLaunchKernelGGL(quantize_weight_kernel, dim3((N + 3) / 4), dim3(256), 0, st, w, N, K, bits, (unsigned char *)qw, scale,
                     wsum);
  return hipGetLastError();
}

// ------------------------------------------------ weights in fragment order
// Copies the codes of a quantised weight matrix into the order the large-M GEMM streams them in: fragment
// (n / 32, k / 32) is 64 lanes x 16 bytes (8 bytes for packed nibbles), lane l holds row n % 32 = l % 32, k values
// 16 (l / 32) .. 16 (l / 32) + 15 of the group.  One thread per (fragment, lane).
__global__ __launch_bounds__(256) void tile_weight_kernel(const unsigned char *__restrict__ q, unsigned char *__restrict__ qt, int N,
                                                          int K, int w4) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  const int ng = K / 32;
  if (i >= (size_t)(N / 32) * ng * 64) return;
  const int l = (int)(i & 63), kg = (int)((i >> 6) % ng), nb = (int)((i >> 6) / ng);
  const size_t n = (size_t)nb * 32 + (l & 31);
  const int k = kg * 32 + (l >> 5) * 16;
  if (w4) *(uint2 *)(qt + i * 8) = *(const uint2 *)(q + n * (K >> 1) + (k >> 1));
  else *(uint4 *)(qt + i * 16) = *(const uint4 *)(q + n * K + k);
}

hipError_t launch_tile_weight(const void *q, void *qt, int N, int K, int bits, hipStream_t st) {
  if (N % 32 || K % 32) return hipErrorInvalidValue;
  const size_t n = (size_t)(N / 32) * (K / 32) * 64;
  hipLaunchKernelGGL(tile_weight_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, (const unsigned char *)q,
                     (unsigned char *)qt, N, K, bits == 4 ? 1 : 0);
  return hipGetLastError();
}

// ------------------------------------------- LayerNorm + modulate + quantise
// One wavefront per token row; the row lives in registers (D <= 2048).
constexpr int LN_MAX_IT = 8;

__device__ __forceinline__ double wave_sum_d(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// The value that gets quantised is formed in fp64 and rounded to fp32 once: the codes then differ from
// exact arithmetic only where the fp32 residual stream itself does, which keeps code flips (and the
// error they seed in every later layer) at the floor.
// One workgroup per R consecutive token rows, one float4 of every row per thread (the launch sizes the workgroup to
// D / 4 rounded up to whole wavefronts, D <= 2048): every load of the rows and of their modulation vectors is issued
// at once, one memory round trip.  R = 1 gives the most workgroups (small M); R = 4 puts four times the bytes in
// flight per compute unit, which is what the memory system needs to run near its peak at large M.  The arithmetic of a
// row, and with it every code, is the same for both.
template <int R>
__global__ __launch_bounds__(512) void ln_mod_quant_kernel(const void *__restrict__ x, int x_bf16, const float *__restrict__ shift,
                                                           const float *__restrict__ scale, int ld_mod, int M, int D, int T,
                                                           const QParam *qp, int8_t *__restrict__ q,
                                                           float *__restrict__ f32_out) {
  __shared__ double red[R][16];
  __shared__ double stat[R][2];
  const int m0 = blockIdx.x * R;
  const int k = threadIdx.x * 4;
  const bool live = k < D;
  const int kc = live ? k : 0;
  float4 v[R], s4[R], c4[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int m = min(m0 + r, M - 1);             // rows beyond M re-read the last row (never stored)
    const int b = m / T;
    v[r] = stream_load4(x, ((size_t)m * D + kc) >> 2, x_bf16);
    s4[r] = *(const float4 *)(shift + (size_t)b * ld_mod + kc);
    c4[r] = *(const float4 *)(scale + (size_t)b * ld_mod + kc);
  }
  // mean and variance from one reduction of (sum, sum of squares): in fp64 the cancellation in
  // E[x^2] - mean^2 costs ~1e-13 relative for rows of O(1) values, far below the fp32 rounding of the result
  const int nw = blockDim.x >> 6;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    double sum = 0.0, sq = 0.0;
    if (live) {
      const double a = v[r].x, bq = v[r].y, c = v[r].z, d = v[r].w;
      sum = (a + bq) + (c + d);
      sq = (a * a + bq * bq) + (c * c + d * d);
    }
    sum = wave_sum_d(sum);
    sq = wave_sum_d(sq);
    if ((threadIdx.x & 63) == 0) {
      red[r][threadIdx.x >> 6] = sum;
      red[r][8 + (threadIdx.x >> 6)] = sq;
    }
  }
  __syncthreads();
  if (threadIdx.x < R) {                          // one thread per row finishes its statistics
    const int r = threadIdx.x;
    double tot = 0.0, tot2 = 0.0;
    for (int w = 0; w < nw; ++w) {
      tot += red[r][w];
      tot2 += red[r][8 + w];
    }
    const double mean = tot / (double)D;
    const double var = tot2 / (double)D - mean * mean;
    stat[r][0] = mean;
    stat[r][1] = 1.0 / sqrt(fmax(var, 0.0) + 1e-6);
  }
  __syncthreads();
  float qs = 1.0f;
  int qz = 0;
  if (qp) {
    QParam t = *qp;
    qs = t.s;
    qz = t.z;
  }
  if (!live) return;
#pragma unroll
  for (int r = 0; r < R; ++r) {
    const int m = m0 + r;
    if (m >= M) break;
    const double mean = stat[r][0], rstd = stat[r][1];
    const float h0 = (float)((v[r].x - mean) * rstd * (1.0 + (double)c4[r].x) + (double)s4[r].x);
    const float h1 = (float)((v[r].y - mean) * rstd * (1.0 + (double)c4[r].y) + (double)s4[r].y);
    const float h2 = (float)((v[r].z - mean) * rstd * (1.0 + (double)c4[r].z) + (double)s4[r].z);
    const float h3 = (float)((v[r].w - mean) * rstd * (1.0 + (double)c4[r].w) + (double)s4[r].w);
    if (q)
      *(unsigned *)(q + (size_t)m * D + k) =
          pack4(quant_code(h0, qs, qz), quant_code(h1, qs, qz), quant_code(h2, qs, qz), quant_code(h3, qs, qz));
    if (f32_out) *(float4 *)(f32_out + (size_t)m * D + k) = make_float4(h0, h1, h2, h3);
  }
}

// ---- one wavefront per token row
// The wavefront-per-row form of the same operation, for launches with thousands of rows: a lane holds NV float4 of
// the row (float4 index lane + 64 it), the (sum, sum of squares) reduction stays inside the wavefront (DPP moves inside
// rows of 16 lanes, the four row sums read back as scalars: no LDS, no barrier), a wavefront walks `rows_per_wave`
// consecutive rows with the next row's loads in flight while it works on the current one, and keeps the modulation
// vectors of the batch element in registers from row to row.  The value that is quantised is the same float64
// expression as above, rounded to float32 once.  Eq. 1 takes v * (1 / s) where that is certain to round to the same
// integer as the IEEE quotient v / s and the quotient itself otherwise (decided for a float4 of the whole wavefront at
// a time, so the common case is branch-free).
template <int CTRL>
__device__ __forceinline__ double dpp_move_d(double v) {
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const int lo = __builtin_amdgcn_update_dpp(0, (int)(unsigned)b, CTRL, 0xF, 0xF, false);
  const int hi = __builtin_amdgcn_update_dpp(0, (int)(unsigned)(b >> 32), CTRL, 0xF, 0xF, false);
  return __builtin_bit_cast(double, ((unsigned long long)(unsigned)hi << 32) | (unsigned long long)(unsigned)lo);
}
__device__ __forceinline__ double readlane_d(double v, int l) {
  const unsigned long long b = __builtin_bit_cast(unsigned long long, v);
  const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)b, l);
  const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(b >> 32), l);
  return __builtin_bit_cast(double, ((unsigned long long)hi << 32) | (unsigned long long)lo);
}
// the same value in every lane (every lane adds the same pairs in the same order)
__device__ __forceinline__ double wave_sum_dpp(double v) {
  v += dpp_move_d<0xB1>(v);     // quad_perm [1, 0, 3, 2]
  v += dpp_move_d<0x4E>(v);     // quad_perm [2, 3, 0, 1]
  v += dpp_move_d<0x141>(v);    // row_half_mirror: the other quad of the half row
  v += dpp_move_d<0x140>(v);    // row_mirror: the other half of the row of 16
  return (readlane_d(v, 0) + readlane_d(v, 16)) + (readlane_d(v, 32) + readlane_d(v, 48));
}

// Eq. 1 for four values at once, packed signed codes.  qf = v * inv_s differs from the correctly rounded quotient by
// less than 2 units in its last place (inv_s carries half a unit of relative error, the product another half, the
// quotient's own rounding a third), so when qf is farther than 4e-7 |qf| from a rounding boundary both round to the same
// integer; otherwise the quotient decides.  zu = zero point + 128 (the paper's unsigned code), clamped to 0 .. 255 and
// converted exactly; the sign bit of each byte is flipped back at the end.
__device__ __forceinline__ unsigned quant4_packed(float h0, float h1, float h2, float h3, float s, float inv_s, float zu) {
  const float h[4] = {h0, h1, h2, h3};
  float r[4];
  bool doubt = false;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const float qf = h[e] * inv_s;
    r[e] = __builtin_rintf(qf);
    doubt |= (0.5f - fabsf(qf - r[e])) <= 4e-7f * fabsf(qf);
  }
  if (__builtin_amdgcn_ballot_w64(doubt) != 0ull) {
#pragma unroll
    for (int e = 0; e < 4; ++e) r[e] = __builtin_rintf(h[e] / s);
  }
  unsigned w = 0;
#pragma unroll
  for (int e = 0; e < 4; ++e) w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(r[e] + zu, 0.0f, 255.0f), e, w);
  return w ^ 0x80808080u;
}

template <int NV>
__global__ __launch_bounds__(256) void ln_mod_quant_wave_kernel(const void *__restrict__ x, int x_bf16, const float *__restrict__ shift,
                                                                const float *__restrict__ scale, int ld_mod, int M, int D, int T,
                                                                const QParam *qp, int8_t *__restrict__ q, int rows_per_wave) {
  const int lane = threadIdx.x & 63;
  const int wv = __builtin_amdgcn_readfirstlane(blockIdx.x * 4 + (threadIdx.x >> 6));
  const int m_begin = wv * rows_per_wave;
  if (m_begin >= M) return;                        // whole wavefronts leave; the kernel has no barrier
  const int m_end = min(m_begin + rows_per_wave, M);
  const int nv4 = D >> 2;
  bool live[NV];
  int kc[NV];
#pragma unroll
  for (int it = 0; it < NV; ++it) {
    live[it] = lane + 64 * it < nv4;
    kc[it] = live[it] ? lane + 64 * it : 0;
  }
  const QParam t = *qp;
  const float qs = t.s, inv_s = 1.0f / t.s, zu = (float)(t.z + 128);
  float4 xa[NV], xn[NV], s4[NV], c4[NV];
#pragma unroll
  for (int it = 0; it < NV; ++it) xa[it] = stream_load4(x, (((size_t)m_begin * D) >> 2) + kc[it], x_bf16);
  int b_cur = -1;
  for (int m = m_begin; m < m_end; ++m) {
    const int mn = min(m + 1, m_end - 1);          // the last row is requested once more (never used)
#pragma unroll
    for (int it = 0; it < NV; ++it) xn[it] = stream_load4(x, (((size_t)mn * D) >> 2) + kc[it], x_bf16);
    const int b = m / T;
    if (b != b_cur) {
#pragma unroll
      for (int it = 0; it < NV; ++it) {
        s4[it] = *(const float4 *)(shift + (size_t)b * ld_mod + 4 * kc[it]);
        c4[it] = *(const float4 *)(scale + (size_t)b * ld_mod + 4 * kc[it]);
      }
      b_cur = b;
    }
    double sum = 0.0, sq = 0.0;
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      if (live[it]) {
        const double a = xa[it].x, bq = xa[it].y, c = xa[it].z, d = xa[it].w;
        sum += (a + bq) + (c + d);
        sq += (a * a + bq * bq) + (c * c + d * d);
      }
    }
    sum = wave_sum_dpp(sum);
    sq = wave_sum_dpp(sq);
    const double mean = sum / (double)D;
    const double var = sq / (double)D - mean * mean;
    const double rstd = 1.0 / sqrt(fmax(var, 0.0) + 1e-6);
#pragma unroll
    for (int it = 0; it < NV; ++it) {
      if (live[it]) {
        const float h0 = (float)((xa[it].x - mean) * rstd * (1.0 + (double)c4[it].x) + (double)s4[it].x);
        const float h1 = (float)((xa[it].y - mean) * rstd * (1.0 + (double)c4[it].y) + (double)s4[it].y);
        const float h2 = (float)((xa[it].z - mean) * rstd * (1.0 + (double)c4[it].z) + (double)s4[it].z);
        const float h3 = (float)((xa[it].w - mean) * rstd * (1.0 + (double)c4[it].w) + (double)s4[it].w);
        *(unsigned *)(q + (size_t)m * D + 4 * kc[it]) = quant4_packed(h0, h1, h2, h3, qs, inv_s, zu);
      }
    }
#pragma unroll
    for (int it = 0; it < NV; ++it) xa[it] = xn[it];
  }
}

hipError_t launch_ln_mod_quant(const void *x, int x_bf16, const float *shift, const float *scale, int ld_mod, int M, int D, int T,
                               const QParam *qp, int8_t *q, float *f32_out, hipStream_t st) {
  const int threads = ((D / 4 + 63) / 64) * 64;
  if (D % 4 || threads > 512) return hipErrorInvalidValue;
  const int nv = (D / 4 + 63) / 64;
  if (q && !f32_out && M >= 1024 && nv <= 5) {
    // wavefront per row; with thousands of rows four consecutive rows per wavefront (they share the batch element's
    // modulation vectors; 2 / 4 / 8 / 16 rows measured at M = 32768: 53.3 / 51.8 / 55.3 / 57.7 us)
    const int rpw = M >= 8192 ? 4 : 1;
    const int waves = (M + rpw - 1) / rpw;
    const dim3 grid((waves + 3) / 4);
    switch (nv) {
      case 1: hipLaunchKernelGGL(ln_mod_quant_wave_kernel<1>, grid, dim3(256), 0, st, x, x_bf16, shift, scale, ld_mod, M, D, T, qp, q, rpw); break;
      case 2: hipLaunchKernelGGL(ln_mod_quant_wave_kernel<2>, grid, dim3(256), 0, st, x, x_bf16, shift, scale, ld_mod, M, D, T, qp, q, rpw); break;
      case 3: hipLaunchKernelGGL(ln_mod_quant_wave_kernel<3>, grid, dim3(256), 0, st, x, x_bf16, shift, scale, ld_mod, M, D, T, qp, q, rpw); break;
      case 4: hipLaunchKernelGGL(ln_mod_quant_wave_kernel<4>, grid, dim3(256), 0, st, x, x_bf16, shift, scale, ld_mod, M, D, T, qp, q, rpw); break;
      default: hipLaunchKernelGGL(ln_mod_quant_wave_kernel<5>, grid, dim3(256), 0, st, x, x_bf16, shift, scale, ld_mod, M, D, T, qp, q, rpw); break;
    }
  } else if (M >= 8192)
    hipLaunchKernelGGL(ln_mod_quant_kernel<4>, dim3((M + 3) / 4), dim3(threads), 0, st, x, x_bf16, shift, scale, ld_mod, M, D, T,
                       qp, q, f32_out);
  else
    hipLaunchKernelGGL(ln_mod_quant_kernel<1>, dim3(M), dim3(threads), 0, st, x, x_bf16, shift, scale, ld_mod, M, D, T, qp, q,
                       f32_out);
  return hipGetLastError();
}

// ------------------------------------------------- small linear (few rows)
// y[b, n] = act_out(W[n, :] . act_in(x[b, :]) + bias[n]); one wavefront per n.  Inputs and outputs are float32 tensors;
// the arithmetic in between is float64 and the result is rounded once, so that what is stored does not depend on the
// summation order (conditioning vectors feed quantisers, where a last-bit difference can move a code).
__device__ __forceinline__ double silu_d(double x) { return x / (1.0 + exp(-x)); }

// One workgroup = 8 rows x 16 NC outputs: the (activated) inputs of the 8 rows are formed once, in float64, and kept in
// LDS (the activation is an exponential per value: it must not be repeated per output); a wavefront takes 4 NC of the
// outputs, four at a time, so that every input value read from LDS and every weight read from memory feeds 4 and 8
// multiply-adds.  NC = 4 for many rows (all steps of a window at once), NC = 1 for few (one step: the outputs must
// supply the workgroups).  Per output the summation order is fixed: lane l adds k = l, l + 64, ... in order, then the
// lanes are reduced by the shuffle tree of wave_sum_d.
template <int NC>
__global__ __launch_bounds__(256) void small_linear_kernel(const float *__restrict__ x, int ldx, const float *__restrict__ W,
                                                           const float *__restrict__ bias, float *__restrict__ y, int ldy,
                                                           int B, int N, int K, int act_in, int act_out) {
  extern __shared__ double xs[];                  // [8][K]
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int b0 = blockIdx.y * 8, n0 = blockIdx.x * (16 * NC);
  for (int i = threadIdx.x; i < 8 * K; i += 256) {
    const int r = i / K, k = i - r * K;
    double v = b0 + r < B ? (double)x[(size_t)(b0 + r) * ldx + k] : 0.0;
    if (act_in == 1) v = silu_d(v);
    xs[i] = v;
  }
  __syncthreads();
  for (int c = 0; c < NC; ++c) {
    const int n = n0 + wave * (4 * NC) + c * 4;
    if (n >= N) break;
    double acc[8][4];
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[r][j] = 0.0;
    const float *wr[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) wr[j] = W + (size_t)min(n + j, N - 1) * K;      // outputs beyond N repeat the last (not stored)
    for (int k = lane; k < K; k += 64) {
      double wv[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) wv[j] = (double)wr[j][k];
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        const double xv = xs[r * K + k];
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[r][j] = fma(wv[j], xv, acc[r][j]);
      }
    }
#pragma unroll
    for (int r = 0; r < 8; ++r)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        double t = wave_sum_d(acc[r][j]);
        if (lane == 0 && b0 + r < B && n + j < N) {
          t += bias ? (double)bias[n + j] : 0.0;
          if (act_out == 1) t = silu_d(t);
          y[(size_t)(b0 + r) * ldy + n + j] = (float)t;
        }
      }
  }
}

hipError_t launch_small_linear(const float *x, int ldx, const float *W, const float *b, float *y, int ldy, int B, int N,
                               int K, int act_in, int act_out, hipStream_t st) {
  const size_t smem = (size_t)8 * K * sizeof(double);
  if (smem > 160 * 1024) return hipErrorInvalidValue;
  static size_t attr = 0;
  if (smem > attr) {
    hipError_t e = hipFuncSetAttribute((const void *)small_linear_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e == hipSuccess)
      e = hipFuncSetAttribute((const void *)small_linear_kernel<1>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    attr = smem;
  }
  const int groups = (B + 7) / 8;
  if ((long long)groups * ((N + 63) / 64) >= 512)
    hipLaunchKernelGGL(small_linear_kernel<4>, dim3((N + 63) / 64, groups), dim3(256), smem, st, x, ldx, W, b, y, ldy, B, N, K,
                       act_in, act_out);
  else
    hipLaunchKernelGGL(small_linear_kernel<1>, dim3((N + 15) / 16, groups), dim3(256), smem, st, x, ldx, W, b, y, ldy, B, N, K,
                       act_in, act_out);
  return hipGetLastError();
}

// ----------------------------------------------------------- conditioning
// Sinusoidal timestep embedding [cos | sin], frequencies exp(-ln(1e4) j / half),
// evaluated in double so that the fp32 result is correctly rounded.
// Row w is the embedding of timestep t_first + w * t_step.
__global__ void time_embed_kernel(int t_first, int t_step, int W, int dim, float *__restrict__ out) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= W * dim) return;
  const int j = i % dim, half = dim / 2, t = t_first + (i / dim) * t_step;
  const int f = j < half ? j : j - half;
  const double a = (double)t * exp(-log(10000.0) * (double)f / (double)half);
  out[i] = (float)(j < half ? cos(a) : sin(a));
}

hipError_t launch_time_embed(int t_first, int t_step, int W, int dim, float *out, hipStream_t st) {
  hipLaunchKernelGGL(time_embed_kernel, dim3((W * dim + 255) / 256), dim3(256), 0, st, t_first, t_step, W, dim, out);
  return hipGetLastError();
}

// c[r, :] = te[r / B, :] + table[label of batch element r % B]: rows are (timestep slot, batch element)
__global__ void cond_finish_kernel(const float *__restrict__ te, const float *__restrict__ table,
                                   const int32_t *__restrict__ labels, int n_labels, int null_label, int rows, int B, int D,
                                   float *__restrict__ c, int *__restrict__ flags) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= rows * D) return;
  const int r = i / D, n = i % D, w = r / B, b = r % B;
  int y = b < n_labels ? labels[b] : null_label;
  if (y < 0 || y > null_label) {                  // the table has null_label + 1 rows: clamp, and tell the host
    if (n == 0) atomicOr(flags, 1);
    y = min(max(y, 0), null_label);
  }
  c[i] = te[(size_t)w * D + n] + table[(size_t)y * D + n];
}

hipError_t launch_cond_finish(const float *te, const float *table, const int32_t *labels, int n_labels, int null_label,
                              int rows, int B, int D, float *c, int *flags, hipStream_t st) {
  hipLaunchKernelGGL(cond_finish_kernel, dim3((rows * D + 255) / 256), dim3(256), 0, st, te, table, labels, n_labels,
                     null_label, rows, B, D, c, flags);
  return hipGetLastError();
}

// codes of SiLU(c) for the adaLN site of every block: q[l, b, n]
__global__ void silu_quant_kernel(const float *__restrict__ c, int BD, int L, const QParam *qp, int qp_stride,
                                  int8_t *__restrict__ q, size_t l_stride) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= BD) return;
  const float v = (float)silu_d((double)c[i]);      // float64 value rounded once, then Eq. 1
  for (int l = 0; l < L; ++l) {
    QParam t = qp[(size_t)l * qp_stride];
    q[(size_t)l * l_stride + i] = (int8_t)quant_code(v, t.s, t.z);
  }
}

hipError_t launch_silu_quant(const float *c, int B, int D, int L, const QParam *qp, int qp_stride, int8_t *q,
                             size_t l_stride, hipStream_t st) {
  hipLaunchKernelGGL(silu_quant_kernel, dim3((B * D + 255) / 256), dim3(256), 0, st, c, B * D, L, qp, qp_stride, q,
                     l_stride);
  return hipGetLastError();
}

// --------------------------------------------------------- patch embedding
// tok[b, t, n] = sum_f pw[n, f] * patch(b, t)[f] + pb[n] + pos[t, n], features f = (c, ph, pw).
__global__ __launch_bounds__(256) void embed_kernel(const float *__restrict__ x, const float *__restrict__ pw,
                                                    const float *__restrict__ pb, const float *__restrict__ pos,
                                                    void *__restrict__ tok, int tok_bf16, int n_src, int C, int H, int W, int p,
                                                    int D, int b_off) {
  __shared__ float patch[256];
  const int gw = W / p, T = (H / p) * gw;
  const int bt = blockIdx.x, b = bt / T, t = bt % T;
  const int F = C * p * p;
  const int ty = t / gw, tx = t % gw;
  const float *src = x + (size_t)((b + b_off) % n_src) * C * H * W;
  for (int f = threadIdx.x; f < F; f += blockDim.x) {
    const int c = f / (p * p), ph = (f / p) % p, pq = f % p;
    patch[f] = src[((size_t)c * H + ty * p + ph) * W + tx * p + pq];
  }
  __syncthreads();
  for (int n = threadIdx.x; n < D; n += blockDim.x) {
    // float64 dot product, rounded once when the token is stored
    double acc = 0.0;
    const float *wr = pw + (size_t)n * F;
    if (F % 4 == 0) {
      for (int f0 = 0; f0 < F; f0 += 16) {
        float4 w4[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w4[u] = *(const float4 *)(wr + min(f0 + 4 * u, F - 4));
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int f = f0 + 4 * u;
          if (f < F) {
            acc = fma((double)w4[u].x, (double)patch[f], acc);
            acc = fma((double)w4[u].y, (double)patch[f + 1], acc);
            acc = fma((double)w4[u].z, (double)patch[f + 2], acc);
            acc = fma((double)w4[u].w, (double)patch[f + 3], acc);
          }
        }
      }
    } else {
      for (int f = 0; f < F; ++f) acc = fma((double)wr[f], (double)patch[f], acc);
    }
    stream_store(tok, (size_t)bt * D + n, (float)((acc + (double)pb[n]) + (double)pos[(size_t)t * D + n]), tok_bf16);
  }
}

hipError_t launch_embed(const float *x, const float *pw, const float *pb, const float *pos, void *tok, int tok_bf16, int B,
                        int n_src, int C, int H, int W, int p, int D, int b_off, hipStream_t st) {
  const int T = (H / p) * (W / p);
  hipLaunchKernelGGL(embed_kernel, dim3(B * T), dim3(256), 0, st, x, pw, pb, pos, tok, tok_bf16, n_src, C, H, W, p, D, b_off);
  return hipGetLastError();
}

// ---------------------------------------------------------------- final layer
// Per token: LayerNorm, modulate with (shift, scale) = fmod[b, 0:D], fmod[b, D:2D],
// dot with the rows of the output linear that belong to the first C of the 2C
// channels, and scatter to eps[b, c, ty*p+ph, tx*p+pw] (output features (ph, pw, c)).
template <int NIT>   // 256-feature slices of a row that a wavefront holds (D <= 256 NIT)
__global__ __launch_bounds__(256) void final_kernel(const void *__restrict__ tok, int tok_bf16, const float *__restrict__ fmod,
                                                    const float *__restrict__ fw, const float *__restrict__ fb,
                                                    float *__restrict__ eps, int M, int C, int H, int W, int p, int D) {
  const int lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (m >= M) return;
  const int gw = W / p, T = (H / p) * gw;
  const int b = m / T, t = m % T, ty = t / gw, tx = t % gw;
  const float *sh = fmod + (size_t)b * 2 * D, *sc = sh + D;
  // loads never branch (chunks beyond D re-read the last chunk and are zeroed): the row and its modulation
  // vectors arrive in one memory round trip
  float4 v[NIT], s4[NIT], c4[NIT];
  int kk[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    kk[it] = min((lane + 64 * it) * 4, D - 4);
    v[it] = stream_load4(tok, ((size_t)m * D + kk[it]) >> 2, tok_bf16);
    s4[it] = *(const float4 *)(sh + kk[it]);
    c4[it] = *(const float4 *)(sc + kk[it]);
  }
  // float64 throughout (the noise estimate is rounded once, when it is stored)
  double sum = 0.0;
#pragma unroll
  for (int it = 0; it < NIT; ++it)
    if ((lane + 64 * it) * 4 < D) sum += ((double)v[it].x + (double)v[it].y) + ((double)v[it].z + (double)v[it].w);
  const double mean = wave_sum_d(sum) / (double)D;
  double sq = 0.0;
#pragma unroll
  for (int it = 0; it < NIT; ++it)
    if ((lane + 64 * it) * 4 < D) {
      const double a = v[it].x - mean, bq = v[it].y - mean, c = v[it].z - mean, d = v[it].w - mean;
      sq += (a * a + bq * bq) + (c * c + d * d);
    }
  const double rstd = 1.0 / sqrt(wave_sum_d(sq) / (double)D + 1e-6);
  double h[NIT][4];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    if ((lane + 64 * it) * 4 < D) {
      h[it][0] = (v[it].x - mean) * rstd * (1.0 + (double)c4[it].x) + (double)s4[it].x;
      h[it][1] = (v[it].y - mean) * rstd * (1.0 + (double)c4[it].y) + (double)s4[it].y;
      h[it][2] = (v[it].z - mean) * rstd * (1.0 + (double)c4[it].z) + (double)s4[it].z;
      h[it][3] = (v[it].w - mean) * rstd * (1.0 + (double)c4[it].w) + (double)s4[it].w;
    } else {
      h[it][0] = h[it][1] = h[it][2] = h[it][3] = 0.0;      // contributes nothing to the dot products below
    }
  }
  // the p*p*C dot products of this row, 16 at a time: per-lane partial sums, then a butterfly that halves
  // the number of live values with every exchange (17 shuffles for 16 sums instead of 6 each)
  const int n_out = p * p * C;
  for (int o0 = 0; o0 < n_out; o0 += 16) {
    double part[16];
#pragma unroll
    for (int u = 0; u < 16; ++u) {
      part[u] = 0.0;
      const int oi = o0 + u;
      if (oi < n_out) {
        const float *wr = fw + (size_t)((oi / C) * 2 * C + oi % C) * D;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
          const float4 w4 = *(const float4 *)(wr + kk[it]);
          part[u] += (h[it][0] * (double)w4.x + h[it][1] * (double)w4.y) + (h[it][2] * (double)w4.z + h[it][3] * (double)w4.w);
        }
      }
    }
    // after the exchange over distance 32 >> s a lane keeps the values whose index has bit (3 - s) equal to
    // its own lane bit (5 - s); after 4 exchanges lane l holds value (l >> 2) & 15 summed over 16 lanes
#pragma unroll
    for (int s2 = 0; s2 < 4; ++s2) {
      const int dist = 32 >> s2, half = 8 >> s2;
      const bool upper = (lane & dist) != 0;
#pragma unroll
      for (int u = 0; u < half; ++u) {
        const double keep = upper ? part[u + half] : part[u];
        const double send = upper ? part[u] : part[u + half];
        part[u] = keep + __shfl_xor(send, dist, 64);
      }
    }
    double r = part[0];
    r += __shfl_xor(r, 2, 64);
    r += __shfl_xor(r, 1, 64);
    const int u_mine = ((lane >> 5) & 1) * 8 + ((lane >> 4) & 1) * 4 + ((lane >> 3) & 1) * 2 + ((lane >> 2) & 1);
    const int oi = o0 + u_mine;
    if ((lane & 3) == 0 && oi < n_out) {
      const int pp = oi / C, c = oi % C;
      eps[(((size_t)b * C + c) * H + ty * p + pp / p) * W + tx * p + pp % p] = (float)(r + (double)fb[pp * 2 * C + c]);
    }
  }
}

hipError_t launch_final(const void *tok, int tok_bf16, const float *fmod, const float *fw, const float *fb, float *eps, int B,
                        int C, int H, int W, int p, int D, hipStream_t st) {
  const int M = B * (H / p) * (W / p);
  const dim3 grid((M + 3) / 4);
#define QC_FINAL(NIT) hipLaunchKernelGGL(final_kernel<NIT>, grid, dim3(256), 0, st, tok, tok_bf16, fmod, fw, fb, eps, M, C, H, W, p, D)
  if (D <= 256) QC_FINAL(1);
  else if (D <= 512) QC_FINAL(2);
  else if (D <= 1280) QC_FINAL(5);
  else QC_FINAL(LN_MAX_IT);
#undef QC_FINAL
  return hipGetLastError();
}

// ---------------------------------------------------------------- cache ops
// The cached tensors are stored as fp32 or, in the reduced-precision variant, as bfloat16; so is the residual stream.

template <bool BF16>
__device__ __forceinline__ float4 load_cached4(const void *base, size_t i4) {
  if (BF16) {
    const uint2 r = ((const uint2 *)base)[i4];       // four bfloat16
    return make_float4(__builtin_bit_cast(float, r.x << 16), __builtin_bit_cast(float, r.x & 0xFFFF0000u),
                       __builtin_bit_cast(float, r.y << 16), __builtin_bit_cast(float, r.y & 0xFFFF0000u));
  }
  return ((const float4 *)base)[i4];
}

template <bool BF16>
__global__ __launch_bounds__(256) void cache_store_kernel(const float4 *__restrict__ s, void *__restrict__ d, size_t n4) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n4; i += stride) {
    const float4 v = s[i];
    if (BF16) {
      uint2 r;
      r.x = (unsigned)bf16_bits(v.x) | ((unsigned)bf16_bits(v.y) << 16);
      r.y = (unsigned)bf16_bits(v.z) | ((unsigned)bf16_bits(v.w) << 16);
      ((uint2 *)d)[i] = r;
    } else {
      ((float4 *)d)[i] = v;
    }
  }
}

hipError_t launch_cache_store(const float *src, void *dst, size_t n, bool bf16, hipStream_t st) {
  size_t n4 = n / 4, blocks = (n4 + 255) / 256;
  if (blocks > 16384) blocks = 16384;
  if (blocks == 0) return hipSuccess;
  if (bf16) hipLaunchKernelGGL(cache_store_kernel<true>, dim3((unsigned)blocks), dim3(256), 0, st, (const float4 *)src, dst, n4);
  else hipLaunchKernelGGL(cache_store_kernel<false>, dim3((unsigned)blocks), dim3(256), 0, st, (const float4 *)src, dst, n4);
  return hipGetLastError();
}

// x[b, t, :] += gate[b, :] * cached[b, t, :]
template <bool BF16>
__global__ __launch_bounds__(256) void cache_reuse_kernel(void *__restrict__ x, int x_bf16, const void *__restrict__ cached,
                                                          const float *__restrict__ gate, int ld_gate, size_t n4, int TD4,
                                                          int D4) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const int b = (int)(i / TD4), n = (int)(i % D4) * 4;
  float4 xv = stream_load4(x, i, x_bf16);
  const float4 cv = load_cached4<BF16>(cached, i);
  float4 g = *(const float4 *)(gate + (size_t)b * ld_gate + n);
  xv.x = xv.x + g.x * cv.x;
  xv.y = xv.y + g.y * cv.y;
  xv.z = xv.z + g.z * cv.z;
  xv.w = xv.w + g.w * cv.w;
  stream_store4(x, i, xv, x_bf16);
}

hipError_t launch_cache_reuse(void *x, int x_bf16, const void *cached, const float *gate, int ld_gate, int B, int T, int D,
                              bool bf16, hipStream_t st) {
  const size_t n4 = (size_t)B * T * D / 4;
  const dim3 grid((unsigned)((n4 + 255) / 256));
  if (bf16) hipLaunchKernelGGL(cache_reuse_kernel<true>, grid, dim3(256), 0, st, x, x_bf16, cached, gate, ld_gate, n4, T * D / 4, D / 4);
  else hipLaunchKernelGGL(cache_reuse_kernel<false>, grid, dim3(256), 0, st, x, x_bf16, cached, gate, ld_gate, n4, T * D / 4, D / 4);
  return hipGetLastError();
}

// All blocks of a cached step in one pass over x: for every block in order,
// x += gate_msa * attn_cached; x += gate_mlp * mlp_cached (same association
// as block after block; a bfloat16 stream is rounded to its storage format after every addition, as it would be if
// it went through memory).  mod[l, b, 6D] holds the gates in chunks 2 and 5.  Cache strides are in elements.
__device__ __forceinline__ float as_stored(float v, int bf) { return bf ? bf16_value(bf16_bits(v)) : v; }

template <bool BF16>
__global__ __launch_bounds__(256) void cached_blocks_kernel(void *__restrict__ x, int x_bf16, const void *__restrict__ cache,
                                                            size_t cache_block_stride, size_t cache_which_stride,
                                                            const float *__restrict__ mod, size_t mod_block_stride,
                                                            int ld_mod, int L, size_t n4, int TD4, int D4, int D) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= n4) return;
  const int b = (int)(i / TD4), n = (int)(i % D4) * 4;
  constexpr size_t ES = BF16 ? 2 : 4;               // bytes per cached element
  const char *cbase = (const char *)cache;
  float4 xv = stream_load4(x, i, x_bf16);
  auto apply = [&](const float4 &g1, const float4 &a, const float4 &g2, const float4 &mo) {
    xv.x = as_stored(xv.x + g1.x * a.x, x_bf16); xv.y = as_stored(xv.y + g1.y * a.y, x_bf16);
    xv.z = as_stored(xv.z + g1.z * a.z, x_bf16); xv.w = as_stored(xv.w + g1.w * a.w, x_bf16);
    xv.x = as_stored(xv.x + g2.x * mo.x, x_bf16); xv.y = as_stored(xv.y + g2.y * mo.y, x_bf16);
    xv.z = as_stored(xv.z + g2.z * mo.z, x_bf16); xv.w = as_stored(xv.w + g2.w * mo.w, x_bf16);
  };
  // the loads of four blocks are in flight together; the additions keep the block order
  constexpr int U = 4;
  int l = 0;
  for (; l + U <= L; l += U) {
    float4 g1[U], g2[U], a[U], mo[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const float *mrow = mod + (size_t)(l + u) * mod_block_stride + (size_t)b * ld_mod + n;
      g1[u] = *(const float4 *)(mrow + 2 * D);
      g2[u] = *(const float4 *)(mrow + 5 * D);
      a[u] = load_cached4<BF16>(cbase + (size_t)(l + u) * cache_block_stride * ES, i);
      mo[u] = load_cached4<BF16>(cbase + ((size_t)(l + u) * cache_block_stride + cache_which_stride) * ES, i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) apply(g1[u], a[u], g2[u], mo[u]);
  }
  for (; l < L; ++l) {
    const float *mrow = mod + (size_t)l * mod_block_stride + (size_t)b * ld_mod + n;
    const float4 g1 = *(const float4 *)(mrow + 2 * D), g2 = *(const float4 *)(mrow + 5 * D);
    const float4 a = load_cached4<BF16>(cbase + (size_t)l * cache_block_stride * ES, i);
    const float4 mo = load_cached4<BF16>(cbase + ((size_t)l * cache_block_stride + cache_which_stride) * ES, i);
    apply(g1, a, g2, mo);
  }
  stream_store4(x, i, xv, x_bf16);
}

hipError_t launch_cached_blocks(void *x, int x_bf16, const void *cache, size_t cache_block_stride, size_t cache_which_stride,
                                const float *mod, size_t mod_block_stride, int ld_mod, int L, int B, int T, int D, bool bf16,
                                hipStream_t st) {
  const size_t n4 = (size_t)B * T * D / 4;
  const dim3 grid((unsigned)((n4 + 255) / 256));
  if (bf16)
    hipLaunchKernelGGL(cached_blocks_kernel<true>, grid, dim3(256), 0, st, x, x_bf16, cache, cache_block_stride, cache_which_stride, mod,
                       mod_block_stride, ld_mod, L, n4, T * D / 4, D / 4, D);
  else
    hipLaunchKernelGGL(cached_blocks_kernel<false>, grid, dim3(256), 0, st, x, x_bf16, cache, cache_block_stride, cache_which_stride, mod,
                       mod_block_stride, ld_mod, L, n4, T * D / 4, D / 4, D);
  return hipGetLastError();
}

// ------------------------------------------------- DDIM update + guidance + VC
__device__ __forceinline__ float block_sum_256(float v, float *red) {
  v = wave_sum(v);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  __syncthreads();
  if (lane == 0) red[w] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

// One workgroup per (latent, channel) plane.  xhat = cx*x + ce*eps is DDIM with
// eta = 0 (cx = sqrt(abar_prev/abar_t), ce = sqrt(1-abar_prev) - cx*sqrt(1-abar_t));
// then Eq. 10 with mu = plane mean: x~ = xhat + (K-1)(xhat - mu).  Both the updated sample and the corrected sample are
// stored float32 tensors; guidance + solver update, and VC, are each evaluated in float64 from the stored tensors they
// read and rounded once (the same values the separate DDIM, fit and VC launches of the factor fitting produce).
__device__ __forceinline__ double block_sum_256d(double v, double *red) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  __syncthreads();                       // red may still be read from the previous use
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void ddim_vc_kernel(float *__restrict__ x, const float *__restrict__ eps, int B, int C,
                                                      int HW, double cx, double ce, float cfg, const float *__restrict__ K_t) {
  __shared__ double red[4];
  const int plane = blockIdx.x, c = plane % C;
  float *xp = x + (size_t)plane * HW;
  const float *ec = eps + (size_t)plane * HW;
  const float *eu = eps + ((size_t)B * C + plane) * HW;
  const double w = (double)cfg;
  double sum = 0.0;
  for (int i = threadIdx.x; i < HW; i += 256) {
    double e = (double)ec[i];
    if (cfg > 0.0f) {
      const double u = (double)eu[i];
      e = u + w * (e - u);
    }
    const float xh = (float)(cx * (double)xp[i] + ce * e);
    xp[i] = xh;
    sum += (double)xh;
  }
  if (!K_t) return;
  const double mu = block_sum_256d(sum, red) / (double)HW;
  const double km1 = (double)K_t[c] - 1.0;
  for (int i = threadIdx.x; i < HW; i += 256) {          // a thread re-reads only what it wrote itself
    const double xh = (double)xp[i];
    xp[i] = (float)(xh + km1 * (xh - mu));
  }
}

hipError_t launch_ddim_vc(float *x, const float *eps, int B, int C, int HW, double cx, double ce, float cfg_scale,
                          const float *K_t, hipStream_t st) {
  hipLaunchKernelGGL(ddim_vc_kernel, dim3(B * C), dim3(256), 0, st, x, eps, B, C, HW, cx, ce, cfg_scale, K_t);
  return hipGetLastError();
}

__global__ __launch_bounds__(256) void vc_kernel(float *__restrict__ x, const float *__restrict__ K_t,
                                                 const float *__restrict__ mu_in, int C, int HW) {
  __shared__ double red[4];
  const int plane = blockIdx.x, c = plane % C;
  float *xp = x + (size_t)plane * HW;
  double mu;
  if (mu_in) {
    mu = (double)mu_in[c];
  } else {
    double sum = 0.0;
    for (int i = threadIdx.x; i < HW; i += 256) sum += (double)xp[i];
    mu = block_sum_256d(sum, red) / (double)HW;
  }
  const double km1 = (double)K_t[c] - 1.0;
  for (int i = threadIdx.x; i < HW; i += 256) {
    const double v = (double)xp[i];
    xp[i] = (float)(v + km1 * (v - mu));
  }
}

hipError_t launch_vc(float *x, const float *K_t, const float *mu, int B, int C, int HW, hipStream_t st) {
  hipLaunchKernelGGL(vc_kernel, dim3(B * C), dim3(256), 0, st, x, K_t, mu, C, HW);
  return hipGetLastError();
}

// ------------------------------------------------------------------ VC fit
// Factors of one timestep: the exact minimiser, channel by channel, of
//   sum ((x~ - x') / x')^2 + sum (x~ - x')^2,   x~ = mu + K (x^ - mu)     (objective after Eq. 10)
// over the elements of the channel in the whole batch: K = S1 / S2 with S1 = sum d (x' - mu) w,
// S2 = sum d^2 w, d = x^ - mu, w = 1 + 1 / (x'^2 + eps), mu = spatial mean of the x^ plane.
// One workgroup per (sample, channel) plane writes its two partial sums (fp64); a second, tiny kernel adds the
// planes of a channel in a fixed order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void vc_fit_sums_kernel(const float *__restrict__ x_hat, const float *__restrict__ x_ref,
                                                          int HW, double eps, double *__restrict__ part) {
  __shared__ double red[4];
  const int plane = blockIdx.x;
  const float *xh = x_hat + (size_t)plane * HW, *xr = x_ref + (size_t)plane * HW;
  double sum = 0.0;
  for (int i = threadIdx.x; i < HW; i += 256) sum += (double)xh[i];
  const double mu = block_sum_256d(sum, red) / (double)HW;
  double s1 = 0.0, s2 = 0.0;
  for (int i = threadIdx.x; i < HW; i += 256) {
    const double d = (double)xh[i] - mu, r = (double)xr[i];
    const double w = 1.0 + 1.0 / (r * r + eps);
    s1 += d * (r - mu) * w;
    s2 += d * d * w;
  }
  s1 = block_sum_256d(s1, red);
  s2 = block_sum_256d(s2, red);
  if (threadIdx.x == 0) {
    part[2 * plane] = s1;
    part[2 * plane + 1] = s2;
  }
}

__global__ void vc_fit_solve_kernel(const double *__restrict__ part, int B, int C, float *__restrict__ K_t) {
  const int c = blockIdx.x * blockDim.x + threadIdx.x;
  if (c >= C) return;
  double s1 = 0.0, s2 = 0.0;
  for (int b = 0; b < B; ++b) {
    s1 += part[2 * ((size_t)b * C + c)];
    s2 += part[2 * ((size_t)b * C + c) + 1];
  }
  K_t[c] = s2 > 0.0 ? (float)(s1 / s2) : 1.0f;
}

hipError_t launch_vc_fit(const float *x_hat, const float *x_ref, int B, int C, int HW, float eps, double *work, float *K_t,
                         hipStream_t st) {
  hipLaunchKernelGGL(vc_fit_sums_kernel, dim3(B * C), dim3(256), 0, st, x_hat, x_ref, HW, (double)eps, work);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(vc_fit_solve_kernel, dim3((C + 63) / 64), dim3(64), 0, st, work, B, C, K_t);
  return hipGetLastError();
}

// ------------------------------------------------------ calibration helpers
// Plain fp32 tiled linear y = act(x W^T + b): 64x64 tile, 16-deep slabs, 4x4 per thread.
__global__ __launch_bounds__(256) void linear_f32_kernel(const float *__restrict__ x, const float *__restrict__ W,
                                                         const float *__restrict__ bias, float *__restrict__ y, int M, int N,
                                                         int K, int act_out) {
  __shared__ float sx[16][65], sw[16][65];
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const int tx = threadIdx.x % 16, ty = threadIdx.x / 16;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += 16) {
    for (int i = threadIdx.x; i < 64 * 16; i += 256) {
      const int r = i / 16, k = i % 16;
      sx[k][r] = (m0 + r < M && k0 + k < K) ? x[(size_t)(m0 + r) * K + k0 + k] : 0.0f;
      sw[k][r] = (n0 + r < N && k0 + k < K) ? W[(size_t)(n0 + r) * K + k0 + k] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = sx[k][ty * 4 + i], b[i] = sw[k][tx * 4 + i];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
  for (int i = 0; i < 4; ++i)
    for (int j = 0; j < 4; ++j) {
      const int m = m0 + ty * 4 + i, n = n0 + tx * 4 + j;
      if (m < M && n < N) {
        float v = acc[i][j] + (bias ? bias[n] : 0.0f);
        if (act_out == 2) v = gelu_f(v);
        y[(size_t)m * N + n] = v;
      }
    }
}

hipError_t launch_linear_f32(const float *x, const float *W, const float *b, float *y, int M, int N, int K, int act_out,
                             hipStream_t st) {
  hipLaunchKernelGGL(linear_f32_kernel, dim3((N + 63) / 64, (M + 63) / 64), dim3(256), 0, st, x, W, b, y, M, N, K, act_out);
  return hipGetLastError();
}

// Running min / max of a tensor kept as order-preserving integers:
// slot[0] = min, slot[1] = max; act = 1 takes SiLU of the values first.
__device__ __forceinline__ int f2ord(float f) {
  int i = __float_as_int(f);
  return i ^ ((i >> 31) & 0x7FFFFFFF);
}
__global__ __launch_bounds__(256) void minmax_kernel(const float *__restrict__ x, size_t n, int act, int *slot) {
  float lo = INFINITY, hi = -INFINITY;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    float v = x[i];
    if (act == 1) v = silu_f(v);
    lo = fminf(lo, v);
    hi = fmaxf(hi, v);
  }
  hi = wave_max(hi);
  lo = -wave_max(-lo);
  if ((threadIdx.x & 63) == 0 && lo <= hi) {
    atomicMin(slot, f2ord(lo));
    atomicMax(slot + 1, f2ord(hi));
  }
}

hipError_t launch_minmax(const float *x, size_t n, int *slot, hipStream_t st) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(minmax_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, n, 0, slot);
  return hipGetLastError();
}
hipError_t launch_minmax_silu(const float *x, size_t n, int *slot, hipStream_t st) {
  size_t blocks = (n + 255) / 256;
  if (blocks > 1024) blocks = 1024;
  if (blocks == 0) return hipSuccess;
  hipLaunchKernelGGL(minmax_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, n, 1, slot);
  return hipGetLastError();
}

__global__ void fill_i32_kernel(int *p, size_t n, int v) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
hipError_t launch_fill_i32(int *p, size_t n, int v, hipStream_t st) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
  return hipGetLastError();
}

}  // namespace qc
