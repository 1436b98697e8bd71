// softmax(Q K^T / sqrt(d)) V per (batch, head) in fp32 on the matrix cores
// (v_mfma_f32_16x16x4_f32), keys streamed through LDS in tiles of 64 with an
// online softmax, so no T x T matrix ever exists.  The output is quantised with
// the attention-projection site's (s, z) on the way out (Eq. 1), or written as
// fp32 for calibration.
//
// Work split: one workgroup = 64 queries of one (batch, head); each of its four
// wavefronts owns 16 queries.  The products are formed transposed so that a
// lane always owns ONE query:
//   S^T = K Q^T : A operand = K rows (keys), B operand = Q^T (queries)
//   O^T = V^T P^T : A operand = V^T rows (features), B operand = P^T
// MFMA 16x16x4 layouts: lane l supplies A[row l%16][k l/16] and B[k l/16][col l%16];
// result register r of lane l is row 4*(l/16)+r, column l%16.  Hence the S^T
// result of lane (q = l%16, g = l/16) holds keys 4g..4g+3 of query q, which is
// exactly the B operand P^T[key][q] needs if the k index of the second product
// enumerates keys as 4g + r; the V^T operand is read with the same enumeration.
// The running max / sum of a query are per-lane scalars, shared across the four
// g groups with two shuffles.
#include "qc_internal.h"

namespace qc {

typedef float v4f __attribute__((ext_vector_type(4)));

template <int DP>   // head dim padded to a multiple of 16
__global__ __launch_bounds__(256) void attention_kernel(const float *__restrict__ qkv, int T, int H, int hd,
                                                        const QParam *qp, int8_t *__restrict__ q_out,
                                                        float *__restrict__ f32_out, float scale_log2e) {
  constexpr int S = DP + 4;          // LDS row stride in floats: 8 consecutive rows hit 8 distinct 16-byte bank groups
  constexpr int NC = DP / 16;        // 16-wide feature chunks
  __shared__ __align__(16) float Ks[64 * S];
  __shared__ __align__(16) float Vs[64 * S];

  const int D = H * hd;
  const int bh = blockIdx.y, b = bh / H, h = bh % H;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int ql = lane & 15, g = lane >> 4;
  const int q_row = blockIdx.x * 64 + wave * 16 + ql;            // query of this lane
  const float *base = qkv + (size_t)b * T * 3 * D + (size_t)h * hd;

  // Q^T operand: features 16c + 4g + u of this lane's query, pre-scaled by log2(e)/sqrt(d)
  v4f qf[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int e = 16 * c + 4 * g;
    v4f v = {0.f, 0.f, 0.f, 0.f};
    if (q_row < T && e < hd) v = *(const v4f *)(base + (size_t)q_row * 3 * D + e);
    qf[c] = v * scale_log2e;
  }

  v4f o[NC];
#pragma unroll
  for (int c = 0; c < NC; ++c) o[c] = (v4f){0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.0f;

  for (int k0 = 0; k0 < T; k0 += 64) {
    __syncthreads();
    // stage K and V tiles (zero padded in features and keys)
    for (int i = tid; i < 64 * (DP / 4); i += 256) {
      const int r = i / (DP / 4), e = (i % (DP / 4)) * 4;
      v4f kv = {0.f, 0.f, 0.f, 0.f}, vv = {0.f, 0.f, 0.f, 0.f};
      if (k0 + r < T && e < hd) {
        const float *src = base + (size_t)(k0 + r) * 3 * D + e;
        kv = *(const v4f *)(src + D);
        vv = *(const v4f *)(src + 2 * D);
      }
      *(v4f *)(Ks + r * S + e) = kv;
      *(v4f *)(Vs + r * S + e) = vv;
    }
    __syncthreads();

    // S^T tile: 4 blocks of 16 keys
    v4f s[4];
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      v4f acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int c = 0; c < NC; ++c) {
        const v4f kf = *(const v4f *)(Ks + (kt * 16 + ql) * S + 16 * c + 4 * g);
#pragma unroll
        for (int u = 0; u < 4; ++u) acc = __builtin_amdgcn_mfma_f32_16x16x4f32(kf[u], qf[c][u], acc, 0, 0, 0);
      }
      s[kt] = acc;
    }
    // mask keys past the end, running max
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        if (k0 + kt * 16 + 4 * g + r >= T) s[kt][r] = -INFINITY;
        mx = fmaxf(mx, s[kt][r]);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);           // finite: every tile holds at least one valid key
    const float alpha = exp2f(m_run - m_new);
    m_run = m_new;
    l_run *= alpha;
#pragma unroll
    for (int c = 0; c < NC; ++c) o[c] *= alpha;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float pv = exp2f(s[kt][r] - m_new);
        s[kt][r] = pv;
        l_run += pv;
      }
    // O^T += V^T P^T
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float *vrow = Vs + (kt * 16 + 4 * g + r) * S + ql;
#pragma unroll
        for (int c = 0; c < NC; ++c) o[c] = __builtin_amdgcn_mfma_f32_16x16x4f32(vrow[16 * c], s[kt][r], o[c], 0, 0, 0);
      }
  }

  l_run += __shfl_xor(l_run, 16, 64);
  l_run += __shfl_xor(l_run, 32, 64);
  if (q_row >= T) return;
  const float inv = 1.0f / l_run;
  float qs = 1.0f;
  int qz = 0;
  if (qp) {
    QParam t = *qp;
    qs = t.s;
    qz = t.z;
  }
  const size_t out_row = ((size_t)b * T + q_row) * D + (size_t)h * hd;
#pragma unroll
  for (int c = 0; c < NC; ++c) {
    const int e = 16 * c + 4 * g;
    if (e >= hd) continue;
    const v4f v = o[c] * inv;
    if (q_out) {
      int c0, c1, c2, c3;
      float r;
      r = rintf(v[0] / qs) + (float)qz; c0 = (int)fminf(fmaxf(r, -128.f), 127.f);
      r = rintf(v[1] / qs) + (float)qz; c1 = (int)fminf(fmaxf(r, -128.f), 127.f);
      r = rintf(v[2] / qs) + (float)qz; c2 = (int)fminf(fmaxf(r, -128.f), 127.f);
      r = rintf(v[3] / qs) + (float)qz; c3 = (int)fminf(fmaxf(r, -128.f), 127.f);
      *(unsigned *)(q_out + out_row + e) = (unsigned)(c0 & 0xFF) | ((unsigned)(c1 & 0xFF) << 8) |
                                           ((unsigned)(c2 & 0xFF) << 16) | ((unsigned)(c3 & 0xFF) << 24);
    }
    if (f32_out) *(v4f *)(f32_out + out_row + e) = v;
  }
}

hipError_t launch_attention(const float *qkv, int B, int T, int H, int hd, const QParam *qp, int8_t *q_out, float *f32_out,
                            hipStream_t st) {
  const float sl2 = 1.4426950408889634f / sqrtf((float)hd);
  dim3 grid((T + 63) / 64, B * H);
  const int dp = (hd + 15) / 16 * 16;
  switch (dp) {
    case 16: hipLaunchKernelGGL(attention_kernel<16>, grid, dim3(256), 0, st, qkv, T, H, hd, qp, q_out, f32_out, sl2); break;
    case 32: hipLaunchKernelGGL(attention_kernel<32>, grid, dim3(256), 0, st, qkv, T, H, hd, qp, q_out, f32_out, sl2); break;
    case 48: hipLaunchKernelGGL(attention_kernel<48>, grid, dim3(256), 0, st, qkv, T, H, hd, qp, q_out, f32_out, sl2); break;
    case 64: hipLaunchKernelGGL(attention_kernel<64>, grid, dim3(256), 0, st, qkv, T, H, hd, qp, q_out, f32_out, sl2); break;
    case 80: hipLaunchKernelGGL(attention_kernel<80>, grid, dim3(256), 0, st, qkv, T, H, hd, qp, q_out, f32_out, sl2); break;
    case 96: hipLaunchKernelGGL(attention_kernel<96>, grid, dim3(256), 0, st, qkv, T, H, hd, qp, q_out, f32_out, sl2); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace qc
