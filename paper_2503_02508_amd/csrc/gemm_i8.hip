// int8 x int8 -> int32 GEMM on the gfx950 matrix cores (v_mfma_i32_32x32x32_i8)
// with the dequantise / GELU+requantise / cache-store+gated-residual epilogues
// of the quantised linears of a DiT block.
//
//   acc[m, n] = sum_k A[m, k] * W[n, k]          A: activation codes, W: weight codes
//   v[m, n]   = a_s * w_s[n] * (acc - a_z * wsum[n]) + bias[n]
//
// Tiling: a 256-thread workgroup (4 wavefronts) owns a BM x BN tile of the
// output and walks K in slabs of 128 bytes.  Both operands are K-contiguous, so
// a slab row is 8 sixteen-byte chunks; slabs are staged in LDS (rows padded by
// 16 bytes so the 128-bit fragment reads of 8 neighbouring rows fall in 8
// different bank groups) and double buffered: the global loads of slab k+1 are
// in flight while slab k feeds the MFMAs.  Each wavefront holds a (BM/WM) x
// (BN/WN) sub-tile as 32x32 int32 accumulator blocks.
//
// MFMA operand layout (32x32x32 i8): lane l supplies 16 bytes of row (l % 32)
// of either operand for k-group (l / 32); the products pair byte j of group g
// of A with byte j of group g of W, so any k order works as long as both
// operands use the same one.  Result layout: register r of lane l is
// row (r/4)*8 + (l/32)*4 + r%4, column l % 32.
#include "qc_internal.h"

namespace qc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int BK = 128;
constexpr int LDS_ROW = BK + 16;

__device__ __forceinline__ int map_col(int j, int sel_D) {
  return sel_D ? (j < sel_D ? j + 2 * sel_D : j + 4 * sel_D) : j;
}

// 8 packed bytes (16 nibbles, element 2j low, 2j+1 high) -> 16 int8 codes.
__device__ __forceinline__ v4i unpack_w4(v2i p) {
  v4i o;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    unsigned w = (unsigned)(h ? p.y : p.x);
    unsigned lo = w & 0x0F0F0F0Fu;
    unsigned hi = (w >> 4) & 0x0F0F0F0Fu;
    lo |= (lo & 0x08080808u) * 0x1Eu;   // sign-extend each nibble inside its byte
    hi |= (hi & 0x08080808u) * 0x1Eu;
    unsigned e0 = __builtin_amdgcn_perm(hi, lo, 0x05010400u);   // l0 h0 l1 h1
    unsigned e1 = __builtin_amdgcn_perm(hi, lo, 0x07030602u);   // l2 h2 l3 h3
    if (h == 0) { o.x = (int)e0; o.y = (int)e1; } else { o.z = (int)e0; o.w = (int)e1; }
  }
  return o;
}

__device__ __forceinline__ float gelu_tanh(float v) {
  const float k0 = 0.7978845608028654f, k1 = 0.044715f;
  float u = k0 * (v + k1 * v * v * v);
  return 0.5f * v * (1.0f + tanhf(u));
}

__device__ __forceinline__ int quant_code(float v, float s, int z_signed) {
  float r = rintf(v / s) + (float)z_signed;
  r = fminf(fmaxf(r, -128.0f), 127.0f);
  return (int)r;
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(256) void gemm_i8_kernel(GemmArgs p) {
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int PA = BM / 32, PB = BN / 32;   // 16-byte chunks per thread per slab
  static_assert(WM * WN == 4 && TM >= 1 && TN >= 1, "four wavefronts per workgroup");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char *sA = smem;
  unsigned char *sB = smem + 2 * BM * LDS_ROW;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int z = blockIdx.z;
  const int ncover = p.sel_D ? 2 * p.sel_D : p.N;
  const int tiles_m = (p.M + BM - 1) / BM;
  const int m0 = (blockIdx.x % tiles_m) * BM;
  const int n0 = (blockIdx.x / tiles_m) * BN;
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  const int8_t *A = p.A + (long long)z * p.zs_A;
  const unsigned char *W = (const unsigned char *)p.W + (long long)z * p.zs_W;   // byte stride
  const long long w_row_bytes = p.w4 ? (p.K >> 1) : p.K;

  const int lr = tid >> 3, lc = tid & 7;   // slab row (per pass of 32) and chunk of this thread
  v4i ra[PA], rb[PB];

  auto load_slab = [&](int k0) {
    const int k = k0 + lc * 16;
    const bool kin = k < p.K;
#pragma unroll
    for (int i = 0; i < PA; ++i) {
      const int m = m0 + lr + 32 * i;
      v4i v = {0, 0, 0, 0};
      if (kin && m < p.M) v = *(const v4i *)(A + (long long)m * p.lda + k);
      ra[i] = v;
    }
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      const int j = n0 + lr + 32 * i;
      v4i v = {0, 0, 0, 0};
      if (kin && j < ncover) {
        const unsigned char *row = W + (long long)map_col(j, p.sel_D) * w_row_bytes;
        if (p.w4) v = unpack_w4(*(const v2i *)(row + (k >> 1)));
        else v = *(const v4i *)(row + k);
      }
      rb[i] = v;
    }
  };
  auto store_slab = [&](int buf) {
#pragma unroll
    for (int i = 0; i < PA; ++i)
      *(v4i *)(sA + (buf * BM + lr + 32 * i) * LDS_ROW + lc * 16) = ra[i];
#pragma unroll
    for (int i = 0; i < PB; ++i)
      *(v4i *)(sB + (buf * BN + lr + 32 * i) * LDS_ROW + lc * 16) = rb[i];
  };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int nk = (p.K + BK - 1) / BK;
  load_slab(0);
  store_slab(0);
  __syncthreads();
  const int frow = lane & 31, fk = (lane >> 5) * 16;
  for (int kt = 0; kt < nk; ++kt) {
    const int cur = kt & 1;
    if (kt + 1 < nk) load_slab((kt + 1) * BK);
    const unsigned char *a_base = sA + (cur * BM + wm0 + frow) * LDS_ROW + fk;
    const unsigned char *b_base = sB + (cur * BN + wn0 + frow) * LDS_ROW + fk;
#pragma unroll
    for (int kk = 0; kk < BK / 32; ++kk) {
      v4i fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *(const v4i *)(a_base + i * 32 * LDS_ROW + kk * 32);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = *(const v4i *)(b_base + j * 32 * LDS_ROW + kk * 32);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) store_slab(cur ^ 1);
    __syncthreads();
  }

  // ------------------------------------------------------------ epilogue
  float a_s = p.a_scale;
  int a_z = p.a_zp;
  if (p.a_qp) {
    QParam q = p.a_qp[(long long)z * p.zs_qp];
    a_s = q.s;
    a_z = q.z;
  }
  float o_s = 1.0f;
  int o_z = 0;
  if (EPI == EPI_GELU_Q) {
    QParam q = *p.o_qp;
    o_s = q.s;
    o_z = q.z;
  }
  const float *w_scale = p.w_scale + (long long)z * p.zs_vecN;
  const int32_t *wsum = p.wsum + (long long)z * p.zs_vecN;
  const float *bias = p.bias ? p.bias + (long long)z * p.zs_vecN : nullptr;
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int jl = n0 + wn0 + j * 32 + (lane & 31);
    if (jl >= ncover) continue;
    const int n = map_col(jl, p.sel_D);
    const float sc = a_s * w_scale[n];
    const int zw = a_z * wsum[n];
    const float bs = bias ? bias[n] : 0.0f;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (m >= p.M) continue;
        const int a = acc[i][j][r];
        const float v = fmaf(sc, (float)(a - zw), bs);
        if (EPI == EPI_F32) {
          float *y = p.y + (long long)z * p.zs_out;
          y[(long long)m * p.ldy + n] = v;
          if (p.acc_out) p.acc_out[(long long)m * p.N + n] = a;
        } else if (EPI == EPI_GELU_Q) {
          p.q_out[(long long)m * p.ldq + n] = (int8_t)quant_code(gelu_tanh(v), o_s, o_z);
        } else {
          const long long o = (long long)m * p.N + n;
          p.cache_out[o] = v;
          const float g = p.gate[(long long)(m / p.rows_per_batch) * p.ld_gate + n];
          p.x[o] = p.x[o] + g * v;
        }
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, int EPI>
static hipError_t launch_cfg(const GemmArgs &a, int nz, hipStream_t st) {
  constexpr int smem = 2 * (BM + BN) * LDS_ROW;
  static bool attr_set = false;
  auto kern = gemm_i8_kernel<BM, BN, WM, WN, EPI>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int ncover = a.sel_D ? 2 * a.sel_D : a.N;
  const int tiles = ((a.M + BM - 1) / BM) * ((ncover + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles, 1, nz), dim3(256), smem, st, a);
  return hipGetLastError();
}

template <int EPI>
static hipError_t launch_epi(const GemmArgs &a, int nz, hipStream_t st) {
  if (a.M <= 32) return launch_cfg<32, 128, 1, 4, EPI>(a, nz, st);
  if (a.M <= 64) return launch_cfg<64, 128, 2, 2, EPI>(a, nz, st);
  return launch_cfg<128, 128, 2, 2, EPI>(a, nz, st);
}

hipError_t launch_gemm(const GemmArgs &a, int epi, int nz, hipStream_t st) {
  switch (epi) {
    case EPI_F32: return launch_epi<EPI_F32>(a, nz, st);
    case EPI_GELU_Q: return launch_epi<EPI_GELU_Q>(a, nz, st);
    default: return launch_epi<EPI_RESID>(a, nz, st);
  }
}

}  // namespace qc
