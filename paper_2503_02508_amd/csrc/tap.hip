// Calibration-set clustering (temporal-aware parallel clustering, TAP; the paper's section of that name and its
// algorithm): similarity matrices on the fp32 matrix cores, degree normalisation, leading singular vectors by block
// power iteration with Cholesky QR and a Jacobi Rayleigh-Ritz step, k-means, aggregation over subsamples.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <math.h>
#include <utility>
#include <vector>
#include "qc_tap.h"
#include "qc_internal.h"

namespace {

#define TAP_FAIL(code, ...)     \
  do {                          \
    qc::set_error(__VA_ARGS__); \
    return (code);              \
  } while (0)

#define TAP_HIP(expr)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) TAP_FAIL(QC_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_));     \
  } while (0)

#define TAP_RC(expr)       \
  do {                     \
    int rc_ = (expr);      \
    if (rc_) return rc_;   \
  } while (0)

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int NUM_XCD = 8;
constexpr int KB_MAX = 128;
constexpr int M_MAX = 8;

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ------------------------------------------------------------------------------------------------ fp32 GEMM
// C[m, n] = sum_k A(m, k) B(n, k) with A(m, k) = A[m * sam + k * sak], B(n, k) = B[n * sbn + k * sbk]; each operand
// is contiguous either along k (KC) or along its own index.  128 x 128 tile per workgroup of four wavefronts (2 x 2,
// each 64 x 64 = 2 x 2 blocks of v_mfma_f32_32x32x2_f32), K walked in slabs of 32 staged through LDS k-major, so that
// an operand fetch is 32 consecutive floats per half wavefront.  The next slab's global loads are in flight while the
// current one is multiplied.
constexpr int TM = 128, TN = 128, TK = 32;
// LDS row stride (floats) of a k-major tile.  An operand contiguous along k is transposed on the way in: lane l
// writes element (k = 4 (l % 8) + i, o = l / 8); 4 * 130 = 8 (mod 64) spreads the 64 lanes over 64 banks.  An operand
// contiguous along its own index is stored with 16-byte writes and needs a stride that is a multiple of 4.
template <bool KC>
constexpr int ldt() { return KC ? 130 : 132; }

enum SgemmEpi { SE_PLAIN = 0, SE_SIM = 1, SE_COLSCALE = 2 };

struct SgemmArgs {
  const float *A, *B;
  float *C;
  long long sam, sak, sbn, sbk, ldc;
  int M, N, K;
  int a_kc, b_kc;     // operand contiguous along k (else along its own index)
  int a_vec, b_vec;   // 16-byte loads are safe (alignment and extents are multiples of 4)
  // SE_SIM: C = alpha * acc * rs[m] * cs[n] + (1 - alpha) * exp(-|tr[m] - tc[n]|);  SE_COLSCALE: C = acc * cs[n]
  const float *rs, *cs, *tr, *tc;
  float alpha;
  // split K (SE_PLAIN only): workgroup (tile, blockIdx.y = s) multiplies k in [s * kchunk, (s + 1) * kchunk) and writes
  // its partial product to C + s * part_stride; a second kernel adds the partial products in order
  int kchunk;
  long long part_stride;
  // symmetric product (SE_PLAIN, B = A with the same strides, M = N): only the tiles on and below the diagonal are
  // computed; the kernel that adds the partial products also writes the mirror image
  int sym;
};

// One operand's share of a slab for this thread: four units of four consecutive elements.
//  KC: unit u -> (o = u / 8, k4 = (u % 8) * 4), elements along k
//  else: unit u -> (k = u / 32, o4 = (u % 32) * 4), elements along o
// Out-of-range elements are loaded from a clamped (valid) address and zeroed only when the slab is written to LDS
// (bit 4 p + i of the returned mask = element i of unit p is in range): nothing touches a loaded register before
// that, so all loads of a slab stay in flight together while the previous slab is multiplied.
template <bool KC, bool vec>
__device__ __forceinline__ unsigned load_units(const float *P, long long so, long long sk, int o0, int O, int k0, int K,
                                               int tid, float4 (&r)[4]) {
  unsigned mask = 0;
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int u = tid + 256 * p;
    if (KC) {
      const int o = o0 + (u >> 3), k = k0 + ((u & 7) << 2);
      if (vec) {
        const bool ok = o < O && k < K;
        r[p] = *reinterpret_cast<const float4 *>(P + (ok ? (long long)o * so + k : 0));
        mask |= ok ? 0xFu << (4 * p) : 0u;
      } else {
        float e[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool ok = o < O && k + i < K;
          e[i] = P[ok ? (long long)o * so + (long long)(k + i) * sk : 0];
          mask |= ok ? 1u << (4 * p + i) : 0u;
        }
        r[p] = make_float4(e[0], e[1], e[2], e[3]);
      }
    } else {
      const int k = k0 + (u >> 5), o = o0 + ((u & 31) << 2);
      if (vec) {
        const bool ok = o < O && k < K;
        r[p] = *reinterpret_cast<const float4 *>(P + (ok ? (long long)k * sk + o : 0));
        mask |= ok ? 0xFu << (4 * p) : 0u;
      } else {
        // element loads: lane l takes o = l % 32 + 32 i, so that every load covers 32 consecutive floats
        const int ob = o0 + (u & 31);
        float e[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const bool ok = ob + 32 * i < O && k < K;
          e[i] = P[ok ? (long long)k * sk + (long long)(ob + 32 * i) * so : 0];
          mask |= ok ? 1u << (4 * p + i) : 0u;
        }
        r[p] = make_float4(e[0], e[1], e[2], e[3]);
      }
    }
  }
  return mask;
}

template <bool KC, bool vec>
__device__ __forceinline__ void store_units(float *T, int tid, unsigned mask, const float4 (&r)[4]) {
  constexpr int LDT = ldt<KC>();
#pragma unroll
  for (int p = 0; p < 4; ++p) {
    const int u = tid + 256 * p;
    const float x = (mask >> (4 * p)) & 1u ? r[p].x : 0.f, y = (mask >> (4 * p + 1)) & 1u ? r[p].y : 0.f;
    const float z = (mask >> (4 * p + 2)) & 1u ? r[p].z : 0.f, w = (mask >> (4 * p + 3)) & 1u ? r[p].w : 0.f;
    if (KC) {
      const int o = u >> 3, k = (u & 7) << 2;
      T[(k + 0) * LDT + o] = x;
      T[(k + 1) * LDT + o] = y;
      T[(k + 2) * LDT + o] = z;
      T[(k + 3) * LDT + o] = w;
    } else {
      const int k = u >> 5;
      if (vec) {
        *reinterpret_cast<float4 *>(T + k * LDT + ((u & 31) << 2)) = make_float4(x, y, z, w);
      } else {
        float *d = T + k * LDT + (u & 31);
        d[0] = x;
        d[32] = y;
        d[64] = z;
        d[96] = w;
      }
    }
  }
}

// entry t of the lower triangle walked row by row -> (row, column), column <= row
__device__ __forceinline__ void tri_decode(int t, int &row, int &col) {
  int r = (int)((sqrtf(8.f * (float)t + 1.f) - 1.f) * 0.5f);
  while (r * (r + 1) / 2 > t) --r;
  while ((r + 1) * (r + 2) / 2 <= t) ++r;
  row = r;
  col = t - r * (r + 1) / 2;
}

// VEC: both operands take 16-byte loads (a compile-time choice: a run-time branch around the loads would make the
// compiler wait for them at the join and expose their latency)
template <bool AKC, bool BKC, int EPI, bool VEC>
__global__ __launch_bounds__(256, 2) void sgemm_kernel(SgemmArgs p) {
  constexpr int LDA = ldt<AKC>(), LDB = ldt<BKC>();
  __shared__ __align__(16) float As[2][TK * LDA];
  __shared__ __align__(16) float Bs[2][TK * LDB];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int tiles_m = (p.M + TM - 1) / TM, tiles_n = (p.N + TN - 1) / TN;
  const int total = p.sym ? tiles_m * (tiles_m + 1) / 2 : tiles_m * tiles_n;
  // workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous run of tiles (n fastest) so that the
  // tiles sharing an A panel meet in one L2
  const int per_xcd = (total + NUM_XCD - 1) / NUM_XCD;
  const int tile = (blockIdx.x % NUM_XCD) * per_xcd + blockIdx.x / NUM_XCD;
  if (blockIdx.x / NUM_XCD >= per_xcd || tile >= total) return;
  int tm, tn;
  if (p.sym) {
    tri_decode(tile, tm, tn);
  } else {
    tm = tile / tiles_n;
    tn = tile % tiles_n;
  }
  const int m0 = tm * TM, n0 = tn * TN;
  const int wm0 = (wave >> 1) * 64, wn0 = (wave & 1) * 64;

  floatx16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // Two LDS buffers: while slab s is multiplied from one, slab s + 1 (already in registers) is written to the other
  // and slab s + 2 is requested from memory; one barrier per slab.  A buffer is overwritten two slabs after it was
  // read, and the barrier in between is passed only by wavefronts that have finished reading it.
  float4 ra[4], rb[4];
  const int kbeg = blockIdx.y * p.kchunk, kend = min(p.K, kbeg + p.kchunk);
  const int nslab = (kend - kbeg + TK - 1) / TK;
  if (EPI == SE_PLAIN) p.C += (long long)blockIdx.y * p.part_stride;
  unsigned ma = load_units<AKC, VEC>(p.A, p.sam, p.sak, m0, p.M, kbeg, kend, tid, ra);
  unsigned mb = load_units<BKC, VEC>(p.B, p.sbn, p.sbk, n0, p.N, kbeg, kend, tid, rb);
  store_units<AKC, VEC>(As[0], tid, ma, ra);
  store_units<BKC, VEC>(Bs[0], tid, mb, rb);
  ma = load_units<AKC, VEC>(p.A, p.sam, p.sak, m0, p.M, kbeg + TK, kend, tid, ra);
  mb = load_units<BKC, VEC>(p.B, p.sbn, p.sbk, n0, p.N, kbeg + TK, kend, tid, rb);
  __syncthreads();
  for (int s = 0; s < nslab; ++s) {
    const int cur = s & 1;
    if (s + 1 < nslab) {
      store_units<AKC, VEC>(As[cur ^ 1], tid, ma, ra);
      store_units<BKC, VEC>(Bs[cur ^ 1], tid, mb, rb);
    }
    if (s + 2 < nslab) {
      ma = load_units<AKC, VEC>(p.A, p.sam, p.sak, m0, p.M, kbeg + (s + 2) * TK, kend, tid, ra);
      mb = load_units<BKC, VEC>(p.B, p.sbn, p.sbk, n0, p.N, kbeg + (s + 2) * TK, kend, tid, rb);
    }
    const float *ap = As[cur] + (lane >> 5) * LDA + wm0 + (lane & 31);
    const float *bp = Bs[cur] + (lane >> 5) * LDB + wn0 + (lane & 31);
    // the fragments of step kk + 1 are read from LDS before the four products of step kk are issued (the
    // scheduling barriers pin that order), so an LDS round trip hides behind 256 cycles of matrix-core work
    float a0 = ap[0], a1 = ap[32], b0 = bp[0], b1 = bp[32];
    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
    for (int kk = 0; kk < TK / 2; ++kk) {
      float na0 = 0.f, na1 = 0.f, nb0 = 0.f, nb1 = 0.f;
      if (kk + 1 < TK / 2) {
        na0 = ap[(kk + 1) * 2 * LDA];
        na1 = ap[(kk + 1) * 2 * LDA + 32];
        nb0 = bp[(kk + 1) * 2 * LDB];
        nb1 = bp[(kk + 1) * 2 * LDB + 32];
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);      // the LDS reads (two paired loads)
      }
      acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b0, acc[0][0], 0, 0, 0);
      acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a0, b1, acc[0][1], 0, 0, 0);
      acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b0, acc[1][0], 0, 0, 0);
      acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x2f32(a1, b1, acc[1][1], 0, 0, 0);
      __builtin_amdgcn_sched_group_barrier(0x008, 4, 0);        // then the four matrix instructions
      a0 = na0;
      a1 = na1;
      b0 = nb0;
      b1 = nb1;
    }
    __syncthreads();
  }

  // epilogue: register r of a 32 x 32 block is row 8 (r / 4) + 4 (lane / 32) + r % 4, column lane % 32.  The row
  // factors of the similarity epilogue are fetched for all 32 rows of this lane in one batch (clamped, branch-free)
  float rsv[2][16], trv[2][16];
  if (EPI == SE_SIM) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        const int mm = m < p.M ? m : p.M - 1;
        rsv[i][r] = p.rs[mm];
        trv[i][r] = p.tr[mm];
      }
  }
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    const int n = n0 + wn0 + j * 32 + (lane & 31);
    const bool nok = n < p.N;
    float csn = 1.f, tcn = 0.f;
    if (EPI != SE_PLAIN) csn = p.cs[nok ? n : 0];
    if (EPI == SE_SIM) tcn = p.tc[nok ? n : 0];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        float v = acc[i][j][r];
        if (EPI == SE_SIM) v = p.alpha * (v * rsv[i][r] * csn) + (1.f - p.alpha) * expf(-fabsf(trv[i][r] - tcn));
        if (EPI == SE_COLSCALE) v *= csn;
        if (nok && m < p.M) p.C[(long long)m * p.ldc + n] = v;
      }
  }
}

__global__ __launch_bounds__(256) void splitk_reduce_kernel(const float *part, int splits, long long stride,
                                                            long long count, float *out) {
  const long long i = (long long)blockIdx.x * 256 + threadIdx.x;
  if (i >= count) return;
  float s = 0.f;
  for (int q = 0; q < splits; ++q) s += part[q * stride + i];
  out[i] = s;
}

// the same for a symmetric n x n product of which only the tiles on and below the diagonal were computed: one
// workgroup per 32 x 32 block on or below the diagonal adds the partial products, writes the block and, through LDS,
// its transpose (`out` may be `part` when there is a single partial product)
__global__ __launch_bounds__(256) void splitk_reduce_sym_kernel(const float *part, int splits, long long stride, int n,
                                                                long long ldc, float *out) {
  __shared__ float tile[32][33];
  int bm, bn;
  tri_decode(blockIdx.x, bm, bn);
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int r = bm * 32 + ty + 8 * rr, c = bn * 32 + tx;
    const bool ok = r < n && c < n;
    float s = 0.f;
    for (int q = 0; q < splits; ++q) s += part[ok ? q * stride + (long long)r * ldc + c : 0];
    if (ok) out[(long long)r * ldc + c] = s;
    tile[ty + 8 * rr][tx] = s;
  }
  __syncthreads();
  if (bm == bn) return;
#pragma unroll
  for (int rr = 0; rr < 4; ++rr) {
    const int r = bn * 32 + ty + 8 * rr, c = bm * 32 + tx;
    if (r < n && c < n) out[(long long)r * ldc + c] = tile[tx][ty + 8 * rr];
  }
}

// `part` (part_elems floats) allows a plain product with few tiles and a long K to be split along K
hipError_t sgemm(SgemmArgs a, int epi, hipStream_t st, float *part = nullptr, size_t part_elems = 0) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  a.a_kc = a.sak == 1;
  a.b_kc = a.sbk == 1;
  if (!a.a_kc && a.sam != 1) return hipErrorInvalidValue;
  if (!a.b_kc && a.sbn != 1) return hipErrorInvalidValue;
  // 16-byte loads: base aligned, the strided dimension's stride and the contiguous extent multiples of 4
  a.a_vec = aligned16(a.A) && (a.a_kc ? (a.sam % 4 == 0 && a.K % 4 == 0) : (a.sak % 4 == 0 && a.M % 4 == 0));
  a.b_vec = aligned16(a.B) && (a.b_kc ? (a.sbn % 4 == 0 && a.K % 4 == 0) : (a.sbk % 4 == 0 && a.N % 4 == 0));
  if (a.sym && (epi != SE_PLAIN || a.M != a.N || a.A != a.B || a.sam != a.sbn || a.sak != a.sbk)) return hipErrorInvalidValue;
  const int tiles_m = (a.M + TM - 1) / TM;
  const int tiles = a.sym ? tiles_m * (tiles_m + 1) / 2 : tiles_m * ((a.N + TN - 1) / TN);
  const int grid = ((tiles + NUM_XCD - 1) / NUM_XCD) * NUM_XCD;
  int splits = 1;
  a.kchunk = a.K > 0 ? a.K : 1;
  a.part_stride = 0;
  float *out = a.C;
  const long long out_elems = (long long)a.M * a.ldc;
  if (epi == SE_PLAIN && part && tiles < 256 && a.K >= 8 * TK) {
    long long want = 512 / tiles;            // at most the 512 workgroups the chip holds at a time
    if (want > 16) want = 16;
    if (want > a.K / (4 * TK)) want = a.K / (4 * TK);
    if (want > (long long)(part_elems / (size_t)out_elems)) want = (long long)(part_elems / (size_t)out_elems);
    if (want > 1) {
      a.kchunk = (int)(((a.K + want - 1) / want + TK - 1) / TK * TK);
      splits = (a.K + a.kchunk - 1) / a.kchunk;
      a.part_stride = out_elems;
      a.C = part;
    }
  }
  const bool vec = a.a_vec && a.b_vec;
#define SG_LAUNCH(AK, BK, E)                                                                                   \
  do {                                                                                                         \
    if (vec) hipLaunchKernelGGL((sgemm_kernel<AK, BK, E, true>), dim3(grid, splits), dim3(256), 0, st, a);     \
    else hipLaunchKernelGGL((sgemm_kernel<AK, BK, E, false>), dim3(grid, splits), dim3(256), 0, st, a);        \
  } while (0)
  if (epi == SE_SIM) {
    if (a.a_kc && a.b_kc) SG_LAUNCH(true, true, SE_SIM);
    else return hipErrorInvalidValue;
  } else if (epi == SE_COLSCALE) {
    if (a.a_kc && a.b_kc) SG_LAUNCH(true, true, SE_COLSCALE);
    else return hipErrorInvalidValue;
  } else {
    if (a.a_kc && a.b_kc) SG_LAUNCH(true, true, SE_PLAIN);
    else if (a.a_kc && !a.b_kc) SG_LAUNCH(true, false, SE_PLAIN);
    else if (!a.a_kc && !a.b_kc) SG_LAUNCH(false, false, SE_PLAIN);
    else return hipErrorInvalidValue;
  }
#undef SG_LAUNCH
  if (a.sym) {
    const int nb = (a.M + 31) / 32;
    hipLaunchKernelGGL(splitk_reduce_sym_kernel, dim3(nb * (nb + 1) / 2), dim3(256), 0, st,
                       splits > 1 ? (const float *)part : (const float *)out, splits, out_elems, a.M, a.ldc, out);
  } else if (splits > 1) {
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((out_elems + 255) / 256)), dim3(256), 0, st, part, splits,
                       out_elems, out_elems, out);
  }
  return hipGetLastError();
}

// --------------------------------------------------------------------------------------- similarity helpers
// 1 / |x_r| of every pool row (fp64 sum of squares); 0 for a zero row
__global__ __launch_bounds__(256) void rownorm_kernel(const float *X, int N, int F, float *rinv) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= N) return;
  const float *x = X + (long long)row * F;
  double s = 0.0;
  for (int j = lane; j < F; j += 64) {
    const double v = x[j];
    s += v * v;
  }
  s = wave_sum(s);
  if (lane == 0) rinv[row] = s > 0.0 ? (float)(1.0 / sqrt(s)) : 0.f;
}

// rows, inverse norms and timestamps of one subsample gathered into dense arrays; an index outside [0, N) raises
// the flag and is replaced by 0
__global__ __launch_bounds__(256) void gather_kernel(const float *X, const float *rinv, const float *t, const int *idx,
                                                     int N, int F, float *Xs, float *cs, float *tc, int *flag) {
  const int h = blockIdx.x;
  int s = idx[h];
  if (s < 0 || s >= N) {
    if (threadIdx.x == 0) atomicOr(flag, 1);
    s = 0;
  }
  const float *src = X + (long long)s * F;
  float *dst = Xs + (long long)h * F;
  for (int j = threadIdx.x; j < F; j += 256) dst[j] = src[j];
  if (threadIdx.x == 0) {
    cs[h] = rinv[s];
    tc[h] = t[s];
  }
}

// d_r: one wavefront per row, fp64 sum
__global__ __launch_bounds__(256) void rowsum_kernel(const float *A, int N, int n, float *dr) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6), lane = threadIdx.x & 63;
  if (row >= N) return;
  const float *a = A + (long long)row * n;
  double s = 0.0;
  for (int j = lane; j < n; j += 64) s += (double)a[j];
  s = wave_sum(s);
  if (lane == 0) dr[row] = (float)s;
}

// d_c in two deterministic stages: partial sums of COL_CHUNKS row ranges, then their sum in order
constexpr int COL_CHUNKS = 64;
__global__ __launch_bounds__(256) void colsum_partial_kernel(const float *A, int N, int n, double *part) {
  __shared__ double red[4][64];
  const int c = threadIdx.x & 63, ph = threadIdx.x >> 6;
  const int col = blockIdx.x * 64 + c;
  const int rows_per = (N + COL_CHUNKS - 1) / COL_CHUNKS;
  const int r0 = blockIdx.y * rows_per, r1 = min(N, r0 + rows_per);
  double s = 0.0;
  if (col < n)
    for (int r = r0 + ph; r < r1; r += 4) s += (double)A[(long long)r * n + col];
  red[ph][c] = s;
  __syncthreads();
  if (ph == 0 && col < n) part[(long long)blockIdx.y * n + col] = ((red[0][c] + red[1][c]) + red[2][c]) + red[3][c];
}

__global__ __launch_bounds__(256) void colsum_final_kernel(const double *part, int n, float *dc) {
  const int col = blockIdx.x * 256 + threadIdx.x;
  if (col >= n) return;
  double s = 0.0;
  for (int b = 0; b < COL_CHUNKS; ++b) s += part[(long long)b * n + col];
  dc[col] = (float)s;
}

__global__ __launch_bounds__(256) void fill_int_kernel(int *p, int count, int v) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < count) p[i] = v;
}

__global__ __launch_bounds__(256) void degree_check_kernel(const float *d, int count, int *flag) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < count) {
    const float v = d[i];
    if (!(v > 0.f) || !isfinite(v)) atomicOr(flag, 1);
  }
}

// `guard` (may be null): a device flag raised by the degree check; the matrix is left alone when it is set
__global__ __launch_bounds__(256) void normalise_kernel(float *A, const float *dr, const float *dc, int N, int n,
                                                        const int *guard) {
  if (guard && *guard) return;
  const int nblk = (n + 255) / 256;
  const int r = blockIdx.x / nblk;
  const int h = (blockIdx.x % nblk) * 256 + threadIdx.x;
  if (h >= n) return;
  const float s = (1.f / sqrtf(dr[r])) * (1.f / sqrtf(dc[h]));
  A[(long long)r * n + h] *= s;
}

// -------------------------------------------------------------------------- orthonormalisation (Cholesky QR)
// partial Gram matrices of kb vectors of length n over ranges of their elements, fp64: part[b][a][c] = sum_j y_a[j]
// y_c[j], vector a's element j at Y[a * sv + j * sj] (rows of a [kb, n] matrix: sv = n, sj = 1; columns of an
// [n, kb] matrix: sv = 1, sj = kb)
__global__ __launch_bounds__(256) void gram_partial_kernel(const float *Y, int kb, int n, long long sv, long long sj,
                                                           int jchunk, double *part) {
  __shared__ float ys[KB_MAX][33];
  const int tid = threadIdx.x, ta = tid >> 4, tb = tid & 15;
  double acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int c = 0; c < 8; ++c) acc[i][c] = 0.0;
  const int j0 = blockIdx.x * jchunk, j1 = min(n, j0 + jchunk);
  for (int jb = j0; jb < j1; jb += 32) {
    __syncthreads();
    for (int u = tid; u < KB_MAX * 32; u += 256) {
      // consecutive lanes along the contiguous direction
      const int a = sj == 1 ? u >> 5 : u & (KB_MAX - 1), j = sj == 1 ? u & 31 : u >> 7;
      const bool ok = a < kb && jb + j < j1;
      const float v = Y[ok ? (long long)a * sv + (long long)(jb + j) * sj : 0];
      ys[a][j] = ok ? v : 0.f;
    }
    __syncthreads();
    for (int j = 0; j < 32; ++j) {
      double av[8], bv[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        av[i] = (double)ys[ta * 8 + i][j];
        bv[i] = (double)ys[tb * 8 + i][j];
      }
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int c = 0; c < 8; ++c) acc[i][c] = fma(av[i], bv[c], acc[i][c]);
    }
  }
  double *out = part + (long long)blockIdx.x * kb * kb;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int a = ta * 8 + i, b = tb * 8 + c;
      if (a < kb && b < kb) out[a * kb + b] = acc[i][c];
    }
}

__global__ __launch_bounds__(256) void gram_reduce_kernel(const double *part, int nparts, int kk, double *W) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= kk) return;
  double s = 0.0;
  int b = 0;
  for (; b + 8 <= nparts; b += 8) {        // eight loads in flight, added in order
    double t[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) t[q] = part[(long long)(b + q) * kk + i];
#pragma unroll
    for (int q = 0; q < 8; ++q) s += t[q];
  }
  for (; b < nparts; ++b) s += part[(long long)b * kk + i];
  W[i] = s;
}

// Inverse Cholesky factor of W + shift I (= Lc Lc^T, Lc lower), one workgroup.  The shift, shift_rel times the largest
// diagonal entry, keeps the factorisation alive when the rows are numerically dependent (shifted Cholesky QR: the
// rows come out better conditioned, not yet orthonormal, and the next pass finishes).
// The sweep is the square-root-free form on one kb x kb array S.  After column j, rows R > j of the columns C > j
// hold the trailing matrix w (kept whole: the copies above the diagonal are updated too and never read, which saves
// every per-lane condition), rows R <= j of the columns C > j hold the inverse being built, r_CR at S[R][C], r's unit
// diagonal implicit.  At column j, with pivot p_j = S[j][j], every element of the columns C > j takes
//   S[R][C] -= g(R) g(C) / p_j,   g(x) = S[x][j] for x != j, g(j) = 1,
// where row j starts from zero (r_Cj = -w_Cj / p_j), which reads only column j.  Wavefront w of the 16 keeps the
// columns w, w + 16, ..., lane l the rows l and l + 64 of each: finished columns are skipped by a test that is
// uniform over the wavefront, and the work stays balanced until the last columns.  The owner of column j publishes it
// through LDS (two buffers in turn, so one barrier per column suffices), with 1 in place of the pivot.
// Then Lc^-1 = diag(p)^-1/2 r.
// Out: Rinv[kb, kb] fp32 = Lc^-1 (lower triangular), so that Rinv Y has orthonormal rows when the shift is
// negligible.  With `check` set (the last pass, whose input should already be near orthonormal) the kernel returns the
// identity at once when W is the identity to 1e-5, and a pivot below 1/4 raises the flag: the block has no full
// rank.  A non-positive pivot always raises it.
__global__ __launch_bounds__(1024) void chol_inv_kernel(const double *W, int kb, double shift_rel, int check,
                                                         float *Rinv, int *flag) {
  __shared__ double colbuf[2][KB_MAX];
  __shared__ double pivbuf[2];
  __shared__ double pivs[KB_MAX];
  __shared__ double red[16];
  __shared__ double dmax;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  constexpr int NC = KB_MAX / 16;
  double S[NC][2];
#pragma unroll
  for (int i = 0; i < NC; ++i)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int R = lane + 64 * h, C = w + 16 * i;
      const bool in = R < kb && C < kb;
      const int lo = R < C ? R : C, hi = R < C ? C : R;
      const double v = W[in ? hi * kb + lo : 0];        // the Gram matrix is read from its lower triangle
      S[i][h] = in ? v : 0.0;
      if (in && R == C) pivs[R] = v;
    }
  // last pass only: rows that are already orthonormal to fp32 level (|W - I| <= 1e-5 everywhere) are left as they are
  if (check) {
    double dev = 0.0;
#pragma unroll
    for (int i = 0; i < NC; ++i)
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int R = lane + 64 * h, C = w + 16 * i;
        const double d = fabs(S[i][h] - (R == C ? 1.0 : 0.0));
        dev = (R < kb && C < kb) ? fmax(dev, d) : dev;
      }
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) dev = fmax(dev, __shfl_xor(dev, o, 64));
    if (lane == 0) red[w] = dev;
  }
  __syncthreads();
  if (tid == 0) {
    double m = 0.0;
    for (int i = 0; i < kb; ++i) m = fmax(m, pivs[i]);
    dmax = m;
  }
  if (check) {
    double dev = 0.0;
    for (int q = 0; q < 16; ++q) dev = fmax(dev, red[q]);
    if (dev <= 1e-5) {                    // the same value in every thread: the whole workgroup leaves together
#pragma unroll
      for (int i = 0; i < NC; ++i)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int R = lane + 64 * h, C = w + 16 * i;
          if (R < kb && C < kb) Rinv[C * kb + R] = R == C ? 1.f : 0.f;
        }
      return;
    }
  }
  __syncthreads();
  const double shift = shift_rel * dmax;
#pragma unroll
  for (int i = 0; i < NC; ++i)
#pragma unroll
    for (int h = 0; h < 2; ++h)
      if (lane + 64 * h == w + 16 * i) S[i][h] += shift;
  for (int j = 0; j < kb; ++j) {
    double *buf = colbuf[j & 1];
    const bool z0 = lane == j, z1 = lane + 64 == j;       // this lane's copy of row j
    if (w == (j & 15)) {
      double v0 = 0.0, v1 = 0.0;
#pragma unroll
      for (int i = 0; i < NC; ++i)
        if (i == (j >> 4)) {
          v0 = S[i][0];
          v1 = S[i][1];
        }
      if (z0) pivbuf[j & 1] = v0;
      if (z1) pivbuf[j & 1] = v1;
      buf[lane] = z0 ? 1.0 : v0;
      buf[lane + 64] = z1 ? 1.0 : v1;
    }
    __syncthreads();
    double piv = pivbuf[j & 1];
    if (!(piv > 0.0) || !isfinite(piv)) {
      if (tid == 0) atomicOr(flag, 2);
      piv = 1.0;
    } else if (check && piv < 0.25) {
      if (tid == 0) atomicOr(flag, 2);
    }
    if (tid == 0) pivs[j] = piv;
    if (w + 16 * (NC - 1) > j) {          // this wavefront still has a column beyond j
      // 1 / p: hardware estimate refined by two Newton steps
      double inv_p = __builtin_amdgcn_rcp(piv);
      inv_p = inv_p * (2.0 - piv * inv_p);
      inv_p = inv_p * (2.0 - piv * inv_p);
      const double g0 = buf[lane], g1 = buf[lane + 64];
#pragma unroll
      for (int i = 0; i < NC; ++i) {
        const int C = w + 16 * i;
        if (C > j && C < kb) {
          const double gc = buf[C] * inv_p;
          const double s0 = z0 ? 0.0 : S[i][0], s1 = z1 ? 0.0 : S[i][1];
          S[i][0] = fma(-g0, gc, s0);
          S[i][1] = fma(-g1, gc, s1);
        }
      }
    }
    // the buffer that column j + 1 is published to was last read at column j - 1, before this column's barrier
  }
  __syncthreads();
#pragma unroll
  for (int i = 0; i < NC; ++i)
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int R = lane + 64 * h, C = w + 16 * i;
      if (R >= kb || C >= kb) continue;
      // S[R][C] with R < C is r_{C, R}: row C of the inverse; everything above the diagonal of Rinv is zero
      float v = 0.f;
      if (R == C) v = (float)(1.0 / sqrt(pivs[R]));
      else if (R < C) v = (float)(S[i][h] / sqrt(pivs[C]));
      Rinv[C * kb + R] = v;
    }
}

// ------------------------------------------------------------------------------- Rayleigh-Ritz (Jacobi)
// sum over each row of 16 lanes, every lane receiving it: four butterfly steps on the data-parallel-primitive paths
// (quad permutes, mirror within 8, mirror within 16), no LDS traffic.  All lanes of a row add the same pairs in the
// same tree, so they hold bitwise the same result.
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
  int lo = __double2loint(v), hi = __double2hiint(v);
  lo = __builtin_amdgcn_update_dpp(0, lo, CTRL, 0xF, 0xF, true);
  hi = __builtin_amdgcn_update_dpp(0, hi, CTRL, 0xF, 0xF, true);
  return __hiloint2double(hi, lo);
}
__device__ __forceinline__ double row16_sum(double v) {
  v += dpp_move<0xB1>(v);    // quad_perm [1, 0, 3, 2]
  v += dpp_move<0x4E>(v);    // quad_perm [2, 3, 0, 1]
  v += dpp_move<0x141>(v);   // row_half_mirror
  v += dpp_move<0x140>(v);   // row_mirror
  return v;
}

// 1 / x and x^-1/2 to fp64 rounding level: hardware estimate, two Newton steps
__device__ __forceinline__ double nr_rcp(double x) {
  double r = __builtin_amdgcn_rcp(x);
  r = r * (2.0 - x * r);
  return r * (2.0 - x * r);
}
__device__ __forceinline__ double nr_rsq(double x) {
  double r = __builtin_amdgcn_rsq(x);
  r = r * (1.5 - 0.5 * x * r * r);
  return r * (1.5 - 0.5 * x * r * r);
}

// Eigenvectors of the symmetric positive semi-definite T[kb, kb] (fp64) by one-sided Jacobi rotations on the rows of
// a copy M of T (LDS): rotations from the left make the rows mutually orthogonal; then row j = lambda_j v_j^T.  The
// kb / 2 pairs of a round are disjoint (round-robin schedule) and rotate concurrently, one pair per row of 16 lanes
// (64 rows in the workgroup), lane e holding elements e, e + 16, ....  The squared row norms are carried along (a
// rotation by tangent t moves t * <x, y> from one to the other) and recomputed at the start of every sweep, so a pair
// costs one reduction.  Rows whose norm is below 10^-11 of the largest are rounding noise and are left alone.  Out:
// the k eigenvectors of largest eigenvalue as rows of Wk[k, kb], sigma[k] = lambda^1/2 (descending) and inv_sigma[k] =
// lambda^-1/2 (0 where lambda = 0).
__global__ __launch_bounds__(1024) void jacobi_kernel(const double *T, int kb, int k, int max_sweeps, float *Wk,
                                                       float *inv_sigma, float *sigma) {
  extern __shared__ double Ms[];
  __shared__ int rotated;
  __shared__ double nrm2[KB_MAX];
  __shared__ double amax;
  const int tid = threadIdx.x, e = tid & 15, grp = tid >> 4;   // grp: 0..63
  const int ldm = kb + 2;
  for (int u = tid; u < kb * kb; u += 1024) {
    const int i = u / kb, j = u % kb;
    Ms[i * ldm + j] = 0.5 * (T[i * kb + j] + T[j * kb + i]);
  }
  if (tid == 0) rotated = 0;
  __syncthreads();
  const int half = kb / 2, ring = kb - 1;
  for (int sweep = 0; sweep <= max_sweeps; ++sweep) {
    for (int j = grp; j < kb; j += 64) {
      double s = 0.0;
      for (int c = e; c < kb; c += 16) {
        const double x = Ms[j * ldm + c];
        s = fma(x, x, s);
      }
      s = row16_sum(s);
      if (e == 0) nrm2[j] = s;
    }
    __syncthreads();
    if (sweep == max_sweeps) break;       // the norms are exact again: ready for the ranking below
    if (tid == 0) {
      double m = 0.0;
      for (int i = 0; i < kb; ++i) m = fmax(m, nrm2[i]);
      amax = m;
    }
    __syncthreads();
    const double floor2 = 1e-22 * amax;
    for (int round = 0; round < ring; ++round) {
      // all 64 lanes of a wavefront run the reduction (the 16-lane groups without a pair add zeros)
      const bool live = grp < half;
      const int pr = live ? grp : 0;
      const int a = pr == 0 ? round : (round + pr) % ring;
      const int b = pr == 0 ? ring : (round - pr + ring) % ring;
      double *ra = Ms + a * ldm, *rb = Ms + b * ldm;
      double x[8], y[8];
      double ga = 0.0;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const int c = e + 16 * i;
        const bool ok = live && c < kb;
        x[i] = ok ? ra[c] : 0.0;
        y[i] = ok ? rb[c] : 0.0;
        ga = fma(x[i], y[i], ga);
      }
      ga = row16_sum(ga);
      const double al = nrm2[a], be = nrm2[b];
      if (live && fmin(al, be) > floor2 && fabs(ga) > 1e-11 * sqrt(al * be)) {
        // the rotation from hardware reciprocal / reciprocal-square-root estimates refined by Newton steps: a
        // correctly rounded division and square root cost several times the rest of the round, and any (c, s) with
        // c^2 + s^2 = 1 to rounding keeps the rows' span; the sweeps converge on the same vectors
        const double zeta = (be - al) * nr_rcp(2.0 * ga);
        const double h2 = fma(zeta, zeta, 1.0);
        const double tt = copysign(1.0, zeta) * nr_rcp(fabs(zeta) + h2 * nr_rsq(h2));
        const double c_ = nr_rsq(fma(tt, tt, 1.0)), s_ = c_ * tt;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const int c = e + 16 * i;
          if (c < kb) {
            ra[c] = c_ * x[i] - s_ * y[i];
            rb[c] = s_ * x[i] + c_ * y[i];
          }
        }
        if (e == 0) {
          nrm2[a] = al - tt * ga;
          nrm2[b] = be + tt * ga;
          rotated = 1;
        }
      }
      __syncthreads();
    }
    const int any = rotated;
    __syncthreads();
    if (tid == 0) rotated = 0;
    __syncthreads();
    if (!any) break;                      // nothing moved in this sweep: the carried norms are the exact ones
  }
  __syncthreads();
  // eigenvalues = row norms; rank them (descending, ties to the lower row)
  for (int j = grp; j < kb; j += 64) {
    int rank = 0;
    const double mine = nrm2[j] > 0.0 ? nrm2[j] : 0.0;
    for (int i = 0; i < kb; ++i) {
      const double o = nrm2[i] > 0.0 ? nrm2[i] : 0.0;
      rank += (o > mine || (o == mine && i < j)) ? 1 : 0;
    }
    if (rank < k) {
      const double lam = sqrt(mine);
      const double inv = lam > 0.0 ? 1.0 / lam : 0.0;
      for (int c = e; c < kb; c += 16) Wk[rank * kb + c] = (float)(Ms[j * ldm + c] * inv);
      if (e == 0) {
        sigma[rank] = (float)sqrt(lam);
        inv_sigma[rank] = lam > 0.0 ? (float)(1.0 / sqrt(lam)) : 0.f;
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------- k-means
__device__ __forceinline__ int clamp_label(int v, int k) { return v < 0 ? 0 : (v >= k ? k - 1 : v); }

__global__ __launch_bounds__(256) void kmeans_init_kernel(const float *U, int N, int d, int k, const int *init_idx,
                                                          float *centres, int *flag) {
  const int c = blockIdx.x;
  int r = init_idx[c];
  if (r < 0 || r >= N) {
    if (threadIdx.x == 0) atomicOr(flag, 1);
    r = 0;
  }
  for (int j = threadIdx.x; j < d; j += 256) centres[c * d + j] = U[(long long)r * d + j];
}

// Control words of one k-means run (device, ints): ctl[0], ctl[1] = labels changed by the passes of even / odd index,
// ctl[2] = 1 once a pass has changed nothing, ctl[3] = assignment passes run.  Every kernel of a pass leaves at once
// when ctl[2] is up, so the host may enqueue passes ahead of knowing whether they are needed.
constexpr int KM_DONE = 2, KM_PASSES = 3;

// assignment pass `it`: 64 rows per workgroup staged in LDS beside the centres (rows padded with zeros to whole
// float4s, which leaves every sum as it is); thread (row, g) scans the centres c = g, g + 4, ... four at a time (one
// 16-byte broadcast read per centre and four dimensions), each sum running over the dimensions in ascending order; the
// four candidates of a row are merged with ties to the lowest centre
__global__ __launch_bounds__(256) void kmeans_assign_kernel(const float *U, int N, int d, const float *centres, int k,
                                                            int *labels, int *ctl, int it) {
  if (ctl[KM_DONE]) return;
  extern __shared__ float sm[];
  const int dp = (d + 3) & ~3;
  float *cs = sm;                       // [k][dp]
  float *us = sm + k * dp;              // [64][dp + 1]
  __shared__ float bd[4][64];
  __shared__ int bi[4][64];
  const int tid = threadIdx.x, row = tid & 63, g = tid >> 6;
  const int r0 = blockIdx.x * 64;
  if (blockIdx.x == 0 && tid == 0) atomicAdd(&ctl[KM_PASSES], 1);
  for (int u = tid; u < k * dp; u += 256) {
    const int c = u / dp, j = u - c * dp;
    const float v = centres[j < d ? c * d + j : 0];
    cs[u] = j < d ? v : 0.f;
  }
  for (int u = tid; u < 64 * dp; u += 256) {
    const int rr = u / dp, j = u - rr * dp;
    const bool ok = r0 + rr < N && j < d;
    const float v = U[ok ? (long long)(r0 + rr) * d + j : 0];
    us[rr * (dp + 1) + j] = ok ? v : 0.f;
  }
  __syncthreads();
  float best = INFINITY;
  int besti = 0x7fffffff;
  const float *u = us + row * (dp + 1);
  for (int c0 = g; c0 < k; c0 += 16) {
    const float *p0 = cs + c0 * dp;
    const float *p1 = cs + (c0 + 4 < k ? c0 + 4 : c0) * dp;
    const float *p2 = cs + (c0 + 8 < k ? c0 + 8 : c0) * dp;
    const float *p3 = cs + (c0 + 12 < k ? c0 + 12 : c0) * dp;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    for (int j = 0; j < dp; j += 4) {
      const float4 a0 = *(const float4 *)(p0 + j), a1 = *(const float4 *)(p1 + j);
      const float4 a2 = *(const float4 *)(p2 + j), a3 = *(const float4 *)(p3 + j);
      const float u0 = u[j], u1 = u[j + 1], u2 = u[j + 2], u3 = u[j + 3];
      float t;
      t = u0 - a0.x; s0 = fmaf(t, t, s0); t = u1 - a0.y; s0 = fmaf(t, t, s0);
      t = u2 - a0.z; s0 = fmaf(t, t, s0); t = u3 - a0.w; s0 = fmaf(t, t, s0);
      t = u0 - a1.x; s1 = fmaf(t, t, s1); t = u1 - a1.y; s1 = fmaf(t, t, s1);
      t = u2 - a1.z; s1 = fmaf(t, t, s1); t = u3 - a1.w; s1 = fmaf(t, t, s1);
      t = u0 - a2.x; s2 = fmaf(t, t, s2); t = u1 - a2.y; s2 = fmaf(t, t, s2);
      t = u2 - a2.z; s2 = fmaf(t, t, s2); t = u3 - a2.w; s2 = fmaf(t, t, s2);
      t = u0 - a3.x; s3 = fmaf(t, t, s3); t = u1 - a3.y; s3 = fmaf(t, t, s3);
      t = u2 - a3.z; s3 = fmaf(t, t, s3); t = u3 - a3.w; s3 = fmaf(t, t, s3);
    }
    if (s0 < best) { best = s0; besti = c0; }
    if (c0 + 4 < k && s1 < best) { best = s1; besti = c0 + 4; }
    if (c0 + 8 < k && s2 < best) { best = s2; besti = c0 + 8; }
    if (c0 + 12 < k && s3 < best) { best = s3; besti = c0 + 12; }
  }
  bd[g][row] = best;
  bi[g][row] = besti;
  __syncthreads();
  if (g == 0 && r0 + row < N) {
    for (int q = 1; q < 4; ++q) {
      const float s = bd[q][row];
      const int c = bi[q][row];
      if (s < best || (s == best && c < besti)) {
        best = s;
        besti = c;
      }
    }
    if (labels[r0 + row] != besti) {
      labels[r0 + row] = besti;
      atomicAdd(&ctl[it & 1], 1);
    }
  }
}

// update pass, stage 1: workgroup b walks its range of rows in ascending order, thread j owning dimension j, and adds
// each row to its cluster's fp64 sums in LDS (LDS adds without return value: the adds of one thread to one address
// are carried out in program order, so the sums are those of the rows in ascending order; 32 rows are loaded ahead);
// stage 2 adds the workgroups' sums in order.  An empty cluster keeps its centre.  Nothing happens when the pass
// changed no label.
__global__ __launch_bounds__(128) void kmeans_partial_kernel(const float *U, int N, int d, const int *labels, int k,
                                                             int rows_per, double *psum, int *pcnt, const int *ctl,
                                                             int it) {
  if (ctl[KM_DONE] || ctl[it & 1] == 0) return;
  extern __shared__ double accs[];      // [k][d]
  __shared__ int cnt[KB_MAX];
  const int j = threadIdx.x;
  for (int u = j; u < k * d; u += 128) accs[u] = 0.0;
  for (int u = j; u < k; u += 128) cnt[u] = 0;
  __syncthreads();
  const int r0 = blockIdx.x * rows_per, r1 = min(N, r0 + rows_per);
  const int jj = j < d ? j : 0;
  int r = r0;
  constexpr int RB = 32;                  // rows per batch; two batches are in flight
  int c[RB], cn[RB];
  float v[RB], vn[RB];
  if (r + RB <= r1) {
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      c[i] = labels[r + i];
      v[i] = U[(long long)(r + i) * d + jj];
    }
  }
  for (; r + RB <= r1; r += RB) {
    // the next batch is requested before this one is added (clamped to the range: the last request repeats rows)
    const int rn = r + 2 * RB <= r1 ? r + RB : r;
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      cn[i] = labels[rn + i];
      vn[i] = U[(long long)(rn + i) * d + jj];
    }
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      const int ci = clamp_label(c[i], k);
      if (j < d) atomicAdd(&accs[ci * d + j], (double)v[i]);
      if (j == 0) atomicAdd(&cnt[ci], 1);
    }
#pragma unroll
    for (int i = 0; i < RB; ++i) {
      c[i] = cn[i];
      v[i] = vn[i];
    }
  }
  for (; r < r1; ++r) {
    const int c = clamp_label(labels[r], k);
    if (j < d) atomicAdd(&accs[c * d + j], (double)U[(long long)r * d + j]);
    if (j == 0) atomicAdd(&cnt[c], 1);
  }
  __syncthreads();
  double *ps = psum + (long long)blockIdx.x * k * d;
  for (int u = j; u < k * d; u += 128) ps[u] = accs[u];
  for (int u = j; u < k; u += 128) pcnt[blockIdx.x * k + u] = cnt[u];
}

// stage 2, and the bookkeeping of pass `it`: a pass that changed nothing raises ctl[2]; otherwise the other pass
// parity's counter is cleared for the next pass (nothing reads it during this kernel)
__global__ __launch_bounds__(64) void kmeans_finish_kernel(const double *psum, const int *pcnt, int nb, int k, int d,
                                                           float *centres, int *ctl, int it) {
  if (ctl[KM_DONE]) return;
  if (ctl[it & 1] == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) ctl[KM_DONE] = 1;
    return;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) ctl[(it + 1) & 1] = 0;
  const int u = blockIdx.x * 64 + threadIdx.x;
  if (u >= k * d) return;
  const int c = u / d;
  double tot = 0.0;
  int m = 0;
  int b = 0;
  for (; b + 16 <= nb; b += 16) {
    double t[16];
    int q[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      t[i] = psum[(long long)(b + i) * k * d + u];
      q[i] = pcnt[(b + i) * k + c];
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      tot += t[i];
      m += q[i];
    }
  }
  for (; b < nb; ++b) {
    tot += psum[(long long)b * k * d + u];
    m += pcnt[b * k + c];
  }
  if (m > 0) centres[u] = (float)(tot / (double)m);
}

// ---------------------------------------------------------------------------------------------- aggregation
__global__ __launch_bounds__(256) void contingency_kernel(const int *a, const int *b, int N, int k, int *T) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r < N) atomicAdd(&T[clamp_label(a[r], k) * k + clamp_label(b[r], k)], 1);
}

// greedy renaming, one workgroup: k times take the largest remaining count (ties to the lowest flat index), fix
// perm[column] = row, retire the row and the column.  The table lives in registers, 16 entries per thread, each as
// the 64-bit key (count << 32) | (2^31 - 1 - flat index), so that the largest key is the entry wanted; retired and
// absent entries are -1.  A round is a maximum over the thread's keys, over the wavefront (shuffles) and over the 16
// wavefronts (LDS, two buffers in turn: one barrier per round).
__global__ __launch_bounds__(1024) void greedy_match_kernel(const int *T, int k, int *perm) {
  constexpr int PER = KB_MAX * KB_MAX / 1024;
  __shared__ long long wbest[2][16];
  const int tid = threadIdx.x;
  long long key[PER];
  int rc[PER];                              // (row << 8) | column of the entry
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    const int u = tid + 1024 * i;
    const bool in = u < k * k;
    const int v = T[in ? u : 0];
    key[i] = in ? ((long long)v << 32) | (long long)(unsigned)(0x7fffffff - u) : -1ll;
    rc[i] = in ? ((u / k) << 8) | (u % k) : 0xffff;
  }
  for (int it = 0; it < k; ++it) {
    long long m = key[0];
#pragma unroll
    for (int i = 1; i < PER; ++i) m = key[i] > m ? key[i] : m;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
      const long long x = __shfl_xor(m, o, 64);
      m = x > m ? x : m;
    }
    if ((tid & 63) == 0) wbest[it & 1][tid >> 6] = m;
    __syncthreads();
    long long g = wbest[it & 1][0];
#pragma unroll
    for (int w = 1; w < 16; ++w) {
      const long long x = wbest[it & 1][w];
      g = x > g ? x : g;
    }
    // rows and columns retire in pairs, so (k - it)^2 entries are still live here and g >= 0
    const int u = 0x7fffffff - (int)(unsigned)(g & 0xffffffffll);
    const int p = u / k, q = u - p * k;
    if (tid == 0) perm[q] = p;
#pragma unroll
    for (int i = 0; i < PER; ++i)
      if ((rc[i] >> 8) == p || (rc[i] & 0xff) == q) key[i] = -1ll;
  }
}

__global__ __launch_bounds__(256) void identity_perm_kernel(int *perm, int k) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < k) perm[i] = i;
}

__global__ __launch_bounds__(256) void vote_kernel(const int *labels, const int *perm, int m, int N, int k, int *out) {
  const int r = blockIdx.x * 256 + threadIdx.x;
  if (r >= N) return;
  int name[M_MAX];
  for (int i = 0; i < m; ++i) name[i] = perm[i * k + clamp_label(labels[(long long)i * N + r], k)];
  int best = 0, pick = name[0];
  for (int i = 0; i < m; ++i) {
    int votes = 0;
    for (int q = 0; q < m; ++q) votes += name[q] == name[i] ? 1 : 0;
    if (votes > best) {      // strict: the earliest vector among the most frequent names wins
      best = votes;
      pick = name[i];
    }
  }
  out[r] = pick;
}

// ------------------------------------------------------------------------------------------- host side
struct Carve {
  char *base;
  size_t off = 0;
  explicit Carve(void *b) : base(static_cast<char *>(b)) {}
  template <class T>
  T *take(size_t count) {
    off = (off + 255) & ~size_t(255);
    T *p = base ? reinterpret_cast<T *>(base + off) : nullptr;
    off += count * sizeof(T);
    return p;
  }
};

// element ranges of the partial Gram matrices: at most 128 of them, whole multiples of the 32 elements the kernel
// stages at a time
int gram_chunk(int len) { return (((len + 127) / 128) + 31) / 32 * 32; }
int gram_parts(int len) { return (len + gram_chunk(len) - 1) / gram_chunk(len); }

// row ranges of the k-means partial sums: at most 256 of them, at least 256 rows each
int kmeans_rows_per(int N) {
  const int r = (N + 255) / 256;
  return r < 256 ? 256 : r;
}
int kmeans_blocks(int N) { return (N + kmeans_rows_per(N) - 1) / kmeans_rows_per(N); }

struct SimWork {
  float *rinv, *Xs, *cs, *tc;
  double *colpart;
  int *flag;
  size_t bytes;
  SimWork(void *w, int N, int F, int n) {
    Carve c(w);
    flag = c.take<int>(64);
    rinv = c.take<float>(N);
    Xs = c.take<float>((size_t)n * F);
    cs = c.take<float>(n);
    tc = c.take<float>(n);
    colpart = c.take<double>((size_t)COL_CHUNKS * n);
    bytes = c.off + 256;
  }
};

struct EmbedWork {
  float *G, *Q, *Y, *Z, *Bm, *Wk, *isig, *Rinv, *spart;
  size_t spart_elems;
  double *part, *W;
  int *flag;
  size_t bytes;
  EmbedWork(void *w, int N, int n, int k, int kb) {
    Carve c(w);
    flag = c.take<int>(64);
    G = c.take<float>((size_t)n * n);
    Q = c.take<float>((size_t)kb * n);
    Y = c.take<float>((size_t)kb * n);
    Z = c.take<float>((size_t)kb * n);
    Bm = c.take<float>((size_t)N * kb);
    Wk = c.take<float>((size_t)k * kb);
    isig = c.take<float>(k);
    Rinv = c.take<float>((size_t)kb * kb);
    spart_elems = (size_t)5 * n * n;
    spart = c.take<float>(spart_elems);
    const int parts = gram_parts(n) > gram_parts(N) ? gram_parts(n) : gram_parts(N);
    part = c.take<double>((size_t)parts * kb * kb);
    W = c.take<double>((size_t)kb * kb);
    bytes = c.off + 256;
  }
};

struct SmallWork {      // k-means (N rows of d dimensions), aggregation, normalisation
  int *flag, *changed, *T, *perm, *pcnt;
  double *psum;
  size_t bytes;
  SmallWork(void *w, int N, int d, int k) {
    Carve c(w);
    flag = c.take<int>(64);
    changed = c.take<int>(64);
    T = c.take<int>((size_t)k * k);
    perm = c.take<int>((size_t)M_MAX * k);
    pcnt = c.take<int>((size_t)kmeans_blocks(N) * k);
    psum = c.take<double>((size_t)kmeans_blocks(N) * k * d);
    bytes = c.off + 256;
  }
};

struct ClusterWork {
  float *A, *dr, *dc, *U, *sigma, *centres;
  int *flags;           // [4]: index, degree, rank, initial-centre checks of a deferred run
  void *sub;            // region handed to the calls above
  size_t sub_bytes, bytes;
  ClusterWork(void *w, int N, int F, int n, int k, int kb) {
    Carve c(w);
    A = c.take<float>((size_t)N * n);
    dr = c.take<float>(N);
    dc = c.take<float>(n);
    U = c.take<float>((size_t)N * k);
    sigma = c.take<float>(k);
    centres = c.take<float>((size_t)k * k);
    flags = c.take<int>(64);
    // the k-means region is sized for rows of up to kb dimensions, so that the one size also covers qc_tap_kmeans
    // on an embedding of the whole iteration block
    size_t s1 = SimWork(nullptr, N, F, n).bytes, s2 = EmbedWork(nullptr, N, n, k, kb).bytes, s3 = SmallWork(nullptr, N, kb, kb).bytes;
    sub_bytes = s1 > s2 ? s1 : s2;
    if (s3 > sub_bytes) sub_bytes = s3;
    sub = c.take<char>(sub_bytes);
    bytes = c.off + 256;
  }
};

int check_dims(int N, int F, int n, int k, int kb) {
  if (N < 1 || F < 1 || n < 1 || k < 1 || kb < 1) TAP_FAIL(QC_ERR_SHAPE, "N, F, n, k, kb must be positive");
  if (kb > KB_MAX || kb % 8) TAP_FAIL(QC_ERR_UNSUPPORTED, "kb must be a multiple of 8 and at most %d (got %d)", KB_MAX, kb);
  if (k > kb) TAP_FAIL(QC_ERR_SHAPE, "k (%d) exceeds kb (%d)", k, kb);
  if (kb > n) TAP_FAIL(QC_ERR_SHAPE, "kb (%d) exceeds the subsample size n (%d)", kb, n);
  if (n > N) TAP_FAIL(QC_ERR_SHAPE, "n (%d) exceeds N (%d)", n, N);
  if ((long long)N * (n > F ? n : F) >= (1ll << 31)) TAP_FAIL(QC_ERR_UNSUPPORTED, "N * max(n, F) must be below 2^31");
  return QC_OK;
}

// reads a device flag word after waiting for the stream
int read_flag(const int *flag, hipStream_t st, int *out) {
  TAP_HIP(hipMemcpyAsync(out, flag, sizeof(int), hipMemcpyDeviceToHost, st));
  TAP_HIP(hipStreamSynchronize(st));
  return QC_OK;
}

// optional timing of the similarity contraction (the dominant kernel) with events on the caller's stream
struct SimProfile {
  bool on = false;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> ev;
  size_t used = 0;
};
SimProfile g_prof;

// Each stage below takes `ext`: null = use the flag word in its own workspace and report the error before returning
// (the stage waits for the stream); non-null = raise that device flag instead and only enqueue (the caller reads the
// flags of several stages, possibly of several streams, later).
// Internal streams and events of one qc_tap_cluster call (default priority).  They belong to the call, not to the
// process: calls from several host threads, or on several devices, share nothing.
constexpr int MAX_SLOTS = 3;
struct CallStreams {
  hipStream_t streams[MAX_SLOTS] = {nullptr, nullptr, nullptr};
  hipEvent_t fork = nullptr;
  hipEvent_t chain[MAX_SLOTS] = {nullptr, nullptr, nullptr};
  ~CallStreams() {
    for (int j = 0; j < MAX_SLOTS; ++j) {
      if (streams[j]) { (void)hipStreamSynchronize(streams[j]); (void)hipStreamDestroy(streams[j]); }
      if (chain[j]) (void)hipEventDestroy(chain[j]);
    }
    if (fork) (void)hipEventDestroy(fork);
  }
};

// `gemm_after` (may be null): the contraction starts after this event.  A caller that runs several subsamples on
// several streams chains them (embed_impl records the matching event after its own large product), so that the
// chip-filling products run one after the other and only the small, latency-bound kernels overlap.
int similarity_impl(const float *X, const float *t, int N, int F, const int *idx, int n, float alpha, float *A,
                    float *d_r, float *d_c, void *work, hipStream_t st, int *ext = nullptr,
                    hipEvent_t gemm_after = nullptr) {
  SimWork w(work, N, F, n);
  int *fl = ext ? ext : w.flag;
  if (!ext) hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(256), 0, st, w.flag, 64, 0);
  hipLaunchKernelGGL(rownorm_kernel, dim3((N + 3) / 4), dim3(256), 0, st, X, N, F, w.rinv);
  hipLaunchKernelGGL(gather_kernel, dim3(n), dim3(256), 0, st, X, w.rinv, t, idx, N, F, w.Xs, w.cs, w.tc, fl);
  TAP_HIP(hipGetLastError());
  SgemmArgs g{};
  g.A = X; g.sam = F; g.sak = 1;
  g.B = w.Xs; g.sbn = F; g.sbk = 1;
  g.C = A; g.ldc = n;
  g.M = N; g.N = n; g.K = F;
  g.rs = w.rinv; g.cs = w.cs; g.tr = t; g.tc = w.tc; g.alpha = alpha;
  if (gemm_after) TAP_HIP(hipStreamWaitEvent(st, gemm_after, 0));
  if (g_prof.on) {
    if (g_prof.used == g_prof.ev.size()) {
      hipEvent_t a, b;
      TAP_HIP(hipEventCreate(&a));
      TAP_HIP(hipEventCreate(&b));
      g_prof.ev.emplace_back(a, b);
    }
    TAP_HIP(hipEventRecord(g_prof.ev[g_prof.used].first, st));
  }
  TAP_HIP(sgemm(g, SE_SIM, st));
  if (g_prof.on) TAP_HIP(hipEventRecord(g_prof.ev[g_prof.used++].second, st));
  hipLaunchKernelGGL(rowsum_kernel, dim3((N + 3) / 4), dim3(256), 0, st, A, N, n, d_r);
  hipLaunchKernelGGL(colsum_partial_kernel, dim3((n + 63) / 64, COL_CHUNKS), dim3(256), 0, st, A, N, n, w.colpart);
  hipLaunchKernelGGL(colsum_final_kernel, dim3((n + 255) / 256), dim3(256), 0, st, w.colpart, n, d_c);
  TAP_HIP(hipGetLastError());
  if (ext) return QC_OK;
  int flag = 0;
  TAP_RC(read_flag(w.flag, st, &flag));
  if (flag) TAP_FAIL(QC_ERR_RANGE, "a subsample index lies outside [0, %d)", N);
  return QC_OK;
}

int normalise_impl(float *A, const float *d_r, const float *d_c, int N, int n, void *work, hipStream_t st,
                   int *ext = nullptr) {
  SmallWork w(work, 1, 1, 1);
  int *fl = ext ? ext : w.flag;
  if (!ext) hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(256), 0, st, w.flag, 64, 0);
  hipLaunchKernelGGL(degree_check_kernel, dim3((N + 255) / 256), dim3(256), 0, st, d_r, N, fl);
  hipLaunchKernelGGL(degree_check_kernel, dim3((n + 255) / 256), dim3(256), 0, st, d_c, n, fl);
  TAP_HIP(hipGetLastError());
  if (!ext) {
    int flag = 0;
    TAP_RC(read_flag(w.flag, st, &flag));
    if (flag) TAP_FAIL(QC_ERR_RANGE, "a degree of the similarity matrix is not positive and finite");
  }
  // with a deferred check the kernel itself leaves the matrix alone when the flag is up
  hipLaunchKernelGGL(normalise_kernel, dim3(((n + 255) / 256) * N), dim3(256), 0, st, A, d_r, d_c, N, n,
                     ext ? (const int *)ext : (const int *)nullptr);
  TAP_HIP(hipGetLastError());
  if (!ext) TAP_HIP(hipStreamSynchronize(st));
  return QC_OK;
}

hipError_t set_lds(const void *kern, size_t bytes) {
  return hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

// one pass of shifted Cholesky QR on the rows of `in` [kb, n] into `out` (`in` and `out` must differ)
int cholqr_pass(const float *in, float *out, int kb, int n, int check, EmbedWork &w, int *fl, hipStream_t st) {
  const int parts = gram_parts(n);
  hipLaunchKernelGGL(gram_partial_kernel, dim3(parts), dim3(256), 0, st, in, kb, n, (long long)n, 1ll, gram_chunk(n),
                     w.part);
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((kb * kb + 255) / 256), dim3(256), 0, st, w.part, parts, kb * kb, w.W);
  hipLaunchKernelGGL(chol_inv_kernel, dim3(1), dim3(1024), 0, st, w.W, kb, 1e-12, check, w.Rinv, fl);
  TAP_HIP(hipGetLastError());
  SgemmArgs g{};
  g.A = w.Rinv; g.sam = kb; g.sak = 1;
  g.B = in; g.sbn = 1; g.sbk = n;
  g.C = out; g.ldc = n;
  g.M = kb; g.N = n; g.K = kb;
  TAP_HIP(sgemm(g, SE_PLAIN, st));
  return QC_OK;
}

// rows of `in` made orthonormal into w.Q: three passes, which is enough for a block whose condition number is as
// large as 10^12 (the power iteration multiplies by L^T L, whose small eigenvalues are rounding noise in fp32); uses
// w.Z and w.Y as intermediates (`in` may be w.Y)
int orthonormalise(const float *in, EmbedWork &w, int kb, int n, int *fl, hipStream_t st) {
  TAP_RC(cholqr_pass(in, w.Z, kb, n, 0, w, fl, st));
  TAP_RC(cholqr_pass(w.Z, w.Y, kb, n, 0, w, fl, st));
  TAP_RC(cholqr_pass(w.Y, w.Q, kb, n, 1, w, fl, st));
  return QC_OK;
}

// Between two multiplications of the power iteration one pass is enough: the next product only needs rows that span
// the same space and are well conditioned (a single shifted pass leaves them orthonormal to about the square of the
// block's condition number times the fp64 rounding, far from dependent); `in` must not be w.Q
int recondition(const float *in, EmbedWork &w, int kb, int n, int *fl, hipStream_t st) {
  return cholqr_pass(in, w.Q, kb, n, 0, w, fl, st);
}

// `big_done` (may be null) is recorded after the one chip-filling product of this stage (L^T L)
int embed_impl(const float *L, int N, int n, int k, int kb, int iters, const float *q0, float *U, float *sigma,
               void *work, hipStream_t st, int *ext = nullptr, hipEvent_t big_done = nullptr) {
  EmbedWork w(work, N, n, k, kb);
  int *fl = ext ? ext : w.flag;
  if (!ext) hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(256), 0, st, w.flag, 64, 0);
  TAP_HIP(hipGetLastError());
  // G = L^T L drives the power iteration (its fp32 rounding only slows the convergence of directions whose singular
  // values are below about 3e-4 of the largest; the Rayleigh-Ritz step below works on L itself)
  SgemmArgs g{};
  g.A = L; g.sam = 1; g.sak = n;
  g.B = L; g.sbn = 1; g.sbk = n;
  g.C = w.G; g.ldc = n;
  g.M = n; g.N = n; g.K = N;
  g.sym = 1;
  TAP_HIP(sgemm(g, SE_PLAIN, st, w.spart, w.spart_elems));
  if (big_done) TAP_HIP(hipEventRecord(big_done, st));
  if (iters > 0) TAP_RC(recondition(q0, w, kb, n, fl, st));
  else TAP_RC(orthonormalise(q0, w, kb, n, fl, st));
  SgemmArgs mul{};
  mul.A = w.Q; mul.sam = n; mul.sak = 1;
  mul.B = w.G; mul.sbn = n; mul.sbk = 1;      // G is symmetric
  mul.C = w.Y; mul.ldc = n;
  mul.M = kb; mul.N = n; mul.K = n;
  for (int it = 0; it < iters; ++it) {
    TAP_HIP(sgemm(mul, SE_PLAIN, st, w.spart, w.spart_elems));
    if (it + 1 < iters) TAP_RC(recondition(w.Y, w, kb, n, fl, st));
    else TAP_RC(orthonormalise(w.Y, w, kb, n, fl, st));      // the final basis: orthonormal to fp32 level
  }
  // Rayleigh-Ritz on B = L Q^T [N, kb]: T = B^T B (fp64), its k leading eigenvectors W, U = B W^T diag(1 / sigma)
  SgemmArgs bm{};
  bm.A = L; bm.sam = n; bm.sak = 1;
  bm.B = w.Q; bm.sbn = n; bm.sbk = 1;
  bm.C = w.Bm; bm.ldc = kb;
  bm.M = N; bm.N = kb; bm.K = n;
  TAP_HIP(sgemm(bm, SE_PLAIN, st));
  const int parts = gram_parts(N);
  hipLaunchKernelGGL(gram_partial_kernel, dim3(parts), dim3(256), 0, st, w.Bm, kb, N, 1ll, (long long)kb, gram_chunk(N),
                     w.part);
  hipLaunchKernelGGL(gram_reduce_kernel, dim3((kb * kb + 255) / 256), dim3(256), 0, st, w.part, parts, kb * kb, w.W);
  const size_t lds = (size_t)kb * (kb + 2) * sizeof(double);
  TAP_HIP(set_lds((const void *)jacobi_kernel, lds));
  hipLaunchKernelGGL(jacobi_kernel, dim3(1), dim3(1024), lds, st, w.W, kb, k, 30, w.Wk, w.isig, sigma);
  TAP_HIP(hipGetLastError());
  SgemmArgs u{};
  u.A = w.Bm; u.sam = kb; u.sak = 1;
  u.B = w.Wk; u.sbn = kb; u.sbk = 1;
  u.C = U; u.ldc = k;
  u.M = N; u.N = k; u.K = kb;
  u.cs = w.isig;
  TAP_HIP(sgemm(u, SE_COLSCALE, st));
  if (ext) return QC_OK;
  int flag = 0;
  TAP_RC(read_flag(w.flag, st, &flag));
  if (flag) TAP_FAIL(QC_ERR_RANGE, "the iteration block has no full rank (a zero start vector, or fewer than kb independent directions)");
  return QC_OK;
}

// One k-means problem of a group that advances in lockstep, each on its own stream
struct KmSlot {
  const float *U;
  const int *init_idx;
  int *labels;
  float *centres;
  void *work;
  hipStream_t st;
  int *ext;            // null, or a device flag for the index check (read by the caller)
  int passes;
  bool active;
};

// Lloyd's iteration on `ns` problems of the same shape, each on its own stream.  The passes decide on the device
// whether they still have work (see the control words above), so the host enqueues KM_BATCH passes on every stream and
// only then reads the control words; a problem leaves the loop when a pass has changed nothing.  With a null `ext` the
// initial-centre indices are checked (and the error reported) before the first pass.
constexpr int KM_BATCH = 8;

int kmeans_multi(KmSlot *slots, int ns, int N, int d, int k, int max_iter) {
  const int dp = (d + 3) & ~3;
  const size_t lds = ((size_t)k * dp + (size_t)64 * (dp + 1)) * sizeof(float);
  TAP_HIP(set_lds((const void *)kmeans_assign_kernel, lds));
  const size_t lds_acc = (size_t)k * d * sizeof(double);
  TAP_HIP(set_lds((const void *)kmeans_partial_kernel, lds_acc));
  const int nb = kmeans_blocks(N);
  for (int i = 0; i < ns; ++i) {
    KmSlot &q = slots[i];
    SmallWork w(q.work, N, d, k);
    if (!q.ext) hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(256), 0, q.st, w.flag, 64, 0);
    hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(256), 0, q.st, w.changed, 64, 0);
    hipLaunchKernelGGL(fill_int_kernel, dim3((N + 255) / 256), dim3(256), 0, q.st, q.labels, N, -1);
    hipLaunchKernelGGL(kmeans_init_kernel, dim3(k), dim3(256), 0, q.st, q.U, N, d, k, q.init_idx, q.centres,
                       q.ext ? q.ext : w.flag);
    TAP_HIP(hipGetLastError());
    q.passes = 0;
    q.active = max_iter > 0;
  }
  for (int i = 0; i < ns; ++i) {
    if (slots[i].ext) continue;
    SmallWork w(slots[i].work, N, d, k);
    int flag = 0;
    TAP_RC(read_flag(w.flag, slots[i].st, &flag));
    if (flag) TAP_FAIL(QC_ERR_RANGE, "an initial-centre index lies outside [0, %d)", N);
  }
  for (int it0 = 0; it0 < max_iter; it0 += KM_BATCH) {
    const int it1 = it0 + KM_BATCH < max_iter ? it0 + KM_BATCH : max_iter;
    bool any = false;
    for (int it = it0; it < it1; ++it) {
      for (int i = 0; i < ns; ++i) {
        KmSlot &q = slots[i];
        if (!q.active) continue;
        any = true;
        SmallWork w(q.work, N, d, k);
        hipLaunchKernelGGL(kmeans_assign_kernel, dim3((N + 63) / 64), dim3(256), lds, q.st, q.U, N, d, q.centres, k,
                           q.labels, w.changed, it);
        hipLaunchKernelGGL(kmeans_partial_kernel, dim3(nb), dim3(128), lds_acc, q.st, q.U, N, d, q.labels, k,
                           kmeans_rows_per(N), w.psum, w.pcnt, w.changed, it);
        hipLaunchKernelGGL(kmeans_finish_kernel, dim3((k * d + 63) / 64), dim3(64), 0, q.st, w.psum, w.pcnt, nb, k, d,
                           q.centres, w.changed, it);
        TAP_HIP(hipGetLastError());
      }
    }
    if (!any) break;
    for (int i = 0; i < ns; ++i) {
      KmSlot &q = slots[i];
      if (!q.active) continue;
      SmallWork w(q.work, N, d, k);
      int ctl[4] = {0, 0, 0, 0};
      TAP_HIP(hipMemcpyAsync(ctl, w.changed, sizeof(ctl), hipMemcpyDeviceToHost, q.st));
      TAP_HIP(hipStreamSynchronize(q.st));
      q.passes = ctl[KM_PASSES];
      if (ctl[KM_DONE]) q.active = false;
    }
  }
  for (int i = 0; i < ns; ++i) TAP_HIP(hipStreamSynchronize(slots[i].st));
  return QC_OK;
}

int kmeans_impl(const float *U, int N, int d, int k, const int *init_idx, int max_iter, int *labels, float *centres,
                int *passes_out, void *work, hipStream_t st) {
  KmSlot q{U, init_idx, labels, centres, work, st, nullptr, 0, false};
  TAP_RC(kmeans_multi(&q, 1, N, d, k, max_iter));
  if (passes_out) *passes_out = q.passes;
  return QC_OK;
}

int aggregate_impl(const int *labels, int m, int N, int k, int *out, int *perm_out, void *work, hipStream_t st) {
  SmallWork w(work, 1, 1, k);
  hipLaunchKernelGGL(identity_perm_kernel, dim3((k + 255) / 256), dim3(256), 0, st, w.perm, k);
  for (int i = 1; i < m; ++i) {
    hipLaunchKernelGGL(fill_int_kernel, dim3((k * k + 255) / 256), dim3(256), 0, st, w.T, k * k, 0);
    hipLaunchKernelGGL(contingency_kernel, dim3((N + 255) / 256), dim3(256), 0, st, labels, labels + (size_t)i * N, N, k, w.T);
    hipLaunchKernelGGL(greedy_match_kernel, dim3(1), dim3(1024), 0, st, w.T, k, w.perm + (size_t)i * k);
  }
  hipLaunchKernelGGL(vote_kernel, dim3((N + 255) / 256), dim3(256), 0, st, labels, w.perm, m, N, k, out);
  TAP_HIP(hipGetLastError());
  if (perm_out) TAP_HIP(hipMemcpyAsync(perm_out, w.perm, (size_t)m * k * sizeof(int), hipMemcpyDeviceToDevice, st));
  return QC_OK;
}

int check_work(const void *work, size_t have, size_t need) {
  if (!work) TAP_FAIL(QC_ERR_NULL, "work is NULL");
  if (!aligned16(work)) TAP_FAIL(QC_ERR_ALIGN, "work must be 16-byte aligned");
  if (have < need) TAP_FAIL(QC_ERR_WORKSPACE, "workspace of %zu bytes is too small (%zu needed)", have, need);
  return QC_OK;
}

}  // namespace

extern "C" {

int qc_tap_workspace_bytes(int N, int F, int n, int k, int kb, size_t *bytes_out) {
  if (!bytes_out) TAP_FAIL(QC_ERR_NULL, "bytes_out is NULL");
  TAP_RC(check_dims(N, F, n, k, kb));
  *bytes_out = ClusterWork(nullptr, N, F, n, k, kb).bytes;
  return QC_OK;
}

int qc_tap_profile_begin(void) {
  g_prof.on = true;
  g_prof.used = 0;
  return QC_OK;
}

int qc_tap_profile_end(float *sim_ms_out, int *launches_out) {
  if (!sim_ms_out || !launches_out) TAP_FAIL(QC_ERR_NULL, "an output pointer is NULL");
  if (!g_prof.on) TAP_FAIL(QC_ERR_STATE, "qc_tap_profile_begin was not called");
  g_prof.on = false;
  float total = 0.f;
  for (size_t i = 0; i < g_prof.used; ++i) {
    TAP_HIP(hipEventSynchronize(g_prof.ev[i].second));
    float ms = 0.f;
    TAP_HIP(hipEventElapsedTime(&ms, g_prof.ev[i].first, g_prof.ev[i].second));
    total += ms;
  }
  *sim_ms_out = total;
  *launches_out = (int)g_prof.used;
  return QC_OK;
}

int qc_tap_similarity(const float *X, const float *t, int N, int F, const int *idx, int n, float alpha, float *A,
                      float *d_r, float *d_c, void *work, size_t work_bytes, void *stream) {
  if (!X || !t || !idx || !A || !d_r || !d_c) TAP_FAIL(QC_ERR_NULL, "a required pointer is NULL");
  if (N < 1 || F < 1 || n < 1) TAP_FAIL(QC_ERR_SHAPE, "N, F, n must be positive");
  if (n > N) TAP_FAIL(QC_ERR_SHAPE, "n (%d) exceeds N (%d)", n, N);
  if ((long long)N * (n > F ? n : F) >= (1ll << 31)) TAP_FAIL(QC_ERR_UNSUPPORTED, "N * max(n, F) must be below 2^31");
  if (!(alpha >= 0.f && alpha <= 1.f)) TAP_FAIL(QC_ERR_RANGE, "alpha must lie in [0, 1]");
  if (!aligned16(X) || !aligned16(A)) TAP_FAIL(QC_ERR_ALIGN, "X and A must be 16-byte aligned");
  TAP_RC(check_work(work, work_bytes, SimWork(nullptr, N, F, n).bytes));
  return similarity_impl(X, t, N, F, idx, n, alpha, A, d_r, d_c, work, static_cast<hipStream_t>(stream));
}

int qc_tap_normalise(float *A, const float *d_r, const float *d_c, int N, int n, void *work, size_t work_bytes,
                     void *stream) {
  if (!A || !d_r || !d_c) TAP_FAIL(QC_ERR_NULL, "a required pointer is NULL");
  if (N < 1 || n < 1) TAP_FAIL(QC_ERR_SHAPE, "N and n must be positive");
  if ((long long)N * n >= (1ll << 31)) TAP_FAIL(QC_ERR_UNSUPPORTED, "N * n must be below 2^31");
  TAP_RC(check_work(work, work_bytes, SmallWork(nullptr, 1, 1, 1).bytes));
  return normalise_impl(A, d_r, d_c, N, n, work, static_cast<hipStream_t>(stream));
}

int qc_tap_embed(const float *L, int N, int n, int k, int kb, int iters, const float *q0, float *U, float *sigma,
                 void *work, size_t work_bytes, void *stream) {
  if (!L || !q0 || !U || !sigma) TAP_FAIL(QC_ERR_NULL, "a required pointer is NULL");
  TAP_RC(check_dims(N, 1, n, k, kb));
  if (iters < 0 || iters > 1000) TAP_FAIL(QC_ERR_RANGE, "iters must lie in [0, 1000]");
  if (!aligned16(L) || !aligned16(q0) || !aligned16(U)) TAP_FAIL(QC_ERR_ALIGN, "L, q0 and U must be 16-byte aligned");
  TAP_RC(check_work(work, work_bytes, EmbedWork(nullptr, N, n, k, kb).bytes));
  return embed_impl(L, N, n, k, kb, iters, q0, U, sigma, work, static_cast<hipStream_t>(stream));
}

int qc_tap_kmeans(const float *U, int N, int d, int k, const int *init_idx, int max_iter, int *labels, float *centres,
                  int *passes_out, void *work, size_t work_bytes, void *stream) {
  if (!U || !init_idx || !labels || !centres) TAP_FAIL(QC_ERR_NULL, "a required pointer is NULL");
  if (N < 1 || d < 1 || k < 1) TAP_FAIL(QC_ERR_SHAPE, "N, d, k must be positive");
  if (d > KB_MAX || k > KB_MAX) TAP_FAIL(QC_ERR_UNSUPPORTED, "d and k must be at most %d", KB_MAX);
  if ((long long)N * d >= (1ll << 31)) TAP_FAIL(QC_ERR_UNSUPPORTED, "N * d must be below 2^31");
  if (max_iter < 1) TAP_FAIL(QC_ERR_RANGE, "max_iter must be at least 1");
  TAP_RC(check_work(work, work_bytes, SmallWork(nullptr, N, d, k).bytes));
  return kmeans_impl(U, N, d, k, init_idx, max_iter, labels, centres, passes_out, work, static_cast<hipStream_t>(stream));
}

int qc_tap_aggregate(const int *labels, int m, int N, int k, int *out, int *perm_out, void *work, size_t work_bytes,
                     void *stream) {
  if (!labels || !out) TAP_FAIL(QC_ERR_NULL, "a required pointer is NULL");
  if (m < 1 || N < 1 || k < 1) TAP_FAIL(QC_ERR_SHAPE, "m, N, k must be positive");
  if (m > M_MAX) TAP_FAIL(QC_ERR_UNSUPPORTED, "at most %d label vectors", M_MAX);
  if (k > KB_MAX) TAP_FAIL(QC_ERR_UNSUPPORTED, "k must be at most %d", KB_MAX);
  if ((long long)m * N >= (1ll << 31)) TAP_FAIL(QC_ERR_UNSUPPORTED, "m * N must be below 2^31");
  TAP_RC(check_work(work, work_bytes, SmallWork(nullptr, 1, 1, k).bytes));
  return aggregate_impl(labels, m, N, k, out, perm_out, work, static_cast<hipStream_t>(stream));
}

int qc_tap_cluster(const float *X, const float *t, int N, int F, const int *subsamples, int m, int n, float alpha,
                   int k, int kb, int iters, const float *q0, const int *init_idx, int max_iter, int *labels_out,
                   int *per_labels, void *work, size_t work_bytes, void *stream) {
  if (!X || !t || !subsamples || !q0 || !init_idx || !labels_out || !per_labels)
    TAP_FAIL(QC_ERR_NULL, "a required pointer is NULL");
  TAP_RC(check_dims(N, F, n, k, kb));
  if (m < 1 || m > M_MAX) TAP_FAIL(QC_ERR_UNSUPPORTED, "m must lie in [1, %d]", M_MAX);
  if (!(alpha >= 0.f && alpha <= 1.f)) TAP_FAIL(QC_ERR_RANGE, "alpha must lie in [0, 1]");
  if (iters < 0 || iters > 1000) TAP_FAIL(QC_ERR_RANGE, "iters must lie in [0, 1000]");
  if (max_iter < 1) TAP_FAIL(QC_ERR_RANGE, "max_iter must be at least 1");
  if (!aligned16(X) || !aligned16(q0)) TAP_FAIL(QC_ERR_ALIGN, "X and q0 must be 16-byte aligned");
  const size_t per = (ClusterWork(nullptr, N, F, n, k, kb).bytes + 255) & ~size_t(255);
  TAP_RC(check_work(work, work_bytes, per));
  hipStream_t st = static_cast<hipStream_t>(stream);
  // as many subsamples at a time as the workspace holds (at most MAX_SLOTS): the first on the caller's stream, the
  // others on internal streams that start after the work already enqueued on the caller's stream
  int slots = (int)(work_bytes / per);
  if (slots > MAX_SLOTS) slots = MAX_SLOTS;
  if (slots > m) slots = m;
  hipStream_t ss[MAX_SLOTS] = {st, nullptr, nullptr};
  CallStreams cs;                                 // destroyed (after a wait on each stream) on every way out
  if (slots > 1) {
    TAP_HIP(hipEventCreateWithFlags(&cs.fork, hipEventDisableTiming));
    TAP_HIP(hipEventRecord(cs.fork, st));
    for (int j = 1; j < slots; ++j) {
      TAP_HIP(hipStreamCreateWithFlags(&cs.streams[j], hipStreamNonBlocking));
      TAP_HIP(hipStreamWaitEvent(cs.streams[j], cs.fork, 0));
      ss[j] = cs.streams[j];
    }
    for (int j = 0; j < slots; ++j) TAP_HIP(hipEventCreateWithFlags(&cs.chain[j], hipEventDisableTiming));
  }
  for (int i0 = 0; i0 < m; i0 += slots) {
    const int ns = m - i0 < slots ? m - i0 : slots;
    KmSlot km[MAX_SLOTS];
    for (int j = 0; j < ns; ++j) {
      ClusterWork w(static_cast<char *>(work) + (size_t)j * per, N, F, n, k, kb);
      const int i = i0 + j;
      hipLaunchKernelGGL(fill_int_kernel, dim3(1), dim3(256), 0, ss[j], w.flags, 64, 0);
      TAP_RC(similarity_impl(X, t, N, F, subsamples + (size_t)i * n, n, alpha, w.A, w.dr, w.dc, w.sub, ss[j], w.flags + 0,
                             j > 0 ? cs.chain[j - 1] : nullptr));
      TAP_RC(normalise_impl(w.A, w.dr, w.dc, N, n, w.sub, ss[j], w.flags + 1));
      TAP_RC(embed_impl(w.A, N, n, k, kb, iters, q0, w.U, w.sigma, w.sub, ss[j], w.flags + 2,
                        slots > 1 ? cs.chain[j] : nullptr));
      km[j] = KmSlot{w.U, init_idx + (size_t)i * k, per_labels + (size_t)i * N, w.centres, w.sub, ss[j], w.flags + 3, 0, false};
    }
    // the first pass of the k-means below runs on whatever the earlier stages left; the flags tell afterwards
    // whether that was meaningful (every kernel stays inside its buffers on any input)
    int rc = kmeans_multi(km, ns, N, k, k, max_iter);
    for (int j = 0; j < ns && rc == QC_OK; ++j) {
      ClusterWork w(static_cast<char *>(work) + (size_t)j * per, N, F, n, k, kb);
      int fl[4] = {0, 0, 0, 0};
      TAP_HIP(hipMemcpyAsync(fl, w.flags, sizeof(fl), hipMemcpyDeviceToHost, ss[j]));
      TAP_HIP(hipStreamSynchronize(ss[j]));
      if (fl[0]) { qc::set_error("a subsample index lies outside [0, %d)", N); rc = QC_ERR_RANGE; }
      else if (fl[1]) { qc::set_error("a degree of the similarity matrix is not positive and finite"); rc = QC_ERR_RANGE; }
      else if (fl[2]) { qc::set_error("the iteration block has no full rank (a zero start vector, or fewer than kb independent directions)"); rc = QC_ERR_RANGE; }
      else if (fl[3]) { qc::set_error("an initial-centre index lies outside [0, %d)", N); rc = QC_ERR_RANGE; }
    }
    if (rc != QC_OK) {
      for (int j = 0; j < slots; ++j) (void)hipStreamSynchronize(ss[j]);
      return rc;
    }
  }
  // every stream has drained (the k-means loop ends with a wait on each): the merge runs on the caller's stream
  TAP_RC(aggregate_impl(per_labels, m, N, k, labels_out, nullptr, work, st));
  TAP_HIP(hipStreamSynchronize(st));
  return QC_OK;
}

}  // extern "C"
