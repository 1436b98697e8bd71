// int8 x int8 -> int32 GEMM on the gfx950 matrix cores (v_mfma_i32_32x32x32_i8)
// with the dequantise / GELU+requantise / cache-store+gated-residual epilogues
// of the quantised linears of a DiT block.
//
//   acc[m, n] = sum_k A[m, k] * W[n, k]          A: activation codes, W: weight codes
//   v[m, n]   = a_s * w_s[n] * (acc - a_z * wsum[n]) + bias[n]
//
// Tiling: a workgroup of 4 or 8 wavefronts owns a BM x BN tile of the
// output and walks K in slabs of 128 bytes.  Both operands are K-contiguous, so
// a slab row is 8 sixteen-byte chunks.  Slabs are staged in LDS (rows padded by
// 16 bytes so the 128-bit fragment reads of 8 neighbouring rows fall in 8
// different bank groups), two LDS buffers.  Global loads run PF slabs ahead of
// the MFMAs through a rotating set of registers: memory latency on this part
// is a few slab-times, so one slab of prefetch leaves the matrix cores idle.
//
// MFMA operand layout (32x32x32 i8): lane l supplies 16 bytes of row (l % 32)
// of either operand for k-group (l / 32); the products pair byte j of group g
// of both operands, so any k order works as long as both use the same one.
// Result layout: register r of lane l is row (r/4)*8 + (l/32)*4 + r%4 of the
// first operand, column l % 32 of the second.  The fp32 epilogues put the
// activations first (a lane owns one output column n, 32 lanes write 128
// contiguous bytes of a row); the int8 epilogue puts the weights first (a lane
// owns one row m and four consecutive n per register group, packed to a dword,
// staged through LDS and written out as 16-byte chunks).
//
// Workgroup -> tile mapping is XCD-aware: hardware deals workgroups round-robin
// to the 8 XCDs, each with its own L2; the mapping gives every XCD a contiguous
// range of weight panels so that a panel is fetched into one L2 only.
#include <cstdlib>
#include <type_traits>

#include "qc_internal.h"

namespace qc {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef unsigned v2u __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));


constexpr int NUM_XCD = 8;
constexpr int GELU_FIX_CAP = 1024;      // queue of fc1 outputs decided again in float64, per tile

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

// tanh-GELU written as v * sigmoid(2u), u = sqrt(2/pi) (v + 0.044715 v^3):
// 0.5 v (1 + tanh u) = v / (1 + exp(-2u)); one exp2 and one reciprocal.
__device__ __forceinline__ float gelu_tanh(float v) {
  const float c1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;   // -2 sqrt(2/pi) log2(e)
  const float c2 = c1 * 0.044715f;
  const float t = v * fmaf(c2, v * v, c1);
  return v * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(t));
}
// the same divided by the quantiser step s: v / (s + s exp(-2u)), the step folded into the denominator
__device__ __forceinline__ float gelu_tanh_over(float v, float s) {
  const float c1 = -2.0f * 0.7978845608028654f * 1.4426950408889634f;
  const float c2 = c1 * 0.044715f;
  const float t = v * fmaf(c2, v * v, c1);
  return v * __builtin_amdgcn_rcpf(fmaf(s, __builtin_amdgcn_exp2f(t), s));
}

// Dequantised output of a quantised linear as it is stored: the float32 rounding of the float64 value
// (a_s * w_s[n]) * (acc - a_z * wsum[n]) + bias[n] (the product of the two scales is exact in float64; one float64
// multiplication, one float64 addition, one rounding to float32).  Stored tensors then carry no rounding of their own
// beyond the storage format, so the codes quantised from them further down do not depend on the order of operations here.
__device__ __forceinline__ float dequant_f32(double sc, int corr, double bs) {
  return (float)__dadd_rn(__dmul_rn(sc, (double)corr), bs);
}

// The fc1 epilogue's exact path for one output element: float64 from the integer accumulator to the GELU value, one
// rounding to float32, Eq. 1 with an IEEE division.  x / (1 + exp(-2u)) = 0.5 x (1 + tanh u).
__device__ __noinline__ int gelu_code_exact(int corr, float a_s, float w_s, float bias, float o_s, int o_z) {
  const double u = __dadd_rn(__dmul_rn((double)a_s * (double)w_s, (double)corr), (double)bias);
  const double k = 0.7978845608028654 * (u + 0.044715 * u * u * u);
  const float g = (float)(u / (1.0 + exp(-2.0 * k)));
  const float r = __builtin_rintf(g / o_s) + (float)o_z;
  return (int)fminf(fmaxf(r, -128.0f), 127.0f);
}

// Eq. 1 on signed codes with the quotient v / s refined to the correctly rounded
// value by one Newton step on the reciprocal estimate.
__device__ __forceinline__ int quant_code(float v, float s, float inv_s, float z) {
  float q = v * inv_s;
  q = fmaf(fmaf(-q, s, v), inv_s, q);
  float r = __builtin_rintf(q) + z;
  r = fminf(fmaxf(r, -128.0f), 127.0f);
  return (int)r;
}

// Epilogue of a tile: acc[i][j] is the 32 x 32 block (i along the rows m of the activations, j along the output
// columns n) of wavefront (wave / WN, wave % WN); for EPI_GELU_Q the weights were the first MFMA operand (register
// index runs along n), otherwise the activations were (register index runs along m).  smem: the workgroup's dynamic
// LDS, free for reuse (every wavefront is past its last fragment read).
// FAST: the launcher has checked that every tile is interior along m and lies in one batch element (and, for the QKV
// scatter, the alignment its staged path needs); the general paths are then not compiled into the kernel.
// RBF: the residual stream or the cache may be bfloat16 (read from the arguments); false: both are known to be float32.
template <int BM, int BN, int WM, int WN, int EPI, bool FAST = false, bool RBF = true>
__device__ __forceinline__ void gemm_epilogue(const GemmArgs &p, v16i (&acc)[BM / WM / 32][BN / WN / 32], unsigned char *smem,
                                              const int m0, const int n0, const int z) {
  constexpr int TM = BM / WM / 32, TN = BN / WN / 32, NT = 64 * WM * WN;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm0 = (wave / WN) * (BM / WM), wn0 = (wave % WN) * (BN / WN);
  const int ncover = p.sel_D ? 2 * p.sel_D : p.N;
  float a_s = p.a_scale;
  int a_z = p.a_zp;
  if (p.a_qp) {
    QParam q = p.a_qp[(long long)z * p.zs_qp];
    a_s = q.s;
    a_z = q.z;
  }
  const float *w_scale = p.w_scale + (long long)z * p.zs_vecN;
  const int32_t *wsum = p.wsum + (long long)z * p.zs_vecN;
  const float *bias = p.bias ? p.bias + (long long)z * p.zs_vecN : nullptr;

  if (EPI == EPI_GELU_Q) {
    // per-column constants into LDS: v = sc[n] * float(acc - zw[n]) + bs[n]
    float *c_sc = (float *)smem;
    int *c_zw = (int *)(smem + BN * 4);
    float *c_bs = (float *)(smem + BN * 8);
    unsigned char *stage = smem + BN * 12;             // [BM][BN + 16] codes
    constexpr int SROW = BN + 16;
    // Elements whose fast evaluation lands too close to a rounding boundary of Eq. 1 to be trusted are queued here and
    // decided again in float64 (gelu_code_exact): the codes are then those of exact arithmetic on the accumulators.
    int *fix_cnt = (int *)(stage + BM * SROW);
    int *fix_ent = fix_cnt + 4;                        // [GELU_FIX_CAP][4]: accumulator minus zero-point term, column, row
    if (tid == 0) *fix_cnt = 0;
    if (tid < BN) {
      const int n = n0 + tid;
      const bool ok = n < p.N;
      c_sc[tid] = ok ? a_s * w_scale[n] : 0.0f;
      c_zw[tid] = ok ? a_z * wsum[n] : 0;
      c_bs[tid] = (ok && bias) ? bias[n] : 0.0f;
    }
    __syncthreads();
    const QParam oq = *p.o_qp;
    // codes are formed as the paper's unsigned ones (zero point + 128, clamped to 0 .. 255, converted and packed by
    // one instruction each); the sign bit of the four bytes is flipped back when the word is stored
    const float o_s = oq.s, o_inv = 1.0f / oq.s, o_zu = (float)(oq.z + 128);
    // Bound of the fast path's error in units of the output step, as a multiple of |v| / s (|GELU(v)| <= |v|):
    // 1.5e-6 covers the float32 dequantisation (accumulators beyond 2^24 are rounded on conversion) and the exp2 /
    // reciprocal estimates with a margin of 2, 2e-7 the unrefined quotient gv * (1 / s); 2e-6 absolute covers the bias
    // rounding.  An element is in doubt when |q - rint(q)| + bound > 1/2.
    const float tol_v = 1.7e-6f * o_inv;
    const float doubt_at = 0.5f - 2e-6f;
    const int g = lane >> 5;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const int nl = wn0 + j * 32 + rg * 8 + g * 4;       // 4 consecutive columns of this lane
        const v4f sc = *(const v4f *)(c_sc + nl);
        const v4i zw = *(const v4i *)(c_zw + nl);
        const v4f bs = *(const v4f *)(c_bs + nl);
#pragma unroll
        for (int i = 0; i < TM; ++i) {
          unsigned w = 0;
          float dist[4];                                      // distance from the rounding boundary plus the error bound
          int corr[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // the large-M kernel's accumulators already carry the zero-point term
            corr[e] = FAST ? acc[i][j][rg * 4 + e] : acc[i][j][rg * 4 + e] - zw[e];
            const float v = fmaf(sc[e], (float)corr[e], bs[e]);
            const float q = gelu_tanh_over(v, o_s);
            const float r = __builtin_rintf(q);
            w = __builtin_amdgcn_cvt_pk_u8_f32(__builtin_amdgcn_fmed3f(r + o_zu, 0.0f, 255.0f), e, w);
            dist[e] = fmaf(tol_v, fabsf(v), fabsf(q - r));
          }
          w ^= 0x80808080u;
          // one comparison and one branch per four outputs; taken by a wavefront about once in a hundred times
          if (fmaxf(fmaxf(dist[0], dist[1]), fmaxf(dist[2], dist[3])) > doubt_at) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (dist[e] > doubt_at) {
                const int slot = atomicAdd(fix_cnt, 1);
                if (slot < GELU_FIX_CAP) {
                  fix_ent[slot * 4 + 0] = corr[e];
                  fix_ent[slot * 4 + 1] = nl + e;
                  fix_ent[slot * 4 + 2] = wm0 + i * 32 + (lane & 31);
                }
              }
          }
          *(unsigned *)(stage + (wm0 + i * 32 + (lane & 31)) * SROW + nl) = w;
        }
      }
    }
    __syncthreads();
    {
      const int nfix = min(*fix_cnt, GELU_FIX_CAP);
      for (int f = tid; f < nfix; f += NT) {
        const int corr = fix_ent[f * 4 + 0], nl = fix_ent[f * 4 + 1], row = fix_ent[f * 4 + 2];
        const int n = n0 + nl;
        if (n < p.N) stage[row * SROW + nl] = (unsigned char)gelu_code_exact(corr, a_s, w_scale[n], bias ? bias[n] : 0.0f, o_s, oq.z);
      }
      if (nfix) __syncthreads();
    }
    // coalesced write-out: 16-byte chunks, 8 lanes cover a 128-byte row segment
    constexpr int CH = BN / 16;
    for (int c = tid; c < BM * CH; c += NT) {
      const int r = c / CH, cc = (c % CH) * 16;
      const int m = m0 + r, n = n0 + cc;
      if (m >= p.M || n >= p.N) continue;
      int8_t *dst = p.q_out + (long long)m * p.ldq + n;
      if (n + 16 <= p.N) {
        // large launches: streaming stores (the tensor is far larger than the L2 and would only evict the operands)
        if (FAST) __builtin_nontemporal_store(*(const v4i *)(stage + r * SROW + cc), (v4i *)dst);
        else *(v4i *)dst = *(const v4i *)(stage + r * SROW + cc);
      } else {
        for (int e = 0; n + e < p.N; ++e) dst[e] = (int8_t)stage[r * SROW + cc + e];
      }
    }
    return;
  }

  if (EPI == EPI_QKV) {
    // float32 values scattered to the head-major layouts of the attention kernel: Q and K [B, H, T, hd], V transposed
    // and key-permuted [B, H, DP, Tp]; p.y, when set, also receives them row-major ([M, 3 D], for inspection)
    const int T = p.rows_per_batch, D = p.N / 3;
    const bool fast_t = (T % 4) == 0;
    const bool tile_one_batch = (T % BM) == 0;      // then every row of the tile belongs to batch element m0 / T
    const int b_tile = m0 / T;
    constexpr int HN = 128;                                   // the tile is handled in column halves of 128
    if (FAST || (BM == 128 && BN % HN == 0 && (BN / WN) <= HN && tile_one_batch && fast_t && m0 + BM <= p.M && D % HN == 0 &&
                 (p.hd & 3) == 0 && (p.Tp & 7) == 0)) {
      // Tile inside one batch element, every 128 columns inside one of Q, K, V: the values go through LDS (free after
      // the K loop) and leave as 16-byte stores along the contiguous direction of their layout (Q / K: features of a
      // token and head; V^T: tokens of a feature).
      const int tb = m0 - b_tile * T;                         // first token of the tile
#pragma unroll
      for (int hn = 0; hn < BN / HN; ++hn) {
        const int n0h = n0 + hn * HN;                         // first column of this half
        if (n0h >= p.N) break;
        const bool mine = wn0 / HN == hn;                     // this wavefront's columns lie in the half
        const int part = n0h / D;
        if (hn) __syncthreads();                              // the previous half has left the staging area
        float *stage = (float *)smem;
        constexpr int SR = HN + 4;                            // Q / K: floats per staged token row
        constexpr int VR = BM + 4;                            // V^T: floats per staged feature row
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (!mine) continue;
          const int nl = wn0 - hn * HN + j * 32 + (lane & 31);
          const double sc = (double)a_s * (double)w_scale[n0h + nl];
          const int zw = a_z * wsum[n0h + nl];
          const double bs = bias ? (double)bias[n0h + nl] : 0.0;
          // the optional row-major copy is not compiled into the large-M kernel (its launcher declines such launches)
          float *ycol = (!FAST && p.y) ? p.y + (long long)m0 * p.ldy + n0h + nl : nullptr;     // 32 lanes write 128 contiguous bytes
#pragma unroll
          for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
              const int ml = wm0 + i * 32 + rg * 8 + (lane >> 5) * 4;
              v4f v;
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                v[q] = dequant_f32(sc, acc[i][j][rg * 4 + q] - zw, bs);
                if (ycol) ycol[(unsigned)(ml + q) * (unsigned)p.ldy] = v[q];
              }
              if (part < 2) {
#pragma unroll
                for (int q = 0; q < 4; ++q) stage[(ml + q) * SR + nl] = v[q];
              } else {
                // four consecutive tokens stay together under the key permutation of the V^T rows
                *(v4f *)(stage + nl * VR + vt_pos(ml)) = v;
              }
            }
            if (TM * TN > 4) __builtin_amdgcn_sched_barrier(0);      // large register tiles: keep the live ranges of a block short
          }
        }
        __syncthreads();
        if (part < 2) {
          // thread -> four features cc .. cc + 3 (inside one head: heads start at multiples of hd, a multiple of 4) of
          // the rows cr, cr + NT / 32, ...
          const int cr = tid >> 5, cc = (tid & 31) * 4;
          const int nn = n0h - part * D + cc, h = nn / p.hd, e = nn - h * p.hd;
          float *dst = (part == 0 ? p.q32 : p.k32) +
                       ((unsigned)(b_tile * p.heads + h) * (unsigned)T + (unsigned)(tb + cr)) * (unsigned)p.hd + (unsigned)e;
#pragma unroll
          for (int q = 0; q < BM * 32 / NT; ++q) {
            const v4f v = *(const v4f *)(stage + (cr + q * (NT / 32)) * SR + cc);
            v4f *d = (v4f *)(dst + (unsigned)(q * (NT / 32)) * (unsigned)p.hd);
            if (FAST) __builtin_nontemporal_store(v, d);      // large launches: streaming stores
            else *d = v;
          }
        } else {
          // thread -> 4 consecutive token positions ch of the features fc, fc + NT / 32, ...
          const int fc = tid >> 5, ch = (tid & 31) * 4;
#pragma unroll
          for (int q = 0; q < HN * 32 / NT; ++q) {
            const int col = fc + q * (NT / 32);
            const int nn = n0h - 2 * D + col, h = nn / p.hd, e = nn - h * p.hd;
            const unsigned o = ((unsigned)(b_tile * p.heads + h) * (unsigned)p.DP + (unsigned)e) * (unsigned)p.Tp + (unsigned)(tb + ch);
            if (FAST) __builtin_nontemporal_store(*(const v4f *)(stage + col * VR + ch), (v4f *)(p.vt32 + o));
            else *(v4f *)(p.vt32 + o) = *(const v4f *)(stage + col * VR + ch);
          }
        }
      }
      return;
    }
    if (FAST) return;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = n0 + wn0 + j * 32 + (lane & 31);
      if (n >= p.N) continue;
      const double sc = (double)a_s * (double)w_scale[n];
      const int zw = a_z * wsum[n];
      const double bs = bias ? (double)bias[n] : 0.0;
      const int part = n / D, nn = n - part * D, h = nn / p.hd, e = nn - h * p.hd;
      float *dqk = part == 0 ? p.q32 : p.k32;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
          const int mb = m0 + wm0 + i * 32 + rg * 8 + (lane >> 5) * 4;   // 4 consecutive rows mb .. mb+3
          if (mb >= p.M) continue;
          v4f v;
#pragma unroll
          for (int q = 0; q < 4; ++q) v[q] = dequant_f32(sc, acc[i][j][rg * 4 + q] - zw, bs);
          const int b0 = tile_one_batch ? b_tile : mb / T, t0 = mb - b0 * T;
          if (part == 2 && fast_t && mb + 3 < p.M) {
            // T is a multiple of 4: the four rows are tokens t0 .. t0 + 3 of one batch element, contiguous in V^T
            *(v4f *)(p.vt32 + ((long long)(b0 * p.heads + h) * p.DP + e) * p.Tp + vt_pos(t0)) = v;
          } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              if (mb + q >= p.M) continue;
              int b = b0, t = t0 + q;
              while (t >= T) { t -= T; ++b; }
              if (part == 2) p.vt32[((long long)(b * p.heads + h) * p.DP + e) * p.Tp + vt_pos(t)] = v[q];
              else dqk[((long long)(b * p.heads + h) * T + t) * p.hd + e] = v[q];
            }
          }
          if (p.y) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
              if (mb + q < p.M) p.y[(long long)(mb + q) * p.ldy + n] = v[q];
          }
        }
      }
    }
    return;
  }

  if (EPI == EPI_RESID) {
    // read-modify-write of the residual stream: the loads of a batch of column blocks are all issued
    // before the first use, so the epilogue pays one memory round trip per batch instead of one per
    // register group; a batch is the whole tile when its values fit in registers beside the accumulators
    constexpr int JB = TM * TN <= 4 ? TN : 1, IB = TM * TN <= 4 ? TM : 1;
    const bool uniform_batch = (p.rows_per_batch % BM) == 0;
    const int b_uniform = m0 / p.rows_per_batch;
    const int x_bf16 = RBF ? p.x_bf16 : 0, cache_bf16 = RBF ? p.cache_bf16 : 0;
    if (FAST && RBF && (x_bf16 || cache_bf16) && p.N % 128 == 0) {
      // A bfloat16 stream or cache: 32 lanes of a wavefront cover only 64 bytes of a row, and 2-byte stores leave
      // every cache line half written.  The dequantised values go through LDS in column halves of 128 instead, and
      // every thread handles four adjacent columns of 16 rows: 8- or 16-byte loads and stores, whole lines per row.
      constexpr int HN = 128, SR = HN + 4, RQ = BM * 32 / NT;
      float *stage = (float *)smem;
      const int cr = tid >> 5, cc = (tid & 31) * 4;     // thread -> rows cr + (NT / 32) q, columns cc .. cc + 3 of a half
#pragma unroll
      for (int hn = 0; hn < BN / HN; ++hn) {
        const int n0h = n0 + hn * HN;
        if (n0h >= p.N) break;
        const bool mine = wn0 / HN == hn;               // this wavefront's columns lie in the half
        if (hn) __syncthreads();                        // the previous half has left the staging area
        const v4f gv = *(const v4f *)(p.gate + (long long)b_uniform * p.ld_gate + n0h + cc);
        const size_t ob4 = ((size_t)m0 * p.N + n0h + cc) >> 2;      // in groups of four elements
        const size_t row4 = (size_t)p.N >> 2;
        // a bfloat16 stream: the thread's 16 pieces of x (8 bytes each) are requested before the staging, which hides
        // their latency (a float32 stream would take twice the registers: its loads stay in the loop below)
        uint2 xraw[RQ];
        if (x_bf16) {
#pragma unroll
          for (int q = 0; q < RQ; ++q) xraw[q] = ((const uint2 *)p.x)[ob4 + (size_t)(cr + q * (NT / 32)) * row4];
        }
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (!mine) continue;
          const int nl = wn0 - hn * HN + j * 32 + (lane & 31);
          const double sc = (double)a_s * (double)w_scale[n0h + nl];
          const int zw = a_z * wsum[n0h + nl];
          const double bs = bias ? (double)bias[n0h + nl] : 0.0;
#pragma unroll
          for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r)
              stage[(wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * SR + nl] = dequant_f32(sc, acc[i][j][r] - zw, bs);
            __builtin_amdgcn_sched_barrier(0);          // one block's values live at a time
          }
        }
        __syncthreads();
#pragma unroll 4
        for (int q = 0; q < RQ; ++q) {
          const int row = cr + q * (NT / 32);
          const v4f v = *(const v4f *)(stage + row * SR + cc);
          const size_t o4 = ob4 + (size_t)row * row4;
          float4 xo;
          if (x_bf16) {
            xo = make_float4(__builtin_bit_cast(float, xraw[q].x << 16), __builtin_bit_cast(float, xraw[q].x & 0xFFFF0000u),
                             __builtin_bit_cast(float, xraw[q].y << 16), __builtin_bit_cast(float, xraw[q].y & 0xFFFF0000u));
          } else {
            xo = stream_load4(p.x, o4, 0);
          }
          stream_store4(p.cache_out, o4, make_float4(v.x, v.y, v.z, v.w), cache_bf16);
          stream_store4(p.x, o4, make_float4(fmaf(gv.x, v.x, xo.x), fmaf(gv.y, v.y, xo.y), fmaf(gv.z, v.z, xo.z), fmaf(gv.w, v.w, xo.w)),
                        x_bf16);
        }
      }
      return;
    }
    if (FAST) {
      // every row of the tile exists and belongs to batch element b_uniform; N is a multiple of 32, so a wavefront's
      // 32-column block lies inside the matrix or outside it as a whole.  Addresses are a wavefront-uniform row pointer
      // (scalar arithmetic) plus one 32-bit lane offset, and the loads of x of XB blocks (16 values per lane each: the
      // registers of the K loop's operand ring and fragments are free now) are issued before the first is used, so a
      // tile's epilogue pays TM x TN / XB memory round trips instead of TM x TN.
      constexpr int XB = (!RBF && TM % 2 == 0) ? 2 : 1;   // the bfloat16 variants have no registers to spare   // the bfloat16 variants have no registers to spare
      const int wv = __builtin_amdgcn_readfirstlane(wave);
      const int wm0u = (wv / WN) * (BM / WM), wn0u = (wv % WN) * (BN / WN);
      const unsigned loff = (unsigned)((lane >> 5) * 4) * (unsigned)p.N + (unsigned)(lane & 31);
      const size_t xsz = x_bf16 ? 2 : 4, csz = cache_bf16 ? 2 : 4;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int nb = n0 + wn0u + j * 32;
        if (nb >= p.N) continue;
        const int n = nb + (lane & 31);
        const double sc = (double)a_s * (double)w_scale[n];
        const int zw = a_z * wsum[n];
        const double bs = bias ? (double)bias[n] : 0.0;
        const float g = p.gate[(long long)b_uniform * p.ld_gate + n];
        const size_t e0 = (size_t)(m0 + wm0u) * p.N + nb;           // first element of the wavefront's block column
#pragma unroll
        for (int i0 = 0; i0 < TM; i0 += XB) {
          float xv[XB][16];
#pragma unroll
          for (int ii = 0; ii < XB; ++ii) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const size_t er = e0 + (size_t)((i0 + ii) * 32 + (r >> 2) * 8 + (r & 3)) * p.N;
              xv[ii][r] = stream_load((const char *)p.x + er * xsz, loff, x_bf16);
            }
          }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int ii = 0; ii < XB; ++ii) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const size_t er = e0 + (size_t)((i0 + ii) * 32 + (r >> 2) * 8 + (r & 3)) * p.N;
              const float v = dequant_f32(sc, acc[i0 + ii][j][r] - zw, bs);
              // the cached tensor is written once and read a step later: a streaming store keeps it out of the L2's way
              if (!RBF) __builtin_nontemporal_store(v, (float *)((char *)p.cache_out + er * csz) + loff);
              else stream_store((char *)p.cache_out + er * csz, loff, v, cache_bf16);
              stream_store((char *)p.x + er * xsz, loff, fmaf(g, v, xv[ii][r]), x_bf16);
            }
            __builtin_amdgcn_sched_barrier(0);                // one block's dequantised values live at a time
          }
        }
      }
      return;
    }
    const bool interior = uniform_batch && m0 + BM <= p.M && n0 + BN <= p.N;
#pragma unroll
    for (int j0 = 0; j0 < TN; j0 += JB)
#pragma unroll
      for (int i0 = 0; i0 < TM; i0 += IB) {
        float xv[JB][IB][16], gv[JB];
        double scv[JB], bsv[JB];
        int zwv[JB];
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
          const int n = min(n0 + wn0 + (j0 + jj) * 32 + (lane & 31), p.N - 1);
#pragma unroll
          for (int ii = 0; ii < IB; ++ii)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const int m = min(m0 + wm0 + (i0 + ii) * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3), p.M - 1);
              xv[jj][ii][r] = stream_load(p.x, (long long)m * p.N + n, x_bf16);
            }
          scv[jj] = (double)a_s * (double)w_scale[n];
          zwv[jj] = a_z * wsum[n];
          bsv[jj] = bias ? (double)bias[n] : 0.0;
          gv[jj] = p.gate[(long long)b_uniform * p.ld_gate + n];
        }
#pragma unroll
        for (int jj = 0; jj < JB; ++jj) {
          const int j = j0 + jj;
          const int n = n0 + wn0 + j * 32 + (lane & 31);
          if (interior) {
            // interior tile inside one batch element: no bounds checks, one gate per column
#pragma unroll
            for (int ii = 0; ii < IB; ++ii)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int i = i0 + ii;
                const float v = dequant_f32(scv[jj], acc[i][j][r] - zwv[jj], bsv[jj]);
                // 32-bit offset inside the tile's rows from one 64-bit base per column
                const long long ob = (long long)m0 * p.N + n;
                const unsigned o = (unsigned)(wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3)) * (unsigned)p.N;
                if (cache_bf16) ((unsigned short *)p.cache_out + ob)[o] = bf16_bits(v);
                else ((float *)p.cache_out + ob)[o] = v;
                stream_store(p.x, ob + o, fmaf(gv[jj], v, xv[jj][ii][r]), x_bf16);
              }
          } else {
            if (n >= p.N) continue;
#pragma unroll
            for (int ii = 0; ii < IB; ++ii)
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int i = i0 + ii;
                const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
                if (m >= p.M) continue;
                const float v = dequant_f32(scv[jj], acc[i][j][r] - zwv[jj], bsv[jj]);
                const long long o = (long long)m * p.N + n;
                if (cache_bf16) ((unsigned short *)p.cache_out)[o] = bf16_bits(v);
                else ((float *)p.cache_out)[o] = v;
                const float g = p.gate[(long long)(m / p.rows_per_batch) * p.ld_gate + n];
                stream_store(p.x, o, fmaf(g, v, xv[jj][ii][r]), x_bf16);
              }
          }
        }
        if (TM * TN > 4) __builtin_amdgcn_sched_barrier(0);      // large register tiles: one batch's values live at a time
      }
    return;
  }

#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int jl = n0 + wn0 + j * 32 + (lane & 31);
    if (jl >= ncover) continue;
    const int n = map_col(jl, p.sel_D);
    const double sc = (double)a_s * (double)w_scale[n];
    const int zw = a_z * wsum[n];
    const double bs = bias ? (double)bias[n] : 0.0;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm0 + i * 32 + (r >> 2) * 8 + (lane >> 5) * 4 + (r & 3);
        if (m >= p.M) continue;
        const int a = acc[i][j][r];
        float *y = p.y + (long long)z * p.zs_out;
        y[(long long)m * p.ldy + n] = dequant_f32(sc, a - zw, bs);
        if (p.acc_out) p.acc_out[(long long)m * p.N + n] = a;
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, int EPI, int TAG, bool W4, int PF, int BK, bool RBF>
__global__ __launch_bounds__(64 * WM * WN, (WM * WN == 4 && BM * BN <= 128 * 128) ? 2 : 1) void gemm_i8_kernel(GemmArgs p) {
  constexpr int WTM = BM / WM, WTN = BN / WN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int NT = 64 * WM * WN;            // threads per workgroup
  constexpr int LDS_ROW = BK + 16;            // padded slab row in LDS
  constexpr int CPR = BK / 16;                // 16-byte chunks per slab row
  constexpr int RP = NT / CPR;                // slab rows covered by one pass of the workgroup
  constexpr int PA = BM / RP, PB = BN / RP;   // 16-byte chunks per thread per slab
  static_assert(TM >= 1 && TN >= 1 && PA >= 1 && PB >= 1, "tile too small for the workgroup");
  extern __shared__ __align__(16) unsigned char smem[];
  unsigned char *sA = smem;
  unsigned char *sB = smem + 2 * BM * LDS_ROW;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int z = blockIdx.z;
  const int ncover = p.sel_D ? 2 * p.sel_D : p.N;
  const int tiles_m = (p.M + BM - 1) / BM;
  // XCD-aware order: workgroup b runs on XCD b % 8.  The 8 XCDs form an xm x xn
  // grid over the tile grid; each XCD owns a contiguous block of cm x cn tiles,
  // so an activation panel is fetched by xn L2s and a weight panel by xm L2s.
  const int tiles_n = (ncover + BN - 1) / BN;
  const int xm = p.xcd_m, xn = NUM_XCD / xm;
  const int cm = (tiles_m + xm - 1) / xm, cn = (tiles_n + xn - 1) / xn;
  const int xcd = blockIdx.x % NUM_XCD, local = blockIdx.x / NUM_XCD;
  const int tm = (xcd % xm) * cm + local % cm, tn = (xcd / xm) * cn + local / cm;
  if (tm >= tiles_m || tn >= tiles_n) return;
  const int m0 = tm * BM;
  const int n0 = tn * BN;
  const int wm0 = (wave / WN) * WTM, wn0 = (wave % WN) * WTN;

  const int8_t *A = p.A + (long long)z * p.zs_A;
  const unsigned char *W = (const unsigned char *)p.W + (long long)z * p.zs_W;   // byte stride
  const int w_row_bytes = W4 ? (p.K >> 1) : p.K;

  // Loads never branch: rows outside the matrix are clamped to the last row
  // (their products land in accumulators that are never stored) and the
  // chunks of a ragged last slab are clamped in k and zeroed by a select.
  const int lr = tid / CPR, lc = tid % CPR;   // slab row (per pass of RP rows) and chunk of this thread
  unsigned oa[PA], ob[PB];                  // byte offsets of this thread's chunk rows
#pragma unroll
  for (int i = 0; i < PA; ++i) oa[i] = (unsigned)min(m0 + lr + RP * i, p.M - 1) * (unsigned)p.lda;
#pragma unroll
  for (int i = 0; i < PB; ++i) ob[i] = (unsigned)map_col(min(n0 + lr + RP * i, ncover - 1), p.sel_D) * (unsigned)w_row_bytes;
  typedef typename std::conditional<W4, v2i, v4i>::type wload_t;
  v4i ra[PF][PA];
  wload_t rb[PF][PB];

  // The loaded values are not touched until store_slab, so that nothing waits
  // on a load right after issuing it.
  auto load_slab = [&](int s, int k0, bool ragged) {
    int k = k0 + lc * 16;
    if (ragged) k = min(k, p.K - 16);
#pragma unroll
    for (int i = 0; i < PA; ++i) ra[s][i] = *(const v4i *)(A + oa[i] + k);
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      if (W4) *(v2i *)&rb[s][i] = *(const v2i *)(W + ob[i] + (k >> 1));
      else *(v4i *)&rb[s][i] = *(const v4i *)(W + ob[i] + k);
    }
  };
  auto store_slab = [&](int s, int buf, bool zero) {   // zero: this thread's chunk lies beyond K
#pragma unroll
    for (int i = 0; i < PA; ++i)
      *(v4i *)(sA + (buf * BM + lr + RP * i) * LDS_ROW + lc * 16) = zero ? (v4i){0, 0, 0, 0} : ra[s][i];
#pragma unroll
    for (int i = 0; i < PB; ++i) {
      v4i v;
      if (W4) v = unpack_w4(*(v2i *)&rb[s][i]);
      else v = *(v4i *)&rb[s][i];
      *(v4i *)(sB + (buf * BN + lr + RP * i) * LDS_ROW + lc * 16) = zero ? (v4i){0, 0, 0, 0} : v;
    }
  };

  // the same, one quarter at a time (chunk c of the PA + PB chunks belongs to part c % NPART): lets the
  // steady-state step spread its memory instructions between the MFMA groups
  constexpr int NPART = BK / 32;
  auto load_part = [&](int s, int k0, int part) {
    const int k = k0 + lc * 16;
#pragma unroll
    for (int i = 0; i < PA; ++i)
      if (i % NPART == part) ra[s][i] = *(const v4i *)(A + oa[i] + k);
#pragma unroll
    for (int i = 0; i < PB; ++i)
      if ((PA + i) % NPART == part) {
        if (W4) *(v2i *)&rb[s][i] = *(const v2i *)(W + ob[i] + (k >> 1));
        else *(v4i *)&rb[s][i] = *(const v4i *)(W + ob[i] + k);
      }
  };
  auto store_part = [&](int s, int buf, int part) {
#pragma unroll
    for (int i = 0; i < PA; ++i)
      if (i % NPART == part) *(v4i *)(sA + (buf * BM + lr + RP * i) * LDS_ROW + lc * 16) = ra[s][i];
#pragma unroll
    for (int i = 0; i < PB; ++i)
      if ((PA + i) % NPART == part) {
        v4i v;
        if (W4) v = unpack_w4(*(v2i *)&rb[s][i]);
        else v = *(v4i *)&rb[s][i];
        *(v4i *)(sB + (buf * BN + lr + RP * i) * LDS_ROW + lc * 16) = v;
      }
  };

  v16i acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

  const int nk = (p.K + BK - 1) / BK;
  const bool k_ragged = (p.K % BK) != 0;
  const int frow = lane & 31, fk = (lane >> 5) * 16;

  auto compute = [&](int cur) {
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
        for (int j = 0; j < TN; ++j) {
          if (EPI == EPI_GELU_Q)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[j], fa[i], acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[i], fb[j], acc[i][j], 0, 0, 0);
        }
    }
  };

  // One steady-state step, software-pipelined inside the wavefront.  LDS reads have a latency of a few
  // hundred cycles and a wavefront is alone on its SIMD when the launch has few workgroups, so a whole
  // slab of fragments (all NPART k-groups) is in flight at once: the reads of the next slab are issued
  // right after the barrier that publishes it, in front of the last MFMA group of the current slab, and a
  // quarter of the next slab's LDS stores and of the global loads PF slabs ahead is issued behind each
  // MFMA group, so that LDS and memory instructions execute under the matrix-core time.
  constexpr bool DEEP = TM * TN <= 4;          // a slab of fragments fits beside the accumulators
  v4i fa[DEEP ? NPART : 1][TM], fb[DEEP ? NPART : 1][TN];
  auto read_group = [&](int buf, int kk) {
    const unsigned char *a_base = sA + (buf * BM + wm0 + frow) * LDS_ROW + fk + kk * 32;
    const unsigned char *b_base = sB + (buf * BN + wn0 + frow) * LDS_ROW + fk + kk * 32;
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[DEEP ? kk : 0][i] = *(const v4i *)(a_base + i * 32 * LDS_ROW);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[DEEP ? kk : 0][j] = *(const v4i *)(b_base + j * 32 * LDS_ROW);
  };
  auto mfma_group = [&](int kk) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int g = DEEP ? kk : 0;
        if (EPI == EPI_GELU_Q)
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fb[g][j], fa[g][i], acc[i][j], 0, 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[g][i], fb[g][j], acc[i][j], 0, 0, 0);
      }
  };
  // precondition: the fragment reads of slab kt (buffer kt & 1) have been issued
  auto step = [&](int s, int kt) {
    const int cur = kt & 1;
#pragma unroll
    for (int kk = 0; kk < NPART; ++kk) {
      if (kk + 1 < NPART) {
        __builtin_amdgcn_sched_barrier(0);
        mfma_group(kk);
      }
      __builtin_amdgcn_sched_barrier(0);
      store_part((s + 1) % PF, cur ^ 1, kk);
      load_part(s, (kt + PF) * BK, kk);
    }
    __builtin_amdgcn_sched_barrier(0);
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk + 1 < NPART; ++kk) read_group(cur ^ 1, kk);
    __builtin_amdgcn_sched_barrier(0);
    mfma_group(NPART - 1);
    __builtin_amdgcn_sched_barrier(0);
    read_group(cur ^ 1, NPART - 1);
    __builtin_amdgcn_sched_barrier(0);
  };

  // Shallow variant for tiles whose accumulators leave no room for a slab of fragments: the fragments of
  // k-group kk+1 are read while the MFMAs of group kk run.
  auto step_shallow = [&](int s, int kt) {
    const int cur = kt & 1;
    const unsigned char *a_base = sA + (cur * BM + wm0 + frow) * LDS_ROW + fk;
    const unsigned char *b_base = sB + (cur * BN + wn0 + frow) * LDS_ROW + fk;
    v4i ga[2][TM], gb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) ga[0][i] = *(const v4i *)(a_base + i * 32 * LDS_ROW);
#pragma unroll
    for (int j = 0; j < TN; ++j) gb[0][j] = *(const v4i *)(b_base + j * 32 * LDS_ROW);
#pragma unroll
    for (int kk = 0; kk < NPART; ++kk) {
      if (kk + 1 < NPART) {
#pragma unroll
        for (int i = 0; i < TM; ++i) ga[(kk + 1) & 1][i] = *(const v4i *)(a_base + i * 32 * LDS_ROW + (kk + 1) * 32);
#pragma unroll
        for (int j = 0; j < TN; ++j) gb[(kk + 1) & 1][j] = *(const v4i *)(b_base + j * 32 * LDS_ROW + (kk + 1) * 32);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) {
          if (EPI == EPI_GELU_Q)
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(gb[kk & 1][j], ga[kk & 1][i], acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ga[kk & 1][i], gb[kk & 1][j], acc[i][j], 0, 0, 0);
        }
      __builtin_amdgcn_sched_barrier(0);
      store_part((s + 1) % PF, cur ^ 1, kk);
      load_part(s, (kt + PF) * BK, kk);
      __builtin_amdgcn_sched_barrier(0);
    }
    __syncthreads();
  };

  // prologue: PF slabs in flight, slab 0 into LDS
#pragma unroll
  for (int s = 0; s < PF; ++s)
    if (s < nk) load_slab(s, s * BK, k_ragged && s == nk - 1);
  store_slab(0, 0, k_ragged && nk == 1 && lc * 16 >= p.K);
  __syncthreads();
  // main loop, unrolled by PF so that the register sets rotate with static indices:
  // at step kt LDS[kt & 1] holds slab kt, registers hold slabs kt+1 .. kt+PF-1.
  // Steady state is straight-line code (every step loads, computes, stores) so
  // that the wait before a store only covers the one slab it needs; the last
  // few steps run in a conditional tail.
  int kb = 0;
  const int nk_steady = k_ragged ? nk - 1 : nk;      // the ragged last slab is loaded by the tail (clamped, zero-filled)
  if (DEEP && 2 * PF - 1 < nk_steady) {
#pragma unroll
    for (int kk = 0; kk < NPART; ++kk) read_group(0, kk);
  }
  for (; kb + 2 * PF - 1 < nk_steady; kb += PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      if (DEEP) step(s, kb + s);
      else step_shallow(s, kb + s);
    }
  }
  for (; kb < nk; kb += PF) {
#pragma unroll
    for (int s = 0; s < PF; ++s) {
      const int kt = kb + s;
      if (kt < nk) {
        if (kt + PF < nk) load_slab(s, (kt + PF) * BK, k_ragged && kt + PF == nk - 1);
        if (kt + 1 < nk) store_slab((s + 1) % PF, (kt + 1) & 1, k_ragged && kt + 2 == nk && (kt + 1) * BK + lc * 16 >= p.K);
        compute(kt & 1);
        __syncthreads();
      }
    }
  }

  gemm_epilogue<BM, BN, WM, WN, EPI, false, RBF>(p, acc, smem, m0, n0, z);
}

// ---------------------------------------------------------------------------------------------------------------
// Large-M kernel.  At M of several thousand rows the tile loop above is bound by LDS traffic (its writes run at a
// quarter of the read rate) and by the 64 bytes per clock a compute unit can pull through its vector memory path,
// so this kernel moves fewer bytes through both:
//   * tile 128 (M) x 256 (N), four wavefronts side by side along N, each 128 x 64 (4 x 2 blocks of 32 x 32: one LDS
//     fragment read feeds two MFMAs, one weight fragment four), two workgroups per compute unit so that one tile's
//     prologue and epilogue run under the other's main loop;
//   * weights never touch LDS: they are stored a second time in MFMA fragment order (fragment (n / 32, k / 32) =
//     64 lanes x 16 bytes, lane l = row n % 32 = l % 32, bytes 16 (l / 32) .. of the 32 k values; packed nibbles:
//     8 bytes per lane) and each wavefront streams the fragments of its own 64 columns straight into a ring of
//     registers, four k-groups deep (slots 2 par, 2 par + 1 for the two k-groups of a slab of parity par);
//   * activations go global -> registers -> LDS in slabs of 64 bytes of K (a thread moves two 16-byte chunks per
//     slab), two slabs in flight in registers, three slab buffers in LDS.  A slab row is 64 bytes, its four 16-byte
//     chunks XOR-swizzled with bits 2..3 of the row so that the fragment reads (32 consecutive rows, one chunk) are
//     free of bank conflicts;
//   * one barrier per slab, between its two k-groups: slab kt + 1 is written to LDS during the first k-group of slab
//     kt and read after that barrier; its buffer was last read in slab kt - 2, two barriers ago;
//   * one memory instruction is issued behind each MFMA (pinned with scheduling barriers), so a wavefront keeps its
//     matrix pipe fed while its loads, LDS writes and fragment reads are in flight.
// Every global load here is an ordinary register load issued through inline assembly (the compiler neither sees nor
// counts them); register loads complete in the order they were issued, so each wait on the vector memory counter below
// is the number of loads issued after the one it is for.  Per slab the order is: two activation loads (slab kt + 3),
// two ring loads (k-group 2 kt + 4), [barrier], two ring loads (k-group 2 kt + 5).
// (A variant that sent the activations straight to LDS (global_load_lds_dwordx4) was measured first: those loads and
// register loads share the counter but complete out of order with respect to each other, so counted waits gave wrong
// fragments on some boxes, and draining the counter before every barrier cost 8 % against this version.)
#define QC_WAIT_VM(n) asm volatile("s_waitcnt vmcnt(" #n ")" ::: "memory")
// the same, tied to registers that become valid with it: their uses cannot be moved above the wait
#define QC_WAIT_VM_FOR2(n, r0, r1) asm volatile("s_waitcnt vmcnt(" #n ")" : "+v"(r0), "+v"(r1)::"memory")
#define QC_WAIT_VM_FOR4(n, r0, r1, r2, r3) asm volatile("s_waitcnt vmcnt(" #n ")" : "+v"(r0), "+v"(r1), "+v"(r2), "+v"(r3)::"memory")
// all LDS writes of this wavefront done, then the workgroup barrier
#define QC_LDS_DONE_BARRIER asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory")

template <int EPI, int TAG, bool W4, bool RBF>
__global__ __launch_bounds__(256, 2) void gemm_i8_big_kernel(GemmArgs p) {
  constexpr int BM = 128, BN = 256, WM = 1, WN = 4, TM = 4, TN = 2, BK = 64;
  constexpr int RB = 4, NB = 3, NS = 2;           // ring depth (k-groups), LDS slab buffers, slabs in flight in registers
  constexpr int SLAB = BM * BK;
  extern __shared__ __align__(16) unsigned char smem[];

  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  // Tile order: XCD x (= workgroup id mod 8) owns a contiguous range of the order "GM tile rows at a time, column by
  // column", GM chosen by the launcher so that the column tiles of a group of rows are resident on the XCD at the same
  // time, walk K in step and share the group's activation slabs through the XCD's L2.
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  const int per_xcd = (gridDim.x + 7) >> 3;
  const int t = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
  if (t >= tiles_m * tiles_n) return;
  const int GM = p.group_m;
  const int grp = t / (GM * tiles_n), gm0 = grp * GM, gsz = min(GM, tiles_m - gm0), rr = t - grp * GM * tiles_n;
  const int tn = rr / gsz, tm = gm0 + rr % gsz;
  const int m0 = __builtin_amdgcn_readfirstlane(tm * BM), n0 = __builtin_amdgcn_readfirstlane(tn * BN);   // the divisions above run on the vector ALU
  const int wn0 = wave * (TN * 32);

  // activations: load i of thread tid covers row 64 i + tid / 4, 16-byte chunk tid % 4 of a slab and is written to
  // LDS at the swizzled position of that chunk.  Rows beyond M re-read row M - 1.
  unsigned aoff[2], lpos[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = i * 64 + (tid >> 2), c = tid & 3;
    aoff[i] = (unsigned)(min(m0 + row, p.M - 1) - m0) * (unsigned)p.lda + c * 16;
    lpos[i] = row * BK + ((c ^ ((row >> 2) & 3)) * 16);
  }
  const int8_t *abase = p.A + (size_t)m0 * p.lda;
  const int nk = p.K / BK, ng = p.K / 32;
  v4i ra[NS][2];
  auto load_a = [&](int q, int kt, int i) {       // slabs past the end re-read the last one (never used)
    asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(ra[q][i]) : "v"(aoff[i]), "s"(abase + min(kt, nk - 1) * BK) : "memory");
  };
  auto write_a = [&](int q, int kt, int i) { *(v4i *)(smem + (kt % NB) * SLAB + lpos[i]) = ra[q][i]; };

  // weight fragment streams of this wavefront: n-blocks (n0 + wn0) / 32 + j (blocks past N re-read the last block)
  constexpr int FRAG = W4 ? 512 : 1024;           // bytes per fragment
  typedef typename std::conditional<W4, v2i, v4i>::type wfrag_t;
  const int nblocks = p.N / 32;
  const int8_t *sb[TN];
#pragma unroll
  for (int j = 0; j < TN; ++j) sb[j] = (const int8_t *)p.Wt + (size_t)min((n0 + wn0) / 32 + j, nblocks - 1) * ng * FRAG;
  const unsigned lane_off = lane * (W4 ? 8 : 16);
  wfrag_t bq[RB][TN];
  auto load_ring = [&](int slot, int g) {         // groups past the end re-read the last one (never used)
    const size_t go = (size_t)min(g, ng - 1) * FRAG;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if (W4) asm volatile("global_load_dwordx2 %0, %1, %2" : "=v"(bq[slot][j]) : "v"(lane_off), "s"(sb[j] + go) : "memory");
      else asm volatile("global_load_dwordx4 %0, %1, %2" : "=v"(bq[slot][j]) : "v"(lane_off), "s"(sb[j] + go) : "memory");
    }
  };

  v16i acc[TM][TN];
  if constexpr (EPI == EPI_GELU_Q) {
    // the accumulators start at minus the zero-point term a_z * wsum[n] of their column (the weights are the first
    // MFMA operand here: register 4 rg + e of block j is column 32 j + 8 rg + 4 (lane / 32) + e), so the epilogue
    // finds acc - a_z * wsum[n] ready; the loads complete under the prologue's wait for the first slabs
    const int a_z = p.a_qp ? p.a_qp[0].z : p.a_zp;
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int rg = 0; rg < 4; ++rg) {
        const v4i ws = *(const v4i *)(p.wsum + min(n0 + wn0 + j * 32 + rg * 8 + (lane >> 5) * 4, p.N - 4));
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int e = 0; e < 4; ++e) acc[i][j][rg * 4 + e] = -(a_z * ws[e]);
      }
  } else {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][j][q] = 0;
  }

  const int frow = lane & 31, fsw = (frow >> 2) & 3;
  v4i fa[2][TM];
  auto read_frag = [&](int f, int kt, int kg, int i) {
    fa[f][i] = *(const v4i *)(smem + (kt % NB) * SLAB + frow * BK + ((((lane >> 5) + 2 * kg) ^ fsw) * 16) + i * 32 * BK);
  };
  v4i wf[TN];
  auto unpack_ring = [&](int slot) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      if constexpr (W4) wf[j] = unpack_w4(bq[slot][j]);
      else wf[j] = bq[slot][j];
    }
  };
  auto mfma = [&](int f, int i, int j) {
    if (EPI == EPI_GELU_Q) acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(wf[j], fa[f][i], acc[i][j], 0, 0, 0);
    else acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(fa[f][i], wf[j], acc[i][j], 0, 0, 0);
  };
#define QC_SB __builtin_amdgcn_sched_barrier(0)

  // prologue: slab 0 -> LDS, slabs 1 and 2 -> the two register sets, ring groups 0 .. 3
  load_a(0, 0, 0); load_a(0, 0, 1);
  load_a(1, 1, 0); load_a(1, 1, 1);
#pragma unroll
  for (int g = 0; g < RB; ++g) load_ring(g, g);
  QC_SB;
  QC_WAIT_VM_FOR4(0, ra[0][0], ra[0][1], ra[1][0], ra[1][1]);
  write_a(0, 0, 0); write_a(0, 0, 1);
  QC_SB;
  load_a(0, 2, 0); load_a(0, 2, 1);
  QC_LDS_DONE_BARRIER;
#pragma unroll
  for (int i = 0; i < TM; ++i) read_frag(0, 0, 0, i);
  QC_SB;

  // Slab kt = k-groups 2 kt and 2 kt + 1, ring slots 2 par and 2 par + 1 (par = kt % 2), register set q = (kt + 1) % 2
  // holds slab kt + 1.  On entry: slab kt is in LDS and published; fa[0] holds (or awaits) the fragments of (kt,
  // group 0); ring groups up to 2 kt + 3 and activation slabs up to kt + 2 are requested.
  // Loads issued after the one a wait is for:
  //   top of the slab, for ring group 2 kt and for slab kt + 1 in registers (both requested in the first half of slab
  //   kt - 2, the activations first): ring group 2 kt - 1 ... (2) and the six loads of slab kt - 1                 = 8
  //   (slab 1 needs the prologue's load of slab 2, which has only the six loads of slab 0 behind it:                 6)
  //   after the barrier, for ring group 2 kt + 1 (requested at the end of slab kt - 2): six loads of slab kt - 1 and
  //   the four of this slab's first half                                                                          = 10
  static_assert(RB == 4 && NB == 3 && NS == 2 && TM == 4 && TN == 2, "waits and slots below are written for this depth");
  auto slab = [&](int kt, int par, auto first) {
    const int q = (kt + 1) % NS;
    if constexpr (decltype(first)::value) QC_WAIT_VM_FOR4(6, bq[2 * par][0], bq[2 * par][1], ra[q][0], ra[q][1]);
    else QC_WAIT_VM_FOR4(8, bq[2 * par][0], bq[2 * par][1], ra[q][0], ra[q][1]);
    unpack_ring(2 * par);
    QC_SB;
    mfma(0, 0, 0); write_a(q, kt + 1, 0); QC_SB;
    mfma(0, 0, 1); write_a(q, kt + 1, 1); QC_SB;
    mfma(0, 1, 0); read_frag(1, kt, 1, 0); QC_SB;
    mfma(0, 1, 1); read_frag(1, kt, 1, 1); QC_SB;
    mfma(0, 2, 0); read_frag(1, kt, 1, 2); QC_SB;
    mfma(0, 2, 1); read_frag(1, kt, 1, 3); QC_SB;
    mfma(0, 3, 0); load_a(q, kt + 3, 0); QC_SB;
    mfma(0, 3, 1); load_a(q, kt + 3, 1); QC_SB;
    load_ring(2 * par, 2 * kt + 4);
    QC_SB;
    QC_LDS_DONE_BARRIER;
    QC_WAIT_VM_FOR2(10, bq[2 * par + 1][0], bq[2 * par + 1][1]);
    unpack_ring(2 * par + 1);
    QC_SB;
    mfma(1, 0, 0); QC_SB;
    mfma(1, 0, 1); QC_SB;
    mfma(1, 1, 0); QC_SB;
    mfma(1, 1, 1); QC_SB;
    mfma(1, 2, 0); read_frag(0, kt + 1, 0, 0); QC_SB;
    mfma(1, 2, 1); read_frag(0, kt + 1, 0, 1); QC_SB;
    mfma(1, 3, 0); read_frag(0, kt + 1, 0, 2); QC_SB;
    mfma(1, 3, 1); read_frag(0, kt + 1, 0, 3); QC_SB;
    load_ring(2 * par + 1, 2 * kt + 5);
    QC_SB;
  };
  // K is a multiple of 128 (checked by the launcher): an even number of slabs, at least two
  slab(0, 0, std::false_type());
  slab(1, 1, std::true_type());
  for (int kt = 2; kt + 2 <= nk; kt += 2) {
    slab(kt, 0, std::false_type());
    slab(kt + 1, 1, std::false_type());
  }
#undef QC_SB
  // the loads that ran past the end (clamped addresses) must have landed before registers are reused, and every
  // wavefront must be past its last fragment read before the epilogue reuses LDS
  QC_WAIT_VM(0);
  __builtin_amdgcn_sched_barrier(0);
  __syncthreads();
  gemm_epilogue<BM, BN, WM, WN, EPI, true, RBF>(p, acc, smem, m0, n0, 0);
}

constexpr int BIG_SMEM_LOOP = 3 * 128 * 64;
constexpr int BIG_SMEM_STAGE = 128 * (128 + 4) * 4;                      // one staged column half, float32 (QKV scatter, residual)
constexpr int BIG_SMEM_GELU = 256 * 12 + 128 * (256 + 16) + 16 + GELU_FIX_CAP * 16;

template <int EPI, int TAG, bool W4, bool RBF>
static hipError_t launch_big_fmt(const GemmArgs &a, hipStream_t st) {
  constexpr int smem_epi = EPI == EPI_GELU_Q ? BIG_SMEM_GELU : BIG_SMEM_STAGE;
  constexpr int smem = smem_epi > BIG_SMEM_LOOP ? smem_epi : BIG_SMEM_LOOP;
  static_assert(2 * smem <= 160 * 1024, "two workgroups per compute unit");
  static bool attr_set = false;
  auto kern = gemm_i8_big_kernel<EPI, TAG, W4, RBF>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tiles = ((a.M + 127) / 128) * ((a.N + 255) / 256);
  GemmArgs b = a;
  {
    // tile rows per group: every column tile of a group resident on its XCD at once (64 workgroup slots), at most 4
    // rows (measured on M = 32768: 4 rows beat 16 by 2 - 9 % on the four linears of DiT-XL/2, 1 - 2 rows lose again)
    const int tiles_n = (a.N + 255) / 256, fit = 64 / tiles_n;
    b.group_m = fit < 1 ? 1 : (fit > 4 ? 4 : fit);
  }
  hipLaunchKernelGGL(kern, dim3(((tiles + 7) / 8) * 8), dim3(256), smem, st, b);
  return hipGetLastError();
}

// the residual epilogue is compiled twice: for float32 stream and cache, and for the bfloat16 variants of either
template <int EPI, int TAG, bool W4>
static hipError_t launch_big(const GemmArgs &a, hipStream_t st) {
  if (EPI == EPI_RESID && (a.x_bf16 || a.cache_bf16)) return launch_big_fmt<EPI, TAG, W4, true>(a, st);
  return launch_big_fmt<EPI, TAG, W4, false>(a, st);
}

// The large-M kernel takes over when the weights exist in fragment order, the shape fits its loop (K a multiple of
// 128, N of 32, 16-byte aligned rows), every 128-row tile is whole and inside one batch element (its epilogues are
// compiled without the general paths) and the launch has enough 128 x 256 tiles for it to pay.
static bool use_big(const GemmArgs &a, int epi, int nz) {
  if (!a.Wt || nz != 1 || a.sel_D || a.acc_out) return false;
  if (a.K % 128 || a.N % 32 || a.lda % 16 || a.M % 128) return false;
  if (epi == EPI_RESID && a.rows_per_batch % 128) return false;
  if (epi == EPI_QKV && (a.y || a.rows_per_batch % 128 || (a.N / 3) % 128 || a.hd % 4 || a.Tp % 8)) return false;
  const long long tiles = (long long)((a.M + 127) / 128) * ((a.N + 255) / 256);
  // measured alone on the chip (DiT-XL/2 shapes): 160 tiles (proj / fc2 at M = 4096) run 20 % faster here than in the
  // tile kernel, 224 - 288 tiles (QKV / fc1 at M = 2048) 0 - 10 % faster, 112 - 144 tiles (M = 1024) 3 - 15 % slower,
  // 80 tiles (proj / fc2 at M = 2048) 15 - 25 % slower
  return tiles >= 150;
}

template <int BM, int BN, int WM, int WN, int EPI, int TAG, bool W4, int PF, int BK = 128, bool RBF = false>
static hipError_t launch_cfg(const GemmArgs &a, int nz, hipStream_t st) {
  // the residual epilogue is compiled for float32 stream and cache, and once more for the bfloat16 variants of either
  if constexpr (EPI == EPI_RESID && !RBF) {
    if (a.x_bf16 || a.cache_bf16) return launch_cfg<BM, BN, WM, WN, EPI, TAG, W4, PF, BK, true>(a, nz, st);
  }
  constexpr int smem_loop = 2 * (BM + BN) * (BK + 16);
  constexpr int smem_epi = BN * 12 + BM * (BN + 16) + 16 + GELU_FIX_CAP * 16;
  constexpr int smem = smem_loop > smem_epi ? smem_loop : smem_epi;
  static bool attr_set = false;
  auto kern = gemm_i8_kernel<BM, BN, WM, WN, EPI, TAG, W4, PF, BK, RBF>;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int ncover = a.sel_D ? 2 * a.sel_D : a.N;
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (ncover + BN - 1) / BN;
  // pick the XCD grid that moves the fewest bytes into the L2s, weighted by load imbalance
  const double bytes_a = (double)a.M * a.K, bytes_w = (double)ncover * a.K * (W4 ? 0.5 : 1.0);
  int best_xm = 1;
  double best = 1e300;
  for (int xm = 1; xm <= NUM_XCD; xm *= 2) {
    const int xn = NUM_XCD / xm;
    const int cm = (tiles_m + xm - 1) / xm, cn = (tiles_n + xn - 1) / xn;
    const double cost = (xn * bytes_a + xm * bytes_w) * ((double)cm * cn * NUM_XCD / ((double)tiles_m * tiles_n));
    if (cost < best) { best = cost; best_xm = xm; }
  }
  GemmArgs b = a;
  b.xcd_m = best_xm;
  const int cm = (tiles_m + best_xm - 1) / best_xm, cn = (tiles_n + NUM_XCD / best_xm - 1) / (NUM_XCD / best_xm);
  const int grid = NUM_XCD * cm * cn;
  hipLaunchKernelGGL(kern, dim3(grid, 1, nz), dim3(64 * WM * WN), smem, st, b);
  return hipGetLastError();
}

template <int EPI, int TAG, bool W4>
static hipError_t launch_shape(const GemmArgs &a, int nz, hipStream_t st) {
  if constexpr (EPI != EPI_F32) {
    if (use_big(a, EPI, nz)) return launch_big<EPI, TAG, W4>(a, st);
  }
  if (a.M <= 32) return launch_cfg<32, 128, 1, 4, EPI, TAG, W4, 3>(a, nz, st);
  if (a.M <= 64) return launch_cfg<64, 128, 2, 2, EPI, TAG, W4, 3>(a, nz, st);
  // Fewer tiles than compute units: a workgroup is alone on its CU and a single wavefront per SIMD cannot
  // keep the LDS and memory pipes busy (they are issue-bound per wavefront), so the tile is shared by 8.
  // The residual epilogue keeps a tile of x in registers, which would leave the 4-wavefront variant one
  // workgroup per CU: it always runs on 8.
  // Inside a block the QKV product runs beside the other sub-batch's kernels: beyond half a chip of tiles it takes
  // the 4-wavefront variant, whose workgroups share a compute unit with the other stream's instead of queueing for a
  // free one (measured on the benchmark's sub-batches, 216 tiles: +1.8 % on the whole pass although the launch itself
  // takes 5 % longer).
  const int n_tiles = ((a.M + 127) / 128) * (((a.sel_D ? 2 * a.sel_D : a.N) + 127) / 128);
  if (EPI == EPI_RESID || n_tiles <= (EPI == EPI_QKV ? 128 : 256))
    return launch_cfg<128, 128, 2, 4, EPI, TAG, W4, 3>(a, nz, st);
  // Otherwise 4 wavefronts per tile and two workgroups per compute unit.
  return launch_cfg<128, 128, 2, 2, EPI, TAG, W4, 3>(a, nz, st);
}

template <int EPI, int TAG>
static hipError_t launch_epi(const GemmArgs &a, int nz, hipStream_t st) {
  return a.w4 ? launch_shape<EPI, TAG, true>(a, nz, st) : launch_shape<EPI, TAG, false>(a, nz, st);
}

// `site` only names the instantiation (so that profiles tell the linears apart).
hipError_t launch_gemm(const GemmArgs &a, int epi, int nz, hipStream_t st, int site) {
  if (epi == EPI_GELU_Q) return launch_epi<EPI_GELU_Q, QC_SITE_FC1>(a, nz, st);
  if (epi == EPI_RESID)
    return site == QC_SITE_FC2 ? launch_epi<EPI_RESID, QC_SITE_FC2>(a, nz, st) : launch_epi<EPI_RESID, QC_SITE_PROJ>(a, nz, st);
  if (epi == EPI_QKV) return launch_epi<EPI_QKV, QC_SITE_QKV>(a, nz, st);
  return site == QC_SITE_ADA ? launch_epi<EPI_F32, QC_SITE_ADA>(a, nz, st) : launch_epi<EPI_F32, QC_SITE_QKV>(a, nz, st);
}

}  // namespace qc

