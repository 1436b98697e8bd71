"""Oracle: uniform affine quantisation (paper section "Quantization and Cache",
Eq. 1-3) and the quantised linear layer built on it.  Test infrastructure.

Readings taken where the paper is silent or garbled:
  * Eq. 3's zero point is printed with a stray "+z" inside the clip; it is read
    as z = clip(round(-l/s), 0, 2^b - 1).
  * the calibration range [l, u] is widened to contain 0, so that 0.0 is a code.
  * a degenerate range (u == l == 0) gives s = 1, z = 0.
  * round() is round-half-to-even; x/s is an IEEE float32 division.
  * weights are "channel-wise" (Comparison on Performance section): one
    symmetric scale per output row, codes in [-qmax, qmax], qmax = 2^(b-1) - 1.
  * activations are "tensor-wise": one (s, z) per quantiser site.
Codes follow Eq. 1 (unsigned, 0 .. 2^b - 1).  int8 hardware stores code - 128
and zero point - 128; `to_signed` gives that representation, and accumulators
are defined on the signed codes.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


# ----------------------------------------------------------------- Eq. 2-3
def act_qparams(lo, hi, bits: int = 8):
    """(s, z) of an activation quantiser from the observed range (Eq. 2-3)."""
    l32 = F32(min(float(lo), 0.0))
    u32 = F32(max(float(hi), 0.0))
    qmax = F32(2 ** bits - 1)
    if not (u32 > l32):
        return F32(1.0), 0
    s = F32(F32(u32 - l32) / qmax)
    z = int(np.clip(np.rint(F32(-l32) / s), F32(0), qmax))
    return s, z


# ------------------------------------------------------------------- Eq. 1
def quantize(x, s, z: int, bits: int = 8) -> np.ndarray:
    """Q(x|b) = clip(round(x/s) + z, 0, 2^b - 1); decision in float32."""
    x32 = np.asarray(x, dtype=F32)
    r = np.rint(x32 / F32(s))
    q = np.clip(r + F32(z), F32(0), F32(2 ** bits - 1))
    return q.astype(np.int32)


def dequantize(q, s, z: int) -> np.ndarray:
    """Real value a code stands for: s * (q - z), in float64."""
    return np.float64(F32(s)) * (np.asarray(q, dtype=np.int64) - int(z)).astype(np.float64)


def to_signed(q, z: int, bits: int = 8):
    """Shift unsigned codes and zero point by 2^(b-1) (same real values)."""
    off = 2 ** (bits - 1)
    return np.asarray(q, dtype=np.int64) - off, int(z) - off


# ------------------------------------------------- channel-wise weight quant
def weight_quant(W, bits: int = 8):
    """Symmetric per-output-row quantisation of W[N, K].
    Returns (codes int8 [N,K], scale float32 [N], row sums int64 [N])."""
    W32 = np.asarray(W, dtype=F32)
    qmax = F32(2 ** (bits - 1) - 1)
    amax = np.max(np.abs(W32), axis=1)
    s = np.where(amax > 0, amax / qmax, F32(1.0)).astype(F32)
    q = np.clip(np.rint(W32 / s[:, None]), -qmax, qmax).astype(np.int8)
    wsum = q.astype(np.int64).sum(axis=1)
    return q, s, wsum


def pack_w4(q: np.ndarray) -> np.ndarray:
    """Pack 4-bit two's-complement codes [N, K] (K even) two per byte:
    element 2j in bits 0-3, element 2j+1 in bits 4-7."""
    q = np.asarray(q, dtype=np.int8)
    lo = (q[:, 0::2].astype(np.uint8)) & 0xF
    hi = (q[:, 1::2].astype(np.uint8)) & 0xF
    return (lo | (hi << 4)).astype(np.uint8)


def unpack_w4(p: np.ndarray) -> np.ndarray:
    p = np.asarray(p, dtype=np.uint8)
    lo = (p & 0xF).astype(np.int16)
    hi = (p >> 4).astype(np.int16)
    lo = np.where(lo >= 8, lo - 16, lo)
    hi = np.where(hi >= 8, hi - 16, hi)
    out = np.empty((p.shape[0], p.shape[1] * 2), dtype=np.int8)
    out[:, 0::2] = lo
    out[:, 1::2] = hi
    return out


# ------------------------------------------------------ integer contraction
def int_matmul(qa, qw) -> np.ndarray:
    """acc[m, n] = sum_k qa[m, k] * qw[n, k], exact, as int64.
    The float64 matrix product of small integers is exact while every partial
    sum stays below 2^53, which holds for 8-bit codes at any K used here."""
    a = np.asarray(qa, dtype=np.float64)
    w = np.asarray(qw, dtype=np.float64)
    return np.rint(a @ w.T).astype(np.int64)


class QLinear:
    """A weight matrix after channel-wise quantisation (plus its fp32 bias)."""

    def __init__(self, W, b, bits: int = 8):
        self.bits = bits
        self.q, self.scale, self.wsum = weight_quant(W, bits)
        self.bias = np.asarray(b, dtype=F32)

    def packed(self):
        return pack_w4(self.q) if self.bits == 4 else self.q


def lin_q(a, lin: QLinear, s_a, z_a: int, act_bits: int = 8, tap: dict | None = None):
    """Quantised linear layer on a[M, K]:
         q_a = Q(a);  acc = sum_k (q_a - 128) * qw;   (signed codes)
         y   = s_a * s_w[n] * (acc - (z_a - 128) * wsum[n]) + b[n]
    i.e. dequantise(q_a) times dequantise(qw) plus bias, with the integer part
    exact."""
    q = quantize(a, s_a, z_a, act_bits)
    qs, zs = to_signed(q, z_a, act_bits)
    acc = int_matmul(qs, lin.q)
    corr = acc - zs * lin.wsum[None, :]
    y = (np.float64(F32(s_a)) * lin.scale.astype(np.float64))[None, :] * corr.astype(np.float64) \
        + lin.bias.astype(np.float64)[None, :]
    if tap is not None:
        tap["codes"] = qs.astype(np.int8) if act_bits == 8 else qs
        tap["acc"] = acc
    return y


def bf16_round(x):
    """Value of x after storage as bfloat16 (8 exponent bits, 7 fraction bits):
    x is first rounded to float32, then to the nearest bfloat16 with ties to
    even, and returned as float64.  Used by the reduced-precision cache variant
    (not in the paper: it halves the bytes a cached step streams)."""
    x32 = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    bits = x32.view(np.uint32).astype(np.uint64)
    bits = (bits + 0x7FFF + ((bits >> 16) & 1)) & 0xFFFF0000
    return bits.astype(np.uint32).view(np.float32).astype(np.float64).reshape(x32.shape)
