"""Pins for the oracle's quantiser, weight quantiser and integer contraction
(Eq. 1-3 of the paper).  CPU only.  Each test checks the oracle against
something other than itself: hand-computed fixtures, invariants of the
definition, brute-force integer loops."""
import os
import itertools

import numpy as np
import pytest

from oracle import quant as Q

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    out = []
    with open(os.path.join(GOLD, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                out.append([float(v) for v in line.split()])
    return out


def test_quantizer_hand_examples():
    for s, z, x, want in _rows("quantizer_worked_examples.txt"):
        got = int(Q.quantize(np.array([x]), s, int(z))[0])
        assert got == int(want), (s, z, x, got, want)


def test_qparams_hand_examples():
    for l, u, s_want, z_want in _rows("qparams_worked_examples.txt"):
        s, z = Q.act_qparams(l, u)
        assert abs(float(s) - s_want) <= 1e-6 * s_want, (l, u, s)
        assert z == int(z_want), (l, u, z)
        assert isinstance(s, np.float32)


@pytest.mark.parametrize("l,u", [(-3.0, 5.0), (-0.37, 0.11), (0.0, 7.3), (-2.0, 0.0), (-100.0, 1e-3)])
def test_roundtrip_error_bound_and_endpoints(l, u):
    s, z = Q.act_qparams(l, u)
    rng = np.random.default_rng(0)
    x = rng.uniform(l, u, size=20000)
    q = Q.quantize(x, s, z)
    assert q.min() >= 0 and q.max() <= 255
    back = Q.dequantize(q, s, z)
    # inside the range the error is at most half a step (plus float32 rounding of x and x/s)
    assert np.max(np.abs(back - x.astype(np.float32))) <= 0.5 * float(s) * (1 + 1e-5) + 1e-6 * max(abs(l), abs(u))
    # end points and zero
    assert int(Q.quantize(np.array([0.0]), s, z)[0]) == z
    assert int(Q.quantize(np.array([l]), s, z)[0]) == (0 if l < 0 else z)
    assert int(Q.quantize(np.array([u]), s, z)[0]) == (255 if u > 0 else z)
    # 0.0 is represented exactly
    assert Q.dequantize(np.array([z]), s, z)[0] == 0.0
    # saturation outside the range
    assert int(Q.quantize(np.array([l - 10 * (u - l)]), s, z)[0]) == 0
    assert int(Q.quantize(np.array([u + 10 * (u - l)]), s, z)[0]) == 255


def test_idempotent_on_all_codes():
    for s, z in [(np.float32(0.013), 7), (np.float32(1.7), 200), (np.float32(1e-3), 128)]:
        codes = np.arange(256)
        again = Q.quantize(Q.dequantize(codes, s, z), s, z)
        assert np.array_equal(again, codes)


def test_ties_to_even_all_codes():
    # s = 2^-3 makes s*(k + 1/2) exact in float32, so every tie is a true tie.
    s, z = np.float32(0.125), 100
    k = np.arange(-100, 155)
    x = (k + 0.5) * 0.125
    q = Q.quantize(x, s, z)
    want = np.where(k % 2 == 0, k, k + 1) + z
    assert np.array_equal(q, np.clip(want, 0, 255))


def test_monotone_and_step():
    s, z = np.float32(0.031), 93
    x = np.linspace(-5, 7, 100001)
    q = Q.quantize(x, s, z)
    d = np.diff(q)
    assert d.min() >= 0 and d.max() <= 1


def test_signed_representation_same_reals():
    s, z = np.float32(0.02), 77
    q = np.arange(256)
    qs, zs = Q.to_signed(q, z)
    assert qs.min() == -128 and qs.max() == 127 and zs == 77 - 128
    assert np.array_equal(qs - zs, q - z)


# --------------------------------------------------------------- weights
@pytest.mark.parametrize("bits,qmax", [(8, 127), (4, 7)])
def test_weight_quant_properties(bits, qmax):
    rng = np.random.default_rng(1)
    W = (rng.standard_normal((37, 64)) * 0.02).astype(np.float32)
    W[5] = 0.0                                     # an all-zero row
    q, s, wsum = Q.weight_quant(W, bits)
    assert q.dtype == np.int8 and s.dtype == np.float32
    assert np.abs(q).max() <= qmax
    nz = [i for i in range(37) if i != 5]
    assert np.all(np.abs(q[nz]).max(axis=1) == qmax)      # the row maximum maps to +-qmax
    assert s[5] == 1.0 and np.all(q[5] == 0)
    err = np.abs(q.astype(np.float64) * s[:, None].astype(np.float64) - W)
    assert np.all(err <= 0.5 * s[:, None] * (1 + 1e-5))
    assert np.array_equal(wsum, q.astype(np.int64).sum(axis=1))
    # sign symmetry: quantising -W negates the codes (symmetric quantiser, ties to even)
    q2, s2, _ = Q.weight_quant(-W, bits)
    assert np.array_equal(q2, -q) and np.array_equal(s2, s)


def test_w4_pack_roundtrip_all_bytes():
    # every (low nibble, high nibble) pair of 4-bit two's-complement values
    vals = np.arange(-8, 8, dtype=np.int8)
    pairs = np.array(list(itertools.product(vals, vals)), dtype=np.int8)    # [256, 2]
    packed = Q.pack_w4(pairs)
    assert packed.shape == (256, 1) and len(np.unique(packed)) == 256
    assert np.array_equal(Q.unpack_w4(packed), pairs)
    # bit layout: element 0 in the low nibble, element 1 in the high nibble
    assert Q.pack_w4(np.array([[1, 0]], dtype=np.int8))[0, 0] == 0x01
    assert Q.pack_w4(np.array([[0, 1]], dtype=np.int8))[0, 0] == 0x10
    assert Q.pack_w4(np.array([[-1, -8]], dtype=np.int8))[0, 0] == 0x8F


# ------------------------------------------------------------ contraction
def test_int_matmul_vs_python_loops():
    rng = np.random.default_rng(2)
    a = rng.integers(-128, 128, size=(5, 48))
    w = rng.integers(-127, 128, size=(7, 48))
    want = [[sum(int(a[m, k]) * int(w[n, k]) for k in range(48)) for n in range(7)] for m in range(5)]
    assert np.array_equal(Q.int_matmul(a, w), np.array(want, dtype=np.int64))


def test_int_matmul_vs_int64_matmul_and_extremes():
    rng = np.random.default_rng(3)
    a = rng.integers(-128, 128, size=(33, 4608)).astype(np.int64)
    w = rng.integers(-127, 128, size=(29, 4608)).astype(np.int64)
    assert np.array_equal(Q.int_matmul(a, w), a @ w.T)
    # extreme magnitudes at the largest K of the workloads stay inside int32
    a = np.full((2, 4608), -128); w = np.full((3, 4608), -127)
    acc = Q.int_matmul(a, w)
    assert np.all(acc == 4608 * 128 * 127) and acc.max() < 2 ** 31
    assert np.all(Q.int_matmul(a, -w) == -4608 * 128 * 127)


def test_lin_q_zero_point_identity_and_dequant_meaning():
    """lin_q must equal 'dequantise both operands, multiply in real numbers'."""
    rng = np.random.default_rng(4)
    a = rng.standard_normal((9, 32)) * 2
    W = (rng.standard_normal((11, 32)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(11) * 0.02).astype(np.float32)
    lin = Q.QLinear(W, b, 8)
    s, z = Q.act_qparams(a.min(), a.max())
    tap = {}
    y = Q.lin_q(a, lin, s, z, tap=tap)
    a_hat = Q.dequantize(Q.quantize(a, s, z), s, z)                        # reals the codes stand for
    w_hat = lin.q.astype(np.float64) * lin.scale[:, None].astype(np.float64)
    want = a_hat @ w_hat.T + b.astype(np.float64)
    assert np.allclose(y, want, rtol=1e-12, atol=1e-12)
    # accumulators are defined on the signed codes, brute force
    codes = tap["codes"].astype(int)
    brute = np.array([[sum(int(codes[m, k]) * int(lin.q[n, k]) for k in range(32)) for n in range(11)]
                      for m in range(9)])
    assert np.array_equal(tap["acc"], brute)
    assert codes.min() >= -128 and codes.max() <= 127


def test_lin_q_w4_uses_packed_codes_consistently():
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((6, 16)) * 0.02).astype(np.float32)
    lin = Q.QLinear(W, np.zeros(6, np.float32), 4)
    assert np.abs(lin.q).max() == 7
    assert np.array_equal(Q.unpack_w4(lin.packed()), lin.q)


def test_lin_q_converges_to_fp_linear_with_fine_codes():
    """With 16-bit activations and weights the quantised layer approaches the real one."""
    rng = np.random.default_rng(6)
    a = rng.standard_normal((20, 64))
    W = (rng.standard_normal((10, 64)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(10) * 0.02).astype(np.float32)
    exact = a @ W.astype(np.float64).T + b
    errs = []
    for bits in (8, 16):
        lin = Q.QLinear.__new__(Q.QLinear)
        lin.bits = bits
        W32 = W
        qmax = 2 ** (bits - 1) - 1
        amax = np.abs(W32).max(axis=1)
        lin.scale = (amax / np.float32(qmax)).astype(np.float32)
        lin.q = np.clip(np.rint(W32 / lin.scale[:, None]), -qmax, qmax).astype(np.int64)
        lin.wsum = lin.q.sum(axis=1)
        lin.bias = b
        s, z = Q.act_qparams(a.min(), a.max(), bits)
        y = Q.lin_q(a, lin, s, z, act_bits=bits)
        errs.append(np.abs(y - exact).max())
    assert errs[0] < 2e-2 and errs[1] < errs[0] / 100


def test_bf16_round_matches_library_conversion_and_ties_to_even():
    import torch
    rng = np.random.default_rng(3)
    x = np.concatenate([rng.normal(size=4000) * 10.0 ** rng.integers(-6, 6, size=4000), [0.0, -0.0, 1.0, -1.0, 3.0e38, 1e-30]])
    want = torch.tensor(x, dtype=torch.float32).to(torch.bfloat16).to(torch.float32).numpy().astype(np.float64)
    got = Q.bf16_round(x)
    assert np.array_equal(got, want)
    # exact halfway cases: 1 + 2^-8 lies between 1 and 1 + 2^-7 -> even (1); 1 + 3 * 2^-8 -> 1 + 2^-6
    assert Q.bf16_round(np.array([1.0 + 2.0 ** -8]))[0] == 1.0
    assert Q.bf16_round(np.array([1.0 + 3 * 2.0 ** -8]))[0] == 1.0 + 2.0 ** -6
    # idempotent, relative error at most 2^-9
    assert np.array_equal(Q.bf16_round(got), got)
    nz = x != 0
    assert np.max(np.abs(got[nz] - np.float32(x[nz]).astype(np.float64)) / np.abs(x[nz])) <= 2.0 ** -8
