"""GPU parity of the single operations, through the C ABI, against the CPU
oracle on identical seeded inputs.  Integer results (codes, accumulators, row
sums) must match bit for bit."""
import numpy as np
import pytest

from oracle import quant as OQ
from oracle import sampler as OS

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def qc():
    import paper_2503_02508_amd as m
    return m


def _cuda(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


# ------------------------------------------------------------- quantize_act
@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 255, 1024, 1_000_003])
@pytest.mark.parametrize("s,z", [(0.0317, 121), (1.0, 0), (2.5e-3, 255)])
def test_quantize_act_bit_exact(qc, n, s, z):
    import torch
    rng = np.random.default_rng(n)
    x = (rng.standard_normal(n) * 3).astype(np.float32)
    if n >= 255:
        k = np.arange(-100, 100)
        x[:200] = ((k + 0.5) * np.float32(s)).astype(np.float32)      # values at / next to rounding ties
        x[200:204] = [1e30, -1e30, 0.0, -0.0]
    xd = _cuda(x)
    q = torch.empty(n + 8, dtype=torch.int8, device="cuda").fill_(77)[:n]
    qc.qc_quantize_act(xd, q, s, z)
    torch.cuda.synchronize()
    want = OQ.quantize(x, np.float32(s), z) - 128
    assert np.array_equal(q.cpu().numpy().astype(np.int32), want)


def test_quantize_act_empty_and_errors(qc):
    import torch
    x = torch.zeros(16, device="cuda")
    q = torch.zeros(16, dtype=torch.int8, device="cuda")
    qc.qc_quantize_act(x[:0], q[:0], 1.0, 0)
    for s, z in [(0.0, 0), (-1.0, 0), (float("nan"), 0), (float("inf"), 0), (1.0, -1), (1.0, 256)]:
        with pytest.raises(qc.QCError) as e:
            qc.qc_quantize_act(x, q, s, z)
        assert e.value.code == -4


# ---------------------------------------------------------- quantize_weight
@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("N,K", [(37, 64), (5, 16), (1152, 1152), (130, 4608)])
def test_quantize_weight_bit_exact(qc, bits, N, K):
    import torch
    rng = np.random.default_rng(N * 7 + K + bits)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    W[N // 2] = 0.0
    qw = torch.empty((N, K if bits == 8 else K // 2), dtype=torch.int8 if bits == 8 else torch.uint8, device="cuda")
    sc = torch.empty(N, dtype=torch.float32, device="cuda")
    ws = torch.empty(N, dtype=torch.int32, device="cuda")
    qc.qc_quantize_weight(_cuda(W), bits, qw, sc, ws)
    torch.cuda.synchronize()
    q, s, wsum = OQ.weight_quant(W, bits)
    want = q if bits == 8 else OQ.pack_w4(q)
    assert np.array_equal(qw.cpu().numpy(), want)
    assert np.array_equal(sc.cpu().numpy(), s)                 # fp32 scale bit-equal
    assert np.array_equal(ws.cpu().numpy().astype(np.int64), wsum)


# -------------------------------------------------------------- w8a8_linear
SHAPES = [(1, 1, 16), (7, 33, 48), (8, 6912, 1152), (130, 200, 144), (256, 1152, 384), (300, 257, 1168),
          (65, 129, 4608), (512, 3456, 1152)]


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("M,N,K", SHAPES)
def test_w8a8_linear_accumulators_bit_exact(qc, bits, M, N, K):
    import torch
    rng = np.random.default_rng(M + 31 * N + 977 * K + bits)
    qx = rng.integers(-128, 128, size=(M, K), dtype=np.int8)
    W = (rng.standard_normal((N, K)) * 0.02).astype(np.float32)
    b = (rng.standard_normal(N) * 0.02).astype(np.float32)
    lin = OQ.QLinear(W, b, bits)
    s_x, z_x = np.float32(0.0213), 117
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    qc.qc_w8a8_linear(_cuda(qx), _cuda(lin.packed()), _cuda(lin.wsum.astype(np.int32)), _cuda(lin.scale), _cuda(b),
                      float(s_x), z_x, bits, y, acc)
    torch.cuda.synchronize()
    want_acc = OQ.int_matmul(qx, lin.q)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), want_acc)
    corr = want_acc - (z_x - 128) * lin.wsum[None, :]
    want_y = (np.float64(s_x) * lin.scale.astype(np.float64))[None, :] * corr + b.astype(np.float64)[None, :]
    got = y.cpu().numpy().astype(np.float64)
    assert np.max(np.abs(got - want_y)) <= 1e-6 * np.max(np.abs(want_y)) + 1e-7


def test_w8a8_linear_extreme_codes_and_no_bias(qc):
    import torch
    M, N, K = 40, 70, 4608
    qx = np.full((M, K), -128, dtype=np.int8)
    qw = np.full((N, K), -127, dtype=np.int8)
    qw[::2] = 127
    wsum = qw.astype(np.int64).sum(axis=1).astype(np.int32)
    sc = np.full(N, 1e-3, dtype=np.float32)
    y = torch.empty((M, N), dtype=torch.float32, device="cuda")
    acc = torch.empty((M, N), dtype=torch.int32, device="cuda")
    qc.qc_w8a8_linear(_cuda(qx), _cuda(qw), _cuda(wsum), _cuda(sc), None, 0.5, 0, 8, y, acc)
    torch.cuda.synchronize()
    want = OQ.int_matmul(qx, qw)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), want) and abs(want).max() == 4608 * 128 * 127
    # zero point 0 (unsigned) = -128 signed: acc - (-128) * wsum = 0 for all-(-128) inputs
    assert np.all(y.cpu().numpy() == 0.0)


def test_w8a8_linear_deterministic(qc):
    import torch
    rng = np.random.default_rng(5)
    M, N, K = 300, 500, 1152
    qx = _cuda(rng.integers(-128, 128, size=(M, K), dtype=np.int8))
    qw = _cuda(rng.integers(-127, 128, size=(N, K), dtype=np.int8))
    ws = _cuda(np.zeros(N, dtype=np.int32)); sc = _cuda(np.ones(N, dtype=np.float32))
    outs = []
    for _ in range(2):
        y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        qc.qc_w8a8_linear(qx, qw, ws, sc, None, 1.0, 128, 8, y, None)
        torch.cuda.synchronize()
        outs.append(y.cpu().numpy())
    assert np.array_equal(outs[0], outs[1])


def test_w8a8_linear_errors(qc):
    import torch
    a = torch.zeros((4, 32), dtype=torch.int8, device="cuda")
    w = torch.zeros((4, 32), dtype=torch.int8, device="cuda")
    v = torch.zeros(4, device="cuda"); vi = torch.zeros(4, dtype=torch.int32, device="cuda")
    y = torch.zeros((4, 4), device="cuda")
    with pytest.raises(qc.QCError) as e:
        qc.qc_w8a8_linear(a[:, :24].contiguous(), w[:, :24].contiguous(), vi, v, None, 1.0, 0, 8, y)
    assert e.value.code == -2                       # K not a multiple of 16
    with pytest.raises(qc.QCError) as e:
        qc.qc_w8a8_linear(a, w, vi, v, None, 1.0, 0, 5, y)
    assert e.value.code == -7
    with pytest.raises(qc.QCError) as e:
        qc.qc_w8a8_linear(a, w, None, v, None, 1.0, 0, 8, y)
    assert e.value.code == -1


# ----------------------------------------------------------------------- VC
@pytest.mark.parametrize("B,C,H,W", [(1, 4, 32, 32), (3, 4, 64, 64), (2, 3, 5, 7)])
def test_vc_correct_vs_oracle(qc, B, C, H, W):
    import torch
    rng = np.random.default_rng(B + C + H)
    x = (rng.standard_normal((B, C, H, W)) * 2 + 0.3).astype(np.float32)
    K = rng.uniform(0.9, 1.05, size=C).astype(np.float32)
    xd = _cuda(x)
    qc.qc_vc_correct(xd, _cuda(K))
    got = xd.cpu().numpy()
    want = OS.vc_correct(x, K)
    assert np.max(np.abs(got - want)) <= 2e-6 * np.max(np.abs(want))
    # K = 1 is a bitwise identity
    xd = _cuda(x)
    qc.qc_vc_correct(xd, _cuda(np.ones(C, dtype=np.float32)))
    assert np.array_equal(xd.cpu().numpy(), x)
    # caller-supplied mean
    mu = rng.standard_normal(C).astype(np.float32)
    xd = _cuda(x)
    qc.qc_vc_correct(xd, _cuda(K), _cuda(mu))
    assert np.max(np.abs(xd.cpu().numpy() - OS.vc_correct(x, K, mu))) <= 2e-6 * np.max(np.abs(want))
