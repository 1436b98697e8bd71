"""The entry point that allocates nothing (qc_vc_fit_static: partial sums in the library's fixed device array)
against qc_vc_fit with a caller-provided workspace, through the C ABI: same kernels, so the factors must be equal bit
for bit - on two calls in a row, the second with a smaller input (the array keeps the first call's contents)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def _pair(B, C, H, W, seed):
    import torch
    rng = np.random.default_rng(seed)
    xr = rng.standard_normal((B, C, H, W)).astype(np.float32) * 2 + 0.3
    xh = (1.07 * (xr - xr.mean(axis=(2, 3), keepdims=True)) + xr.mean(axis=(2, 3), keepdims=True)
          + 0.05 * rng.standard_normal((B, C, H, W))).astype(np.float32)
    return torch.from_numpy(xh).cuda(), torch.from_numpy(xr).cuda()


def test_static_scratch_entry_point_matches_workspace_entry_point():
    import torch
    import paper_2503_02508_amd as qc
    from oracle import vc_fit
    for (B, C, H, W, seed) in [(6, 4, 32, 32, 1), (2, 3, 9, 7, 2)]:       # second call: smaller input
        xh, xr = _pair(B, C, H, W, seed)
        work = torch.full((B * C * 2,), float("nan"), dtype=torch.float64, device="cuda")
        K_ws = torch.zeros(C, dtype=torch.float32, device="cuda")
        K_st = torch.zeros(C, dtype=torch.float32, device="cuda")
        qc.qc_vc_fit(xh, xr, 1e-3, work, K_ws)
        qc.qc_vc_fit_static(xh, xr, 1e-3, K_st)
        torch.cuda.synchronize()
        assert torch.equal(K_st, K_ws), (K_st, K_ws)
        want = vc_fit.fit_factor(xh.cpu().numpy(), xr.cpu().numpy(), 1e-3)
        assert np.max(np.abs(K_st.cpu().numpy().astype(np.float64) - want)) <= 2e-6
    # beyond the fixed array: a clear error, nothing launched
    import ctypes as C_
    big = torch.zeros((1,), device="cuda")
    p = C_.c_void_p(big.data_ptr())
    assert qc.lib.qc_vc_fit_static(p, p, 4097, 4, 1, 1, 0.0, p, None) == -6
    assert "planes" in qc.last_error()
