"""Helpers shared by the GPU parity tests: build the oracle model and the HIP
context from the same seeded inputs, and the error measures of the parity bar."""
from __future__ import annotations

import numpy as np

from oracle import dit, sampler
from synthetic import dit_inputs as I

# parity bar for floating-point outputs (block outputs, noise estimates, latents)
MAX_ABS = 1e-2
REL_RMS = 1e-3


def rel_rms(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    return float(np.sqrt(np.mean((got - want) ** 2)) / max(np.sqrt(np.mean(want ** 2)), 1e-30))


def max_abs(got, want):
    return float(np.max(np.abs(np.asarray(got, dtype=np.float64) - np.asarray(want, dtype=np.float64))))


def assert_close(got, want, what, max_abs_tol=MAX_ABS, rel_rms_tol=REL_RMS):
    ma, rr = max_abs(got, want), rel_rms(got, want)
    assert ma <= max_abs_tol and rr <= rel_rms_tol, "%s: max-abs %.3e (tol %.1e), rel-RMS %.3e (tol %.1e)" % (
        what, ma, max_abs_tol, rr, rel_rms_tol)
    return ma, rr


def code_flip_stats(got_codes, want_codes):
    """Fraction of differing codes and the largest code distance."""
    g = np.asarray(got_codes).astype(np.int32).reshape(-1)
    w = np.asarray(want_codes).astype(np.int32).reshape(-1)
    d = np.abs(g - w)
    return float(np.mean(d != 0)), int(d.max()) if d.size else 0


def qkv_rows_from_heads(ctx, model, max_batch, B):
    """The last QKV projection as a row-major [B * T, 3 D] device tensor, gathered from the head-major buffers the
    attention kernel reads (Q and K [max_batch, H, T, d], V transposed [max_batch, H, dp, Tp] with the keys of each group
    of 32 interleaved in units of 4).  Unlike the optional row-major copy this needs no extra output of the QKV GEMM,
    so the launch under test is the one the sampler makes."""
    import torch
    H, T, D = model.heads, model.tokens, model.hidden
    d = D // H
    dp, Tp = (d + 15) // 16 * 16, (T + 63) // 64 * 64
    n = max_batch * H * T * d
    buf = ctx.workspace("qkv_heads", (2 * n + max_batch * H * dp * Tp,), torch.float32)
    q = buf[:n].view(max_batch, H, T, d)[:B].permute(0, 2, 1, 3).reshape(B * T, D)
    k = buf[n:2 * n].view(max_batch, H, T, d)[:B].permute(0, 2, 1, 3).reshape(B * T, D)
    t = torch.arange(T, device=buf.device)
    u = (t >> 2) & 7
    pos = (t & ~31) | ((((u & 3) << 1) | (u >> 2)) << 2) | (t & 3)
    v = buf[2 * n:].view(max_batch, H, dp, Tp)[:B, :, :d][:, :, :, pos].permute(0, 3, 1, 2).reshape(B * T, D)
    return torch.cat([q, k, v], dim=1)


def oracle_calibration(model, w, wl=None, lat=None, lab=None, t=None):
    """Activation parameters from the oracle's un-quantised forward."""
    if lat is None:
        lat, lab, step_idx = I.calibration_inputs(wl)
        if wl.fixed_t is not None:
            t = np.full((lat.shape[0],), wl.fixed_t)
        else:
            tt, _, _ = sampler.ddim_schedule(wl.steps)
            t = tt[step_idx]
    qp, ranges = sampler.calibrate(model, w, lat, lab, t)
    return qp, ranges, (lat, lab, np.asarray(t))


def make_pair(model, w, qp, max_batch, cache_interval=1):
    """(oracle linears, HIP context) with identical weights and activation parameters."""
    import paper_2503_02508_amd as qc
    lin = dit.QLinears(w, qp, model.weight_bits)
    ctx = qc.Context(model, max_batch, cache_interval)
    ctx.load_weights(w)
    for (blk, site), (s, z) in qp.items():
        ctx.set_act_qparams(blk, dit.SITES.index(site), float(s), int(z))
    return lin, ctx
