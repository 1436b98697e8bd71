"""Oracle: fitting the variance-compensation factors K[St, C] ("Variance Align
for Exposure Bias" section: the argmin objective that follows Eq. 10, and the
closed form printed after it).  Test infrastructure.  float64.

The objective for one timestep and one channel, over all N elements of that
channel in a small batch of intermediate samples (N = batch x height x width):

    L(K) = sum_n ((x~_n - x'_n) / x'_n)^2  +  sum_n (x~_n - x'_n)^2,
    x~_n = mu + K (x^_n - mu)                                        (Eq. 10)

x^ is the accelerated (quantised + cached) sampler's intermediate sample, x'
the full-precision sampler's sample at the same step (the target), mu the
spatial mean of the x^ plane the element lies in (the same mu Eq. 10 uses when
the correction is applied).  The first term is the squared inverse root
quantisation-to-noise ratio taken element by element (relative error), the
second the squared error.

Readings taken where the paper is silent or garbled:
  * the printed closed form has a self-evidently damaged exponent in its last
    denominator term ("2+") and its second numerator term equals the exact
    derivative only when mu = 0.  This oracle uses the exact minimiser of L,

        K = sum_n d_n (x'_n - mu) w_n / sum_n d_n^2 w_n,
        d_n = x^_n - mu,  w_n = 1 + 1 / (x'_n^2 + eps),

    which reduces to the printed expression for mu = 0 and eps = 0 (pinned by
    a test).  eps > 0 (the "+" that survives in the printed exponent) keeps
    elements with x' near 0 finite; it is an input.
  * K is fitted step by step along the trajectory: at step i the accelerated
    sample before VC is fitted against the reference sample, the fitted K_i is
    applied, and both samplers go on; so K_i sees the corrections of the steps
    before it, as it will when it is used.
  * a channel whose d is identically 0 gets K = 1.
"""
from __future__ import annotations

import numpy as np

from . import sampler
from .dit import FPLinears, st

F64 = np.float64


def _planes(x_hat, x_ref):
    xh = np.asarray(x_hat, dtype=F64)
    xr = np.asarray(x_ref, dtype=F64)
    if xh.shape != xr.shape or xh.ndim != 4:
        raise ValueError("x_hat and x_ref must both be [B, C, H, W]")
    mu = xh.mean(axis=(2, 3), keepdims=True)
    return xh, xr, mu


def objective(K, x_hat, x_ref, eps: float):
    """L(K) per channel ([C]) for factors K[C]."""
    xh, xr, mu = _planes(x_hat, x_ref)
    Kc = np.asarray(K, dtype=F64).reshape(1, -1, 1, 1)
    e = mu + Kc * (xh - mu) - xr
    return (e * e / (xr * xr + eps) + e * e).sum(axis=(0, 2, 3))


def fit_sums(x_hat, x_ref, eps: float):
    """(S1[C], S2[C]) = (sum d (x' - mu) w, sum d^2 w) over batch and plane."""
    xh, xr, mu = _planes(x_hat, x_ref)
    d = xh - mu
    w = 1.0 + 1.0 / (xr * xr + eps)
    return (d * (xr - mu) * w).sum(axis=(0, 2, 3)), (d * d * w).sum(axis=(0, 2, 3))


def fit_factor(x_hat, x_ref, eps: float = 1e-6):
    """K[C] that minimises L for this batch of (accelerated, reference) samples."""
    s1, s2 = fit_sums(x_hat, x_ref, eps)
    K = np.ones_like(s1)
    nz = s2 > 0
    K[nz] = s1[nz] / s2[nz]
    return K


def fit_sampler(x0, labels, steps, interval, desc, w, linear_q, cfg_scale=0.0, eps: float = 1e-6):
    """Runs the full-precision, un-cached sampler and the accelerated sampler
    from the same initial latents and labels and fits K step by step.
    Returns (K[steps, C], accelerated final sample, reference final sample)."""
    tt, at, ap = sampler.ddim_schedule(steps)
    fp = FPLinears(w)
    x_ref = np.asarray(x0, dtype=F64)
    x_hat = np.asarray(x0, dtype=F64)
    cache_q: dict = {}
    K = np.ones((steps, x_hat.shape[1]), dtype=F64)
    for i in range(steps):
        x_ref, _ = sampler.sample_step(x_ref, labels, i, int(tt[i]), at[i], ap[i], desc, w, fp, {}, 1, cfg_scale, None,
                                       force_full=True)
        x_hat, _ = sampler.sample_step(x_hat, labels, i, int(tt[i]), at[i], ap[i], desc, w, linear_q, cache_q, interval,
                                       cfg_scale, None)
        K[i] = st(fit_factor(x_hat, x_ref, eps))              # the factors are a stored (float32) table
        x_hat = st(sampler.vc_correct(x_hat, K[i]))
    return K, x_hat, x_ref
