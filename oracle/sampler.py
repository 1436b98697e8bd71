"""Oracle: sampler step with the step-level cache rule and the variance
compensation (VC) of the paper, plus the min/max calibration that yields the
activation quantiser parameters.  Test infrastructure.  float64.

Readings taken where the paper is silent:
  * cache rule ("Quantization and Cache" section: recompute when the step
    counter mod N is 0, reuse for the following N-1 steps): the counter is the
    sampling-step index i = 0, 1, ...; step 0 is always a refresh.
  * solver: deterministic DDIM (eta = 0) on the 1000-step linear-beta schedule
    (1e-4 .. 2e-2), timesteps t_i = (St-1-i) * floor(1000/St); abar_prev = 1
    on the last step; no clipping of the predicted x0.
  * VC (Eq. 10) acts on the sample after the solver update; mu is the spatial
    mean of each (sample, channel) plane of that sample, so the correction
    keeps every plane's mean and scales its variance by K^2 (Eq. 9).  It is
    evaluated as x + (K-1)(x-mu), which is Eq. 10 rearranged.
  * classifier-free guidance (not in the paper; used by one workload): the
    batch is [conditional ; null-label], eps = eps_u + w (eps_c - eps_u).
  * storage precision: the sample after the solver update and the sample after
    VC are float32 tensors (dit.st); each of the two is evaluated in float64
    from the stored tensors it reads.
"""
from __future__ import annotations

import numpy as np

from .dit import FPLinears, QLinears, denoiser, block_full, SITES, st
from .quant import act_qparams

F64 = np.float64
TRAIN_STEPS = 1000


def abar_table(n: int = TRAIN_STEPS, beta0: float = 1e-4, beta1: float = 2e-2):
    betas = np.linspace(beta0, beta1, n, dtype=F64)
    return np.cumprod(1.0 - betas)


def ddim_schedule(steps: int):
    """(t[St], abar_t[St], abar_prev[St]) for a descending timestep list."""
    ab = abar_table()
    stride = TRAIN_STEPS // steps
    t = np.array([(steps - 1 - i) * stride for i in range(steps)], dtype=np.int64)
    abar_t = ab[t]
    abar_prev = np.concatenate([ab[t[1:]], [1.0]])
    return t, abar_t, abar_prev


def is_refresh_step(i: int, interval: int) -> bool:
    return i % interval == 0


def ddim_update(x, eps, abar_t: float, abar_prev: float):
    x0 = (x - np.sqrt(1.0 - abar_t) * eps) / np.sqrt(abar_t)
    return np.sqrt(abar_prev) * x0 + np.sqrt(1.0 - abar_prev) * eps


def cfg_combine(eps_c, eps_u, w: float):
    return eps_u + w * (eps_c - eps_u)


def vc_correct(x, K_t, mu=None):
    """Eq. 10, channel-wise: x~ = mu + K_t (x - mu).  x[B, C, H, W], K_t[C].
    mu defaults to the per-(sample, channel) spatial mean; a caller-supplied
    mu[C] is the other reading of the equation."""
    x = np.asarray(x, dtype=F64)
    K = np.asarray(K_t, dtype=F64).reshape(1, -1, 1, 1)
    if mu is None:
        m = x.mean(axis=(2, 3), keepdims=True)
    else:
        m = np.asarray(mu, dtype=F64).reshape(1, -1, 1, 1)
    return x + (K - 1.0) * (x - m)


def sample_step(x, labels, i, t, abar_t, abar_prev, desc, w, linear, cache, interval,
                cfg_scale=0.0, K_t=None, force_full=None, taps=None, cache_bf16=False):
    """One sampler step: denoiser (full or cached by the cache rule), guidance,
    solver update, VC.  force_full: None = the rule, a boolean = that mode, an
    array [depth, 2] = a per-(block, module) schedule for this step."""
    if force_full is None:
        full = is_refresh_step(i, interval)
    elif isinstance(force_full, (bool, np.bool_, int)):
        full = bool(force_full)
    else:
        full = np.asarray(force_full, dtype=bool)
    B = x.shape[0]
    if cfg_scale > 0:
        xin = np.concatenate([x, x], axis=0)
        yin = np.concatenate([np.asarray(labels), np.full((B,), desc.num_classes)])
    else:
        xin, yin = x, np.asarray(labels)
    tt = np.full((xin.shape[0],), t)
    eps = denoiser(xin, tt, yin, desc, w, linear, cache, full, taps, cache_bf16)
    if cfg_scale > 0:
        eps = cfg_combine(eps[:B], eps[B:], cfg_scale)
    xn = st(ddim_update(np.asarray(x, dtype=F64), eps, abar_t, abar_prev))      # the updated sample is a stored tensor ...
    if K_t is not None:
        xn = st(vc_correct(xn, K_t))                                           # ... and so is the corrected one
    return xn, eps


def sample(x, labels, steps, interval, desc, w, linear, cfg_scale=0.0, K=None,
           max_steps=None, trace=None, mask=None, cache_bf16=False):
    """Run the sampler for `steps` steps (or only the first `max_steps`).
    mask[steps, depth, 2] (1 = recompute) replaces the interval rule."""
    t, abar_t, abar_prev = ddim_schedule(steps)
    cache: dict = {}
    x = np.asarray(x, dtype=F64)
    n = steps if max_steps is None else min(steps, max_steps)
    for i in range(n):
        K_t = None if K is None else K[i]
        x, eps = sample_step(x, labels, i, int(t[i]), abar_t[i], abar_prev[i], desc, w, linear,
                             cache, interval, cfg_scale, K_t, None if mask is None else np.asarray(mask)[i],
                             cache_bf16=cache_bf16)
        if trace is not None:
            trace.append((x.copy(), eps.copy()))
    return x


# ------------------------------------------------------------- calibration
def calibrate(desc, w, latents, labels, timesteps):
    """Activation quantiser parameters from calibration data (Eq. 2-3): an
    un-quantised forward of every calibration input, the global min / max of
    each site's input over all of them, then act_qparams.
    Returns {(block, site): (s, z)} and the raw ranges."""
    fp = FPLinears(w)
    for n in range(latents.shape[0]):
        denoiser(latents[n:n + 1], np.array([timesteps[n]]), labels[n:n + 1], desc, w, fp,
                 cache={}, full=True)
    return {k: act_qparams(lo, hi) for k, (lo, hi) in fp.ranges.items()}, fp.ranges


def calibrate_block(desc, w, tokens, cond):
    """Single-block variant: ranges from full-block forwards of tokens[n, T, D]
    with conditioning cond[n, D]."""
    fp = FPLinears(w)
    for n in range(tokens.shape[0]):
        block_full(np.asarray(tokens[n:n + 1], dtype=F64), np.asarray(cond[n:n + 1], dtype=F64),
                   0, desc.heads, fp)
    return {k: act_qparams(lo, hi) for k, (lo, hi) in fp.ranges.items()}, fp.ranges
