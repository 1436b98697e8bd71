"""Pins for the VC-factor fit of the oracle: brute-force minimisation of the
objective, the cases with a known answer, and the printed closed form in the
case where it is exact."""
import numpy as np
import pytest

from oracle import vc_fit, sampler


def _pair(seed, B=3, C=4, H=6, W=5, noise=0.1, shift=0.3):
    rng = np.random.default_rng(seed)
    x_ref = rng.normal(size=(B, C, H, W)) + shift
    scale = rng.uniform(0.8, 1.2, size=(1, C, 1, 1))
    mu = x_ref.mean(axis=(2, 3), keepdims=True)
    x_hat = mu + scale * (x_ref - mu) + noise * rng.normal(size=x_ref.shape)
    return x_hat, x_ref


def _golden_min(f, lo, hi, it=200):
    g = (np.sqrt(5.0) - 1.0) / 2.0
    a, b = lo, hi
    c, d = b - g * (b - a), a + g * (b - a)
    for _ in range(it):
        if f(c) < f(d):
            b, d = d, c
            c = b - g * (b - a)
        else:
            a, c = c, d
            d = a + g * (b - a)
    return 0.5 * (a + b)


@pytest.mark.parametrize("seed,eps", [(1, 1e-6), (2, 1e-2), (3, 1.0)])
def test_closed_form_is_the_brute_force_minimiser(seed, eps):
    x_hat, x_ref = _pair(seed)
    K = vc_fit.fit_factor(x_hat, x_ref, eps)
    for c in range(x_hat.shape[1]):
        def f(k, c=c):
            Kc = K.copy()
            Kc[c] = k
            return vc_fit.objective(Kc, x_hat, x_ref, eps)[c]
        # coarse grid first (the objective is a parabola in k, but do not assume it), then golden section
        grid = np.linspace(-2.0, 4.0, 601)
        k0 = grid[np.argmin([f(k) for k in grid])]
        kb = _golden_min(f, k0 - 0.02, k0 + 0.02)
        assert abs(kb - K[c]) < 1e-7, (c, kb, K[c])
        # and it is a strict minimum
        assert f(K[c]) < f(K[c] + 1e-3) and f(K[c]) < f(K[c] - 1e-3)


def test_identical_samples_give_one():
    x_hat, _ = _pair(4)
    np.testing.assert_allclose(vc_fit.fit_factor(x_hat, x_hat.copy(), 1e-6), 1.0, rtol=0, atol=1e-14)


def test_pure_variance_scaling_is_recovered():
    """x' = mu + a (x^ - mu) plane by plane: the fit must return a."""
    rng = np.random.default_rng(5)
    x_hat = rng.normal(size=(2, 3, 4, 4)) + 0.5
    a = np.array([0.9, 1.0, 1.3])
    mu = x_hat.mean(axis=(2, 3), keepdims=True)
    x_ref = mu + a.reshape(1, 3, 1, 1) * (x_hat - mu)
    np.testing.assert_allclose(vc_fit.fit_factor(x_hat, x_ref, 1e-3), a, rtol=1e-12)
    # and applying the fitted factor reproduces the reference (Eq. 10)
    np.testing.assert_allclose(sampler.vc_correct(x_hat, a), x_ref, rtol=0, atol=1e-13)


def test_reduces_to_the_printed_closed_form_when_plane_means_vanish():
    """Closed form printed after the argmin objective, evaluated literally with mu = 0."""
    rng = np.random.default_rng(6)
    x_hat = rng.normal(size=(2, 2, 4, 4))
    x_hat -= x_hat.mean(axis=(2, 3), keepdims=True)          # mu = 0 exactly up to rounding
    x_ref = x_hat * 1.1 + 0.05 * rng.normal(size=x_hat.shape)
    x_ref[np.abs(x_ref) < 0.05] = 0.05                       # keep 1 / x' finite at eps = 0
    num = (x_ref * x_hat).sum(axis=(0, 2, 3)) + (x_hat / x_ref).sum(axis=(0, 2, 3))
    den = (x_hat ** 2).sum(axis=(0, 2, 3)) + (x_hat ** 2 / x_ref ** 2).sum(axis=(0, 2, 3))
    np.testing.assert_allclose(vc_fit.fit_factor(x_hat, x_ref, 0.0), num / den, rtol=1e-10)


def test_zero_deviation_channel_gets_one():
    x_hat = np.ones((2, 2, 3, 3))
    x_hat[:, 1] += np.arange(9.0).reshape(3, 3)
    x_ref = x_hat * 1.5
    K = vc_fit.fit_factor(x_hat, x_ref, 1e-6)
    assert K[0] == 1.0 and np.isfinite(K[1])


def test_sums_are_additive_over_the_batch():
    x_hat, x_ref = _pair(7, B=4)
    a1, a2 = vc_fit.fit_sums(x_hat[:2], x_ref[:2], 1e-4)
    b1, b2 = vc_fit.fit_sums(x_hat[2:], x_ref[2:], 1e-4)
    s1, s2 = vc_fit.fit_sums(x_hat, x_ref, 1e-4)
    np.testing.assert_allclose(a1 + b1, s1, rtol=1e-13)
    np.testing.assert_allclose(a2 + b2, s2, rtol=1e-13)


def test_fit_along_a_trajectory_reduces_the_objective():
    """Tiny model: the fitted K never does worse than K = 1 at the step it is fitted on, and the loop
    returns one factor per (step, channel)."""
    from synthetic import dit_inputs as I
    from oracle import dit
    from tests.qc_testlib import oracle_calibration
    model = I.ModelDesc(depth=1, hidden=32, heads=2, mlp_dim=64, patch=2, latent_c=4, latent_h=8, latent_w=8,
                        num_classes=10, freq_dim=16, weight_bits=8)
    steps, interval = 6, 2
    w = I.make_weights(model, 11, std=0.15)
    tt, at, ap = sampler.ddim_schedule(steps)
    clat = np.concatenate([I.make_latents(1, model, 4000 + i) for i in range(4)])
    qp, _, _ = oracle_calibration(model, w, lat=clat, lab=I.make_labels(4, model, 12), t=tt[[0, 2, 4, 5]])
    lin = dit.QLinears(w, qp, 8)
    x0, lab = I.make_latents(2, model, 13), I.make_labels(2, model, 14)
    K, x_hat, x_ref = vc_fit.fit_sampler(x0, lab, steps, interval, model, w, lin, 0.0, 1e-3)
    assert K.shape == (steps, 4) and np.all(np.isfinite(K))
    # replay: at every step the fitted factor beats the identity on the objective it minimises
    fp = dit.FPLinears(w)
    xr = x0.astype(np.float64)
    xh = x0.astype(np.float64)
    cache = {}
    for i in range(steps):
        xr, _ = sampler.sample_step(xr, lab, i, int(tt[i]), at[i], ap[i], model, w, fp, {}, 1, 0.0, None, force_full=True)
        xh, _ = sampler.sample_step(xh, lab, i, int(tt[i]), at[i], ap[i], model, w, lin, cache, interval, 0.0, None)
        assert np.all(vc_fit.objective(K[i], xh, xr, 1e-3) <= vc_fit.objective(np.ones(4), xh, xr, 1e-3) + 1e-12)
        xh = dit.st(sampler.vc_correct(xh, K[i]))          # the corrected sample is a stored (float32) tensor
    np.testing.assert_allclose(xh, x_hat, rtol=0, atol=1e-12)
    np.testing.assert_allclose(xr, x_ref, rtol=0, atol=1e-12)
