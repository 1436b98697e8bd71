"""Pins for the oracle's network pieces, cache rule, solver and VC.  CPU only.
Each piece is checked against a library routine, a closed form or an invariant
of its definition, never against the oracle's own formula."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import dit, sampler, quant
from synthetic import dit_inputs as I

TINY = I.ModelDesc(depth=2, hidden=32, heads=2, mlp_dim=64, patch=2, latent_c=4, latent_h=8, latent_w=8,
                   num_classes=10)


@pytest.fixture
def exact_storage():
    """The formulas against library routines: stored tensors keep float64 (no rounding to the float32 storage format)."""
    with dit.storage("f64"):
        yield


def _tiny_setup(seed=0, std=0.2):
    w = I.make_weights(TINY, seed, std=std)
    lat = I.make_latents(3, TINY, seed + 1)
    lab = I.make_labels(3, TINY, seed + 2)
    return w, lat, lab


# ------------------------------------------------------- library routines
def test_layer_norm_vs_torch():
    x = np.random.default_rng(0).standard_normal((2, 5, 32)) * 3 + 1
    want = F.layer_norm(torch.from_numpy(x), (32,), eps=1e-6).numpy()
    assert np.allclose(dit.layer_norm(x), want, rtol=1e-12, atol=1e-12)
    out = dit.layer_norm(x)
    assert np.allclose(out.mean(-1), 0, atol=1e-12) and np.allclose(out.var(-1), 1, atol=1e-5)


def test_gelu_silu_vs_torch():
    x = np.linspace(-6, 6, 1001)
    assert np.allclose(dit.gelu_tanh(x), F.gelu(torch.from_numpy(x), approximate="tanh").numpy(), atol=1e-14)
    assert np.allclose(dit.silu(x), F.silu(torch.from_numpy(x)).numpy(), atol=1e-14)


def test_attention_vs_torch_sdpa():
    rng = np.random.default_rng(1)
    B, T, H, d = 2, 7, 3, 8
    D = H * d
    qkv = rng.standard_normal((B, T, 3 * D))
    got = dit.attention(qkv, H)
    t = torch.from_numpy(qkv).reshape(B, T, 3, H, d).permute(2, 0, 3, 1, 4)
    want = F.scaled_dot_product_attention(t[0], t[1], t[2]).permute(0, 2, 1, 3).reshape(B, T, D).numpy()
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)


def test_attention_uniform_when_keys_equal():
    # identical keys -> uniform weights -> output is the mean of V
    B, T, H, d = 1, 6, 2, 4
    D = H * d
    rng = np.random.default_rng(2)
    qkv = rng.standard_normal((B, T, 3 * D))
    qkv[:, :, D:2 * D] = qkv[:, :1, D:2 * D]
    out = dit.attention(qkv, H)
    assert np.allclose(out, np.broadcast_to(qkv[:, :, 2 * D:].mean(axis=1, keepdims=True), out.shape))


def test_timestep_embedding_closed_forms():
    e = dit.timestep_embedding([0, 500], 256)
    assert e.shape == (2, 256)
    assert np.all(e[0, :128] == 1.0) and np.all(e[0, 128:] == 0.0)
    assert math.isclose(e[1, 0], math.cos(500.0)) and math.isclose(e[1, 128], math.sin(500.0))
    j = 64                                        # f_64 = 10^-2
    assert math.isclose(e[1, j], math.cos(5.0), rel_tol=1e-12)
    assert math.isclose(e[1, 128 + j], math.sin(5.0), rel_tol=1e-12)
    assert np.allclose(e[:, :128] ** 2 + e[:, 128:] ** 2, 1.0)


def test_patchify_vs_torch_unfold_and_unpatchify_inverse():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 4, 8, 6))
    got = dit.patchify(x, 2)
    want = F.unfold(torch.from_numpy(x), kernel_size=2, stride=2).transpose(1, 2).numpy()
    assert np.array_equal(got, want)
    # unpatchify places feature (ph, pw, c) of token (i, j) at pixel (c, i*p+ph, j*p+pw)
    tok = rng.standard_normal((2, 12, 2 * 2 * 8))
    img = dit.unpatchify(tok, 2, 8, 8, 6)
    for (b, i, j, ph, pw, c) in [(0, 0, 0, 0, 0, 0), (1, 3, 2, 1, 0, 5), (0, 2, 1, 1, 1, 7)]:
        assert img[b, c, i * 2 + ph, j * 2 + pw] == tok[b, i * 3 + j, (ph * 2 + pw) * 8 + c]


# ------------------------------------------------ the block, un-quantised
class _TorchBlock:
    """The adaLN-Zero block written with torch library ops only."""

    def __init__(self, bw, heads):
        self.w = {k: torch.from_numpy(v.astype(np.float64)) for k, v in bw.items()}
        self.h = heads

    def __call__(self, x, c):
        w = self.w
        x = torch.from_numpy(x); c = torch.from_numpy(c)
        B, T, D = x.shape
        mod = F.linear(F.silu(c), w["ada_w"], w["ada_b"])
        sm, cm, gm, sl, cl, gl = mod.chunk(6, dim=1)
        h = F.layer_norm(x, (D,), eps=1e-6) * (1 + cm.unsqueeze(1)) + sm.unsqueeze(1)
        qkv = F.linear(h, w["qkv_w"], w["qkv_b"]).reshape(B, T, 3, self.h, D // self.h).permute(2, 0, 3, 1, 4)
        o = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2]).transpose(1, 2).reshape(B, T, D)
        x = x + gm.unsqueeze(1) * F.linear(o, w["proj_w"], w["proj_b"])
        h2 = F.layer_norm(x, (D,), eps=1e-6) * (1 + cl.unsqueeze(1)) + sl.unsqueeze(1)
        m = F.linear(F.gelu(F.linear(h2, w["fc1_w"], w["fc1_b"]), approximate="tanh"), w["fc2_w"], w["fc2_b"])
        return (x + gl.unsqueeze(1) * m).numpy()


def test_fp_block_vs_torch_library_block(exact_storage):
    w, _, _ = _tiny_setup()
    rng = np.random.default_rng(4)
    x = rng.standard_normal((2, TINY.tokens, TINY.hidden))
    c = rng.standard_normal((2, TINY.hidden))
    got = dit.block_full(x, c, 1, TINY.heads, dit.FPLinears(w))
    want = _TorchBlock(w["blocks"][1], TINY.heads)(x, c)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)


def _qparams_for(w, x_lat, lab, t):
    qp, ranges = sampler.calibrate(TINY, w, x_lat, lab, t)
    return qp, ranges


def test_quantised_block_close_to_fp_and_converges_with_bits(exact_storage):
    w, lat, lab = _tiny_setup()
    t = np.array([500, 500, 500])
    qp8, ranges = _qparams_for(w, lat, lab, t)
    assert set(ranges) == {(b, s) for b in range(TINY.depth) for s in dit.SITES}
    fp = dit.denoiser(lat, t, lab, TINY, w, dit.FPLinears(w), {}, True)
    e8 = dit.denoiser(lat, t, lab, TINY, w, dit.QLinears(w, qp8, 8, 8), {}, True)
    qp16 = {k: quant.act_qparams(lo, hi, 16) for k, (lo, hi) in ranges.items()}

    class Fine(dit.QLinears):
        def __init__(self, weights, qparams):
            self.qparams = qparams; self.act_bits = 16; self.taps = None
            self.lin = []
            for b in weights["blocks"]:
                d = {}
                for s in dit.SITES:
                    lin = quant.QLinear.__new__(quant.QLinear)
                    W = b[s + "_w"]; qmax = 2 ** 15 - 1
                    lin.bits = 16
                    lin.scale = (np.abs(W).max(axis=1) / np.float32(qmax)).astype(np.float32)
                    lin.q = np.clip(np.rint(W / lin.scale[:, None]), -qmax, qmax).astype(np.int64)
                    lin.wsum = lin.q.sum(axis=1); lin.bias = b[s + "_b"]
                    d[s] = lin
                self.lin.append(d)

    e16 = dit.denoiser(lat, t, lab, TINY, w, Fine(w, qp16), {}, True)
    r8 = np.sqrt(np.mean((e8 - fp) ** 2)) / np.sqrt(np.mean(fp ** 2))
    r16 = np.sqrt(np.mean((e16 - fp) ** 2)) / np.sqrt(np.mean(fp ** 2))
    assert r8 < 5e-2 and r16 < r8 / 50


def test_block_is_identity_when_gates_are_zero():
    w, _, _ = _tiny_setup()
    D = TINY.hidden
    bw = w["blocks"][0]
    bw["ada_w"][2 * D:3 * D] = 0; bw["ada_b"][2 * D:3 * D] = 0      # gate_msa
    bw["ada_w"][5 * D:6 * D] = 0; bw["ada_b"][5 * D:6 * D] = 0      # gate_mlp
    rng = np.random.default_rng(5)
    x = dit.st(rng.standard_normal((2, TINY.tokens, D))); c = rng.standard_normal((2, D))      # a stored (float32) stream
    qp = {(0, s): quant.act_qparams(-4, 4) for s in dit.SITES}
    out = dit.block_full(x, c, 0, TINY.heads, dit.QLinears(w, qp))
    assert np.array_equal(out, x)


# ---------------------------------------------------------------- cache
def test_cached_step_equals_full_step_on_fresh_cache_bitwise():
    w, lat, lab = _tiny_setup()
    t = np.array([500, 500, 500])
    qp, _ = _qparams_for(w, lat, lab, t)
    lin = dit.QLinears(w, qp)
    cache = {}
    full = dit.denoiser(lat, t, lab, TINY, w, lin, cache, True)
    assert set(cache) == {(b, k) for b in range(TINY.depth) for k in ("attn", "mlp")}
    again = dit.denoiser(lat, t, lab, TINY, w, lin, cache, False)
    assert np.array_equal(full, again)
    # at another timestep only the gates change: the result differs from both
    other = dit.denoiser(lat, t - 20, lab, TINY, w, lin, cache, False)
    assert not np.array_equal(other, full)


@pytest.mark.parametrize("St,N", [(50, 2), (100, 3), (250, 5), (7, 3), (5, 1)])
def test_refresh_count(St, N):
    n = sum(sampler.is_refresh_step(i, N) for i in range(St))
    assert n == -(-St // N) and sampler.is_refresh_step(0, N)


def test_interval_one_is_no_cache():
    w, lat, lab = _tiny_setup()
    t = np.array([500, 500, 500])
    qp, _ = _qparams_for(w, lat, lab, t)
    a = sampler.sample(lat, lab, 5, 1, TINY, w, dit.QLinears(w, qp))
    # reference run: every step forced full with a throw-away cache
    tt, at, ap = sampler.ddim_schedule(5)
    x = lat.astype(np.float64)
    for i in range(5):
        x, _ = sampler.sample_step(x, lab, i, int(tt[i]), at[i], ap[i], TINY, w, dit.QLinears(w, qp), {}, 1,
                                   force_full=True)
    assert np.array_equal(a, x)


def test_per_module_schedule_special_cases():
    """The per-(block, module) schedule: all ones is the full step, all zeros the cached step, the schedule
    built from the interval rule is the interval sampler, and recomputing one module on an unchanged input
    reproduces its stored output (so a mixed step on a fresh cache equals the full step) - all bitwise."""
    w, lat, lab = _tiny_setup()
    t = np.array([500, 500, 500])
    qp, _ = _qparams_for(w, lat, lab, t)
    lin = dit.QLinears(w, qp)
    L = TINY.depth
    cache = {}
    full = dit.denoiser(lat, t, lab, TINY, w, lin, cache, True)
    ones, zeros = np.ones((L, 2), bool), np.zeros((L, 2), bool)
    assert np.array_equal(dit.denoiser(lat, t, lab, TINY, w, lin, {}, ones), full)
    assert np.array_equal(dit.denoiser(lat, t, lab, TINY, w, lin, dict(cache), zeros), full)
    for sched in ([[1, 0]] * L, [[0, 1]] * L, [[1, 0], [0, 1]][:L] + [[0, 0]] * (L - 2)):
        c2 = {k: v.copy() for k, v in cache.items()}
        assert np.array_equal(dit.denoiser(lat, t, lab, TINY, w, lin, c2, np.array(sched, bool)), full)
    # at another timestep a recomputed module differs from its stored output, and is stored again
    c3 = {k: v.copy() for k, v in cache.items()}
    sched = np.zeros((L, 2), bool)
    sched[0, 1] = True
    mixed = dit.denoiser(lat, t - 40, lab, TINY, w, lin, c3, sched)
    cached = dit.denoiser(lat, t - 40, lab, TINY, w, lin, dict(cache), False)
    assert not np.array_equal(mixed, cached)
    assert not np.array_equal(c3[(0, "mlp")], cache[(0, "mlp")]) and np.array_equal(c3[(0, "attn")], cache[(0, "attn")])
    # the interval rule written as a mask
    steps, N = 7, 3
    mask = np.zeros((steps, L, 2), bool)
    mask[::N] = True
    a = sampler.sample(lat, lab, steps, N, TINY, w, lin)
    b = sampler.sample(lat, lab, steps, 1, TINY, w, lin, mask=mask)
    assert np.array_equal(a, b)


def test_bf16_cache_variant():
    """Reduced-precision cache: the refresh step itself is unchanged (it uses the exact module outputs), what it
    stores is the bfloat16 rounding of what the fp32 cache stores, and a cached step differs from the fp32-cache
    one by at most the rounding of the stored tensors times the gates."""
    w, lat, lab = _tiny_setup()
    t = np.array([500, 500, 500])
    qp, _ = _qparams_for(w, lat, lab, t)
    lin = dit.QLinears(w, qp)
    c32, c16 = {}, {}
    f32 = dit.denoiser(lat, t, lab, TINY, w, lin, c32, True)
    f16 = dit.denoiser(lat, t, lab, TINY, w, lin, c16, True, cache_bf16=True)
    assert np.array_equal(f32, f16)
    for k in c32:
        assert np.array_equal(c16[k], quant.bf16_round(c32[k]))
        assert not np.array_equal(c16[k], c32[k])
    a = dit.denoiser(lat, t - 20, lab, TINY, w, lin, c32, False)
    b = dit.denoiser(lat, t - 20, lab, TINY, w, lin, c16, False, cache_bf16=True)
    assert not np.array_equal(a, b)
    assert np.sqrt(np.mean((a - b) ** 2)) <= 2.0 ** -8 * np.sqrt(np.mean(a ** 2)) * 4
    # the sampler threads the option through
    s32 = sampler.sample(lat, lab, 6, 2, TINY, w, lin)
    s16 = sampler.sample(lat, lab, 6, 2, TINY, w, lin, cache_bf16=True)
    assert not np.array_equal(s32, s16) and np.sqrt(np.mean((s32 - s16) ** 2)) < 2e-2 * np.sqrt(np.mean(s32 ** 2))


def test_cached_run_differs_but_tracks_uncached_run():
    w, lat, lab = _tiny_setup()
    qp, _ = _qparams_for(w, lat, lab, np.array([500, 500, 500]))
    a = sampler.sample(lat, lab, 6, 1, TINY, w, dit.QLinears(w, qp))
    b = sampler.sample(lat, lab, 6, 2, TINY, w, dit.QLinears(w, qp))
    assert not np.array_equal(a, b)
    assert np.sqrt(np.mean((a - b) ** 2)) < 0.2 * np.sqrt(np.mean(a ** 2))


# --------------------------------------------------------------- solver
def test_abar_table_and_schedule():
    ab = sampler.abar_table()
    want = torch.cumprod(1 - torch.linspace(1e-4, 2e-2, 1000, dtype=torch.float64), 0).numpy()
    assert np.allclose(ab, want, rtol=1e-13)
    assert math.isclose(ab[0], 1 - 1e-4) and np.all(np.diff(ab) < 0) and 3.9e-5 < ab[-1] < 4.2e-5
    t, at, ap = sampler.ddim_schedule(50)
    assert list(t[:3]) == [980, 960, 940] and t[-1] == 0 and len(t) == 50
    assert ap[-1] == 1.0 and np.array_equal(ap[:-1], at[1:]) and np.array_equal(at, ab[t])


def test_ddim_identity_and_exact_denoise_and_hand_case():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((2, 4, 8, 8))
    assert np.allclose(sampler.ddim_update(x, np.zeros_like(x), 0.3, 0.3), x, rtol=1e-15)
    # if eps is the true noise, a jump to abar_prev = 1 returns x0 exactly
    x0 = rng.standard_normal(x.shape); eps = rng.standard_normal(x.shape); ab = 0.37
    xt = math.sqrt(ab) * x0 + math.sqrt(1 - ab) * eps
    assert np.allclose(sampler.ddim_update(xt, eps, ab, 1.0), x0, atol=1e-13)
    # and a jump to another noise level lands on the same (x0, eps) line
    assert np.allclose(sampler.ddim_update(xt, eps, ab, 0.81), 0.9 * x0 + math.sqrt(0.19) * eps, atol=1e-13)
    # hand case: x=1, eps=0.5, abar_t=0.25, abar_prev=0.64: x0=(1-sqrt(.75)/2)/0.5, out=0.8 x0+0.6*0.5
    x0h = (1 - math.sqrt(0.75) * 0.5) / 0.5
    assert math.isclose(float(sampler.ddim_update(np.array(1.0), np.array(0.5), 0.25, 0.64)), 0.8 * x0h + 0.3)


def test_cfg_combine_special_cases():
    a = np.array([1.0, 2.0]); b = np.array([0.5, -1.0])
    assert np.array_equal(sampler.cfg_combine(a, b, 1.0), a)
    assert np.array_equal(sampler.cfg_combine(a, b, 0.0), b)
    assert np.allclose(sampler.cfg_combine(a, b, 1.5), 1.5 * a - 0.5 * b)


# -------------------------------------------------------------------- VC
def test_vc_identity_mean_variance_and_collapse():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((3, 4, 8, 8)) * 2 + 0.7
    assert np.array_equal(sampler.vc_correct(x, np.ones(4)), x)          # K = 1: bitwise identity
    K = np.array([0.9, 1.0, 1.1, 0.5])
    y = sampler.vc_correct(x, K)
    assert np.allclose(y.mean(axis=(2, 3)), x.mean(axis=(2, 3)), atol=1e-14)      # Eq. 9: mean kept
    assert np.allclose(y.var(axis=(2, 3)), x.var(axis=(2, 3)) * K[None, :] ** 2)   # variance times K^2
    z = sampler.vc_correct(x, np.zeros(4))
    assert np.allclose(z, np.broadcast_to(x.mean(axis=(2, 3), keepdims=True), x.shape))
    # caller-supplied mu reading: mu + K (x - mu)
    mu = np.array([0.1, 0.2, 0.3, 0.4])
    y2 = sampler.vc_correct(x, K, mu)
    assert np.allclose(y2, mu.reshape(1, 4, 1, 1) + K.reshape(1, 4, 1, 1) * (x - mu.reshape(1, 4, 1, 1)))


def test_vc_matches_gaussian_rescale_statistically():
    # Eq. 9: f ~ N(mu, sigma^2) rescaled with sigma_new/sigma has std sigma_new
    rng = np.random.default_rng(8)
    f = rng.normal(1.5, 2.0, size=(1, 1, 400, 400))
    y = sampler.vc_correct(f, np.array([0.25]))
    assert abs(y.std() - 0.5) < 5e-3 and abs(y.mean() - 1.5) < 2e-2


def test_guidance_step_uses_null_label_for_second_half(exact_storage):
    w, lat, lab = _tiny_setup()
    qp, _ = _qparams_for(w, lat, lab, np.array([500, 500, 500]))
    lin = dit.QLinears(w, qp)
    x1, eps = sampler.sample_step(lat.astype(np.float64), lab, 0, 500, 0.3, 0.4, TINY, w, lin, {}, 2, cfg_scale=1.5)
    ec = dit.denoiser(lat, np.full(3, 500), lab, TINY, w, lin, {}, True)
    eu = dit.denoiser(lat, np.full(3, 500), np.full(3, TINY.num_classes), TINY, w, lin, {}, True)
    assert np.allclose(eps, eu + 1.5 * (ec - eu), atol=1e-14)


# ------------------------------------- head, tail and calibration of the network
class _TorchDiT:
    """The whole un-quantised network (the cited DiT architecture) written with torch library
    routines only: conv2d patch embedding, embedding lookup, linear / silu / layer_norm, scaled-dot-
    product attention, fold for the un-patchify.  Returns the noise estimate and, per block, the
    inputs of the five linears (the quantiser sites)."""

    def __init__(self, w, desc):
        self.w = {k: torch.from_numpy(np.asarray(v, dtype=np.float64)) for k, v in w.items() if k != "blocks"}
        self.blocks = [{k: torch.from_numpy(v.astype(np.float64)) for k, v in b.items()} for b in w["blocks"]]
        self.d = desc

    def cond(self, t, y):
        w, half = self.w, self.d.freq_dim // 2
        freqs = torch.pow(torch.tensor(10000.0, dtype=torch.float64), -torch.arange(half, dtype=torch.float64) / half)
        args = torch.as_tensor(np.asarray(t), dtype=torch.float64)[:, None] * freqs[None]
        emb = torch.cat([torch.cos(args), torch.sin(args)], dim=1)
        te = F.linear(F.silu(F.linear(emb, w["t_w1"], w["t_b1"])), w["t_w2"], w["t_b2"])
        return te + F.embedding(torch.as_tensor(np.asarray(y), dtype=torch.long), w["label_table"])

    def embed(self, x):
        w, d = self.w, self.d
        k = w["patch_w"].reshape(d.hidden, d.latent_c, d.patch, d.patch)
        tok = F.conv2d(torch.from_numpy(np.asarray(x, dtype=np.float64)), k, w["patch_b"], stride=d.patch)
        return tok.flatten(2).transpose(1, 2) + w["pos"][None]

    def final(self, x, c):
        w, d = self.w, self.d
        p, C2 = d.patch, 2 * d.latent_c
        shift, scale = F.linear(F.silu(c), w["fada_w"], w["fada_b"]).chunk(2, dim=1)
        h = F.layer_norm(x, (d.hidden,), eps=1e-6) * (1 + scale.unsqueeze(1)) + shift.unsqueeze(1)
        out = F.linear(h, w["flin_w"], w["flin_b"])                      # [B, T, p*p*2C], features (ph, pw, c)
        B, T, _ = out.shape
        cols = out.reshape(B, T, p, p, C2).permute(0, 4, 2, 3, 1).reshape(B, C2 * p * p, T)   # fold wants (c, ph, pw)
        img = F.fold(cols, output_size=(d.latent_h, d.latent_w), kernel_size=p, stride=p)
        return img[:, :d.latent_c]

    def forward(self, x, t, y):
        c = self.cond(t, y)
        h = self.embed(x)
        sites = []
        for bw in self.blocks:
            B, T, D = h.shape
            H = self.d.heads
            a_in = F.silu(c)
            sm, cm, gm, sl, cl, gl = F.linear(a_in, bw["ada_w"], bw["ada_b"]).chunk(6, dim=1)
            q_in = F.layer_norm(h, (D,), eps=1e-6) * (1 + cm.unsqueeze(1)) + sm.unsqueeze(1)
            qkv = F.linear(q_in, bw["qkv_w"], bw["qkv_b"]).reshape(B, T, 3, H, D // H).permute(2, 0, 3, 1, 4)
            p_in = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2]).transpose(1, 2).reshape(B, T, D)
            h = h + gm.unsqueeze(1) * F.linear(p_in, bw["proj_w"], bw["proj_b"])
            f1_in = F.layer_norm(h, (D,), eps=1e-6) * (1 + cl.unsqueeze(1)) + sl.unsqueeze(1)
            f2_in = F.gelu(F.linear(f1_in, bw["fc1_w"], bw["fc1_b"]), approximate="tanh")
            h = h + gl.unsqueeze(1) * F.linear(f2_in, bw["fc2_w"], bw["fc2_b"])
            sites.append({"ada": a_in, "qkv": q_in, "proj": p_in, "fc1": f1_in, "fc2": f2_in})
        return self.final(h, c).numpy(), sites


def test_conditioning_vs_torch_library(exact_storage):
    w, _, _ = _tiny_setup()
    t = np.array([0, 37, 999]); y = np.array([3, 0, TINY.num_classes])          # last row of the table = null label
    got = dit.conditioning(t, y, w)
    want = _TorchDiT(w, TINY).cond(t, y).numpy()
    assert got.shape == (3, TINY.hidden) and np.allclose(got, want, rtol=1e-11, atol=1e-13)
    # each label moves the vector by exactly the difference of its table rows; the timestep part is shared
    other = dit.conditioning(t, np.array([4, 0, 1]), w)
    assert np.allclose(other[0] - got[0], w["label_table"][4].astype(np.float64) - w["label_table"][3])
    assert np.array_equal(other[1], got[1])
    # the hidden layer of the timestep MLP has a SiLU: zeroing the second layer's weights leaves bias + label row only
    w2 = dict(w); w2["t_w2"] = np.zeros_like(w["t_w2"])
    assert np.allclose(dit.conditioning(t, y, w2), w["t_b2"].astype(np.float64) + w["label_table"][y])


def test_embed_vs_conv2d_patch_embedding(exact_storage):
    w, lat, _ = _tiny_setup()
    got = dit.embed(lat, w, TINY.patch)
    want = _TorchDiT(w, TINY).embed(lat).numpy()
    assert got.shape == (3, TINY.tokens, TINY.hidden) and np.allclose(got, want, rtol=1e-11, atol=1e-13)
    # a zero latent embeds to bias + position table
    z = dit.embed(np.zeros_like(lat), w, TINY.patch)
    assert np.allclose(z, (w["patch_b"].astype(np.float64) + w["pos"].astype(np.float64))[None])
    # one hot pixel (c, i*p+ph, j*p+pw) excites column (c, ph, pw) of the kernel in token i*gw+j only
    p, gw = TINY.patch, TINY.latent_w // TINY.patch
    x1 = np.zeros((1, TINY.latent_c, TINY.latent_h, TINY.latent_w)); x1[0, 2, 1 * p + 1, 3 * p + 0] = 1.0
    d = dit.embed(x1, w, p) - z[:1]
    col = w["patch_w"].astype(np.float64)[:, (2 * p + 1) * p + 0]
    assert np.allclose(d[0, 1 * gw + 3], col) and np.count_nonzero(np.abs(d).sum(-1)) == 1


def test_final_layer_vs_torch_library_and_closed_forms(exact_storage):
    w, _, _ = _tiny_setup()
    rng = np.random.default_rng(12)
    x = rng.standard_normal((2, TINY.tokens, TINY.hidden)); c = rng.standard_normal((2, TINY.hidden))
    got = dit.final_layer(x, c, w, TINY.patch, TINY.latent_c, TINY.latent_h, TINY.latent_w)
    want = _TorchDiT(w, TINY).final(torch.from_numpy(x), torch.from_numpy(c)).numpy()
    assert got.shape == (2, TINY.latent_c, TINY.latent_h, TINY.latent_w)
    assert np.allclose(got, want, rtol=1e-10, atol=1e-12)
    # zero linear weights: every pixel shows the bias of its (ph, pw, c) feature, c among the FIRST C of the 2C channels
    w0 = dict(w); w0["flin_w"] = np.zeros_like(w["flin_w"])
    e = dit.final_layer(x, c, w0, TINY.patch, TINY.latent_c, TINY.latent_h, TINY.latent_w)
    p, C = TINY.patch, TINY.latent_c
    for (ch, r, col) in [(0, 0, 0), (3, 5, 2), (1, 7, 7)]:
        assert e[1, ch, r, col] == np.float64(w["flin_b"][((r % p) * p + (col % p)) * 2 * C + ch])
    # modulation: first half of the adaLN output is the shift, second half the scale (scale = -1 wipes the normalised
    # activations, shift = s then makes every feature s, so the output is s * row-sums of the linear + bias)
    D = TINY.hidden
    w1 = dict(w); w1["fada_w"] = np.zeros_like(w["fada_w"])
    w1["fada_b"] = np.concatenate([np.full(D, 0.25, np.float32), np.full(D, -1.0, np.float32)])
    e1 = dit.final_layer(x, c, w1, p, C, TINY.latent_h, TINY.latent_w)
    feat = 0.25 * w["flin_w"].astype(np.float64).sum(axis=1) + w["flin_b"]
    assert np.allclose(e1[0, 2, 4, 5], feat[((4 % p) * p + (5 % p)) * 2 * C + 2])


def test_fp_denoiser_vs_torch_library_network(exact_storage):
    w, lat, lab = _tiny_setup()
    t = np.array([500, 20, 980])
    got = dit.denoiser(lat, t, lab, TINY, w, dit.FPLinears(w), {}, True)
    want, _ = _TorchDiT(w, TINY).forward(lat, t, lab)
    assert np.allclose(got, want, rtol=1e-9, atol=1e-11)


def test_calibration_ranges_are_site_inputs_over_all_calibration_data(exact_storage):
    """Eq. 2 on calibration data: for every (block, site) the range is the min / max of that linear's INPUT, taken
    over all calibration samples together; Eq. 3 then gives (s, z).  The inputs come from the torch-library network."""
    w, lat, lab = _tiny_setup()
    t = np.array([980, 500, 20])
    qp, ranges = sampler.calibrate(TINY, w, lat, lab, t)
    net = _TorchDiT(w, TINY)
    per_sample = [net.forward(lat[n:n + 1], t[n:n + 1], lab[n:n + 1])[1] for n in range(3)]
    for blk in range(TINY.depth):
        for site in dit.SITES:
            lo = min(float(s[blk][site].min()) for s in per_sample)
            hi = max(float(s[blk][site].max()) for s in per_sample)
            glo, ghi = ranges[(blk, site)]
            assert math.isclose(glo, lo, rel_tol=1e-9, abs_tol=1e-12) and math.isclose(ghi, hi, rel_tol=1e-9, abs_tol=1e-12)
            s, z = qp[(blk, site)]
            ws, wz = quant.act_qparams(lo, hi)
            assert z == wz and math.isclose(float(s), float(ws), rel_tol=1e-6)
            # the range covers 0 and the grid reaches both ends (reading of Eq. 2-3 pinned in the quantiser tests)
            assert float(s) * (0 - z) <= min(lo, 0) + float(s) / 2 and float(s) * (255 - z) >= max(hi, 0) - float(s) / 2
    # a single sample gives a narrower (or equal) range everywhere, and strictly narrower somewhere
    _, r1 = sampler.calibrate(TINY, w, lat[:1], lab[:1], t[:1])
    assert all(r1[k][0] >= ranges[k][0] and r1[k][1] <= ranges[k][1] for k in ranges)
    assert any(r1[k] != ranges[k] for k in ranges)


def test_calibrate_block_ranges_vs_torch_block_inputs(exact_storage):
    w, _, _ = _tiny_setup()
    rng = np.random.default_rng(13)
    tok = rng.standard_normal((3, TINY.tokens, TINY.hidden)); cond = rng.standard_normal((3, TINY.hidden))
    qp, ranges = sampler.calibrate_block(TINY, w, tok, cond)
    bw = {k: torch.from_numpy(v.astype(np.float64)) for k, v in w["blocks"][0].items()}
    x, c = torch.from_numpy(tok), torch.from_numpy(cond)
    D, H = TINY.hidden, TINY.heads
    sm, cm, gm, sl, cl, gl = F.linear(F.silu(c), bw["ada_w"], bw["ada_b"]).chunk(6, dim=1)
    q_in = F.layer_norm(x, (D,), eps=1e-6) * (1 + cm.unsqueeze(1)) + sm.unsqueeze(1)
    qkv = F.linear(q_in, bw["qkv_w"], bw["qkv_b"]).reshape(3, TINY.tokens, 3, H, D // H).permute(2, 0, 3, 1, 4)
    p_in = F.scaled_dot_product_attention(qkv[0], qkv[1], qkv[2]).transpose(1, 2).reshape(3, TINY.tokens, D)
    x2 = x + gm.unsqueeze(1) * F.linear(p_in, bw["proj_w"], bw["proj_b"])
    f1_in = F.layer_norm(x2, (D,), eps=1e-6) * (1 + cl.unsqueeze(1)) + sl.unsqueeze(1)
    f2_in = F.gelu(F.linear(f1_in, bw["fc1_w"], bw["fc1_b"]), approximate="tanh")
    want = {"ada": F.silu(c), "qkv": q_in, "proj": p_in, "fc1": f1_in, "fc2": f2_in}
    assert set(ranges) == {(0, s) for s in dit.SITES}
    for site, v in want.items():
        assert np.allclose(ranges[(0, site)], (float(v.min()), float(v.max())), rtol=1e-9, atol=1e-12)
        assert qp[(0, site)][1] == quant.act_qparams(float(v.min()), float(v.max()))[1]


def test_storage_format_rounds_the_stored_tensors_only():
    """Default storage: every tensor kept between two operations is a float32 value, and the result stays within
    float32 rounding of the pure-float64 evaluation of the same formulas."""
    w, lat, lab = _tiny_setup()
    t = np.array([500, 20, 980])
    with dit.storage("f64"):
        c64 = dit.conditioning(t, lab, w); e64 = dit.embed(lat, w, TINY.patch)
        fp64 = dit.denoiser(lat, t, lab, TINY, w, dit.FPLinears(w), {}, True)
    c32 = dit.conditioning(t, lab, w); e32 = dit.embed(lat, w, TINY.patch)
    cache, taps = {}, []
    qp, _ = sampler.calibrate(TINY, w, lat, lab, t)
    fp32 = dit.denoiser(lat, t, lab, TINY, w, dit.FPLinears(w), {}, True)
    dit.denoiser(lat, t, lab, TINY, w, dit.QLinears(w, qp), cache, True, taps)
    f32_exact = lambda a: np.array_equal(np.asarray(a, dtype=np.float32).astype(np.float64), a)
    assert f32_exact(c32) and f32_exact(e32) and f32_exact(fp32) and not f32_exact(c64)
    assert all(f32_exact(v) for v in cache.values())
    assert all(f32_exact(tp[k]) for tp in taps for k in ("qkv", "A", "Mo", "x"))
    assert not any(f32_exact(tp[k]) for tp in taps for k in ("h", "o", "u", "g"))      # quantised where produced, never stored
    assert np.allclose(c32, c64, rtol=1e-5, atol=1e-7) and not np.array_equal(c32, c64)
    assert np.allclose(e32, e64, rtol=1e-7, atol=1e-9) and np.allclose(fp32, fp64, rtol=1e-4, atol=1e-6)
    assert dit.st(np.float64(1.0) + 2.0 ** -30) == 1.0
    with dit.storage("f64"):
        assert dit.st(np.float64(1.0) + 2.0 ** -30) != 1.0
    x1, _ = sampler.sample_step(lat.astype(np.float64), lab, 0, 500, 0.3, 0.4, TINY, w, dit.QLinears(w, qp), {}, 2, K_t=np.full(4, 0.97))
    assert f32_exact(x1)


def test_bf16_stream_format_rounds_the_token_tensor_only():
    """stream_format("bf16"): the embedding's output and the residual stream after every gated add are bfloat16
    values (8 significant bits: the low 16 bits of their float32 pattern are zero), every other stored tensor keeps
    float32, and the noise estimate stays within bfloat16 rounding of the float32-stream one.  The rounding itself
    is pinned bit by bit: ties go to the even 16-bit pattern, 1 + 2^-8 rounds down to 1, 1 + 3 * 2^-8 up to 1 + 2^-6."""
    w, lat, lab = _tiny_setup()
    t = np.array([500, 20, 980])
    qp, _ = sampler.calibrate(TINY, w, lat, lab, t)
    is_bf16 = lambda a: np.all((np.asarray(a, dtype=np.float32).view(np.uint32) & 0xFFFF) == 0) and np.array_equal(
        np.asarray(a, dtype=np.float32).astype(np.float64), a)
    f32_exact = lambda a: np.array_equal(np.asarray(a, dtype=np.float32).astype(np.float64), a)
    taps32, taps16 = [], []
    e32 = dit.denoiser(lat, t, lab, TINY, w, dit.QLinears(w, qp), {}, True, taps32)
    with dit.stream_format("bf16"):
        assert dit.st_x(1.0 + 2.0 ** -8) == 1.0 and dit.st_x(1.0 + 3 * 2.0 ** -8) == 1.0 + 2.0 ** -6
        assert dit.st_x(1.0 + 2.0 ** -8 + 2.0 ** -20) == 1.0 + 2.0 ** -7          # above the tie: up
        assert dit.st(1.0 + 2.0 ** -8) == 1.0 + 2.0 ** -8                            # other tensors: float32
        tok = dit.embed(lat, w, TINY.patch)
        cache = {}
        e16 = dit.denoiser(lat, t, lab, TINY, w, dit.QLinears(w, qp), cache, True, taps16)
        e16c = dit.denoiser(lat, t, lab, TINY, w, dit.QLinears(w, qp), cache, False)
    assert is_bf16(tok) and all(is_bf16(tp["x"]) for tp in taps16)
    assert all(f32_exact(tp[k]) and not is_bf16(tp[k]) for tp in taps16 for k in ("qkv", "A", "Mo"))
    assert not any(is_bf16(tp["x"]) for tp in taps32)
    assert f32_exact(e16) and not np.array_equal(e16, e32)
    # bfloat16 keeps 8 bits: the stream's relative error is 2^-9 per store, the estimate moves by a few times that
    rel = lambda a, b: np.sqrt(np.mean((a - b) ** 2) / np.mean(b ** 2))
    assert rel(e16, e32) < 5e-2 and rel(e16c, e16) < 1.0
    assert dit.st_x(1.0 + 2.0 ** -8) == 1.0 + 2.0 ** -8                              # back to float32 outside the block
