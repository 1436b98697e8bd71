"""Seeded, synthetic DiT-shaped inputs.

Nothing here computes any step of the method (no quantiser, no network layer,
no sampler arithmetic): the functions only describe workload shapes and draw
random tensors.  Both the CPU oracle's callers and the HIP path's callers take
their inputs from here so that the two sides see identical bytes.

Workloads stand in for the paper's ImageNet / pre-trained DiT-XL/2 setting
(Experimental Settings section): shapes are the real architecture's, values
are random draws.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np

FREQ_DIM = 256          # width of the sinusoidal timestep embedding
NUM_CLASSES = 1000      # label table has NUM_CLASSES + 1 rows (last = null label)


@dataclass(frozen=True)
class ModelDesc:
    depth: int
    hidden: int
    heads: int
    mlp_dim: int
    patch: int
    latent_c: int
    latent_h: int
    latent_w: int
    num_classes: int = NUM_CLASSES
    freq_dim: int = FREQ_DIM
    weight_bits: int = 8

    @property
    def tokens(self) -> int:
        return (self.latent_h // self.patch) * (self.latent_w // self.patch)

    @property
    def head_dim(self) -> int:
        return self.hidden // self.heads

    @property
    def patch_dim(self) -> int:
        return self.latent_c * self.patch * self.patch


@dataclass(frozen=True)
class Workload:
    """One benchmark configuration: model + batch + sampler settings + seeds."""
    name: str
    model: ModelDesc
    batch: int              # latents (before classifier-free-guidance doubling)
    steps: int              # sampler steps St
    cache_interval: int     # N
    cfg_scale: float        # <= 0: guidance off
    seed_weights: int
    seed_latents: int
    seed_labels: int
    seed_k: int
    calib_seeds: tuple = (4000, 4001, 4002, 4003)
    fixed_t: int | None = None      # single-step workloads (config 0)


DIT_S2_1BLOCK = ModelDesc(depth=1, hidden=384, heads=6, mlp_dim=1536, patch=2,
                          latent_c=4, latent_h=32, latent_w=32)
DIT_XL2_256 = ModelDesc(depth=28, hidden=1152, heads=16, mlp_dim=4608, patch=2,
                        latent_c=4, latent_h=32, latent_w=32)
DIT_XL2_512 = replace(DIT_XL2_256, latent_h=64, latent_w=64)
DIT_XL2_256_W4 = replace(DIT_XL2_256, weight_bits=4)


def _wl(i, name, model, batch, steps, interval, cfg=0.0, fixed_t=None):
    return Workload(name=name, model=model, batch=batch, steps=steps,
                    cache_interval=interval, cfg_scale=cfg,
                    seed_weights=1000 + i, seed_latents=2000 + i,
                    seed_labels=3000 + i, seed_k=5000 + i, fixed_t=fixed_t)


WORKLOADS = {
    "cfg0": _wl(0, "dit_s2_block_b1", DIT_S2_1BLOCK, 1, 1, 1, fixed_t=500),
    "cfg1": _wl(1, "dit_xl2_256_w8a8_b8_ddim50_n2", DIT_XL2_256, 8, 50, 2),
    "cfg2": _wl(2, "dit_xl2_256_w8a8_b64_cfg_ddim100_n3", DIT_XL2_256, 64, 100, 3, cfg=1.5),
    "cfg3": _wl(3, "dit_xl2_512_w8a8_b16_ddim50_n2", DIT_XL2_512, 16, 50, 2),
    "cfg4": _wl(4, "dit_xl2_256_w4a8_b32_ddim250_n5", DIT_XL2_256_W4, 32, 250, 5),
}


def shrink(model: ModelDesc, depth: int) -> ModelDesc:
    """Same layer shapes, fewer blocks (for parity cases the oracle can finish)."""
    return replace(model, depth=depth)


# --------------------------------------------------------------------------
# random tensors
# --------------------------------------------------------------------------

def _normal(rng: np.random.Generator, shape, std) -> np.ndarray:
    return (rng.standard_normal(size=shape, dtype=np.float32) * np.float32(std))


def _pos_table(model: ModelDesc) -> np.ndarray:
    """Fixed 2-D sine/cosine position table of shape [T, D] (a constant input
    tensor of the network, like any other weight)."""
    gh = model.latent_h // model.patch
    gw = model.latent_w // model.patch
    d = model.hidden
    quarter = d // 4
    omega = 1.0 / (10000.0 ** (np.arange(quarter, dtype=np.float64) / quarter))
    ys, xs = np.meshgrid(np.arange(gh, dtype=np.float64),
                         np.arange(gw, dtype=np.float64), indexing="ij")
    def enc(p):
        a = p.reshape(-1, 1) * omega.reshape(1, -1)
        return np.concatenate([np.sin(a), np.cos(a)], axis=1)
    tab = np.concatenate([enc(xs), enc(ys)], axis=1)
    out = np.zeros((gh * gw, d), dtype=np.float64)
    out[:, :tab.shape[1]] = tab
    return out.astype(np.float32)


def make_weights(model: ModelDesc, seed: int, std: float = 0.02) -> dict:
    """All fp32 parameters of the network, weights and biases ~ N(0, std)."""
    rng = np.random.default_rng(seed)
    D, R = model.hidden, model.mlp_dim
    out_dim = model.patch * model.patch * 2 * model.latent_c
    w = {
        "patch_w": _normal(rng, (D, model.patch_dim), std),
        "patch_b": _normal(rng, (D,), std),
        "pos": _pos_table(model),
        "t_w1": _normal(rng, (D, model.freq_dim), std),
        "t_b1": _normal(rng, (D,), std),
        "t_w2": _normal(rng, (D, D), std),
        "t_b2": _normal(rng, (D,), std),
        "label_table": _normal(rng, (model.num_classes + 1, D), std),
        "fada_w": _normal(rng, (2 * D, D), std),
        "fada_b": _normal(rng, (2 * D,), std),
        "flin_w": _normal(rng, (out_dim, D), std),
        "flin_b": _normal(rng, (out_dim,), std),
        "blocks": [],
    }
    for _ in range(model.depth):
        w["blocks"].append({
            "ada_w": _normal(rng, (6 * D, D), std), "ada_b": _normal(rng, (6 * D,), std),
            "qkv_w": _normal(rng, (3 * D, D), std), "qkv_b": _normal(rng, (3 * D,), std),
            "proj_w": _normal(rng, (D, D), std), "proj_b": _normal(rng, (D,), std),
            "fc1_w": _normal(rng, (R, D), std), "fc1_b": _normal(rng, (R,), std),
            "fc2_w": _normal(rng, (D, R), std), "fc2_b": _normal(rng, (D,), std),
        })
    return w


def make_latents(batch: int, model: ModelDesc, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.standard_normal(size=(batch, model.latent_c, model.latent_h, model.latent_w),
                               dtype=np.float32)


def make_labels(batch: int, model: ModelDesc, seed: int) -> np.ndarray:
    rng = np.random.default_rng(seed)
    return rng.integers(0, model.num_classes, size=(batch,), dtype=np.int32)


def make_vc_factors(steps: int, channels: int, seed: int, lo=0.95, hi=1.0) -> np.ndarray:
    """VC factor table K[St, C]; values slightly below one (the variance of the
    quantised+cached trajectory drifts upwards late in sampling, motivation of
    the variance-compensation section)."""
    rng = np.random.default_rng(seed)
    return rng.uniform(lo, hi, size=(steps, channels)).astype(np.float32)


def make_tokens(batch: int, model: ModelDesc, seed: int, std: float = 1.0) -> np.ndarray:
    """Random residual-stream tokens [B, T, D] for single-block cases."""
    rng = np.random.default_rng(seed)
    return _normal(rng, (batch, model.tokens, model.hidden), std)


def make_cond(batch: int, model: ModelDesc, seed: int, std: float = 1.0) -> np.ndarray:
    """Random conditioning vectors c[B, D] for single-block cases."""
    rng = np.random.default_rng(seed)
    return _normal(rng, (batch, model.hidden), std)


def calibration_inputs(wl: Workload, n: int = 4):
    """The n calibration inputs of a workload: N(0,1) latents from the workload's
    calibration seeds, seeded labels, and the indices of the sampler steps whose
    timesteps they are taken at (first, one third, two thirds, last).  A
    single-step workload uses its fixed timestep for all of them (index -1)."""
    m = wl.model
    lat = np.concatenate([make_latents(1, m, s) for s in wl.calib_seeds[:n]], axis=0)
    lab = make_labels(n, m, wl.seed_labels + 500)
    if wl.fixed_t is not None:
        step_idx = np.full((n,), -1, dtype=np.int32)
    else:
        St = wl.steps
        step_idx = np.array([0, St // 3, (2 * St) // 3, St - 1], dtype=np.int32)[:n]
    return lat, lab, step_idx
