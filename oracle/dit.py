"""Oracle: the class-conditional DiT denoiser with quantised linears and the
attention / MLP output cache.  Test infrastructure.  float64 throughout.

The paper does not define the network; it uses the DiT-XL/2 of the DiT paper
it cites (Experimental Settings).  Conventions of that architecture followed
here: adaLN-Zero block; LayerNorm without affine, eps 1e-6, biased variance;
modulate(h) = h*(1+scale) + shift; six modulation chunks in the order
(shift_msa, scale_msa, gate_msa, shift_mlp, scale_mlp, gate_mlp); SiLU before
every adaLN linear; tanh-GELU; softmax(QK^T/sqrt(d)); 256-wide sinusoidal
timestep embedding [cos | sin] with frequencies exp(-ln(1e4) j/128); learned
sigma (2C output channels, the noise estimate is the first C).

What is quantised (Comparison on Performance section: channel-wise weights,
tensor-wise activations): the inputs and weights of the five linears of each
block - adaLN projection, QKV, attention output projection, MLP fc1 and fc2.
Embedders, attention products, softmax, LayerNorm and the final layer stay in
floating point.

What is cached ("outputs from self-attention and MLP layers", same section):
the output of the attention projection and of fc2, bias included, before the
adaLN gate.  A cached block recomputes only the gates at the current timestep.

Storage precision (the paper fixes none): every tensor the sampler keeps in
memory between two operations - conditioning vectors, tokens, modulation
vectors, Q | K | V, the module outputs that are cached, the residual stream
after every gated add, the noise estimate - is a float32 tensor; `st()` below
rounds to it.  The arithmetic between two stored tensors is float64 (exact
integer contractions, float64 everywhere else).  Values that are quantised
right where they are produced (LayerNorm + modulation output, attention
output, GELU output) are never stored: Eq. 1 rounds the float64 value to
float32 once and decides there.  `storage("f64")` switches the rounding off
(used to check the formulas against library routines to 1e-10).

Reduced-precision residual stream (not in the paper: a storage variant that
halves the bytes every block reads and writes of it): under
`stream_format("bf16")` the token tensor - the patch embedding's output and
the residual stream after every gated add - is stored as bfloat16 (`st_x()`:
the float64 value rounded to float32, then to bfloat16, ties to even); every
other stored tensor keeps float32.
"""
from __future__ import annotations

import numpy as np

from .quant import QLinear, lin_q, bf16_round

import contextlib

SITES = ("ada", "qkv", "proj", "fc1", "fc2")
F64 = np.float64
_STORE_F32 = True


def st(x):
    """The value of x after it is stored as a float32 tensor."""
    x = np.asarray(x, dtype=F64)
    return x.astype(np.float32).astype(F64) if _STORE_F32 else x


_STREAM_BF16 = False


def st_x(x):
    """The value of the token tensor / residual stream x after it is stored (float32, or bfloat16 under
    stream_format("bf16"))."""
    return bf16_round(st(x)) if (_STREAM_BF16 and _STORE_F32) else st(x)


@contextlib.contextmanager
def stream_format(kind: str):
    """stream_format("bf16"): the residual stream is stored as bfloat16; stream_format("f32"): the default."""
    global _STREAM_BF16
    old = _STREAM_BF16
    _STREAM_BF16 = {"f32": False, "bf16": True}[kind]
    try:
        yield
    finally:
        _STREAM_BF16 = old


@contextlib.contextmanager
def storage(kind: str):
    """storage("f64"): stored tensors keep float64 (pure mathematics); storage("f32"): the default."""
    global _STORE_F32
    old = _STORE_F32
    _STORE_F32 = {"f32": True, "f64": False}[kind]
    try:
        yield
    finally:
        _STORE_F32 = old


# ------------------------------------------------------------ linear modes
class FPLinears:
    """Un-quantised linears; records the min / max of every quantiser site's
    input (used to derive (s, z) from calibration data, Eq. 2)."""

    def __init__(self, weights: dict):
        self.w = weights
        self.ranges: dict = {}

    def __call__(self, blk: int, site: str, a: np.ndarray) -> np.ndarray:
        lo, hi = float(a.min()), float(a.max())
        old = self.ranges.get((blk, site))
        self.ranges[(blk, site)] = (lo, hi) if old is None else (min(old[0], lo), max(old[1], hi))
        W = self.w["blocks"][blk][site + "_w"].astype(F64)
        b = self.w["blocks"][blk][site + "_b"].astype(F64)
        return a @ W.T + b


class QLinears:
    """Quantised linears with static per-site activation parameters."""

    def __init__(self, weights: dict, qparams: dict, weight_bits: int = 8, act_bits: int = 8):
        self.qparams = qparams
        self.act_bits = act_bits
        self.lin = [{s: QLinear(b[s + "_w"], b[s + "_b"], weight_bits) for s in SITES}
                    for b in weights["blocks"]]
        self.taps: dict | None = None      # set to {} to record codes / accumulators

    def __call__(self, blk: int, site: str, a: np.ndarray) -> np.ndarray:
        s, z = self.qparams[(blk, site)]
        tap = None
        if self.taps is not None:
            tap = self.taps.setdefault((blk, site), {})
        return lin_q(a, self.lin[blk][site], s, z, self.act_bits, tap)


# --------------------------------------------------------------- primitives
def silu(x):
    return x / (1.0 + np.exp(-x))


def gelu_tanh(x):
    return 0.5 * x * (1.0 + np.tanh(np.sqrt(2.0 / np.pi) * (x + 0.044715 * x ** 3)))


def layer_norm(x, eps: float = 1e-6):
    mu = x.mean(axis=-1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=-1, keepdims=True)
    return (x - mu) / np.sqrt(var + eps)


def modulate(h, shift, scale):
    return h * (1.0 + scale[:, None, :]) + shift[:, None, :]


def attention(qkv, heads: int):
    """softmax(Q K^T / sqrt(d)) V per (batch, head).  qkv[B, T, 3D] holds
    Q | K | V, each split head-major into d = D/heads columns per head."""
    B, T, D3 = qkv.shape
    D = D3 // 3
    d = D // heads
    q, k, v = (qkv[:, :, i * D:(i + 1) * D].reshape(B, T, heads, d).transpose(0, 2, 1, 3)
               for i in range(3))
    s = (q @ k.transpose(0, 1, 3, 2)) / np.sqrt(F64(d))
    s = s - s.max(axis=-1, keepdims=True)
    p = np.exp(s)
    p = p / p.sum(axis=-1, keepdims=True)
    o = p @ v
    return o.transpose(0, 2, 1, 3).reshape(B, T, D)


# ------------------------------------------------------------------- blocks
def block_mod(c, blk: int, linear):
    """adaLN projection of a block: Lin(SiLU(c)) split into its six chunks."""
    mod = st(linear(blk, "ada", silu(c)))
    return np.split(mod, 6, axis=1)


def block_full(x, c, blk: int, heads: int, linear, cache: dict | None = None, tap: dict | None = None,
               cache_bf16: bool = False):
    """One adaLN-Zero DiT block, fully computed; stores the attention and MLP
    module outputs into `cache` when given (rounded to bfloat16 storage with
    cache_bf16; the block itself always uses the exact module outputs)."""
    B, T, D = x.shape
    shift_msa, scale_msa, gate_msa, shift_mlp, scale_mlp, gate_mlp = block_mod(c, blk, linear)
    h = modulate(layer_norm(x), shift_msa, scale_msa)
    qkv = st(linear(blk, "qkv", h.reshape(B * T, D))).reshape(B, T, 3 * D)
    o = attention(qkv, heads)
    A = st(linear(blk, "proj", o.reshape(B * T, D))).reshape(B, T, D)
    x = st_x(x + gate_msa[:, None, :] * A)
    h2 = modulate(layer_norm(x), shift_mlp, scale_mlp)
    u = linear(blk, "fc1", h2.reshape(B * T, D))
    g = gelu_tanh(u)
    Mo = st(linear(blk, "fc2", g)).reshape(B, T, D)
    x = st_x(x + gate_mlp[:, None, :] * Mo)
    if cache is not None:
        cache[(blk, "attn")] = bf16_round(A) if cache_bf16 else A
        cache[(blk, "mlp")] = bf16_round(Mo) if cache_bf16 else Mo
    if tap is not None:
        tap.update(h=h, qkv=qkv, o=o, A=A, h2=h2, u=u, g=g, Mo=Mo, x=x)
    return x


def block_cached(x, c, blk: int, linear, cache: dict):
    """A block on a non-refresh step: the stored module outputs are reused and
    only the gates come from the current conditioning."""
    _, _, gate_msa, _, _, gate_mlp = block_mod(c, blk, linear)
    x = st_x(x + gate_msa[:, None, :] * cache[(blk, "attn")])
    x = st_x(x + gate_mlp[:, None, :] * cache[(blk, "mlp")])
    return x


def block_mixed(x, c, blk: int, heads: int, linear, cache: dict, attn_full: bool, mlp_full: bool,
                cache_bf16: bool = False):
    """A block under a per-module cache schedule (the cache rule of the
    "Quantization and Cache" section applied module by module, as a learned
    layer-caching policy would): each of the two modules is either recomputed,
    which also refreshes its stored output, or replaced by its stored output;
    gates always come from the current conditioning."""
    B, T, D = x.shape
    shift_msa, scale_msa, gate_msa, shift_mlp, scale_mlp, gate_mlp = block_mod(c, blk, linear)
    if attn_full:
        h = modulate(layer_norm(x), shift_msa, scale_msa)
        qkv = st(linear(blk, "qkv", h.reshape(B * T, D))).reshape(B, T, 3 * D)
        A = st(linear(blk, "proj", attention(qkv, heads).reshape(B * T, D))).reshape(B, T, D)
        cache[(blk, "attn")] = bf16_round(A) if cache_bf16 else A
    else:
        A = cache[(blk, "attn")]
    x = st_x(x + gate_msa[:, None, :] * A)
    if mlp_full:
        h2 = modulate(layer_norm(x), shift_mlp, scale_mlp)
        Mo = st(linear(blk, "fc2", gelu_tanh(linear(blk, "fc1", h2.reshape(B * T, D))))).reshape(B, T, D)
        cache[(blk, "mlp")] = bf16_round(Mo) if cache_bf16 else Mo
    else:
        Mo = cache[(blk, "mlp")]
    x = st_x(x + gate_mlp[:, None, :] * Mo)
    return x


# ------------------------------------------------- embedders and final layer
def timestep_embedding(t, dim: int = 256):
    t = np.asarray(t, dtype=F64).reshape(-1)
    half = dim // 2
    freqs = np.exp(-np.log(10000.0) * np.arange(half, dtype=F64) / half)
    args = t[:, None] * freqs[None, :]
    return np.concatenate([np.cos(args), np.sin(args)], axis=1)


def conditioning(t, y, w: dict):
    """c = MLP(sinusoid(t)) + label_table[y]."""
    e = st(timestep_embedding(t, w["t_w1"].shape[1]))
    h = st(silu(e @ w["t_w1"].astype(F64).T + w["t_b1"].astype(F64)))
    te = st(h @ w["t_w2"].astype(F64).T + w["t_b2"].astype(F64))
    return st(te + w["label_table"].astype(F64)[np.asarray(y, dtype=np.int64)])


def patchify(x, p: int):
    """x[B, C, H, W] -> [B, T, C*p*p]; token = (row-patch, col-patch) row-major,
    features ordered (c, ph, pw)."""
    B, C, H, W = x.shape
    x = x.reshape(B, C, H // p, p, W // p, p)
    return x.transpose(0, 2, 4, 1, 3, 5).reshape(B, (H // p) * (W // p), C * p * p)


def unpatchify(tok, p: int, c_out: int, H: int, W: int):
    """tok[B, T, p*p*c_out] (features ordered (ph, pw, c)) -> [B, c_out, H, W]."""
    B = tok.shape[0]
    gh, gw = H // p, W // p
    t = tok.reshape(B, gh, gw, p, p, c_out)
    return t.transpose(0, 5, 1, 3, 2, 4).reshape(B, c_out, H, W)


def embed(x_lat, w: dict, p: int):
    tok = patchify(np.asarray(x_lat, dtype=F64), p)
    return st_x(tok @ w["patch_w"].astype(F64).T + w["patch_b"].astype(F64) + w["pos"].astype(F64)[None])


def final_layer(x, c, w: dict, p: int, C: int, H: int, W: int):
    """adaLN-modulated LayerNorm, linear to p*p*2C features, unpatchify; returns
    the noise estimate = first C of the 2C channels."""
    mod = st(silu(c) @ w["fada_w"].astype(F64).T + w["fada_b"].astype(F64))
    shift, scale = np.split(mod, 2, axis=1)
    h = modulate(layer_norm(x), shift, scale)
    out = st(h @ w["flin_w"].astype(F64).T + w["flin_b"].astype(F64))
    img = unpatchify(out, p, 2 * C, H, W)
    return img[:, :C]


def denoiser(x_lat, t, y, desc, w: dict, linear, cache: dict, full: bool, taps: list | None = None,
             cache_bf16: bool = False):
    """Noise estimate of the network for latents x_lat[B, C, H, W] at timesteps
    t[B] with labels y[B].  `full` = True recomputes every block and refreshes
    the cache, False reuses it in every block; an array [depth, 2] of booleans
    decides per (block, module) with module 0 = attention, 1 = MLP."""
    c = conditioning(t, y, w)
    x = embed(x_lat, w, desc.patch)
    if not isinstance(full, (bool, np.bool_)):
        sched = np.asarray(full, dtype=bool).reshape(desc.depth, 2)
        for blk in range(desc.depth):
            x = block_mixed(x, c, blk, desc.heads, linear, cache, bool(sched[blk, 0]), bool(sched[blk, 1]), cache_bf16)
        return final_layer(x, c, w, desc.patch, desc.latent_c, desc.latent_h, desc.latent_w)
    for blk in range(desc.depth):
        if full:
            tap = None
            if taps is not None:
                tap = {}
                taps.append(tap)
            x = block_full(x, c, blk, desc.heads, linear, cache, tap, cache_bf16)
        else:
            x = block_cached(x, c, blk, linear, cache)
    return final_layer(x, c, w, desc.patch, desc.latent_c, desc.latent_h, desc.latent_w)
