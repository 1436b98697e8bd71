"""ctypes binding of include/qc.h: same names, argument marshalling only.

Tensors are torch CUDA (ROCm) tensors; the binding passes their data pointers
and the current torch stream.  There is no fallback: importing fails loudly if
libqc.so has not been built (python paper_2503_02508_amd/build.py)."""
from __future__ import annotations

import ctypes as C
import os

__all__ = [
    "lib", "QCError", "ModelDesc", "Context", "QC_FULL", "QC_CACHED", "QC_CACHE_ATTN", "QC_CACHE_MLP", "SITES",
    "qc_quantize_act", "qc_quantize_weight", "qc_w8a8_linear", "qc_vc_correct", "qc_vc_fit", "qc_vc_fit_static", "qc_ddim_schedule", "last_error",
    "LIB_PATH", "WS", "KERNEL_CLASSES",
    "qc_tap_workspace_bytes", "qc_tap_similarity", "qc_tap_normalise", "qc_tap_embed", "qc_tap_kmeans",
    "qc_tap_aggregate", "qc_tap_cluster", "qc_tap_profile_begin", "qc_tap_profile_end",
]

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libqc.so")
if not os.path.exists(LIB_PATH):
    raise ImportError("libqc.so is missing: build it with `python paper_2503_02508_amd/build.py` "
                      "(there is no CPU fallback)")
lib = C.CDLL(LIB_PATH)

QC_FULL, QC_CACHED = 0, 1
QC_CACHE_ATTN, QC_CACHE_MLP = 0, 1
SITES = ("ada", "qkv", "proj", "fc1", "fc2")
WS = {"tokens": 0, "qact_ln": 1, "qact_attn": 2, "qact_mlp": 3, "qkv": 4, "mod": 5, "cond": 6, "eps": 7, "qkv_heads": 8}

vp, i32, f32, f64, sz = C.c_void_p, C.c_int, C.c_float, C.c_double, C.c_size_t


class ModelDesc(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("depth", "hidden", "heads", "mlp_dim", "patch", "latent_c", "latent_h",
                                         "latent_w", "num_classes", "freq_dim", "weight_bits", "cache_interval")]


class BlockWeights(C.Structure):
    _fields_ = [(n, vp) for n in ("ada_w", "ada_b", "qkv_w", "qkv_b", "proj_w", "proj_b", "fc1_w", "fc1_b",
                                  "fc2_w", "fc2_b")]


class Weights(C.Structure):
    _fields_ = [(n, vp) for n in ("patch_w", "patch_b", "pos", "t_w1", "t_b1", "t_w2", "t_b2", "label_table",
                                  "fada_w", "fada_b", "flin_w", "flin_b")] + [("blocks", C.POINTER(BlockWeights))]


_SIGS = {
    "qc_last_error": (C.c_char_p, []),
    "qc_arena_bytes": (i32, [C.POINTER(ModelDesc), i32, C.POINTER(sz)]),
    "qc_create": (i32, [C.POINTER(ModelDesc), vp, sz, i32, C.POINTER(vp)]),
    "qc_destroy": (i32, [vp]),
    "qc_load_weights_f32": (i32, [vp, C.POINTER(Weights), vp]),
    "qc_set_act_qparams": (i32, [vp, i32, i32, f32, i32]),
    "qc_get_act_qparams": (i32, [vp, i32, i32, C.POINTER(f32), C.POINTER(i32)]),
    "qc_calibrate_minmax": (i32, [vp, C.POINTER(Weights), vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), i32, vp]),
    "qc_quantize_act": (i32, [vp, vp, sz, f32, i32, vp]),
    "qc_quantize_weight": (i32, [vp, i32, i32, i32, vp, vp, vp, vp]),
    "qc_w8a8_linear": (i32, [vp, vp, vp, vp, vp, f32, i32, i32, i32, i32, i32, vp, vp, vp]),
    "qc_vc_correct": (i32, [vp, vp, vp, i32, i32, i32, i32, vp]),
    "qc_set_cache_mask": (i32, [vp, vp, i32]),
    "qc_set_cache_format": (i32, [vp, i32]),
    "qc_vc_fit": (i32, [vp, vp, i32, i32, i32, i32, f32, vp, vp, vp]),
    "qc_vc_fit_static": (i32, [vp, vp, i32, i32, i32, i32, f32, vp, vp]),
    "qc_denoise_f32": (i32, [vp, C.POINTER(Weights), vp, i32, vp, i32, i32, vp, vp]),
    "qc_vc_fit_sampler": (i32, [vp, C.POINTER(Weights), vp, vp, vp, i32, i32, f32, f32, vp, vp]),
    "qc_ddim_schedule": (i32, [i32, C.POINTER(C.c_int32), C.POINTER(f64), C.POINTER(f64)]),
    "qc_dit_block": (i32, [vp, i32, i32, vp, vp, i32, vp]),
    "qc_cache_store": (i32, [vp, i32, i32, vp, i32, vp]),
    "qc_cache_reuse": (i32, [vp, i32, i32, vp, vp, i32, i32, vp]),
    "qc_cache_ptr": (i32, [vp, i32, i32, C.POINTER(vp)]),
    "qc_workspace_ptr": (i32, [vp, i32, C.POINTER(vp), C.POINTER(sz)]),
    "qc_denoise": (i32, [vp, vp, i32, vp, i32, i32, i32, vp, vp]),
    "qc_sample_step": (i32, [vp, vp, vp, i32, i32, i32, f64, f64, f32, vp, i32, vp]),
    "qc_sample": (i32, [vp, vp, vp, i32, i32, f32, vp, vp]),
    "qc_keep_qkv_f32": (i32, [vp, i32]),
    "qc_check": (i32, [vp, vp]),
    "qc_set_stream_format": (i32, [vp, i32]),
    "qc_tap_workspace_bytes": (i32, [i32, i32, i32, i32, i32, C.POINTER(sz)]),
    "qc_tap_similarity": (i32, [vp, vp, i32, i32, vp, i32, f32, vp, vp, vp, vp, sz, vp]),
    "qc_tap_normalise": (i32, [vp, vp, vp, i32, i32, vp, sz, vp]),
    "qc_tap_embed": (i32, [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]),
    "qc_tap_kmeans": (i32, [vp, i32, i32, i32, vp, i32, vp, vp, C.POINTER(i32), vp, sz, vp]),
    "qc_tap_aggregate": (i32, [vp, i32, i32, i32, vp, vp, vp, sz, vp]),
    "qc_tap_cluster": (i32, [vp, vp, i32, i32, vp, i32, i32, f32, i32, i32, i32, vp, vp, i32, vp, vp, vp, sz, vp]),
    "qc_tap_profile_begin": (i32, []),
    "qc_tap_profile_end": (i32, [C.POINTER(f32), C.POINTER(i32)]),
    "qc_profile_begin": (i32, [vp]),
    "qc_profile_end": (i32, [vp, i32, C.POINTER(C.c_int32), C.POINTER(f32), vp]),
}
KERNEL_CLASSES = ("gemm_adaln", "ln_mod_quant", "gemm_qkv", "attention", "gemm_proj", "gemm_fc1", "gemm_fc2",
                  "cached_blocks", "ddim_vc")
for _n, (_r, _a) in _SIGS.items():
    _f = getattr(lib, _n)
    _f.restype, _f.argtypes = _r, _a


class QCError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("qc error %d: %s" % (code, msg))
        self.code = code


def last_error() -> str:
    return lib.qc_last_error().decode()


def _chk(rc):
    if rc != 0:
        raise QCError(rc, last_error())


def _p(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


# ---------------------------------------------------------------- single ops
def qc_quantize_act(x, q, scale: float, zero_point: int):
    _chk(lib.qc_quantize_act(_p(x), _p(q), x.numel(), scale, zero_point, _stream()))


def qc_quantize_weight(w, bits, qw, w_scale, wsum):
    N, K = w.shape
    _chk(lib.qc_quantize_weight(_p(w), N, K, bits, _p(qw), _p(w_scale), _p(wsum), _stream()))


def qc_w8a8_linear(qx, qw, wsum, w_scale, bias, x_scale, x_zp, weight_bits, y, acc=None):
    M, K = qx.shape
    N = qw.shape[0]
    _chk(lib.qc_w8a8_linear(_p(qx), _p(qw), _p(wsum), _p(w_scale), _p(bias), x_scale, x_zp, M, N, K, weight_bits,
                            _p(y), _p(acc), _stream()))


def qc_vc_fit(x_hat, x_ref, eps, work, K_t):
    B, Cc, H, W = x_hat.shape
    _chk(lib.qc_vc_fit(_p(x_hat), _p(x_ref), B, Cc, H, W, float(eps), _p(work), _p(K_t), _stream()))


def qc_vc_fit_static(x_hat, x_ref, eps, K_t):
    B, Cc, H, W = x_hat.shape
    _chk(lib.qc_vc_fit_static(_p(x_hat), _p(x_ref), B, Cc, H, W, float(eps), _p(K_t), _stream()))


def qc_vc_correct(x, K_t, mu=None):
    B, Cc, H, W = x.shape
    _chk(lib.qc_vc_correct(_p(x), _p(K_t), _p(mu), B, Cc, H, W, _stream()))


# ------------------------------------------------ calibration-set clustering (include/qc_tap.h)
def qc_tap_workspace_bytes(N, F, n, k, kb) -> int:
    out = sz()
    _chk(lib.qc_tap_workspace_bytes(N, F, n, k, kb, C.byref(out)))
    return out.value


def _wb(work):
    return work.numel() * work.element_size()


def qc_tap_similarity(X, t, idx, alpha, A, d_r, d_c, work):
    N, F = X.shape
    _chk(lib.qc_tap_similarity(_p(X), _p(t), N, F, _p(idx), idx.numel(), float(alpha), _p(A), _p(d_r), _p(d_c),
                               _p(work), _wb(work), _stream()))


def qc_tap_normalise(A, d_r, d_c, work):
    N, n = A.shape
    _chk(lib.qc_tap_normalise(_p(A), _p(d_r), _p(d_c), N, n, _p(work), _wb(work), _stream()))


def qc_tap_embed(L, k, iters, q0, U, sigma, work):
    N, n = L.shape
    _chk(lib.qc_tap_embed(_p(L), N, n, k, q0.shape[0], iters, _p(q0), _p(U), _p(sigma), _p(work), _wb(work), _stream()))


def qc_tap_kmeans(U, init_idx, max_iter, labels, centres, work) -> int:
    N, d = U.shape
    passes = i32(0)
    _chk(lib.qc_tap_kmeans(_p(U), N, d, init_idx.numel(), _p(init_idx), max_iter, _p(labels), _p(centres),
                           C.byref(passes), _p(work), _wb(work), _stream()))
    return passes.value


def qc_tap_aggregate(labels, k, out, work, perm_out=None):
    m, N = labels.shape
    _chk(lib.qc_tap_aggregate(_p(labels), m, N, k, _p(out), _p(perm_out), _p(work), _wb(work), _stream()))


def qc_tap_cluster(X, t, subsamples, alpha, k, iters, q0, init_idx, max_iter, labels_out, per_labels, work):
    N, F = X.shape
    m, n = subsamples.shape
    _chk(lib.qc_tap_cluster(_p(X), _p(t), N, F, _p(subsamples), m, n, float(alpha), k, q0.shape[0], iters, _p(q0),
                            _p(init_idx), max_iter, _p(labels_out), _p(per_labels), _p(work), _wb(work), _stream()))


def qc_tap_profile_begin():
    _chk(lib.qc_tap_profile_begin())


def qc_tap_profile_end():
    """(summed milliseconds, launches) of the similarity contraction since qc_tap_profile_begin."""
    ms, n = f32(0), i32(0)
    _chk(lib.qc_tap_profile_end(C.byref(ms), C.byref(n)))
    return ms.value, n.value


def qc_ddim_schedule(steps: int):
    t = (C.c_int32 * steps)()
    a = (f64 * steps)()
    b = (f64 * steps)()
    _chk(lib.qc_ddim_schedule(steps, t, a, b))
    return list(t), list(a), list(b)


# ------------------------------------------------------------------ context
class Context:
    """Owns the device arena (a torch uint8 tensor) and the qc_ctx handle."""

    def __init__(self, model, max_batch: int, cache_interval: int = 1):
        import torch
        self.desc = ModelDesc(model.depth, model.hidden, model.heads, model.mlp_dim, model.patch, model.latent_c,
                              model.latent_h, model.latent_w, model.num_classes, model.freq_dim, model.weight_bits,
                              cache_interval)
        self.model = model
        self.max_batch = max_batch
        n = sz()
        _chk(lib.qc_arena_bytes(C.byref(self.desc), max_batch, C.byref(n)))
        self.arena = torch.empty(n.value + 256, dtype=torch.uint8, device="cuda")
        base = (self.arena.data_ptr() + 255) & ~255
        self.h = vp()
        _chk(lib.qc_create(C.byref(self.desc), vp(base), n.value, max_batch, C.byref(self.h)))
        self._keep = None
        self._cache_bf16 = False

    def close(self):
        if self.h:
            lib.qc_destroy(self.h)
            self.h = vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # weights: dict of numpy fp32 arrays as produced by synthetic.dit_inputs.make_weights
    def _marshal_weights(self, w):
        import torch
        dev = {k: torch.from_numpy(v).cuda() for k, v in w.items() if k != "blocks"}
        blocks = [{k: torch.from_numpy(v).cuda() for k, v in b.items()} for b in w["blocks"]]
        arr = (BlockWeights * len(blocks))()
        for i, b in enumerate(blocks):
            for k, _ in BlockWeights._fields_:
                setattr(arr[i], k, b[k].data_ptr())
        ws = Weights()
        for k, _ in Weights._fields_:
            if k != "blocks":
                setattr(ws, k, dev[k].data_ptr())
        ws.blocks = C.cast(arr, C.POINTER(BlockWeights))
        return ws, (dev, blocks, arr)

    def load_weights(self, w, keep_fp32: bool = False):
        import torch
        ws, keep = self._marshal_weights(w)
        _chk(lib.qc_load_weights_f32(self.h, C.byref(ws), _stream()))
        torch.cuda.synchronize()
        if keep_fp32:
            self._keep = (ws, keep)

    def calibrate(self, x, t, y):
        """x: cuda float32 [n, C, H, W]; t, y: python int sequences."""
        if self._keep is None:
            raise QCError(-5, "load_weights(..., keep_fp32=True) is needed before calibrate")
        n = x.shape[0]
        ta = (C.c_int32 * n)(*[int(v) for v in t])
        ya = (C.c_int32 * n)(*[int(v) for v in y])
        _chk(lib.qc_calibrate_minmax(self.h, C.byref(self._keep[0]), _p(x), ta, ya, n, _stream()))

    def denoise_f32(self, x, t, labels, B, eps_out):
        if self._keep is None:
            raise QCError(-5, "load_weights(..., keep_fp32=True) is needed before denoise_f32")
        _chk(lib.qc_denoise_f32(self.h, C.byref(self._keep[0]), _p(x), int(t), _p(labels), labels.numel(), B, _p(eps_out),
                                _stream()))

    def vc_fit_sampler(self, x_hat, x_ref, labels, steps, cfg_scale, vc_eps, K_out):
        if self._keep is None:
            raise QCError(-5, "load_weights(..., keep_fp32=True) is needed before vc_fit_sampler")
        _chk(lib.qc_vc_fit_sampler(self.h, C.byref(self._keep[0]), _p(x_hat), _p(x_ref), _p(labels), x_hat.shape[0], steps,
                                   float(cfg_scale), float(vc_eps), _p(K_out), _stream()))

    def drop_fp32(self):
        self._keep = None

    def set_act_qparams(self, block, site, scale, zp):
        _chk(lib.qc_set_act_qparams(self.h, block, site, float(scale), int(zp)))

    def get_act_qparams(self, block, site):
        s, z = f32(), i32()
        _chk(lib.qc_get_act_qparams(self.h, block, site, C.byref(s), C.byref(z)))
        return s.value, z.value

    def set_cache_mask(self, mask):
        """mask: numpy array [steps, depth, 2] of 0/1 (1 = recompute), or None for the interval rule."""
        if mask is None:
            _chk(lib.qc_set_cache_mask(self.h, None, 0))
            return
        import numpy as np
        m = np.ascontiguousarray(np.asarray(mask, dtype=np.uint8))
        _chk(lib.qc_set_cache_mask(self.h, m.ctypes.data_as(vp), m.shape[0]))

    def keep_qkv_f32(self, on=True):
        _chk(lib.qc_keep_qkv_f32(self.h, int(on)))

    def set_stream_format(self, fmt):
        """"fp32" (default) or "bf16": storage of the residual stream inside denoise / sample_step / sample."""
        _chk(lib.qc_set_stream_format(self.h, {"fp32": 0, "bf16": 1}[fmt]))

    def check(self):
        """Waits for the current stream; raises if a kernel flagged an out-of-range class label since the last call."""
        _chk(lib.qc_check(self.h, _stream()))

    def dit_block(self, block, mode, x, c):
        _chk(lib.qc_dit_block(self.h, block, mode, _p(x), _p(c), x.shape[0], _stream()))

    def cache_store(self, block, which, src):
        _chk(lib.qc_cache_store(self.h, block, which, _p(src), src.shape[0], _stream()))

    def cache_reuse(self, block, which, x, gate):
        _chk(lib.qc_cache_reuse(self.h, block, which, _p(x), _p(gate), gate.stride(0), x.shape[0], _stream()))

    def _view(self, ptr, shape, dtype):
        """Wraps arena memory at `ptr` as a tensor (a view of self.arena)."""
        import torch
        off = ptr - self.arena.data_ptr()
        n = 1
        for s in shape:
            n *= s
        nbytes = n * torch.empty((), dtype=dtype).element_size()
        return self.arena[off:off + nbytes].view(dtype).view(*shape)

    def cache_tensor(self, block, which, B):
        import torch
        p = vp()
        _chk(lib.qc_cache_ptr(self.h, block, which, C.byref(p)))
        m = self.model
        return self._view(p.value, (B, m.tokens, m.hidden), torch.bfloat16 if self._cache_bf16 else torch.float32)

    def set_cache_format(self, fmt):
        """fmt: "fp32" (default) or "bf16"."""
        code = {"fp32": 0, "bf16": 1}[fmt]
        _chk(lib.qc_set_cache_format(self.h, code))
        self._cache_bf16 = code == 1

    def workspace(self, name, shape, dtype):
        p, n = vp(), sz()
        _chk(lib.qc_workspace_ptr(self.h, WS[name], C.byref(p), C.byref(n)))
        return self._view(p.value, shape, dtype)

    def denoise(self, x, t, labels, B, mode, eps_out):
        _chk(lib.qc_denoise(self.h, _p(x), int(t), _p(labels), labels.numel(), B, mode, _p(eps_out), _stream()))

    def sample_step(self, x, labels, step_index, t, abar_t, abar_prev, cfg_scale=0.0, K_t=None, force_mode=-1):
        _chk(lib.qc_sample_step(self.h, _p(x), _p(labels), x.shape[0], step_index, int(t), abar_t, abar_prev,
                                cfg_scale, _p(K_t), force_mode, _stream()))

    def profile_pass(self, fn):
        """Runs fn() with per-launch event timing on; returns {class: {name, launches, total_ms}}."""
        n = len(KERNEL_CLASSES)
        cnt, ms = (C.c_int32 * n)(), (f32 * n)()
        _chk(lib.qc_profile_begin(self.h))
        try:
            fn()
        finally:
            _chk(lib.qc_profile_end(self.h, n, cnt, ms, _stream()))
        return {k: {"name": k, "launches": int(cnt[i]), "total_ms": float(ms[i])}
                for i, k in enumerate(KERNEL_CLASSES) if cnt[i]}

    def sample(self, x, labels, steps, cfg_scale=0.0, K=None):
        _chk(lib.qc_sample(self.h, _p(x), _p(labels), x.shape[0], steps, cfg_scale, _p(K), _stream()))
