"""Each fused quantiser of a DiT block checked ALONE: the oracle recomputes the value to be quantised from
the device's own upstream tensor (the tensor the kernel actually read), so a differing code can only come from
the arithmetic of that one kernel, not from a difference further upstream.

  * LayerNorm + modulate + quantise (second site): input = the device's residual stream after the attention
    branch (read back with the MLP gate set to zero, which makes the block output equal to it bit for bit) and the
    device's modulation vectors.  Required: the oracle's codes, all of them.
  * GELU + requantise (fc1 epilogue): input = the device's LayerNorm codes; the oracle forms the exact integer
    accumulators from them.  Required: the oracle's codes, all of them.
  * attention + quantise: input = the device's fp32 Q | K | V.  The kernel multiplies fp16 pairs (22 significant
    bits) and exponentiates in fp32, and decides again in float64 where the value sits within that error of a
    rounding boundary.  Required: the oracle's codes, all of them.
  * stored tensors (modulation vectors, Q | K | V, projection and fc2 outputs, residual stream): float32 values that
    must equal the oracle's stored tensors bit for bit, given the device's codes.

Eq. 1 decides in fp32 on both sides: the oracle evaluates the pre-quantiser value in fp64 and rounds it to fp32."""
import numpy as np
import pytest

from oracle import dit, quant, sampler
from synthetic import dit_inputs as I
from qc_testlib import make_pair, code_flip_stats, rel_rms, max_abs, qkv_rows_from_heads

pytestmark = pytest.mark.gpu



def _cuda(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _signed_codes(x, s, z):
    return (quant.quantize(x, s, z) - 128).astype(np.int8)


@pytest.mark.parametrize("name,model,B,wb,std", [
    ("dit_s2", I.DIT_S2_1BLOCK, 2, 8, 0.02),
    ("xl_256", I.DIT_XL2_256, 2, 8, 0.02),
    ("xl_256_w4", I.DIT_XL2_256, 2, 4, 0.02),
    # M = 12288 rows: all four linears take the large-M GEMM kernel (fragment-ordered weights)
    # M = 2048 and 4096 rows: launches on both sides of the tile count from which the large-M kernel takes over
    # (M = 2048: QKV and fc1 large-M, proj and fc2 tile kernel; M = 4096: all four large-M)
    ("xl_256_m2048", I.DIT_XL2_256, 8, 8, 0.02),
    ("xl_256_m4096_w4", I.DIT_XL2_256, 16, 4, 0.02),
    ("xl_256_large_m", I.DIT_XL2_256, 48, 8, 0.02),
    ("xl_256_large_m_w4", I.DIT_XL2_256, 48, 4, 0.02),
    ("ragged", I.ModelDesc(depth=1, hidden=80, heads=4, mlp_dim=176, patch=1, latent_c=3, latent_h=5, latent_w=7,
                           num_classes=7), 3, 8, 0.15),
])
def test_each_fused_quantiser_alone(name, model, B, wb, std):
    import torch
    import paper_2503_02508_amd as qc
    from dataclasses import replace
    model = replace(I.shrink(model, 1), weight_bits=wb)
    seed = 77
    w = I.make_weights(model, seed, std=std)
    D, R, T, H = model.hidden, model.mlp_dim, model.tokens, model.heads
    # gate of the MLP branch = 0: the block's output is then the residual stream after the attention branch
    w["blocks"][0]["ada_w"][5 * D:6 * D] = 0
    w["blocks"][0]["ada_b"][5 * D:6 * D] = 0
    tok = I.make_tokens(B, model, seed + 1)
    cond = I.make_cond(B, model, seed + 2, std=0.5)
    qp, _ = sampler.calibrate_block(model, w, I.make_tokens(4, model, seed + 3), I.make_cond(4, model, seed + 4, std=0.5))
    lin, ctx = make_pair(model, w, qp, B)
    # large launches: Q | K | V are read back from the head-major buffers, so that the QKV GEMM runs without the optional
    # row-major copy, i.e. through the large-M kernel as in the sampler; the small cases read that copy (and check it)
    big = B * T >= 2048
    ctx.keep_qkv_f32(not big)
    x = _cuda(tok)
    ctx.dit_block(0, qc.QC_FULL, x, _cuda(cond))
    torch.cuda.synchronize()
    M = B * T
    x_mid = x.cpu().numpy().astype(np.float64)                                   # device, fp32 values
    mod = ctx.workspace("mod", (ctx.max_batch if ctx.max_batch > 512 else 512, 6 * D), torch.float32).cpu().numpy()[:B].astype(np.float64)
    qkv_heads = qkv_rows_from_heads(ctx, model, B, B).cpu().numpy().astype(np.float64)
    qkv_dev = qkv_heads if big else ctx.workspace("qkv", (M, 3 * D), torch.float32).cpu().numpy().astype(np.float64)
    assert np.array_equal(qkv_dev, qkv_heads), "the head-major Q | K | V differ from the row-major copy"
    c_attn = ctx.workspace("qact_attn", (M, D), torch.int8).cpu().numpy()
    c_ln2 = ctx.workspace("qact_ln", (M, D), torch.int8).cpu().numpy()
    c_gelu = ctx.workspace("qact_mlp", (M, R), torch.int8).cpu().numpy()
    A_dev = ctx.cache_tensor(0, qc.QC_CACHE_ATTN, B).cpu().numpy().reshape(M, D)
    Mo_dev = ctx.cache_tensor(0, qc.QC_CACHE_MLP, B).cpu().numpy().reshape(M, D)
    ctx.close()
    L = lin.lin[0]
    report = {}
    f32 = lambda a: np.asarray(a, dtype=np.float64).astype(np.float32)

    def frac_ne(got, want):
        return float(np.mean(np.asarray(got) != np.asarray(want)))

    # modulation: adaLN projection, stored as float32 -> bit-equal to the oracle's stored tensor
    mod_or = np.concatenate(dit.block_mod(cond.astype(np.float64), 0, lin), axis=1)
    assert np.array_equal(mod.astype(np.float32), f32(mod_or)), "adaLN projection: %.2e of the stored values differ" % frac_ne(mod.astype(np.float32), f32(mod_or))
    assert np.all(mod[:, 5 * D:] == 0)

    # ---- first LayerNorm site, through the stored Q | K | V (bit-equal when its codes are the oracle's)
    s, z = qp[(0, "qkv")]
    h1 = dit.modulate(dit.layer_norm(tok.astype(np.float64)), mod[:, 0:D], mod[:, D:2 * D]).reshape(M, D)
    corr = quant.int_matmul(_signed_codes(h1, s, z), L["qkv"].q) - (z - 128) * L["qkv"].wsum[None]
    qkv_or = (np.float64(np.float32(s)) * L["qkv"].scale.astype(np.float64))[None] * corr + L["qkv"].bias.astype(np.float64)[None]
    rows_off = int(np.count_nonzero(np.any(qkv_dev.astype(np.float32) != f32(qkv_or), axis=1)))
    report["ln1 + qkv rows that differ"] = "%d of %d" % (rows_off, M)
    assert rows_off == 0

    # ---- attention + quantise, from the device's own Q | K | V (the one approximate kernel: fp16-pair products)
    s, z = qp[(0, "proj")]
    o = dit.attention(qkv_dev.reshape(B, T, 3 * D), H).reshape(M, D)
    f_attn = code_flip_stats(c_attn, _signed_codes(o, s, z))
    report["attention codes"] = "%.2e (dist %d)" % f_attn

    # ---- projection output from the device's codes: exact dequantisation, stored as float32
    corr = quant.int_matmul(c_attn, L["proj"].q) - (z - 128) * L["proj"].wsum[None]
    A_or = (np.float64(np.float32(s)) * L["proj"].scale.astype(np.float64))[None] * corr + L["proj"].bias.astype(np.float64)[None]
    report["proj out differing"] = "%.1e" % frac_ne(A_dev, f32(A_or))
    assert np.array_equal(A_dev, f32(A_or))

    # ---- residual after the attention branch: x + gate * A with the device's A (one fused multiply-add; the oracle
    # rounds the float64 sum when it stores it, which differs from the single rounding only at double-rounding ties)
    x_or = tok.astype(np.float64) + mod[:, None, 2 * D:3 * D] * A_dev.reshape(B, T, D).astype(np.float64)
    off = frac_ne(x_mid.astype(np.float32), f32(x_or))
    report["stream differing"] = "%.1e" % off
    assert off <= 1e-6

    # ---- second LayerNorm + modulate + quantise, from the device's residual stream
    s, z = qp[(0, "fc1")]
    h2 = dit.modulate(dit.layer_norm(x_mid), mod[:, 3 * D:4 * D], mod[:, 4 * D:5 * D]).reshape(M, D)
    f_ln2 = code_flip_stats(c_ln2, _signed_codes(h2, s, z))
    report["ln2 codes"] = "%.2e (dist %d)" % f_ln2

    # ---- fc1 + GELU + requantise, from the device's LayerNorm codes
    corr = quant.int_matmul(c_ln2, L["fc1"].q) - (z - 128) * L["fc1"].wsum[None]
    u = (np.float64(np.float32(s)) * L["fc1"].scale.astype(np.float64))[None] * corr + L["fc1"].bias.astype(np.float64)[None]
    s2, z2 = qp[(0, "fc2")]
    f_gelu = code_flip_stats(c_gelu, _signed_codes(dit.gelu_tanh(u), s2, z2))
    report["gelu codes"] = "%.2e (dist %d)" % f_gelu

    # ---- fc2 output from the device's codes
    corr = quant.int_matmul(c_gelu, L["fc2"].q) - (z2 - 128) * L["fc2"].wsum[None]
    Mo_or = (np.float64(np.float32(s2)) * L["fc2"].scale.astype(np.float64))[None] * corr + L["fc2"].bias.astype(np.float64)[None]
    report["fc2 out differing"] = "%.1e" % frac_ne(Mo_dev, f32(Mo_or))
    assert np.array_equal(Mo_dev, f32(Mo_or))

    print(name, "; ".join("%s: %s" % kv for kv in report.items()))
    # LayerNorm (float64 on the device), the fc1 epilogue and the attention kernel (fast path + exact decision near
    # rounding boundaries) give the oracle's codes
    assert f_ln2[0] == 0.0, "second LayerNorm quantiser: %.2e of its codes differ" % f_ln2[0]
    assert f_gelu[0] == 0.0, "GELU quantiser: %.2e of its codes differ" % f_gelu[0]
    assert f_attn[0] == 0.0, "attention quantiser: %.2e of its codes differ" % f_attn[0]


@pytest.mark.parametrize("wb", [8, 4])
def test_large_m_linears_every_tile_at_32768_rows(wb):
    """The four linears of a DiT-XL/2 block at M = 32768 rows (128 latents, the launch shape of the guided workload):
    the large-M GEMM kernel streams activations and weights with hand-counted waits, so a wait that is one load short
    shows up as a few wrong 32-row fragments somewhere in the 4608 tiles and not in a small product.  Four rows of
    every 128-row tile (one per 32-row fragment) are recomputed by the oracle from the device's own upstream codes:
    Q | K | V, projection output, GELU codes and fc2 output must equal it exactly; and a second run from the same
    input must reproduce every stored tensor bit for bit."""
    import torch
    import paper_2503_02508_amd as qc
    from dataclasses import replace
    model = replace(I.shrink(I.DIT_XL2_256, 1), weight_bits=wb)
    B, seed = 128, 91
    w = I.make_weights(model, seed, std=0.02)
    D, R, T = model.hidden, model.mlp_dim, model.tokens
    tok = I.make_tokens(B, model, seed + 1)
    cond = I.make_cond(B, model, seed + 2, std=0.5)
    qp, _ = sampler.calibrate_block(model, w, I.make_tokens(4, model, seed + 3), I.make_cond(4, model, seed + 4, std=0.5))
    lin, ctx = make_pair(model, w, qp, B)
    M = B * T
    rows = (np.arange(M // 128)[:, None] * 128 + np.array([5, 44, 83, 122])[None]).reshape(-1)
    rows_t = torch.from_numpy(rows).cuda()
    L = lin.lin[0]
    f32 = lambda a: np.asarray(a, dtype=np.float64).astype(np.float32)
    cond_d, tok_d = _cuda(cond), _cuda(tok)

    def run():
        x = tok_d.clone()
        ctx.dit_block(0, qc.QC_FULL, x, cond_d)
        torch.cuda.synchronize()
        return dict(x=x.reshape(M, D),
                    qkv=qkv_rows_from_heads(ctx, model, B, B),      # from the head-major buffers: no row-major copy is asked for, so the large-M kernel runs
                    c_attn=ctx.workspace("qact_attn", (M, D), torch.int8).clone(),
                    c_ln2=ctx.workspace("qact_ln", (M, D), torch.int8).clone(),
                    c_gelu=ctx.workspace("qact_mlp", (M, R), torch.int8).clone(),
                    A=ctx.cache_tensor(0, qc.QC_CACHE_ATTN, B).reshape(M, D).clone(),
                    Mo=ctx.cache_tensor(0, qc.QC_CACHE_MLP, B).reshape(M, D).clone())

    first = run()
    mod = ctx.workspace("mod", (512, 6 * D), torch.float32).cpu().numpy()[:B].astype(np.float64)
    for rep in range(3):
        again = run()
        for k in first:
            assert torch.equal(first[k], again[k]), "%s differs between two runs from the same input (run %d)" % (k, rep + 2)
    ctx.close()
    g = {k: v[rows_t].cpu().numpy() for k, v in first.items()}
    bidx = rows // T

    # Q | K | V from the oracle's first-LayerNorm codes of the sampled rows
    s, z = qp[(0, "qkv")]
    xr = tok.reshape(M, D)[rows].astype(np.float64)
    h1 = dit.layer_norm(xr) * (1.0 + mod[bidx, D:2 * D]) + mod[bidx, 0:D]
    corr = quant.int_matmul(_signed_codes(h1, s, z), L["qkv"].q) - (z - 128) * L["qkv"].wsum[None]
    want = (np.float64(np.float32(s)) * L["qkv"].scale.astype(np.float64))[None] * corr + L["qkv"].bias.astype(np.float64)[None]
    assert np.array_equal(g["qkv"], f32(want)), "Q | K | V: %d sampled rows differ" % np.count_nonzero(np.any(g["qkv"] != f32(want), axis=1))
    # projection output from the device's attention codes
    s, z = qp[(0, "proj")]
    corr = quant.int_matmul(g["c_attn"], L["proj"].q) - (z - 128) * L["proj"].wsum[None]
    want = (np.float64(np.float32(s)) * L["proj"].scale.astype(np.float64))[None] * corr + L["proj"].bias.astype(np.float64)[None]
    assert np.array_equal(g["A"], f32(want)), "projection: %d sampled rows differ" % np.count_nonzero(np.any(g["A"] != f32(want), axis=1))
    # GELU codes from the device's second-LayerNorm codes
    s, z = qp[(0, "fc1")]
    corr = quant.int_matmul(g["c_ln2"], L["fc1"].q) - (z - 128) * L["fc1"].wsum[None]
    u = (np.float64(np.float32(s)) * L["fc1"].scale.astype(np.float64))[None] * corr + L["fc1"].bias.astype(np.float64)[None]
    s2, z2 = qp[(0, "fc2")]
    want = _signed_codes(dit.gelu_tanh(u), s2, z2)
    assert np.array_equal(g["c_gelu"], want), "fc1 + GELU: %d sampled rows differ" % np.count_nonzero(np.any(g["c_gelu"] != want, axis=1))
    # fc2 output from the device's GELU codes
    corr = quant.int_matmul(g["c_gelu"], L["fc2"].q) - (z2 - 128) * L["fc2"].wsum[None]
    want = (np.float64(np.float32(s2)) * L["fc2"].scale.astype(np.float64))[None] * corr + L["fc2"].bias.astype(np.float64)[None]
    assert np.array_equal(g["Mo"], f32(want)), "fc2: %d sampled rows differ" % np.count_nonzero(np.any(g["Mo"] != f32(want), axis=1))
