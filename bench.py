#!/usr/bin/env python3
"""Benchmark of the W8A8 + step-cache + VC DiT sampler on one MI355X.

One benchmark "step" is one pass of the whole hot path over one batch: the
complete DDIM sampling loop of the workload (for the default workload: 8
latents, 50 sampler steps, cache refreshed every 2nd step, VC every step), all
inputs resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg1] [--no-cpu-baseline]

`--workload tap1` measures the calibration-set clustering instead (one "step" = the whole algorithm over the sample
pool of the paper's setting); the default run and the headline metric are the sampler's.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_MFMA_PEAK_TOPS = 5000.0     # MI355X dense int8 matrix peak (published), TOP/s
FP16_MFMA_PEAK_TFLOPS = 2500.0   # MI355X dense fp16 matrix peak (published), TFLOP/s
HBM_PEAK_GBS = 8000.0            # MI355X HBM3E peak (published), GB/s
FP32_MFMA_PEAK_TFLOPS = 157.3    # MI355X dense fp32 matrix peak (published), TFLOP/s
TAP_ITERS, TAP_MAX_PASSES = 8, 100   # power-iteration rounds and k-means pass limit of the clustering workload

# HBM bytes per launch of a kernel class from the hardware counters (two rocprofv3 --pmc runs, FETCH_SIZE and
# WRITE_SIZE, scaled by what the same counters read for a copy of known size); filled in from the summaries
# under profiles/, keyed by (workload, kernel class).  None where no counter run covers the pair.
TRAFFIC = {
    # profiles/sampler_cfg1_dit_xl2_b8_hbm_traffic.txt: (FETCH_SIZE * 2.0 + WRITE_SIZE * 1.0) KiB per dispatch
    ("dit_xl2_256_w8a8_b8_ddim50_n2", "gemm_fc2"): (17402.7 * 2.0 + 9216.0) * 1024,
    ("dit_xl2_256_w8a8_b8_ddim50_n2", "gemm_qkv"): (6389.1 * 2.0 + 13824.0) * 1024,
    ("dit_xl2_256_w8a8_b8_ddim50_n2", "gemm_fc1"): (7751.1 * 2.0 + 4608.0) * 1024,
    ("dit_xl2_256_w8a8_b8_ddim50_n2", "gemm_proj"): (6167.5 * 2.0 + 9216.0) * 1024,
    ("dit_xl2_256_w8a8_b8_ddim50_n2", "attention"): (7326.0 * 2.0 + 1536.0) * 1024,
    # profiles/sampler_cfg2_dit_xl2_b64_cfg_hbm_traffic.txt
    ("dit_xl2_256_w8a8_b64_cfg_ddim100_n3", "gemm_fc2"): (332125.0 * 2.0 + 294912.0) * 1024,
    ("dit_xl2_256_w8a8_b64_cfg_ddim100_n3", "gemm_qkv"): (154249.9 * 2.0 + 454764.7) * 1024,
    ("dit_xl2_256_w8a8_b64_cfg_ddim100_n3", "gemm_fc1"): (254733.6 * 2.0 + 147456.0) * 1024,
    ("dit_xl2_256_w8a8_b64_cfg_ddim100_n3", "gemm_proj"): (120028.1 * 2.0 + 294912.0) * 1024,
    ("dit_xl2_256_w8a8_b64_cfg_ddim100_n3", "attention"): (268460.4 * 2.0 + 49152.0) * 1024,
    # profiles/sampler_cfg3_dit_xl2_512_b16_hbm_traffic.txt
    ("dit_xl2_512_w8a8_b16_ddim50_n2", "gemm_fc2"): (147087.0 * 2.0 + 147456.0) * 1024,
    ("dit_xl2_512_w8a8_b16_ddim50_n2", "gemm_qkv"): (76425.0 * 2.0 + 226030.6) * 1024,
    ("dit_xl2_512_w8a8_b16_ddim50_n2", "gemm_fc1"): (124429.6 * 2.0 + 73728.0) * 1024,
    ("dit_xl2_512_w8a8_b16_ddim50_n2", "gemm_proj"): (58563.5 * 2.0 + 147456.0) * 1024,
    ("dit_xl2_512_w8a8_b16_ddim50_n2", "attention"): (143814.6 * 2.0 + 24576.0) * 1024,
    # profiles/clustering_tap1_counters.txt
    ("tap1", "similarity"): (1706789.6 * 2.0 + 279926.8) * 1024,
}


def int8_ops_per_full_step(m, B):
    """int8 multiply-accumulate work (2 ops per MAC) of the five quantised linears of all blocks."""
    M = B * m.tokens
    D, R = m.hidden, m.mlp_dim
    per_block = M * (3 * D * D + D * D + 2 * R * D) + B * 6 * D * D
    return 2 * per_block * m.depth


def cpu_baseline(wl):
    """The CPU oracle, as it stands, on a bounded sample of the same workload:
    one latent, one refresh step and one cached step of the full-depth network;
    scaled to the workload's (refresh, cached) step counts."""
    import numpy as np
    from oracle import dit, sampler
    from synthetic import dit_inputs as I
    m = wl.model
    w = I.make_weights(m, wl.seed_weights)
    clat, clab, idx = I.calibration_inputs(wl, n=1)
    tt, at, ap = sampler.ddim_schedule(wl.steps)
    qp, _ = sampler.calibrate(m, w, clat, clab, tt[idx])
    lin = dit.QLinears(w, qp, m.weight_bits)
    lat = I.make_latents(1, m, wl.seed_latents)
    lab = I.make_labels(1, m, wl.seed_labels)
    K = I.make_vc_factors(wl.steps, m.latent_c, wl.seed_k)
    cache = {}
    x = lat.astype(np.float64)
    times = []
    for i in range(2):
        t0 = time.perf_counter()
        x, _ = sampler.sample_step(x, lab, i, int(tt[i]), at[i], ap[i], m, w, lin, cache, 2, wl.cfg_scale, K[i])
        times.append(time.perf_counter() - t0)
    n_full = -(-wl.steps // wl.cache_interval)
    per_latent = n_full * times[0] + (wl.steps - n_full) * times[1]
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": 1.0 / per_latent, "unit": "latents/sec", "cores": int(cores), "kind": "oracle",
            "sample": "1 latent, 1 refresh step (%.2f s) + 1 cached step (%.2f s) of the full-depth network, "
                      "scaled to %d refresh + %d cached steps" % (times[0], times[1], n_full, wl.steps - n_full)}


def per_shape_rates(model, weight_bits):
    """The four quantised linears, the attention kernel and the LayerNorm + quantise kernel of ONE block of the
    workload's network at M = 2048 and M = 32768 token rows (batch 8 and 128 at 256 tokens), each launch alone on
    the chip (block-level call, one stream), timed with HIP events around every launch: achieved TOP/s (TFLOP/s for
    the attention, GB/s for the bandwidth-bound kernel) per shape."""
    import numpy as np
    import torch
    from dataclasses import replace
    import paper_2503_02508_amd as qc
    from synthetic import dit_inputs as I
    m1 = replace(I.shrink(model, 1), weight_bits=weight_bits)
    w = I.make_weights(m1, 1)
    D, R, T = m1.hidden, m1.mlp_dim, m1.tokens
    out = {}
    for M in (2048, 32768):
        B = M // T
        if B < 1 or B * T != M:
            continue
        ctx = qc.Context(m1, B, 2)
        ctx.load_weights(w)
        for site, (sc, z) in enumerate([(0.01, 128), (0.04, 128), (0.002, 128), (0.04, 128), (0.02, 10)]):
            ctx.set_act_qparams(0, site, sc, z)
        x = torch.from_numpy(I.make_tokens(B, m1, 2)).cuda()
        c = torch.from_numpy(I.make_cond(B, m1, 3, std=0.5)).cuda()

        def blocks():
            for _ in range(5):
                ctx.dit_block(0, qc.QC_FULL, x, c)
        blocks()
        torch.cuda.synchronize()
        prof = ctx.profile_pass(blocks)
        ops = {"gemm_qkv": 2.0 * M * 3 * D * D, "gemm_proj": 2.0 * M * D * D, "gemm_fc1": 2.0 * M * R * D,
               "gemm_fc2": 2.0 * M * D * R}
        row = {}
        for k, p in prof.items():
            us = p["total_ms"] * 1e3 / max(p["launches"], 1)
            if k in ops:
                row[k] = {"avg_us": us, "TOP/s": ops[k] / (us * 1e-6) / 1e12, "frac": ops[k] / (us * 1e-6) / 1e12 / INT8_MFMA_PEAK_TOPS}
            elif k == "ln_mod_quant":      # fp32 row in, int8 codes out
                row[k] = {"avg_us": us, "GB/s": 5.0 * M * D / (us * 1e-6) / 1e9, "frac": 5.0 * M * D / (us * 1e-6) / 1e9 / HBM_PEAK_GBS}
            elif k == "attention":
                fl = 4.0 * B * m1.heads * T * T * m1.head_dim
                row[k] = {"avg_us": us, "TFLOP/s": fl / (us * 1e-6) / 1e12, "frac": fl / (us * 1e-6) / 1e12 / FP16_MFMA_PEAK_TFLOPS}
        out["m%d" % M] = row
        ctx.close()
        del ctx, x, c
        torch.cuda.empty_cache()
    return out


def tap_block(k):
    """Size of the iteration block: k rounded up to a multiple of 8 plus 24 guard vectors, at most 128."""
    return min(128, (k + 7) // 8 * 8 + 24)


def tap_cpu_baseline(wl):
    """The clustering oracle, as it stands, on the first 6144 samples of the same pool (subsamples of 1/20 of them,
    the workload's k, alpha and number of subsamples)."""
    import numpy as np
    from oracle import tap
    from synthetic import tap_inputs as TI
    Ns = min(wl.N, 6144)
    ns = max(wl.k, Ns // 20)
    X, t, _, _ = TI.make_pool(wl.N, wl.F, wl.steps, wl.classes, wl.seed)
    X, t = X[:Ns], t[:Ns]
    subs = TI.make_subsamples(Ns, ns, wl.m, wl.seed + 1)
    init = TI.make_init(Ns, wl.k, wl.m, wl.seed + 2)
    t0 = time.perf_counter()
    tap.tap(X, t, subs, wl.alpha, wl.k, init, TAP_MAX_PASSES)
    dt = time.perf_counter() - t0
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    return {"value": Ns / dt, "unit": "samples/sec", "cores": int(cores), "kind": "oracle",
            "sample": "the first %d pool samples with subsamples of %d (%.1f s); the cost per sample grows with the "
                      "pool (similarity and singular vectors are N x n with n = N / 20), so the full pool would be "
                      "slower per sample" % (Ns, ns, dt)}


def bench_tap(args):
    import numpy as np
    import torch
    import paper_2503_02508_amd as qc
    from synthetic import tap_inputs as TI
    wl = TI.TAP_WORKLOADS[args.workload]
    kb = tap_block(wl.k)
    torch.cuda.set_device(0)
    X, t, _, _ = TI.make_pool(wl.N, wl.F, wl.steps, wl.classes, wl.seed)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    Xd, td = dev(X), dev(t)
    subs = dev(TI.make_subsamples(wl.N, wl.n, wl.m, wl.seed + 1))
    init = dev(TI.make_init(wl.N, wl.k, wl.m, wl.seed + 2))
    q0 = dev(TI.make_start_block(kb, wl.n, wl.seed + 3))
    del X
    # room for all subsamples at once (at most 3 are worked on together)
    slots = min(wl.m, 3)
    per = (qc.qc_tap_workspace_bytes(wl.N, wl.F, wl.n, wl.k, kb) + 255) // 256 * 256
    work = torch.empty(slots * per, dtype=torch.uint8, device="cuda")
    final = torch.empty(wl.N, dtype=torch.int32, device="cuda")
    per = torch.empty((wl.m, wl.N), dtype=torch.int32, device="cuda")

    def run_once():
        qc.qc_tap_cluster(Xd, td, subs, wl.alpha, wl.k, TAP_ITERS, q0, init, TAP_MAX_PASSES, final, per, work)

    for _ in range(args.warmup):
        run_once()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_once()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert int(final.min()) >= 0 and int(final.max()) < wl.k
    # dominant kernel: the similarity contraction, events around its launches in one more pass
    qc.qc_tap_profile_begin()
    run_once()
    sim_ms, launches = qc.qc_tap_profile_end()
    flops = 2.0 * wl.N * wl.n * wl.F
    ach = flops / (sim_ms / launches * 1e-3) / 1e12
    out = {
        "metric": "pool samples clustered/sec, calibration-set clustering (TAP)",
        "value": wl.N * args.steps / dt, "unit": "samples/sec", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt / args.steps * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": wl.name, "pool": wl.N, "features": wl.F, "subsample": wl.n, "subsamples": wl.m,
                   "clusters": wl.k, "alpha": wl.alpha, "iteration_block": kb, "power_iterations": TAP_ITERS,
                   "concurrent_subsamples": slots,
                   "kmeans_pass_limit": TAP_MAX_PASSES},
        "roofline": {"bound": "mfma", "kernel": "similarity (sgemm_kernel, cosine + temporal epilogue)", "achieved": ach,
                     "peak": FP32_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": ach / FP32_MFMA_PEAK_TFLOPS,
                     "traffic": TRAFFIC.get((wl.name, "similarity")), "avg_launch_us": sim_ms / launches * 1e3,
                     "launches": launches},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = tap_cpu_baseline(wl)
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cache-format", choices=["fp32", "bf16"], default="fp32",
                    help="storage of the cached module outputs (fp32 is the headline configuration)")
    ap.add_argument("--stream-format", choices=["fp32", "bf16"], default="fp32",
                    help="storage of the residual stream (fp32 is the headline configuration)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (latents are independent, so more GPUs would each run "
              "this same program on their share of the batch); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    if args.workload.startswith("tap"):
        return bench_tap(args)

    import numpy as np
    import torch
    import paper_2503_02508_amd as qc
    from synthetic import dit_inputs as I

    wl = I.WORKLOADS[args.workload]
    m = wl.model
    B = wl.batch
    Beff = 2 * B if wl.cfg_scale > 0 else B
    torch.cuda.set_device(0)

    # ---- setup (untimed): weights, on-device weight quantisation, on-device calibration
    w = I.make_weights(m, wl.seed_weights)
    ctx = qc.Context(m, Beff, wl.cache_interval)
    ctx.load_weights(w, keep_fp32=True)
    clat, clab, idx = I.calibration_inputs(wl)
    tt, _, _ = qc.qc_ddim_schedule(wl.steps)
    ctx.calibrate(torch.from_numpy(clat).cuda(), [tt[i] for i in idx], clab)
    ctx.drop_fp32()
    ctx.set_cache_format(args.cache_format)
    ctx.set_stream_format(args.stream_format)
    del w
    lat = torch.from_numpy(I.make_latents(B, m, wl.seed_latents)).cuda()
    lab = torch.from_numpy(I.make_labels(B, m, wl.seed_labels).astype(np.int32)).cuda()
    K = torch.from_numpy(I.make_vc_factors(wl.steps, m.latent_c, wl.seed_k)).cuda()
    x = torch.empty_like(lat)

    def run_once():
        x.copy_(lat)
        ctx.sample(x, lab, wl.steps, wl.cfg_scale, K)

    for _ in range(args.warmup):
        run_once()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_once()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert torch.isfinite(x).all()
    ms_per_step = dt / args.steps * 1e3
    value = B * args.steps / dt

    # ---- full-step and cached-step latency (same batch, forced modes)
    tt_, at_, ap_ = qc.qc_ddim_schedule(wl.steps)
    def step_us(mode, reps=6):
        x.copy_(lat)
        ctx.sample_step(x, lab, 0, tt_[0], at_[0], ap_[0], wl.cfg_scale, K[0], qc.QC_FULL)   # fills the cache
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            ctx.sample_step(x, lab, 1, tt_[1], at_[1], ap_[1], wl.cfg_scale, K[1], mode)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / reps * 1e6
    full_us, cached_us = step_us(qc.QC_FULL), step_us(qc.QC_CACHED)

    # ---- dominant kernel: instrumented repeat of the same pass with HIP events around its launches
    prof = ctx.profile_pass(run_once)
    n_full = -(-wl.steps // wl.cache_interval)
    roofline = None
    if prof:
        dom = max(prof.values(), key=lambda p: p["total_ms"])
        for p in prof.values():
            p["avg_us"] = p["total_ms"] * 1e3 / max(p["launches"], 1)
        MT, D, R = Beff * m.tokens, m.hidden, m.mlp_dim
        per_pass = n_full * m.depth        # full blocks in one pass
        sb = 2 if args.stream_format == "bf16" else 4      # bytes per residual-stream element
        # algorithmic work of each class in one pass; a pass may cut the batch into sub-batches that are
        # launched separately, so the work of one launch is the class's work over its launches
        work = {
            "gemm_qkv": ("mfma", 2.0 * MT * 3 * D * D * per_pass),
            "gemm_proj": ("mfma", 2.0 * MT * D * D * per_pass),
            "gemm_fc1": ("mfma", 2.0 * MT * R * D * per_pass),
            "gemm_fc2": ("mfma", 2.0 * MT * D * R * per_pass),
            "attention": ("mfma16", 4.0 * Beff * m.heads * m.tokens * m.tokens * m.head_dim * per_pass),
            # residual-stream row in, int8 codes out
            "ln_mod_quant": ("hbm", (sb + 1.0) * MT * D * 2 * per_pass),
            # both cached tensors of every block read once, the residual stream read and written once
            "cached_blocks": ("hbm", (2.0 * m.depth * (2 if args.cache_format == "bf16" else 4) + 2.0 * sb) * MT * D
                              * (wl.steps - n_full)),
            # sample and noise estimate(s) read, sample written; one launch per step
            "ddim_vc": ("hbm", (4.0 * (B + Beff) + 4.0 * B) * m.latent_c * m.latent_h * m.latent_w * wl.steps),
            # all steps' adaLN projections of every block in one launch per window of steps
            "gemm_adaln": ("mfma", 2.0 * wl.steps * Beff * 6 * D * D * m.depth),
        }
        peaks = {"mfma": (INT8_MFMA_PEAK_TOPS, "TOP/s"), "mfma16": (FP16_MFMA_PEAK_TFLOPS, "TFLOP/s"),
                 "hbm": (HBM_PEAK_GBS, "GB/s")}
        for k, (bound, wk) in work.items():
            if k not in prof:
                continue
            peak, unit = peaks[bound]
            per_launch = wk / prof[k]["launches"]
            ach = per_launch / (prof[k]["avg_us"] * 1e-6) / (1e9 if bound == "hbm" else 1e12)
            prof[k].update({"bound": "mfma" if bound != "hbm" else "hbm", "achieved": ach, "peak": peak, "unit": unit,
                            "frac": ach / peak})
        if "achieved" in dom:
            roofline = {"bound": dom["bound"], "kernel": dom["name"], "achieved": dom["achieved"], "peak": dom["peak"],
                        "unit": dom["unit"], "frac": dom["frac"], "traffic": TRAFFIC.get((wl.name, dom["name"])),
                        "avg_launch_us": dom["avg_us"], "launches": dom["launches"]}
    total_int8 = int8_ops_per_full_step(m, Beff) * n_full
    out = {
        "metric": "latents/sec, DiT-XL/2 W%dA8+cache %d^2 at %d steps; int8 GEMM %% of MFMA peak" % (
            m.weight_bits, 8 * m.latent_h, wl.steps),
        "value": value, "unit": "latents/sec", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": wl.name, "latents": B, "effective_batch": Beff, "sampler_steps": wl.steps,
                   "cache_interval": wl.cache_interval, "refresh_steps": n_full, "cfg_scale": wl.cfg_scale,
                   "weight_bits": m.weight_bits, "vc": True,
                   "cache_format": args.cache_format, "stream_format": args.stream_format},
        "int8_tops_end_to_end": total_int8 / (ms_per_step * 1e-3) / 1e12,
        "full_step_us": full_us, "cached_step_us": cached_us,
        "roofline": roofline,
        "kernels": prof,
    }
    # per-shape rates of one block's kernels, each launch alone on the chip
    ctx.close()
    del ctx
    torch.cuda.empty_cache()
    out["per_shape"] = per_shape_rates(m, m.weight_bits)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
