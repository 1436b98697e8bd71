#!/usr/bin/env python3
"""Short, profiler-friendly run of the sampler: a few sampler steps of one
workload plus a plain copy of known size, for hardware-counter collection.

Counter collection serialises kernels and slows every dispatch, so the full
benchmark is too long for it; the kernels of one refresh step and one cached
step are the same ones the benchmark launches (same shapes, same launch
configuration).  The copies at the end are the yardstick that converts the
FETCH_SIZE / WRITE_SIZE counter readings into bytes: a plain device-to-device
copy of 512 MiB (far larger than the L2s and the memory-side cache, so every
byte is fetched from and written to HBM once).

    rocprofv3 --pmc FETCH_SIZE --kernel-trace -d <out> -- python3 paper_2503_02508_amd/profile_driver.py
    rocprofv3 --pmc WRITE_SIZE --kernel-trace -d <out> -- python3 paper_2503_02508_amd/profile_driver.py

With `--workload tap1` the run is one subsample of the calibration-set clustering instead (similarity, degree
normalisation, embedding, k-means at the benchmark's sizes and settings), followed by the same copies.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="cfg1")
    ap.add_argument("--sampler-steps", type=int, default=2, help="sampler steps to run (from step 0)")
    ap.add_argument("--copies", type=int, default=3)
    ap.add_argument("--copy-mib", type=int, default=512)
    args = ap.parse_args()

    import numpy as np
    import torch
    import paper_2503_02508_amd as qc

    if args.workload.startswith("tap"):
        run_tap(args, qc, np, torch)
        copies(args, torch)
        return
    from synthetic import dit_inputs as I

    wl = I.WORKLOADS[args.workload]
    m = wl.model
    B = wl.batch
    Beff = 2 * B if wl.cfg_scale > 0 else B
    torch.cuda.set_device(0)
    w = I.make_weights(m, wl.seed_weights)
    ctx = qc.Context(m, Beff, wl.cache_interval)
    ctx.load_weights(w, keep_fp32=True)
    clat, clab, idx = I.calibration_inputs(wl)
    tt, at, ap_ = qc.qc_ddim_schedule(wl.steps)
    ctx.calibrate(torch.from_numpy(clat).cuda(), [tt[i] for i in idx], clab)
    ctx.drop_fp32()
    del w
    x = torch.from_numpy(I.make_latents(B, m, wl.seed_latents)).cuda()
    lab = torch.from_numpy(I.make_labels(B, m, wl.seed_labels).astype(np.int32)).cuda()
    K = torch.from_numpy(I.make_vc_factors(wl.steps, m.latent_c, wl.seed_k)).cuda()
    print("profile_driver: %s, %d sampler steps" % (wl.name, args.sampler_steps), flush=True)
    for i in range(args.sampler_steps):
        ctx.sample_step(x, lab, i, tt[i], at[i], ap_[i], wl.cfg_scale, K[i])
    torch.cuda.synchronize()
    copies(args, torch)


def run_tap(args, qc, np, torch):
    from synthetic import tap_inputs as TI
    wl = TI.TAP_WORKLOADS[args.workload]
    kb = min(128, (wl.k + 7) // 8 * 8 + 24)
    torch.cuda.set_device(0)
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    X, t, _, _ = TI.make_pool(wl.N, wl.F, wl.steps, wl.classes, wl.seed)
    Xd, td = dev(X), dev(t)
    idx = dev(TI.make_subsamples(wl.N, wl.n, wl.m, wl.seed + 1)[0])
    init = dev(TI.make_init(wl.N, wl.k, wl.m, wl.seed + 2)[0])
    q0 = dev(TI.make_start_block(kb, wl.n, wl.seed + 3))
    work = torch.empty(qc.qc_tap_workspace_bytes(wl.N, wl.F, wl.n, wl.k, kb), dtype=torch.uint8, device="cuda")
    A = torch.empty((wl.N, wl.n), device="cuda")
    dr, dc = torch.empty(wl.N, device="cuda"), torch.empty(wl.n, device="cuda")
    U, sig = torch.empty((wl.N, wl.k), device="cuda"), torch.empty(wl.k, device="cuda")
    lab, cen = torch.empty(wl.N, dtype=torch.int32, device="cuda"), torch.empty((wl.k, wl.k), device="cuda")
    print("profile_driver: %s, one subsample" % wl.name, flush=True)
    qc.qc_tap_similarity(Xd, td, idx, wl.alpha, A, dr, dc, work)
    qc.qc_tap_normalise(A, dr, dc, work)
    qc.qc_tap_embed(A, wl.k, 8, q0, U, sig, work)
    qc.qc_tap_kmeans(U, init, 100, lab, cen, work)
    torch.cuda.synchronize()


def copies(args, torch):
    n = args.copy_mib * (1 << 20) // 4
    src = torch.ones(n, device="cuda")
    dst = torch.empty_like(src)
    torch.cuda.synchronize()
    for _ in range(args.copies):
        dst.copy_(src)
    torch.cuda.synchronize()
    print("profile_driver: copy yardstick = %d bytes read and %d bytes written per copy kernel launch"
          % (n * 4, n * 4), flush=True)


if __name__ == "__main__":
    main()
