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
