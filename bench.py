#!/usr/bin/env python3
"""Benchmark of the local training step on one MI355X.

A *step* is one pass of the whole hot path over one batch per block of the workload
(default: the ResNet-18-style configuration, 17 local layers in 4 blocks at batch
64/128/256/512): for every block, gather its batch from the previous block's activation
cache at the block's own batch size (nf_cache_read with a shuffled index list; block 1
gathers raw inputs), run nf_local_step for each of its layers (forward, head, loss, local
gradients, SGD with momentum), and store the block's emitted activations in the next cache
(nf_cache_write).  All inputs are synthetic, seeded, and resident in HBM before timing.

Prints ONE JSON line: images/s over the timed steps, plus `roofline` for the kernel that
takes the most time (per-launch algorithmic FLOPs / HIP-event duration against the fp32
MFMA peak) and `cpu_baseline` (the CPU oracle timed on a bounded sample of the same work).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix peak
MFMA_BF16_PEAK_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
HBM_PEAK_GBS = 8000.0          # MI355X HBM3E

# HBM-side bytes per launch (fabric reads + writes) of the kernels that can dominate the default
# workload, from `rocprofv3 --pmc FETCH_SIZE` and `--pmc WRITE_SIZE` passes over this script, each
# scaled by what the same counter reads for a plain 1 GiB copy (`--traffic-calib`): FETCH_SIZE x 2.0,
# WRITE_SIZE x 1.0.  Averages over the launches of one step; summary under profiles/.
TRAFFIC_BYTES_PER_LAUNCH = {
    ("cfg3_resnet18", "igemm_wgrad_fast_128x128"): 66.7e6 + 37.9e6,
    ("cfg3_resnet18", "igemm_fwd_fast_128x128"): 67.6e6 + 16.8e6,
}
TRAFFIC_SOURCE = ("offline: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes over this script, scaled by a 1 GiB copy "
                  "(FETCH x 2.0, WRITE x 1.0); summary in profiles/local_step_cfg3_hbm_traffic.md; not re-measured "
                  "by this run")
# The same counters for the HBM-bound kernels of the default workload, per (kernel symbol, grid in
# threads): (counter bytes per launch, rocprofv3 kernel-trace duration in us); same passes, same
# scaling, durations from the --kernel-trace --stats run.  HIP-event pairs (the `hbm` figures measured
# live below) add about 3 us to every launch, which halves the apparent rate of a 6 us copy.
HBM_OFFLINE = {
    "cfg3_resnet18": [
        ("cache_copy_kernel", 1048576, 33.59e6, 6.41), ("cache_copy_kernel", 2097152, 67.15e6, 14.84),
        ("wgrad_reduce_kernel", 325376, 17.62e6, 7.39), ("wgrad_reduce_kernel", 1283584, 50.11e6, 15.29),
        ("wgrad_reduce_kernel", 402944, 76.87e6, 17.70), ("wgrad_reduce_kernel", 697856, 141.74e6, 25.85),
        ("head_wide_kernel<4>", 215040, 22.45e6, 17.78), ("head_wide_kernel<4>", 149504, 6.45e6, 10.78),
        ("head_sample_kernel<4, false>", 83968, 4.34e6, 12.78),
    ],
}
HBM_OFFLINE_SOURCE = "profiles/local_step_cfg3_hbm_traffic.md (offline rocprofv3 passes; not re-measured by this run)"
# kernels judged against the HBM roofline (everything that is not a contraction)
HBM_KERNELS = ("cache_read", "cache_write", "cache_copy", "wgrad_reduce_sgd", "wgrad_reduce", "head_pool", "head_fc",
               "head_sample", "head_wide", "head_bwd", "maxpool_fwd", "maxpool_bwd", "fwd_finish", "sgd", "loss_mean")


def layer_flops(ls, B, n_classes):
    """Algorithmic FLOPs of one local step: fwd + wgrad for the layer (and projection),
    fwd + wgrad + dgrad for the aux conv and the linear layer (dense formula)."""
    f_layer = 2.0 * B * ls.Ho * ls.Wo * ls.C_out * ls.C_in * ls.R * ls.S
    f_proj = 2.0 * B * ls.Ho * ls.Wo * ls.C_out * ls.skip_C if ls.skip_kind == 2 else 0.0
    f_aux = 2.0 * B * ls.Hp * ls.Wp * ls.A * ls.C_out * 9
    f_fc = 2.0 * B * 4 * ls.A * n_classes
    return 2.0 * (f_layer + f_proj) + 3.0 * f_aux + 3.0 * f_fc


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="cfg3")
    ap.add_argument("--samples", type=int, default=0, help="synthetic data-set size (default: the config's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-prof", action="store_true")
    ap.add_argument("--lr", type=float, default=None, help="override the configuration's learning rate")
    ap.add_argument("--head-pool", choices=["avg", "max"], default="avg", help="the heads' down-sampling F_n")
    ap.add_argument("--loss", choices=["ce", "mse"], default="ce", help="the local loss of Eq. 3")
    ap.add_argument("--contraction", choices=["f32", "bf16x6", "bf16x9"], default="f32",
                    help="how the wide contractions run: fp32 matrix-core instructions (the default), or "
                         "bf16 matrix-core instructions on three-way split fp32 operands (six or all nine piece "
                         "products; same accuracy)")
    ap.add_argument("--trace-loss", action="store_true", help="print every layer's loss after each step (syncs)")
    ap.add_argument("--traffic-calib", action="store_true",
                    help="only run 5 plain copies of 1 GiB (nf_cache_read, contiguous rows): the known-size kernel "
                         "the FETCH_SIZE / WRITE_SIZE counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import workloads
    from paper_2402_14139_amd import binding as nf
    from paper_2402_14139_amd import layout
    from paper_2402_14139_amd.layer import LocalLayer

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the library has no CPU path", file=sys.stderr)
        sys.exit(2)
    nf.lib()
    modes = {"f32": nf.NF_CONTRACT_F32, "bf16x6": nf.NF_CONTRACT_BF16X6, "bf16x9": nf.NF_CONTRACT_BF16X9}
    nf.nf_contraction(modes[args.contraction])
    dev = "cuda:0"
    torch.cuda.set_device(0)
    if args.traffic_calib:
        rows, se = 4096, 65536  # 4096 rows of 256 KiB: reads 1 GiB, writes 1 GiB per launch
        src = torch.ones((rows, se), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            nf.nf_cache_read(src, None, rows, se, 0, None, rows, dst, None)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_calib": "cache_copy_kernel", "launches": 5, "read_bytes": rows * se * 4,
                          "write_bytes": rows * se * 4}))
        return
    cfg = workloads.config(args.config)
    if args.lr is not None:
        cfg.lr = args.lr
    N = args.samples or cfg.n_samples
    maxB = max(b.batch for b in cfg.blocks)
    N = max(N // maxB, 1) * maxB
    cls = cfg.n_classes
    log = lambda *a: print(*a, file=sys.stderr, flush=True)  # noqa: E731
    log(f"[bench] {cfg.name}: {len(cfg.layers)} layers, {len(cfg.blocks)} blocks, N={N}")

    # ---- parameters and per-layer device state ------------------------------------------------
    layers = []
    for li, ls in enumerate(cfg.layers):
        p = workloads.gen_layer_params(cfg.seed, li, ls, cls)
        d, a = nf.LayerDesc(**ls.layer_desc_fields()), nf.AuxDesc(**ls.aux_desc_fields(cls))
        a.head_pool, a.loss_kind = int(args.head_pool == "max"), int(args.loss == "mse")
        B = cfg.blocks[ls.block].batch
        L = LocalLayer(d, a, layout.params_to_lib(p, ls.A), B, momentum=cfg.momentum != 0, device=dev)
        L.y = L.new_output(B)
        layers.append(L)

    # ---- synthetic data set (rows = samples, NHWC) and the caches between blocks ---------------
    g = workloads.rng_for(cfg.seed, "bench-data")
    C0, H0, W0 = cfg.in_shape
    se0 = C0 * H0 * W0
    data = torch.empty((N, se0), dtype=torch.float32, device=dev)
    chunk = 1024
    for i in range(0, N, chunk):
        n = min(chunk, N - i)
        data[i:i + n] = torch.from_numpy(g.standard_normal((n, se0)).astype(np.float32)).to(dev)
    labels = torch.from_numpy(g.integers(0, cls, size=(N,)).astype(np.int32)).to(dev)
    nblk = len(cfg.blocks)
    se = [se0]
    for b in cfg.blocks:
        last = cfg.layers[b.layers[-1]]
        se.append(last.C_out * last.Hp * last.Wp)
    caches = [data] + [torch.empty((N, se[k + 1]), dtype=torch.float32, device=dev) for k in range(nblk - 1)]
    clabels = [labels] + [torch.empty((N,), dtype=torch.int32, device=dev) for _ in range(nblk - 1)]
    # Timed steps write each block's output into a second set of caches: in the method a cache is
    # written once, after its block has been trained, and only read afterwards; writing the
    # half-trained outputs into the caches the next block is reading from would feed the blocks'
    # evolving weights back into their own inputs.
    wcaches = [None] + [torch.empty_like(c) for c in caches[1:]]
    wlabels = [None] + [torch.empty_like(c) for c in clabels[1:]]
    xin = []
    lin = []
    for k, b in enumerate(cfg.blocks):
        f = cfg.layers[b.layers[0]]
        xin.append(torch.empty((b.batch, f.H_in, f.W_in, f.C_in), dtype=torch.float32, device=dev))
        lin.append(torch.empty((b.batch,), dtype=torch.int32, device=dev))
    perms = [torch.from_numpy(workloads.rng_for(cfg.seed, "perm", k).permutation(N).astype(np.int64)).to(dev)
             for k in range(nblk)]

    def skip_of(li, x_block):
        ls = cfg.layers[li]
        if not ls.skip_kind:
            return None
        src = ls.skip_src  # the layer whose INPUT is the shortcut tensor
        first = cfg.blocks[ls.block].layers[0]
        return x_block if src == first else layers[src - 1].y

    def block_forward(k, x):
        b = cfg.blocks[k]
        cur = x
        for li in b.layers:
            layers[li].forward(cur, skip_of(li, x), layers[li].y)
            cur = layers[li].y
        return cur

    def block_step(k, x, lab):
        b = cfg.blocks[k]
        cur = x
        for li in b.layers:
            layers[li].step(cur, skip_of(li, x), lab, cfg.lr, cfg.momentum, layers[li].y)
            cur = layers[li].y
        return cur

    # fill the caches once with the initial weights so deeper blocks see real activations
    t0 = time.time()
    for k in range(nblk - 1):
        B = cfg.blocks[k].batch
        for first in range(0, N, B):
            nf.nf_cache_read(caches[k], clabels[k], N, se[k], first, None, B, xin[k], lin[k])
            y = block_forward(k, xin[k])
            nf.nf_cache_write(caches[k + 1], clabels[k + 1], N, se[k + 1], first, B, y, lin[k])
    torch.cuda.synchronize()
    log(f"[bench] caches filled in {time.time() - t0:.1f}s "
        f"({sum(c.numel() for c in caches[1:]) * 4 / 2**30:.2f} GiB)")

    def one_step(s):
        for k in range(nblk):
            B = cfg.blocks[k].batch
            j = s % (N // B)
            nf.nf_cache_read(caches[k], clabels[k], N, se[k], 0, perms[k][j * B:(j + 1) * B], B, xin[k], lin[k])
            y = block_step(k, xin[k], lin[k])
            if k + 1 < nblk:
                nf.nf_cache_write(wcaches[k + 1], wlabels[k + 1], N, se[k + 1], j * B, B, y, lin[k])
        if args.trace_loss:
            torch.cuda.synchronize()
            log(f"[loss] step {s}: " + " ".join(f"{float(L.loss.item()):.3f}" for L in layers)
                + " | ymax " + " ".join(f"{float(L.y.max()):.1f}" for L in layers))

    for s in range(args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(args.warmup, args.warmup + args.steps):
        one_step(s)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / args.steps
    images_per_step = sum(b.batch for b in cfg.blocks)
    flops_per_step = sum(layer_flops(ls, cfg.blocks[ls.block].batch, cls) for ls in cfg.layers)
    losses = [float(L.loss.item()) for L in layers]
    finite = bool(all(np.isfinite(losses)))
    if not finite:
        # un-normalised synthetic training can diverge at a configuration's own learning rate
        # (the VGG-11 configuration names lr = 0.05); the default workload must stay finite
        log(f"[bench] WARNING: non-finite losses after the timed steps: {losses}")
        assert args.config != "cfg3", losses
    log(f"[bench] {ms_per_step:.3f} ms/step, {flops_per_step / 1e9:.1f} GFLOP/step, "
        f"{flops_per_step / dt * args.steps / 1e12:.2f} TFLOP/s ({args.contraction})")

    # ---- the same steps in the other contraction mode (reported beside the headline, never as it) ----
    other_name = "bf16x6" if args.contraction == "f32" else "f32"
    prev_mode = nf.nf_contraction(modes[other_name])
    s0 = args.warmup + args.steps
    for s in range(s0, s0 + args.warmup):
        one_step(s)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(s0 + args.warmup, s0 + args.warmup + args.steps):
        one_step(s)
    torch.cuda.synchronize()
    ms_other = (time.perf_counter() - t0) * 1e3 / args.steps
    nf.nf_contraction(prev_mode)
    other_mode = {"contraction": other_name, "ms_per_step": round(ms_other, 4),
                  "value": round(images_per_step / (ms_other * 1e-3), 1), "unit": "images/s",
                  "tflops": round(flops_per_step / (ms_other * 1e-3) / 1e12, 2),
                  "losses_finite": bool(all(np.isfinite([float(L.loss.item()) for L in layers]))),
                  "note": "same workload, same fp32 operands and results; the wide convolutions and weight gradients "
                          "run on the bf16 matrix cores with every operand cut into three bfloat16 pieces "
                          "(six piece products, fp32 accumulation); parity tests pass at the same tolerance"
                          if other_name == "bf16x6" else "the default mode: fp32 matrix-core instructions"}
    log(f"[bench] other contraction mode ({other_name}): {ms_other:.3f} ms/step, {other_mode['tflops']:.2f} TFLOP/s")

    # ---- per-kernel timing with HIP events: the same steps again ------------------------------
    roofline, kernels, hbm = None, [], []
    if not args.no_prof:
        psteps = min(args.steps, 5)
        nf.nf_prof_begin()
        for s in range(psteps):
            one_step(args.warmup + args.steps + s)
        recs = nf.nf_prof_end()
        tot = sum(r["ms"] for r in recs)
        for r in recs:
            kernels.append({"kernel": r["kernel"], "launches_per_step": r["launches"] / psteps,
                            "ms_per_step": round(r["ms"] / psteps, 4), "share": round(r["ms"] / tot, 4),
                            "avg_us": round(1e3 * r["ms"] / r["launches"], 2),
                            "tflops": round(r["flops"] / (r["ms"] * 1e-3) / 1e12, 2) if r["flops"] else 0.0,
                            "gbs": round(r["bytes"] / (r["ms"] * 1e-3) / 1e9, 1)})
        dom = recs[0]
        if dom["kernel"].startswith("igemm"):
            ach = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
            # a split-operand kernel spends six bf16 matrix-core multiply-adds per algorithmic one
            split = 6 if "_split_" in dom["kernel"] else 9 if "_split9_" in dom["kernel"] else 0
            peak = round(MFMA_BF16_PEAK_TFLOPS / split, 1) if split else MFMA_F32_PEAK_TFLOPS
            roofline = {"kernel": dom["kernel"], "bound": "mfma", "achieved": round(ach, 2),
                        "peak": peak, "unit": "TFLOP/s", "frac": round(ach / peak, 4),
                        "peak_note": (f"bf16 dense matrix peak 2500 TFLOP/s / {split} piece products per fp32 multiply-add"
                                      if split else "fp32 dense matrix peak"),
                        "traffic": TRAFFIC_BYTES_PER_LAUNCH.get((cfg.name, dom["kernel"])),
                        "traffic_source": TRAFFIC_SOURCE,
                        "launches": dom["launches"], "avg_launch_us": round(1e3 * dom["ms"] / dom["launches"], 2),
                        "measured_over": f"{psteps} further steps with one HIP-event pair per kernel launch"}
        else:
            ach = dom["bytes"] / (dom["ms"] * 1e-3) / 1e9
            roofline = {"kernel": dom["kernel"], "bound": "hbm", "achieved": round(ach, 1), "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(ach / HBM_PEAK_GBS, 4), "traffic": None,
                        "launches": dom["launches"], "avg_launch_us": round(1e3 * dom["ms"] / dom["launches"], 2),
                        "measured_over": f"{psteps} further steps with one HIP-event pair per kernel launch"}
        # HBM-bound kernels: algorithmic bytes (the library's per-launch formula) / HIP-event duration
        # against the published 8 TB/s; counter bytes per launch where an offline pass collected them
        for r in recs:
            if r["kernel"] in HBM_KERNELS and r["ms"] > 0:
                gbs = r["bytes"] / (r["ms"] * 1e-3) / 1e9
                hbm.append({"kernel": r["kernel"], "launches_per_step": r["launches"] / psteps,
                            "algorithmic_bytes_per_launch": round(r["bytes"] / r["launches"]),
                            "avg_us": round(1e3 * r["ms"] / r["launches"], 2), "achieved_gbs": round(gbs, 1),
                            "frac_of_8tbs": round(gbs / HBM_PEAK_GBS, 4),
                            "ms_per_step": round(r["ms"] / psteps, 4)})
        for kr in kernels:
            log(f"[kernel] {kr['kernel']:<26} {kr['launches_per_step']:6.1f}/step {kr['ms_per_step']:9.4f} ms "
                f"{100 * kr['share']:5.1f}%  avg {kr['avg_us']:9.2f} us  {kr['tflops']:7.2f} TFLOP/s {kr['gbs']:8.1f} GB/s")

    # ---- per-layer step times (one event pair per local step) ---------------------------------
    per_layer = []
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in cfg.layers]
    acc = [0.0] * len(cfg.layers)
    reps = 3
    for r in range(reps):
        for k in range(nblk):
            b = cfg.blocks[k]
            cur = xin[k]
            for li in b.layers:
                evs[li][0].record()
                layers[li].step(cur, skip_of(li, xin[k]), lin[k], cfg.lr, cfg.momentum, layers[li].y)
                evs[li][1].record()
                cur = layers[li].y
        torch.cuda.synchronize()
        for li in range(len(cfg.layers)):
            acc[li] += evs[li][0].elapsed_time(evs[li][1])
    for li, ls in enumerate(cfg.layers):
        B = cfg.blocks[ls.block].batch
        ms = acc[li] / reps
        fl = layer_flops(ls, B, cls)
        per_layer.append({"layer": ls.name, "block": ls.block, "B": B, "ms": round(ms, 4),
                          "images_per_s": round(B / (ms * 1e-3), 1), "tflops": round(fl / (ms * 1e-3) / 1e12, 2)})
        log(f"[layer] {li:2d} {ls.name:<8} blk{ls.block} B={B:<4d} {ms:8.3f} ms {B / (ms * 1e-3):10.0f} img/s "
            f"{fl / (ms * 1e-3) / 1e12:7.2f} TFLOP/s")

    per_block = []
    for k, b in enumerate(cfg.blocks):
        ms = sum(per_layer[li]["ms"] for li in b.layers)
        per_block.append({"block": k, "B": b.batch, "layers": len(b.layers), "ms": round(ms, 4),
                          "images_per_s": round(b.batch / (ms * 1e-3), 1)})

    # ---- the device's own figures: fp32 MFMA peak from CU count x clock (64 flop/clk/SIMD, 4 SIMDs
    # per CU), and a measured plain-copy bandwidth (1 GiB read + 1 GiB written) as the practical
    # HBM ceiling next to the published 8 TB/s
    prop = torch.cuda.get_device_properties(0)
    cus, clock_khz = nf.nf_device_info()
    device = {"name": prop.name, "compute_units": cus, "clock_mhz": round(clock_khz / 1e3, 1),
              "mfma_f32_peak_tflops_from_props": round(cus * 256 * clock_khz * 1e3 / 1e12, 1)}
    if not args.no_prof:
        rows, se_c = 4096, 65536
        src = torch.ones((rows, se_c), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        nf.nf_cache_read(src, None, rows, se_c, 0, None, rows, dst, None)
        e0.record()
        for _ in range(5):
            nf.nf_cache_read(src, None, rows, se_c, 0, None, rows, dst, None)
        e1.record()
        torch.cuda.synchronize()
        device["copy_1gib_gbs"] = round(5 * 2 * rows * se_c * 4 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1)
        del src, dst
    log(f"[device] {device}")

    # ---- cache streams at the step's own sizes: 20 launches back to back, captured in a HIP graph
    # and replayed between ONE event pair (the per-launch event pairs above add ~3 us to every
    # launch, and 20 eager launches of a 6 us copy are bound by the host's call rate): the shuffled
    # row gather of every block's batch, and the write of its output
    cache_stream = []
    if not args.no_prof:
        reps = 20

        def timed_graph(fn):
            try:
                gph = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gph):
                    for r in range(reps):
                        fn(r)
                torch.cuda.synchronize()
                gph.replay()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                gph.replay()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) * 1e3 / reps
            except Exception as exc:  # noqa: BLE001
                log(f"[cache] HIP-graph capture not available: {exc}")
                torch.cuda.synchronize()
                return None

        for k in range(nblk):
            B = cfg.blocks[k].batch
            nb = N // B
            sl = [perms[k][(r % nb) * B:(r % nb + 1) * B] for r in range(reps)]
            us = timed_graph(lambda r: nf.nf_cache_read(caches[k], clabels[k], N, se[k], 0, sl[r], B, xin[k], lin[k]))
            by = 8.0 * se[k] * B + 16.0 * B
            if us:
                cache_stream.append({"op": "cache_read", "block": k, "B": B, "bytes_per_launch": by, "us": round(us, 2),
                                     "gbs": round(by / us / 1e3, 1), "frac_of_8tbs": round(by / us / 1e3 / HBM_PEAK_GBS, 4)})
            if k + 1 < nblk:
                y = layers[cfg.blocks[k].layers[-1]].y
                us = timed_graph(lambda r: nf.nf_cache_write(wcaches[k + 1], wlabels[k + 1], N, se[k + 1], (r % nb) * B, B,
                                                             y, lin[k]))
                by = 8.0 * se[k + 1] * B + 8.0 * B
                if us:
                    cache_stream.append({"op": "cache_write", "block": k, "B": B, "bytes_per_launch": by,
                                         "us": round(us, 2), "gbs": round(by / us / 1e3, 1),
                                         "frac_of_8tbs": round(by / us / 1e3 / HBM_PEAK_GBS, 4)})
        for c in cache_stream:
            log(f"[cache] {c['op']:<11} block {c['block']} B={c['B']:<4d} {c['bytes_per_launch'] / 1e6:7.1f} MB "
                f"{c['us']:7.2f} us {c['gbs']:8.1f} GB/s ({100 * c['frac_of_8tbs']:.1f} % of 8 TB/s)")

    # ---- the same work through the block-level calls (Worker loop inside the library) ----------
    # per block: nf_block_train_epoch over `steps` shuffled batches of its cache, without and with
    # the prefetch stream (read of batch j+1 overlapping the training of batch j); then the
    # forward-only sweep that fills the next block's cache over all N samples.
    block_driver = None
    if not args.no_prof:
        main_s, side_s = torch.cuda.Stream(), torch.cuda.Stream()
        tot = {"plain": 0.0, "prefetch": 0.0, "graph": 0.0}
        fill_ms, eval_ms = 0.0, 0.0
        n_eval = min(N, 2048)
        epred = torch.empty((n_eval,), dtype=torch.int32, device=dev)
        ecnt = torch.zeros((1,), dtype=torch.int32, device=dev)
        for k, b in enumerate(cfg.blocks):
            Ls = [layers[li] for li in b.layers]
            skip = [(-1 if not cfg.layers[li].skip_kind else cfg.layers[li].skip_src - b.layers[0]) for li in b.layers]
            mom = cfg.momentum != 0
            blk = nf.make_block([l.d for l in Ls], [l.a for l in Ls], skip, [l.sp for l in Ls], [l.sa for l in Ls],
                                [l.sgp for l in Ls], [l.sga for l in Ls], [l.svp for l in Ls] if mom else None,
                                [l.sva for l in Ls] if mom else None)
            bws = torch.empty(nf.nf_block_workspace_bytes(blk, b.batch), dtype=torch.uint8, device=dev)
            nb = min(args.steps, N // b.batch)
            bl = torch.zeros((nb, len(Ls)), dtype=torch.float32, device=dev)
            torch.cuda.synchronize()
            for mode, pf in (("plain", None), ("prefetch", side_s), ("plain", None), ("prefetch", side_s)):
                t0 = time.perf_counter()
                nf.nf_block_train_epoch(blk, cfg.lr, cfg.momentum, b.batch, nb * b.batch, caches[k], clabels[k], N,
                                        perms[k], bl, bws, stream=main_s, prefetch_stream=pf)
                main_s.synchronize()
                tot[mode] += (time.perf_counter() - t0) * 1e3 / nb / 2
            # the same pass captured once by the library in a HIP graph (nf_block_graph_create) and
            # launched twice (an extra figure: a failure to capture must not cost the benchmark line)
            if tot["graph"] is not None:
                try:
                    graph = nf.nf_block_graph_create(blk, cfg.lr, cfg.momentum, b.batch, nb * b.batch, caches[k],
                                                     clabels[k], N, perms[k], bl, bws)
                    torch.cuda.synchronize()
                    for _ in range(2):
                        t0 = time.perf_counter()
                        nf.nf_block_graph_launch(graph, stream=main_s)
                        main_s.synchronize()
                        tot["graph"] += (time.perf_counter() - t0) * 1e3 / nb / 2
                    nf.nf_block_graph_destroy(graph)
                except Exception as exc:  # noqa: BLE001
                    log(f"[block] HIP-graph capture not available: {exc}")
                    tot["graph"] = None
                    torch.cuda.synchronize()
            if k + 1 < nblk:
                t0 = time.perf_counter()
                nf.nf_block_fill_cache(blk, b.batch, N, caches[k], clabels[k], N, wcaches[k + 1], wlabels[k + 1], N,
                                       bws, stream=main_s)
                main_s.synchronize()
                fill_ms += (time.perf_counter() - t0) * 1e3
            # early-exit evaluation at the block's last layer over n_eval samples of its input cache
            t0 = time.perf_counter()
            nf.nf_block_evaluate(blk, len(Ls) - 1, b.batch, n_eval, caches[k], clabels[k], N, epred, ecnt, bws,
                                 stream=main_s)
            main_s.synchronize()
            eval_ms += (time.perf_counter() - t0) * 1e3
            del bws
        block_driver = {"ms_per_step": round(tot["plain"], 4), "ms_per_step_prefetch": round(tot["prefetch"], 4),
                        "ms_per_step_hip_graph": None if tot["graph"] is None else round(tot["graph"], 4),
                        "note": "nf_block_train_epoch per block (no cache write inside a training pass), summed "
                                "over blocks per batch; prefetch = cache read of the next batch on a second stream",
                        "fill_cache_sweep_ms": round(fill_ms, 2),
                        "fill_cache_images_per_s": round((nblk - 1) * N / (fill_ms * 1e-3), 1) if fill_ms else None,
                        "evaluate_images_per_s": round(nblk * n_eval / (eval_ms * 1e-3), 1),
                        "evaluate_note": f"nf_block_evaluate at each block's last exit over {n_eval} samples of "
                                         "its input cache (forward of the block + that exit's head + arg-max)"}
        log(f"[block] train pass {tot['plain']:.3f} ms/step, with prefetch {tot['prefetch']:.3f} ms/step, "
            f"replayed from a HIP graph {tot['graph'] if tot['graph'] is not None else float('nan'):.3f} ms/step; "
            f"cache-fill sweeps of {nblk - 1} blocks x {N} samples {fill_ms:.1f} ms; evaluation of {nblk} exits x "
            f"{n_eval} samples {eval_ms:.1f} ms")

    # ---- CPU oracle on a bounded sample of the same workload ----------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as O
        # One local step of each layer at its block's batch size, in network order, until about
        # 25 s of CPU time have been spent (the whole step if it fits); scaled by FLOPs to the
        # full step.  Block inputs are synthetic post-ReLU tensors of the right shape.
        budget_s, t_cpu, fl_sample, done = 25.0, 0.0, 0.0, []
        gcpu = workloads.rng_for(cfg.seed, "cpu-baseline")
        for k, blk in enumerate(cfg.blocks):
            if t_cpu >= budget_s:
                break
            B = blk.batch
            f = cfg.layers[blk.layers[0]]
            xb = gcpu.standard_normal((B, f.C_in, f.H_in, f.W_in)).astype(np.float32)
            if k > 0:
                xb = np.maximum(xb, 0)
            yb = gcpu.integers(0, cls, size=(B,)).astype(np.int32)
            cur, outs = xb, {}
            for li in blk.layers:
                if t_cpu >= budget_s:
                    break
                ls = cfg.layers[li]
                pr = workloads.gen_layer_params(cfg.seed, li, ls, cls)
                mo = {kk: (None if v is None else np.zeros_like(v)) for kk, v in pr.items()}
                xs = None
                if ls.skip_kind:
                    xs = xb if ls.skip_src == blk.layers[0] else outs[ls.skip_src - 1]
                od, oa = O.layer_desc(**ls.layer_desc_fields()), O.aux_desc(**ls.aux_desc_fields(cls))
                t0 = time.perf_counter()
                Y, _, _ = O.local_step(od, oa, cur, xs, yb, pr, mo, cfg.lr, cfg.momentum)
                t_cpu += time.perf_counter() - t0
                fl_sample += layer_flops(ls, B, cls)
                outs[li] = Y
                cur = Y
                done.append(li)
        scaled_step_s = t_cpu * flops_per_step / fl_sample
        # the same oracle on ONE thread: the first layers of the step until about 8 s are spent
        nthreads = O.num_threads()
        O.set_num_threads(1)
        t1, fl1, done1 = 0.0, 0.0, []
        blk0 = cfg.blocks[0]
        f0 = cfg.layers[blk0.layers[0]]
        x1 = gcpu.standard_normal((blk0.batch, f0.C_in, f0.H_in, f0.W_in)).astype(np.float32)
        y1 = gcpu.integers(0, cls, size=(blk0.batch,)).astype(np.int32)
        cur1, outs1 = x1, {}
        for li in blk0.layers:
            if t1 >= 8.0:
                break
            ls = cfg.layers[li]
            pr = workloads.gen_layer_params(cfg.seed, li, ls, cls)
            xs = None
            if ls.skip_kind:
                xs = x1 if ls.skip_src == blk0.layers[0] else outs1[ls.skip_src - 1]
            od, oa = O.layer_desc(**ls.layer_desc_fields()), O.aux_desc(**ls.aux_desc_fields(cls))
            t0 = time.perf_counter()
            Y, _, _ = O.local_step(od, oa, cur1, xs, y1, pr, None, cfg.lr, 0.0)
            t1 += time.perf_counter() - t0
            fl1 += layer_flops(ls, blk0.batch, cls)
            outs1[li] = Y
            cur1 = Y
            done1.append(li)
        O.set_num_threads(nthreads)
        cpu = {"value": round(images_per_step / scaled_step_s, 3), "unit": "images/s", "cores": nthreads,
               "kind": "oracle",
               "value_1thread": round(images_per_step / (t1 * flops_per_step / fl1), 3),
               "gflops_1thread": round(fl1 / t1 / 1e9, 2),
               "sample_1thread": f"one local step of layers {done1[0]}..{done1[-1]} at batch {blk0.batch} "
                                 f"({fl1 / 1e9:.1f} GFLOP) took {t1:.2f} s on one thread; scaled by FLOPs",
               "sample": f"one local step of layers {done[0]}..{done[-1]} of {cfg.name} at their block batch sizes "
                         f"({fl_sample / 1e9:.1f} of the step's {flops_per_step / 1e9:.1f} GFLOP) took {t_cpu:.2f} s; "
                         f"scaled by FLOPs to the full step",
               "gflops": round(fl_sample / t_cpu / 1e9, 2)}
        log(f"[cpu] oracle {t_cpu:.2f}s on {nthreads} threads, {fl_sample / t_cpu / 1e9:.2f} GFLOP/s; "
            f"one thread {fl1 / t1 / 1e9:.2f} GFLOP/s")

    tflops = flops_per_step / (ms_per_step * 1e-3) / 1e12
    out = {
        "metric": "local_step_images_per_sec", "value": round(images_per_step / (ms_per_step * 1e-3), 1),
        "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic", "contraction": args.contraction, "other_contraction_mode": other_mode,
        "config": {"workload": f"{cfg.name}: one local step of each of {len(cfg.layers)} layers at block batches "
                               f"{'/'.join(str(b.batch) for b in cfg.blocks)}, {cls} classes, SGD lr {cfg.lr} "
                               f"momentum {cfg.momentum}, cache read (shuffled gather) before and cache write after "
                               f"every block" + ("" if (args.head_pool, args.loss) == ("avg", "ce") else
                                                 f"; heads: {args.head_pool} pooling, {args.loss} loss"), "images_per_step": images_per_step, "samples": N,
                   "gflop_per_step": round(flops_per_step / 1e9, 1)},
        "tflops": round(tflops, 2), "mfma_f32_peak_frac": round(tflops / MFMA_F32_PEAK_TFLOPS, 4),
        "losses_finite": finite,
        "roofline": roofline, "cpu_baseline": cpu, "hbm": hbm, "cache_stream": cache_stream,
        "hbm_offline": {"source": HBM_OFFLINE_SOURCE,
                        "rows": [{"kernel": k, "grid_threads": g, "counter_bytes_per_launch": by, "rocprof_us": us,
                                  "gbs": round(by / us / 1e3, 1), "frac_of_8tbs": round(by / us / 1e3 / HBM_PEAK_GBS, 3)}
                                 for k, g, by, us in HBM_OFFLINE.get(cfg.name, [])]},
        "block_driver": block_driver, "kernels": kernels,
        "layers": per_layer, "blocks": per_block, "device": device,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
