#!/usr/bin/env python3
"""Benchmark of the NeuS2 training-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2]

A step is one pass of the whole path over one synthetic batch: hash encode (+ Jacobian),
SDF network forward + analytic normal, colour network, compositing, loss, the backward pass
including the second-order term, scatter-add into the table gradient, and Adam on every
parameter (which also clears the gradient buffers).  Inputs and parameters are resident in
HBM before the timed region.  Prints ONE JSON line.

Besides the headline rate the line carries
  roofline      for the kernel that takes the largest share of the step, its algorithmic
                bytes (or flops) per launch divided by its average duration, measured here
                with events on the stream the kernels run on;
  kernels       the same figures for every kernel of the step;
  cpu_baseline  the float64 numpy oracle timed on this machine's host cores on a bounded sample
                of the same workload (a reported baseline, not a target).
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

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix rate: the network kernels run their products as split-bf16 terms

# Bytes that crossed the L2 <-> fabric boundary per call, from the two rocprofv3 --pmc runs
# summarised in profiles/hbm_traffic_cfg2-static-4096x64.txt (FETCH_SIZE x 2.000 + WRITE_SIZE
# x 1.000, the factors a 256 MiB device copy gives), in MiB {read, written}.  Only this
# workload has been measured; other workloads report null.
MEASURED_TRAFFIC_MIB = {
    "cfg2-static-4096x64": {
        "hash_encode": (86.1, 128.0), "sdf_fwd_grad": (128.5, 55.0), "color_fwd": (22.7, 7.0),
        "render_loss_bwd": (22.2, 8.1), "color_bwd": (37.0, 28.4), "sdf_mlp_bwd": (155.3, 48.0),
        "hash_scatter_bwd": (83.9 + 310.7, 232.7 + 56.4),      # bin_rows_kernel + scatter_owner_kernel
        "adam_all": (186.4, 209.6),
    },
}

# the HIP kernels behind each timed call (names as rocprofv3 prints them)
KERNELS_OF_CALL = {
    "hash_encode": "encode_kernel", "sdf_fwd_grad": "sdf_fwd_kernel", "sdf_mlp_bwd": "sdf_bwd_kernel",
    "sdf_bwd_2nd": "sdf_bwd_kernel + zero_kernel + bin_rows_kernel + scatter_owner_kernel + pos_hessian_kernel + sum_levels_kernel",
    "hash_scatter_bwd": "zero_kernel + bin_rows_kernel + scatter_owner_kernel (scatter_kernel below 2^16 points)",
    "adam_all": "adam_tables_kernel (tables, and the networks' matrices in a last row of workgroups)", "color_fwd": "color_fwd_kernel", "color_bwd": "color_bwd_kernel",
    "render_loss_bwd": "render_loss_kernel", "render_rays": "render_fwd_kernel", "render_rays_bwd": "render_bwd_kernel", "loss": "loss_kernel",
}


def algorithmic_cost(cfg, n):
    """Per-launch algorithmic bytes and flops of every kernel, from per-sample figures.

    Table gathers are counted at element size (8 corners x F x element bytes per level),
    atomics as read + write, every streamed array once.  Flops count the multiply-adds the
    method needs (2 per weight per use); recomputation inside the backward kernels and
    padding of narrow layers are NOT counted.
    """
    lam, D, F = cfg.active_levels, cfg.enc_dim, cfg.n_features
    et = 2 if cfg.table_dtype == "f16" else 4
    K = len(cfg.sdf_dims) - 1
    sd = cfg.sdf_dims
    sdf_w = sum(sd[i] * sd[i + 1] for i in range(K))             # weights of the SDF network
    sweep_w = sum(sd[i] * sd[i + 1] for i in range(K - 1))       # weights the reverse/forward sweeps use
    cost = {
        "hash_encode": {"bytes": 12 + lam * 8 * F * et + D * 4 + D * 12, "flops": 0},
        "sdf_fwd_grad": {"bytes": D * 4 + D * 12 + 64 + D * 4 + 12 + 8 * (K - 1), "flops": 2 * sdf_w + 2 * sweep_w + 2 * D * 3},
        "sdf_mlp_bwd": {"bytes": D * 4 + D * 12 + 64 + 12 + D * 4 + 8 * (K - 1),
                        # first order: data + weight gradients; second order: t_0 = J nbar, the t sweep and the
                        # outer products S_l^T t_{l-1}^T (S_K is a unit row: only row 0 of the last matrix)
                        "flops": 4 * sdf_w + 2 * D * 3 + 2 * sweep_w + 2 * (sdf_w - sd[K - 1] * (sd[K] - 1))},
        "hash_scatter_bwd": {"bytes": 12 + 12 + 2 * D * 4 + lam * 8 * F * 4 * 2, "flops": 0},
    }
    if cfg.loss_kind == 1:
        cd = cfg.color_dims
        col_w = sum(cd[i] * cd[i + 1] for i in range(3))
        cost.update({
            "color_fwd": {"bytes": 12 + 12 + 64 + 12 + 16, "flops": 2 * col_w},
            "color_bwd": {"bytes": 12 + 12 + 64 + 12 + 12 + 4 + 64 + 24 + 16, "flops": 2 * col_w + 4 * col_w},
            "render_rays": {"bytes": 4 + 12 + 4, "flops": 0},
            "render_loss_bwd": {"bytes": 4 + 12 + 12 + 4 + 4 + 12 + 12, "flops": 0},
            "render_rays_bwd": {"bytes": 4 + 12 + 4 + 12, "flops": 0},
            "loss": {"bytes": 12 + 12, "flops": 0},
        })
    else:
        cost["loss"] = {"bytes": 12 + 12 + 4 + 64, "flops": 0}
    # What the network kernels ISSUE on the bf16 matrix cores: every fp32 product is taken as products of
    # bf16 terms (six for forward-type products, whose results decide ReLU masks; three for adjoint-type
    # products and weight gradients), on v_mfma_f32_32x32x16_bf16 (32768 flop for a tile of 32 points),
    # including recomputation (three products where the forward kernels hand over their masks, as here) and the
    # padding of narrow layers.  Instruction counts per tile follow the
    # kernels' structure; the backward kernels add 32 narrow fp32 instructions (2048 flop each).
    ks1, k3 = sd[0] // 16, 1 if K == 3 else 0
    issued = {
        "sdf_fwd_grad": 6 * (2 * ks1 + 8 * k3 + 4 + 8 * k3 + 4),
        "sdf_mlp_bwd": 3 * (2 * ks1 + 8 * k3) + 3 * (2 + 8 * k3 + 4 + 8 * k3 + 2 * ks1 + 8 * k3) + 3 * 2 * (4 * k3 + 2) * 2,
        "color_fwd": 6 * (6 + 8), "color_bwd": 3 * (6 + 8) + 3 * (2 + 8 + 4) + 3 * 2 * (4 + 4),
    }
    out = {k: {"bytes": v["bytes"] * n, "flops": v["flops"] * n} for k, v in cost.items()}
    for k, mf in issued.items():
        if k in out:
            out[k]["issued_flops"] = (mf * 32768 + (32 * 2048 if k.endswith("bwd") else 0)) * n // 32
    # parameters a point can address: a dense level uses (res+1)^3 of its T slots
    n_tab = sum(((r + 1) ** 3 if d else cfg.table_size) for r, d in zip(cfg.res, cfg.dense)) * F
    # read grad, m, v, fp32 value; write m, v, fp32 value, cleared grad (+ the fp16 copy)
    per_param = 16 + 16 + (2 if cfg.table_dtype == "f16" else 0)
    out["adam_tables"] = {"bytes": n_tab * per_param, "flops": 0}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=2, help="1..5 (benchmark configuration number; 5 = one frame of the dynamic scene: rigid "
                         "transform in front of the step, its gradient behind it)")
    ap.add_argument("--rays", type=int, default=None, help="override the number of rays (points for workload 1)")
    ap.add_argument("--ragged", action="store_true",
                    help="rays with their own sample counts (the length mix of a ray marcher) instead of a fixed count")
    ap.add_argument("--marched", action="store_true",
                    help="samples come from the ray marcher: camera rays through a 128^3 occupancy grid around a surface, marched "
                         "inside every timed step (workloads 2..4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one plain device copy of 256 MiB (a kernel of known traffic for counter runs)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures ONE GPU; no multi-GPU path exists; every ray is independent, so the step would shard over rays with one gradient sum per step.",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2212_05231_amd import binding as nb
    from paper_2212_05231_amd import workloads as wl

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    nb.lib()                               # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    w = wl.make_workload(args.workload, n_rays=args.rays)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    if args.ragged:
        if cfg.loss_kind == 0:
            print("bench.py: --ragged needs a workload with rays (2..4)", file=sys.stderr)
            return 2
        # about as many samples as the fixed workload: the mix averages 43 samples per ray
        batch = wl.make_ragged_rays(args.rays or (wl.default_rays(args.workload) * cfg.samples_per_ray) // 43, seed=2000 + args.workload)
        cfg.name = f"cfg{args.workload}-ragged-{batch['dirs'].shape[0]}rays"
    n = batch["pos"].shape[0]
    dynamic = "omega" in batch
    grid = None
    if args.marched:
        if cfg.loss_kind == 0 or dynamic or args.ragged:
            print("bench.py: --marched needs one of the workloads 2..4 and excludes --ragged", file=sys.stderr)
            return 2
        import math
        from paper_2212_05231_amd import occupancy
        R = args.rays or wl.default_rays(args.workload)
        cam = wl.make_camera_rays(R, seed=2000 + args.workload)
        cfg.name = f"cfg{args.workload}-marched-{R}rays"
        step = nb.Step(cfg, params, 128 * R, n_rays=R)
        step.dirs.copy_(torch.from_numpy(cam["dirs"]))
        step.target.copy_(torch.from_numpy(cam["target"]))
        # the grid of a trained scene, made by the library's own update from an analytic SDF: cells whose
        # centre is within 0.03 of a sphere of radius 0.3 (threshold = the logistic density at that distance)
        log2_res, band = 7, 0.03
        e = math.exp(-cfg.s * band)
        grid = occupancy.OccupancyGrid(step, log2_res=log2_res, threshold=cfg.s * e / (1.0 + e) ** 2)
        all_cells = torch.arange(grid.n_cells, dtype=torch.int32, device="cuda")
        nb.occupancy_points(log2_res, all_cells, torch.full((grid.n_cells, 3), 0.5, device="cuda"), grid.pos)
        sdf = ((grid.pos - 0.5).norm(dim=1) - 0.3).contiguous()
        nb.occupancy_update(log2_res, grid.density, all_cells, sdf, 1, grid.n_cells, cfg.s, 1.0, grid.threshold, grid.bitfield)
        origins, jitter = torch.from_numpy(cam["origins"]).cuda(), torch.from_numpy(cam["jitter"]).cuda()
        march_dt, march_steps = math.sqrt(3.0) / 1024, 1024
        n = grid.march(origins, step.dirs, jitter, march_dt, march_steps)
    else:
        step = nb.Step(cfg, params, n, n_rays=batch["dirs"].shape[0] if args.ragged else None, want_pos_grad=dynamic)
        step.set_batch(batch)
    step.zero_grads()
    step.init_optimizer()
    if dynamic:
        # Eq. 9: the frame's points go through x_c = R (x + T) and the map to the unit cube; the
        # gradient with respect to (R, T) is reduced on the device to M (3x3) and b (3)
        from paper_2212_05231_amd import rigid
        rot = rigid.rotation(batch["omega"]).astype(np.float32).reshape(-1)
        shift = batch["shift"].astype(np.float32)
        world = torch.as_tensor(batch["pos"]).cuda()
        Mb = torch.zeros(12, device="cuda")

    def one_step():
        if dynamic:
            nb.rigid_fwd(world, rot, shift, 0.5, 0.5, step.pos)
        if grid is not None:
            # the host reads the sample count back before it can size the step's launches
            step.train_step(grid.march(origins, step.dirs, jitter, march_dt, march_steps))
        else:
            step.train_step()
        if dynamic:
            Mb.zero_()
            nb.rigid_bwd(world, shift, step.d_pos, 0.5, Mb)
        step.adam()

    if args.copy_calibration:
        src = torch.ones(1 << 26, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = 1e3 * dt / args.steps
    value = n * args.steps / dt
    loss_now = [float(x) for x in step.loss.cpu().numpy()[:2]]

    # ---- per-call durations: the same step, driven call by call through the C-ABI in the order
    # neus2_train_step uses, with an event on the kernels' stream between calls, so that every
    # kernel sees the cache state it has inside a step (a call timed alone in a loop runs up to
    # 15 % faster than in the step and would not agree with a rocprofv3 trace of this command)
    kernels = {}
    roofline = None
    if not args.no_kernel_timing:
        c, s = step.c, step
        rays = s.rays
        o = s.opt
        half = 1 if cfg.table_dtype == "f16" else 0
        seq = []
        if grid is not None:
            seq += [("ray_march", lambda: nb.march_rays(grid.log2_res, grid.bitfield, origins, s.dirs, jitter, march_dt, march_steps,
                                                        s.n, s.ray_offsets, s.pos, s.sample_ray))]
        if dynamic:
            seq += [("rigid_fwd", lambda: nb.rigid_fwd(world, rot, shift, 0.5, 0.5, s.pos))]
        seq += [("hash_encode", lambda: nb.hash_encode(c, s.pos[:n], s.tables, s.enc, s.jac)),
               ("sdf_fwd_grad", lambda: nb.sdf_fwd_grad(c, s.enc, s.jac, s.H, n, s.y, s.q, s.normal, masks=s.sdf_masks))]
        if cfg.loss_kind != 0:
            seq += [
                ("color_fwd", lambda: nb.color_fwd(c, s.pos, s.normal, s.dirs, s.y, s.W, n, s.rgb, sample_ray=s.sample_ray,
                                                   masks=s.color_masks)),
                ("render_loss_bwd", (lambda: nb.render_loss_bwd_ragged(c, s.y, s.rgb, s.normal, s.target, s.ray_offsets, rays, n,
                                                                       s.C, s.weights, s.loss, s.dC, s.d_sdf, s.d_rgb, s.d_normal))
                 if s.ragged else
                 (lambda: nb.render_loss_bwd(c, s.y, s.rgb, s.normal, s.target, rays, s.C, s.weights, s.loss,
                                             s.dC, s.d_sdf, s.d_rgb, s.d_normal))),
                ("color_bwd", lambda: nb.color_bwd(c, s.pos, s.normal, s.dirs, s.y, s.W, s.rgb, s.d_rgb, s.d_sdf, n, s.dW,
                                                   s.d_y, s.d_normal, s.d_pos, sample_ray=s.sample_ray, masks=s.color_masks)),
            ]
        else:
            seq += [("loss", lambda: nb.loss(c, None, None, s.normal, s.y, 0, n, s.loss, None, s.d_normal, s.d_y))]
        if dynamic:
            # with the position gradient the two halves share work (the scatter's gather pass adds the
            # first-order part): timed as the one call the step makes
            seq += [("sdf_bwd_2nd", lambda: nb.sdf_bwd_2nd(c, s.pos, s.tables, s.enc, s.jac, s.H, s.q, s.d_y, s.d_normal, n,
                                                           s.dH, s.d_tables, s.d_enc, s.d_pos, workspace=s.workspace,
                                                           masks=s.sdf_masks))]
        else:
            seq += [
                ("sdf_mlp_bwd", lambda: nb.sdf_mlp_bwd(c, s.enc, s.jac, s.H, s.d_y, s.d_normal, n, s.dH, s.d_enc, masks=s.sdf_masks)),
                ("hash_scatter_bwd", lambda: nb.hash_scatter_bwd(c, s.pos[:n], s.tables, s.q, s.d_enc, s.d_normal, n, s.d_tables,
                                                                 workspace=s.workspace)),
            ]
        if dynamic:
            seq += [("rigid_bwd", lambda: nb.rigid_bwd(world, shift, s.d_pos, 0.5, Mb))]
        seq += [
            ("adam_all", lambda: nb.adam_all(c, s.tables, o["master"], s.d_tables, o["m_t"], o["v_t"], s.small, s.d_small,
                                             o["m_s"], o["v_s"], o["lr"], o["b1"], o["b2"], o["eps"], o["t"], True)),
        ]
        cost = algorithmic_cost(cfg, n)
        cost["adam_all"] = {"bytes": cost["adam_tables"]["bytes"] + 32 * int(s.small.numel()), "flops": 0}
        cost["sdf_bwd_2nd"] = {"bytes": cost["sdf_mlp_bwd"]["bytes"] + cost["hash_scatter_bwd"]["bytes"] + 24 * n,
                               "flops": cost["sdf_mlp_bwd"]["flops"], "issued_flops": cost["sdf_mlp_bwd"]["issued_flops"]}
        cost["rigid_fwd"] = {"bytes": 24 * n, "flops": 0}
        cost["rigid_bwd"] = {"bytes": 24 * n, "flops": 0}
        cost["ray_march"] = {"bytes": 32 * rays + 16 * n, "flops": 0}       # a ray's 32 bytes in, a sample's pos + owner out
        reps = max(5, min(args.steps, 100))
        total = {name: 0.0 for name, _ in seq}
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(seq) + 1)] for _ in range(reps)]
        one_step()                                       # the state a step starts from
        for r in range(reps):
            o["t"] += 1
            s.loss.zero_()
            for k, (name, fn) in enumerate(seq):
                events[r][k].record()
                fn()
            events[r][len(seq)].record()
        torch.cuda.synchronize()
        for r in range(reps):
            for k, (name, _) in enumerate(seq):
                total[name] += events[r][k].elapsed_time(events[r][k + 1])
        for name, _ in seq:
            us = 1e3 * total[name] / reps
            k = {"us": round(us, 2), "bytes": cost[name]["bytes"], "flops": cost[name]["flops"],
                 "GBps": round(cost[name]["bytes"] / us * 1e-3, 1)}
            if cost[name]["flops"]:
                k["TFLOPs"] = round(cost[name]["flops"] / us * 1e-6, 2)
            if cost[name].get("issued_flops"):
                k["issued_flops"] = cost[name]["issued_flops"]
                k["issued_TFLOPs"] = round(cost[name]["issued_flops"] / us * 1e-6, 2)
            kernels[name] = k
        dom = max(kernels, key=lambda kk: kernels[kk]["us"])
        kd = kernels[dom]
        # a network kernel is priced by what it issues on the bf16 matrix cores against their peak;
        # everything else by its algorithmic bytes against HBM
        if kd.get("issued_flops") and kd["issued_flops"] / (MFMA_BF16_PEAK_TFLOPS * 1e12) > kd["bytes"] / (HBM_PEAK_GBS * 1e9):
            roofline = {"kernel": dom, "bound": "mfma", "achieved": kd["issued_TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(kd["issued_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4),
                        "algorithmic_fp32_TFLOPs": kd["TFLOPs"]}
        else:
            roofline = {"kernel": dom, "bound": "hbm", "achieved": kd["GBps"], "peak": HBM_PEAK_GBS,
                        "unit": "GB/s", "frac": round(kd["GBps"] / HBM_PEAK_GBS, 4)}
        roofline["us_per_launch"] = kd["us"]
        roofline["hip_kernels"] = KERNELS_OF_CALL.get(dom)
        roofline["algorithmic_bytes"] = kd["bytes"]
        if grid is not None:
            # one refresh of the grid with every cell a candidate (encode + SDF network on 128^3 points, then the update):
            # runs every 16th iteration, outside the timed step
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
            grid.update()
            ev[0].record()
            for _ in range(5):
                grid.update()
            ev[1].record()
            torch.cuda.synchronize()
            kernels["occupancy_refresh"] = {"us": round(1e3 * ev[0].elapsed_time(ev[1]) / 5, 1), "candidate_cells": grid.n_cells,
                                            "note": "every 16th iteration, not part of the timed step"}
        mt = MEASURED_TRAFFIC_MIB.get(cfg.name, {}).get(dom) if n == wl.default_rays(args.workload) * cfg.samples_per_ray else None
        roofline["traffic"] = int((mt[0] + mt[1]) * 1048576) if mt else None

    # ---- CPU baseline: the oracle as it stands, one thread, bounded sample
    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_limits
        from oracle import neus2_oracle as o
        sample_rays = min(128 if step.ragged else 512, step.rays)
        ws = wl.make_workload(args.workload, n_rays=sample_rays)
        if step.ragged:
            ws["batch"] = wl.make_ragged_rays(sample_rays, seed=2000 + args.workload)
        with threadpool_limits(limits=1):
            t0 = time.perf_counter()
            reps = 0
            while True:
                o.train_step(ws["cfg"], ws["params"], ws["batch"])
                reps += 1
                el = time.perf_counter() - t0
                if el > 10.0 or reps >= 8:
                    break
        ns = ws["batch"]["pos"].shape[0]
        cpu = {"value": round(ns * reps / el, 1), "unit": "ray-samples/s", "cores": 1, "kind": "oracle",
               "sample": f"{reps} forward+backward steps of the float64 numpy oracle on {sample_rays} rays "
                         f"({ns} samples) of the same workload (no Adam), {el:.1f} s, BLAS limited to 1 thread"}

    line = {
        "metric": "ray-samples/sec per training step (fwd+2nd-order bwd)",
        "value": round(value, 1), "unit": "ray-samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "points_per_step": n, "rays": step.rays,
                   "samples_per_ray": ("0..128 per ray (ray marcher's mix)" if args.ragged else
                                       f"marched, step sqrt(3)/1024, {n / max(step.rays, 1):.1f} per ray on average" if args.marched else
                                       cfg.samples_per_ray), "levels": cfg.n_levels, "active_levels": cfg.active_levels,
                   "log2_table_size": cfg.log2_table_size, "table_dtype": cfg.table_dtype,
                   "sdf_mlp": cfg.sdf_dims, "color_mlp": cfg.color_dims, "includes_adam": True,
                   "matrix_products": "fp32 values as sums of bf16 terms on the bf16 matrix cores, fp32 accumulation: 3 terms x 6 products "
                                      "where a result is compared at forward tolerance or decides a ReLU mask, 2 terms x 3 products in the adjoint sweeps and weight gradients"},
        "loss": loss_now,
        "roofline": roofline, "cpu_baseline": cpu, "kernels": kernels,
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
