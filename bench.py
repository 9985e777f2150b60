#!/usr/bin/env python3
"""Benchmark of the NeuS2 training-step hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 4]

A step is one pass of the whole path over one synthetic batch: hash encode (+ Jacobian),
SDF network forward + analytic normal, colour network, compositing, loss, the backward pass
including the second-order term, scatter-add into the table gradient, and Adam on every
parameter (which also clears the gradient buffers).  Inputs and parameters are resident in
HBM before the timed region; two batches are kept there and the steps alternate between
them, so that no step finds the previous step's table lines and streams in the caches.
The default workload is the largest single-GPU configuration (2^20 samples, tables of 2^21
entries).  Prints ONE JSON line.

Besides the headline rate (Adam included) the line carries
  without_adam  the same loop without the optimiser (forward + first- and second-order
                backward only, the quantity the metric's name describes);
  roofline      for the call that takes the largest share of the step: its algorithmic bytes
                (or flops) per launch divided by its average duration, measured here with
                events on the stream the kernels run on;
  kernels       the same figures for every call of the step;
  other_workloads  ms per step and rate of the other benchmark configurations (short runs);
  cpu_baseline  the float64 numpy oracle timed on this machine's host cores on a bounded sample
                of the same workload (a reported baseline, not a target).
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F32_PEAK_TFLOPS = 157.3   # MI355X dense fp32 matrix rate: what the same products would be priced against as fp32 instructions
MFMA_BF16_PEAK_TFLOPS = 2500.0 # MI355X dense bf16 matrix rate: the network kernels run their products as split-bf16 terms

# the HIP kernels behind each timed call (names as rocprofv3 prints them)
KERNELS_OF_CALL = {
    "hash_encode": ["encode_kernel"], "sdf_fwd_grad": ["sdf_fwd_kernel"], "sdf_mlp_bwd": ["sdf_bwd_kernel"],
    "sdf_bwd_2nd": ["sdf_bwd_kernel", "zero_kernel", "bin_rows_kernel", "scatter_owner_kernel", "pos_hessian_kernel", "sum_levels_kernel"],
    "hash_scatter_bwd": ["zero_kernel", "bin_rows_kernel", "scatter_owner_kernel"],
    "adam_all": ["adam_tables_kernel"], "color_fwd": ["color_fwd_kernel"], "color_bwd": ["color_bwd_kernel"],
    "render_loss_bwd": ["render_loss_kernel"], "loss": ["loss_kernel"],
}


def measured_traffic(workload_name, call):
    """HBM-side bytes of one launch of `call` from the committed rocprofv3 counter summary of this
    workload (profiles/hbm_traffic_<workload>.txt: FETCH_SIZE and WRITE_SIZE per dispatch, scaled by
    what the same counters read for a device copy of known size), or None if there is none."""
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{workload_name}.txt")
    if not os.path.exists(path):
        return None
    rows = {}
    for line in open(path):
        m = re.match(r"^(.*?)\s+([\d.]+)\s+([\d.]+)\s+([\d.]+)\s+([\d.]+)\s*$", line)
        if m:
            rows[m.group(1).split("<")[0].strip()] = (float(m.group(4)), float(m.group(5)))      # scaled MiB read, written
    total, found = 0.0, False
    for kern in KERNELS_OF_CALL.get(call, []):
        if kern in rows:
            total += sum(rows[kern])
            found = True
    return int(total * 1048576) if found else None


def algorithmic_cost(cfg, n):
    """Per-launch algorithmic bytes and flops of every call, from per-sample figures.

    Table gathers are counted at element size (8 corners x F x element bytes per level),
    atomics as read + write, every streamed array once.  Flops count the multiply-adds the
    method needs (2 per weight per use); recomputation inside the backward kernels and
    padding of narrow layers are NOT counted.  The encode's figure is the method's (position,
    gathers, encoding); the Jacobian this design also stores (12 bytes per feature) is listed
    separately as `bytes_with_stored_jacobian`.
    """
    lam, D, F = cfg.active_levels, cfg.enc_dim, cfg.n_features
    et = 2 if cfg.table_dtype == "f16" else 4
    K = len(cfg.sdf_dims) - 1
    sd = cfg.sdf_dims
    sdf_w = sum(sd[i] * sd[i + 1] for i in range(K))             # weights of the SDF network
    sweep_w = sum(sd[i] * sd[i + 1] for i in range(K - 1))       # weights the reverse/forward sweeps use
    cost = {
        "hash_encode": {"bytes": 12 + lam * 8 * F * et + D * 4, "flops": 0, "bytes_with_stored_jacobian": 12 + lam * 8 * F * et + D * 4 + D * 12},
        "sdf_fwd_grad": {"bytes": D * 4 + D * 12 + 64 + D * 4 + 12 + 8 * (K - 1), "flops": 2 * sdf_w + 2 * sweep_w + 2 * D * 3},
        "sdf_mlp_bwd": {"bytes": D * 4 + D * 12 + 64 + 12 + D * 4 + 8 * (K - 1),
                        # first order: data + weight gradients; second order: t_0 = J nbar, the t sweep and the
                        # outer products S_l^T t_{l-1}^T (S_K is a unit row: only row 0 of the last matrix)
                        "flops": 4 * sdf_w + 2 * D * 3 + 2 * sweep_w + 2 * (sdf_w - sd[K - 1] * (sd[K] - 1))},
        # position and dL/dn, dd/de and dL/de, and per active level 8 corners x F atomics (read + write)
        "hash_scatter_bwd": {"bytes": 12 + 12 + 2 * D * 4 + lam * 8 * F * 4 * 2, "flops": 0,
                             "bytes_atomics_counted_once": 12 + 12 + 2 * D * 4 + lam * 8 * F * 4},
    }
    if cfg.loss_kind == 1:
        cd = cfg.color_dims
        col_w = sum(cd[i] * cd[i + 1] for i in range(3))
        cost.update({
            "color_fwd": {"bytes": 12 + 12 + 64 + 12 + 16, "flops": 2 * col_w},
            "color_bwd": {"bytes": 12 + 12 + 64 + 12 + 12 + 4 + 64 + 24 + 16, "flops": 2 * col_w + 4 * col_w},
            "render_loss_bwd": {"bytes": 4 + 12 + 12 + 4 + 4 + 12 + 12, "flops": 0},
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
    out = {}
    for k, v in cost.items():
        out[k] = {kk: vv * n for kk, vv in v.items()}
    for k, mf in issued.items():
        if k in out:
            out[k]["issued_flops"] = (mf * 32768 + (32 * 2048 if k.endswith("bwd") else 0)) * n // 32
    # parameters a point can address: a dense level uses (res+1)^3 of its T slots; the levels beyond the
    # active ones have never had a gradient and the step leaves them out (NEUS2_ADAM_ACTIVE_LEVELS)
    n_tab = sum(((r + 1) ** 3 if d else cfg.table_size) for r, d in list(zip(cfg.res, cfg.dense))[:cfg.active_levels]) * F
    # read grad, m, v, fp32 value; write m, v, fp32 value, cleared grad (+ the fp16 copy)
    per_param = 16 + 16 + (2 if cfg.table_dtype == "f16" else 0)
    out["adam_tables"] = {"bytes": n_tab * per_param, "flops": 0}
    return out


class Runner:
    """One workload set up on the GPU: `one_step()` is a whole step (Adam included),
    `one_step(adam=False)` the same without the optimiser."""

    def __init__(self, k, args, torch, nb, wl, np):
        self.k, self.torch, self.nb = k, torch, nb
        rays = args.rays if args.rays and k == args.workload else None
        w = wl.make_workload(k, n_rays=rays)
        self.cfg, params, batch = w["cfg"], w["params"], w["batch"]
        cfg = self.cfg
        self.dynamic = k == 5
        self.grid = None
        self.seq = None
        ragged = args.ragged and k == args.workload
        marched = args.marched and k == args.workload
        if ragged:
            # about as many samples as the fixed workload: the mix averages 43 samples per ray
            batch = wl.make_ragged_rays(rays or (wl.default_rays(k) * cfg.samples_per_ray) // 43, seed=2000 + k)
            cfg.name = f"cfg{k}-ragged-{batch['dirs'].shape[0]}rays"
        self.n = batch["pos"].shape[0]
        dev = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).cuda()
        if self.dynamic:
            # the 20-frame sequence (Sec. 5): every frame its own rays, resident on the device; tables, networks and
            # Adam state carried over; the frame's transform trained, alone for the first iterations of a frame
            from paper_2212_05231_amd import sequence
            R = rays or wl.default_rays(5)
            self.frames = []
            for f in range(20):
                b = wl.make_workload(5, n_rays=R, frame=f)["batch"]
                self.frames.append((dev(b["pos"]), dev(b["dirs"]), dev(b["target"]), b["omega"], b["shift"]))
            self.iters_per_frame = max(5, math.ceil(args.steps / 20))
            self.seq = sequence.DynamicSequence(cfg, params, self.n, transform_only=max(1, self.iters_per_frame // 10))
            self.step = self.seq.step
            self.frame_at, self.done_in_frame = 0, 0
            self.seq.begin_frame(*self.frames[0])
            return
        if marched:
            from paper_2212_05231_amd import occupancy
            R = rays or wl.default_rays(k)
            cam = wl.make_camera_rays(R, seed=2000 + k)
            cfg.name = f"cfg{k}-marched-{R}rays"
            self.step = nb.Step(cfg, params, 128 * R, n_rays=R)
            self.step.dirs.copy_(torch.from_numpy(cam["dirs"]))
            self.step.target.copy_(torch.from_numpy(cam["target"]))
            # the grid of a trained scene, made by the library's own update from an analytic SDF: cells whose
            # centre is within 0.03 of a sphere of radius 0.3 (threshold = the logistic density at that distance)
            log2_res, band = 7, 0.03
            e = math.exp(-cfg.s * band)
            self.grid = grid = occupancy.OccupancyGrid(self.step, log2_res=log2_res, threshold=cfg.s * e / (1.0 + e) ** 2)
            all_cells = torch.arange(grid.n_cells, dtype=torch.int32, device="cuda")
            nb.occupancy_points(log2_res, all_cells, torch.full((grid.n_cells, 3), 0.5, device="cuda"), grid.pos)
            sdf = ((grid.pos - 0.5).norm(dim=1) - 0.3).contiguous()
            nb.occupancy_update(log2_res, grid.density, all_cells, sdf, 1, grid.n_cells, cfg.s, 1.0, grid.threshold, grid.bitfield)
            self.origins, self.jitter = torch.from_numpy(cam["origins"]).cuda(), torch.from_numpy(cam["jitter"]).cuda()
            self.march_dt, self.march_steps = math.sqrt(3.0) / 1024, 1024
            self.n = grid.march(self.origins, self.step.dirs, self.jitter, self.march_dt, self.march_steps)
        else:
            self.step = nb.Step(cfg, params, self.n, n_rays=batch["dirs"].shape[0] if ragged else None)
            self.step.set_batch(batch)
        self.step.zero_grads()
        self.step.init_optimizer()
        # a second batch of the same recipe, resident beside the first; steps alternate between them
        self.batches = [(self.step.pos, self.step.dirs, self.step.target)]
        if not (ragged or marched):
            if k == 1:
                self.batches.append((dev(wl.make_points(self.n, 1500 + k)), self.step.dirs, self.step.target))
            else:
                b2 = wl.make_rays(self.n // cfg.samples_per_ray, cfg.samples_per_ray, 1500 + k)
                self.batches.append((dev(b2["pos"]), dev(b2["dirs"]), dev(b2["target"])))
        self.turn = 0

    def one_step(self, adam=True):
        if self.seq is not None:
            if self.done_in_frame == self.iters_per_frame:
                self.frame_at = (self.frame_at + 1) % 20
                self.done_in_frame = 0
                self.seq.begin_frame(*self.frames[self.frame_at])
            self.seq.iterate()
            self.done_in_frame += 1
            return
        s = self.step
        if len(self.batches) > 1:
            self.turn ^= 1
            pos, dirs, target = self.batches[self.turn]
            s.bind_inputs(pos=pos, dirs=dirs, target=target)
        if self.grid is not None:
            # the host reads the sample count back before it can size the step's launches
            s.train_step(self.grid.march(self.origins, s.dirs, self.jitter, self.march_dt, self.march_steps))
        else:
            s.train_step()
        if adam:
            s.adam()

    def timed(self, steps, warmup, adam=True):
        for _ in range(warmup):
            self.one_step(adam)
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.one_step(adam)
        self.torch.cuda.synchronize()
        return time.perf_counter() - t0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", type=int, default=4,
                    help="1..5 (benchmark configuration number; default 4, the largest single-GPU configuration; 5 = the 20-frame "
                         "dynamic sequence: per-frame rays, trained frame transform, carried state)")
    ap.add_argument("--rays", type=int, default=None, help="override the number of rays (points for workload 1)")
    ap.add_argument("--ragged", action="store_true",
                    help="rays with their own sample counts (the length mix of a ray marcher) instead of a fixed count")
    ap.add_argument("--marched", action="store_true",
                    help="samples come from the ray marcher: camera rays through a 128^3 occupancy grid around a surface, marched "
                         "inside every timed step (workloads 2..4)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-timing", action="store_true")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the short runs of the other configurations")
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
    if (args.ragged or args.marched) and args.workload not in (2, 3, 4):
        print("bench.py: --ragged and --marched need one of the workloads 2..4", file=sys.stderr)
        return 2
    if args.ragged and args.marched:
        print("bench.py: --marched excludes --ragged", file=sys.stderr)
        return 2

    run = Runner(args.workload, args, torch, nb, wl, np)
    cfg, step, n, grid = run.cfg, run.step, run.n, run.grid
    dynamic = run.dynamic
    rays = step.rays
    sequence_info = ({"frames": 20, "iterations_per_frame": run.iters_per_frame, "transform_only_iterations": run.seq.transform_only}
                     if dynamic else None)

    if args.copy_calibration:
        src = torch.ones(1 << 26, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        dst.copy_(src)                      # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    dt = run.timed(args.steps, args.warmup, adam=True)
    ms_per_step = 1e3 * dt / args.steps
    value = n * args.steps / dt
    loss_now = [float(x) for x in step.loss.cpu().numpy()[:2]]
    without_adam = None
    if not dynamic:
        # forward + first- and second-order backward alone (gradients pile up in their buffers meanwhile)
        dt2 = run.timed(args.steps, 2, adam=False)
        without_adam = {"ms_per_step": round(1e3 * dt2 / args.steps, 4), "value": round(n * args.steps / dt2, 1), "unit": "ray-samples/s"}
        step.zero_grads()

    # ---- per-call durations: the same step, driven call by call through the C-ABI in the order
    # neus2_train_step uses, with an event on the kernels' stream between calls, so that every
    # kernel sees the cache state it has inside a step (a call timed alone in a loop runs up to
    # 15 % faster than in the step and would not agree with a rocprofv3 trace of this command)
    kernels = {}
    roofline = None
    if not args.no_kernel_timing:
        c, s = step.c, step
        o = s.opt
        seq = []
        if grid is not None:
            seq += [("ray_march", lambda: nb.march_rays(grid.log2_res, grid.bitfield, run.origins, s.dirs, run.jitter, run.march_dt,
                                                        run.march_steps, s.n, s.ray_offsets, s.pos, s.sample_ray))]
        if dynamic:
            sq = run.seq
            seq += [("rigid_fwd", lambda: nb.rigid_fwd_dev(sq.world, sq.pose, 0.5, 0.5, s.pos))]
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
                                                           masks=s.sdf_masks)),
                    ("rigid_bwd", lambda: nb.rigid_bwd_dev(sq.world, sq.pose, s.d_pos, 0.5, sq.Mb)),
                    ("pose_update", lambda: nb.pose_update(sq.param, sq.m, sq.v, sq.prev, sq.Mb, sq.pose, sq.pose_lr, o["b1"], o["b2"],
                                                           o["eps"], max(sq.t_pose, 1), apply=True))]
        else:
            seq += [
                ("sdf_mlp_bwd", lambda: nb.sdf_mlp_bwd(c, s.enc, s.jac, s.H, s.d_y, s.d_normal, n, s.dH, s.d_enc, masks=s.sdf_masks)),
                ("hash_scatter_bwd", lambda: nb.hash_scatter_bwd(c, s.pos[:n], s.tables, s.q, s.d_enc, s.d_normal, n, s.d_tables,
                                                                 workspace=s.workspace)),
            ]
        seq += [
            ("adam_all", lambda: nb.adam_all(c, s.tables, o["master"], s.d_tables, o["m_t"], o["v_t"], s.small, s.d_small,
                                             o["m_s"], o["v_s"], o["lr"], o["b1"], o["b2"], o["eps"], o["t"], True,
                                             active_levels_only=True)),
        ]
        cost = algorithmic_cost(cfg, n)
        cost["adam_all"] = {"bytes": cost["adam_tables"]["bytes"] + 32 * int(s.small.numel()), "flops": 0}
        cost["sdf_bwd_2nd"] = {"bytes": cost["sdf_mlp_bwd"]["bytes"] + cost["hash_scatter_bwd"]["bytes"] + 24 * n,
                               "flops": cost["sdf_mlp_bwd"]["flops"], "issued_flops": cost["sdf_mlp_bwd"]["issued_flops"]}
        cost["rigid_fwd"] = {"bytes": 24 * n, "flops": 0}
        cost["rigid_bwd"] = {"bytes": 24 * n, "flops": 0}
        cost["pose_update"] = {"bytes": 400, "flops": 0}
        cost["ray_march"] = {"bytes": 32 * rays + 16 * n, "flops": 0}       # a ray's 32 bytes in, a sample's pos + owner out
        reps = max(5, min(args.steps, 100))
        total = {name: 0.0 for name, _ in seq}
        events = [[torch.cuda.Event(enable_timing=True) for _ in range(len(seq) + 1)] for _ in range(reps)]
        run.one_step()                                   # the state a step starts from
        for r in range(reps):
            o["t"] += 1
            if not dynamic and len(run.batches) > 1:
                run.turn ^= 1
                s.bind_inputs(*run.batches[run.turn])
            s.loss.zero_()
            for k, (name, fn) in enumerate(seq):
                events[r][k].record()
                fn()
            events[r][len(seq)].record()
        torch.cuda.synchronize()
        # An event pair also spans any time the stream sat idle waiting for the host (a scheduling hiccup of
        # the Python loop): the average is taken over the repetitions within three times the call's median.
        per_rep = {name: [] for name, _ in seq}
        for r in range(reps):
            for k, (name, _) in enumerate(seq):
                per_rep[name].append(events[r][k].elapsed_time(events[r][k + 1]))
        for name, _ in seq:
            med = sorted(per_rep[name])[len(per_rep[name]) // 2]
            kept = [t for t in per_rep[name] if t <= 3.0 * med]
            total[name] = sum(kept)
            us = 1e3 * total[name] / len(kept)
            k = {"us": round(us, 2), "bytes": cost[name]["bytes"], "flops": cost[name]["flops"],
                 "GBps": round(cost[name]["bytes"] / us * 1e-3, 1)}
            for extra in ("bytes_with_stored_jacobian", "bytes_atomics_counted_once"):
                if extra in cost[name]:
                    k[extra] = cost[name][extra]
                    k["GBps_" + extra[6:]] = round(cost[name][extra] / us * 1e-3, 1)
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
            if "GBps_atomics_counted_once" in kd:
                roofline["frac_atomics_counted_once"] = round(kd["GBps_atomics_counted_once"] / HBM_PEAK_GBS, 4)
        roofline["us_per_launch"] = kd["us"]
        roofline["hip_kernels"] = " + ".join(KERNELS_OF_CALL.get(dom, []))
        roofline["algorithmic_bytes"] = kd["bytes"]
        full_size = n == wl.default_rays(args.workload) * (cfg.samples_per_ray if args.workload != 1 else 1)
        roofline["traffic"] = measured_traffic(cfg.name, dom) if full_size else None
        # the roofline fractions of the two encoder-side calls and the matrix-pipe rates of the network calls, side by side
        roofline["by_call"] = {name: {"us": v["us"], "frac_of_hbm_peak": round(v["GBps"] / HBM_PEAK_GBS, 4),
                                      **({"frac_of_bf16_mfma_peak_issued": round(v["issued_TFLOPs"] / MFMA_BF16_PEAK_TFLOPS, 4),
                                          # the same work counted as the fp32 products it stands for, against the fp32 matrix peak
                                          "frac_of_fp32_mfma_peak_algorithmic": round(v["TFLOPs"] / MFMA_F32_PEAK_TFLOPS, 4)}
                                         if "issued_TFLOPs" in v else {})} for name, v in kernels.items()}
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

    # ---- the other benchmark configurations, short runs (their own lines come from --workload k)
    others = None
    if not args.no_other_workloads and not (args.ragged or args.marched or args.rays):
        others = {}
        del run, step
        torch.cuda.empty_cache()
        for k in (1, 2, 3, 4, 5):
            if k == args.workload:
                continue
            r = Runner(k, argparse.Namespace(rays=None, ragged=False, marched=False, workload=k, steps=40), torch, nb, wl, np)
            d = r.timed(40, 5, adam=True)
            others[r.cfg.name] = {"points_per_step": r.n, "ms_per_step": round(1e3 * d / 40, 4), "value": round(r.n * 40 / d, 1),
                                  "unit": "ray-samples/s", "steps": 40, "includes_adam": True}
            if k == 5:
                others[r.cfg.name]["iterations_per_frame"] = r.iters_per_frame
            del r
            torch.cuda.empty_cache()

    # ---- CPU baseline: the oracle as it stands on a bounded sample, one thread, then all cores
    cpu = None
    if not args.no_cpu_baseline:
        from threadpoolctl import threadpool_limits
        from oracle import neus2_oracle as orc
        ragged = args.ragged
        sample_rays = 128 if ragged else (512 if args.workload != 1 else 4096)
        ws = wl.make_workload(args.workload, n_rays=sample_rays)
        if ragged:
            ws["batch"] = wl.make_ragged_rays(sample_rays, seed=2000 + args.workload)
        if args.workload == 5:
            Rm = orc.rotation_from_axis_angle(ws["batch"]["omega"])
            ws["batch"]["pos"] = orc.rigid_forward(ws["batch"]["pos"], Rm, ws["batch"]["shift"], 0.5, 0.5).astype(np.float32)
        ns = ws["batch"]["pos"].shape[0]
        cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
        # the machine's CPU share for one GPU is 16 threads, whatever the affinity mask shows
        many = min(cores, int(os.environ.get("OMP_NUM_THREADS", "16") or 16))

        def time_oracle(threads, budget):
            with threadpool_limits(limits=threads):
                t0 = time.perf_counter()
                reps = 0
                while True:
                    orc.train_step(ws["cfg"], ws["params"], ws["batch"], want_pos_grad=args.workload == 5)
                    reps += 1
                    el = time.perf_counter() - t0
                    if el > budget or reps >= 8:
                        return reps, el
        reps1, el1 = time_oracle(1, 8.0)
        repsN, elN = time_oracle(many, 8.0)
        cpu = {"value": round(ns * reps1 / el1, 1), "unit": "ray-samples/s", "cores": 1, "kind": "oracle",
               "sample": f"{reps1} forward+backward steps of the float64 numpy oracle on {sample_rays} rays "
                         f"({ns} samples) of the same workload (no Adam), {el1:.1f} s, BLAS limited to 1 thread",
               "all_cores": {"value": round(ns * repsN / elN, 1), "cores": many, "host_cores_visible": cores,
                             "sample": f"{repsN} steps, {elN:.1f} s, BLAS limited to {many} threads (numpy parallelises the matrix "
                                       f"products only; gathers and scatters of the oracle stay on one thread)"}}

    line = {
        "metric": "ray-samples/sec per training step (fwd+2nd-order bwd)",
        "value": round(value, 1), "unit": "ray-samples/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32 (3xbf16 split fwd, 2xbf16 split bwd)", "data": "synthetic",
        "config": {"workload": cfg.name, "points_per_step": n, "rays": rays,
                   "samples_per_ray": ("0..128 per ray (ray marcher's mix)" if args.ragged else
                                       f"marched, step sqrt(3)/1024, {n / max(rays, 1):.1f} per ray on average" if args.marched else
                                       cfg.samples_per_ray), "levels": cfg.n_levels, "active_levels": cfg.active_levels,
                   "log2_table_size": cfg.log2_table_size, "table_dtype": cfg.table_dtype,
                   "sdf_mlp": cfg.sdf_dims, "color_mlp": cfg.color_dims, "includes_adam": True,
                   "batches": "two seeded batches resident in HBM, steps alternate between them" if not dynamic else
                              "20 frames resident in HBM, each with its own rays",
                   "matrix_products": "fp32 values as sums of bf16 terms on the bf16 matrix cores, fp32 accumulation: 3 terms x 6 products "
                                      "where a result is compared at forward tolerance or decides a ReLU mask, 2 terms x 3 products in the adjoint sweeps and weight gradients"},
        "loss": loss_now, "without_adam": without_adam,
        "roofline": roofline, "cpu_baseline": cpu, "other_workloads": others, "kernels": kernels,
    }
    if dynamic:
        line["config"]["sequence"] = sequence_info
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
