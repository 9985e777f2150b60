"""A small end-to-end training run on an analytic scene (no dataset is needed): a shaded sphere
of radius 0.5 seen from cameras on a sphere of radius 3, black background.

    python -m paper_2212_05231_amd.demo [--steps 400] [--rays 4096] [--march]

Every iteration draws new rays, renders their target colour analytically, and runs the
library's training step (forward, second-order backward, Adam) with the progressive level
schedule of Sec. 4.3.  Prints the loss as it falls and, at the end, how well the sign of the
learnt SDF separates inside from outside on fresh points.  It exercises the step as a
training loop; it is not one of the paper's experiments.

With --march the samples come from the ray marcher instead (supplement Sec. E.3): an occupancy
grid is refreshed from the learnt SDF every 16 iterations and each ray keeps only the lattice
points in occupied cells, so rays have their own sample counts and the batch shrinks as the
grid empties.
"""
from __future__ import annotations

import argparse
import json

import numpy as np

RADIUS = 0.5


def make_batch(rng, n_rays: int, spr: int):
    u = rng.normal(size=(n_rays, 3))
    u /= np.linalg.norm(u, axis=1, keepdims=True)
    o = 3.0 * u
    tgt = rng.uniform(-0.6, 0.6, size=(n_rays, 3))
    v = tgt - o
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    b = np.sum(o * v, axis=1)
    oo = np.sum(o * o, axis=1)
    root = np.sqrt(np.maximum(b * b - (oo - 1.0), 0.0))
    near, far = -b - root, -b + root
    t = near[:, None] + (np.arange(spr)[None, :] + rng.uniform(size=(n_rays, spr))) * ((far - near)[:, None] / spr)
    p = o[:, None, :] + t[:, :, None] * v[:, None, :]
    pos = np.clip((p + 1.0) * 0.5, 0.0, 1.0 - 2.0 ** -24)
    # analytic target: first hit of the sphere |x| = RADIUS, colour 0.5 + 0.5 * normal
    disc = b * b - (oo - RADIUS * RADIUS)
    hit = disc > 0
    th = -b - np.sqrt(np.where(hit, disc, 0.0))
    ph = o + th[:, None] * v
    target = np.where(hit[:, None], 0.5 + 0.5 * ph / RADIUS, 0.0)
    return {"pos": pos.reshape(-1, 3).astype(np.float32), "dirs": v.astype(np.float32), "target": target.astype(np.float32),
            "t": t, "hit": hit, "t_hit": th, "origin": o}


def geometric_init(cfg, params, rng, radius_cube: float) -> None:
    """Start the SDF network near d(x) = |x - centre| - r (the paper initialises geometrically,
    Sec. 4.1, and feeds the position to the network for that: e = (x, h(x)) in Eq. 1).  Here the
    position reaches the network through the encoding itself: trilinear interpolation reproduces
    linear functions exactly, so the two coarsest (dense) levels are filled with the vertex
    coordinates (x, y | z, 1) and declared frozen (inputs, not parameters): the bias-free network
    gets the position and a constant beside 14 trained levels.  The matrices
    follow the usual sphere initialisation of ReLU networks: Gaussian hidden weights of
    variance 2/width on the position channels, a constant sqrt(pi/width) last row, and -r
    carried by a hidden unit that passes the constant through."""
    tab = np.array(params["tables"], dtype=np.float32)
    for level, (c0, c1) in enumerate((("x", "y"), ("z", "one"))):
        assert cfg.dense[level]
        r1 = cfg.res[level] + 1
        idx = np.arange(r1 ** 3)
        coord = {"x": (idx % r1) / cfg.res[level] - 0.5, "y": ((idx // r1) % r1) / cfg.res[level] - 0.5,
                 "z": (idx // (r1 * r1)) / cfg.res[level] - 0.5, "one": np.ones(r1 ** 3)}
        tab[level, :r1 ** 3, 0] = coord[c0]
        tab[level, :r1 ** 3, 1] = coord[c1]
    params["tables"] = tab.astype(params["tables"].dtype)
    H = [np.zeros_like(h, dtype=np.float32) for h in params["H"]]
    width = H[0].shape[0]
    H[0][1:, 0:3] = rng.normal(size=(width - 1, 3)) * np.sqrt(2.0 / (width - 1))
    H[0][0, 3] = 1.0
    for l in range(1, len(H) - 1):
        H[l][1:, 1:] = rng.normal(size=(width - 1, width - 1)) * np.sqrt(2.0 / (width - 1))
        H[l][0, 0] = 1.0
    H[-1][0, 1:] = np.sqrt(np.pi / (width - 1)) + rng.normal(size=width - 1) * 1e-4
    H[-1][0, 0] = -radius_cube
    H[-1][1:, :] = rng.normal(size=(H[-1].shape[0] - 1, width)) * 0.05
    params["H"] = H


def run(steps: int, n_rays: int, seed: int = 0, log=print, march: bool = False):
    import torch
    from . import binding as nb, occupancy, schedule, workloads as wl
    cfg = wl.make_config(2)
    cfg.log2_table_size = 15
    cfg.res = wl.level_resolutions(16, 16, 512)
    cfg.dense = wl.dense_flags(cfg.res, cfg.table_size)
    params = wl.make_params(cfg, seed + 1)
    geometric_init(cfg, params, np.random.default_rng(seed + 2), radius_cube=0.5 * 0.6)
    cfg.frozen_levels = 2          # the two coordinate levels stay what they are: e = (x, h(x))
    n = n_rays * cfg.samples_per_ray
    rng = np.random.default_rng(seed)
    history, marched = [], []
    if march:
        # room for 3 times the fixed batch; marching step 1/128 of the cube's edge
        step = nb.Step(cfg, params, 3 * n, n_rays=n_rays)
        grid = occupancy.OccupancyGrid(step, log2_res=6, decay=0.95, threshold=0.3 * cfg.s / 4)
        dt, max_steps = 1.0 / 128, 256
        gen = torch.Generator(device="cuda")
        gen.manual_seed(seed)
    else:
        step = nb.Step(cfg, params, n)
    step.init_optimizer(lr=1e-2)
    for it in range(steps):
        step.c.active_levels = schedule.active_levels(it, steps, cfg.n_levels)
        if march:
            if it % 16 == 0:
                grid.update(gen)
            b = make_batch(rng, n_rays, 1)
            step.dirs.copy_(torch.from_numpy(b["dirs"]))
            step.target.copy_(torch.from_numpy(b["target"]))
            origins = torch.from_numpy(((b["origin"] + 1.0) * 0.5).astype(np.float32)).cuda()
            jitter = torch.from_numpy(rng.uniform(size=n_rays).astype(np.float32)).cuda()
            n_it = grid.march(origins, step.dirs, jitter, dt, max_steps)
            marched.append(n_it)
            step.train_step(n_it)
        else:
            step.set_batch(make_batch(rng, n_rays, cfg.samples_per_ray))
            step.train_step()
        step.adam()
        if it % 25 == 0 or it == steps - 1:
            l = step.loss.cpu().numpy()
            history.append((it, float(l[0]), float(l[1])))
            log(f"step {it:5d}  levels {step.c.active_levels:2d}  colour loss {l[0]:.4f}  eikonal term {l[1]:.4f}"
                + (f"  samples {marched[-1]:7d}  occupied cells {100 * grid.occupied_fraction():5.1f} %" if march else ""))
    # sign of the learnt SDF against the true one on fresh sample points
    probe = make_batch(rng, 2048, cfg.samples_per_ray)
    step2 = nb.Step(cfg, {"tables": step.tables.cpu().numpy(), "H": [h.cpu().numpy() for h in step.H],
                          "W": [w.cpu().numpy() for w in step.W]}, 2048 * cfg.samples_per_ray)
    step2.set_batch(probe)
    step2.train_step()
    torch.cuda.synchronize()
    d = step2.y[:, 0].cpu().numpy()
    world = probe["pos"].astype(np.float64) * 2.0 - 1.0
    true = np.linalg.norm(world, axis=1) - RADIUS
    # outside the object the rays supervise the field; behind the first surface the transmittance is
    # zero and nothing but the eikonal term constrains it, so the sign is judged outside only
    outside = true > 0.05
    agree = float(np.mean(d[outside] > 0))
    # where the rendered surface is: expected distance of the compositing weights along rays that hit
    wgt = step2.weights.cpu().numpy().reshape(2048, cfg.samples_per_ray).astype(np.float64)
    mass = wgt.sum(axis=1)
    seen = probe["hit"] & (mass > 0.5)
    depth = (wgt * probe["t"]).sum(axis=1) / np.maximum(mass, 1e-12)
    depth_err = float(np.mean(np.abs(depth[seen] - probe["t_hit"][seen])))
    found = float(np.mean(mass[probe["hit"]] > 0.5))
    log(f"outside the sphere the learnt SDF is positive on {100 * agree:.1f} % of {int(outside.sum())} probe points; "
        f"{100 * found:.1f} % of the rays that hit the sphere render a surface, at a mean distance error of {depth_err:.4f} "
        f"(sphere radius {RADIUS}, sample spacing {2.0 / cfg.samples_per_ray:.3f})")
    out = {"history": history, "outside_positive": agree, "surface_found": found, "depth_error": depth_err}
    if march:
        out.update({"samples_first": marched[0], "samples_last": marched[-1], "occupied_fraction": grid.occupied_fraction()})
    return out


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--steps", type=int, default=400)
    ap.add_argument("--rays", type=int, default=4096)
    ap.add_argument("--march", action="store_true", help="sample with the occupancy grid and the ray marcher")
    a = ap.parse_args()
    out = run(a.steps, a.rays, march=a.march)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
