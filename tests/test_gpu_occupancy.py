"""Parity of the occupancy-grid and ray-marching entry points (through the C ABI) with their
oracle.  Integer results (which lattice points are kept, offsets, owners) and the sample
positions, which are single-rounded binary32 expressions on both sides, must agree bit for
bit; densities to 1e-5 relative; occupancy bits exactly wherever the density is not within
that tolerance of the threshold.  Needs an MI355X."""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import neus2_oracle as o
from oracle import occupancy_oracle as oc
from paper_2212_05231_amd import binding as nb
from paper_2212_05231_amd import workloads as wl

pytestmark = pytest.mark.gpu

DENSITY_TOL = 1e-5


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    nb.lib()


def cuda(a, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(a)).to(dtype=dtype).cuda().contiguous()


def words_to_bits(words):
    w = words.cpu().numpy().view(np.uint32)
    return ((w[:, None] >> np.arange(32, dtype=np.uint32)) & 1).astype(bool).reshape(-1)


def morton_bits(cells_xyz, log2_res):
    G = 1 << log2_res
    g = np.arange(G)
    X, Y, Z = np.meshgrid(g, g, g, indexing="ij")
    bits = np.zeros(G ** 3, bool)
    bits[oc.morton3(X.ravel(), Y.ravel(), Z.ravel(), log2_res)] = cells_xyz.ravel()
    return bits


def gpu_march(log2_res, bits, rays, dt, max_steps, capacity, want_t=True):
    R = rays["origins"].shape[0]
    off = torch.full((R + 1,), -7, dtype=torch.int32, device="cuda")
    pos = torch.full((max(capacity, 1), 3), -1.0, device="cuda")
    owner = torch.full((max(capacity, 1),), -1, dtype=torch.int32, device="cuda")
    t = torch.full((max(capacity, 1),), -1.0, device="cuda") if want_t else None
    words = cuda(oc.pack_bits(bits).view(np.int32), torch.int32)
    nb.march_rays(log2_res, words, cuda(rays["origins"]), cuda(rays["dirs"]), cuda(rays["jitter"]), dt, max_steps,
                  capacity, off, pos, owner, t)
    torch.cuda.synchronize()
    return off.cpu().numpy(), pos.cpu().numpy(), owner.cpu().numpy(), (t.cpu().numpy() if want_t else None)


@pytest.mark.parametrize("log2_res", [2, 5, 8])
def test_candidate_points_bit_exact(log2_res):
    m = 5000 + 13
    cand = wl.make_candidate_cells(log2_res, m, 4)
    pos = torch.zeros(m, 3, device="cuda")
    nb.occupancy_points(log2_res, cuda(cand["cells"], torch.int32), cuda(cand["jitter"]), pos)
    torch.cuda.synchronize()
    assert np.array_equal(pos.cpu().numpy(), oc.cell_points(cand["cells"], cand["jitter"], log2_res))


@pytest.mark.parametrize("log2_res,learned", [(2, False), (5, True), (7, False)])
def test_grid_update_against_oracle(log2_res, learned):
    """Three refreshes in a row: decay, maximum at the candidates (with duplicates), threshold."""
    rng = np.random.default_rng(log2_res)
    n_cells = 1 << (3 * log2_res)
    s, decay, thr = 24.0, 0.95, 1.0
    dens_ref = rng.uniform(0.0, 2.0, size=n_cells).astype(np.float32).astype(np.float64)
    dens = cuda(dens_ref)
    words = torch.zeros(max(n_cells // 32, 4), dtype=torch.int32, device="cuda")
    s_dev = cuda(np.array([s], np.float32)) if learned else None
    for it in range(3):
        m = min(n_cells // 2, 40000) if it < 2 else 0
        cand = wl.make_candidate_cells(log2_res, m, 10 + it)
        sdf = (rng.normal(size=(m, 16)) * 0.08).astype(np.float32)
        if m:
            sdf[:3, 0] = [0.0, np.inf, np.nan]                       # s/4; density 0; skipped
        nb.occupancy_update(log2_res, dens, cuda(cand["cells"], torch.int32) if m else None, cuda(sdf) if m else None,
                            16, m, 0.0 if learned else s, decay, thr, words, s_dev=s_dev)
        torch.cuda.synchronize()
        sdf0 = sdf[:, 0].astype(np.float64)
        ok = np.isfinite(sdf0)
        dens_ref, bits_ref = oc.occupancy_update(dens_ref, cand["cells"][ok], sdf0[ok], s, decay, thr)
        got = dens.cpu().numpy().astype(np.float64)
        assert np.all(np.abs(got - dens_ref) <= DENSITY_TOL * np.maximum(dens_ref, 1e-30)), it
        clear = np.abs(dens_ref - thr) > 2 * DENSITY_TOL * thr
        bits = words_to_bits(words)[:n_cells]
        assert np.array_equal(bits[clear], bits_ref[clear]), it
        assert np.array_equal(bits, dens.cpu().numpy() > np.float32(thr)), it   # the bit is the kernel's own comparison
        assert 0.02 < bits.mean() < 0.98
        dens_ref = got                                                # next round starts from what the GPU holds


@pytest.mark.parametrize("log2_res,n_rays,dt,max_steps", [(3, 300, math.sqrt(3) / 200, 400),
                                                          (5, 2500, 1.0 / 64, 150),
                                                          (7, 700, math.sqrt(3) / 1024, 1024)])
def test_marcher_bit_exact(log2_res, n_rays, dt, max_steps):
    """Offsets, owners, positions and parameters of every sample, against the brute-force
    lattice definition; rays that miss the cube, start inside it, stop at max_steps."""
    G = 1 << log2_res
    rng = np.random.default_rng(log2_res)
    cells = wl.make_shell_cells(log2_res, 0.3, 0.06) | (rng.uniform(size=(G, G, G)) < 0.03)
    bits = morton_bits(cells, log2_res)
    rays = wl.make_camera_rays(n_rays, 20 + log2_res)
    rays["origins"][0], rays["dirs"][0] = [0.5, 0.5, -1.0], [0.0, 0.0, 1.0]            # axis-parallel
    rays["origins"][1], rays["dirs"][1] = [1.5, 0.5, -1.0], [0.0, 0.0, 1.0]            # parallel and outside
    off_r, pos_r, own_r, t_r = oc.march_rays(bits, log2_res, rays["origins"], rays["dirs"], rays["jitter"], dt,
                                             max_steps, 10 ** 8)
    n = int(off_r[-1])
    counts = np.diff(off_r)
    assert n > 2 * n_rays and (counts == 0).any() and (counts.max() > 64 or log2_res < 7)
    off, pos, own, t = gpu_march(log2_res, bits, rays, dt, max_steps, n + 100)
    assert np.array_equal(off, off_r)
    assert np.array_equal(own[:n], own_r)
    assert np.array_equal(pos[:n].view(np.uint32), pos_r.view(np.uint32))
    assert np.array_equal(t[:n].view(np.uint32), t_r.view(np.uint32))
    assert (own[n:] == -1).all() and (pos[n:] == -1).all()                  # nothing written past the end
    # a batch with less room: the crossing ray is cut, later rays are empty; t may be left out
    cap = int(off_r[n_rays // 2] + 5)
    off2, pos2, own2, _ = gpu_march(log2_res, bits, rays, dt, max_steps, cap, want_t=False)
    assert np.array_equal(off2, np.minimum(off_r, cap))
    assert np.array_equal(pos2[:cap].view(np.uint32), pos_r[:cap].view(np.uint32))
    assert np.array_equal(own2[:cap], own_r[:cap])


def test_marcher_degenerate_inputs():
    log2_res = 4
    rays = wl.make_camera_rays(130, 3)
    full, empty = np.ones(4096, bool), np.zeros(4096, bool)
    off, pos, own, t = gpu_march(log2_res, empty, rays, 1 / 64, 200, 1000)
    assert (off == 0).all() and (own == -1).all()
    ref = oc.march_rays(full, log2_res, rays["origins"], rays["dirs"], rays["jitter"], 1 / 64, 200, 10 ** 6)
    off, pos, own, t = gpu_march(log2_res, full, rays, 1 / 64, 200, int(ref[0][-1]))
    assert np.array_equal(off, ref[0]) and np.array_equal(pos.view(np.uint32), ref[1].view(np.uint32))
    off, pos, own, t = gpu_march(log2_res, full, rays, 1 / 64, 200, 0)           # no room at all
    assert (off == 0).all()
    none = {k: v[:0] for k, v in rays.items()}
    off, pos, own, t = gpu_march(log2_res, full, none, 1 / 64, 200, 10)         # no rays
    assert off.tolist() == [0]
    with pytest.raises(nb.Neus2Error):
        gpu_march(9, full, rays, 1 / 64, 200, 10)
    with pytest.raises(nb.Neus2Error):
        gpu_march(log2_res, full, rays, 0.0, 200, 10)
    with pytest.raises(nb.Neus2Error):
        gpu_march(log2_res, full, rays, 1 / 64, 0, 10)


def test_marcher_full_size_properties_and_sampled_rays():
    """The benchmark's shape: 4096 camera rays, a 128^3 grid around a surface, step sqrt(3)/1024.
    Every sample lies in an occupied cell and on its ray; 48 rays are recomputed one by one."""
    log2_res, n_rays, dt, max_steps = 7, 4096, math.sqrt(3) / 1024, 1024
    bits = morton_bits(wl.make_shell_cells(log2_res, 0.3, 0.03), log2_res)
    rays = wl.make_camera_rays(n_rays, 1002)
    capacity = 1 << 19
    off, pos, own, t = gpu_march(log2_res, bits, rays, dt, max_steps, capacity)
    n = int(off[-1])
    assert 30 * n_rays < n < capacity and off[0] == 0 and (np.diff(off) >= 0).all()
    assert np.array_equal(own[:n], np.repeat(np.arange(n_rays), np.diff(off)))
    c = np.clip(np.floor(pos[:n] * np.float32(128)).astype(np.int64), 0, 127)
    assert bits[oc.morton3(c[:, 0], c[:, 1], c[:, 2], log2_res)].all()
    line = rays["origins"][own[:n]].astype(np.float64) + t[:n, None].astype(np.float64) * rays["dirs"][own[:n]]
    assert np.abs(pos[:n] - line).max() < 1e-6
    for r in np.random.default_rng(0).choice(n_rays, 48, replace=False):
        _, t_r, p_r = oc.march_ray(bits, log2_res, rays["origins"][r], rays["dirs"][r], rays["jitter"][r], dt, max_steps)
        assert np.array_equal(pos[off[r]:off[r + 1]].view(np.uint32), p_r.view(np.uint32)), r
        assert np.array_equal(t[off[r]:off[r + 1]].view(np.uint32), t_r.view(np.uint32)), r


def test_marched_batch_through_the_training_step():
    """What the marcher writes (offsets, owners, positions, all on the device) is what the step
    for rays of unequal length reads: one step on a marched batch, in buffers sized for more
    samples than the marcher found, against the oracle's step on the oracle's marched batch."""
    log2_res, dt, max_steps = 5, 1.0 / 48, 200
    bits = morton_bits(wl.make_shell_cells(log2_res, 0.3, 0.08), log2_res)
    rays = wl.make_camera_rays(90, 8)
    w = wl.make_workload(2, n_rays=8)
    cfg, params = w["cfg"], w["params"]
    params["tables"] = (params["tables"].astype(np.float64) * 2000.0).astype(params["tables"].dtype)
    off_r, pos_r, own_r, _ = oc.march_rays(bits, log2_res, rays["origins"], rays["dirs"], rays["jitter"], dt, max_steps, 10 ** 6)
    n = int(off_r[-1])
    capacity = n + 333
    step = nb.Step(cfg, params, capacity, n_rays=90)
    step.dirs.copy_(cuda(rays["dirs"]))
    step.target.copy_(cuda(rays["target"]))
    words = cuda(oc.pack_bits(bits).view(np.int32), torch.int32)
    nb.march_rays(log2_res, words, cuda(rays["origins"]), cuda(rays["dirs"]), cuda(rays["jitter"]), dt, max_steps, capacity,
                  step.ray_offsets, step.pos, step.sample_ray)
    n_gpu = int(step.ray_offsets[-1].item())
    assert n_gpu == n and 500 < n
    step.zero_grads()
    step.train_step(n)
    torch.cuda.synchronize()
    batch = {"pos": pos_r, "dirs": rays["dirs"], "target": rays["target"], "ray_offsets": off_r.astype(np.int32),
             "sample_ray": own_r.astype(np.int32)}
    ref = o.train_step(cfg, params, batch)
    rel = lambda a, b: float(np.linalg.norm(np.asarray(a, np.float64) - b) / np.linalg.norm(b))
    L = cfg.n_levels
    flat = lambda tns: tns.cpu().numpy().reshape(-1)[:L * n * 2].reshape(L, n, 2)
    assert rel(np.transpose(flat(step.enc), (1, 0, 2)).reshape(n, -1), ref["he"]["enc"]) <= 1e-5
    assert rel(step.y.cpu().numpy()[:n], ref["y"]) <= 1e-5
    assert rel(step.C.cpu().numpy(), ref["C"]) <= 1e-5
    loss = step.loss.cpu().numpy()
    assert abs(float(loss[0] + loss[1]) - ref["loss"]) <= 1e-5 * abs(ref["loss"])
    assert rel(step.d_tables.cpu().numpy(), ref["dtables"]) <= 1e-4
    for a, b in zip(list(step.dH) + list(step.dW), list(ref["dH"]) + list(ref["dW"])):
        assert rel(a.cpu().numpy(), b) <= 1e-4


def test_grid_refresh_from_the_network_and_candidate_schedule():
    """OccupancyGrid.update strings points -> encode -> SDF network -> update together; its result
    is the oracle's update fed with the oracle's SDF at the same points.  Then the schedule: all
    cells while warming up, afterwards half of the candidates among the occupied cells."""
    from paper_2212_05231_amd import occupancy
    w = wl.make_workload(2, n_rays=8)
    cfg, params = w["cfg"], w["params"]
    params["tables"] = (params["tables"].astype(np.float64) * 3000.0).astype(params["tables"].dtype)
    step = nb.Step(cfg, params, 64, n_rays=1)
    log2_res = 4
    grid = occupancy.OccupancyGrid(step, log2_res=log2_res, decay=0.9, threshold=4.0, warm_updates=1)
    assert grid.occupied_fraction() == 1.0
    m = grid.update()
    torch.cuda.synchronize()
    assert m == 4096
    pos = grid.pos.cpu().numpy()
    assert np.array_equal(pos, oc.cell_points(np.arange(4096), grid.jitter.cpu().numpy(), log2_res))
    he = o.hash_encode(cfg, params["tables"].astype(np.float64), pos.astype(np.float64))
    y = o.mlp_forward([np.asarray(h, np.float64) for h in params["H"]], he["enc"])[0]
    dens_ref, bits_ref = oc.occupancy_update(np.zeros(4096), np.arange(4096), y[:, 0], cfg.s, 0.9, 4.0)
    got = grid.density.cpu().numpy()
    assert np.all(np.abs(got - dens_ref) <= 1e-4 * dens_ref + 1e-30)
    clear = np.abs(dens_ref - 4.0) > 1e-3
    bits = words_to_bits(grid.bitfield)[:4096]
    assert np.array_equal(bits[clear], bits_ref[clear]) and 0.0 < bits.mean() < 1.0
    cand = grid.candidates().cpu().numpy()
    assert len(cand) == 2048 and bits[cand[1024:]].all() and not bits[cand[:1024]].all()


def test_training_loop_with_marched_samples():
    """The demo's loop with the marcher: the grid is refreshed from the learnt SDF, rays keep the
    lattice points in occupied cells, and the rendered surface ends up where the sphere is."""
    from paper_2212_05231_amd import demo
    out = demo.run(steps=200, n_rays=2048, log=lambda *_: None, march=True)
    first, last = out["history"][0][1], out["history"][-1][1]
    assert last < 0.35 * first
    assert out["surface_found"] > 0.95 and out["depth_error"] < 0.06
    assert 0.05 < out["occupied_fraction"] < 0.95 and out["samples_last"] > 2048
