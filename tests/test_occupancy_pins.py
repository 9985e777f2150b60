"""Pins of the occupancy-grid / ray-marcher oracle (supplement Sec. E.3 of arXiv 2212.05231 and
the ray-marching appendix of the publication it cites) against things other than itself.
No GPU, no HIP library."""
import math

import numpy as np
import pytest

from oracle import occupancy_oracle as oc
from paper_2212_05231_amd import workloads as wl


def interleave_by_digits(x, y, z, bits):
    """Morton code built as a string of binary digits, z y x per bit from the top."""
    s = ""
    for b in reversed(range(bits)):
        s += str((z >> b) & 1) + str((y >> b) & 1) + str((x >> b) & 1)
    return int(s, 2)


def test_morton_code_against_digit_interleaving():
    assert oc.morton3(1, 0, 0, 3) == 1 and oc.morton3(0, 1, 0, 3) == 2 and oc.morton3(0, 0, 1, 3) == 4
    assert oc.morton3(7, 7, 7, 3) == 511 and oc.morton3(2, 0, 0, 3) == 8
    rng = np.random.default_rng(0)
    for bits in (1, 4, 7, 8):
        c = rng.integers(0, 1 << bits, size=(200, 3))
        code = oc.morton3(c[:, 0], c[:, 1], c[:, 2], bits)
        want = [interleave_by_digits(int(a), int(b), int(d), bits) for a, b, d in c]
        assert code.tolist() == want
        x, y, z = oc.morton3_inverse(code, bits)
        assert np.array_equal(np.stack([x, y, z], 1), c)
    # a bijection on the whole grid
    g = np.arange(16)
    X, Y, Z = np.meshgrid(g, g, g, indexing="ij")
    assert sorted(oc.morton3(X.ravel(), Y.ravel(), Z.ravel(), 4).tolist()) == list(range(4096))


def test_logistic_density_is_derivative_of_logistic_cdf():
    """phi_s = d/dx of Phi_s(x) = 1 / (1 + e^{-s x}); maximum s/4 at 0; integrates to 1."""
    s = 37.0
    x = np.linspace(-0.4, 0.4, 41)
    h = 1e-6
    cdf = lambda v: 1.0 / (1.0 + np.exp(-s * v))
    fd = (cdf(x + h) - cdf(x - h)) / (2 * h)
    assert np.allclose(oc.logistic_density(x, s), fd, rtol=1e-7, atol=1e-9)
    assert oc.logistic_density(0.0, s) == pytest.approx(s / 4)
    assert np.array_equal(oc.logistic_density(x, s), oc.logistic_density(-x, s))
    xs = np.linspace(-2, 2, 400001)
    assert np.trapezoid(oc.logistic_density(xs, s), xs) == pytest.approx(1.0, abs=1e-9)
    assert np.isfinite(oc.logistic_density(np.array([1e6, -1e6]), 1e3)).all()     # no overflow far away


def test_cell_points_lie_in_their_cells():
    cand = wl.make_candidate_cells(5, 500, 3)
    p = oc.cell_points(cand["cells"], cand["jitter"], 5)
    c = np.floor(p.astype(np.float64) * 32).astype(np.int64)
    assert np.array_equal(oc.morton3(c[:, 0], c[:, 1], c[:, 2], 5), cand["cells"])
    assert p.dtype == np.float32 and (p >= 0).all() and (p < 1).all()


def test_update_decay_maximum_threshold():
    rng = np.random.default_rng(1)
    n = 512
    dens = rng.uniform(0.0, 4.0, size=n)
    s, decay, thr = 16.0, 0.95, 1.5
    # no candidates: k updates multiply by decay^k
    d = dens.copy()
    for _ in range(5):
        d, bits = oc.occupancy_update(d, np.zeros(0, int), np.zeros(0), s, decay, thr)
    assert np.allclose(d, dens * decay ** 5, rtol=1e-14)
    assert np.array_equal(bits, dens * decay ** 5 > thr)
    # candidates: the larger of the decayed value and phi_s(sdf); duplicates keep the maximum
    cells = np.array([3, 3, 7, 100, 100, 100])
    sdf = np.array([0.2, 0.0, 0.5, -0.01, 0.3, 0.02])
    d1, bits = oc.occupancy_update(dens, cells, sdf, s, decay, thr)
    phi = lambda v: s * math.exp(-s * v) / (1 + math.exp(-s * v)) ** 2
    assert d1[3] == pytest.approx(max(dens[3] * decay, phi(0.0)))               # = s/4 = 4
    assert d1[7] == pytest.approx(max(dens[7] * decay, phi(0.5)))
    assert d1[100] == pytest.approx(max(dens[100] * decay, phi(-0.01)))
    untouched = np.ones(n, bool)
    untouched[cells] = False
    assert np.allclose(d1[untouched], dens[untouched] * decay)
    assert bits[3] and np.array_equal(bits, d1 > thr)
    # a value equal to the threshold does not set the bit
    d2, b2 = oc.occupancy_update(np.array([2.0, 2.0]), np.zeros(0, int), np.zeros(0), s, 0.5, 1.0)
    assert not b2.any()
    words = oc.pack_bits(np.arange(64) % 3 == 0)
    assert words[0] == sum(1 << i for i in range(32) if i % 3 == 0)
    assert words[1] == sum(1 << (i - 32) for i in range(32, 64) if i % 3 == 0)


# ---- an independent cell-by-cell traversal in float64 (Amanatides & Woo) ---------------------

def traverse(cells_xyz, o, d):
    """[(ix,iy,iz,t_in,t_out)] of the cells of a [G,G,G] grid over [0,1]^3 that the ray crosses."""
    G = cells_xyz.shape[0]
    o = np.asarray(o, np.float64)
    d = np.asarray(d, np.float64)
    lo, hi = 0.0, math.inf
    for a in range(3):
        if d[a] == 0:
            if not 0 <= o[a] < 1:
                return []
            continue
        t1, t2 = (0 - o[a]) / d[a], (1 - o[a]) / d[a]
        lo, hi = max(lo, min(t1, t2)), min(hi, max(t1, t2))
    if not lo < hi:
        return []
    p = o + (lo + 1e-12) * d
    idx = np.clip(np.floor(p * G).astype(int), 0, G - 1)
    out, t = [], lo
    while t < hi and (idx >= 0).all() and (idx < G).all():
        nxt = [((idx[a] + (1 if d[a] > 0 else 0)) / G - o[a]) / d[a] if d[a] != 0 else math.inf for a in range(3)]
        a = int(np.argmin(nxt))
        t_out = min(nxt[a], hi)
        out.append((idx[0], idx[1], idx[2], t, t_out))
        t = t_out
        idx = idx.copy()
        idx[a] += 1 if d[a] > 0 else -1
    return out


def bits_from_xyz(cells_xyz, log2_res):
    """Morton-ordered bool vector from a [x,y,z] bool array, by the digit-interleaving code."""
    G = 1 << log2_res
    bits = np.zeros(G ** 3, bool)
    for x, y, z in zip(*np.nonzero(cells_xyz)):
        bits[interleave_by_digits(int(x), int(y), int(z), log2_res)] = True
    return bits


@pytest.mark.parametrize("log2_res,seed", [(3, 0), (5, 1)])
def test_marcher_against_cell_traversal(log2_res, seed):
    """Every lattice point well inside an occupied cell is kept, every one well inside an empty
    cell or beyond the cube is not, and kept points lie on the ray at the lattice parameters."""
    G = 1 << log2_res
    rng = np.random.default_rng(seed)
    cells_xyz = wl.make_shell_cells(log2_res, 0.3, 0.08) | (rng.uniform(size=(G, G, G)) < 0.05)
    bits = bits_from_xyz(cells_xyz, log2_res)
    rays = wl.make_camera_rays(60, seed + 10)
    dt = math.sqrt(3) / 200
    margin = 2e-6
    kept_total = 0
    for r in range(60):
        o, d, jit = rays["origins"][r], rays["dirs"][r], rays["jitter"][r]
        k, t, p = oc.march_ray(bits, log2_res, o, d, jit, dt, 400)
        segs = traverse(cells_xyz, o, d)
        if not segs:
            assert len(k) == 0
            continue
        t_near, t_far = segs[0][3], segs[-1][4]
        t0 = t_near + float(jit) * dt
        kept = set(k.tolist())
        assert np.allclose(t, t0 + k * dt, atol=1e-5)
        assert np.allclose(p, o.astype(np.float64) + t[:, None].astype(np.float64) * d, atol=1e-6)
        for kk in range(400):
            tk = t0 + kk * dt
            if tk > t_far + margin:
                assert kk not in kept
                continue
            for (ix, iy, iz, a, b) in segs:
                if a + margin < tk < b - margin:
                    assert (kk in kept) == bool(cells_xyz[ix, iy, iz]), (r, kk)
        kept_total += len(kept)
    assert kept_total > 200


def test_marcher_full_and_empty_grid_and_capacity():
    log2_res = 4
    n_cells = 1 << 12
    rays = wl.make_camera_rays(40, 5)
    dt = 1.0 / 64
    empty = oc.march_rays(np.zeros(n_cells, bool), log2_res, rays["origins"], rays["dirs"], rays["jitter"], dt, 300, 10 ** 6)
    assert empty[0].tolist() == [0] * 41 and len(empty[1]) == 0
    off, pos, owner, t = oc.march_rays(np.ones(n_cells, bool), log2_res, rays["origins"], rays["dirs"],
                                        rays["jitter"], dt, 300, 10 ** 6)
    counts = np.diff(off)
    for r in range(40):
        segs = traverse(np.ones((16, 16, 16), bool), rays["origins"][r], rays["dirs"][r])
        if not segs:
            assert counts[r] == 0
            continue
        chord = segs[-1][4] - segs[0][3] - float(rays["jitter"][r]) * dt
        assert abs(counts[r] - math.ceil(chord / dt)) <= 1          # closed form: lattice points in the chord
        tr = t[off[r]:off[r + 1]]
        assert np.allclose(np.diff(tr), dt, atol=1e-5)
    assert np.array_equal(owner, np.repeat(np.arange(40), counts))
    assert (pos >= -1e-6).all() and (pos <= 1 + 1e-6).all()
    # a step limit cuts each ray, a capacity cuts the batch
    off2 = oc.march_rays(np.ones(n_cells, bool), log2_res, rays["origins"], rays["dirs"], rays["jitter"], dt, 7, 10 ** 6)[0]
    assert np.array_equal(np.diff(off2), np.minimum(counts, 7))
    cap = int(off[17] + 3)
    off3, pos3, owner3, t3 = oc.march_rays(np.ones(n_cells, bool), log2_res, rays["origins"], rays["dirs"],
                                           rays["jitter"], dt, 300, cap)
    assert np.array_equal(off3, np.minimum(off, cap)) and len(pos3) == cap
    assert np.array_equal(pos3, pos[:cap]) and np.array_equal(owner3, owner[:cap])


def test_ray_box_special_cases():
    assert oc.ray_box([0.5, 0.5, -1.0], [0, 0, 1]) == (1.0, 2.0)
    assert oc.ray_box([0.5, 0.5, 0.25], [0, 0, 1]) == (0.0, 0.75)            # starts inside: t_near = 0
    assert oc.ray_box([1.5, 0.5, -1.0], [0, 0, 1]) is None                    # parallel, outside the slab
    assert oc.ray_box([0.5, 0.5, 2.0], [0, 0, 1]) is None                     # cube behind the origin
    n, f = oc.ray_box([-1.0, -1.0, -1.0], np.ones(3) / math.sqrt(3))
    assert n == pytest.approx(math.sqrt(3), rel=1e-6) and f == pytest.approx(2 * math.sqrt(3), rel=1e-6)
