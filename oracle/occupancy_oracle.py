"""CPU oracle for the occupancy grid and the ray marcher that feed the NeuS2 training step
(arXiv 2212.05231, supplement Sec. E.3 "Ray Marching Acceleration").

TEST INFRASTRUCTURE ONLY.  Imported by the tests, never by the product path; shares no code
with the HIP sources.

What the paper fixes: a grid over the unit cube marks each cell empty or non-empty; ray
marching skips the empty cells; the grid is refreshed periodically from the SDF the model
predicts, through the logistic density phi_s(d) = s e^{-s d} / (1 + e^{-s d})^2 with the
trained s, "in the same way as" the publication it cites for the grid.  That publication
(Mueller et al. 2022, appendix on ray marching) gives the steps taken here: each cell keeps a
density value; an update multiplies every value by a decay factor, then raises the values of
a set of candidate cells to the density found at a random point inside each, then sets a
cell's bit when its value exceeds a threshold; cells are numbered along the Morton curve;
samples sit at a fixed step along the ray and those in cells with a clear bit are left out.

Readings where both texts are silent:
  * The threshold and the decay are arguments (the cited publication prints 0.95 and a
    threshold for ITS density; phi_s has another scale, so no constant is taken over).
  * Which cells are candidates, and the point inside each, are random draws: they are inputs.
  * A ray's samples are the lattice points t_k = t_0 + k dt, k = 0, 1, ..., with
    t_0 = t_near + jitter dt, that lie before t_far and whose cell has its bit set; t_near and
    t_far are where the ray enters and leaves the unit cube (slab test, t_near >= 0).  Skipping
    empty cells is an optimisation of the marcher and must not change that set.
  * Whether a lattice point is kept is decided by binary32 arithmetic (the precision of the
    kernel that takes the same decision): every operation below that feeds the decision is a
    single correctly rounded binary32 operation, in the order written, so that the kept set is
    reproducible bit for bit.  The density values are float64.
  * A batch has room for `capacity` samples: rays are laid out in order, the ray that crosses
    the capacity is cut there and all later rays are empty.

Pins (tests/test_occupancy_pins.py): Morton codes against digit-by-digit interleaving; phi_s as
the derivative of the logistic CDF, its maximum s/4 and unit integral; decay^k closed form,
maximum and threshold semantics of the update; the marcher against an independent float64
cell-by-cell traversal (Amanatides-Woo) and against closed forms for a full and an empty grid.
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def morton3(x: np.ndarray, y: np.ndarray, z: np.ndarray, bits: int) -> np.ndarray:
    """Morton code of integer cell coordinates: bit b of x, y, z goes to bit 3b, 3b+1, 3b+2."""
    x = np.asarray(x, dtype=np.int64)
    y = np.asarray(y, dtype=np.int64)
    z = np.asarray(z, dtype=np.int64)
    code = np.zeros_like(x)
    for b in range(bits):
        code |= ((x >> b) & 1) << (3 * b)
        code |= ((y >> b) & 1) << (3 * b + 1)
        code |= ((z >> b) & 1) << (3 * b + 2)
    return code


def morton3_inverse(code: np.ndarray, bits: int):
    code = np.asarray(code, dtype=np.int64)
    x = np.zeros_like(code)
    y = np.zeros_like(code)
    z = np.zeros_like(code)
    for b in range(bits):
        x |= ((code >> (3 * b)) & 1) << b
        y |= ((code >> (3 * b + 1)) & 1) << b
        z |= ((code >> (3 * b + 2)) & 1) << b
    return x, y, z


def logistic_density(d: np.ndarray, s: float) -> np.ndarray:
    """phi_s(d) = s e^{-s d} / (1 + e^{-s d})^2 (supplement Sec. E.3); even in d."""
    e = np.exp(-s * np.abs(np.asarray(d, dtype=np.float64)))
    return s * e / (1.0 + e) ** 2


def cell_points(cells: np.ndarray, jitter: np.ndarray, log2_res: int) -> np.ndarray:
    """The point (cell coordinate + jitter) / G inside each candidate cell, binary32 [M,3]."""
    G = 1 << log2_res
    x, y, z = morton3_inverse(cells, log2_res)
    c = np.stack([x, y, z], axis=1).astype(F32)
    return ((c + np.asarray(jitter, dtype=F32)) * F32(1.0 / G)).astype(F32)


def occupancy_update(density: np.ndarray, cells: np.ndarray, sdf: np.ndarray, s: float,
                     decay: float, threshold: float):
    """One refresh of the grid.  density [G^3] (Morton order) -> (new density, bits [G^3] bool).

    Steps in the cited order: decay every cell; raise each candidate cell to the density at
    its sample point (a cell named twice keeps the larger); a bit is set where the value
    exceeds the threshold.
    """
    out = np.asarray(density, dtype=np.float64) * decay
    phi = logistic_density(sdf, s)
    for c, p in zip(np.asarray(cells, dtype=np.int64), phi):
        if p > out[c]:
            out[c] = p
    return out, out > threshold


def pack_bits(bits: np.ndarray) -> np.ndarray:
    """bool [G^3] -> uint32 words, cell c in bit c % 32 of word c // 32."""
    b = np.asarray(bits, dtype=np.uint32).reshape(-1, 32)
    return (b << np.arange(32, dtype=np.uint32)).sum(axis=1, dtype=np.uint64).astype(np.uint32)


def ray_box(o: np.ndarray, d: np.ndarray):
    """Entry and exit parameter of one ray against [0,1]^3 in binary32, or None on a miss.

    Per axis with d_a != 0: inv = 1/d_a, the two slab parameters (0 - o_a) inv and
    (1 - o_a) inv; with d_a == 0 the ray misses unless 0 <= o_a < 1.  t_near is the largest
    lower parameter and at least 0, t_far the smallest upper one; a miss when t_near >= t_far.
    """
    o = np.asarray(o, dtype=F32)
    d = np.asarray(d, dtype=F32)
    near, far = F32(0.0), F32(np.inf)
    for a in range(3):
        if d[a] == F32(0.0):
            if not (F32(0.0) <= o[a] < F32(1.0)):
                return None
            continue
        with np.errstate(over="ignore"):
            inv = F32(1.0) / d[a]
            t1 = (F32(0.0) - o[a]) * inv
            t2 = (F32(1.0) - o[a]) * inv
        near = max(near, min(t1, t2))
        far = min(far, max(t1, t2))
    if not near < far:
        return None
    return near, far


def march_ray(bits: np.ndarray, log2_res: int, o, d, jitter: float, dt: float, max_steps: int):
    """Lattice indices k, parameters t_k and points of the samples one ray keeps (binary32).

    t_k = t_0 + k dt with t_0 = t_near + jitter dt; point = o + t_k d (a product, then a sum);
    cell = clamp(floor(point G), 0, G-1) per axis; kept when t_k < t_far, k < max_steps and
    the cell's bit is set.
    """
    G = 1 << log2_res
    box = ray_box(o, d)
    if box is None:
        return np.zeros(0, np.int64), np.zeros(0, F32), np.zeros((0, 3), F32)
    near, far = box
    o = np.asarray(o, dtype=F32)
    d = np.asarray(d, dtype=F32)
    dt = F32(dt)
    t0 = F32(near + F32(F32(jitter) * dt))
    k = np.arange(max_steps, dtype=np.int64)
    t = (t0 + (k.astype(F32) * dt).astype(F32)).astype(F32)
    p = (o[None, :] + (t[:, None] * d[None, :]).astype(F32)).astype(F32)
    c = np.clip(np.floor((p * F32(G)).astype(F32)).astype(np.int64), 0, G - 1)
    code = morton3(c[:, 0], c[:, 1], c[:, 2], log2_res)
    keep = (t < far) & np.asarray(bits, dtype=bool)[code]
    return k[keep], t[keep], p[keep]


def march_rays(bits: np.ndarray, log2_res: int, origins, dirs, jitter, dt: float, max_steps: int,
               capacity: int):
    """All rays in order.  Returns ray_offsets [R+1], pos [n,3], sample_ray [n], t [n]."""
    R = len(origins)
    offsets = np.zeros(R + 1, dtype=np.int64)
    pos, ts, owner = [], [], []
    for r in range(R):
        _, t, p = march_ray(bits, log2_res, origins[r], dirs[r], jitter[r], dt, max_steps)
        room = capacity - offsets[r]
        t, p = t[:room], p[:room]
        offsets[r + 1] = offsets[r] + len(t)
        pos.append(p)
        ts.append(t)
        owner.append(np.full(len(t), r, dtype=np.int64))
    return (offsets, np.concatenate(pos) if pos else np.zeros((0, 3), F32),
            np.concatenate(owner) if owner else np.zeros(0, np.int64),
            np.concatenate(ts) if ts else np.zeros(0, F32))
