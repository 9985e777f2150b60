"""Pins of the float64 oracle against things other than itself: closed forms,
invariants, brute force on tiny inputs, and central finite differences of the
scalar loss.  None of these tests needs a GPU or the HIP library.

Each test names the passage of the paper (arXiv 2212.05231) that fixes the fact
it checks.  The paper prints no worked numeric example, so there are no golden
numbers from it; tests/golden holds two values computed with Python integers.
"""
import copy
import math
import os

import numpy as np
import pytest

from oracle import neus2_oracle as o
from paper_2212_05231_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def tiny_cfg(L=3, log2T=8, active=None, loss_kind=1, spr=8, sdf=(6, 8, 8, 16), res=(4, 7, 13)):
    dense = wl.dense_flags(list(res), 1 << log2T)
    color = [38, 8, 8, 3] if loss_kind >= 1 else []
    return wl.Config(L, 2, log2T, L if active is None else active, "f32", list(res), dense,
                     list(sdf), color, spr, loss_kind, 20.0, 0.1, "tiny")


def tiny_problem(seed=0, rays=5, **kw):
    cfg = tiny_cfg(**kw)
    rng = np.random.default_rng(seed)
    tables = rng.uniform(-0.5, 0.5, size=(cfg.n_levels, cfg.table_size, 2))
    H = [rng.uniform(-1, 1, size=(cfg.sdf_dims[i + 1], cfg.sdf_dims[i])) * 0.6 for i in range(len(cfg.sdf_dims) - 1)]
    W = [rng.uniform(-1, 1, size=(cfg.color_dims[i + 1], cfg.color_dims[i])) * 0.5 for i in range(len(cfg.color_dims) - 1)]
    if cfg.loss_kind >= 1:
        batch = wl.make_rays(rays, cfg.samples_per_ray, seed + 7)
        batch = {k: v.astype(np.float64) for k, v in batch.items()}
    else:
        batch = {"pos": rng.uniform(0.05, 0.95, size=(rays * cfg.samples_per_ray, 3))}
    return cfg, {"tables": tables, "H": H, "W": W}, batch


# ------------------------------------------------------------------ indexing

def test_dense_levels_are_collision_free_and_lexicographic():
    """Sec. 3 'InstantNGP' (grid vertices of a level map into a table of T slots): when
    (res+1)^3 <= T every vertex has its own slot, in x-fastest order."""
    for k in (1, 2, 4):
        cfg = wl.make_config(k)
        for l, res in enumerate(cfg.res):
            if not cfg.dense[l]:
                assert (res + 1) ** 3 > cfg.table_size
                continue
            g = np.arange(res + 1)
            v = np.stack(np.meshgrid(g, g, g, indexing="ij"), axis=-1).reshape(-1, 3)
            idx = o.vertex_index(v, res, 1, cfg.table_size)
            assert idx.max() < cfg.table_size and idx.min() >= 0
            assert len(np.unique(idx)) == (res + 1) ** 3
            brute = [int(x) + int(y) * (res + 1) + int(z) * (res + 1) ** 2 for x, y, z in v[:: max(1, len(v) // 500)]]
            assert brute == list(idx[:: max(1, len(v) // 500)])


def test_hashed_index_against_python_integers():
    """Spatial hash cited by Sec. 3: xor of coordinate*prime with 32-bit wrap-around, mod T."""
    rng = np.random.default_rng(3)
    v = rng.integers(0, 4097, size=(2000, 3))
    v[:50] = rng.integers(60000, 2 ** 20, size=(50, 3))          # products overflow 32 bits
    for log2T in (14, 19, 21):
        T = 1 << log2T
        idx = o.vertex_index(v, 4096, 0, T)
        for (x, y, z), got in zip(v.tolist(), idx.tolist()):
            want = ((x & 0xFFFFFFFF) ^ ((y * 2654435761) & 0xFFFFFFFF) ^ ((z * 805459861) & 0xFFFFFFFF)) % T
            assert got == want
    with open(os.path.join(GOLDEN, "hash_index.txt")) as fh:
        for line in fh:
            if line.startswith("#") or not line.strip():
                continue
            x, y, z, log2T, want = (int(t) for t in line.split())
            assert int(o.vertex_index(np.array([[x, y, z]]), 4096, 0, 1 << log2T)[0]) == want


def test_cell_is_taken_from_the_fp32_product():
    """The cell index is the floor of the binary32 product, so that an fp32 kernel can match it
    exactly; for some points that floor differs from the float64 one, and the oracle must
    follow binary32 there."""
    x32 = np.float32(0.7)
    for res in (10, 30, 100, 1000, 2048):
        p = o.grid_coords(np.array([[x32, x32, x32]], dtype=np.float32), res)
        assert p[0, 0] == float(np.float32(x32 * np.float32(res)))
    # a case where the two roundings fall into different cells
    found = False
    rng = np.random.default_rng(0)
    xs = rng.uniform(0, 1, size=200000).astype(np.float32)
    for res in (111, 153, 561):
        c32 = np.floor((xs * np.float32(res)).astype(np.float32)).astype(np.int64)
        c64 = np.floor(xs.astype(np.float64) * res).astype(np.int64)
        bad = np.nonzero(c32 != c64)[0]
        if len(bad):
            found = True
            pos = np.stack([xs[bad], xs[bad], xs[bad]], axis=1)
            c0, _ = o.cell_and_fraction(o.grid_coords(pos, res), res)
            assert np.array_equal(c0[:, 0], c32[bad])
    assert found


def test_edge_positions_stay_inside_the_grid():
    pos = np.array([[0.0, 1.0, np.nan], [1.0 - 2.0 ** -24, -3.0, 7.0]], dtype=np.float32)
    for res in (16, 22, 2048, 4096):
        c0, w = o.cell_and_fraction(o.grid_coords(pos, res), res)
        assert c0.min() >= 0 and c0.max() <= res - 1
        assert w.min() >= 0.0 and w.max() <= 1.0
    assert o.cell_and_fraction(o.grid_coords(pos, 16), 16)[1][0, 1] == 1.0   # x=1 -> last cell, w=1


# ------------------------------------------------------------------ interpolation

def test_trilinear_weights_partition_unity():
    rng = np.random.default_rng(1)
    w = rng.uniform(0, 1, size=(1000, 3))
    wc, dwc, d2wc = o.corner_weights(w)
    assert np.all(wc >= 0)
    np.testing.assert_allclose(wc.sum(0), 1.0, atol=1e-15)
    np.testing.assert_allclose(dwc.sum(0), 0.0, atol=1e-15)
    np.testing.assert_allclose(d2wc.sum(0), 0.0, atol=1e-15)
    # derivative of the weights by finite differences
    h = 1e-6
    for a in range(3):
        e = np.zeros(3)
        e[a] = h
        fd = (o.corner_weights(w + e)[0] - o.corner_weights(w - e)[0]) / (2 * h)
        np.testing.assert_allclose(dwc[:, :, a], fd, atol=1e-9)
        fd2 = (o.corner_weights(w + e)[1] - o.corner_weights(w - e)[1]) / (2 * h)
        np.testing.assert_allclose(d2wc[:, :, :, a], fd2, atol=1e-9)


def test_interpolation_reproduces_affine_and_trilinear_tables():
    """Interpolating the surrounding vertices (Sec. 3) is exact for a table that samples an
    affine function, and for v_x v_y v_z it gives p_x p_y p_z with the known Jacobian/Hessian."""
    res, log2T = 6, 9
    cfg = wl.Config(1, 2, log2T, 1, "f32", [res], [1], [2, 4, 16], [], 1, 0, 20.0, 0.1)
    g = np.arange(res + 1)
    v = np.stack(np.meshgrid(g, g, g, indexing="ij"), axis=-1).reshape(-1, 3)
    idx = o.vertex_index(v, res, 1, 1 << log2T)
    a, b = np.array([0.3, -1.1, 0.7]), 0.25
    tab = np.zeros((1, 1 << log2T, 2))
    tab[0, idx, 0] = v @ a + b
    tab[0, idx, 1] = v[:, 0] * v[:, 1] * v[:, 2]
    rng = np.random.default_rng(5)
    pos = rng.uniform(0, 1, size=(300, 3))
    he = o.hash_encode(cfg, tab, pos, fp32_product=False, want_hess=True)
    p = pos * res
    np.testing.assert_allclose(he["enc"][:, 0], p @ a + b, atol=1e-12)
    np.testing.assert_allclose(he["jac"][:, 0, :], np.broadcast_to(a * res, (300, 3)), atol=1e-11)
    np.testing.assert_allclose(he["hess"][:, 0], 0.0, atol=1e-9)
    np.testing.assert_allclose(he["enc"][:, 1], p[:, 0] * p[:, 1] * p[:, 2], atol=1e-11)
    jac = np.stack([p[:, 1] * p[:, 2], p[:, 0] * p[:, 2], p[:, 0] * p[:, 1]], axis=1) * res
    np.testing.assert_allclose(he["jac"][:, 1, :], jac, atol=1e-10)
    for (i, j, k) in ((0, 1, 2), (0, 2, 1), (1, 2, 0)):
        np.testing.assert_allclose(he["hess"][:, 1, i, j], p[:, k] * res * res, atol=1e-9)
        np.testing.assert_allclose(he["hess"][:, 1, j, i], p[:, k] * res * res, atol=1e-9)
        np.testing.assert_allclose(he["hess"][:, 1, i, i], 0.0, atol=1e-12)


def test_encoding_by_brute_force_python_loops():
    """Tiny case written out with Python scalars and integers only."""
    cfg, params, batch = tiny_problem(seed=2, rays=2)
    pos = batch["pos"][:5]
    he = o.hash_encode(cfg, params["tables"], pos, fp32_product=False)
    T = cfg.table_size
    for n in range(pos.shape[0]):
        for l, res in enumerate(cfg.res):
            px, py, pz = (float(pos[n, a]) * res for a in range(3))
            cx, cy, cz = (min(int(math.floor(t)), res - 1) for t in (px, py, pz))
            fx, fy, fz = px - cx, py - cy, pz - cz
            acc = [0.0, 0.0]
            dacc = [0.0, 0.0]
            for dz in (0, 1):
                for dy in (0, 1):
                    for dx in (0, 1):
                        X, Y, Z = cx + dx, cy + dy, cz + dz
                        if cfg.dense[l]:
                            slot = X + Y * (res + 1) + Z * (res + 1) ** 2
                        else:
                            slot = ((X & 0xFFFFFFFF) ^ ((Y * 2654435761) & 0xFFFFFFFF) ^ ((Z * 805459861) & 0xFFFFFFFF)) % T
                        wx = fx if dx else 1 - fx
                        wy = fy if dy else 1 - fy
                        wz = fz if dz else 1 - fz
                        for f in range(2):
                            acc[f] += wx * wy * wz * float(params["tables"][l, slot, f])
                            dacc[f] += res * wx * (1.0 if dy else -1.0) * wz * float(params["tables"][l, slot, f])
                        assert he["idx"][n, l, dx + 2 * dy + 4 * dz] == slot
            for f in range(2):
                assert abs(he["enc"][n, 2 * l + f] - acc[f]) < 1e-13
                assert abs(he["jac"][n, 2 * l + f, 1] - dacc[f]) < 1e-11


def test_jacobian_and_hessian_by_finite_differences():
    cfg, params, batch = tiny_problem(seed=4, rays=4)
    pos = batch["pos"]
    he = o.hash_encode(cfg, params["tables"], pos, fp32_product=False, want_hess=True)
    h = 1e-6
    for a in range(3):
        e = np.zeros(3)
        e[a] = h
        hp = o.hash_encode(cfg, params["tables"], pos + e, fp32_product=False, want_hess=True)
        hm = o.hash_encode(cfg, params["tables"], pos - e, fp32_product=False, want_hess=True)
        same = np.all(hp["idx"] == hm["idx"], axis=(1, 2))            # no cell boundary crossed
        assert same.sum() > 0.8 * len(same)
        np.testing.assert_allclose(he["jac"][same, :, a], ((hp["enc"] - hm["enc"]) / (2 * h))[same], rtol=1e-6, atol=1e-7)
        np.testing.assert_allclose(he["hess"][same, :, :, a], ((hp["jac"] - hm["jac"]) / (2 * h))[same], rtol=1e-5, atol=1e-5)


def test_progressive_mask_equals_truncated_model():
    """Sec. 4.3: w_i(lambda) = I[i <= lambda]; a masked run equals a model that only has the
    first lambda levels and the matching columns of H_1."""
    cfg, params, batch = tiny_problem(seed=6, rays=4, active=2)
    full = o.train_step(cfg, params, batch, fp32_product=False)
    cfg2 = copy.deepcopy(cfg)
    cfg2.n_levels, cfg2.active_levels = 2, 2
    cfg2.res, cfg2.dense = cfg.res[:2], cfg.dense[:2]
    cfg2.sdf_dims = [4] + cfg.sdf_dims[1:]
    p2 = {"tables": params["tables"][:2], "H": [params["H"][0][:, :4]] + params["H"][1:], "W": params["W"]}
    cut = o.train_step(cfg2, p2, batch, fp32_product=False)
    assert abs(full["loss"] - cut["loss"]) < 1e-14
    np.testing.assert_allclose(full["dtables"][:2], cut["dtables"], atol=1e-15)
    assert np.all(full["dtables"][2:] == 0.0)
    assert np.all(full["he"]["enc"][:, 4:] == 0.0)
    np.testing.assert_allclose(full["dH"][0][:, :4], cut["dH"][0], atol=1e-15)
    assert np.all(full["dH"][0][:, 4:] == 0.0)
    for a, b in zip(full["dH"][1:] + full["dW"], cut["dH"][1:] + cut["dW"]):
        np.testing.assert_allclose(a, b, atol=1e-15)


# ------------------------------------------------------------------ MLP, Definition 1, Theorem 1

def test_single_matrix_mlp_is_a_matrix_product():
    rng = np.random.default_rng(0)
    H = [rng.normal(size=(5, 7))]
    x = rng.normal(size=(9, 7))
    y, acts, masks = o.mlp_forward(H, x)
    np.testing.assert_allclose(y, x @ H[0].T)
    S, q = o.mlp_input_gradient(H, masks, 2)
    np.testing.assert_allclose(q[0], H[0][2])


def test_hand_computed_2_2_1_network():
    """y = H_2 g(H_1 x) with H_1 = [[1,-2],[3,1]], H_2 = [[2,-1]], x = (1,1):
    z = (-1, 4), a = (0, 4), y = -4, dy/dx = H_2 diag(0,1) H_1 = (-3, -1)."""
    H = [np.array([[1.0, -2.0], [3.0, 1.0]]), np.array([[2.0, -1.0]])]
    y, acts, masks = o.mlp_forward(H, np.array([[1.0, 1.0]]))
    assert y[0, 0] == -4.0 and list(masks[0][0]) == [0.0, 1.0]
    S, q = o.mlp_input_gradient(H, masks, 0)
    assert list(q[0]) == [-3.0, -1.0] and list(S[0][0]) == [0.0, -1.0]
    # the mask is 0 at a pre-activation of exactly zero (Definition 1: G = 1 only if > 0)
    y, acts, masks = o.mlp_forward(H, np.array([[2.0, 1.0]]))
    assert list(masks[0][0]) == [0.0, 1.0]


def _random_mlp(rng, dims):
    return [rng.normal(size=(dims[i + 1], dims[i])) for i in range(len(dims) - 1)]


def test_input_gradient_by_finite_differences_and_zero_second_derivative():
    """Supplement Sec. B: dy/dx = H_L G_L ... G_2 H_1, and Theorem 1's d2y/dx2 = 0 (the
    gradient does not move under a perturbation that flips no mask)."""
    rng = np.random.default_rng(11)
    for dims in ([6, 8, 16], [6, 8, 8, 16], [5, 7, 6, 4, 3]):
        H = _random_mlp(rng, dims)
        x = rng.normal(size=(20, dims[0]))
        y, acts, masks = o.mlp_forward(H, x)
        for i in (0, dims[-1] - 1):
            S, q = o.mlp_input_gradient(H, masks, i)
            h = 1e-7
            for k in range(dims[0]):
                e = np.zeros(dims[0])
                e[k] = h
                yp, _, mp = o.mlp_forward(H, x + e)
                ym, _, mm = o.mlp_forward(H, x - e)
                ok = np.array([all(np.array_equal(a[n], b[n]) for a, b in zip(mp, mm)) for n in range(20)])
                np.testing.assert_allclose(q[ok, k], ((yp - ym) / (2 * h))[ok, i], rtol=1e-6, atol=1e-7)
            dx = 1e-9 * rng.normal(size=x.shape)
            _, _, m2 = o.mlp_forward(H, x + dx)
            same = np.array([all(np.array_equal(a[n], b[n]) for a, b in zip(masks, m2)) for n in range(20)])
            _, q2 = o.mlp_input_gradient(H, m2, i)
            assert same.sum() >= 18
            assert np.array_equal(q[same], q2[same])


def test_theorem1_outer_product_by_finite_differences():
    """Theorem 1: d (dy/dx)_(i,j) / dH_l = (P_l^j S_l^i)^T, with P and S as in Definition 1."""
    rng = np.random.default_rng(12)
    dims = [4, 6, 5, 3]
    H = _random_mlp(rng, dims)
    x = rng.normal(size=(1, dims[0]))
    _, _, masks = o.mlp_forward(H, x)
    K = len(H)
    h = 1e-6
    for i in range(dims[-1]):
        S, _ = o.mlp_input_gradient(H, masks, i)
        S_full = S + [np.eye(dims[-1])[i][None, :]]           # S_K^i = unit row
        for j in range(dims[0]):
            P = [np.eye(dims[0])[j]]                            # P_1^j = column j of the identity
            for l in range(K - 1):
                P.append(masks[l][0] * (H[l] @ P[-1]))          # P_{l+1}^j = G H_l P_l^j
            for l in range(K):
                want = np.outer(S_full[l][0], P[l])             # [n_l, n_{l-1}]
                got = np.zeros_like(H[l])
                for r in range(H[l].shape[0]):
                    for c in range(H[l].shape[1]):
                        Hp = [m.copy() for m in H]
                        Hm = [m.copy() for m in H]
                        Hp[l][r, c] += h
                        Hm[l][r, c] -= h
                        # masks are held fixed: they are piecewise constant in H (proof of Theorem 1)
                        qp = o.mlp_input_gradient(Hp, masks, i)[1][0, j]
                        qm = o.mlp_input_gradient(Hm, masks, i)[1][0, j]
                        got[r, c] = (qp - qm) / (2 * h)
                np.testing.assert_allclose(got, want, atol=1e-8)


# ------------------------------------------------------------------ rendering

def test_logistic_cdf_and_density():
    """Supplement Sec. E.3: phi_s = s e^{-sx}/(1+e^{-sx})^2 is the derivative of Phi_s."""
    x = np.linspace(-0.4, 0.4, 41)
    s, h = 20.0, 1e-6
    fd = (o.logistic_cdf(x + h, s) - o.logistic_cdf(x - h, s)) / (2 * h)
    dens = s * np.exp(-s * x) / (1 + np.exp(-s * x)) ** 2
    np.testing.assert_allclose(fd, dens, rtol=1e-7)
    assert o.logistic_cdf(np.array([0.0]), s)[0] == 0.5


def test_render_closed_forms():
    """Constant ratio Phi_{i+1}/Phi_i = 1-a gives alpha = a on n-1 intervals and
    C = c (1 - (1-a)^(n-1)); weights and the residual transmittance sum to one; an SDF
    that increases along the ray renders black."""
    n, s, a = 12, 20.0, 0.2
    phi = 0.9 * (1 - a) ** np.arange(n)
    sdf = (np.log(phi / (1 - phi)) / s)[None, :]
    rgb = np.broadcast_to(np.array([0.2, 0.5, 0.9]), (1, n, 3))
    C, wgt, alpha, trans = o.render_rays(sdf, rgb, s)
    np.testing.assert_allclose(alpha[0, :-1], a, atol=1e-13)
    assert alpha[0, -1] == 0.0
    np.testing.assert_allclose(C[0], np.array([0.2, 0.5, 0.9]) * (1 - (1 - a) ** (n - 1)), atol=1e-13)
    rng = np.random.default_rng(2)
    sdf = rng.normal(size=(50, n)) * 0.1
    C, wgt, alpha, trans = o.render_rays(sdf, rng.uniform(size=(50, n, 3)), s)
    assert np.all(alpha >= 0) and np.all(alpha <= 1)
    np.testing.assert_allclose(wgt.sum(1) + np.prod(1 - alpha, axis=1), 1.0, atol=1e-13)
    # the division-free form used on the GPU: (1-Phi_{i+1}) (1 - exp(-s (d_i - d_{i+1})))
    alt = (1 - o.logistic_cdf(sdf[:, 1:], s)) * (1 - np.exp(-s * (sdf[:, :-1] - sdf[:, 1:])))
    np.testing.assert_allclose(alpha[:, :-1], np.maximum(alt, 0), atol=1e-14)
    inc = np.sort(sdf, axis=1)
    C, wgt, alpha, _ = o.render_rays(inc, rng.uniform(size=(50, n, 3)), s)
    assert np.all(alpha == 0) and np.all(C == 0)


def test_render_backward_by_finite_differences():
    rng = np.random.default_rng(3)
    R, n, s = 3, 7, 20.0
    sdf = rng.normal(size=(R, n)) * 0.05
    rgb = rng.uniform(size=(R, n, 3))
    dC = rng.normal(size=(R, 3))
    d_sdf, d_rgb = o.render_rays_backward(sdf, rgb, s, dC)
    f = lambda sd, c: float(np.sum(o.render_rays(sd, c, s)[0] * dC))
    h = 1e-6
    for r in range(R):
        for i in range(n):
            e = np.zeros((R, n))
            e[r, i] = h
            assert abs((f(sdf + e, rgb) - f(sdf - e, rgb)) / (2 * h) - d_sdf[r, i]) < 1e-7
            for ch in range(3):
                e3 = np.zeros((R, n, 3))
                e3[r, i, ch] = h
                assert abs((f(sdf, rgb + e3) - f(sdf, rgb - e3)) / (2 * h) - d_rgb[r, i, ch]) < 1e-8


def test_slope_gradient_by_finite_differences():
    """s of Phi_s is a learnable parameter in the paper (supplement Sec. E.3)."""
    rng = np.random.default_rng(8)
    R, n, s = 4, 9, 20.0
    sdf = rng.normal(size=(R, n)) * 0.05
    rgb = rng.uniform(size=(R, n, 3))
    dC = rng.normal(size=(R, 3))
    _, _, d_s = o.render_rays_backward(sdf, rgb, s, dC, want_ds=True)
    f = lambda ss: float(np.sum(o.render_rays(sdf, rgb, ss)[0] * dC))
    h = 1e-5
    assert abs((f(s + h) - f(s - h)) / (2 * h) - d_s) < 1e-8 * max(1.0, abs(d_s))
    assert abs(d_s) > 1e-6


def test_coordinate_levels_feed_the_position_itself():
    """Eq. 1 feeds e = (x, h(x)).  Trilinear interpolation reproduces linear functions exactly, so a
    dense level filled with the vertex coordinates encodes to the position, with the identity as
    Jacobian; declared frozen, such a level gets no table gradient."""
    cfg = tiny_cfg(L=3, log2T=10, res=(4, 7, 13), loss_kind=0)
    rng = np.random.default_rng(3)
    tables = rng.uniform(-0.5, 0.5, size=(3, cfg.table_size, 2))
    for level, cols in enumerate(((0, 1), (2, None))):
        assert cfg.dense[level]
        r1 = cfg.res[level] + 1
        idx = np.arange(r1 ** 3)
        coords = [(idx % r1) / cfg.res[level], ((idx // r1) % r1) / cfg.res[level], (idx // (r1 * r1)) / cfg.res[level]]
        tables[level, :r1 ** 3, 0] = coords[cols[0]]
        tables[level, :r1 ** 3, 1] = coords[cols[1]] if cols[1] is not None else 1.0
    pos = rng.uniform(0.02, 0.98, size=(50, 3))
    he = o.hash_encode(cfg, tables, pos, fp32_product=False)
    np.testing.assert_allclose(he["enc"][:, 0:3], pos, atol=1e-13)
    np.testing.assert_allclose(he["enc"][:, 3], 1.0, atol=1e-13)
    np.testing.assert_allclose(he["jac"][:, 0:3, :], np.broadcast_to(np.eye(3), (50, 3, 3)), atol=1e-11)
    np.testing.assert_allclose(he["jac"][:, 3, :], 0.0, atol=1e-11)
    cfg.frozen_levels = 2
    H = [rng.uniform(-1, 1, size=(cfg.sdf_dims[i + 1], cfg.sdf_dims[i])) * 0.6 for i in range(len(cfg.sdf_dims) - 1)]
    out = o.train_step(cfg, {"tables": tables, "H": H, "W": []}, {"pos": pos}, fp32_product=False)
    assert np.all(out["dtables"][:2] == 0) and np.linalg.norm(out["dtables"][2]) > 0


def test_ragged_rays_reduce_to_rows_and_to_finite_differences():
    """Rays with their own sample counts (supplement Sec. E.3, ray marching): with equal counts the
    ragged compositing is the fixed one; its gradient matches central differences; a ray without
    samples renders black and has no gradient."""
    rng = np.random.default_rng(12)
    R, n, s = 5, 7, 20.0
    sdf = rng.normal(size=(R, n)) * 0.05
    rgb = rng.uniform(size=(R, n, 3))
    off = np.arange(R + 1) * n
    C, w, a = o.render_rays_ragged(sdf.reshape(-1), rgb.reshape(-1, 3), off, s)
    Cf, wf, af, _ = o.render_rays(sdf, rgb, s)
    assert np.array_equal(C, Cf) and np.array_equal(w, wf.reshape(-1)) and np.array_equal(a, af.reshape(-1))
    off = np.array([0, 3, 3, 11, 12, 35])              # lengths 3, 0, 8, 1, 23
    N = off[-1]
    sdf = rng.normal(size=N) * 0.05
    sdf[12:35] = np.linspace(0.2, -0.2, 23)            # a ray that crosses the surface
    rgb = rng.uniform(size=(N, 3))
    dC = rng.normal(size=(5, 3))
    C, w, a = o.render_rays_ragged(sdf, rgb, off, s)
    assert np.all(C[1] == 0) and a[2] == 0 and a[10] == 0 and a[11] == 0 and a[34] == 0    # last samples, empty ray
    assert np.sum(w[12:35]) > 0.9
    d_sdf, d_rgb, d_s = o.render_rays_ragged_backward(sdf, rgb, off, s, dC)
    f = lambda sd, c, ss: float(np.sum(o.render_rays_ragged(sd, c, off, ss)[0] * dC))
    h = 1e-6
    for i in range(N):
        e = np.zeros(N); e[i] = h
        assert abs((f(sdf + e, rgb, s) - f(sdf - e, rgb, s)) / (2 * h) - d_sdf[i]) < 1e-7
    for i in (0, 5, 20):
        e = np.zeros((N, 3)); e[i, 1] = h
        assert abs((f(sdf, rgb + e, s) - f(sdf, rgb - e, s)) / (2 * h) - d_rgb[i, 1]) < 1e-8
    assert abs((f(sdf, rgb, s + 1e-5) - f(sdf, rgb, s - 1e-5)) / 2e-5 - d_s) < 1e-8
    assert d_sdf[11] == 0                              # a single sample has alpha 0: no gradient


def test_huber_closed_forms():
    """Eq. 4 names the Huber loss for the colour term."""
    r = np.array([-0.5, -0.1, -0.03, 0.0, 0.02, 0.1, 0.7])
    d = 0.1
    np.testing.assert_allclose(o.huber(r, d), [0.1 * 0.45, 0.005, 0.00045, 0.0, 0.0002, 0.005, 0.1 * 0.65], atol=1e-15)
    h = 1e-7
    np.testing.assert_allclose(o.huber_derivative(r, d), (o.huber(r + h, d) - o.huber(r - h, d)) / (2 * h), atol=1e-6)


# ------------------------------------------------------------------ spherical harmonics

def test_sh16_addition_theorem_and_orthonormality():
    rng = np.random.default_rng(4)
    v = rng.normal(size=(500, 3))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    Y = o.sh16(v)
    for l in range(4):
        np.testing.assert_allclose((Y[:, l * l:(l + 1) ** 2] ** 2).sum(1), (2 * l + 1) / (4 * math.pi), atol=1e-13)
    # Gauss-Legendre in cos(theta) x uniform in phi integrates degree-6 polynomials exactly
    xs, ws = np.polynomial.legendre.leggauss(8)
    ph = (np.arange(16) + 0.5) * (2 * math.pi / 16)
    ct, pp = np.meshgrid(xs, ph, indexing="ij")
    st = np.sqrt(1 - ct ** 2)
    pts = np.stack([st * np.cos(pp), st * np.sin(pp), ct], axis=-1).reshape(-1, 3)
    wq = np.repeat(ws, 16) * (2 * math.pi / 16)
    Yq = o.sh16(pts)
    np.testing.assert_allclose((Yq * wq[:, None]).T @ Yq, np.eye(16), atol=1e-13)


def test_sh16_index_and_sign_at_the_axes_and_against_the_library_harmonics():
    """Addition theorem and orthonormality do not see a permutation or a sign flip within one
    degree; these do.  At the pole z only the zonal harmonics m = 0 are non-zero and
    Y_l0(z) = sqrt((2l+1)/4 pi) (textbook); at x the values written here by hand.  For general
    directions: scipy's complex Y_l^m (Condon-Shortley phase), from which the real harmonics are
    sqrt(2) (-1)^m Re Y_l^m for m > 0 and sqrt(2) (-1)^m Im Y_l^|m| for m < 0, index l^2 + l + m."""
    Y = o.sh16(np.array([[0.0, 0.0, 1.0], [1.0, 0.0, 0.0]]))
    pole = np.zeros(16)
    pole[[0, 2, 6, 12]] = [0.2820947918, 0.4886025119, 0.6307831305, 0.7463526652]      # sqrt((2l+1)/(4 pi))
    np.testing.assert_allclose(Y[0], pole, atol=1e-9)
    xhat = np.zeros(16)
    xhat[0] = 0.2820947918          # l = 0
    xhat[3] = 0.4886025119          # l = 1, m = +1: sqrt(3/4pi) x
    xhat[6] = -0.3153915653         # l = 2, m = 0: sqrt(5/16pi) (3 z^2 - 1)
    xhat[8] = 0.5462742153          # l = 2, m = +2: sqrt(15/16pi) (x^2 - y^2)
    xhat[13] = -0.4570457995        # l = 3, m = +1: sqrt(21/32pi) x (5 z^2 - 1)
    xhat[15] = 0.5900435899         # l = 3, m = +3: sqrt(35/32pi) x (x^2 - 3 y^2)
    np.testing.assert_allclose(Y[1], xhat, atol=1e-9)
    from scipy.special import sph_harm_y
    rng = np.random.default_rng(9)
    v = rng.normal(size=(200, 3))
    v /= np.linalg.norm(v, axis=1, keepdims=True)
    theta, phi = np.arccos(v[:, 2]), np.arctan2(v[:, 1], v[:, 0])
    want = np.empty((200, 16))
    for l in range(4):
        for m in range(-l, l + 1):
            c = sph_harm_y(l, abs(m), theta, phi)
            want[:, l * l + l + m] = c.real if m == 0 else math.sqrt(2.0) * (-1) ** m * (c.real if m > 0 else c.imag)
    np.testing.assert_allclose(o.sh16(v), want, atol=1e-12)


# ------------------------------------------------------------------ the whole step

def test_loss_scalar_by_hand():
    """The scalar of Eq. 4 as `forward` assembles it (colour term summed over channels, averaged
    over rays; eikonal term averaged over samples, times beta), on a scene small enough to do by
    hand.  One dense level holds (z, 1) at its vertices, so the encoding is e = (z, 1) exactly
    and de/dx = ((0,0,1),(0,0,0)); a single matrix gives d = 1 - 2 z, so n = (0,0,-2), |n| = 2 and
    the eikonal term is (2-1)^2 = 1.  The colour network's last matrix is zero: c = sigmoid(0) = 1/2.
    Ray A: z = 0.475, 0.525 -> d = +0.05, -0.05, s = 20: alpha_0 = 1 - Phi(-1)/Phi(1) = 1 - 1/e,
    alpha_1 = 0, C = (1 - 1/e)/2 per channel.  Ray B: z = 0.525, 0.475 -> d increases, alpha = 0, C = 0."""
    cfg = wl.Config(1, 2, 13, 1, "f32", [16], [1], [2, 16], [38, 8, 8, 3], 2, 1, 20.0, 0.1, "hand")
    tables = np.zeros((1, cfg.table_size, 2))
    v = np.arange(17 ** 3)
    tables[0, :17 ** 3, 0] = (v // (17 * 17)) / 16.0
    tables[0, :17 ** 3, 1] = 1.0
    H = [np.zeros((16, 2))]
    H[0][0] = [-2.0, 1.0]
    rng = np.random.default_rng(0)
    W = [rng.normal(size=(8, 38)), rng.normal(size=(8, 8)), np.zeros((3, 8))]
    pos = np.array([[0.3, 0.6, 0.475], [0.3, 0.6, 0.525], [0.7, 0.2, 0.525], [0.7, 0.2, 0.475]])
    target = np.array([[0.1, 0.5, 0.9], [0.25, 0.0, 0.5]])
    batch = {"pos": pos, "dirs": np.array([[0.0, 0.0, 1.0], [0.0, 0.0, -1.0]]), "target": target}
    fw = o.forward(cfg, {"tables": tables, "H": H, "W": W}, batch)
    np.testing.assert_allclose(fw["y"][:, 0], [0.05, -0.05, -0.05, 0.05], atol=1e-7)      # fp32 grid product
    np.testing.assert_allclose(fw["normal"], np.tile([0.0, 0.0, -2.0], (4, 1)), atol=1e-6)
    c_a = 0.5 * 0.6321205588                                   # (1 - 1/e) / 2
    np.testing.assert_allclose(fw["C"], [[c_a] * 3, [0.0] * 3], atol=1e-7)
    # colour term: ray A |0.3160603 - (0.1, 0.5, 0.9)| = 0.2160603 + 0.1839397 + 0.5839397 = 0.9839397;
    # ray B |0 - (0.25, 0, 0.5)| = 0.75; mean over the two rays 0.86696985; eikonal 0.1 * 1
    assert abs(fw["loss"] - (0.86696985 + 0.1)) < 1e-6
    cfg.loss_kind, cfg.huber_delta = 2, 0.25
    fw = o.forward(cfg, {"tables": tables, "H": H, "W": W}, batch)
    # Huber, delta 1/4: residuals 0.2160603, 0.1839397 are quadratic (r^2/2 = 0.02334103, 0.01691691),
    # 0.5839397 linear (0.25 (r - 0.125) = 0.11473493); ray B: 0.25 quadratic (0.03125), 0, 0.5 linear (0.09375)
    want = (0.02334103 + 0.01691691 + 0.11473493 + 0.03125 + 0.0 + 0.09375) / 2 + 0.1
    assert abs(fw["loss"] - want) < 1e-6

def _fd_param(cfg, params, batch, getter, index, h=1e-6):
    pp, pm = copy.deepcopy(params), copy.deepcopy(params)
    getter(pp)[index] += h
    getter(pm)[index] -= h
    fp = o.forward(cfg, pp, batch, fp32_product=False)
    fm = o.forward(cfg, pm, batch, fp32_product=False)
    same = all(np.array_equal(a, b) for a, b in zip(fp["masks"], fm["masks"]))
    if cfg.loss_kind >= 1:
        same = same and all(np.array_equal(a, b) for a, b in zip(fp["cmasks"], fm["cmasks"]))
        same = same and np.array_equal(np.sign(fp["diff"]), np.sign(fm["diff"]))
        if cfg.loss_kind == 2:
            same = same and np.array_equal(np.abs(fp["diff"]) <= cfg.huber_delta, np.abs(fm["diff"]) <= cfg.huber_delta)
        same = same and np.array_equal(fp["alpha"] > 0, fm["alpha"] > 0)
    return (fp["loss"] - fm["loss"]) / (2 * h), same


def _check_all_grads(cfg, params, batch, out, rng, n_table=60, n_weight=40, tol=2e-6):
    checked = 0
    mats = [("H", l) for l in range(len(params["H"]))] + [("W", l) for l in range(len(params["W"]))]
    for name, l in mats:
        g = out["d" + name][l]
        for _ in range(n_weight):
            r, c = rng.integers(g.shape[0]), rng.integers(g.shape[1])
            fd, same = _fd_param(cfg, params, batch, lambda p: p[name][l], (r, c))
            if same:
                assert abs(fd - g[r, c]) <= tol * max(1.0, abs(fd)), (name, l, r, c, fd, g[r, c])
                checked += 1
    touched = np.argwhere(out["dtables"] != 0.0)
    assert len(touched) > 0
    for t in touched[rng.choice(len(touched), size=min(n_table, len(touched)), replace=False)]:
        fd, same = _fd_param(cfg, params, batch, lambda p: p["tables"], tuple(t))
        if same:
            assert abs(fd - out["dtables"][tuple(t)]) <= tol * max(1.0, abs(fd)), (t, fd, out["dtables"][tuple(t)])
            checked += 1
    # entries no sample touches have exactly zero gradient, and the loss does not depend on them
    used = np.zeros(out["dtables"].shape[:2], dtype=bool)
    for l in range(cfg.active_levels):
        used[l, np.unique(out["he"]["idx"][:, l, :])] = True
    assert np.all(out["dtables"][~used] == 0.0)
    free = np.argwhere(~used)
    if len(free):
        t = tuple(free[0]) + (0,)
        fd, _ = _fd_param(cfg, params, batch, lambda p: p["tables"], t)
        assert fd == 0.0
    return checked


@pytest.mark.parametrize("loss_kind,sdf", [(0, (6, 8, 16)), (0, (6, 8, 8, 16)), (1, (6, 8, 16)), (1, (6, 8, 8, 16)),
                                           (2, (6, 8, 8, 16))])
def test_whole_step_gradients_by_finite_differences(loss_kind, sdf):
    """Eq. 4 loss; Eqs. 5-8 gradients.  Central differences of the scalar loss in float64 wrt
    weights of both networks and touched table entries."""
    cfg, params, batch = tiny_problem(seed=21 + loss_kind, rays=5, loss_kind=loss_kind, sdf=sdf)
    out = o.train_step(cfg, params, batch, fp32_product=False)
    rng = np.random.default_rng(9)
    assert _check_all_grads(cfg, params, batch, out, rng) > 100
    if loss_kind >= 1:
        assert np.any(out["alpha"] > 0.01)           # the render path is really exercised
        # dL/ds against a central difference of the loss in s
        import copy as _copy
        cp, cm = _copy.deepcopy(cfg), _copy.deepcopy(cfg)
        cp.s += 1e-5
        cm.s -= 1e-5
        fd = (o.loss_value(cp, params, batch, False) - o.loss_value(cm, params, batch, False)) / 2e-5
        assert abs(fd - out["d_s"]) < 1e-7 * max(1.0, abs(fd))
    if loss_kind == 2:
        d = np.abs(out["diff"])
        assert np.any(d <= cfg.huber_delta) and np.any(d > cfg.huber_delta)   # both branches of Huber


def test_whole_step_gradients_with_ragged_rays():
    """The same finite-difference check with rays of different lengths (0, 1, short, long)."""
    cfg, params, _ = tiny_problem(seed=27, rays=5, loss_kind=1, sdf=(6, 8, 8, 16))
    batch = wl.make_ragged_rays(14, seed=5, max_len=40)
    batch = {k: (v.astype(np.float64) if v.dtype == np.float32 else v) for k, v in batch.items()}
    lengths = np.diff(batch["ray_offsets"])
    assert np.any(lengths == 0) and np.any(lengths > 20)
    out = o.train_step(cfg, params, batch, fp32_product=False)
    rng = np.random.default_rng(10)
    assert _check_all_grads(cfg, params, batch, out, rng) > 100
    assert np.any(out["alpha"] > 0.01)


def test_second_order_terms_alone_and_negative_controls(monkeypatch):
    """With beta*L_eikonal as the only loss every gradient is a second-order term (Eqs. 7, 8).
    Dropping either kept term must break the finite-difference check; adding the two terms
    Theorem 1 proves zero changes nothing (they are not in the oracle, and FD agrees)."""
    cfg, params, batch = tiny_problem(seed=31, rays=6, loss_kind=0, sdf=(6, 8, 8, 16))
    eik = lambda p: cfg.beta * o.forward(cfg, p, batch, fp32_product=False)["eikonal"]
    out = o.train_step(cfg, params, batch, fp32_product=False)
    rng = np.random.default_rng(1)
    h = 1e-6
    # gradient of the eikonal part alone = total - first-order gradient of mean(d^2)
    y = out["y"]
    N = y.shape[0]
    d_y = np.zeros_like(y)
    d_y[:, 0] = 2 * y[:, 0] / N
    g1, d_enc1, _ = o.mlp_backward(params["H"], out["acts"], out["masks"], d_y)
    for l in range(len(params["H"])):
        g_eik = out["dH"][l] - g1[l]
        assert np.linalg.norm(g_eik) > 1e-6
        nonzero = 0
        for _ in range(25):
            r, c = rng.integers(g_eik.shape[0]), rng.integers(g_eik.shape[1])
            pp, pm = copy.deepcopy(params), copy.deepcopy(params)
            pp["H"][l][r, c] += h
            pm["H"][l][r, c] -= h
            fd = (eik(pp) - eik(pm)) / (2 * h)
            assert abs(fd - g_eik[r, c]) < 2e-6 * max(1, abs(fd))
            nonzero += abs(fd) > 1e-5
        assert nonzero > 0       # the second-order weight gradient is not negligible

    # negative control 1: an oracle without the S^T t^T term fails the whole-step check
    real_einsum = np.einsum

    def no_t(sub, *ops):
        r = real_einsum(sub, *ops)
        return np.zeros_like(r) if sub == "nka,na->nk" else r
    monkeypatch.setattr(o.np, "einsum", no_t)
    broken = o.train_step(cfg, params, batch, fp32_product=False)
    monkeypatch.setattr(o.np, "einsum", real_einsum)
    with pytest.raises(AssertionError):
        _check_all_grads(cfg, params, batch, broken, np.random.default_rng(9))

    # negative control 2: dropping Eq. 7's table term (q * d(dw)/dOmega) fails as well
    broken = dict(out)
    d_enc_only = np.zeros_like(out["dtables"])
    for l in range(cfg.n_levels):
        p = o.grid_coords(batch["pos"], cfg.res[l], False)
        c0, w = o.cell_and_fraction(p, cfg.res[l])
        wc, _, _ = o.corner_weights(w)
        for c, bits in enumerate(o.CORNERS):
            idx = o.vertex_index(c0 + np.array(bits), cfg.res[l], cfg.dense[l], cfg.table_size)
            for f in range(2):
                d_enc_only[l, :, f] += np.bincount(idx, weights=wc[c] * out["d_enc"][:, 2 * l + f], minlength=cfg.table_size)
    broken["dtables"] = d_enc_only
    assert np.linalg.norm(d_enc_only - out["dtables"]) > 1e-3 * np.linalg.norm(out["dtables"])
    with pytest.raises(AssertionError):
        _check_all_grads(cfg, params, batch, broken, np.random.default_rng(9))
    _check_all_grads(cfg, params, batch, out, np.random.default_rng(9))


def test_position_gradient_by_finite_differences():
    """The gradient wrt the encoder's input position includes the mixed second derivative of
    the interpolation (through n) and the colour network's direct use of x."""
    cfg, params, batch = tiny_problem(seed=41, rays=4)
    out = o.train_step(cfg, params, batch, fp32_product=False, want_pos_grad=True)
    h = 1e-6
    rng = np.random.default_rng(2)
    checked = 0
    for _ in range(40):
        n, a = rng.integers(batch["pos"].shape[0]), rng.integers(3)
        bp = dict(batch)
        bm = dict(batch)
        bp["pos"] = batch["pos"].copy()
        bm["pos"] = batch["pos"].copy()
        bp["pos"][n, a] += h
        bm["pos"][n, a] -= h
        fp = o.forward(cfg, params, bp, fp32_product=False)
        fm = o.forward(cfg, params, bm, fp32_product=False)
        if not np.array_equal(fp["he"]["idx"], fm["he"]["idx"]):
            continue
        if not all(np.array_equal(x, y) for x, y in zip(fp["masks"] + fp["cmasks"], fm["masks"] + fm["cmasks"])):
            continue
        fd = (fp["loss"] - fm["loss"]) / (2 * h)
        assert abs(fd - out["dpos"][n, a]) < 2e-6 * max(1, abs(fd))
        checked += 1
    assert checked > 25


# ------------------------------------------------------------------ rigid transform

def test_rotation_and_accumulation_identity():
    """Eq. 9 and the accumulation rule below Eq. 10: R^c_i (x + T^c_i) = R^c_{i-1}(R_i (x + T_i) + T^c_{i-1})."""
    rng = np.random.default_rng(0)
    R1 = o.rotation_from_axis_angle(rng.normal(size=3) * 0.3)
    np.testing.assert_allclose(R1 @ R1.T, np.eye(3), atol=1e-14)
    assert abs(np.linalg.det(R1) - 1) < 1e-14
    np.testing.assert_allclose(o.rotation_from_axis_angle(np.array([0, 0, math.pi / 2])),
                               [[0, -1, 0], [1, 0, 0], [0, 0, 1]], atol=1e-15)
    Rc, Tc = o.rotation_from_axis_angle(rng.normal(size=3) * 0.2), rng.normal(size=3)
    T1 = rng.normal(size=3)
    x = rng.normal(size=(10, 3))
    Rn, Tn = o.accumulate_transform(Rc, Tc, R1, T1)
    lhs = o.rigid_forward(x, Rn, Tn)
    rhs = o.rigid_forward(o.rigid_forward(x, R1, T1), Rc, Tc)
    np.testing.assert_allclose(lhs, rhs, atol=1e-13)
    np.testing.assert_allclose(o.rigid_forward(x, np.eye(3), np.zeros(3)), x)


def test_transform_gradient_by_finite_differences():
    cfg, params, batch = tiny_problem(seed=51, rays=4)
    world = (batch["pos"] * 2 - 1) * 0.8
    omega, T = np.array([0.03, -0.02, 0.05]), np.array([0.02, 0.01, -0.03])

    def loss_of(om, tt):
        b = dict(batch)
        b["pos"] = o.rigid_forward(world, o.rotation_from_axis_angle(om), tt, 0.5, 0.5)
        return o.forward(cfg, params, b, fp32_product=False)["loss"], b
    _, b0 = loss_of(omega, T)
    out = o.train_step(cfg, params, b0, fp32_product=False, want_pos_grad=True)
    Rm = o.rotation_from_axis_angle(omega)
    M, dT, bsum = o.rigid_backward(world, Rm, T, out["dpos"], 0.5)
    dom = o.axis_angle_gradient(omega, M)
    h = 1e-6
    for k in range(3):
        e = np.zeros(3)
        e[k] = h
        fd_t = (loss_of(omega, T + e)[0] - loss_of(omega, T - e)[0]) / (2 * h)
        fd_o = (loss_of(omega + e, T)[0] - loss_of(omega - e, T)[0]) / (2 * h)
        assert abs(fd_t - dT[k]) < 1e-5 * max(1, abs(fd_t)), (k, fd_t, dT[k])
        assert abs(fd_o - dom[k]) < 1e-5 * max(1, abs(fd_o)), (k, fd_o, dom[k])


# ------------------------------------------------------------------ Adam

def test_frame_chain_equals_the_accumulated_transform_and_its_gradient_by_finite_differences():
    """Eq. 9 down the chain of frames against the accumulation rule printed after Eq. 10
    (R_i^c = R_{i-1}^c R_i, T_i^c = T_i + R_i^{-1} T_{i-1}^c): the two routes to the canonical
    frame agree; and `pose_gradient` against central differences of a point loss."""
    rng = np.random.default_rng(12)
    x = rng.normal(size=(30, 3))
    omega, T = np.array([0.05, -0.03, 0.02]), np.array([0.01, 0.04, -0.02])
    R_prev = o.rotation_from_axis_angle(np.array([0.3, 0.1, -0.2]))
    T_prev = np.array([0.2, -0.1, 0.05])
    Rc, Tc = o.accumulate_transform(R_prev, T_prev, o.rotation_from_axis_angle(omega), T)
    np.testing.assert_allclose(o.frame_to_canonical(x, omega, T, R_prev, T_prev), o.rigid_forward(x, Rc, Tc), atol=1e-14)
    np.testing.assert_allclose(o.frame_to_canonical(x, omega, T, np.eye(3), np.zeros(3)),
                               o.rigid_forward(x, o.rotation_from_axis_angle(omega), T), atol=1e-14)
    g = rng.normal(size=(30, 3))
    loss = lambda w, t: float(np.sum(g * o.frame_to_canonical(x, w, t, R_prev, T_prev)))
    d_omega, d_T = o.pose_gradient(x, omega, T, R_prev, T_prev, g)
    h = 1e-6
    for k in range(3):
        e = np.zeros(3)
        e[k] = h
        assert abs((loss(omega + e, T) - loss(omega - e, T)) / (2 * h) - d_omega[k]) < 1e-7
        assert abs((loss(omega, T + e) - loss(omega, T - e)) / (2 * h) - d_T[k]) < 1e-7
    # from the reductions the library keeps: M = sum g (x + Tc)^T and b = sum g give the same gradient
    M, _, b = o.rigid_backward(x, Rc, Tc, g)
    R = o.rotation_from_axis_angle(omega)
    G = R_prev.T @ (M - np.outer(b, R.T @ T_prev))
    np.testing.assert_allclose(o.axis_angle_gradient(omega, G), d_omega, atol=1e-7)
    np.testing.assert_allclose(Rc.T @ b, d_T, atol=1e-12)


def test_adam_closed_forms():
    g = np.array([0.3, -2.0, 0.0, 1e-8])
    p = np.array([1.0, 2.0, 3.0, 4.0])
    lr, eps = 1e-2, 1e-15
    p1, m1, v1 = o.adam_step(p, g, np.zeros(4), np.zeros(4), 1, lr, 0.9, 0.99, eps)
    np.testing.assert_allclose(p1, p - lr * g / (np.abs(g) + eps), rtol=1e-12)
    assert p1[2] == 3.0
    np.testing.assert_allclose(m1, 0.1 * g)
    np.testing.assert_allclose(v1, 0.01 * g * g)
    # second step written out
    g2 = np.array([0.1, 0.1, 0.1, 0.1])
    p2, m2, v2 = o.adam_step(p1, g2, m1, v1, 2, lr, 0.9, 0.99, eps)
    m_want = 0.9 * 0.1 * g + 0.1 * g2
    v_want = 0.99 * 0.01 * g * g + 0.01 * g2 * g2
    want = p1 - lr * (m_want / (1 - 0.81)) / (np.sqrt(v_want / (1 - 0.99 ** 2)) + eps)
    np.testing.assert_allclose(p2, want, rtol=1e-12)


def test_lazy_adam_skips_untouched_entries_only():
    """The sparse form: an entry with a zero gradient keeps value and moments; entries with a
    gradient get the dense update; written out for an entry touched at steps 1 and 3 only."""
    lr, eps, b1, b2 = 1e-2, 1e-15, 0.9, 0.99
    rng = np.random.default_rng(4)
    p, m, v = rng.normal(size=50), rng.normal(size=50) * 1e-2, np.abs(rng.normal(size=50)) * 1e-4
    g = rng.normal(size=50)
    g[::3] = 0.0
    pd, md, vd = o.adam_step(p, g, m, v, 4, lr, b1, b2, eps)
    pl, ml, vl = o.adam_step(p, g, m, v, 4, lr, b1, b2, eps, lazy=True)
    hit = g != 0
    assert np.array_equal(pl[hit], pd[hit]) and np.array_equal(ml[hit], md[hit]) and np.array_equal(vl[hit], vd[hit])
    assert np.array_equal(pl[~hit], p[~hit]) and np.array_equal(ml[~hit], m[~hit]) and np.array_equal(vl[~hit], v[~hit])
    assert not np.array_equal(md[~hit], m[~hit])                   # the dense form decays them
    # one entry, gradients g1, 0, g3
    g1, g3 = 0.5, -0.2
    x, mm, vv = 1.0, 0.0, 0.0
    for t, gt in ((1, g1), (2, 0.0), (3, g3)):
        x, mm, vv = (float(a[0]) for a in o.adam_step([x], [gt], [mm], [vv], t, lr, b1, b2, eps, lazy=True))
    m_want = b1 * (1 - b1) * g1 + (1 - b1) * g3                    # one decay, not two
    v_want = b2 * (1 - b2) * g1 * g1 + (1 - b2) * g3 * g3
    x_want = (1.0 - lr * np.sign(g1)) - lr * (m_want / (1 - b1 ** 3)) / (np.sqrt(v_want / (1 - b2 ** 3)) + eps)
    assert mm == pytest.approx(m_want, rel=1e-14) and vv == pytest.approx(v_want, rel=1e-14)
    assert x == pytest.approx(x_want, rel=1e-12)

