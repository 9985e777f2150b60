"""Float64 CPU oracle for one NeuS2 training step (arXiv 2212.05231).

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what the
HIP library must compute.  It is imported by the tests, by the smoke check and
by the benchmark's CPU-baseline leg, never by the product path, and it shares no
code with the HIP sources.  Everything is numpy in float64 (vectorised over
points, explicit loops over levels, corners, layers and ray samples) so that a
reader can hold each function against the passage of the paper it cites.

What the paper fixes and what it leaves open:
  * Sec. 3 "InstantNGP": L levels, each a table of T feature vectors of size d;
    a point's feature at a level is the interpolation of the vectors at the
    surrounding grid vertices; levels are concatenated.  The paper prints no
    hash function, vertex convention or level spacing; this oracle uses the
    spatial hash of the publication that passage cites (xor of the vertex
    coordinates times the primes 1, 2654435761, 805459861, modulo T), vertices
    at integer coordinates 0..res, and dense lexicographic indexing when all
    (res+1)^3 vertices fit in the table.
  * Eq. 1: (d, g) = f_Theta(e), a bias-free ReLU MLP as in Definition 1.
  * Eq. 2: n = grad_x d, evaluated analytically as (dd/de)(de/dx) with
    dy/dx = H_K G_{K-1} ... G_1 H_1 (Sec. B of the supplement, first display).
  * Eq. 3: c = c_Upsilon(x, n, v, d, g).
  * Supplement Sec. E.3 "Unbiased Volume Rendering": Phi_s, alpha, T, C-hat.
  * Eq. 4: L = L_color + beta * L_eikonal.
  * Eqs. 5-8 and Theorem 1: the gradient that dL/dn sends into Omega and Theta.
  * Sec. 4.3: levels above lambda contribute zeros.
  * Eq. 9: x_{i-1} = R_i (x_i + T_i).

Readings taken where the text is silent are listed at each function.

Parity pins (tests marked "not gpu") cover every function here: central finite
differences of the loss, closed forms, invariants and brute force on tiny
inputs.  The paper prints no worked numeric example, so beyond those pins the
only numeric comparison is oracle <-> HIP.
"""
from __future__ import annotations

import math
from typing import Dict, List, Optional, Sequence

import numpy as np

PRIME_Y = 2654435761
PRIME_Z = 805459861
CORNERS = [((c >> 0) & 1, (c >> 1) & 1, (c >> 2) & 1) for c in range(8)]  # corner c -> (cx, cy, cz)


# --------------------------------------------------------------------------------------
# Hash-grid encoding (Sec. 3 "InstantNGP"; Sec. 4.1 first paragraph)
# --------------------------------------------------------------------------------------

def grid_coords(pos: np.ndarray, res: int, fp32_product: bool = True) -> np.ndarray:
    """Continuous grid coordinate p = x * res of each point at one level, float64 [N,3].

    Reading: x is first clamped to [0,1] (NaN -> 0).  With `fp32_product` the
    product is the single IEEE binary32 multiply fl32(x) * fl32(res) and is only
    then promoted; this is the normative definition, because the cell index
    floor(p) must agree bit for bit with an fp32 kernel.  `fp32_product=False`
    keeps everything in float64 and exists for finite-difference tests, which
    need a function that is continuous in x.
    """
    if fp32_product:
        x = np.nan_to_num(np.asarray(pos, dtype=np.float32), nan=0.0)
        x = np.clip(x, np.float32(0.0), np.float32(1.0))
        p = (x * np.float32(res)).astype(np.float32)
        return p.astype(np.float64)
    x = np.clip(np.nan_to_num(np.asarray(pos, dtype=np.float64), nan=0.0), 0.0, 1.0)
    return x * float(res)


def cell_and_fraction(p: np.ndarray, res: int):
    """Lower cell vertex c0 = min(floor(p), res-1) (int64) and offset w = p - c0 in [0,1]."""
    c0 = np.minimum(np.floor(p), res - 1).astype(np.int64)
    return c0, p - c0


def vertex_index(v: np.ndarray, res: int, dense: int, table_size: int) -> np.ndarray:
    """Table slot of integer vertices v[...,3] (0 <= v <= res) at one level."""
    vx, vy, vz = (v[..., a].astype(np.uint64) for a in range(3))
    if dense:
        stride = np.uint64(res + 1)
        return (vx + vy * stride + vz * stride * stride).astype(np.int64)
    m32 = np.uint64(0xFFFFFFFF)
    h = (vx & m32) ^ ((vy * np.uint64(PRIME_Y)) & m32) ^ ((vz * np.uint64(PRIME_Z)) & m32)
    return (h % np.uint64(table_size)).astype(np.int64)


def corner_weights(w: np.ndarray):
    """Trilinear weights of the 8 cell corners and their derivatives wrt the offset w.

    Returns (wc [8,N], dwc [8,N,3], d2wc [8,N,3,3]).
    """
    n = w.shape[0]
    wc = np.empty((8, n))
    dwc = np.empty((8, n, 3))
    d2wc = np.zeros((8, n, 3, 3))
    for c, bits in enumerate(CORNERS):
        f = [w[:, a] if bits[a] else 1.0 - w[:, a] for a in range(3)]      # factor per axis
        sgn = [1.0 if bits[a] else -1.0 for a in range(3)]                  # its derivative
        wc[c] = f[0] * f[1] * f[2]
        for a in range(3):
            b, k = (a + 1) % 3, (a + 2) % 3
            dwc[c, :, a] = sgn[a] * f[b] * f[k]
            d2wc[c, :, a, b] = sgn[a] * sgn[b] * f[k]
            d2wc[c, :, b, a] = sgn[a] * sgn[b] * f[k]
    return wc, dwc, d2wc


def hash_encode(cfg, tables: np.ndarray, pos: np.ndarray, fp32_product: bool = True,
                want_hess: bool = False) -> Dict[str, np.ndarray]:
    """Multi-resolution encoding h(x), its Jacobian de/dx and (optionally) Hessian.

    tables [L,T,F] (any float dtype; promoted to float64 as stored).
    Returns enc [N,D], jac [N,D,3], hess [N,D,3,3] or None, idx [N,L,8] (int64),
    with feature k = level*F + f.  Levels >= active_levels give zeros
    (Sec. 4.3: w_i(lambda) = I[i <= lambda]); their idx is still reported.
    """
    L, F, T = cfg.n_levels, cfg.n_features, cfg.table_size
    tab = np.asarray(tables).astype(np.float64)
    N = pos.shape[0]
    enc = np.zeros((N, L * F))
    jac = np.zeros((N, L * F, 3))
    hess = np.zeros((N, L * F, 3, 3)) if want_hess else None
    idx_all = np.zeros((N, L, 8), dtype=np.int64)
    for l in range(L):
        res = cfg.res[l]
        p = grid_coords(pos, res, fp32_product)
        c0, w = cell_and_fraction(p, res)
        wc, dwc, d2wc = corner_weights(w)
        for c, bits in enumerate(CORNERS):
            idx = vertex_index(c0 + np.array(bits, dtype=np.int64), res, cfg.dense[l], T)
            idx_all[:, l, c] = idx
            if l >= cfg.active_levels:
                continue
            val = tab[l, idx, :]                                   # [N,F]
            for f in range(F):
                k = l * F + f
                enc[:, k] += wc[c] * val[:, f]
                jac[:, k, :] += res * dwc[c] * val[:, f, None]
                if want_hess:
                    hess[:, k] += float(res) ** 2 * d2wc[c] * val[:, f, None, None]
    return {"enc": enc, "jac": jac, "hess": hess, "idx": idx_all}


# --------------------------------------------------------------------------------------
# SDF network (Eq. 1, Definition 1) and its input gradient (supplement Sec. B)
# --------------------------------------------------------------------------------------

def mlp_forward(H: Sequence[np.ndarray], x: np.ndarray):
    """y = H_K g(H_{K-1} ... g(H_1 x)), g = ReLU, no biases (Definition 1).

    Returns (y [N,n_K], acts [a_0..a_{K-1}], masks [m_1..m_{K-1}]) where the mask
    is 1 where the pre-activation is strictly positive, else 0.
    """
    acts = [np.asarray(x, dtype=np.float64)]
    masks = []
    for Hl in H[:-1]:
        z = acts[-1] @ np.asarray(Hl, dtype=np.float64).T
        m = (z > 0.0).astype(np.float64)
        masks.append(m)
        acts.append(m * z)
    y = acts[-1] @ np.asarray(H[-1], dtype=np.float64).T
    return y, acts, masks


def mlp_input_gradient(H: Sequence[np.ndarray], masks: Sequence[np.ndarray], i: int = 0):
    """Row i of dy/dx = H_K G_{K-1} ... G_1 H_1 for every point.

    Returns (S, q): S[l-1] = S_l^i of Definition 1 for l = 1..K-1 (the row vector
    H_K^(i,_) G ... H_{l+1} G, shape [N,n_l]) and q = S_1^i H_1 [N,n_0].
    """
    K = len(H)
    n_pts = masks[0].shape[0] if masks else None
    row = np.asarray(H[-1], dtype=np.float64)[i]
    if K == 1:
        return [], row[None, :]
    S: List[Optional[np.ndarray]] = [None] * (K - 1)
    S[K - 2] = row[None, :] * masks[K - 2]
    for l in range(K - 2, 0, -1):                       # S_l from S_{l+1}
        S[l - 1] = (S[l] @ np.asarray(H[l], dtype=np.float64)) * masks[l - 1]
    q = S[0] @ np.asarray(H[0], dtype=np.float64)
    assert n_pts is None or q.shape[0] == n_pts
    return S, q


# --------------------------------------------------------------------------------------
# Colour network (Eq. 3)
# --------------------------------------------------------------------------------------

def sh16(dirs: np.ndarray) -> np.ndarray:
    """Real orthonormal spherical harmonics of degree 0..3 at unit vectors, [R,16].

    Index l*l + l + m, m = -l..l.  (The direction encoding is the benchmark
    configuration's; the paper only says v is an input.)
    """
    d = np.asarray(dirs, dtype=np.float64)
    x, y, z = d[:, 0], d[:, 1], d[:, 2]
    pi = math.pi
    out = np.empty((d.shape[0], 16))
    out[:, 0] = 0.5 * math.sqrt(1.0 / pi)
    c1 = math.sqrt(3.0 / (4.0 * pi))
    out[:, 1] = c1 * y
    out[:, 2] = c1 * z
    out[:, 3] = c1 * x
    out[:, 4] = 0.5 * math.sqrt(15.0 / pi) * x * y
    out[:, 5] = 0.5 * math.sqrt(15.0 / pi) * y * z
    out[:, 6] = 0.25 * math.sqrt(5.0 / pi) * (3.0 * z * z - 1.0)
    out[:, 7] = 0.5 * math.sqrt(15.0 / pi) * x * z
    out[:, 8] = 0.25 * math.sqrt(15.0 / pi) * (x * x - y * y)
    out[:, 9] = 0.25 * math.sqrt(35.0 / (2.0 * pi)) * y * (3.0 * x * x - y * y)
    out[:, 10] = 0.5 * math.sqrt(105.0 / pi) * x * y * z
    out[:, 11] = 0.25 * math.sqrt(21.0 / (2.0 * pi)) * y * (5.0 * z * z - 1.0)
    out[:, 12] = 0.25 * math.sqrt(7.0 / pi) * z * (5.0 * z * z - 3.0)
    out[:, 13] = 0.25 * math.sqrt(21.0 / (2.0 * pi)) * x * (5.0 * z * z - 1.0)
    out[:, 14] = 0.25 * math.sqrt(105.0 / pi) * z * (x * x - y * y)
    out[:, 15] = 0.25 * math.sqrt(35.0 / (2.0 * pi)) * x * (x * x - 3.0 * y * y)
    return out


def color_input(pos, normal, dirs, y, samples_per_ray) -> np.ndarray:
    """[x(3), n(3), SH16(v)(16), (d,g)(16)] per sample; v is the sample's ray direction.
    `samples_per_ray` is one count for all rays or an array with one count per ray."""
    sh = np.repeat(sh16(dirs), samples_per_ray, axis=0)
    return np.concatenate([np.asarray(pos, dtype=np.float64), normal, sh, y], axis=1)


def color_forward(W: Sequence[np.ndarray], cin: np.ndarray):
    """c = sigmoid(W_3 g(W_2 g(W_1 cin))), bias-free; returns (rgb, acts, masks)."""
    u, acts, masks = mlp_forward(W, cin)
    return 1.0 / (1.0 + np.exp(-u)), acts, masks


# --------------------------------------------------------------------------------------
# Volume rendering (supplement Sec. E.3)
# --------------------------------------------------------------------------------------

def logistic_cdf(x: np.ndarray, s: float) -> np.ndarray:
    return 1.0 / (1.0 + np.exp(-s * x))


def render_rays(sdf: np.ndarray, rgb: np.ndarray, s: float):
    """alpha_i = max((Phi(d_i)-Phi(d_{i+1}))/Phi(d_i), 0), T_i = prod_{j<i}(1-alpha_j),
    C = sum_i T_i alpha_i c_i.  Reading: the last sample has no successor, alpha_{n-1} = 0.

    sdf [R,n], rgb [R,n,3] -> (C [R,3], weights T*alpha [R,n], alpha [R,n], trans [R,n]).
    """
    R, n = sdf.shape
    phi = logistic_cdf(sdf, s)
    alpha = np.zeros((R, n))
    alpha[:, :-1] = np.maximum((phi[:, :-1] - phi[:, 1:]) / phi[:, :-1], 0.0)
    trans = np.ones((R, n))
    for i in range(1, n):
        trans[:, i] = trans[:, i - 1] * (1.0 - alpha[:, i - 1])
    wgt = trans * alpha
    C = np.sum(wgt[:, :, None] * rgb, axis=1)
    return C, wgt, alpha, trans


def render_rays_backward(sdf, rgb, s, dC, want_ds: bool = False):
    """Gradient of sum(dC * C) wrt sdf [R,n] and rgb [R,n,3], straight from the definitions;
    with `want_ds` also wrt the slope s of Phi_s (the paper keeps s learnable, supplement
    Sec. E.3), returned as a third value.

    dC/dalpha_i is written out with the explicit product over the other factors
    (no division by 1-alpha_i).
    """
    R, n = sdf.shape
    C, wgt, alpha, trans = render_rays(sdf, rgb, s)
    d_rgb = wgt[:, :, None] * dC[:, None, :]
    cbar = np.sum(rgb * dC[:, None, :], axis=2)            # [R,n]  dC . c_j
    d_alpha = np.zeros((R, n))
    for i in range(n - 1):
        acc = trans[:, i] * cbar[:, i]
        for j in range(i + 1, n):
            prod = np.ones(R)
            for k in range(j):
                if k != i:
                    prod = prod * (1.0 - alpha[:, k])
            acc = acc - prod * alpha[:, j] * cbar[:, j]
        d_alpha[:, i] = acc
    phi = logistic_cdf(sdf, s)
    dphi = s * phi * (1.0 - phi)
    live = (phi[:, :-1] - phi[:, 1:]) > 0.0                 # max(.,0) passes gradient only here
    d_sdf = np.zeros((R, n))
    # alpha_i = 1 - Phi_{i+1}/Phi_i
    d_sdf[:, :-1] += np.where(live, d_alpha[:, :-1] * phi[:, 1:] * dphi[:, :-1] / phi[:, :-1] ** 2, 0.0)
    d_sdf[:, 1:] += np.where(live, -d_alpha[:, :-1] * dphi[:, 1:] / phi[:, :-1], 0.0)
    if want_ds:
        # dPhi_s(x)/ds = x Phi (1 - Phi);  alpha_i = 1 - Phi_{i+1}/Phi_i
        ps = sdf * phi * (1.0 - phi)
        da_ds = -(ps[:, 1:] * phi[:, :-1] - phi[:, 1:] * ps[:, :-1]) / phi[:, :-1] ** 2
        return d_sdf, d_rgb, float(np.sum(np.where(live, d_alpha[:, :-1] * da_ds, 0.0)))
    return d_sdf, d_rgb


# --------------------------------------------------------------------------------------
# Rigid transform (Eq. 9)
# --------------------------------------------------------------------------------------

def rotation_from_axis_angle(omega: np.ndarray) -> np.ndarray:
    """R = exp([omega]_x) by Rodrigues' formula."""
    omega = np.asarray(omega, dtype=np.float64)
    th = float(np.linalg.norm(omega))
    K = np.array([[0.0, -omega[2], omega[1]], [omega[2], 0.0, -omega[0]], [-omega[1], omega[0], 0.0]])
    if th < 1e-12:
        return np.eye(3) + K + 0.5 * K @ K
    return np.eye(3) + (math.sin(th) / th) * K + ((1.0 - math.cos(th)) / th ** 2) * (K @ K)


def rigid_forward(x: np.ndarray, R: np.ndarray, T: np.ndarray, scale: float = 1.0, offset: float = 0.0):
    """x_c = R (x + T) (Eq. 9), followed by the affine map scale * x_c + offset that
    takes world coordinates to the unit cube."""
    xc = (np.asarray(x, dtype=np.float64) + np.asarray(T, dtype=np.float64)[None, :]) @ np.asarray(R, dtype=np.float64).T
    return scale * xc + offset


def accumulate_transform(Rc_prev, Tc_prev, R, T):
    """R_i^c = R_{i-1}^c R_i,  T_i^c = T_i + R_i^{-1} T_{i-1}^c (text after Eq. 10)."""
    return Rc_prev @ R, T + np.linalg.inv(R) @ Tc_prev


# --------------------------------------------------------------------------------------
# One training step: forward, loss (Eq. 4), backward (Eqs. 5-8, Theorem 1)
# --------------------------------------------------------------------------------------

def forward(cfg, params, batch, fp32_product: bool = True, want_hess: bool = False) -> Dict[str, object]:
    """Everything the loss needs, from the definitions.

    batch: pos [N,3] (unit-cube coordinates); for loss_kind 1 (L1 colour term) and 2 (Huber colour
    term, Eq. 4) also dirs [R,3], target [R,3].
    """
    pos = batch["pos"]
    N = pos.shape[0]
    H = params["H"]
    he = hash_encode(cfg, params["tables"], pos, fp32_product, want_hess)
    y, acts, masks = mlp_forward(H, he["enc"])
    S, q = mlp_input_gradient(H, masks, 0)
    q = np.broadcast_to(q, he["enc"].shape)
    normal = np.einsum("nk,nka->na", q, he["jac"])                      # Eq. 2
    nrm = np.sqrt(np.sum(normal * normal, axis=1))
    eik = np.mean((nrm - 1.0) ** 2)
    out = {"he": he, "y": y, "acts": acts, "masks": masks, "S": S, "q": q, "normal": normal,
           "nrm": nrm, "eikonal": eik}
    if cfg.loss_kind == 0:
        out["loss"] = np.mean(y[:, 0] ** 2) + cfg.beta * eik
        return out
    if "ray_offsets" in batch:                       # rays with their own sample counts
        offsets = np.asarray(batch["ray_offsets"], dtype=np.int64)
        R = len(offsets) - 1
        cin = color_input(pos, normal, batch["dirs"], y, np.diff(offsets))
        rgb, cacts, cmasks = color_forward(params["W"], cin)
        C, wgt, alpha = render_rays_ragged(y[:, 0], rgb, offsets, cfg.s)
        trans = None
    else:
        n = cfg.samples_per_ray
        R = N // n
        cin = color_input(pos, normal, batch["dirs"], y, n)
        rgb, cacts, cmasks = color_forward(params["W"], cin)
        C, wgt, alpha, trans = render_rays(y[:, 0].reshape(R, n), rgb.reshape(R, n, 3), cfg.s)
    diff = C - np.asarray(batch["target"], dtype=np.float64)
    out.update({"cin": cin, "rgb": rgb, "cacts": cacts, "cmasks": cmasks, "C": C, "weights": wgt,
                "alpha": alpha, "trans": trans, "diff": diff})
    if cfg.loss_kind == 2:
        out["loss"] = np.sum(huber(diff, cfg.huber_delta)) / R + cfg.beta * eik
    else:
        out["loss"] = np.sum(np.abs(diff)) / R + cfg.beta * eik
    return out


def render_rays_ragged(sdf, rgb, offsets, s: float):
    """Rays with their own sample counts, as an occupancy-grid ray marcher produces them
    (supplement Sec. E.3, "Ray Marching Strategy"): ray r owns samples offsets[r]..offsets[r+1]-1
    of the flat arrays sdf [N], rgb [N,3].  Every ray is composited by `render_rays` on its own
    slice; a ray without samples has colour 0.  -> (C [R,3], weights [N], alpha [N])."""
    R = len(offsets) - 1
    C = np.zeros((R, 3))
    wgt = np.zeros(sdf.shape[0])
    alpha = np.zeros(sdf.shape[0])
    for r in range(R):
        a, b = int(offsets[r]), int(offsets[r + 1])
        if b > a:
            Cr, wr, ar, _ = render_rays(sdf[a:b][None, :], rgb[a:b][None, :, :], s)
            C[r], wgt[a:b], alpha[a:b] = Cr[0], wr[0], ar[0]
    return C, wgt, alpha


def render_rays_ragged_backward(sdf, rgb, offsets, s: float, dC):
    """Backward of `render_rays_ragged`, ray by ray -> (d_sdf [N], d_rgb [N,3], d_s)."""
    d_sdf = np.zeros(sdf.shape[0])
    d_rgb = np.zeros((sdf.shape[0], 3))
    d_s = 0.0
    for r in range(len(offsets) - 1):
        a, b = int(offsets[r]), int(offsets[r + 1])
        if b > a:
            ds, dr, dss = render_rays_backward(sdf[a:b][None, :], rgb[a:b][None, :, :], s, dC[r][None, :], want_ds=True)
            d_sdf[a:b], d_rgb[a:b], d_s = ds[0], dr[0], d_s + dss
    return d_sdf, d_rgb, d_s


def huber(r: np.ndarray, delta: float) -> np.ndarray:
    """Huber loss of a residual: r^2/2 for |r| <= delta, delta (|r| - delta/2) beyond (Eq. 4 names
    it for the colour term; delta is not given in the paper and is a configuration value)."""
    a = np.abs(r)
    return np.where(a <= delta, 0.5 * r * r, delta * (a - 0.5 * delta))


def huber_derivative(r: np.ndarray, delta: float) -> np.ndarray:
    return np.clip(r, -delta, delta)


def loss_value(cfg, params, batch, fp32_product: bool = True) -> float:
    return float(forward(cfg, params, batch, fp32_product)["loss"])


def mlp_backward(Wm: Sequence[np.ndarray], acts, masks, d_out):
    """Ordinary back-propagation through a bias-free ReLU MLP.

    Returns (grads per matrix, gradient wrt the input, deltas [delta_1..delta_K]).
    """
    K = len(Wm)
    grads = [None] * K
    deltas = [None] * K
    delta = d_out
    for l in range(K - 1, -1, -1):
        deltas[l] = delta
        grads[l] = delta.T @ acts[l]
        back = delta @ np.asarray(Wm[l], dtype=np.float64)
        delta = back * masks[l - 1] if l > 0 else back
    return grads, delta, deltas


def train_step(cfg, params, batch, fp32_product: bool = True, want_pos_grad: bool = False) -> Dict[str, object]:
    """Forward values and all gradients of one step.

    Gradients returned: dH (list), dW (list), dtables [L,T,F], and, if asked,
    dpos [N,3] (gradient wrt the encoder's input position, incl. the colour
    network's direct dependence on x).  Intermediate adjoints d_y, d_normal,
    d_enc are returned as well so that each library call can be checked alone.
    """
    fw = forward(cfg, params, batch, fp32_product, want_hess=want_pos_grad)
    pos = batch["pos"]
    N = pos.shape[0]
    H = params["H"]
    K = len(H)
    L, F, T = cfg.n_levels, cfg.n_features, cfg.table_size
    y, normal, nrm, q = fw["y"], fw["normal"], fw["nrm"], fw["q"]
    jac = fw["he"]["jac"]

    d_y = np.zeros_like(y)
    d_normal = (2.0 * cfg.beta / N) * ((nrm - 1.0) / np.maximum(nrm, 1e-30))[:, None] * normal
    d_pos_color = np.zeros((N, 3))
    dW: List[np.ndarray] = []
    if cfg.loss_kind == 0:
        d_y[:, 0] += 2.0 * y[:, 0] / N
    else:
        ragged = "ray_offsets" in batch
        n = cfg.samples_per_ray
        R = len(batch["ray_offsets"]) - 1 if ragged else N // n
        if cfg.loss_kind == 2:
            dC = huber_derivative(fw["diff"], cfg.huber_delta) / R
        else:
            dC = np.sign(fw["diff"]) / R
        if ragged:
            d_sdf, d_rgb, d_s = render_rays_ragged_backward(y[:, 0], fw["rgb"], np.asarray(batch["ray_offsets"], dtype=np.int64),
                                                            cfg.s, dC)
        else:
            d_sdf, d_rgb, d_s = render_rays_backward(y[:, 0].reshape(R, n), fw["rgb"].reshape(R, n, 3), cfg.s, dC, want_ds=True)
        fw["d_s"] = d_s
        rgb = fw["rgb"]
        d_u = d_rgb.reshape(N, 3) * rgb * (1.0 - rgb)
        dW, d_cin, _ = mlp_backward(params["W"], fw["cacts"], fw["cmasks"], d_u)
        d_pos_color = d_cin[:, 0:3]
        d_normal = d_normal + d_cin[:, 3:6]
        d_y = d_y + d_cin[:, 22:38]
        d_y[:, 0] += d_sdf.reshape(N)
        fw["d_rgb"] = d_rgb.reshape(N, 3)
        fw["d_sdf_render"] = d_sdf.reshape(N)
        fw["dC"] = dC

    # first order through the SDF network
    dH, d_enc, _ = mlp_backward(H, fw["acts"], fw["masks"], d_y)

    # second order, Theorem 1: d n_a / d H_l = S_l^T (P_l^a)^T with P started from column a of
    # de/dx; summed over a with weights dL/dn_a this is one forward-mode sweep t.
    t = np.einsum("nka,na->nk", jac, d_normal)                    # t_0 = (de/dx) dL/dn
    for l in range(K):
        S_l = fw["S"][l] if l < K - 1 else None
        if S_l is None:                                           # S_K = unit row selecting d
            dH[l][0, :] += np.sum(t, axis=0)
        else:
            dH[l] += S_l.T @ t
            t = fw["masks"][l] * (t @ np.asarray(H[l], dtype=np.float64).T)

    dtables = table_gradient(cfg, pos, q, d_enc, d_normal, fp32_product)
    # Levels below frozen_levels are inputs, not parameters (they carry the position x into the
    # network, Eq. 1 feeds e = (x, h(x))): no gradient.
    dtables[:getattr(cfg, "frozen_levels", 0)] = 0.0

    out = dict(fw)
    out.update({"d_y": d_y, "d_normal": d_normal, "d_enc": d_enc, "dH": dH, "dW": dW, "dtables": dtables})
    if want_pos_grad:
        hess = fw["he"]["hess"]
        d_pos = np.einsum("nka,nk->na", jac, d_enc)
        d_pos += np.einsum("na,nk,nkab->nb", d_normal, q, hess)
        out["dpos"] = d_pos + d_pos_color
    return out


def table_gradient(cfg, pos, q, d_enc, d_normal, fp32_product: bool = True) -> np.ndarray:
    """dL/dOmega [L,T,F]: the first-order term w_c * dL/de plus Eq. 7's term
    (dd/de) * d(de/dx)/dOmega contracted with dL/dn, i.e. for corner c of the cell of point i
    at level l:  dOmega[l, slot_c, f] += w_c * d_enc[i, lF+f] + q[i, lF+f] * res_l * sum_a d_normal[i,a] * d_a w_c.
    Active levels only."""
    L, F, T = cfg.n_levels, cfg.n_features, cfg.table_size
    q = np.asarray(q, dtype=np.float64)
    d_enc = np.asarray(d_enc, dtype=np.float64)
    d_normal = np.asarray(d_normal, dtype=np.float64)
    dtables = np.zeros((L, T, F))
    for l in range(min(L, cfg.active_levels)):
        res = cfg.res[l]
        p = grid_coords(pos, res, fp32_product)
        c0, w = cell_and_fraction(p, res)
        wc, dwc, _ = corner_weights(w)
        for c, bits in enumerate(CORNERS):
            idx = vertex_index(c0 + np.array(bits, dtype=np.int64), res, cfg.dense[l], T)
            dn_dw = res * np.sum(dwc[c] * d_normal, axis=1)        # res * sum_a dL/dn_a d_a w_c
            for f in range(F):
                k = l * F + f
                coef = wc[c] * d_enc[:, k] + q[:, k] * dn_dw
                dtables[l, :, f] += np.bincount(idx, weights=coef, minlength=T)
    return dtables


def rigid_backward(x, R, T, d_xc, scale: float = 1.0):
    """Reductions for the transform gradient: M = sum dL/dx_c (x+T)^T, b = sum dL/dx_c,
    where d_xc is the gradient wrt the mapped coordinate scale*x_c + offset.
    Returns (M [3,3] = dL/dR, dL/dT = R^T b, b)."""
    g = scale * np.asarray(d_xc, dtype=np.float64)
    xt = np.asarray(x, dtype=np.float64) + np.asarray(T, dtype=np.float64)[None, :]
    M = g.T @ xt
    b = np.sum(g, axis=0)
    return M, np.asarray(R, dtype=np.float64).T @ b, b


def axis_angle_gradient(omega, M, h: float = 1e-6):
    """dL/domega_k = sum_ij dR_ij/domega_k M_ij, with dR/domega by central differences
    of Rodrigues' formula in float64."""
    g = np.zeros(3)
    for k in range(3):
        e = np.zeros(3)
        e[k] = h
        dR = (rotation_from_axis_angle(omega + e) - rotation_from_axis_angle(omega - e)) / (2 * h)
        g[k] = np.sum(dR * M)
    return g


# --------------------------------------------------------------------------------------
# A frame's transform as six parameters (Sec. 5, Eqs. 9-10)
# --------------------------------------------------------------------------------------

def frame_to_canonical(x, omega, T, R_prev, T_prev):
    """Eq. 9 applied down the chain of frames: a point x of the current frame goes to the previous
    frame by R(omega) (x + T), and from there to the canonical (first) frame by the transform
    accumulated so far, x_c = R_prev (x_prev + T_prev)."""
    R = rotation_from_axis_angle(omega)
    x_prev = (np.asarray(x, dtype=np.float64) + np.asarray(T, dtype=np.float64)[None, :]) @ R.T
    return (x_prev + np.asarray(T_prev, dtype=np.float64)[None, :]) @ np.asarray(R_prev, dtype=np.float64).T


def pose_gradient(x, omega, T, R_prev, T_prev, d_xc, h: float = 1e-6):
    """Gradient of a loss with respect to the frame's (omega, T), given dL/dx_c per point, from
    the definition above: dL/dT = sum (R_prev R)^T g, dL/domega_k = sum g . R_prev (dR/domega_k) (x + T)
    with dR/domega_k by central differences of Rodrigues' formula."""
    g = np.asarray(d_xc, dtype=np.float64)
    R = rotation_from_axis_angle(omega)
    Rp = np.asarray(R_prev, dtype=np.float64)
    u = np.asarray(x, dtype=np.float64) + np.asarray(T, dtype=np.float64)[None, :]
    d_T = (Rp @ R).T @ np.sum(g, axis=0)
    d_omega = np.zeros(3)
    for k in range(3):
        e = np.zeros(3)
        e[k] = h
        dR = (rotation_from_axis_angle(np.asarray(omega, dtype=np.float64) + e)
              - rotation_from_axis_angle(np.asarray(omega, dtype=np.float64) - e)) / (2 * h)
        d_omega[k] = np.sum(g * (u @ dR.T @ Rp.T))
    return d_omega, d_T


def dynamic_frame_iteration(cfg, params, opt, pose, frame_batch, joint: bool, lr: float, pose_lr: float,
                            b1: float = 0.9, b2: float = 0.99, eps: float = 1e-15, pos_override=None):
    """One training iteration of a frame of a dynamic scene (Sec. 5; supplement Sec. E.3: the first
    iterations of a frame optimise the transform alone, `joint` False).

    params: tables (as stored), master (float64 copy of fp16 tables, or None), H, W.
    opt: Adam state {"t", "m_tables", "v_tables", "m_H", "v_H", "m_W", "v_W"}.
    pose: {"omega", "T", "m", "v", "t", "R_prev", "T_prev"}.
    frame_batch: world-space pos [N,3], dirs, target.
    `pos_override`: the encoder's input positions to use instead of this function's own float64
    transform rounded to binary32 (the cell of a point is decided in binary32, so a parity test
    hands both sides the same binary32 positions).
    Returns (new params, new opt, new pose, the step's outputs); inputs are not modified.
    """
    world = np.asarray(frame_batch["pos"], dtype=np.float64)
    Rc, Tc = accumulate_transform(pose["R_prev"], pose["T_prev"], rotation_from_axis_angle(pose["omega"]), pose["T"])
    pos = rigid_forward(world, Rc, Tc, 0.5, 0.5).astype(np.float32) if pos_override is None else pos_override
    out = train_step(cfg, params, {"pos": pos, "dirs": frame_batch["dirs"], "target": frame_batch["target"]}, want_pos_grad=True)
    d_omega, d_T = pose_gradient(world, pose["omega"], pose["T"], pose["R_prev"], pose["T_prev"], 0.5 * out["dpos"])
    out["d_pose"] = np.concatenate([d_omega, d_T])
    t_pose = pose["t"] + 1
    p6, m6, v6 = adam_step(np.concatenate([pose["omega"], pose["T"]]), out["d_pose"], pose["m"], pose["v"], t_pose, pose_lr, b1, b2, eps)
    new_pose = dict(pose, omega=p6[:3], T=p6[3:], m=m6, v=v6, t=t_pose)
    if not joint:
        return params, opt, new_pose, out
    t = opt["t"] + 1
    new_params, new_opt = dict(params), dict(opt, t=t)
    half = np.asarray(params["tables"]).dtype == np.float16
    full = params["master"] if half else np.asarray(params["tables"], dtype=np.float64)
    full, new_opt["m_tables"], new_opt["v_tables"] = adam_step(full, out["dtables"], opt["m_tables"], opt["v_tables"], t, lr, b1, b2, eps)
    if half:
        new_params["master"] = full.astype(np.float32).astype(np.float64)          # the master copy is binary32
        new_params["tables"] = full.astype(np.float32).astype(np.float16)
    else:
        new_params["tables"] = full.astype(np.float32)
    for name, grads in (("H", out["dH"]), ("W", out["dW"])):
        mats, ms, vs = [], [], []
        for k, g in enumerate(grads):
            p1, m1, v1 = adam_step(params[name][k], g, opt["m_" + name][k], opt["v_" + name][k], t, lr, b1, b2, eps)
            mats.append(p1.astype(np.float32))
            ms.append(m1)
            vs.append(v1)
        new_params[name], new_opt["m_" + name], new_opt["v_" + name] = mats, ms, vs
    return new_params, new_opt, new_pose, out


# --------------------------------------------------------------------------------------
# Optimiser (the paper names none; the benchmark contract asks for Adam)
# --------------------------------------------------------------------------------------

def adam_step(param, grad, m, v, t: int, lr: float, b1: float, b2: float, eps: float, lazy: bool = False):
    """Textbook Adam, bias-corrected.  Returns (param, m, v) in float64.

    The paper names no optimiser.  `lazy` is the sparse form used for hash tables: an entry
    whose gradient is exactly zero keeps its value and both moments (no decay); reading: the
    bias correction uses the global step number t for every entry.
    """
    g = np.asarray(grad, dtype=np.float64)
    p0, m0, v0 = (np.asarray(a, dtype=np.float64) for a in (param, m, v))
    m1 = b1 * m0 + (1.0 - b1) * g
    v1 = b2 * v0 + (1.0 - b2) * g * g
    mhat = m1 / (1.0 - b1 ** t)
    vhat = v1 / (1.0 - b2 ** t)
    p1 = p0 - lr * mhat / (np.sqrt(vhat) + eps)
    if lazy:
        keep = g == 0.0
        return np.where(keep, p0, p1), np.where(keep, m0, m1), np.where(keep, v0, v1)
    return p1, m1, v1
