"""Parity of the HIP library (through its C ABI) with the float64 oracle, element by element
on the same seeded inputs.  All tests here need an MI355X.

Tolerances (stated by the benchmark contract): table indices bit-exact; forward values
relative L2 error <= 1e-5 per tensor; gradients <= 1e-4 per tensor (5e-3 / 2e-3 are allowed
with fp16 tables, but the oracle sees the same fp16-rounded tables, so the fp32 bars are
applied throughout).
"""
import math

import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import neus2_oracle as o
from paper_2212_05231_amd import binding as nb
from paper_2212_05231_amd import workloads as wl

pytestmark = pytest.mark.gpu

FWD_TOL = 1e-5
GRAD_TOL = 1e-4


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    nb.lib()


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a))


def from_level_major(t, n):
    """[L][n][F] -> [n, L*F]"""
    a = t.detach().cpu().numpy().astype(np.float64)
    return np.transpose(a, (1, 0, 2)).reshape(n, -1)


def jac_from_level_major(t, n):
    """library layout [L][3 pairs][n][2] -> [n, L*F, 3]"""
    a = t.detach().cpu().numpy().astype(np.float64).reshape(-1, 3, n, 2)
    return np.transpose(a, (2, 0, 1, 3)).reshape(n, -1, 3)      # [n][L][pair][2] = [n][L][F*3] -> [n, L*F, 3]


def jac_to_level_major(J, n, L):
    """[n, L*F, 3] -> torch, library layout [L][3 pairs][n][2]"""
    a = np.asarray(J, dtype=np.float64).reshape(n, L, 3, 2)
    return cuda(np.ascontiguousarray(np.transpose(a, (1, 2, 0, 3))))


def decode_masks(words, n, layers):
    """library mask buffer [2][n][2] -> list of bool [n, 64] per hidden layer (bit 16 b + r of word
    (layer, i, h) is neuron 32 b + 8 (r / 4) + 4 h + r % 4)"""
    w = words.detach().cpu().numpy().astype(np.uint32).reshape(2, n, 2)
    out = []
    for layer in range(layers):
        m = np.zeros((n, 64), dtype=bool)
        for h in range(2):
            for b in range(2):
                for r in range(16):
                    m[:, 32 * b + 8 * (r // 4) + 4 * h + r % 4] = (w[layer, :, h] >> np.uint32(16 * b + r)) & np.uint32(1)
        out.append(m)
    return out


def to_level_major(a, L):
    """[n, L*F] -> torch [L][n][F]"""
    n = a.shape[0]
    return torch.as_tensor(np.ascontiguousarray(np.transpose(a.reshape(n, L, 2), (1, 0, 2))), dtype=torch.float32).cuda()


def cuda(a, dtype=torch.float32):
    return torch.as_tensor(np.ascontiguousarray(a)).to(dtype=dtype).cuda().contiguous()


def run_step(k, n_rays, want_pos=False, scale_tables=None, active=None, spr=None, keep_masks=True):
    w = wl.make_workload(k, n_rays=n_rays)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    if active is not None:
        cfg.active_levels = active
    if scale_tables is not None:
        params["tables"] = (params["tables"].astype(np.float64) * scale_tables).astype(params["tables"].dtype)
    if k == 5:
        R = o.rotation_from_axis_angle(batch["omega"])
        batch["pos"] = np.clip(o.rigid_forward(batch["pos"], R, batch["shift"], 0.5, 0.5), 0, 1 - 2.0 ** -24).astype(np.float32)
    n = batch["pos"].shape[0]
    step = nb.Step(cfg, params, n, want_pos_grad=want_pos, keep_masks=keep_masks)
    step.set_batch(batch)
    step.zero_grads()
    step.train_step()
    torch.cuda.synchronize()
    ref = o.train_step(cfg, params, batch, want_pos_grad=want_pos)
    return cfg, step, ref, n


def assert_elementwise(name, got, ref, tol, outliers=0.0):
    """|got - ref| <= tol * (|ref| + largest |ref| of the tensor), element by element.  An element
    is a sum of up to 64 products, so its error scales with the magnitude of the terms, not of the
    result: the tensor's largest magnitude stands for it.  `outliers`: the fraction of elements
    allowed outside (a ReLU mask that flips between binary32-class and float64 arithmetic at a
    pre-activation within rounding of zero moves that one point's q and normal)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    bad = np.abs(got - ref) > tol * (np.abs(ref) + np.max(np.abs(ref)))
    assert np.mean(bad) <= outliers, (name, int(bad.sum()), bad.size, float(np.max(np.abs(got - ref))), float(np.max(np.abs(ref))))


def check_step(cfg, step, ref, n, want_pos=False, outliers=0.0):
    errs = {}
    assert_elementwise("enc", from_level_major(step.enc, n), ref["he"]["enc"], FWD_TOL)
    assert_elementwise("jac", jac_from_level_major(step.jac, n), ref["he"]["jac"], FWD_TOL)
    assert_elementwise("y", step.y.cpu().numpy(), ref["y"], FWD_TOL, outliers)
    assert_elementwise("q", from_level_major(step.q, n), ref["q"], FWD_TOL, outliers)
    assert_elementwise("normal", step.normal.cpu().numpy(), ref["normal"], FWD_TOL, outliers)
    if cfg.loss_kind != 0:
        assert_elementwise("rgb", step.rgb.cpu().numpy(), ref["rgb"], FWD_TOL, outliers)
        assert_elementwise("C", step.C.cpu().numpy(), ref["C"], FWD_TOL, outliers)
    errs["enc"] = rel(from_level_major(step.enc, n), ref["he"]["enc"])
    errs["jac"] = rel(jac_from_level_major(step.jac, n), ref["he"]["jac"])
    errs["y"] = rel(step.y.cpu().numpy(), ref["y"])
    errs["q"] = rel(from_level_major(step.q, n), ref["q"])
    errs["normal"] = rel(step.normal.cpu().numpy(), ref["normal"])
    loss = step.loss.cpu().numpy()
    errs["loss"] = abs(float(loss[0] + loss[1]) - ref["loss"]) / abs(ref["loss"])
    if cfg.loss_kind != 0:
        errs["rgb"] = rel(step.rgb.cpu().numpy(), ref["rgb"])
        errs["C"] = rel(step.C.cpu().numpy(), ref["C"])
        errs["weights"] = rel(step.weights.cpu().numpy().reshape(ref["weights"].shape), ref["weights"])
    for name, e in errs.items():
        assert e <= FWD_TOL, (name, e, errs)
    g = {}
    g["d_y"] = rel(step.d_y.cpu().numpy(), ref["d_y"])
    g["d_normal"] = rel(step.d_normal.cpu().numpy(), ref["d_normal"])
    act = cfg.active_levels * 2
    g["d_enc"] = rel(from_level_major(step.d_enc, n)[:, :act], ref["d_enc"][:, :act])
    for l, (a, b) in enumerate(zip(step.dH, ref["dH"])):
        g[f"dH{l}"] = rel(a.cpu().numpy(), b)
    for l, (a, b) in enumerate(zip(step.dW, ref["dW"])):
        g[f"dW{l}"] = rel(a.cpu().numpy(), b)
    g["d_tables"] = rel(step.d_tables.cpu().numpy(), ref["dtables"])
    if want_pos:
        g["d_pos"] = rel(step.d_pos.cpu().numpy(), ref["dpos"])
    for name, e in g.items():
        assert e <= GRAD_TOL, (name, e, g)
    errs.update(g)
    return errs


# ------------------------------------------------------------------ encoding

@pytest.mark.parametrize("k,n_rays", [(1, 4096 + 77), (2, 50), (4, 9)])
def test_hash_encode_indices_bit_exact_and_values(k, n_rays):
    w = wl.make_workload(k, n_rays=n_rays)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    pos = batch["pos"].copy()
    pos[:4] = np.array([[0, 0, 0], [1, 1, 1], [1 - 2.0 ** -24, 0.5, 0.25], [np.nan, -1.0, 2.0]], dtype=np.float32)
    n = pos.shape[0]
    c = nb.make_config(cfg)
    L = cfg.n_levels
    tables = cuda(params["tables"], torch.float16 if cfg.table_dtype == "f16" else torch.float32)
    enc = torch.empty(L, n, 2, device="cuda")
    jac = torch.empty(L, 3, n, 2, device="cuda")
    idx = torch.zeros(n, L, 8, dtype=torch.int32, device="cuda")
    nb.hash_encode(c, cuda(pos), tables, enc, jac, idx)
    torch.cuda.synchronize()
    ref = o.hash_encode(cfg, params["tables"], pos)
    got_idx = idx.cpu().numpy().astype(np.int64) & 0xFFFFFFFF
    assert np.array_equal(got_idx, ref["idx"])
    assert rel(from_level_major(enc, n), ref["enc"]) <= FWD_TOL
    assert rel(jac_from_level_major(jac, n), ref["jac"]) <= FWD_TOL
    # per-element check as well (fp32 sums of 8 products)
    np.testing.assert_allclose(from_level_major(enc, n), ref["enc"], rtol=FWD_TOL, atol=1e-9)


def test_hash_encode_large_tables_and_batch_every_value():
    """Workload 4's tables (2^21 entries a level: 8 MiB in fp16, 16 MiB in fp32, several times an L2) on a
    quarter of a million points: every value and every Jacobian entry against the oracle, with edge
    positions and a ragged last block."""
    w = wl.make_workload(4, n_rays=4096 + 3)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    pos = batch["pos"][:262144 + 77].copy()
    pos[:4] = np.array([[0, 0, 0], [1, 1, 1], [1 - 2.0 ** -24, 0.5, 0.25], [np.nan, -1.0, 2.0]], dtype=np.float32)
    n = pos.shape[0]
    c = nb.make_config(cfg)
    L = cfg.n_levels
    tables = cuda(params["tables"], torch.float16)
    enc = torch.full((L, n, 2), 7.0, device="cuda")
    jac = torch.full((L, 3, n, 2), 7.0, device="cuda")
    nb.hash_encode(c, cuda(pos), tables, enc, jac)
    torch.cuda.synchronize()
    ref = o.hash_encode(cfg, params["tables"], pos)
    assert rel(from_level_major(enc, n), ref["enc"]) <= FWD_TOL
    assert rel(jac_from_level_major(jac, n), ref["jac"]) <= FWD_TOL
    np.testing.assert_allclose(from_level_major(enc, n), ref["enc"], rtol=FWD_TOL, atol=1e-9)
    got_j, want_j = jac_from_level_major(jac, n), ref["jac"]
    for l in range(L):
        sl = slice(2 * l, 2 * l + 2)
        np.testing.assert_allclose(got_j[:, sl], want_j[:, sl], rtol=FWD_TOL, atol=1e-9 * cfg.res[l])
    # the same through fp32 tables
    cfg.table_dtype = "f32"
    c = nb.make_config(cfg)
    tab32 = params["tables"].astype(np.float32) * np.float32(1.37)
    nb.hash_encode(c, cuda(pos), cuda(tab32), enc, jac)
    torch.cuda.synchronize()
    ref = o.hash_encode(cfg, tab32, pos)
    assert rel(from_level_major(enc, n), ref["enc"]) <= FWD_TOL
    assert rel(jac_from_level_major(jac, n), ref["jac"]) <= FWD_TOL


def test_fp16_subnormal_table_entries_are_not_flushed():
    cfg = wl.make_config(2)
    c = nb.make_config(cfg)
    tab = np.full((cfg.n_levels, cfg.table_size, 2), 3e-6, dtype=np.float16)      # subnormal in fp16
    pos = wl.make_points(257, 5)
    enc = torch.empty(cfg.n_levels, 257, 2, device="cuda")
    jac = torch.empty(cfg.n_levels, 3, 257, 2, device="cuda")
    nb.hash_encode(c, cuda(pos), cuda(tab, torch.float16), enc, jac)
    np.testing.assert_allclose(enc.cpu().numpy(), float(np.float16(3e-6)), rtol=1e-6)


def test_progressive_mask_zeroes_inactive_levels():
    cfg, step, ref, n = run_step(3, 8)
    assert torch.all(step.enc[cfg.active_levels:] == 0) and torch.all(step.jac[cfg.active_levels:] == 0)
    assert torch.all(step.d_tables[cfg.active_levels:] == 0)
    check_step(cfg, step, ref, n)


# ------------------------------------------------------------------ single calls

def test_sdf_fwd_grad_alone_with_large_values():
    """Random encodings of order one (the workloads' are ~1e-4) so that masks are mixed."""
    rng = np.random.default_rng(0)
    for k, n in ((1, 1000 + 19), (2, 2048 + 5)):
        cfg = wl.make_config(k)
        c = nb.make_config(cfg)
        L, D = cfg.n_levels, cfg.enc_dim
        H = [rng.normal(size=(cfg.sdf_dims[i + 1], cfg.sdf_dims[i])).astype(np.float32) * 0.3 for i in range(len(cfg.sdf_dims) - 1)]
        e = rng.normal(size=(n, D)).astype(np.float32)
        J = rng.normal(size=(n, D, 3)).astype(np.float32)
        y = torch.empty(n, 16, device="cuda")
        q = torch.empty(L, n, 2, device="cuda")
        nrm = torch.empty(n, 3, device="cuda")
        jac_lm = jac_to_level_major(J, n, L)
        nb.sdf_fwd_grad(c, to_level_major(e, L), jac_lm, [cuda(h) for h in H], n, y, q, nrm)
        torch.cuda.synchronize()
        yr, acts, masks = o.mlp_forward(H, e)
        S, qr = o.mlp_input_gradient(H, masks, 0)
        assert rel(y.cpu().numpy(), yr) <= FWD_TOL
        assert rel(from_level_major(q, n), qr) <= FWD_TOL
        assert rel(nrm.cpu().numpy(), np.einsum("nk,nka->na", qr, J.astype(np.float64))) <= FWD_TOL


@pytest.mark.parametrize("enc_scale,w_scale", [(1e-12, 1.0), (1e-4, 30.0), (1.0, 1e-6), (3e4, 0.3), (1e15, 1e-3)])
def test_network_products_over_a_wide_range_of_magnitudes(enc_scale, w_scale):
    """The matrix products take fp32 factors as sums of bf16 terms; bf16 has the exponent range of
    fp32, so accuracy must not depend on the magnitude of encodings, weights or adjoints (an fp16
    split would underflow here).  Forward of the SDF network alone, then its backward (first and
    second order) alone, each per-point feature with a scale of its own within a factor 1e3."""
    rng = np.random.default_rng(11)
    cfg = wl.make_config(2)
    c = nb.make_config(cfg)
    n, L, D = 1500 + 7, cfg.n_levels, cfg.enc_dim
    H = [(rng.normal(size=(cfg.sdf_dims[i + 1], cfg.sdf_dims[i])) * w_scale / 8).astype(np.float32) for i in range(3)]
    feat = 10.0 ** rng.uniform(-1.5, 1.5, size=D)
    e = (rng.normal(size=(n, D)) * feat * enc_scale).astype(np.float32)
    J = (rng.normal(size=(n, D, 3)) * enc_scale).astype(np.float32)
    Hg = [cuda(h) for h in H]
    enc_lm, jac_lm = to_level_major(e, L), jac_to_level_major(J, n, L)
    y, q, nrm = torch.empty(n, 16, device="cuda"), torch.empty(L, n, 2, device="cuda"), torch.empty(n, 3, device="cuda")
    nb.sdf_fwd_grad(c, enc_lm, jac_lm, Hg, n, y, q, nrm)
    yr, acts, masks = o.mlp_forward(H, e)
    S, qr = o.mlp_input_gradient(H, masks, 0)
    assert rel(y.cpu().numpy(), yr) <= FWD_TOL
    assert rel(from_level_major(q, n), qr) <= FWD_TOL
    # backward: adjoints of y and of the normal, also of widely different sizes
    d_y = (rng.normal(size=(n, 16)) * 10.0 ** rng.uniform(-3, 3, size=16) * 1e-6).astype(np.float32)
    d_n = (rng.normal(size=(n, 3)) * 1e-3).astype(np.float32)
    dH = [torch.zeros_like(h) for h in Hg]
    d_enc = torch.zeros(L, n, 2, device="cuda")
    nb.sdf_mlp_bwd(c, enc_lm, jac_lm, Hg, cuda(d_y), cuda(d_n), n, dH, d_enc)
    torch.cuda.synchronize()
    H64 = [h.astype(np.float64) for h in H]
    gH, d_in, _ = o.mlp_backward(H64, acts, masks, d_y.astype(np.float64))
    # second order (Theorem 1): dL/dH_l += S_l^T t_{l-1}^T with t_0 = J nbar
    t = np.einsum("nka,na->nk", J.astype(np.float64), d_n.astype(np.float64))
    Ssweep = [None, None, None]
    s_vec = np.tile(H64[2][0], (n, 1)) * masks[1]
    Ssweep[1] = s_vec
    Ssweep[0] = (s_vec @ H64[1]) * masks[0]
    gH[0] += Ssweep[0].T @ t
    t1 = (t @ H64[0].T) * masks[0]
    gH[1] += Ssweep[1].T @ t1
    t2 = (t1 @ H64[1].T) * masks[1]
    gH[2][0] += t2.sum(axis=0)
    assert rel(from_level_major(d_enc, n), d_in) <= GRAD_TOL
    for a, b in zip(dH, gH):
        assert rel(a.cpu().numpy(), b) <= GRAD_TOL


@pytest.mark.parametrize("D,K", [(16, 2), (16, 3), (32, 2), (32, 3)])
def test_sdf_network_every_kernel_shape(D, K):
    """The four shapes the SDF kernels are built for (input width 16 or 32, one or two hidden
    layers), forward and first/second-order backward alone, with a ragged last tile."""
    rng = np.random.default_rng(100 * D + K)
    cfg = wl.make_config(2)
    cfg.n_levels = cfg.active_levels = D // 2
    cfg.res, cfg.dense = cfg.res[:D // 2], cfg.dense[:D // 2]
    cfg.sdf_dims = [D] + [64] * (K - 1) + [16]
    c = nb.make_config(cfg)
    n, L = 32 * 37 + 11, cfg.n_levels
    H = [(rng.normal(size=(cfg.sdf_dims[i + 1], cfg.sdf_dims[i])) * 0.3).astype(np.float32) for i in range(K)]
    e = rng.normal(size=(n, D)).astype(np.float32)
    J = rng.normal(size=(n, D, 3)).astype(np.float32)
    Hg = [cuda(h) for h in H]
    enc_lm, jac_lm = to_level_major(e, L), jac_to_level_major(J, n, L)
    y, q, nrm = torch.empty(n, 16, device="cuda"), torch.empty(L, n, 2, device="cuda"), torch.empty(n, 3, device="cuda")
    kept = torch.zeros(2, n, 2, dtype=torch.int32, device="cuda")
    nb.sdf_fwd_grad(c, enc_lm, jac_lm, Hg, n, y, q, nrm, masks=kept)
    yr, acts, masks = o.mlp_forward(H, e)
    S, qr = o.mlp_input_gradient(H, masks, 0)
    assert rel(y.cpu().numpy(), yr) <= FWD_TOL
    assert rel(from_level_major(q, n), qr) <= FWD_TOL
    assert rel(nrm.cpu().numpy(), np.einsum("nk,nka->na", qr, J.astype(np.float64))) <= FWD_TOL
    # the masks handed to the backward kernel are the oracle's, but for pre-activations that round to
    # the other side of zero
    for got, want in zip(decode_masks(kept, n, K - 1), masks):
        assert np.mean(got != (want > 0)) < 1e-4
    d_y = rng.normal(size=(n, 16)).astype(np.float32)
    d_n = rng.normal(size=(n, 3)).astype(np.float32)
    H64 = [h.astype(np.float64) for h in H]
    gH, d_in, _ = o.mlp_backward(H64, acts, masks, d_y.astype(np.float64))
    # second order (Theorem 1 for the SDF output): dL/dH_l += S_l^T t_{l-1}^T, t_0 = J nbar
    t = np.einsum("nka,na->nk", J.astype(np.float64), d_n.astype(np.float64))
    s_vec = np.tile(H64[K - 1][0], (n, 1)) * masks[K - 2]
    sweep = [None] * (K - 1)
    sweep[K - 2] = s_vec
    for l in range(K - 3, -1, -1):
        sweep[l] = (sweep[l + 1] @ H64[l + 1]) * masks[l]
    for l in range(K - 1):
        gH[l] += sweep[l].T @ t
        t = (t @ H64[l].T) * masks[l]
    gH[K - 1][0] += t.sum(axis=0)
    # the backward kernel in both forms: masks from the forward kernel, or worked out again
    for given in (kept, None):
        dH = [torch.zeros_like(h) for h in Hg]
        d_enc = torch.zeros(L, n, 2, device="cuda")
        nb.sdf_mlp_bwd(c, enc_lm, jac_lm, Hg, cuda(d_y), cuda(d_n), n, dH, d_enc, masks=given)
        torch.cuda.synchronize()
        assert rel(from_level_major(d_enc, n), d_in) <= GRAD_TOL
        for a, b in zip(dH, gH):
            assert rel(a.cpu().numpy(), b) <= GRAD_TOL


def test_render_forward_backward_alone():
    rng = np.random.default_rng(1)
    for spr, rays in ((64, 37), (17, 9), (1, 5), (2, 3)):
        cfg = wl.make_config(2)
        cfg.samples_per_ray = spr
        c = nb.make_config(cfg)
        n = rays * spr
        sdf = (rng.normal(size=(rays, spr)) * 0.05).astype(np.float32)
        if spr == 64:
            sdf[0] = np.linspace(0.3, -0.3, spr)             # a ray that crosses the surface
            sdf[1] = np.sort(sdf[1])                         # increasing: renders nothing
        rgb = rng.uniform(size=(rays, spr, 3)).astype(np.float32)
        dC = rng.normal(size=(rays, 3)).astype(np.float32)
        y = np.zeros((n, 16), dtype=np.float32)
        y[:, 0] = sdf.reshape(-1)
        Cg = torch.empty(rays, 3, device="cuda")
        wg = torch.empty(n, device="cuda")
        yg = cuda(y)
        nb.render_rays(c, yg, 16, cuda(rgb.reshape(n, 3)), rays, Cg, wg)
        ds = torch.empty(n, device="cuda")
        dr = torch.empty(n, 3, device="cuda")
        nb.render_rays_bwd(c, yg, 16, cuda(rgb.reshape(n, 3)), cuda(dC), rays, ds, dr)
        torch.cuda.synchronize()
        Cr, wr, alpha, _ = o.render_rays(sdf.astype(np.float64), rgb.astype(np.float64), cfg.s)
        d_sdf, d_rgb = o.render_rays_backward(sdf.astype(np.float64), rgb.astype(np.float64), cfg.s, dC.astype(np.float64))
        assert rel(Cg.cpu().numpy(), Cr) <= FWD_TOL
        assert rel(wg.cpu().numpy().reshape(rays, spr), wr) <= FWD_TOL
        assert rel(dr.cpu().numpy().reshape(rays, spr, 3), d_rgb) <= GRAD_TOL
        if spr > 1:
            assert rel(ds.cpu().numpy().reshape(rays, spr), d_sdf) <= GRAD_TOL
        else:
            assert torch.all(ds == 0)
        if spr == 64:
            assert np.all(wg.cpu().numpy().reshape(rays, spr)[1] == 0)
        # the slope read from device memory (a trained parameter) and its gradient, added into d_s
        s_dev = cuda(np.array([33.0], dtype=np.float32))
        d_s = cuda(np.array([0.5], dtype=np.float32))
        nb.render_rays(c, yg, 16, cuda(rgb.reshape(n, 3)), rays, Cg, wg, s_dev=s_dev)
        nb.render_rays_bwd(c, yg, 16, cuda(rgb.reshape(n, 3)), cuda(dC), rays, ds, dr, s_dev=s_dev, d_s=d_s)
        torch.cuda.synchronize()
        Cr, wr, _, _ = o.render_rays(sdf.astype(np.float64), rgb.astype(np.float64), 33.0)
        d_sdf, d_rgb, ref_ds = o.render_rays_backward(sdf.astype(np.float64), rgb.astype(np.float64), 33.0,
                                                      dC.astype(np.float64), want_ds=True)
        assert rel(Cg.cpu().numpy(), Cr) <= FWD_TOL
        assert rel(ds.cpu().numpy().reshape(rays, spr), d_sdf) <= GRAD_TOL
        # dL/ds is a sum of terms of both signs: measure the error against their magnitude
        scale = float(np.sum(np.abs(d_sdf * sdf))) / 33.0
        assert abs(float(d_s.cpu()[0]) - 0.5 - ref_ds) <= GRAD_TOL * max(scale, 1e-30) + 1e-7


def test_compositing_backward_with_saturated_alpha():
    """A sample pair whose alpha rounds to exactly 1 in binary32 (s (d_i - d_{i+1}) and -s d_{i+1}
    beyond about 17): the transmittance behind it is 0 and the backward pass divides a zero sum
    by 1 - alpha.  The adjoints must stay finite and equal the oracle's, which writes the product
    over the other samples out instead of dividing; stand-alone, fused and ragged kernels."""
    rng = np.random.default_rng(60)
    for s_val, jump in ((20.0, (0.5, -0.9)), (800.0, (0.01, -0.025))):
        cfg = wl.make_config(2)
        cfg.s = s_val
        c = nb.make_config(cfg)
        rays, spr = 6, cfg.samples_per_ray
        n = rays * spr
        sdf = (rng.normal(size=(rays, spr)) * (0.4 / s_val)).astype(np.float32)
        sdf[0, 20], sdf[0, 21] = jump                       # mid-ray
        sdf[1, 0], sdf[1, 1] = jump                         # first pair
        sdf[2, spr - 2], sdf[2, spr - 1] = jump             # last pair
        sdf[3, 10:14] = (jump[0], jump[1], jump[0], jump[1])   # twice on one ray
        f32 = np.float32
        assert f32(1) / (f32(1) + np.exp(f32(s_val) * f32(jump[1]))) * -np.expm1(-f32(s_val) * (f32(jump[0]) - f32(jump[1]))) == f32(1)
        rgb = rng.uniform(size=(rays, spr, 3)).astype(np.float32)
        normal = (rng.normal(size=(n, 3)) * 0.7).astype(np.float32)
        target = rng.uniform(size=(rays, 3)).astype(np.float32)
        dC = rng.normal(size=(rays, 3)).astype(np.float32)
        y = np.zeros((n, 16), dtype=np.float32)
        y[:, 0] = sdf.reshape(-1)
        s64, r64 = sdf.astype(np.float64), rgb.astype(np.float64)
        z = lambda *sh: torch.zeros(*sh, device="cuda")
        yg, rg = cuda(y), cuda(rgb.reshape(n, 3))
        # stand-alone backward
        ds, dr, d_s = z(n), z(n, 3), z(1)
        nb.render_rays_bwd(c, yg, 16, rg, cuda(dC), rays, ds, dr, d_s=d_s)
        torch.cuda.synchronize()
        want_ds, want_dr, want_s = o.render_rays_backward(s64, r64, s_val, dC.astype(np.float64), want_ds=True)
        assert torch.isfinite(ds).all() and torch.isfinite(dr).all() and torch.isfinite(d_s).all()
        assert rel(ds.cpu().numpy().reshape(rays, spr), want_ds) <= GRAD_TOL
        assert rel(dr.cpu().numpy().reshape(rays, spr, 3), want_dr) <= GRAD_TOL
        # fused: compositing + loss + backward; fixed sample count, then the same rays as ragged rays
        Cr, wr, _, _ = o.render_rays(s64, r64, s_val)
        g = np.sign(Cr - target) / rays
        want_ds, want_dr = o.render_rays_backward(s64, r64, s_val, g)
        off = cuda(np.arange(rays + 1) * spr, torch.int32)
        for ragged in (False, True):
            Cg, wg, loss, dCg, ds, dr, dn, d_s = z(rays, 3), z(n), z(2), z(rays, 3), z(n), z(n, 3), z(n, 3), z(1)
            if ragged:
                nb.render_loss_bwd_ragged(c, yg, rg, cuda(normal), cuda(target), off, rays, n, Cg, wg, loss, dCg, ds, dr, dn, d_s=d_s)
            else:
                nb.render_loss_bwd(c, yg, rg, cuda(normal), cuda(target), rays, Cg, wg, loss, dCg, ds, dr, dn, d_s=d_s)
            torch.cuda.synchronize()
            for t in (Cg, wg, loss, ds, dr, d_s):
                assert torch.isfinite(t).all()
            assert rel(Cg.cpu().numpy(), Cr) <= FWD_TOL and rel(wg.cpu().numpy().reshape(rays, spr), wr) <= FWD_TOL
            assert rel(ds.cpu().numpy().reshape(rays, spr), want_ds) <= GRAD_TOL
            assert rel(dr.cpu().numpy().reshape(rays, spr, 3), want_dr) <= GRAD_TOL


@pytest.mark.parametrize("loss_kind", [1, 2])
def test_fused_render_loss_backward_against_oracle(loss_kind):
    """neus2_render_loss_bwd = render + loss + render backward in one launch."""
    rng = np.random.default_rng(40 + loss_kind)
    for spr, rays in ((64, 1500), (17, 9), (1, 5)):
        cfg = wl.make_config(2)
        cfg.samples_per_ray, cfg.loss_kind, cfg.huber_delta = spr, loss_kind, 0.05
        c = nb.make_config(cfg)
        n = rays * spr
        sdf = (rng.normal(size=(rays, spr)) * 0.05)
        sdf[0] = np.linspace(0.3, -0.3, spr)
        sdf = sdf.astype(np.float32)
        rgb = rng.uniform(size=(rays, spr, 3)).astype(np.float32)
        normal = (rng.normal(size=(n, 3)) * 0.7).astype(np.float32)
        target = rng.uniform(size=(rays, 3)).astype(np.float32)
        y = np.zeros((n, 16), dtype=np.float32)
        y[:, 0] = sdf.reshape(-1)
        z = lambda *sh: torch.zeros(*sh, device="cuda")
        Cg, wg, loss, dC, ds, dr, dn, d_s = z(rays, 3), z(n), z(2), z(rays, 3), z(n), z(n, 3), z(n, 3), z(1)
        nb.render_loss_bwd(c, cuda(y), cuda(rgb.reshape(n, 3)), cuda(normal), cuda(target), rays, Cg, wg, loss, dC, ds, dr, dn,
                           d_s=d_s)
        torch.cuda.synchronize()
        s64, r64 = sdf.astype(np.float64), rgb.astype(np.float64)
        Cr, wr, _, _ = o.render_rays(s64, r64, cfg.s)
        diff = Cr - target
        if loss_kind == 1:
            first, g = np.sum(np.abs(diff)) / rays, np.sign(diff) / rays
        else:
            first, g = np.sum(o.huber(diff, cfg.huber_delta)) / rays, o.huber_derivative(diff, cfg.huber_delta) / rays
        ln = np.linalg.norm(normal.astype(np.float64), axis=1)
        eik = cfg.beta * np.mean((ln - 1.0) ** 2)
        d_normal = (2.0 * cfg.beta / n) * ((ln - 1.0) / ln)[:, None] * normal
        d_sdf, d_rgb, ref_ds = o.render_rays_backward(s64, r64, cfg.s, g, want_ds=True)
        got_loss = loss.cpu().numpy()
        assert abs(got_loss[0] - first) <= FWD_TOL * first and abs(got_loss[1] - eik) <= FWD_TOL * eik
        assert rel(Cg.cpu().numpy(), Cr) <= FWD_TOL
        assert rel(wg.cpu().numpy().reshape(rays, spr), wr) <= FWD_TOL
        # a colour within rounding of its target may take the other branch of |.|' in fp32: compare where it is clear
        clear = np.abs(diff) > 1e-6
        assert np.array_equal(dC.cpu().numpy()[clear] > 0, g[clear] > 0)
        assert rel(dn.cpu().numpy(), d_normal) <= GRAD_TOL
        assert rel(dr.cpu().numpy().reshape(rays, spr, 3), d_rgb) <= GRAD_TOL
        if spr > 1:
            assert rel(ds.cpu().numpy().reshape(rays, spr), d_sdf) <= GRAD_TOL
            scale = float(np.sum(np.abs(d_sdf * s64))) / cfg.s
            assert abs(float(d_s.cpu()[0]) - ref_ds) <= GRAD_TOL * scale + 1e-9


@pytest.mark.parametrize("loss_kind", [1, 2])
def test_ragged_render_loss_backward_against_oracle(loss_kind):
    """Rays with their own sample counts: none, one, short, longer than one and than three wavefronts."""
    rng = np.random.default_rng(50 + loss_kind)
    cfg = wl.make_config(2)
    cfg.loss_kind, cfg.huber_delta = loss_kind, 0.05
    c = nb.make_config(cfg)
    lengths = np.array([3, 0, 64, 1, 65, 128, 200, 0, 17, 63, 129, 2] + list(rng.integers(0, 90, size=300)))
    off = np.zeros(len(lengths) + 1, dtype=np.int64)
    off[1:] = np.cumsum(lengths)
    rays, n = len(lengths), int(off[-1])
    sdf = (rng.normal(size=n) * 0.05)
    sdf[off[6]:off[7]] = np.linspace(0.4, -0.4, 200)          # a long ray that crosses the surface in its third chunk
    sdf = sdf.astype(np.float32)
    rgb = rng.uniform(size=(n, 3)).astype(np.float32)
    normal = (rng.normal(size=(n, 3)) * 0.7).astype(np.float32)
    target = rng.uniform(size=(rays, 3)).astype(np.float32)
    y = np.zeros((n, 16), dtype=np.float32)
    y[:, 0] = sdf
    z = lambda *sh: torch.zeros(*sh, device="cuda")
    Cg, wg, loss, dC, ds, dr, dn, d_s = z(rays, 3), z(n), z(2), z(rays, 3), z(n), z(n, 3), z(n, 3), z(1)
    nb.render_loss_bwd_ragged(c, cuda(y), cuda(rgb), cuda(normal), cuda(target), cuda(off, torch.int32), rays, n, Cg, wg, loss,
                              dC, ds, dr, dn, d_s=d_s)
    torch.cuda.synchronize()
    s64, r64 = sdf.astype(np.float64), rgb.astype(np.float64)
    Cr, wr, _ = o.render_rays_ragged(s64, r64, off, cfg.s)
    diff = Cr - target
    if loss_kind == 1:
        first, g = np.sum(np.abs(diff)) / rays, np.sign(diff) / rays
    else:
        first, g = np.sum(o.huber(diff, cfg.huber_delta)) / rays, o.huber_derivative(diff, cfg.huber_delta) / rays
    ln = np.linalg.norm(normal.astype(np.float64), axis=1)
    eik = cfg.beta * np.mean((ln - 1.0) ** 2)
    d_normal = (2.0 * cfg.beta / n) * ((ln - 1.0) / ln)[:, None] * normal
    d_sdf, d_rgb, ref_ds = o.render_rays_ragged_backward(s64, r64, off, cfg.s, g)
    got_loss = loss.cpu().numpy()
    assert abs(got_loss[0] - first) <= FWD_TOL * first and abs(got_loss[1] - eik) <= FWD_TOL * eik
    assert rel(Cg.cpu().numpy(), Cr) <= FWD_TOL
    assert np.all(Cg.cpu().numpy()[[1, 7]] == 0)                 # rays without samples
    assert rel(wg.cpu().numpy(), wr) <= FWD_TOL
    assert rel(dn.cpu().numpy(), d_normal) <= GRAD_TOL
    assert rel(dr.cpu().numpy(), d_rgb) <= GRAD_TOL
    assert rel(ds.cpu().numpy(), d_sdf) <= GRAD_TOL
    long_ray = slice(off[6], off[7])
    assert rel(ds.cpu().numpy()[long_ray], d_sdf[long_ray]) <= GRAD_TOL and np.linalg.norm(d_sdf[long_ray]) > 0
    scale = float(np.sum(np.abs(d_sdf * s64))) / cfg.s
    assert abs(float(d_s.cpu()[0]) - ref_ds) <= GRAD_TOL * scale


def test_step_with_ragged_rays():
    """A whole step on rays of different lengths (the colour network looks its direction up by
    the sample's ray), against the oracle."""
    w = wl.make_workload(2, n_rays=8)
    cfg, params = w["cfg"], w["params"]
    params["tables"] = (params["tables"].astype(np.float64) * 2000.0).astype(params["tables"].dtype)
    batch = wl.make_ragged_rays(150, seed=77)
    n, rays = batch["pos"].shape[0], batch["dirs"].shape[0]
    lengths = np.diff(batch["ray_offsets"])
    assert np.any(lengths == 0) and np.any(lengths > 64) and n % cfg.samples_per_ray != 0
    step = nb.Step(cfg, params, n, n_rays=rays)
    step.set_batch(batch)
    step.zero_grads()
    step.train_step()
    torch.cuda.synchronize()
    ref = o.train_step(cfg, params, batch)
    assert np.any(ref["alpha"] > 0.05)
    print(check_step(cfg, step, ref, n))


def test_color_forward_backward_alone():
    rng = np.random.default_rng(2)
    cfg = wl.make_config(2)
    c = nb.make_config(cfg)
    rays, spr = 21, cfg.samples_per_ray
    n = rays * spr
    W = [rng.normal(size=(cfg.color_dims[i + 1], cfg.color_dims[i])).astype(np.float32) * 0.3 for i in range(3)]
    pos = rng.uniform(size=(n, 3)).astype(np.float32)
    nrm = rng.normal(size=(n, 3)).astype(np.float32)
    dirs = rng.normal(size=(rays, 3))
    dirs = (dirs / np.linalg.norm(dirs, axis=1, keepdims=True)).astype(np.float32)
    y = rng.normal(size=(n, 16)).astype(np.float32)
    d_rgb = rng.normal(size=(n, 3)).astype(np.float32)
    d_sdf = rng.normal(size=(n,)).astype(np.float32)
    dn0 = rng.normal(size=(n, 3)).astype(np.float32)
    Wg = [cuda(w) for w in W]
    rgb = torch.empty(n, 3, device="cuda")
    args = (cuda(pos), cuda(nrm), cuda(dirs), cuda(y))
    kept = torch.zeros(2, n, 2, dtype=torch.int32, device="cuda")
    nb.color_fwd(c, *args, Wg, n, rgb, masks=kept)
    cin = o.color_input(pos, nrm.astype(np.float64), dirs, y.astype(np.float64), spr)
    rgb_r, acts, masks = o.color_forward(W, cin)
    assert rel(rgb.cpu().numpy(), rgb_r) <= FWD_TOL
    for got, want in zip(decode_masks(kept, n, 2), masks):
        assert np.mean(got != (want > 0)) < 1e-4
    d_u = d_rgb * rgb_r * (1 - rgb_r)
    gW, d_cin, _ = o.mlp_backward(W, acts, masks, d_u)
    want_dy = d_cin[:, 22:38].copy()
    want_dy[:, 0] += d_sdf
    # the backward kernel in both forms: masks from the forward kernel, or worked out again
    for given in (kept, None):
        dW = [torch.zeros_like(w) for w in Wg]
        d_y = torch.empty(n, 16, device="cuda")
        d_normal = cuda(dn0)
        d_pos = torch.empty(n, 3, device="cuda")
        nb.color_bwd(c, *args, Wg, rgb, cuda(d_rgb), cuda(d_sdf), n, dW, d_y, d_normal, d_pos, masks=given)
        torch.cuda.synchronize()
        for a, b in zip(dW, gW):
            assert rel(a.cpu().numpy(), b) <= GRAD_TOL
        assert rel(d_y.cpu().numpy(), want_dy) <= GRAD_TOL
        assert rel(d_normal.cpu().numpy(), dn0 + d_cin[:, 3:6]) <= GRAD_TOL
        assert rel(d_pos.cpu().numpy(), d_cin[:, 0:3]) <= GRAD_TOL


def test_adam_fp32_and_fp16():
    rng = np.random.default_rng(3)
    cnt = 100003
    p = rng.normal(size=cnt).astype(np.float32) * 1e-3
    g = rng.normal(size=cnt).astype(np.float32) * 1e-4
    g[:10] = 0.0
    m = rng.normal(size=cnt).astype(np.float32) * 1e-5
    v = np.abs(rng.normal(size=cnt)).astype(np.float32) * 1e-9
    for dtype in (0, 1):
        for t in (1, 7):
            m0 = np.zeros_like(m) if t == 1 else m
            v0 = np.zeros_like(v) if t == 1 else v
            pg, gg, mg, vg = cuda(p), cuda(g), cuda(m0), cuda(v0)
            if dtype == 1:
                half = cuda(p, torch.float16)
                nb.adam_step(half, pg, gg, mg, vg, 1, 1e-2, 0.9, 0.99, 1e-15, t)
            else:
                nb.adam_step(pg, None, gg, mg, vg, 0, 1e-2, 0.9, 0.99, 1e-15, t)
            torch.cuda.synchronize()
            pr, mr, vr = o.adam_step(p, g, m0, v0, t, 1e-2, 0.9, 0.99, 1e-15)
            # fp32 against float64: a few ulp of the largest term of each sum
            for got, want in ((pg, pr), (mg, mr), (vg, vr)):
                got = got.cpu().numpy().astype(np.float64)
                assert rel(got, want) <= 1e-6
                assert np.max(np.abs(got - want)) <= 1e-6 * np.max(np.abs(want))
            assert torch.all(gg == 0)
            if t == 1:
                assert np.array_equal(pg.cpu().numpy()[:10], p[:10])      # zero gradient: unchanged
            if dtype == 1:
                # the fp16 copy is the round-to-nearest-even of the fp32 master the kernel wrote
                assert torch.equal(half, pg.to(torch.float16))


@pytest.mark.parametrize("lazy", [False, True])
def test_adam_lazy_form_and_vector_tails(lazy):
    """Entries with a zero gradient: left alone in the lazy form, decayed in the dense one; both
    entry points, table sizes whose addressable part is not a multiple of four parameters."""
    rng = np.random.default_rng(5)
    cnt = 4099
    p = rng.normal(size=cnt).astype(np.float32) * 1e-3
    g = rng.normal(size=cnt).astype(np.float32) * 1e-4
    g[rng.uniform(size=cnt) < 0.6] = 0.0
    m = rng.normal(size=cnt).astype(np.float32) * 1e-5
    v = np.abs(rng.normal(size=cnt)).astype(np.float32) * 1e-9
    pg, gg, mg, vg = cuda(p), cuda(g), cuda(m), cuda(v)
    nb.adam_step(pg, None, gg, mg, vg, 0, 1e-2, 0.9, 0.99, 1e-15, 3, zero_grad=True, lazy=lazy)
    pr, mr, vr = o.adam_step(p, g, m, v, 3, 1e-2, 0.9, 0.99, 1e-15, lazy=lazy)
    for got, want in ((pg, pr), (mg, mr), (vg, vr)):
        assert rel(got.cpu().numpy(), want) <= 1e-6
    if lazy:
        z = g == 0
        assert np.array_equal(pg.cpu().numpy()[z], p[z]) and np.array_equal(mg.cpu().numpy()[z], m[z])
    assert torch.all(gg == 0)
    # tables: dense levels with (res+1)^3 * 2 parameters (2 mod 4), hashed levels, whole groups of zeros
    cfg = wl.make_config(2)
    cfg.log2_table_size, cfg.n_levels, cfg.active_levels = 12, 8, 8
    cfg.res = [4, 6, 10, 14, 40, 80, 100, 120]
    cfg.dense = [1 if (r + 1) ** 3 <= cfg.table_size else 0 for r in cfg.res]
    cfg.sdf_dims = [16] + cfg.sdf_dims[1:]
    assert cfg.dense == [1, 1, 1, 1, 0, 0, 0, 0] and ((cfg.res[0] + 1) ** 3 * 2) % 4 == 2
    c = nb.make_config(cfg)
    L, T = cfg.n_levels, cfg.table_size
    p = (rng.normal(size=(L, T, 2)) * 1e-3).astype(np.float32)
    g, m, v = np.zeros((L, T, 2), np.float32), np.zeros((L, T, 2), np.float32), np.zeros((L, T, 2), np.float32)
    for l in range(L):
        used = (cfg.res[l] + 1) ** 3 if cfg.dense[l] else T
        g[l, :used] = rng.normal(size=(used, 2)) * 1e-4
        g[l, :used][rng.uniform(size=used) < 0.7] = 0.0
        m[l, :used] = rng.normal(size=(used, 2)) * 1e-5
        v[l, :used] = np.abs(rng.normal(size=(used, 2))) * 1e-9
    tab, master, gg, mg, vg = cuda(p, torch.float16), cuda(p), cuda(g), cuda(m), cuda(v)
    nb.adam_tables(c, tab, master, gg, mg, vg, 1e-2, 0.9, 0.99, 1e-15, 9, zero_grad=True, lazy=lazy)
    torch.cuda.synchronize()
    pr, mr, vr = o.adam_step(p, g, m, v, 9, 1e-2, 0.9, 0.99, 1e-15, lazy=lazy)
    for got, want in ((master, pr), (mg, mr), (vg, vr)):
        got = got.cpu().numpy().astype(np.float64)
        assert rel(got, want) <= 1e-6 and np.max(np.abs(got - want)) <= 1e-6 * np.max(np.abs(want))
    assert torch.all(gg == 0)
    touched = torch.as_tensor(g != 0).cuda() if lazy else torch.ones_like(master, dtype=torch.bool)
    assert torch.equal(tab[touched], master.to(torch.float16)[touched])
    with pytest.raises(nb.Neus2Error):
        nb.lib()  # keep the import used
        nb._check(nb.lib().neus2_adam_step(pg.data_ptr(), None, gg.data_ptr(), mg.data_ptr(), vg.data_ptr(), 4, 0, 1e-2, 0.9, 0.99,
                                           1e-15, 1, 7, None))


@pytest.mark.parametrize("lazy", [False, True])
def test_adam_active_levels_flag_is_the_dense_update_while_the_other_levels_are_untouched(lazy):
    """NEUS2_ADAM_ACTIVE_LEVELS: with zero gradient and zero moments beyond the active levels (the state
    the progressive schedule of Sec. 4.3 keeps them in) the result is the oracle's update over every
    level; those levels are left bit for bit, also when something was written there."""
    rng = np.random.default_rng(15)
    cfg = wl.make_config(2)
    cfg.log2_table_size, cfg.n_levels, cfg.active_levels = 12, 8, 5
    cfg.res = [4, 6, 10, 14, 40, 80, 100, 120]
    cfg.dense = [1 if (r + 1) ** 3 <= cfg.table_size else 0 for r in cfg.res]
    cfg.sdf_dims = [16] + cfg.sdf_dims[1:]
    c = nb.make_config(cfg)
    L, T, A = cfg.n_levels, cfg.table_size, cfg.active_levels
    p = (rng.normal(size=(L, T, 2)) * 1e-3).astype(np.float32)
    p = p.astype(np.float16).astype(np.float32)                   # tables and master agree at the start
    g, m, v = (np.zeros((L, T, 2), np.float32) for _ in range(3))
    for l in range(A):
        used = (cfg.res[l] + 1) ** 3 if cfg.dense[l] else T
        g[l, :used] = rng.normal(size=(used, 2)) * 1e-4
        g[l, :used][rng.uniform(size=used) < 0.5] = 0.0
        m[l, :used] = rng.normal(size=(used, 2)) * 1e-5
        v[l, :used] = np.abs(rng.normal(size=(used, 2))) * 1e-9
    tab, master, gg, mg, vg = cuda(p, torch.float16), cuda(p), cuda(g), cuda(m), cuda(v)
    nb.adam_tables(c, tab, master, gg, mg, vg, 1e-2, 0.9, 0.99, 1e-15, 4, zero_grad=True, lazy=lazy, active_levels_only=True)
    torch.cuda.synchronize()
    pr, mr, vr = o.adam_step(p, g, m, v, 4, 1e-2, 0.9, 0.99, 1e-15, lazy=lazy)
    assert np.array_equal(pr[A:], p[A:].astype(np.float64)) and not mr[A:].any()      # the oracle's dense update leaves them too
    for got, want in ((master, pr), (mg, mr), (vg, vr)):
        got = got.cpu().numpy().astype(np.float64)
        assert rel(got, want) <= 1e-6 and np.max(np.abs(got - want)) <= 1e-6 * np.max(np.abs(want))
    assert torch.all(gg == 0)
    assert torch.equal(tab[A:], cuda(p[A:], torch.float16)) and torch.equal(master[A:], cuda(p[A:]))
    # the flag means "skip", whatever those levels hold: a gradient written there stays, uncleared
    gg[A + 1, 7, 1] = 1.0
    before = [t.clone() for t in (tab, master, mg, vg)]
    nb.adam_tables(c, tab, master, gg, mg, vg, 1e-2, 0.9, 0.99, 1e-15, 5, zero_grad=True, lazy=lazy, active_levels_only=True)
    torch.cuda.synchronize()
    assert float(gg[A + 1, 7, 1]) == 1.0
    for t, b in zip((tab, master, mg, vg), before):
        assert torch.equal(t[A:], b[A:])
    # and without the flag the same call updates it
    nb.adam_tables(c, tab, master, gg, mg, vg, 1e-2, 0.9, 0.99, 1e-15, 6, zero_grad=True, lazy=lazy)
    torch.cuda.synchronize()
    assert float(gg[A + 1, 7, 1]) == 0.0 and float(mg[A + 1, 7, 1]) > 0.0


def test_adam_all_equals_the_two_separate_calls():
    """Tables and the flat buffer of matrices in one launch: what neus2_adam_tables (bit for bit) and
    neus2_adam_step (to rounding) give, dense and lazy; the flat buffer against the oracle."""
    rng = np.random.default_rng(6)
    cfg = wl.make_config(2)
    cfg.log2_table_size = 13
    cfg.dense = [1 if (r + 1) ** 3 <= cfg.table_size else 0 for r in cfg.res]
    c = nb.make_config(cfg)
    L, T = cfg.n_levels, cfg.table_size
    small_n = 11 * 1000 + 3
    for lazy in (False, True):
        p = (rng.normal(size=(L, T, 2)) * 1e-3).astype(np.float32)
        g = (rng.normal(size=(L, T, 2)) * 1e-4).astype(np.float32)
        g[rng.uniform(size=g.shape) < 0.5] = 0.0
        for l in range(L):
            if cfg.dense[l]:
                g[l, (cfg.res[l] + 1) ** 3:] = 0.0
        m = (rng.normal(size=g.shape) * 1e-5).astype(np.float32) * (g != 0)
        v = (np.abs(rng.normal(size=g.shape)) * 1e-9).astype(np.float32) * (g != 0)
        sp, sg = rng.normal(size=small_n).astype(np.float32), rng.normal(size=small_n).astype(np.float32) * 1e-3
        sm, sv = rng.normal(size=small_n).astype(np.float32) * 1e-4, np.abs(rng.normal(size=small_n)).astype(np.float32) * 1e-7
        a = [cuda(p, torch.float16), cuda(p), cuda(g), cuda(m), cuda(v), cuda(sp), cuda(sg), cuda(sm), cuda(sv)]
        b = [t.clone() for t in a]
        nb.adam_all(c, a[0], a[1], a[2], a[3], a[4], a[5], a[6], a[7], a[8], 1e-2, 0.9, 0.99, 1e-15, 4, True, lazy)
        nb.adam_tables(c, b[0], b[1], b[2], b[3], b[4], 1e-2, 0.9, 0.99, 1e-15, 4, True, lazy)
        nb.adam_step(b[5], None, b[6], b[7], b[8], 0, 1e-2, 0.9, 0.99, 1e-15, 4, True, False)
        torch.cuda.synchronize()
        for x, y in zip(a[:5], b[:5]):
            assert torch.equal(x, y)                                  # the same kernel code
        for x, y in zip(a[5:], b[5:]):                                # two kernels: the compiler may fuse multiply-adds differently
            assert rel(x.cpu().numpy(), y.cpu().numpy()) <= 1e-6
        pr, mr, vr = o.adam_step(sp, sg, sm, sv, 4, 1e-2, 0.9, 0.99, 1e-15)
        assert rel(a[5].cpu().numpy(), pr) <= 1e-6 and rel(a[7].cpu().numpy(), mr) <= 1e-6 and rel(a[8].cpu().numpy(), vr) <= 1e-6
        assert torch.all(a[6] == 0)
        # with the levels beyond the active ones left out: the flat buffer rides along as before, the tables as
        # neus2_adam_tables with the same flag leaves them
        c.active_levels = 9
        a2, b2 = [t.clone() for t in a], [t.clone() for t in a]
        for t in (a2, b2):
            t[2].copy_(cuda(g)); t[6].copy_(cuda(sg))
        nb.adam_all(c, *a2, 1e-2, 0.9, 0.99, 1e-15, 5, True, lazy, active_levels_only=True)
        nb.adam_tables(c, b2[0], b2[1], b2[2], b2[3], b2[4], 1e-2, 0.9, 0.99, 1e-15, 5, True, lazy, active_levels_only=True)
        torch.cuda.synchronize()
        for x, y in zip(a2[:5], b2[:5]):
            assert torch.equal(x, y)
        assert torch.equal(a2[2][9:], cuda(g)[9:]) and torch.all(a2[2][:9] == 0) and torch.all(a2[6] == 0)
        assert torch.equal(a2[1][9:], a[1][9:]) and not torch.equal(a2[1][:9], a[1][:9])
        c.active_levels = cfg.active_levels


def test_adam_tables_skips_only_unaddressable_slots():
    """The table update leaves out the slots of dense levels no point can reach; the result must
    be the dense update of every parameter (their gradient and moments are zero)."""
    for k in (2, 4):
        cfg = wl.make_config(k)
        cfg.log2_table_size, cfg.n_levels, cfg.active_levels = 14, 8, 8      # small tables, dense and hashed levels
        cfg.res = cfg.res[:8]
        cfg.dense = [1 if (r + 1) ** 3 <= cfg.table_size else 0 for r in cfg.res]
        cfg.sdf_dims = [16] + cfg.sdf_dims[1:]
        assert 0 < sum(cfg.dense) < 8
        c = nb.make_config(cfg)
        rng = np.random.default_rng(30 + k)
        L, T = cfg.n_levels, cfg.table_size
        p = (rng.normal(size=(L, T, 2)) * 1e-3).astype(np.float32)
        g = np.zeros((L, T, 2), dtype=np.float32)
        m = np.zeros_like(g)
        v = np.zeros_like(g)
        for l in range(L):
            used = (cfg.res[l] + 1) ** 3 if cfg.dense[l] else T
            g[l, :used] = rng.normal(size=(used, 2)) * 1e-4
            m[l, :used] = rng.normal(size=(used, 2)) * 1e-5
            v[l, :used] = np.abs(rng.normal(size=(used, 2))) * 1e-9
        half = cfg.table_dtype == "f16"
        tab = cuda(p, torch.float16) if half else cuda(p)
        master = cuda(p) if half else None
        gg, mg, vg = cuda(g), cuda(m), cuda(v)
        nb.adam_tables(c, tab, master, gg, mg, vg, 1e-2, 0.9, 0.99, 1e-15, 5)
        torch.cuda.synchronize()
        pr, mr, vr = o.adam_step(p, g, m, v, 5, 1e-2, 0.9, 0.99, 1e-15)
        full = master if half else tab
        for got, want in ((full, pr), (mg, mr), (vg, vr)):
            got = got.cpu().numpy().astype(np.float64)
            assert rel(got, want) <= 1e-6
            assert np.max(np.abs(got - want)) <= 1e-6 * np.max(np.abs(want))
        assert torch.all(gg == 0)
        if half:
            assert torch.equal(tab, master.to(torch.float16))


def test_rigid_forward_backward():
    rng = np.random.default_rng(4)
    n = 5000
    x = rng.uniform(-1, 1, size=(n, 3)).astype(np.float32)
    tr = wl.make_rigid(9)
    R = o.rotation_from_axis_angle(tr["omega"])
    out = torch.empty(n, 3, device="cuda")
    nb.rigid_fwd(cuda(x), R.reshape(-1), tr["shift"], 0.5, 0.5, out)
    R32 = R.astype(np.float32).astype(np.float64)
    T32 = tr["shift"].astype(np.float32).astype(np.float64)
    assert rel(out.cpu().numpy(), o.rigid_forward(x, R32, T32, 0.5, 0.5)) <= 1e-6
    d_out = rng.normal(size=(n, 3)).astype(np.float32)
    Mb = torch.zeros(12, device="cuda")
    nb.rigid_bwd(cuda(x), tr["shift"], cuda(d_out), 0.5, Mb)
    torch.cuda.synchronize()
    M, dT, b = o.rigid_backward(x, R32, T32, d_out, 0.5)
    got = Mb.cpu().numpy()
    assert rel(got[:9].reshape(3, 3), M) <= GRAD_TOL
    assert rel(got[9:], b) <= GRAD_TOL


# ------------------------------------------------------------------ whole steps

def test_step_config1_full_size():
    cfg, step, ref, n = run_step(1, 4096)
    print(check_step(cfg, step, ref, n))


def test_step_config1_ragged_tail_and_position_gradient():
    cfg, step, ref, n = run_step(1, 1000 + 13, want_pos=True, scale_tables=3000.0)
    print(check_step(cfg, step, ref, n, want_pos=True))


@pytest.mark.parametrize("k,n_rays", [(2, 96), (3, 40), (4, 24)])
def test_step_ray_configs_small(k, n_rays):
    cfg, step, ref, n = run_step(k, n_rays)
    print(check_step(cfg, step, ref, n))


@pytest.mark.parametrize("k,n_rays", [(1, 300), (2, 96)])
def test_step_whose_backward_kernels_work_the_masks_out_again(k, n_rays):
    """Without mask buffers the backward kernels repeat the forward kernels' arithmetic."""
    cfg, step, ref, n = run_step(k, n_rays, keep_masks=False)
    assert step.buffers.sdf_masks is None and step.buffers.color_masks is None
    print(check_step(cfg, step, ref, n))


def test_step_config2_with_order_one_tables_and_position_gradient():
    """Tables scaled so that SDF values, alphas and masks are non-degenerate."""
    cfg, step, ref, n = run_step(2, 64, want_pos=True, scale_tables=2000.0)
    assert np.any(ref["alpha"] > 0.05)
    print(check_step(cfg, step, ref, n, want_pos=True))


def test_step_huber_loss_and_trained_slope():
    """Eq. 4's Huber colour term, and s of Phi_s as a parameter on the device that Adam updates
    together with the matrices (supplement Sec. E.3)."""
    w = wl.make_workload(2, n_rays=64)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    cfg.loss_kind, cfg.huber_delta = 2, 0.25
    params["tables"] = (params["tables"].astype(np.float64) * 2000.0).astype(params["tables"].dtype)
    n = batch["pos"].shape[0]
    step = nb.Step(cfg, params, n, learn_s=True)
    cfg_s = cfg.s
    step.s_dev.fill_(cfg_s * 1.5)          # the device value wins over the descriptor's
    cfg.s = cfg_s * 1.5                    # (the oracle reads cfg.s)
    step.set_batch(batch)
    step.zero_grads()
    step.train_step()
    torch.cuda.synchronize()
    ref = o.train_step(cfg, params, batch)
    r = np.abs(ref["diff"])
    assert np.any(r <= cfg.huber_delta) and np.any(r > cfg.huber_delta)
    print(check_step(cfg, step, ref, n))
    d_sdf = step.d_sdf.cpu().numpy().astype(np.float64)
    scale = float(np.sum(np.abs(d_sdf * ref["y"][:, 0]))) / cfg.s
    got = float(step.d_s.cpu()[0])
    assert abs(got - ref["d_s"]) <= GRAD_TOL * scale, (got, ref["d_s"], scale)
    assert abs(ref["d_s"]) > 1e-3 * scale          # not a vacuous comparison
    step.init_optimizer()
    step.adam()
    torch.cuda.synchronize()
    s_new, _, _ = o.adam_step(np.array([cfg.s]), np.array([got]), np.zeros(1), np.zeros(1), 1, 1e-2, 0.9, 0.99, 1e-15)
    assert abs(float(step.s_dev.cpu()[0]) - s_new[0]) <= 1e-6 * cfg.s
    assert float(step.d_s.cpu()[0]) == 0.0


@pytest.mark.parametrize("n_rays", [48, 1024 + 5])
def test_step_with_frozen_coordinate_levels(n_rays):
    """Eq. 1 feeds e = (x, h(x)): the two coarsest levels hold the vertex coordinates and are frozen
    (no table gradient, no Adam update); the position gradient still flows through them.  Small
    batch (atomic scatter) and large batch (LDS scatter + gather pass)."""
    w = wl.make_workload(2, n_rays=n_rays)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    tab = params["tables"].astype(np.float32) * 2000.0
    for level, cols in enumerate(((0, 1), (2, None))):
        r1 = cfg.res[level] + 1
        idx = np.arange(r1 ** 3)
        coords = [(idx % r1) / cfg.res[level] - 0.5, ((idx // r1) % r1) / cfg.res[level] - 0.5, (idx // (r1 * r1)) / cfg.res[level] - 0.5]
        tab[level, :r1 ** 3, 0] = coords[cols[0]]
        tab[level, :r1 ** 3, 1] = coords[cols[1]] if cols[1] is not None else 1.0
    params["tables"] = tab.astype(np.float16)
    cfg.frozen_levels = 2
    n = batch["pos"].shape[0]
    step = nb.Step(cfg, params, n, want_pos_grad=True)
    step.set_batch(batch)
    step.zero_grads()
    step.train_step()
    torch.cuda.synchronize()
    # the encoding of the frozen levels IS the position (and a constant)
    enc = from_level_major(step.enc, n)
    assert np.max(np.abs(enc[:, 0:3] - (batch["pos"] - 0.5))) <= 1e-3 and np.max(np.abs(enc[:, 3] - 1.0)) <= 1e-6
    if n_rays < 100:
        ref = o.train_step(cfg, params, batch, want_pos_grad=True)
        assert np.all(ref["dtables"][:2] == 0) and np.linalg.norm(ref["dtables"][2:]) > 0
        check_step(cfg, step, ref, n, want_pos=True)
    else:
        pick = np.arange(0, n_rays, 40)
        spr = cfg.samples_per_ray
        pts = (pick[:, None] * spr + np.arange(spr)[None, :]).reshape(-1)
        sub = {"pos": batch["pos"][pts], "dirs": batch["dirs"][pick], "target": batch["target"][pick]}
        ref = o.train_step(cfg, params, sub, want_pos_grad=True)
        assert rel(step.d_pos.cpu().numpy()[pts], ref["dpos"] * (len(pick) / n_rays)) <= GRAD_TOL
        want_t = o.table_gradient(cfg, batch["pos"], from_level_major(step.q, n), from_level_major(step.d_enc, n),
                                  step.d_normal.cpu().numpy())
        want_t[:2] = 0.0
        assert rel(step.d_tables.cpu().numpy(), want_t) <= GRAD_TOL
    assert float(step.d_tables[:2].abs().sum()) == 0.0
    before = step.tables[:2].clone()
    step.init_optimizer()
    step.adam()
    torch.cuda.synchronize()
    assert torch.equal(step.tables[:2], before) and not torch.equal(step.tables[2:4], cuda(params["tables"][2:4], torch.float16))


def test_step_config5_frames_with_transform_gradient():
    w = wl.make_workload(5, n_rays=32, frame=1)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    params["tables"] = (params["tables"].astype(np.float64) * 2000).astype(np.float16)
    world = batch["pos"]
    n = world.shape[0]
    R = o.rotation_from_axis_angle(batch["omega"]).astype(np.float32)
    T = batch["shift"].astype(np.float32)
    step = nb.Step(cfg, params, n, want_pos_grad=True)
    step.set_batch(batch)
    wg = cuda(world)
    nb.rigid_fwd(wg, R.reshape(-1), T, 0.5, 0.5, step.pos)
    step.zero_grads()
    step.train_step()
    Mb = torch.zeros(12, device="cuda")
    nb.rigid_bwd(wg, T, step.d_pos, 0.5, Mb)
    torch.cuda.synchronize()
    # the oracle gets the SAME fp32 transformed positions (index parity), checked to 1e-6 against its own transform
    pos_gpu = step.pos.cpu().numpy()
    assert rel(pos_gpu, o.rigid_forward(world, R, T, 0.5, 0.5)) <= 1e-6
    b2 = dict(batch)
    b2["pos"] = pos_gpu
    ref = o.train_step(cfg, params, b2, want_pos_grad=True)
    check_step(cfg, step, ref, n, want_pos=True)
    M, dT, bsum = o.rigid_backward(world, R, T, ref["dpos"], 0.5)
    got = Mb.cpu().numpy()
    assert rel(got[:9].reshape(3, 3), M) <= GRAD_TOL
    assert rel(got[9:], bsum) <= GRAD_TOL


def test_concentrated_batch_overflows_the_record_lists():
    """65536 samples inside a cube of side 2e-3: on every hashed level they share a handful of
    cells, so the per-range record lists of the LDS scatter overflow and the surplus goes
    through global atomics; also the worst case for same-address contention."""
    w = wl.make_workload(2, n_rays=1024)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    rng = np.random.default_rng(5)
    n = batch["pos"].shape[0]
    batch["pos"] = (0.37 + 2e-3 * rng.uniform(size=(n, 3))).astype(np.float32)
    step = nb.Step(cfg, params, n)
    assert step.workspace is not None
    step.set_batch(batch)
    step.zero_grads()
    step.train_step()
    torch.cuda.synchronize()
    # Points this close share near-zero pre-activations, so fp32 and float64 disagree on many
    # ReLU masks; the scatter is therefore checked on the adjoints the GPU itself produced.
    want = o.table_gradient(cfg, batch["pos"], from_level_major(step.q, n), from_level_major(step.d_enc, n),
                            step.d_normal.cpu().numpy())
    assert rel(step.d_tables.cpu().numpy(), want) <= GRAD_TOL
    # and the same adjoints through the atomic kernel alone (no workspace)
    c = step.c
    alone = torch.zeros_like(step.d_tables)
    nb.hash_scatter_bwd(c, step.pos, step.tables, step.q, step.d_enc, step.d_normal, n, alone)
    torch.cuda.synchronize()
    assert rel(alone.cpu().numpy(), want) <= GRAD_TOL


def test_training_loop_on_an_analytic_scene_learns():
    """The step used as a training loop (new rays every iteration, progressive levels, Adam): on a
    shaded sphere the colour loss falls and the rays that hit the sphere render a surface at the
    right distance, starting from a sphere of the wrong radius."""
    from paper_2212_05231_amd import demo
    out = demo.run(steps=200, n_rays=2048, log=lambda *_: None)
    first, last = out["history"][0][1], np.mean([h[1] for h in out["history"][-3:]])
    assert last < 0.3 * first, out["history"]
    # (the sign of the field in empty space is not asserted: without a mask term a black surface in
    # front of the background fits the photometric loss as well as no surface does)
    assert out["surface_found"] > 0.9 and out["depth_error"] < 0.06, out


@pytest.mark.parametrize("n_rays", [40, 1100])
def test_step_with_no_active_or_no_trained_level(n_rays):
    """Degenerate level settings on both scatter paths: lambda = 0 (every encoding is zero: the
    networks see zeros, all table gradients are zero) and frozen_levels = active_levels (levels
    feed the network but none is trained)."""
    for active, frozen in ((0, 0), (3, 3)):
        w = wl.make_workload(2, n_rays=n_rays)
        cfg, params, batch = w["cfg"], w["params"], w["batch"]
        params["tables"] = (params["tables"].astype(np.float64) * 2000.0).astype(params["tables"].dtype)
        cfg.active_levels, cfg.frozen_levels = active, frozen
        n = batch["pos"].shape[0]
        step = nb.Step(cfg, params, n)
        step.set_batch(batch)
        step.zero_grads()
        step.train_step()
        torch.cuda.synchronize()
        assert float(step.d_tables.abs().sum()) == 0.0
        assert torch.isfinite(step.loss).all()
        if active == 0:
            assert float(step.enc.abs().sum()) == 0.0 and float(step.y.abs().sum()) == 0.0
        if n_rays < 100:
            ref = o.train_step(cfg, params, batch)
            check_step(cfg, step, ref, n)


def test_empty_batch_is_a_no_op():
    cfg = wl.make_config(2)
    params = wl.make_params(cfg, 1)
    step = nb.Step(cfg, params, 0)
    step.train_step()
    torch.cuda.synchronize()
    assert float(step.d_tables.abs().sum()) == 0.0


def weight_gradients_from_adjoints(cfg, params, batch, d_y, d_normal, d_rgb):
    """dL/dH_l and dL/dW_l of a whole batch by the oracle's own functions, given the adjoints of
    (d,g), n and c of every sample: the oracle's forward pass over all points, ordinary
    back-propagation of d_y, Theorem 1's term S_l^T t_{l-1}^T from t_0 = (de/dx) d_normal, and the
    colour network's back-propagation of d_rgb.  What the sums over points must give when the
    per-sample adjoints (checked on sampled rays) are right."""
    H = params["H"]
    K = len(H)
    he = o.hash_encode(cfg, params["tables"], batch["pos"])
    y, acts, masks = o.mlp_forward(H, he["enc"])
    S, q = o.mlp_input_gradient(H, masks, 0)
    normal = np.einsum("nk,nka->na", q, he["jac"])
    dH, _, _ = o.mlp_backward(H, acts, masks, np.asarray(d_y, dtype=np.float64))
    t = np.einsum("nka,na->nk", he["jac"], np.asarray(d_normal, dtype=np.float64))
    for l in range(K):
        if l < K - 1:
            dH[l] += S[l].T @ t
            t = masks[l] * (t @ np.asarray(H[l], dtype=np.float64).T)
        else:
            dH[l][0, :] += np.sum(t, axis=0)
    cin = o.color_input(batch["pos"], normal, batch["dirs"], y, cfg.samples_per_ray)
    rgb, cacts, cmasks = o.color_forward(params["W"], cin)
    dW, _, _ = o.mlp_backward(params["W"], cacts, cmasks, np.asarray(d_rgb, dtype=np.float64) * rgb * (1.0 - rgb))
    return dH, dW


@pytest.mark.parametrize("k", [2, 3, 4])
def test_full_size_sampled_rays(k):
    """At the workload's full size and launch configuration: per-ray outputs of a random
    sample of rays against the oracle run on those rays alone; adjoints scale with 1/rays.
    The reductions over all points are checked element by element against the oracle applied to
    the per-sample adjoints the GPU produced: the table gradient (workload 4: 256 record lists
    per hashed level and a dense level that goes through record lists), and the weight gradients
    of both networks including the second-order term."""
    w = wl.make_workload(k)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    n = batch["pos"].shape[0]
    spr = cfg.samples_per_ray
    R = n // spr
    step = nb.Step(cfg, params, n)
    step.set_batch(batch)
    step.zero_grads()
    step.train_step()
    torch.cuda.synchronize()
    rng = np.random.default_rng(0)
    pick = np.sort(rng.choice(R, size=48, replace=False))
    pts = (pick[:, None] * spr + np.arange(spr)[None, :]).reshape(-1)
    sub = {"pos": batch["pos"][pts], "dirs": batch["dirs"][pick], "target": batch["target"][pick]}
    ref = o.train_step(cfg, params, sub)
    scale = len(pick) / R
    ptsg = torch.as_tensor(pts).cuda()
    assert rel(step.y[ptsg].cpu().numpy(), ref["y"]) <= FWD_TOL
    assert rel(step.normal[ptsg].cpu().numpy(), ref["normal"]) <= FWD_TOL
    assert rel(step.rgb[ptsg].cpu().numpy(), ref["rgb"]) <= FWD_TOL
    assert rel(step.C[torch.as_tensor(pick).cuda()].cpu().numpy(), ref["C"]) <= FWD_TOL
    assert_elementwise("y", step.y[ptsg].cpu().numpy(), ref["y"], FWD_TOL)
    assert_elementwise("normal", step.normal[ptsg].cpu().numpy(), ref["normal"], FWD_TOL)
    assert_elementwise("rgb", step.rgb[ptsg].cpu().numpy(), ref["rgb"], FWD_TOL)
    assert rel(step.d_y[ptsg].cpu().numpy(), ref["d_y"] * scale) <= GRAD_TOL
    assert rel(step.d_normal[ptsg].cpu().numpy(), ref["d_normal"] * scale) <= GRAD_TOL
    assert rel(step.d_rgb[ptsg].cpu().numpy(), ref["d_rgb"] * scale) <= GRAD_TOL
    assert rel(from_level_major(step.d_enc[:, ptsg], len(pts)), ref["d_enc"] * scale) <= GRAD_TOL
    assert float(step.d_tables[cfg.active_levels:].abs().sum()) == 0.0
    # the table gradient of ALL points, element by element and level by level
    q_all, d_enc_all = from_level_major(step.q, n), from_level_major(step.d_enc, n)
    want_t = o.table_gradient(cfg, batch["pos"], q_all, d_enc_all, step.d_normal.cpu().numpy())
    got_t = step.d_tables.cpu().numpy().astype(np.float64)
    for l in range(cfg.active_levels):
        assert rel(got_t[l], want_t[l]) <= GRAD_TOL, (l, rel(got_t[l], want_t[l]))
    bound = GRAD_TOL * (np.abs(want_t) + np.max(np.abs(want_t), axis=(1, 2), keepdims=True))
    assert np.all(np.abs(got_t - want_t) <= bound)
    del q_all, d_enc_all, want_t, got_t
    # the weight gradients of both networks, first and second order, summed over ALL points
    dH, dW = weight_gradients_from_adjoints(cfg, params, batch, step.d_y.cpu().numpy(), step.d_normal.cpu().numpy(),
                                            step.d_rgb.cpu().numpy())
    for l, (a, b) in enumerate(zip(step.dH, dH)):
        assert rel(a.cpu().numpy(), b) <= GRAD_TOL, ("dH", l, rel(a.cpu().numpy(), b))
    for l, (a, b) in enumerate(zip(step.dW, dW)):
        assert rel(a.cpu().numpy(), b) <= GRAD_TOL, ("dW", l, rel(a.cpu().numpy(), b))


def test_dense_level_through_record_lists_and_its_range_crossings():
    """Workload 4's descriptor at 2^16 points, the smallest batch that takes the LDS scatter: its
    level of resolution 101 is dense with 130 ranges of 8192 slots, more than the in-place path
    takes, so its rows go through record lists; a row whose x+1 corner is the first slot of the
    next range is split (that corner goes straight to the gradient).  Every tensor of the step,
    the table gradient level by level, against the full oracle."""
    w = wl.make_workload(4, n_rays=1024)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    params["tables"] = (params["tables"].astype(np.float64) * 2000.0).astype(params["tables"].dtype)
    level = 5
    assert cfg.dense[level] == 1 and (cfg.res[level] + 1) ** 3 > 64 * 8192
    n = batch["pos"].shape[0]
    assert n == 1 << 16
    step = nb.Step(cfg, params, n)
    assert step.workspace is not None
    step.set_batch(batch)
    step.zero_grads()
    step.train_step()
    torch.cuda.synchronize()
    ref = o.train_step(cfg, params, batch)
    # rows of that level whose two x corners fall into different ranges exist in this batch
    idx = ref["he"]["idx"][:, level, :]
    crossing = (idx[:, 0::2] >> 13) != (idx[:, 1::2] >> 13)
    assert crossing.sum() >= 4
    check_step(cfg, step, ref, n, outliers=1e-4)
    got_t = step.d_tables.cpu().numpy().astype(np.float64)
    for l in range(cfg.n_levels):
        assert rel(got_t[l], ref["dtables"][l]) <= GRAD_TOL, (l, rel(got_t[l], ref["dtables"][l]))
    # the slots those crossing rows touch, one by one
    slots = np.unique(idx[:, 1::2][crossing])
    np.testing.assert_allclose(got_t[level, slots], ref["dtables"][level, slots], rtol=GRAD_TOL,
                               atol=GRAD_TOL * np.max(np.abs(ref["dtables"][level])))


@pytest.mark.parametrize("seed", [0, 1, 2, 3, 4, 5, 6, 7])
def test_grid_shapes_other_than_the_benchmark_ones(seed):
    """Encode and scatter-add (the path that keeps ranges of the gradient in LDS) on grids drawn at random:
    8 or 16 levels, 2^12 .. 2^21 entries a level, resolutions from 2 up to 8192 with any mix of dense and hashed
    levels (none, all), any number of active and frozen levels, both table types, ray-shaped and uniform points,
    a ragged number of points.  Indices bit for bit, values and the table gradient of every level against the
    oracle: the host-side plan of the scatter (which level takes which kind of list, how many ranges, how the
    lists are cut) must hold for shapes nobody tuned it for."""
    rng = np.random.default_rng(4000 + seed)
    L = int(rng.choice([8, 16]))
    log2_T = int(rng.integers(12, 22))
    T = 1 << log2_T
    res_min = int(rng.integers(2, 40))
    res_max = int(rng.choice([64, 200, 777, 2048, 8192]))
    res = wl.level_resolutions(L, res_min, max(res_max, res_min + L))
    if seed % 4 == 3:
        res = sorted(int(r) for r in rng.integers(2, 3000, size=L))          # not geometric at all
    dense = wl.dense_flags(res, T)
    if seed == 5:
        dense = [0] * L                                                       # hashed although they would fit
    cfg = wl.make_config(2)
    cfg.n_levels, cfg.log2_table_size, cfg.res, cfg.dense = L, log2_T, res, dense
    cfg.active_levels = int(rng.integers(1, L + 1)) if seed % 2 else L
    cfg.frozen_levels = min(1 + seed % 2, cfg.active_levels - 1) if seed % 3 == 1 else 0
    cfg.table_dtype = "f16" if seed % 2 == 0 else "f32"
    cfg.sdf_dims = [2 * L, 64, 64, 16]
    c = nb.make_config(cfg)
    n = (1 << 16) + int(rng.integers(1, 40000))
    if seed % 2:
        pos = wl.make_points(n, 4100 + seed)
    else:
        pos = wl.make_rays((n + 63) // 64, 64, 4100 + seed)["pos"][:n]
    tab = rng.uniform(-1.0, 1.0, size=(L, T, 2))
    tab = tab.astype(np.float16 if cfg.table_dtype == "f16" else np.float32)
    tables = cuda(tab, torch.float16 if cfg.table_dtype == "f16" else torch.float32)
    print(f"seed {seed}: L {L}, T 2^{log2_T}, res {res}, dense {dense}, active {cfg.active_levels}, frozen {cfg.frozen_levels}, "
          f"{cfg.table_dtype}, n {n}", flush=True)
    enc = torch.full((L, n, 2), 7.0, device="cuda")
    jac = torch.full((L, 3, n, 2), 7.0, device="cuda")
    idx = torch.zeros(n, L, 8, dtype=torch.int32, device="cuda")
    nb.hash_encode(c, cuda(pos), tables, enc, jac, idx)
    torch.cuda.synchronize()
    ref = o.hash_encode(cfg, tab, pos)
    assert np.array_equal(idx.cpu().numpy().astype(np.int64) & 0xFFFFFFFF, ref["idx"])
    del idx
    assert rel(from_level_major(enc, n), ref["enc"]) <= FWD_TOL
    assert rel(jac_from_level_major(jac, n), ref["jac"]) <= FWD_TOL
    q = rng.normal(size=(n, 2 * L)).astype(np.float32)
    d_enc = (rng.normal(size=(n, 2 * L)) / n).astype(np.float32)
    d_normal = (rng.normal(size=(n, 3)) / n * 1e-2).astype(np.float32)
    to_lm = lambda a: cuda(a.reshape(n, L, 2).transpose(1, 0, 2))
    want = o.table_gradient(cfg, pos, q, d_enc, d_normal)
    want[:cfg.frozen_levels] = 0.0
    ws = torch.zeros(nb.workspace_bytes(c, n) // 4, dtype=torch.int32, device="cuda")
    for workspace in (ws, None):                                  # LDS path, atomic path
        got = torch.zeros(L, T, 2, device="cuda")
        nb.hash_scatter_bwd(c, cuda(pos), tables, to_lm(q), to_lm(d_enc), cuda(d_normal), n, got, workspace=workspace)
        torch.cuda.synchronize()
        got = got.cpu().numpy().astype(np.float64)
        for l in range(L):
            if l < cfg.frozen_levels or l >= cfg.active_levels:
                assert not got[l].any(), l
            else:
                assert rel(got[l], want[l]) <= GRAD_TOL, (workspace is not None, l, res[l], dense[l], rel(got[l], want[l]))
        bound = GRAD_TOL * (np.abs(want) + np.max(np.abs(want), axis=(1, 2), keepdims=True))
        assert np.all(np.abs(got - want) <= bound), workspace is not None


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_whole_step_on_shapes_other_than_the_benchmark_ones(seed):
    """The whole training step against the full oracle on descriptors drawn at random: 8 or 16 levels, one or two
    hidden SDF layers, table sizes and resolutions that no benchmark workload has, 64, 40, 7 or 3 samples per ray,
    L1 or Huber, fp16 or fp32 tables, a batch below or above the size at which the scatter-add changes path."""
    rng = np.random.default_rng(4200 + seed)
    L = (8, 16, 16, 8)[seed]
    log2_T = (15, 17, 13, 18)[seed]
    res = wl.level_resolutions(L, int(rng.integers(3, 30)), int(rng.choice([300, 1000, 3000])))
    cfg = wl.make_config(2)
    cfg.n_levels, cfg.log2_table_size, cfg.res, cfg.dense = L, log2_T, res, wl.dense_flags(res, 1 << log2_T)
    cfg.active_levels = L if seed != 2 else 11
    cfg.table_dtype = "f16" if seed % 2 == 0 else "f32"
    cfg.sdf_dims = [2 * L, 64, 64, 16] if seed != 1 else [2 * L, 64, 16]
    cfg.samples_per_ray = (64, 40, 7, 3)[seed]
    cfg.loss_kind = 1 + seed % 2
    n_rays = (1024 + 9, 700, 9500, 1000)[seed]
    params = wl.make_params(cfg, 4300 + seed)
    params["tables"] = (params["tables"].astype(np.float64) * 3000.0).astype(params["tables"].dtype)
    batch = wl.make_rays(n_rays, cfg.samples_per_ray, 4400 + seed)
    n = batch["pos"].shape[0]
    print(f"seed {seed}: L {L}, T 2^{log2_T}, res {res}, dense {cfg.dense}, active {cfg.active_levels}, {cfg.table_dtype}, "
          f"sdf {cfg.sdf_dims}, {cfg.samples_per_ray} samples per ray, loss {cfg.loss_kind}, n {n}", flush=True)
    want_pos = seed >= 2              # the gradient with respect to the positions as well (seed 2: from stored second derivatives)

    def both(batch):
        n = batch["pos"].shape[0]
        step = nb.Step(cfg, params, n, want_pos_grad=want_pos)
        step.set_batch(batch)
        step.zero_grads()
        step.train_step()
        torch.cuda.synchronize()
        ref = o.train_step(cfg, params, batch, want_pos_grad=want_pos)
        # points at which a ReLU mask differs between the kernels' arithmetic and float64: a pre-activation within
        # rounding of zero; either side of it is a valid decision, but the unit's weight then enters dd/de or not
        flipped = np.zeros(n, dtype=bool)
        for words, want in ((step.sdf_masks, ref["masks"]), (step.color_masks, ref["cmasks"])):
            for got_m, want_m in zip(decode_masks(words, n, len(want)), want):
                flipped |= np.any(got_m != (np.asarray(want_m) != 0), axis=1)
        return step, ref, n, flipped

    step, ref, n, flipped = both(batch)
    if flipped.any():
        # with order-one tables one such point is visible in every sum at the 1e-4 bar: the rays that hold one are
        # taken out of the batch and the step is compared on the rest (the other points' values do not change)
        spr = cfg.samples_per_ray
        rays = np.unique(np.nonzero(flipped)[0] // spr)
        print(f"seed {seed}: {int(flipped.sum())} points with a mask decided differently, rays {rays.tolist()} left out", flush=True)
        assert len(rays) <= 6
        keep = np.setdiff1d(np.arange(n // spr), rays)
        batch = {"pos": batch["pos"].reshape(-1, spr, 3)[keep].reshape(-1, 3), "dirs": batch["dirs"][keep],
                 "target": batch["target"][keep]}
        step, ref, n, flipped = both(batch)
        assert not flipped.any()
    if seed in (0, 2):
        assert n >= 1 << 16                      # the scatter-add's path for large batches
    check_step(cfg, step, ref, n, want_pos=want_pos)
    got_t = step.d_tables.cpu().numpy().astype(np.float64)
    for l in range(cfg.active_levels):
        assert rel(got_t[l], ref["dtables"][l]) <= GRAD_TOL, (l, rel(got_t[l], ref["dtables"][l]))


def test_large_batch_position_gradient():
    """Batches of 2^16 points and more take the path that keeps the table gradient in LDS; the
    position gradient then comes from a gather pass of its own.  Against the oracle on a sample
    of rays (adjoints scale with 1/rays), and against the atomic path on all points."""
    w = wl.make_workload(2, n_rays=1024 + 3)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    params["tables"] = (params["tables"].astype(np.float64) * 2000.0).astype(params["tables"].dtype)
    n = batch["pos"].shape[0]
    spr = cfg.samples_per_ray
    R = n // spr
    assert n >= 1 << 16
    outs = []
    for use_ws in (True, False):
        step = nb.Step(cfg, params, n, want_pos_grad=True, use_workspace=use_ws)
        step.set_batch(batch)
        step.zero_grads()
        step.train_step()
        torch.cuda.synchronize()
        outs.append((step.d_pos.cpu().numpy().astype(np.float64), step.d_tables.cpu().numpy().astype(np.float64)))
    assert rel(outs[0][0], outs[1][0]) <= 1e-5 and rel(outs[0][1], outs[1][1]) <= 1e-5
    rng = np.random.default_rng(1)
    pick = np.sort(rng.choice(R, size=40, replace=False))
    pts = (pick[:, None] * spr + np.arange(spr)[None, :]).reshape(-1)
    sub = {"pos": batch["pos"][pts], "dirs": batch["dirs"][pick], "target": batch["target"][pick]}
    ref = o.train_step(cfg, params, sub, want_pos_grad=True)
    assert np.linalg.norm(ref["dpos"]) > 0
    assert rel(outs[0][0][pts], ref["dpos"] * (len(pick) / R)) <= GRAD_TOL


def test_full_size_dynamic_frame_sampled_rays():
    """Workload 5 at full size as bench.py runs it: rigid transform, step with the position
    gradient (gather pass of the large-batch scatter), reduction to (M, b).  Sampled rays against
    the oracle on those rays alone; the reduction against the oracle's applied to the GPU's
    position gradient."""
    w = wl.make_workload(5)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    params["tables"] = (params["tables"].astype(np.float64) * 2000).astype(np.float16)
    world = batch["pos"]
    n = world.shape[0]
    spr = cfg.samples_per_ray
    R = o.rotation_from_axis_angle(batch["omega"]).astype(np.float32)
    T = batch["shift"].astype(np.float32)
    step = nb.Step(cfg, params, n, want_pos_grad=True)
    step.set_batch(batch)
    wg = cuda(world)
    nb.rigid_fwd(wg, R.reshape(-1), T, 0.5, 0.5, step.pos)
    step.zero_grads()
    step.train_step()
    Mb = torch.zeros(12, device="cuda")
    nb.rigid_bwd(wg, T, step.d_pos, 0.5, Mb)
    torch.cuda.synchronize()
    pos_gpu = step.pos.cpu().numpy()
    rng = np.random.default_rng(2)
    rays = n // spr
    pick = np.sort(rng.choice(rays, size=40, replace=False))
    pts = (pick[:, None] * spr + np.arange(spr)[None, :]).reshape(-1)
    assert rel(pos_gpu[pts], o.rigid_forward(world[pts], R, T, 0.5, 0.5)) <= 1e-6
    sub = {"pos": pos_gpu[pts], "dirs": batch["dirs"][pick], "target": batch["target"][pick]}
    ref = o.train_step(cfg, params, sub, want_pos_grad=True)
    scale = len(pick) / rays
    d_pos = step.d_pos.cpu().numpy().astype(np.float64)
    assert rel(step.y.cpu().numpy()[pts], ref["y"]) <= FWD_TOL
    assert rel(step.C.cpu().numpy()[pick], ref["C"]) <= FWD_TOL
    assert np.linalg.norm(ref["dpos"]) > 0 and rel(d_pos[pts], ref["dpos"] * scale) <= GRAD_TOL
    M, dT, bsum = o.rigid_backward(world, R, T, d_pos, 0.5)
    got = Mb.cpu().numpy()
    assert rel(got[:9].reshape(3, 3), M) <= GRAD_TOL and rel(got[9:], bsum) <= GRAD_TOL


def test_full_size_config2_against_full_oracle():
    """The whole benchmark step, all gradients, against the oracle at full size (about a minute of CPU)."""
    cfg, step, ref, n = run_step(2, None)
    errs = check_step(cfg, step, ref, n, outliers=1e-4)
    print({k: f"{v:.2e}" for k, v in errs.items()})
