"""ctypes binding of libneus2.so: the same names as include/neus2.h, argument marshalling
only.  Tensors are torch tensors on the GPU (torch owns memory and streams); every step of
the computation runs inside the library's HIP kernels.  There is no fallback: if the
library has not been built, `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libneus2.so")

MAX_LEVELS = 32
MAX_MATS = 4

ERROR_NAMES = {0: "OK", -1: "ERR_NULL", -2: "ERR_SHAPE", -3: "ERR_CONFIG", -4: "ERR_ALIGN",
               -5: "ERR_UNSUPPORTED", -6: "ERR_HIP"}


class Neus2Config(C.Structure):
    _fields_ = [
        ("n_levels", C.c_int32), ("n_features", C.c_int32), ("log2_table_size", C.c_int32),
        ("active_levels", C.c_int32), ("table_dtype", C.c_int32),
        ("res", C.c_int32 * MAX_LEVELS), ("dense", C.c_int32 * MAX_LEVELS),
        ("n_sdf_mats", C.c_int32), ("sdf_dims", C.c_int32 * (MAX_MATS + 1)),
        ("n_color_mats", C.c_int32), ("color_dims", C.c_int32 * (MAX_MATS + 1)),
        ("samples_per_ray", C.c_int32), ("loss_kind", C.c_int32),
        ("s", C.c_float), ("beta", C.c_float), ("huber_delta", C.c_float),
        ("frozen_levels", C.c_int32),
    ]


_P = C.c_void_p


class Neus2StepBuffers(C.Structure):
    _fields_ = [(name, _P) for name in (
        "pos", "dirs", "target", "tables", "H", "W",
        "enc", "jac", "y", "q", "normal", "rgb", "C", "weights", "loss",
        "dC", "d_sdf", "d_rgb", "d_y", "d_normal", "d_enc", "d_pos", "dH", "dW", "d_tables", "workspace")] + [
        ("workspace_bytes", C.c_int64), ("s_dev", _P), ("d_s", _P), ("ray_offsets", _P), ("sample_ray", _P),
        ("n_rays", C.c_int64), ("sdf_masks", _P), ("color_masks", _P)]


class Neus2Error(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"libneus2: {ERROR_NAMES.get(code, code)}: {message}")
        self.code = code


_lib = None

_SIGNATURES = {
    "neus2_last_error": (C.c_char_p, []),
    "neus2_version": (C.c_int, []),
    "neus2_validate_config": (C.c_int, [C.POINTER(Neus2Config)]),
    "neus2_workspace_bytes": (C.c_int64, [C.POINTER(Neus2Config), C.c_int64]),
    "neus2_hash_encode": (C.c_int, [C.POINTER(Neus2Config), _P, _P, C.c_int64, _P, _P, _P, _P]),
    "neus2_sdf_fwd_grad": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, C.c_int64, _P, _P, _P, _P, _P]),
    "neus2_color_fwd": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, _P, C.c_int64, _P, _P, _P]),
    "neus2_color_bwd": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, _P, _P, _P, _P, C.c_int64, _P, _P, _P, _P, _P, _P]),
    "neus2_render_loss_bwd_ragged": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, _P, C.c_int64, C.c_int64, _P, _P, _P,
                                               _P, _P, _P, _P, _P, _P]),
    "neus2_render_rays": (C.c_int, [C.POINTER(Neus2Config), _P, C.c_int64, _P, _P, C.c_int64, _P, _P, _P]),
    "neus2_render_rays_bwd": (C.c_int, [C.POINTER(Neus2Config), _P, C.c_int64, _P, _P, _P, C.c_int64, _P, _P, _P, _P]),
    "neus2_render_loss_bwd": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, C.c_int64, _P, _P, _P, _P, _P, _P, _P, _P, _P]),
    "neus2_loss": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, C.c_int64, C.c_int64, _P, _P, _P, _P, _P]),
    "neus2_sdf_bwd_2nd": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, _P, _P, _P, C.c_int64, _P, _P, _P, _P, _P,
                                    C.c_int64, _P, _P]),
    "neus2_sdf_mlp_bwd": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, C.c_int64, _P, _P, _P, _P, _P]),
    "neus2_sdf_deep_workspace_bytes": (C.c_int64, [C.c_int32, C.c_int64]),
    "neus2_sdf_deep_fwd_grad": (C.c_int, [C.c_int32, C.c_int32, _P, _P, _P, C.c_int64, _P, _P, _P, _P, C.c_int64, _P]),
    "neus2_sdf_deep_bwd": (C.c_int, [C.c_int32, C.c_int32, _P, _P, _P, _P, _P, C.c_int64, _P, _P, _P, C.c_int64, _P]),
    "neus2_hash_scatter_bwd": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, C.c_int64, _P, _P, _P, C.c_int64, _P]),
    "neus2_hash_scatter_bwd_static": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, C.c_int64, _P, _P]),
    "neus2_adam_step": (C.c_int, [_P, _P, _P, _P, _P, C.c_int64, C.c_int, C.c_float, C.c_float, C.c_float,
                                  C.c_float, C.c_int, C.c_int, _P]),
    "neus2_adam_tables": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, C.c_float, C.c_float, C.c_float,
                                    C.c_float, C.c_int, C.c_int, _P]),
    "neus2_adam_all": (C.c_int, [C.POINTER(Neus2Config), _P, _P, _P, _P, _P, _P, _P, _P, _P, C.c_int64, C.c_float, C.c_float,
                                 C.c_float, C.c_float, C.c_int, C.c_int, _P]),
    "neus2_rigid_fwd": (C.c_int, [_P, _P, _P, C.c_float, C.c_float, C.c_int64, _P, _P]),
    "neus2_rigid_bwd": (C.c_int, [_P, _P, _P, C.c_float, C.c_int64, _P, _P]),
    "neus2_rigid_fwd_dev": (C.c_int, [_P, _P, C.c_float, C.c_float, C.c_int64, _P, _P]),
    "neus2_rigid_bwd_dev": (C.c_int, [_P, _P, _P, C.c_float, C.c_int64, _P, _P]),
    "neus2_pose_update": (C.c_int, [_P, _P, _P, _P, _P, _P, C.c_float, C.c_float, C.c_float, C.c_float, C.c_int, C.c_int, _P]),
    "neus2_occupancy_points": (C.c_int, [C.c_int, _P, _P, C.c_int64, _P, _P]),
    "neus2_occupancy_update": (C.c_int, [C.c_int, _P, _P, _P, C.c_int64, C.c_int64, _P, C.c_float, C.c_float, C.c_float, _P, _P]),
    "neus2_march_rays": (C.c_int, [C.c_int, _P, _P, _P, _P, C.c_int64, C.c_float, C.c_int32, C.c_int64, _P, _P, _P, _P, _P]),
    "neus2_train_step": (C.c_int, [C.POINTER(Neus2Config), C.POINTER(Neus2StepBuffers), C.c_int64, _P]),
}

EXPORTS = tuple(_SIGNATURES)


def lib():
    """The loaded library; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2212_05231_amd.build` first")
        handle = C.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(handle, name)
            fn.restype = res
            fn.argtypes = args
        _lib = handle
    return _lib


def _check(code: int) -> None:
    if code != 0:
        raise Neus2Error(code, lib().neus2_last_error().decode())


def make_config(cfg) -> Neus2Config:
    """`cfg` is a workloads.Config (or anything with the same attributes)."""
    c = Neus2Config()
    c.n_levels, c.n_features, c.log2_table_size = cfg.n_levels, cfg.n_features, cfg.log2_table_size
    c.active_levels = cfg.active_levels
    c.table_dtype = 1 if cfg.table_dtype == "f16" else 0
    for l in range(cfg.n_levels):
        c.res[l] = cfg.res[l]
        c.dense[l] = cfg.dense[l]
    c.n_sdf_mats = len(cfg.sdf_dims) - 1
    for i, d in enumerate(cfg.sdf_dims):
        c.sdf_dims[i] = d
    c.n_color_mats = max(len(cfg.color_dims) - 1, 0)
    for i, d in enumerate(cfg.color_dims):
        c.color_dims[i] = d
    c.samples_per_ray, c.loss_kind, c.s, c.beta = cfg.samples_per_ray, cfg.loss_kind, cfg.s, cfg.beta
    c.huber_delta = getattr(cfg, "huber_delta", 0.0)
    c.frozen_levels = getattr(cfg, "frozen_levels", 0)
    return c


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if not t.is_contiguous():
        raise ValueError("tensors passed to libneus2 must be contiguous")
    return t.data_ptr()


def _ptr_array(ts: Sequence):
    arr = (C.c_void_p * max(len(ts), 1))()
    for i, t in enumerate(ts):
        arr[i] = _ptr(t)
    return arr


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def validate_config(c: Neus2Config) -> int:
    return lib().neus2_validate_config(C.byref(c))


def hash_encode(c, pos, tables, enc, jac, dbg_idx=None):
    _check(lib().neus2_hash_encode(C.byref(c), _ptr(pos), _ptr(tables), pos.shape[0], _ptr(enc), _ptr(jac),
                                   _ptr(dbg_idx), _stream()))


def sdf_fwd_grad(c, enc, jac, H, n, y, q, normal, masks=None):
    _check(lib().neus2_sdf_fwd_grad(C.byref(c), _ptr(enc), _ptr(jac), _ptr_array(H), n, _ptr(y), _ptr(q),
                                    _ptr(normal), _ptr(masks), _stream()))


def color_fwd(c, pos, normal, dirs, y, W, n, rgb, sample_ray=None, masks=None):
    _check(lib().neus2_color_fwd(C.byref(c), _ptr(pos), _ptr(normal), _ptr(dirs), _ptr(sample_ray), _ptr(y), _ptr_array(W), n,
                                 _ptr(rgb), _ptr(masks), _stream()))


def color_bwd(c, pos, normal, dirs, y, W, rgb, d_rgb, d_sdf, n, dW, d_y, d_normal, d_pos=None, sample_ray=None, masks=None):
    _check(lib().neus2_color_bwd(C.byref(c), _ptr(pos), _ptr(normal), _ptr(dirs), _ptr(sample_ray), _ptr(y), _ptr_array(W),
                                 _ptr(rgb), _ptr(d_rgb), _ptr(d_sdf), n, _ptr_array(dW), _ptr(d_y), _ptr(d_normal),
                                 _ptr(d_pos), _ptr(masks), _stream()))


def render_rays(c, sdf, sdf_stride, rgb, rays, Cout, weights, s_dev=None):
    _check(lib().neus2_render_rays(C.byref(c), _ptr(sdf), sdf_stride, _ptr(rgb), _ptr(s_dev), rays, _ptr(Cout),
                                   _ptr(weights), _stream()))


def render_rays_bwd(c, sdf, sdf_stride, rgb, dC, rays, d_sdf, d_rgb, s_dev=None, d_s=None):
    _check(lib().neus2_render_rays_bwd(C.byref(c), _ptr(sdf), sdf_stride, _ptr(rgb), _ptr(dC), _ptr(s_dev), rays,
                                       _ptr(d_sdf), _ptr(d_rgb), _ptr(d_s), _stream()))


def render_loss_bwd(c, y, rgb, normal, target, rays, Cout, weights, loss_out, dC, d_sdf, d_rgb, d_normal, s_dev=None, d_s=None):
    _check(lib().neus2_render_loss_bwd(C.byref(c), _ptr(y), _ptr(rgb), _ptr(normal), _ptr(target), _ptr(s_dev), rays,
                                       _ptr(Cout), _ptr(weights), _ptr(loss_out), _ptr(dC), _ptr(d_sdf), _ptr(d_rgb),
                                       _ptr(d_normal), _ptr(d_s), _stream()))


def render_loss_bwd_ragged(c, y, rgb, normal, target, ray_offsets, rays, n, Cout, weights, loss_out, dC, d_sdf, d_rgb,
                           d_normal, s_dev=None, d_s=None):
    _check(lib().neus2_render_loss_bwd_ragged(C.byref(c), _ptr(y), _ptr(rgb), _ptr(normal), _ptr(target), _ptr(ray_offsets),
                                              _ptr(s_dev), rays, n, _ptr(Cout), _ptr(weights), _ptr(loss_out), _ptr(dC),
                                              _ptr(d_sdf), _ptr(d_rgb), _ptr(d_normal), _ptr(d_s), _stream()))


def loss(c, Cimg, target, normal, y, rays, n, loss_out, dC, d_normal, d_y):
    _check(lib().neus2_loss(C.byref(c), _ptr(Cimg), _ptr(target), _ptr(normal), _ptr(y), rays, n, _ptr(loss_out),
                            _ptr(dC), _ptr(d_normal), _ptr(d_y), _stream()))


def workspace_bytes(c, n) -> int:
    return lib().neus2_workspace_bytes(C.byref(c), n)


def sdf_bwd_2nd(c, pos, tables, enc, jac, H, q, d_y, d_normal, n, dH, d_tables, d_enc, d_pos=None, workspace=None,
                masks=None):
    _check(lib().neus2_sdf_bwd_2nd(C.byref(c), _ptr(pos), _ptr(tables), _ptr(enc), _ptr(jac), _ptr_array(H),
                                   _ptr(q), _ptr(d_y), _ptr(d_normal), n, _ptr_array(dH), _ptr(d_tables),
                                   _ptr(d_enc), _ptr(d_pos), _ptr(workspace),
                                   workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                   _ptr(masks), _stream()))


def sdf_mlp_bwd(c, enc, jac, H, d_y, d_normal, n, dH, d_enc, d_pos=None, masks=None):
    _check(lib().neus2_sdf_mlp_bwd(C.byref(c), _ptr(enc), _ptr(jac), _ptr_array(H), _ptr(d_y), _ptr(d_normal), n,
                                   _ptr_array(dH), _ptr(d_enc), _ptr(d_pos), _ptr(masks), _stream()))


def _bytes(t) -> int:
    return t.numel() * t.element_size() if t is not None else 0


def sdf_deep_workspace_bytes(n_mats: int, n: int) -> int:
    return lib().neus2_sdf_deep_workspace_bytes(n_mats, n)


def sdf_deep_fwd_grad(enc_dim, enc, jac, H, n, y, q, normal, workspace):
    _check(lib().neus2_sdf_deep_fwd_grad(len(H), enc_dim, _ptr(enc), _ptr(jac), _ptr_array(H), n, _ptr(y), _ptr(q),
                                         _ptr(normal), _ptr(workspace), _bytes(workspace), _stream()))


def sdf_deep_bwd(enc_dim, enc, jac, H, d_y, d_normal, n, dH, d_enc, workspace):
    _check(lib().neus2_sdf_deep_bwd(len(H), enc_dim, _ptr(enc), _ptr(jac), _ptr_array(H), _ptr(d_y), _ptr(d_normal), n,
                                    _ptr_array(dH), _ptr(d_enc), _ptr(workspace), _bytes(workspace), _stream()))


def hash_scatter_bwd(c, pos, tables, q, d_enc, d_normal, n, d_tables, d_pos=None, workspace=None):
    _check(lib().neus2_hash_scatter_bwd(C.byref(c), _ptr(pos), _ptr(tables), _ptr(q), _ptr(d_enc), _ptr(d_normal),
                                        n, _ptr(d_tables), _ptr(d_pos), _ptr(workspace),
                                        workspace.numel() * workspace.element_size() if workspace is not None else 0,
                                        _stream()))


def hash_scatter_bwd_static(c, pos, tables, q, d_enc, d_normal, n, d_tables):
    _check(lib().neus2_hash_scatter_bwd_static(C.byref(c), _ptr(pos), _ptr(tables), _ptr(q), _ptr(d_enc), _ptr(d_normal),
                                               n, _ptr(d_tables), _stream()))


def adam_step(param, master, grad, m, v, dtype, lr, beta1, beta2, eps, t, zero_grad=True, lazy=False):
    _check(lib().neus2_adam_step(_ptr(param), _ptr(master), _ptr(grad), _ptr(m), _ptr(v), grad.numel(), dtype,
                                 lr, beta1, beta2, eps, t, (1 if zero_grad else 0) | (2 if lazy else 0), _stream()))


def adam_tables(c, tables, master, grad, m, v, lr, beta1, beta2, eps, t, zero_grad=True, lazy=False, active_levels_only=False):
    _check(lib().neus2_adam_tables(C.byref(c), _ptr(tables), _ptr(master), _ptr(grad), _ptr(m), _ptr(v),
                                   lr, beta1, beta2, eps, t,
                                   (1 if zero_grad else 0) | (2 if lazy else 0) | (4 if active_levels_only else 0), _stream()))


def adam_all(c, tables, master, grad, m, v, small, small_grad, small_m, small_v, lr, beta1, beta2, eps, t, zero_grad=True,
             lazy=False, active_levels_only=False):
    _check(lib().neus2_adam_all(C.byref(c), _ptr(tables), _ptr(master), _ptr(grad), _ptr(m), _ptr(v), _ptr(small),
                                _ptr(small_grad), _ptr(small_m), _ptr(small_v), small.numel(), lr, beta1, beta2, eps, t,
                                (1 if zero_grad else 0) | (2 if lazy else 0) | (4 if active_levels_only else 0), _stream()))


def rigid_fwd(pos, R, T, scale, offset, out):
    Ra = (C.c_float * 9)(*[float(x) for x in R])
    Ta = (C.c_float * 3)(*[float(x) for x in T])
    _check(lib().neus2_rigid_fwd(_ptr(pos), Ra, Ta, scale, offset, pos.shape[0], _ptr(out), _stream()))


def rigid_bwd(pos, T, d_out, scale, Mb):
    Ta = (C.c_float * 3)(*[float(x) for x in T])
    _check(lib().neus2_rigid_bwd(_ptr(pos), Ta, _ptr(d_out), scale, pos.shape[0], _ptr(Mb), _stream()))


def rigid_fwd_dev(pos, pose, scale, offset, out):
    _check(lib().neus2_rigid_fwd_dev(_ptr(pos), _ptr(pose), scale, offset, pos.shape[0], _ptr(out), _stream()))


def rigid_bwd_dev(pos, pose, d_out, scale, Mb):
    _check(lib().neus2_rigid_bwd_dev(_ptr(pos), _ptr(pose), _ptr(d_out), scale, pos.shape[0], _ptr(Mb), _stream()))


def pose_update(param, m, v, prev, Mb, pose, lr, beta1, beta2, eps, t, apply=True):
    _check(lib().neus2_pose_update(_ptr(param), _ptr(m), _ptr(v), _ptr(prev), _ptr(Mb), _ptr(pose), lr, beta1, beta2, eps, t,
                                   1 if apply else 0, _stream()))


def occupancy_points(log2_res, cells, jitter, pos):
    _check(lib().neus2_occupancy_points(log2_res, _ptr(cells), _ptr(jitter), cells.shape[0], _ptr(pos), _stream()))


def occupancy_update(log2_res, density, cells, sdf, sdf_stride, m, s, decay, threshold, bitfield, s_dev=None):
    _check(lib().neus2_occupancy_update(log2_res, _ptr(density), _ptr(cells), _ptr(sdf), sdf_stride, m, _ptr(s_dev),
                                        s, decay, threshold, _ptr(bitfield), _stream()))


def march_rays(log2_res, bitfield, origins, dirs, jitter, dt, max_steps, capacity, ray_offsets, pos, sample_ray, t=None):
    _check(lib().neus2_march_rays(log2_res, _ptr(bitfield), _ptr(origins), _ptr(dirs), _ptr(jitter), origins.shape[0],
                                  dt, max_steps, capacity, _ptr(ray_offsets), _ptr(pos), _ptr(sample_ray), _ptr(t),
                                  _stream()))


class Step:
    """All device buffers of one training step, allocated once with torch, plus the
    `neus2_step_buffers` struct that `train_step` hands to the library."""

    def __init__(self, cfg, params: Dict[str, object], n: int, want_pos_grad: bool = False, device="cuda",
                 use_workspace: bool = True, learn_s: bool = False, n_rays: Optional[int] = None,
                 keep_masks: bool = True):
        """`n_rays` given: rays have their own sample counts (set_batch then wants "ray_offsets"
        and "sample_ray"); otherwise n / samples_per_ray rays of equal length.  `keep_masks`: the
        forward kernels hand their ReLU masks to the backward kernels (16 bytes per sample and
        network) instead of the backward kernels working them out again."""
        import torch
        self.cfg, self.c, self.n = cfg, make_config(cfg), n
        L, F, T = cfg.n_levels, cfg.n_features, cfg.table_size
        self.ragged = n_rays is not None
        self.rays = n_rays if self.ragged else n // cfg.samples_per_ray
        f32 = dict(dtype=torch.float32, device=device)
        tdt = torch.float16 if cfg.table_dtype == "f16" else torch.float32
        self.tables = torch.as_tensor(params["tables"]).to(device=device, dtype=tdt).contiguous()
        # all matrices of both networks live in one flat buffer (one Adam launch covers them);
        # each matrix starts on a 16-byte boundary
        mats = [torch.as_tensor(m, dtype=torch.float32) for m in list(params["H"]) + list(params["W"])]
        offs, total = [], 0
        for m in mats:
            offs.append(total)
            total += (m.numel() + 3) // 4 * 4
        # a trained slope s of Phi_s sits behind the matrices: Adam updates it in the same launch
        s_off = total
        total += 4 if learn_s else 0
        self.small = torch.zeros(max(total, 4), **f32)
        self.d_small = torch.zeros_like(self.small)
        self.s_dev = self.small[s_off:s_off + 1] if learn_s else None
        self.d_s = self.d_small[s_off:s_off + 1] if learn_s else None
        if learn_s:
            self.s_dev.fill_(cfg.s)
        self.mat_slices = [(o, tuple(m.shape)) for o, m in zip(offs, mats)]     # where each matrix sits in the flat buffer
        views = [self.small[o:o + m.numel()].view(m.shape) for o, m in zip(offs, mats)]
        gviews = [self.d_small[o:o + m.numel()].view(m.shape) for o, m in zip(offs, mats)]
        for v, m in zip(views, mats):
            v.copy_(m)
        nH = len(params["H"])
        self.H, self.W = views[:nH], views[nH:]
        self.pos = torch.zeros(n, 3, **f32)
        self.dirs = torch.zeros(max(self.rays, 1), 3, **f32)
        self.target = torch.zeros(max(self.rays, 1), 3, **f32)
        z = lambda *shape: torch.zeros(*shape, **f32)
        self.enc, self.jac, self.q, self.d_enc = z(L, n, F), z(L, 3, n, F), z(L, n, F), z(L, n, F)
        self.y, self.d_y = z(n, 16), z(n, 16)
        self.normal, self.d_normal = z(n, 3), z(n, 3)
        self.rgb, self.d_rgb = z(n, 3), z(n, 3)
        self.C, self.dC = z(max(self.rays, 1), 3), z(max(self.rays, 1), 3)
        self.weights, self.d_sdf = z(n), z(n)
        self.loss = z(4)
        self.ray_offsets = torch.zeros(self.rays + 1, dtype=torch.int32, device=device) if self.ragged else None
        self.sample_ray = torch.zeros(max(n, 1), dtype=torch.int32, device=device) if self.ragged else None
        self.d_pos = z(n, 3) if want_pos_grad else None
        self.sdf_masks = torch.zeros(2, max(n, 1), 2, dtype=torch.int32, device=device) if keep_masks else None
        self.color_masks = torch.zeros(2, max(n, 1), 2, dtype=torch.int32, device=device) if keep_masks else None
        self.dH, self.dW = gviews[:nH], gviews[nH:]
        self.opt = None
        self.d_tables = z(L, T, F)
        ws = workspace_bytes(self.c, n) if use_workspace else 0
        self.workspace = torch.zeros(ws // 4, dtype=torch.int32, device=device) if ws > 0 else None
        self._H, self._W = _ptr_array(self.H), _ptr_array(self.W)
        self._dH, self._dW = _ptr_array(self.dH), _ptr_array(self.dW)
        b = Neus2StepBuffers()
        for name in ("pos", "dirs", "target", "tables", "enc", "jac", "y", "q", "normal", "rgb", "C", "weights",
                     "loss", "dC", "d_sdf", "d_rgb", "d_y", "d_normal", "d_enc", "d_pos", "d_tables", "workspace",
                     "s_dev", "d_s", "ray_offsets", "sample_ray", "sdf_masks", "color_masks"):
            setattr(b, name, _ptr(getattr(self, name)))
        b.H, b.W = C.cast(self._H, _P), C.cast(self._W, _P)
        b.dH, b.dW = C.cast(self._dH, _P), C.cast(self._dW, _P)
        b.workspace_bytes = ws if self.workspace is not None else 0
        b.n_rays = self.rays
        self.buffers = b

    def set_batch(self, batch: Dict[str, object]) -> None:
        import torch
        self.pos.copy_(torch.as_tensor(batch["pos"], dtype=torch.float32))
        if "dirs" in batch:
            self.dirs.copy_(torch.as_tensor(batch["dirs"], dtype=torch.float32))
            self.target.copy_(torch.as_tensor(batch["target"], dtype=torch.float32))
        if self.ragged:
            self.ray_offsets.copy_(torch.as_tensor(batch["ray_offsets"], dtype=torch.int32))
            if self.n > 0:
                self.sample_ray.copy_(torch.as_tensor(batch["sample_ray"], dtype=torch.int32))

    def bind_inputs(self, pos=None, dirs=None, target=None) -> None:
        """Point the step at other input tensors already on the device (another batch kept
        resident, a frame of a sequence) instead of copying into its own."""
        for name, t in (("pos", pos), ("dirs", dirs), ("target", target)):
            if t is not None:
                if t.shape != getattr(self, name).shape or t.dtype != getattr(self, name).dtype:
                    raise ValueError(f"{name}: shape or dtype differs from the step's")
                setattr(self, name, t)
                setattr(self.buffers, name, _ptr(t))

    def zero_grads(self) -> None:
        self.d_small.zero_()
        self.d_tables.zero_()

    def init_optimizer(self, lr=1e-2, beta1=0.9, beta2=0.99, eps=1e-15, lazy_tables=False) -> None:
        """Adam state: moments for tables and matrices, fp32 master copy of fp16 tables.
        `lazy_tables`: table entries whose gradient is zero in a step are left as they are."""
        import torch
        self.opt = {"lr": lr, "b1": beta1, "b2": beta2, "eps": eps, "t": 0, "lazy": lazy_tables,
                    "m_t": torch.zeros_like(self.d_tables), "v_t": torch.zeros_like(self.d_tables),
                    "m_s": torch.zeros_like(self.small), "v_s": torch.zeros_like(self.small),
                    "master": self.tables.float() if self.tables.dtype == torch.float16 else None}

    def adam(self) -> None:
        """One Adam step on every parameter; the gradient buffers are cleared in the same pass.
        Levels that have never been active (the progressive schedule only adds levels; the largest number of active
        levels a step or an update has seen is kept) have zero gradients and moments, so the dense update leaves
        them as they are: they are skipped."""
        o = self.opt
        o["t"] += 1
        self.most_active_levels = max(getattr(self, "most_active_levels", 0), self.c.active_levels)
        skip = self.c.active_levels >= self.most_active_levels
        adam_all(self.c, self.tables, o["master"], self.d_tables, o["m_t"], o["v_t"], self.small, self.d_small, o["m_s"],
                 o["v_s"], o["lr"], o["b1"], o["b2"], o["eps"], o["t"], True, o["lazy"], active_levels_only=skip)

    def train_step(self, n: Optional[int] = None) -> None:
        """`n` (at most the n the buffers were sized for) runs the step on the first n samples:
        what a ray marcher that filled part of the buffers wants.  Per-point arrays are laid
        out for that n, so every call of one step must be given the same value."""
        n = self.n if n is None else n
        if not 0 <= n <= self.n:
            raise ValueError(f"n = {n} outside 0..{self.n}")
        self.most_active_levels = max(getattr(self, "most_active_levels", 0), self.c.active_levels)
        _check(lib().neus2_train_step(C.byref(self.c), C.byref(self.buffers), n, _stream()))
