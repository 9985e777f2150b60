"""Second-order backward of the SDF network: this library against torch.autograd's double
backward (the comparison of the paper's Fig. 7, "speed-up of our 2nd-order derivative over
PyTorch across MLP layer numbers and batch sizes").

    python -m paper_2212_05231_amd.ablation [--log2-min 14] [--log2-max 20] [--reps 20]

Both sides compute, for a batch of encodings e [n, 32] with Jacobians J = de/dx [n, 32, 3]:
    (d, g) = f(e),  q = dd/de,  normal = q J,
    loss = mean(d^2) + beta * mean((|normal| - 1)^2),
and the gradient of the loss with respect to every matrix of f (which needs the second-order
term of Theorem 1 because the loss depends on normal) and with respect to e.
The library runs neus2_sdf_fwd_grad + neus2_loss + neus2_sdf_mlp_bwd (the fused kernels of the
training step: 1 and 2 hidden layers of 64) or, for the figure's deeper networks (4 and 8 hidden
layers), neus2_sdf_deep_fwd_grad + neus2_loss + neus2_sdf_deep_bwd (one launch per matrix and
direction); PyTorch runs the same network with autograd.grad(create_graph=True) for q and
.backward() for the rest.  Prints one line per case and a JSON summary; the gradients of the two
sides are compared as a sanity check (the parity tests proper are against the float64 oracle).
"""
from __future__ import annotations

import argparse
import json

import numpy as np


def make_case(hidden: int, n: int, beta: float = 0.1, seed: int = 7, layer_by_layer=None):
    """One case of the comparison: the network (hidden layers of 64), a batch of n encodings and
    Jacobians, and the two ways to compute the gradients.  Returns a dict with the inputs
    (`H`, `e`, `J`), `ours()` -> (dH list, d_enc [n,32]) and `theirs()` -> (dH list, d_enc [n,32]).
    `layer_by_layer`: which of the library's two paths runs; default: the fused kernels where they
    exist (up to two hidden layers)."""
    import torch
    from . import binding as nb, workloads as wl
    dev = "cuda"
    if layer_by_layer is None:
        layer_by_layer = hidden > 2
    cfg = wl.make_config(1)
    cfg.sdf_dims = [32] + [64] * min(hidden, 2) + [16]          # the descriptor only serves the fused path and the loss
    cfg.n_levels, cfg.active_levels = 16, 16
    cfg.res, cfg.dense = wl.make_config(2).res, wl.make_config(2).dense
    cfg.log2_table_size = wl.make_config(2).log2_table_size
    cfg.loss_kind, cfg.beta = 0, beta
    c = nb.make_config(cfg)
    g = torch.Generator(device="cpu").manual_seed(seed + hidden)
    dims = [32] + [64] * hidden + [16]
    Hs = [(torch.randn(dims[i + 1], dims[i], generator=g) * (2.0 / dims[i]) ** 0.5).to(dev) for i in range(hidden + 1)]
    e = torch.randn(n, 32, generator=g).to(dev)
    J = (torch.randn(n, 32, 3, generator=g) * 0.3).to(dev)
    # library layout: level-major [L][n][F]; the Jacobian as three planes of pairs per level
    enc = e.view(n, 16, 2).permute(1, 0, 2).contiguous()
    jac = J.view(n, 16, 3, 2).permute(1, 2, 0, 3).contiguous()      # the library's [L][3 pairs][n][2]
    y = torch.empty(n, 16, device=dev); q = torch.empty(16, n, 2, device=dev); normal = torch.empty(n, 3, device=dev)
    loss = torch.zeros(4, device=dev); d_y = torch.empty(n, 16, device=dev); d_normal = torch.empty(n, 3, device=dev)
    d_enc = torch.empty(16, n, 2, device=dev)
    kept = torch.zeros(2, n, 2, dtype=torch.int32, device=dev)      # ReLU masks, forward -> backward
    dH = [torch.zeros_like(h) for h in Hs]
    ws = torch.empty(nb.sdf_deep_workspace_bytes(len(Hs), n), dtype=torch.uint8, device=dev) if layer_by_layer else None

    def ours():
        if layer_by_layer:
            nb.sdf_deep_fwd_grad(32, enc, jac, Hs, n, y, q, normal, ws)
            nb.loss(c, None, None, normal, y, 0, n, loss, None, d_normal, d_y)
            nb.sdf_deep_bwd(32, enc, jac, Hs, d_y, d_normal, n, dH, d_enc, ws)
        else:
            nb.sdf_fwd_grad(c, enc, jac, Hs, n, y, q, normal, masks=kept)
            nb.loss(c, None, None, normal, y, 0, n, loss, None, d_normal, d_y)
            nb.sdf_mlp_bwd(c, enc, jac, Hs, d_y, d_normal, n, dH, d_enc, masks=kept)
        return dH, d_enc.permute(1, 0, 2).reshape(n, 32)

    params = [h.clone().requires_grad_(True) for h in Hs]

    def theirs():
        for p in params:
            p.grad = None
        x = e.detach().requires_grad_(True)
        a = x
        for l, h in enumerate(params):
            a = a @ h.t()
            if l < len(params) - 1:
                a = torch.relu(a)
        d = a[:, 0]
        (qq,) = torch.autograd.grad(d.sum(), x, create_graph=True)
        nrm = torch.einsum("nk,nkc->nc", qq, J)
        ls = (d * d).mean() + beta * ((nrm.norm(dim=1) - 1.0) ** 2).mean()
        ls.backward()
        return [p.grad for p in params], x.grad

    return {"H": Hs, "e": e, "J": J, "beta": beta, "ours": ours, "theirs": theirs, "dH": dH,
            "path": "layer by layer" if layer_by_layer else "fused"}


def run(log2_min: int, log2_max: int, reps: int, beta: float = 0.1):
    import torch
    out = []
    for hidden, layered in ((1, False), (2, False), (2, True), (4, True), (8, True)):
        for lg in range(log2_min, log2_max + 1):
            n = 1 << lg
            case = make_case(hidden, n, beta, layer_by_layer=layered)
            ours, theirs = case["ours"], case["theirs"]

            def timed(fn):
                for _ in range(3):
                    fn()
                torch.cuda.synchronize()
                t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                t0.record()
                for _ in range(reps):
                    fn()
                t1.record()
                torch.cuda.synchronize()
                return t0.elapsed_time(t1) / reps

            for h in case["dH"]:
                h.zero_()
            dH, gx_ours = ours()
            gH, gx = theirs()
            torch.cuda.synchronize()
            err = max(float((a - b).norm() / b.norm()) for a, b in zip(dH, gH))
            err_x = float((gx_ours - gx).norm() / gx.norm())
            t_ours, t_torch = timed(ours), timed(theirs)
            row = {"hidden_layers": hidden, "path": case["path"], "batch": n, "ours_ms": round(t_ours, 4), "autograd_ms": round(t_torch, 4),
                   "speedup": round(t_torch / t_ours, 2), "grad_rel_diff": err, "input_grad_rel_diff": err_x}
            print(f"hidden {hidden} ({case['path']:14s})  batch 2^{lg:<2d}  ours {t_ours:8.3f} ms   autograd {t_torch:8.3f} ms   speed-up {t_torch / t_ours:6.2f}x   "
                  f"grad diff {err:.1e} / {err_x:.1e}", flush=True)
            out.append(row)
    return out


def main() -> None:
    ap = argparse.ArgumentParser()
    ap.add_argument("--log2-min", type=int, default=14)
    ap.add_argument("--log2-max", type=int, default=20)
    ap.add_argument("--reps", type=int, default=20)
    a = ap.parse_args()
    rows = run(a.log2_min, a.log2_max, a.reps)
    print(json.dumps({"ablation": "second-order backward vs torch.autograd double backward", "rows": rows}))


if __name__ == "__main__":
    main()
