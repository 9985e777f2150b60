"""Frame loop of a dynamic scene (Sec. 5 of the paper; training schedule of supplement Sec. E.3).

Every frame brings its own rays.  Hash tables, both networks and their Adam state are carried
over from frame to frame (incremental training); the frame's global transform (Eq. 9) is six
trained parameters (omega, T) that start from a given estimate, are optimised alone for the first
iterations of the frame and jointly with everything else afterwards, and are folded into the
accumulated transform (R^c, T^c of Eq. 10) when the next frame begins.

This module only orders calls of the library: all state, including the transform's parameters,
their moments and the accumulated transform, lives in device memory, and nothing is read back
inside the loop.
"""
from __future__ import annotations

from typing import Callable, Optional

from . import binding as nb
from . import schedule

SCALE, OFFSET = 0.5, 0.5          # world cube [-1,1]^3 -> unit cube


class DynamicSequence:
    def __init__(self, cfg, params, n: int, lr: float = 1e-2, pose_lr: float = 1e-3, transform_only: int = 100,
                 beta1: float = 0.9, beta2: float = 0.99, eps: float = 1e-15, device="cuda"):
        import torch
        self.step = nb.Step(cfg, params, n, want_pos_grad=True, device=device)
        self.step.zero_grads()
        self.step.init_optimizer(lr=lr, beta1=beta1, beta2=beta2, eps=eps)
        self.pose_lr, self.transform_only = pose_lr, transform_only
        # one allocation, every part on a 16-byte boundary
        self.state = torch.zeros(64, dtype=torch.float32, device=device)
        self.param, self.m, self.v = self.state[0:6], self.state[8:14], self.state[16:22]
        self.prev, self.pose, self.Mb = self.state[24:36], self.state[36:48], self.state[48:60]
        self.prev[0] = self.prev[4] = self.prev[8] = 1.0            # identity: the first frame is the canonical one
        self.world = None
        self.frame, self.iteration, self.t_pose = -1, 0, 0

    def begin_frame(self, world_pos, dirs, target, omega, shift) -> None:
        """`world_pos` [n,3], `dirs`, `target` [rays,3]: device tensors of the new frame (world
        coordinates); `omega`, `shift`: the estimate the frame's transform starts from."""
        import torch
        if self.frame >= 0:
            self.prev.copy_(self.pose)                               # R^c_i = R^c_{i-1} R_i, T^c_i = T_i + R_i^{-1} T^c_{i-1}
        self.frame += 1
        self.iteration, self.t_pose = 0, 0
        self.world = world_pos
        self.step.bind_inputs(dirs=dirs, target=target)
        self.param.copy_(torch.as_tensor([*omega, *shift], dtype=torch.float32))
        self.m.zero_()
        self.v.zero_()
        nb.pose_update(self.param, None, None, self.prev, self.Mb, self.pose, 0.0, 0.0, 0.0, 0.0, 1, apply=False)

    def phase(self) -> str:
        """'transform' while only the frame's transform is optimised (not in the first frame,
        which has nothing to start from), then 'joint'."""
        return "joint" if self.frame == 0 else schedule.dynamic_frame_phase(self.iteration, self.transform_only)

    def iterate(self, probe: Optional[Callable[["DynamicSequence"], None]] = None) -> str:
        """One training iteration of the current frame; returns its phase.  `probe` is called
        between the backward pass and the parameter updates (tests look at the gradients there)."""
        s, o = self.step, self.step.opt
        phase = self.phase()
        nb.rigid_fwd_dev(self.world, self.pose, SCALE, OFFSET, s.pos)
        s.train_step()
        nb.rigid_bwd_dev(self.world, self.pose, s.d_pos, SCALE, self.Mb)
        if probe is not None:
            probe(self)
        self.t_pose += 1
        nb.pose_update(self.param, self.m, self.v, self.prev, self.Mb, self.pose, self.pose_lr, o["b1"], o["b2"], o["eps"],
                       self.t_pose, apply=True)
        if phase == "joint":
            s.adam()
        else:
            s.zero_grads()
        self.iteration += 1
        return phase
