"""Host side of the occupancy grid (supplement Sec. E.3 "Ray Marching Acceleration"): owns the
grid's device buffers, draws the candidate cells of an update, and strings the library calls
together.  All arithmetic on the grid and on the rays runs in the library's kernels
(`neus2_occupancy_points`, `neus2_hash_encode`, `neus2_sdf_fwd_grad`, `neus2_occupancy_update`,
`neus2_march_rays`); this module only decides WHICH cells are looked at and WHEN.

The paper refreshes the grid "periodically" as the publication it cites does; that
publication's schedule is what `candidates` follows: during the first updates every cell is a
candidate; afterwards half of the candidates are drawn uniformly from all cells and half from
the cells whose bit is set.
"""
from __future__ import annotations

from . import binding as nb


class OccupancyGrid:
    def __init__(self, step: "nb.Step", log2_res: int = 6, decay: float = 0.95, threshold: float = 0.1,
                 warm_updates: int = 16, later_fraction: float = 0.5, device: str = "cuda"):
        """`step` supplies the configuration, the tables and the SDF matrices the grid is
        refreshed from.  Until the first update every cell counts as occupied."""
        import torch
        self.step, self.log2_res = step, log2_res
        self.n_cells = 1 << (3 * log2_res)
        self.decay, self.threshold = decay, threshold
        self.warm_updates, self.later_fraction = warm_updates, later_fraction
        self.updates = 0
        self.density = torch.zeros(self.n_cells, dtype=torch.float32, device=device)
        self.bitfield = torch.full((max(self.n_cells // 32, 4),), -1, dtype=torch.int32, device=device)
        self.m_max = self.n_cells
        cfg = step.cfg
        L, F = cfg.n_levels, cfg.n_features
        f32 = dict(dtype=torch.float32, device=device)
        self._all, self.last_cells = None, None
        self.jitter = torch.zeros(self.m_max, 3, **f32)
        self.pos = torch.zeros(self.m_max, 3, **f32)
        self.enc, self.jac = torch.zeros(L * self.m_max * F, **f32), torch.zeros(L * self.m_max * F * 3, **f32)
        self.y, self.q = torch.zeros(self.m_max, 16, **f32), torch.zeros(L * self.m_max * F, **f32)
        self.normal = torch.zeros(self.m_max, 3, **f32)

    def _bits(self):
        """bool [n_cells] on the grid's device, unpacked from the bitfield."""
        import torch
        words = self.bitfield[: self.n_cells // 32]
        shifts = torch.arange(32, dtype=torch.int32, device=words.device)
        return ((words[:, None] >> shifts) & 1).reshape(-1).bool()

    def candidates(self, gen=None):
        """Cell numbers (Morton order, int32 tensor on the grid's device) of the next update;
        `gen` is the torch generator the draws come from."""
        import torch
        dev = self.density.device
        if self.updates < self.warm_updates:
            if self._all is None:
                self._all = torch.arange(self.n_cells, dtype=torch.int32, device=dev)
            return self._all
        m = int(self.n_cells * self.later_fraction)
        uniform = torch.randint(0, self.n_cells, (m // 2,), generator=gen, device=dev, dtype=torch.int32)
        occupied = torch.nonzero(self._bits()).reshape(-1).to(torch.int32)
        if occupied.numel() == 0:
            return uniform
        pick = torch.randint(0, occupied.numel(), (m - m // 2,), generator=gen, device=dev)
        return torch.cat([uniform, occupied[pick]])

    def update(self, gen=None, cells=None) -> int:
        """One refresh from the current SDF; the candidate cells and the point inside each are
        drawn on the device from `gen`.  Returns the number of candidate cells."""
        import torch
        step = self.step
        cells = self.candidates(gen) if cells is None else cells.to(device=self.density.device, dtype=torch.int32).contiguous()
        m = int(cells.numel())
        if m > self.m_max:
            raise ValueError(f"{m} candidate cells, room for {self.m_max}")
        if m:
            jitter = self.jitter[:m]
            torch.rand(m, 3, generator=gen, out=jitter)
            jitter.clamp_(max=1.0 - 2.0 ** -24)
            pos_m = self.pos[:m]
            nb.occupancy_points(self.log2_res, cells, jitter, pos_m)
            nb.hash_encode(step.c, pos_m, step.tables, self.enc, self.jac)
            nb.sdf_fwd_grad(step.c, self.enc, self.jac, step.H, m, self.y, self.q, self.normal)
        nb.occupancy_update(self.log2_res, self.density, cells if m else None, self.y if m else None, 16, m,
                            float(step.cfg.s), self.decay, self.threshold, self.bitfield, s_dev=step.s_dev)
        self.last_cells = cells
        self.updates += 1
        return m

    def march(self, origins, dirs, jitter, dt: float, max_steps: int, t=None) -> int:
        """Fills the step's pos / ray_offsets / sample_ray from the rays (device tensors, unit-cube
        coordinates) and returns the number of samples found (one 4-byte read-back: the host
        has to know n to size the launches of the step)."""
        step = self.step
        if not step.ragged:
            raise ValueError("the step must be built for rays of unequal length (n_rays=...)")
        nb.march_rays(self.log2_res, self.bitfield, origins, dirs, jitter, dt, max_steps, step.n,
                      step.ray_offsets, step.pos, step.sample_ray, t)
        return int(step.ray_offsets[-1].item())

    def occupied_fraction(self) -> float:
        return float(self._bits().float().mean().item())
