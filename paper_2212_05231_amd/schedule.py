"""Host-side schedules of the training loop (no arithmetic of the step itself).

Sec. 4.3 of the paper: the level mask w_i(lambda) = [i <= lambda] starts at lambda = 2 and
grows by one level every 2.5 % of the total training steps.  Supplement Sec. E.3: a frame of a
dynamic scene is trained for 1.1k iterations, of which the first 100 optimise the global
transformation alone.
"""
from __future__ import annotations


def active_levels(step: int, total_steps: int, n_levels: int, start: int = 2, every: float = 0.025) -> int:
    """lambda for 0-based iteration `step` of `total_steps`."""
    if total_steps <= 0:
        return n_levels
    period = max(int(round(every * total_steps)), 1)
    return max(1, min(n_levels, start + step // period))


def dynamic_frame_phase(step: int, transform_only: int = 100) -> str:
    """'transform' while only the rigid transform of a new frame is optimised, then 'joint'."""
    return "transform" if step < transform_only else "joint"
