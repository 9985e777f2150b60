"""Host-side schedules (Sec. 4.3; supplement Sec. E.3)."""
from paper_2212_05231_amd import schedule


def test_progressive_levels_start_at_two_and_grow_every_2_5_percent():
    total, L = 15000, 16                       # the static-scene run of the paper: 15k iterations
    lam = [schedule.active_levels(i, total, L) for i in range(total)]
    assert lam[0] == 2 and lam[374] == 2 and lam[375] == 3 and lam[749] == 3 and lam[750] == 4
    assert all(b - a in (0, 1) for a, b in zip(lam, lam[1:]))
    assert lam.index(16) == 375 * 14 and lam[-1] == 16          # all 16 levels after 35 % of the run
    assert schedule.active_levels(10, 0, 8) == 8
    assert schedule.active_levels(5, 10, 4) <= 4


def test_dynamic_frame_phases():
    phases = [schedule.dynamic_frame_phase(i) for i in range(1100)]
    assert phases.count("transform") == 100 and phases[:100] == ["transform"] * 100 and phases[100] == "joint"
