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


def test_step_leaves_levels_out_of_the_optimiser_only_while_they_were_never_active(monkeypatch):
    """The binding's Step passes NEUS2_ADAM_ACTIVE_LEVELS while the schedule has only added levels (Sec. 4.3):
    once a larger number of levels has been active, those levels hold gradients and moments and every level
    is updated again.  Host logic only: the library call is replaced by a recorder."""
    import types
    from paper_2212_05231_amd import binding as nb
    seen = []
    monkeypatch.setattr(nb, "adam_all", lambda *a, **k: seen.append(k["active_levels_only"]))
    step = object.__new__(nb.Step)
    step.c = types.SimpleNamespace(active_levels=4)
    step.opt = {"t": 0, "master": None, "m_t": None, "v_t": None, "m_s": None, "v_s": None, "lr": 1e-2, "b1": 0.9,
                "b2": 0.99, "eps": 1e-15, "lazy": False}
    step.tables = step.d_tables = step.small = step.d_small = None
    for levels in (4, 6, 6, 3, 6, 8, 7):
        step.c.active_levels = levels
        step.adam()
    assert seen == [True, True, True, False, True, True, False]
    assert step.opt["t"] == 7
