"""The 20-frame dynamic sequence (Sec. 5, Eqs. 9-10; schedule of supplement Sec. E.3) on the GPU
against the oracle: tables, networks and Adam state carried from frame to frame, the frame's
transform as six trained parameters, transform-only iterations at the start of a frame, the
accumulated transform.

A ReLU mask is a decision taken from a floating-point value.  A pre-activation within rounding of
zero can fall on different sides in the kernels' arithmetic and in float64; the unit's weight then
enters or leaves dd/de, which moves that one point's normal by about a percent, and through it the
ray's colour and every sum over points.  At a thousand points a single such point is visible in
the sums at the 1e-4 bar.  The masks the kernels used are available (they hand them from the
forward to the backward kernels), so the test finds such points exactly: rays that hold one are
left out of the per-sample comparisons, and an iteration that has one is left out of the
comparisons of sums; most checked iterations, and one in each of the frames 0, 1 and 19, must be
free of them.

Two kinds of comparison.  (1) Iteration by iteration from the same state: before a checked
iteration the GPU's whole state is downloaded, the oracle performs the iteration from it, and
every stage is compared at its own bar (positions 1e-6, step outputs and gradients 1e-4, Adam
on the GPU's own gradients 1e-6).  Frames 0, 1 and 19, both phases.  (2) Free running: the
oracle trains the same 20 frames with its own Adam from the same start; losses and transforms of
the two runs are compared at a looser, stated bar, because Adam divides by the gradient's
magnitude: a gradient entry within rounding of zero moves its parameter by the full learning
rate in either direction, and such entries exist in every step.
"""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import neus2_oracle as o
from paper_2212_05231_amd import binding as nb
from paper_2212_05231_amd import sequence
from paper_2212_05231_amd import workloads as wl

pytestmark = pytest.mark.gpu

FWD_TOL, GRAD_TOL = 1e-5, 1e-4
LR, POSE_LR = 1e-2, 1e-3
FRAMES, ITERS, TRANSFORM_ONLY, RAYS = 20, 3, 1, 16


def rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    den = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / den) if den > 0 else float(np.linalg.norm(a))


def f64(t):
    return t.detach().cpu().numpy().astype(np.float64)


def lm(t, n):
    return np.transpose(f64(t), (1, 0, 2)).reshape(n, -1)


def flipped_points(step, out, n):
    """Points at which a ReLU mask of either network differs between the GPU and the oracle."""
    from test_gpu_parity import decode_masks
    bad = np.zeros(n, dtype=bool)
    for words, want in ((step.sdf_masks, out["masks"]), (step.color_masks, out["cmasks"])):
        for got_m, want_m in zip(decode_masks(words, n, len(want)), want):
            bad |= np.any(got_m != (want_m > 0), axis=1)
    return bad


def make_problem(table_scale=2000.0, active_levels=None):
    w = wl.make_workload(5, n_rays=RAYS)
    cfg, params = w["cfg"], w["params"]
    if active_levels is not None:
        cfg.active_levels = active_levels
    params["tables"] = (params["tables"].astype(np.float64) * table_scale).astype(np.float16)
    frames = [wl.make_workload(5, n_rays=RAYS, frame=f)["batch"] for f in range(FRAMES)]
    return cfg, params, frames


def snapshot(seq):
    """The GPU's state in the oracle's terms."""
    s, op = seq.step, seq.step.opt
    nH = len(s.H)
    mats = lambda flat: [f64(flat[a:a + int(np.prod(sh))]).reshape(sh) for a, sh in s.mat_slices]
    small, ms, vs = mats(s.small), mats(op["m_s"]), mats(op["v_s"])
    params = {"tables": s.tables.cpu().numpy(), "master": f64(op["master"]),
              "H": [m.astype(np.float32) for m in small[:nH]], "W": [m.astype(np.float32) for m in small[nH:]]}
    opt = {"t": op["t"], "m_tables": f64(op["m_t"]), "v_tables": f64(op["v_t"]),
           "m_H": ms[:nH], "v_H": vs[:nH], "m_W": ms[nH:], "v_W": vs[nH:]}
    st = f64(seq.state)
    pose = {"omega": st[0:3], "T": st[3:6], "m": st[8:14], "v": st[16:22], "t": seq.t_pose,
            "R_prev": st[24:33].reshape(3, 3), "T_prev": st[33:36], "Rc": st[36:45].reshape(3, 3), "Tc": st[45:48]}
    return params, opt, pose


def upload_frame(batch):
    dev = lambda a: torch.as_tensor(np.ascontiguousarray(a), dtype=torch.float32).cuda()
    return dev(batch["pos"]), dev(batch["dirs"]), dev(batch["target"])


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    nb.lib()


def test_sequence_iteration_by_iteration_from_the_same_state():
    cfg, params, frames = make_problem()
    n = frames[0]["pos"].shape[0]
    seq = sequence.DynamicSequence(cfg, params, n, lr=LR, pose_lr=POSE_LR, transform_only=TRANSFORM_ONLY)
    checked = {(0, 0), (0, 1), (0, 2), (1, 0), (1, 1), (1, 2), (10, 0), (19, 0), (19, 1), (19, 2)}
    seen_phases = set()
    clean_iterations = []
    for f in range(FRAMES):
        world, dirs, target = upload_frame(frames[f])
        end_of_last = snapshot(seq)[2] if f > 0 else None
        seq.begin_frame(world, dirs, target, frames[f]["omega"], frames[f]["shift"])
        _, _, pose0 = snapshot(seq)
        if f > 0:
            # the transform accumulated so far is what the last frame ended with (text after Eq. 10)
            np.testing.assert_array_equal(pose0["R_prev"], end_of_last["Rc"])
            np.testing.assert_array_equal(pose0["T_prev"], end_of_last["Tc"])
            Rc, Tc = o.accumulate_transform(end_of_last["R_prev"], end_of_last["T_prev"],
                                            o.rotation_from_axis_angle(end_of_last["omega"]), end_of_last["T"])
            np.testing.assert_allclose(pose0["R_prev"], Rc, atol=2e-7)
            np.testing.assert_allclose(pose0["T_prev"], Tc, atol=2e-7)
        np.testing.assert_allclose(pose0["omega"], frames[f]["omega"], rtol=1e-6, atol=1e-9)
        for it in range(ITERS):
            if (f, it) not in checked:
                seq.iterate()
                continue
            before_params, before_opt, before_pose = snapshot(seq)
            got = {}

            def probe(sq):
                st = sq.step
                got.update(pos=st.pos.cpu().numpy(), d_pos=f64(st.d_pos), d_tables=f64(st.d_tables), d_small=f64(st.d_small),
                           Mb=f64(sq.Mb), loss=f64(st.loss), y=f64(st.y), C=f64(st.C), normal=f64(st.normal))
            phase = seq.iterate(probe)
            seen_phases.add((f > 0, phase))
            assert phase == ("transform" if f > 0 and it < TRANSFORM_ONLY else "joint")
            after_params, after_opt, after_pose = snapshot(seq)
            new_params, new_opt, new_pose, out = o.dynamic_frame_iteration(
                cfg, before_params, before_opt, before_pose, frames[f], phase == "joint", LR, POSE_LR, pos_override=got["pos"])
            # --- Eq. 9 through the accumulated transform
            want_pos = o.frame_to_canonical(frames[f]["pos"], before_pose["omega"], before_pose["T"], before_pose["R_prev"],
                                            before_pose["T_prev"]) * 0.5 + 0.5
            assert rel(got["pos"], want_pos) <= 1e-6
            # --- the step on those positions; rays with a point whose mask differs are set aside
            spr = cfg.samples_per_ray
            bad_pts = flipped_points(seq.step, out, n)
            bad_rays = np.any(bad_pts.reshape(-1, spr), axis=1)
            ok_rays = ~bad_rays
            ok = np.repeat(ok_rays, spr)
            assert bad_pts.sum() <= 3 and ok_rays.sum() >= RAYS - 3
            assert rel(got["y"][ok], out["y"][ok]) <= FWD_TOL and rel(got["normal"][ok], out["normal"][ok]) <= FWD_TOL
            assert rel(got["C"][ok_rays], out["C"][ok_rays]) <= FWD_TOL
            assert np.linalg.norm(out["dpos"]) > 0 and rel(got["d_pos"][ok], out["dpos"][ok]) <= GRAD_TOL
            clean = not bad_pts.any()
            clean_iterations.append((f, it, phase, clean))
            s = seq.step
            nH = len(s.H)
            if clean:
                assert abs(got["loss"][0] + got["loss"][1] - out["loss"]) <= FWD_TOL * abs(out["loss"])
                assert rel(got["d_tables"], out["dtables"]) <= GRAD_TOL
                for k, (a, sh) in enumerate(s.mat_slices):
                    want_g = (out["dH"] + out["dW"])[k]
                    assert rel(got["d_small"][a:a + want_g.size].reshape(sh), want_g) <= GRAD_TOL, k
                # --- the reductions and the gradient of the six parameters (seen through Adam's first moment)
                M, _, b = o.rigid_backward(frames[f]["pos"], before_pose["Rc"], before_pose["Tc"], out["dpos"], 0.5)
                assert rel(got["Mb"][:9].reshape(3, 3), M) <= GRAD_TOL and rel(got["Mb"][9:], b) <= GRAD_TOL
                assert rel(after_pose["m"], new_pose["m"]) <= GRAD_TOL, (after_pose["m"], new_pose["m"])
                assert rel(after_pose["v"], new_pose["v"]) <= 2 * GRAD_TOL
                # the parameters: Adam's step is lr * mhat / sqrt(vhat), a gradient error of 1e-4 moves it by about 1e-4 lr
                want_p = np.concatenate([new_pose["omega"], new_pose["T"]])
                got_p = np.concatenate([after_pose["omega"], after_pose["T"]])
                np.testing.assert_allclose(got_p, want_p, atol=1e-3 * POSE_LR + 1e-7)
            # the reductions from the GPU's own position gradient, and the six parameters from them: always
            M, _, b = o.rigid_backward(frames[f]["pos"], before_pose["Rc"], before_pose["Tc"], got["d_pos"], 0.5)
            assert rel(got["Mb"][:9].reshape(3, 3), M) <= GRAD_TOL and rel(got["Mb"][9:], b) <= GRAD_TOL
            R_now = o.rotation_from_axis_angle(before_pose["omega"])
            G = before_pose["R_prev"].T @ (M - np.outer(b, R_now.T @ before_pose["T_prev"]))
            d_pose = np.concatenate([o.axis_angle_gradient(before_pose["omega"], G), before_pose["Rc"].T @ b])
            p6, m6, v6 = o.adam_step(np.concatenate([before_pose["omega"], before_pose["T"]]), d_pose, before_pose["m"],
                                     before_pose["v"], before_pose["t"] + 1, POSE_LR, 0.9, 0.99, 1e-15)
            assert rel(after_pose["m"], m6) <= GRAD_TOL and rel(after_pose["v"], v6) <= 2 * GRAD_TOL
            np.testing.assert_allclose(np.concatenate([after_pose["omega"], after_pose["T"]]), p6, atol=1e-3 * POSE_LR + 1e-7)
            assert after_pose["t"] == before_pose["t"] + 1
            # the composed transform the next iteration applies
            Rc, Tc = o.accumulate_transform(before_pose["R_prev"], before_pose["T_prev"],
                                            o.rotation_from_axis_angle(after_pose["omega"]), after_pose["T"])
            np.testing.assert_allclose(after_pose["Rc"], Rc, atol=2e-7)
            np.testing.assert_allclose(after_pose["Tc"], Tc, atol=2e-7)
            assert float(seq.Mb.abs().sum()) == 0.0
            if phase == "transform":
                # nothing but the transform moved; no gradient is left behind
                assert np.array_equal(after_params["master"], before_params["master"])
                assert np.array_equal(after_params["tables"], before_params["tables"])
                for a, b2 in zip(after_params["H"] + after_params["W"], before_params["H"] + before_params["W"]):
                    assert np.array_equal(a, b2)
                assert after_opt["t"] == before_opt["t"]
                assert float(s.d_tables.abs().sum()) == 0.0 and float(s.d_small.abs().sum()) == 0.0
            else:
                # Adam on the gradients the GPU itself produced, carried state included
                assert after_opt["t"] == before_opt["t"] + 1
                pr, mr, vr = o.adam_step(before_params["master"], got["d_tables"], before_opt["m_tables"], before_opt["v_tables"],
                                         after_opt["t"], LR, 0.9, 0.99, 1e-15)
                assert rel(after_params["master"], pr) <= 1e-6 and rel(after_opt["m_tables"], mr) <= 1e-6
                assert rel(after_opt["v_tables"], vr) <= 1e-6
                assert np.array_equal(after_params["tables"], after_params["master"].astype(np.float32).astype(np.float16))
                # and against the oracle's own update from its own gradients: equal but for entries whose
                # gradient is within rounding of zero (their step has the other sign)
                if clean:
                    step_err = np.abs(after_params["master"] - new_params["master"])
                    assert np.mean(step_err > 1e-3 * LR) <= 1e-3, float(np.mean(step_err > 1e-3 * LR))
                    for a, b2 in zip(after_params["H"] + after_params["W"], new_params["H"] + new_params["W"]):
                        assert np.mean(np.abs(a - b2) > 1e-3 * LR) <= 2e-3
                assert float(s.d_tables.abs().sum()) == 0.0 and float(s.d_small.abs().sum()) == 0.0
    assert seen_phases == {(False, "joint"), (True, "transform"), (True, "joint")}
    print("checked iterations (frame, iteration, phase, free of mask differences):", clean_iterations)
    assert sum(c for _, _, _, c in clean_iterations) >= len(clean_iterations) - 3
    for frame in (0, 1, 19):
        assert any(c for f2, _, ph, c in clean_iterations if f2 == frame and ph == "joint"), frame
    assert after_opt["t"] == ITERS + (FRAMES - 1) * (ITERS - TRANSFORM_ONLY)      # carried over all frames


@pytest.mark.parametrize("LR,POSE_LR", [(1e-3, 1e-4)])
def test_sequence_free_running_against_the_oracle(LR, POSE_LR):
    """Both sides train all 20 frames on their own, each transforming the frames' points itself
    (the GPU in binary32, the oracle in float64 rounded to binary32: a point's offset inside its
    cell differs by up to res * 2^-24 between them, which is why the eight coarsest levels are
    used here, and the differences then grow from iteration to iteration through Adam).  Stated
    bar: losses within 2 % of each other in every iteration, final accumulated rotation and
    translation within 2e-3."""
    cfg, params, frames = make_problem(table_scale=300.0, active_levels=8)
    n = frames[0]["pos"].shape[0]
    seq = sequence.DynamicSequence(cfg, params, n, lr=LR, pose_lr=POSE_LR, transform_only=TRANSFORM_ONLY)
    op = {"tables": params["tables"], "master": params["tables"].astype(np.float64), "H": params["H"], "W": params["W"]}
    zeros = lambda mats: [np.zeros(m.shape) for m in mats]
    oopt = {"t": 0, "m_tables": np.zeros(params["tables"].shape), "v_tables": np.zeros(params["tables"].shape),
            "m_H": zeros(params["H"]), "v_H": zeros(params["H"]), "m_W": zeros(params["W"]), "v_W": zeros(params["W"])}
    R_prev, T_prev = np.eye(3), np.zeros(3)
    gpu_losses, ref_losses = [], []
    loss_dev = []
    for f in range(FRAMES):
        world, dirs, target = upload_frame(frames[f])
        seq.begin_frame(world, dirs, target, frames[f]["omega"], frames[f]["shift"])
        opose = {"omega": np.asarray(frames[f]["omega"], dtype=np.float32).astype(np.float64),
                 "T": np.asarray(frames[f]["shift"], dtype=np.float32).astype(np.float64),
                 "m": np.zeros(6), "v": np.zeros(6), "t": 0, "R_prev": R_prev, "T_prev": T_prev}
        for it in range(ITERS):
            seq.iterate(lambda sq: loss_dev.append(sq.step.loss.clone()))
            joint = f == 0 or it >= TRANSFORM_ONLY
            op, oopt, opose, out = o.dynamic_frame_iteration(cfg, op, oopt, opose, frames[f], joint, LR, POSE_LR)
            ref_losses.append(out["loss"])
        R_prev, T_prev = o.accumulate_transform(R_prev, T_prev, o.rotation_from_axis_angle(opose["omega"]), opose["T"])
    torch.cuda.synchronize()
    gpu_losses = [float(l[0] + l[1]) for l in loss_dev]
    dev = np.abs(np.array(gpu_losses) - np.array(ref_losses)) / np.array(ref_losses)
    print("largest relative loss deviation", dev.max(), "losses", gpu_losses[:3], gpu_losses[-3:])
    print("deviation by iteration", [float(f"{d:.1e}") for d in dev])
    assert dev.max() <= 2e-2
    st = f64(seq.state)
    print("accumulated transform deviation", np.abs(st[36:45].reshape(3, 3) - R_prev).max(), np.abs(st[45:48] - T_prev).max())
    np.testing.assert_allclose(st[36:45].reshape(3, 3), R_prev, atol=2e-3)
    np.testing.assert_allclose(st[45:48], T_prev, atol=2e-3)
    # the networks were trained, not only replayed: the loss of the last frames is below the first frame's first
    assert np.mean(gpu_losses[-ITERS:]) < gpu_losses[0]
