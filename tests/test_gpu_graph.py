"""neus2_train_step recorded into a HIP graph and replayed.

The library launches kernels only (every clear is a kernel, nothing is allocated, nothing waits for the
stream), so a caller may record a step once and replay it.  A replayed step must do what the eager step
does: forward outputs bit for bit (those kernels have no atomics), gradients up to the order of their
atomic additions.  The graph is replayed several times with eager work and synchronisations in between,
and every replay is checked, not just the first."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from paper_2212_05231_amd import binding as nb, workloads as wl

pytestmark = pytest.mark.gpu


def rel(a, b):
    a, b = a.double(), b.double()
    return float((a - b).norm() / b.norm())


@pytest.mark.parametrize("k,n_rays", [(1, 4096), (2, 1024 + 5)])
def test_replayed_step_equals_the_eager_step(k, n_rays):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    w = wl.make_workload(k, n_rays=n_rays)
    cfg, params, batch = w["cfg"], w["params"], w["batch"]
    n = batch["pos"].shape[0]
    eager = nb.Step(cfg, params, n)
    eager.set_batch(batch)
    eager.zero_grads()
    eager.train_step()
    torch.cuda.synchronize()
    fwd = ("enc", "y", "q", "normal", "rgb", "C") if cfg.loss_kind != 0 else ("enc", "y", "q", "normal")
    want_fwd = {name: getattr(eager, name).clone() for name in fwd}
    want_grad = {"d_tables": eager.d_tables.clone(), "d_small": eager.d_small.clone(), "loss": eager.loss.clone()}

    step = nb.Step(cfg, params, n)
    step.set_batch(batch)
    step.zero_grads()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step.train_step()                                  # once outside the graph: first-call set-up of the library
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    step.zero_grads()
    with torch.cuda.graph(graph):
        step.train_step()
    for replay in range(4):
        # eager work of the same library between the replays: another step on the other object, cleared gradients
        eager.zero_grads()
        eager.train_step()
        step.zero_grads()
        for name in fwd:
            getattr(step, name).fill_(7.0)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for name in fwd:
            assert torch.equal(getattr(step, name), want_fwd[name]), (replay, name)
        assert rel(step.d_tables, want_grad["d_tables"]) <= 1e-5, replay
        assert rel(step.d_small, want_grad["d_small"]) <= 1e-5, replay
        assert rel(step.loss[:2], want_grad["loss"][:2]) <= 1e-6, replay
