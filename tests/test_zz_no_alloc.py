"""The scatter-add entry point that allocates nothing (its record lists live in a static device
array) against the entry point that takes a caller's workspace: same inputs, two calls in a row,
the second with a smaller batch."""
import numpy as np
import pytest

torch = pytest.importorskip("torch")

from oracle import neus2_oracle as o
from paper_2212_05231_amd import binding as nb
from paper_2212_05231_amd import workloads as wl

pytestmark = pytest.mark.gpu

GRAD_TOL = 1e-4


def rel(a, b):
    a, b = np.asarray(a, dtype=np.float64), np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / np.linalg.norm(b))


def test_static_scratch_scatter_matches_the_workspace_scatter_twice():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    cfg = wl.make_config(2)
    c = nb.make_config(cfg)
    L, T = cfg.n_levels, cfg.table_size
    tables = torch.as_tensor(wl.make_params(cfg, 7)["tables"]).cuda()
    for call, n in enumerate((80000, (1 << 16) + 7)):
        rng = np.random.default_rng(100 + call)
        pos = torch.as_tensor(wl.make_rays(n // 64 + 1, 64, 50 + call)["pos"][:n]).cuda().contiguous()
        q = torch.as_tensor(rng.normal(size=(L, n, 2)).astype(np.float32)).cuda()
        d_enc = torch.as_tensor(rng.normal(size=(L, n, 2)).astype(np.float32)).cuda()
        d_normal = torch.as_tensor(rng.normal(size=(n, 3)).astype(np.float32) * 1e-3).cuda()
        need = nb.workspace_bytes(c, n)
        assert 0 < need - 24 * L * n <= 128 * 1024 * 1024          # the owner path, and it fits the static buffer
        ws = torch.zeros(need // 4, dtype=torch.int32, device="cuda")
        want = torch.zeros(L, T, 2, device="cuda")
        nb.hash_scatter_bwd(c, pos, tables, q, d_enc, d_normal, n, want, workspace=ws)
        got = torch.full((L, T, 2), 0.25, device="cuda")             # the gradient is ADDED into
        nb.hash_scatter_bwd_static(c, pos, tables, q, d_enc, d_normal, n, got)
        torch.cuda.synchronize()
        got = got.cpu().numpy().astype(np.float64) - 0.25
        assert rel(got, want.cpu().numpy()) <= 1e-6                  # same kernels, sums in another order
        if call == 1:                                                # and once against the oracle itself
            lm = lambda t: np.transpose(t.cpu().numpy().astype(np.float64), (1, 0, 2)).reshape(n, -1)
            ref = o.table_gradient(cfg, pos.cpu().numpy(), lm(q), lm(d_enc), d_normal.cpu().numpy())
            assert rel(got, ref) <= GRAD_TOL
    # a batch whose lists do not fit is refused before anything is launched
    n_big = 1 << 18
    assert nb.workspace_bytes(c, n_big) - 24 * L * n_big > 128 * 1024 * 1024
    with pytest.raises(nb.Neus2Error) as err:
        nb.hash_scatter_bwd_static(c, pos, tables, q, d_enc, d_normal, n_big, want)
    assert err.value.code == -2
