"""The entry point that allocates nothing (mgk_pairs_noalloc) against mgk_pairs: same
values bit for bit on two calls in a row, the second with a smaller input, and its limits."""
import numpy as np
import pytest

import mgk_workloads as W
import paper_1910_06310_amd as M
from oracle import c_oracle as C

pytestmark = pytest.mark.gpu


def _run(torch, fn, B, pi, pj):
    n = len(pi)
    K = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    it = torch.zeros((n,), dtype=torch.int32, device="cuda")
    fl = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    fn(B, B, pi, pj, K, it, fl)
    torch.cuda.synchronize()
    return K.cpu().numpy(), it.cpu().numpy(), fl.cpu().numpy()


def test_noalloc_entry_point_matches_pairs():
    import torch
    solver = M.Solver(0)
    wb = W.config1(40)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    rng = np.random.default_rng(17)
    # first call: 3000 pairs; second call: 257 other pairs (the array still holds the first list)
    for n in (3000, 257):
        pi = rng.integers(0, 40, n).astype(np.int32)
        pj = rng.integers(0, 40, n).astype(np.int32)
        K0, it0, fl0 = _run(torch, solver.pairs, B, pi, pj)
        K1, it1, fl1 = _run(torch, solver.pairs_noalloc, B, pi, pj)
        assert (K1 == K0).all() and (it1 == it0).all() and (fl1 == fl0).all()
        assert (fl1 == 0).all() and np.isfinite(K1).all()
        sel = rng.choice(n, 40, replace=False)
        np.testing.assert_allclose(K1[sel].astype(np.float64), C.pairs(wb, pi[sel], pj[sel], tier=1), rtol=1e-4)
    # limits: too many pairs, and a pair that needs the global-memory solver
    big = np.zeros(65537, np.int32)
    K = torch.zeros(65537, dtype=torch.float32, device="cuda")
    with pytest.raises(M.MgkError) as ei:
        solver.pairs_noalloc(B, B, big, big, K)
    assert ei.value.status == 5
    wl = W.config2(0.05, 2)
    solver.configure(wl.params)
    BL = solver.load_batch(wl)
    with pytest.raises(M.MgkError) as ei:
        solver.pairs_noalloc(BL, BL, [0], [1], K)
    assert ei.value.status == 5
    # the context still works afterwards
    solver.configure(wb.params)
    pi = np.arange(10, dtype=np.int32); pj = pi[::-1].copy()
    K0, _, _ = _run(torch, solver.pairs, B, pi, pj)
    K1, _, _ = _run(torch, solver.pairs_noalloc, B, pi, pj)
    assert (K1 == K0).all()
