"""Full-size parity of the tile-density sweep (n = 256) and the geometric
graphs (n = 2048): sampled pairs against the matrix-free fp64 oracle, closed
forms where the system collapses, and cross-checks that hold at any size."""
import math

import numpy as np
import pytest

import mgk_workloads as W
import paper_1910_06310_amd as M
from oracle import c_oracle as C

pytestmark = pytest.mark.gpu
RTOL = 1e-4


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


@pytest.fixture(scope="module")
def solver(torch):
    return M.Solver(0)


def run_pairs(torch, solver, B, pi, pj):
    n = len(pi)
    K = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    it = torch.zeros((n,), dtype=torch.int32, device="cuda")
    fl = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    solver.pairs(B, B, pi, pj, K, it, fl)
    torch.cuda.synchronize()
    return K.cpu().numpy().astype(np.float64), it.cpu().numpy(), fl.cpu().numpy()


def run_pairs_nodal(torch, solver, B, wb, pi, pj):
    """Kernel values and the solutions x of Eq. 1 themselves (original vertex numbering)."""
    n = len(pi)
    sizes = wb.sizes()
    lens = sizes[pi] * sizes[pj]
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    K = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    it = torch.zeros((n,), dtype=torch.int32, device="cuda")
    fl = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    x = torch.full((int(off[-1]),), float("nan"), dtype=torch.float32, device="cuda")
    solver.pairs_nodal(B, B, pi, pj, K, x, off[:-1], it, fl)
    torch.cuda.synchronize()
    xs = x.cpu().numpy().astype(np.float64)
    return (K.cpu().numpy().astype(np.float64), [xs[off[k]:off[k + 1]] for k in range(n)],
            it.cpu().numpy(), fl.cpu().numpy())


def posterior_error_bound(wb, i, j, x):
    """Bound on |K_true - p_x^T x| for an approximate solution x of the system S of Eq. 1,
    from one fp64 residual of the oracle's matrix-free operator.

    K_true - p_x^T x = p_x^T S^{-1} rho with rho = b - S x.  Write S = M^{1/2} (I - T) M^{1/2}
    with M = diag(S) = D_x V_x^{-1}.  T is symmetric and similar to M^{-1} (M - S), whose
    entries are all >= 0, so ||T||_2 = its spectral radius <= tau = the largest row sum of
    M^{-1} (M - S) = max (M 1 - S 1) / M, which one more application of S gives; tau < 1 is the
    strict diagonal dominance of S.  Hence
    |p_x^T S^{-1} rho| <= ||M^{-1/2} p_x|| ||M^{-1/2} rho|| / (1 - tau)."""
    from oracle import mgk_oracle as O
    prm = wb.params
    g1, g2 = wb.graph(int(i)), wb.graph(int(j))
    n1, n2 = g1[0], g2[0]

    def deg(g):
        n, _lab, s, d, w, _e = g
        return (np.bincount(s, weights=w.astype(np.float64), minlength=n)
                + np.bincount(d, weights=w.astype(np.float64), minlength=n) + prm.q)

    dd = np.outer(deg(g1), deg(g2))
    kv = O.vertex_kernel(g1[1][:, None], g2[1][None, :], prm.h)
    Mdiag = (dd / kv).reshape(-1)
    b = (dd * prm.q * prm.q).reshape(-1)
    px = np.full(n1 * n2, 1.0 / (n1 * n2))
    rho = b - C.apply(g1, g2, prm.q, prm.h, prm.length_scale, x)
    m = 1.0 / np.sqrt(Mdiag)
    one = np.ones_like(Mdiag)
    tau = float(np.max((Mdiag - C.apply(g1, g2, prm.q, prm.h, prm.length_scale, one)) / Mdiag))
    assert 0.0 <= tau < 1.0
    bound = float(np.linalg.norm(m * px) * np.linalg.norm(m * rho) / (1.0 - tau))
    return bound, float(px @ x), float(np.linalg.norm(rho) / np.linalg.norm(b))


def assert_all_pairs_by_residual(wb, pi, pj, K, xs):
    """Every pair: the value the library returned is p_x^T x of the x it returned, and that x
    is within 1e-4 of the exact solution's value by the a-posteriori bound."""
    worst = 0.0
    for k, (i, j) in enumerate(zip(pi, pj)):
        bound, kx, relres = posterior_error_bound(wb, i, j, xs[k])
        assert abs(K[k] - kx) <= 1e-5 * abs(kx), (k, K[k], kx)
        assert bound + abs(K[k] - kx) <= RTOL * abs(K[k]), (k, bound, K[k], relres)
        worst = max(worst, (bound + abs(K[k] - kx)) / abs(K[k]))
    return worst


@pytest.mark.parametrize("density,n_graphs,n_check", [(0.01, 128, 6), (0.05, 128, 4), (0.2, 16, 2)])
def test_config2_density_sweep(torch, solver, density, n_graphs, n_check):
    wb = W.config2(density, n_graphs)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi = np.arange(0, n_graphs, 2, dtype=np.int32)
    pj = pi + 1
    K, it, fl = run_pairs(torch, solver, B, pi, pj)
    assert np.isfinite(K).all() and (fl == 0).all() and (it > 0).all()
    ref = C.pairs(wb, pi[:n_check], pj[:n_check], tier=1)
    np.testing.assert_allclose(K[:n_check], ref, rtol=RTOL)
    # K(G,G') = K(G',G), and Cauchy-Schwarz with the self-similarities
    Ks, _, _ = run_pairs(torch, solver, B, pj[:8], pi[:8])
    np.testing.assert_allclose(Ks, K[:8], rtol=2e-5)
    Kii, _, _ = run_pairs(torch, solver, B, pi[:8], pi[:8])
    Kjj, _, _ = run_pairs(torch, solver, B, pj[:8], pj[:8])
    assert (K[:8] ** 2 <= Kii * Kjj * (1 + 1e-4)).all()


def test_config2_fully_connected_closed_form(torch, solver):
    """Density 1.0 at n = 256.  With one weight, one edge label per graph and
    one vertex label per graph the system of Eq. 1 collapses to a scalar:
    x == d d' q^2 / (d d' / h - k k' w w' g)."""
    from mgk_workloads.generators import _assemble
    n, q, h, ls = 256, 0.05, 0.5, 1.0
    iu, ju = np.triu_indices(n, 1)
    m = len(iu)
    w1, w2, e1, e2 = 0.75, 0.5, 0.25, 1.0
    g1 = (n, np.zeros(n, np.int32), iu, ju, np.full(m, w1), np.full(m, e1))
    g2 = (n, np.ones(n, np.int32), iu, ju, np.full(m, w2), np.full(m, e2))
    prm = W.KernelParams(q=q, h=h, length_scale=ls)
    wb = _assemble([g1, g2], prm, "complete")
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    K, it, fl = run_pairs(torch, solver, B, np.array([0, 0, 1], np.int32), np.array([1, 0, 1], np.int32))
    k = n - 1
    d1, d2 = k * w1 + q, k * w2 + q
    g = math.exp(-(e1 - e2) ** 2 / (2 * ls * ls))
    assert K[0] == pytest.approx(d1 * d2 * q * q / (d1 * d2 / h - k * k * w1 * w2 * g), rel=RTOL)
    assert fl[0] == 0
    # A graph against itself has kappa == 1 everywhere: the smallest eigenvalue of the
    # system is d^2 - (k w)^2 ~ 2 q k w against a diagonal of d^2, a condition number of
    # several thousand, and b lies along that eigenvector.  fp32 cancellation in
    # a = M p - y then limits the accuracy to about eps32 * cond whatever the stopping
    # rule.  The library says so: the solution is far above the Jacobi guess, the true
    # residual is recomputed with one more product, and the pairs come back with flag 3
    # (value still within eps32 * cond of the closed form) instead of a silent flag 0.
    for val, d, kw in ((K[1], d1, k * w1), (K[2], d2, k * w2)):
        cond = (d * d + kw * kw) / (d * d - kw * kw)
        assert val == pytest.approx(d * d * q * q / (d * d - kw * kw), rel=50 * 6e-8 * cond)
    assert fl[1] == 3 and fl[2] == 3


def test_config2_dense_random_labels_reduced_size(torch, solver):
    # density 1.0 with random weights and labels, n = 96 so the oracle stays cheap
    wb = W.config2(1.0, 4, 96)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi = np.array([0, 2, 0], np.int32); pj = np.array([1, 3, 0], np.int32)
    K, it, fl = run_pairs(torch, solver, B, pi, pj)
    np.testing.assert_allclose(K, C.pairs(wb, pi, pj, tier=1), rtol=RTOL)
    assert (fl == 0).all()


@pytest.mark.parametrize("density,stride", [(0.2, 1), (1.0, 4)])
def test_config2_pairs_by_posterior_residual(torch, solver, density, stride):
    """The real 128-graph batch at the two upper densities (1.0 takes the dense tile-pair
    product), all 64 pairs solved in one call: fp64 residual of the returned x with the
    oracle's operator, for every pair at 0.2 and every fourth pair at 1.0 (two applications
    of the fp64 operator on a pair of complete graphs take several seconds of host time)."""
    wb = W.config2(density, 128)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi = np.arange(0, 128, 2, dtype=np.int32)
    pj = pi + 1
    K, xs, it, fl = run_pairs_nodal(torch, solver, B, wb, pi, pj)
    assert np.isfinite(K).all() and (fl == 0).all() and (it > 0).all()
    sel = np.arange(0, 64, stride)
    worst = assert_all_pairs_by_residual(wb, pi[sel], pj[sel], K[sel], [xs[k] for k in sel])
    print("config 2 density %g: worst a-posteriori bound / K = %.2e" % (density, worst))
    B.free()


def test_config2_dense_random_labels_full_size_against_oracle(torch, solver):
    """One pair of density 1.0 at n = 256 with the configuration's random weights, edge and
    vertex labels, dense tile-pair product, against the matrix-free fp64 oracle."""
    wb = W.config2(1.0, 2)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi = np.array([0], np.int32); pj = np.array([1], np.int32)
    K, it, fl = run_pairs(torch, solver, B, pi, pj)
    np.testing.assert_allclose(K, C.pairs(wb, pi, pj, tier=1), rtol=RTOL)
    assert (fl == 0).all()
    B.free()


def test_config3_geometric_graphs_full_size(torch, solver):
    wb = W.config3()
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    pi = np.arange(0, 32, 2, dtype=np.int32)
    pj = pi + 1
    results = {}
    stats = {}
    for reorder in (M.REORDER_PBR, M.REORDER_NONE):
        B = solver.load_batch(wb, reorder=reorder)
        stats[reorder] = B.stats()
        K, it, fl = run_pairs(torch, solver, B, pi, pj)
        assert np.isfinite(K).all() and (fl == 0).all()
        results[reorder] = K
        B.free()
    # reordering changes the tiles, never the values
    np.testing.assert_allclose(results[M.REORDER_PBR], results[M.REORDER_NONE], rtol=2e-5)
    assert stats[M.REORDER_PBR]["n_tiles"] < 0.25 * stats[M.REORDER_NONE]["n_tiles"]
    ref = C.pairs(wb, pi[:1], pj[:1], tier=1)
    np.testing.assert_allclose(results[M.REORDER_PBR][:1], ref, rtol=RTOL)
    # every one of the 16 pairs: fp64 residual of the returned x with the oracle's operator
    B = solver.load_batch(wb, reorder=M.REORDER_PBR)
    K, xs, it, fl = run_pairs_nodal(torch, solver, B, wb, pi, pj)
    np.testing.assert_allclose(K, results[M.REORDER_PBR], rtol=2e-5)
    worst = assert_all_pairs_by_residual(wb, pi, pj, K, xs)
    print("config 3: worst a-posteriori bound / K = %.2e" % worst)
    B.free()


def test_geometric_graphs_reduced_size_all_pairs(torch, solver):
    wb = W.config3(4, 512)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi, pj = W.gram_pairs(4)
    K, it, fl = run_pairs(torch, solver, B, pi, pj)
    np.testing.assert_allclose(K, C.pairs(wb, pi, pj, tier=1), rtol=RTOL)
    assert (fl == 0).all()


def test_geometric_graphs_with_rows_of_p_not_a_multiple_of_four(torch, solver):
    """n' = 259: the rows of p do not start on 16-byte boundaries, so the sparse product
    stages them element by element, several rounds per thread."""
    wb = W.config3(3, 259)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi, pj = W.gram_pairs(3)
    K, it, fl = run_pairs(torch, solver, B, pi, pj)
    np.testing.assert_allclose(K, C.pairs(wb, pi, pj, tier=1), rtol=RTOL)
    assert (fl == 0).all()


def test_mixed_density_pairs(torch, solver):
    """Pairs of one complete and one sparse graph (the middle band of the paper's
    dense / sparse primitive study, Section IV-B): n = 256 at densities 1.0 x 0.05 with both
    tile paths by the a-posteriori residual, and n = 64 against the dense fp64 oracle."""
    wb = W.concat_batches([W.config2(1.0, 4), W.config2(0.05, 4)], name="mixed")
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi = np.arange(0, 4, dtype=np.int32)
    pj = pi + 4
    values = {}
    try:
        for path in (M.TILE_AUTO, M.TILE_SPARSE, M.TILE_DENSE):
            solver.set_tile_path(path)
            K, xs, it, fl = run_pairs_nodal(torch, solver, B, wb, pi, pj)
            assert (fl == 0).all() and (it > 0).all()
            assert_all_pairs_by_residual(wb, pi[:2], pj[:2], K[:2], xs[:2])
            values[path] = K
        np.testing.assert_allclose(values[M.TILE_SPARSE], values[M.TILE_DENSE], rtol=2e-5)
        np.testing.assert_allclose(values[M.TILE_AUTO], values[M.TILE_SPARSE], rtol=2e-5)
        B.free()
        ws = W.concat_batches([W.config2(1.0, 2, 64), W.config2(0.05, 2, 64)], name="mixed small")
        solver.set_onchip_limit(0)   # the same kernels at a size the dense oracle can take
        Bs = solver.load_batch(ws)
        pi = np.array([0, 1, 0], np.int32); pj = np.array([2, 3, 3], np.int32)
        ref = C.pairs(ws, pi, pj, tier=0)
        for path in (M.TILE_SPARSE, M.TILE_DENSE):
            solver.set_tile_path(path)
            K, it, fl = run_pairs(torch, solver, Bs, pi, pj)
            np.testing.assert_allclose(K, ref, rtol=RTOL)
            assert (fl == 0).all()
    finally:
        solver.set_tile_path(M.TILE_AUTO)
        solver.set_onchip_limit(16384)
