"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle.

Tolerance: |K_gpu - K_oracle| <= 1e-4 |K_oracle| per pair (fp32 arithmetic on
the device, PCG stopped at a relative residual of 1e-6)."""
import numpy as np
import pytest

import mgk_workloads as W
import paper_1910_06310_amd as M
from oracle import c_oracle as C
from oracle import mgk_oracle as O

pytestmark = pytest.mark.gpu
RTOL = 1e-4


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


@pytest.fixture(scope="module")
def solver(torch):
    return M.Solver(0)


def run_gram(torch, solver, wb, reorder=M.REORDER_PBR):
    solver.configure(wb.params)
    B = solver.load_batch(wb, reorder=reorder)
    G = wb.n_graphs
    K = torch.full((G, G), float("nan"), dtype=torch.float32, device="cuda")
    it = torch.zeros((G, G), dtype=torch.int32, device="cuda")
    fl = torch.full((G, G), -1, dtype=torch.int32, device="cuda")
    solver.gram(B, K, it, fl)
    torch.cuda.synchronize()
    return K.cpu().numpy().astype(np.float64), it.cpu().numpy(), fl.cpu().numpy()


def run_pairs(torch, solver, BX, BY, pi, pj):
    n = len(pi)
    K = torch.full((n,), float("nan"), dtype=torch.float32, device="cuda")
    it = torch.zeros((n,), dtype=torch.int32, device="cuda")
    fl = torch.full((n,), -1, dtype=torch.int32, device="cuda")
    solver.pairs(BX, BY, pi, pj, K, it, fl)
    torch.cuda.synchronize()
    return K.cpu().numpy().astype(np.float64), it.cpu().numpy(), fl.cpu().numpy()


def test_config0_full_gram(torch, solver):
    wb = W.config0()
    solver.set_solver(1e-6, 0)
    solver.set_launch(0)
    K, it, fl = run_gram(torch, solver, wb)
    pi, pj = W.gram_pairs(4)
    ref = np.zeros((4, 4))
    ref[pi, pj] = ref[pj, pi] = O.gram_values(wb, pi, pj)
    np.testing.assert_allclose(K, ref, rtol=RTOL)
    assert (K == K.T).all()
    assert (fl == 0).all() and (it > 0).all()


@pytest.mark.parametrize("waves", [0, 1, 2, 4, 8, 16])
def test_config1_full_gram_all_workgroup_sizes(torch, solver, waves):
    wb = W.config1()
    solver.set_solver(1e-6, 0)
    solver.set_launch(waves)
    K, it, fl = run_gram(torch, solver, wb)
    solver.set_launch(0)
    pi, pj = W.gram_pairs(100)
    ref = C.pairs(wb, pi, pj, tier=1)
    err = np.abs(K[pi, pj] - ref) / ref
    assert err.max() <= RTOL, (err.max(), int(err.argmax()))
    assert (K == K.T).all() and (fl == 0).all()
    ev = np.linalg.eigvalsh(K)
    assert ev.min() >= -1e-5 * ev.max()
    if waves == 4:  # dense tier on a sample as well
        sel = np.random.default_rng(0).choice(len(pi), 300, replace=False)
        ref0 = C.pairs(wb, pi[sel], pj[sel], tier=0)
        np.testing.assert_allclose(K[pi[sel], pj[sel]], ref0, rtol=RTOL)


@pytest.mark.parametrize("reorder", [M.REORDER_NONE, M.REORDER_RCM, M.REORDER_PBR])
def test_reordering_does_not_change_values(torch, solver, reorder):
    wb = W.permute_vertices(W.config1(24), np.random.default_rng(3))
    solver.set_solver(1e-6, 0)
    K, _, fl = run_gram(torch, solver, wb, reorder=reorder)
    pi, pj = W.gram_pairs(24)
    ref = C.pairs(wb, pi, pj, tier=0)
    np.testing.assert_allclose(K[pi, pj], ref, rtol=RTOL)
    assert (fl == 0).all()


def _graph_batch(graphs, params):
    from mgk_workloads.generators import _assemble
    return _assemble(graphs, params, "adhoc")


def test_closed_forms_on_device(torch, solver):
    prm = W.KernelParams(q=0.05, h=0.5, length_scale=1.0)
    e = np.zeros(0)
    tri = (3, [0, 0, 0], [0, 0, 1], [1, 2, 2], np.ones(3), np.ones(3))
    single_a = (1, [0], [], [], e, e)
    single_b = (1, [1], [], [], e, e)
    edgeless3 = (3, [0, 1, 1], [], [], e, e)
    edgeless2 = (2, [0, 1], [], [], e, e)
    wb = _graph_batch([tri, single_a, single_b, edgeless3, edgeless2], prm)
    solver.set_solver(1e-6, 0)
    K, it, fl = run_gram(torch, solver, wb)
    assert K[0, 0] == pytest.approx(1681.0 / 32400.0, rel=RTOL)     # two triangles, all kappa = 1
    assert K[1, 1] == pytest.approx(0.0025, rel=1e-6)
    assert K[1, 2] == pytest.approx(0.00125, rel=1e-6)
    assert K[3, 4] == pytest.approx(0.001875, rel=1e-6)
    assert (fl == 0).all()


def test_weighted_graphs_and_separate_batches(torch, solver):
    rng = np.random.default_rng(5)
    prm = W.KernelParams(q=0.05, h=0.4, length_scale=0.7)
    X = W.erdos_renyi_batch(rng, 6, 5, 30, 0.3, (0.2, 2.0), (0.0, 2.0), 3, prm)
    Y = W.erdos_renyi_batch(rng, 5, 9, 70, 0.1, (0.2, 2.0), (0.0, 2.0), 3, prm)
    both = W.concat_batches([X, Y], prm)
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    BX = solver.load_batch(X)
    BY = solver.load_batch(Y, reorder=M.REORDER_RCM)
    pi = np.repeat(np.arange(6), 5).astype(np.int32)
    pj = np.tile(np.arange(5), 6).astype(np.int32)
    K, it, fl = run_pairs(torch, solver, BX, BY, pi, pj)
    ref = C.pairs(both, pi, pj + 6, tier=0)
    np.testing.assert_allclose(K, ref, rtol=RTOL)
    assert (fl == 0).all()
    # same batch on both sides, arbitrary (ordered) pair list incl. repeats
    pi2 = np.array([0, 3, 3, 5, 2], np.int32); pj2 = np.array([5, 3, 1, 0, 2], np.int32)
    K2, _, _ = run_pairs(torch, solver, BX, BX, pi2, pj2)
    np.testing.assert_allclose(K2, C.pairs(X, pi2, pj2, tier=0), rtol=RTOL)
    assert K2[0] == K2[3]


def test_rows_longer_than_a_lane_group(torch, solver):
    # dense small graphs: rows of more than 16 nonzeros take the atomic row-combine path,
    # pairs of a dense and a sparse graph put the sparse one on the lanes
    rng = np.random.default_rng(12)
    prm = W.KernelParams(q=0.05, h=0.5, length_scale=0.8)
    dense = W.erdos_renyi_batch(rng, 4, 20, 40, 0.8, (0.2, 1.0), (0.0, 2.0), 3, prm)
    sparse = W.erdos_renyi_batch(rng, 3, 20, 40, 0.1, (0.2, 1.0), (0.0, 2.0), 3, prm)
    wb = W.concat_batches([dense, sparse], prm)
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    K, it, fl = run_gram(torch, solver, wb)
    pi, pj = W.gram_pairs(7)
    np.testing.assert_allclose(K[pi, pj], C.pairs(wb, pi, pj, tier=0), rtol=RTOL)
    assert (fl == 0).all()
    BX = solver.load_batch(dense); BY = solver.load_batch(sparse)
    qi = np.repeat(np.arange(4), 3).astype(np.int32); qj = np.tile(np.arange(3), 4).astype(np.int32)
    K2, _, _ = run_pairs(torch, solver, BX, BY, qi, qj)
    np.testing.assert_allclose(K2, C.pairs(wb, qi, qj + 4, tier=0), rtol=RTOL)
    K3, _, _ = run_pairs(torch, solver, BY, BX, qj, qi)
    np.testing.assert_allclose(K3, K2, rtol=1e-5)


def test_unlabeled_random_walk_kernel(torch, solver):
    # h = 1 and a constant edge kernel of 1 give Eq. 2
    wb = W.config1(12)
    solver.set_stop_prob(0.05)
    solver.set_vertex_kernel_delta(1.0)
    solver.set_edge_kernel_const(1.0)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    pi, pj = W.gram_pairs(12)
    K, it, fl = run_pairs(torch, solver, B, B, pi, pj)
    wb.params = W.KernelParams(q=0.05, h=1.0, length_scale=1e9)
    np.testing.assert_allclose(K, C.pairs(wb, pi, pj, tier=0), rtol=RTOL)
    # constant kernel 0.5 on weighted graphs: same as labels e, e' at a fixed distance
    rng = np.random.default_rng(8)
    prm = W.KernelParams(q=0.1, h=0.6, length_scale=1.0)
    wb2 = W.erdos_renyi_batch(rng, 4, 6, 20, 0.4, (0.3, 1.5), (0.0, 0.0), 2, prm)
    solver.set_stop_prob(0.1); solver.set_vertex_kernel_delta(0.6); solver.set_edge_kernel_const(1.0)
    B2 = solver.load_batch(wb2)
    pi, pj = W.gram_pairs(4)
    K2, _, _ = run_pairs(torch, solver, B2, B2, pi, pj)
    np.testing.assert_allclose(K2, C.pairs(wb2, pi, pj, tier=0), rtol=RTOL)  # all labels 0 -> kappa_e = 1


@pytest.mark.parametrize("q", [0.005, 0.0005])
def test_small_stopping_probabilities(torch, solver, q):
    """The paper reports solves down to q = 0.0005 on labeled graphs (Section VI): long
    walks dominate, the system stays well conditioned through the vertex and edge kernels."""
    import dataclasses
    wb = W.config1(30)
    wb.params = dataclasses.replace(wb.params, q=q)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    solver.set_launch(0)
    B = solver.load_batch(wb)
    pi, pj = W.gram_pairs(30)
    ref = C.pairs(wb, pi, pj, tier=0)
    try:
        for cache in (True, False):
            solver.set_product_cache(cache)
            K, it, fl = run_pairs(torch, solver, B, B, pi, pj)
            np.testing.assert_allclose(K, ref, rtol=RTOL)
            assert (fl == 0).all()
    finally:
        solver.set_product_cache(True)


def test_iteration_cap_sets_flag(torch, solver):
    wb = W.config1(8)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 1)
    B = solver.load_batch(wb)
    pi, pj = W.gram_pairs(8)
    K, it, fl = run_pairs(torch, solver, B, B, pi, pj)
    assert (it == 1).all() and (fl == 1).all() and np.isfinite(K).all()
    solver.set_solver(1e-6, 0)


def test_start_probabilities(torch, solver):
    wb = W.config1(6)
    rng = np.random.default_rng(2)
    sp = rng.random(int(wb.vtx_off[-1])).astype(np.float32)
    for g in range(6):
        sl = slice(int(wb.vtx_off[g]), int(wb.vtx_off[g + 1]))
        sp[sl] /= sp[sl].sum()
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb, start_prob=sp)
    pi, pj = W.gram_pairs(6)
    K, _, _ = run_pairs(torch, solver, B, B, pi, pj)
    ref = C.pairs(wb, pi, pj, tier=0, start_prob=sp.astype(np.float64))
    np.testing.assert_allclose(K, ref, rtol=RTOL)


def test_config4_full_size_sampled(torch, solver):
    """The 2000-graph Gram in the launch configuration the benchmark times:
    sampled pairs against the oracle, plus properties of the whole matrix."""
    wb = W.config4()
    solver.set_solver(1e-6, 0)
    solver.set_launch(0)
    K, it, fl = run_gram(torch, solver, wb)
    assert np.isfinite(K).all() and (fl == 0).all() and (it > 0).all()
    assert (K == K.T).all()
    pi, pj = W.gram_pairs(2000)
    sel = np.random.default_rng(4).choice(len(pi), 400, replace=False)
    ref = C.pairs(wb, pi[sel], pj[sel], tier=1)
    np.testing.assert_allclose(K[pi[sel], pj[sel]], ref, rtol=RTOL)
    ev = np.linalg.eigvalsh(K)
    assert ev.min() >= -1e-5 * ev.max()
    dg = np.diag(K)
    assert (K * K <= np.outer(dg, dg) * (1 + 1e-4)).all()


# ---- global-memory solver (pairs too large for the on-chip one) ----------------
def test_global_memory_solver_agrees_with_oracle_and_onchip(torch, solver):
    wb = W.config1(20)
    solver.set_solver(1e-6, 0)
    K_chip, it_chip, _ = run_gram(torch, solver, wb)
    solver.set_onchip_limit(0)
    try:
        K_glob, it_glob, fl = run_gram(torch, solver, wb)
    finally:
        solver.set_onchip_limit(16384)
    pi, pj = W.gram_pairs(20)
    ref = C.pairs(wb, pi, pj, tier=0)
    np.testing.assert_allclose(K_glob[pi, pj], ref, rtol=RTOL)
    np.testing.assert_allclose(K_glob, K_chip, rtol=2e-5)
    assert (fl == 0).all() and (K_glob == K_glob.T).all()
    assert np.abs(it_glob - it_chip).max() <= 1


def test_global_memory_solver_weighted_long_rows_two_batches(torch, solver):
    rng = np.random.default_rng(21)
    prm = W.KernelParams(q=0.05, h=0.5, length_scale=0.8)
    X = W.erdos_renyi_batch(rng, 3, 30, 60, 0.6, (0.2, 1.0), (0.0, 2.0), 3, prm)   # rows > 16
    Y = W.erdos_renyi_batch(rng, 4, 40, 90, 0.05, (0.2, 1.0), (0.0, 2.0), 3, prm)  # sparse
    both = W.concat_batches([X, Y], prm)
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    solver.set_onchip_limit(0)
    try:
        BX = solver.load_batch(X); BY = solver.load_batch(Y)
        pi = np.repeat(np.arange(3), 4).astype(np.int32); pj = np.tile(np.arange(4), 3).astype(np.int32)
        K, it, fl = run_pairs(torch, solver, BX, BY, pi, pj)
        np.testing.assert_allclose(K, C.pairs(both, pi, pj + 3, tier=0), rtol=RTOL)
        K2, _, _ = run_pairs(torch, solver, BY, BX, pj, pi)
        np.testing.assert_allclose(K2, K, rtol=1e-5)
        qi, qj = W.gram_pairs(3)
        K3, _, fl3 = run_pairs(torch, solver, BX, BX, qi, qj)       # dense x dense: atomic row sums
        np.testing.assert_allclose(K3, C.pairs(X, qi, qj, tier=0), rtol=RTOL)
        assert (fl == 0).all() and (fl3 == 0).all()
        solver.set_solver(1e-6, 2)                                   # iteration cap
        K4, it4, fl4 = run_pairs(torch, solver, BX, BY, pi, pj)
        assert (it4 == 2).all() and (fl4 == 1).all()
    finally:
        solver.set_onchip_limit(16384)
        solver.set_solver(1e-6, 0)


def test_many_pairs_in_global_memory_are_solved_in_groups(torch, solver):
    """More pairs than one group of the global-memory solver takes (4096): the whole
    config 1 Gram with the on-chip solvers switched off."""
    wb = W.config1()
    solver.set_solver(1e-6, 0)
    solver.set_launch(0)
    solver.set_onchip_limit(0)
    try:
        K, it, fl = run_gram(torch, solver, wb)
    finally:
        solver.set_onchip_limit(16384)
    pi, pj = W.gram_pairs(100)
    ref = C.pairs(wb, pi, pj, tier=1)
    np.testing.assert_allclose(K[pi, pj], ref, rtol=RTOL)
    assert (K == K.T).all() and (fl == 0).all() and (it > 0).all()


def test_mixed_sizes_in_one_call(torch, solver):
    # one Gram whose pairs are split between the on-chip and the global-memory solver
    rng = np.random.default_rng(33)
    prm = W.KernelParams(q=0.05, h=0.5, length_scale=1.0)
    small = W.erdos_renyi_batch(rng, 3, 10, 30, 0.2, (0.5, 1.0), (0.0, 1.0), 4, prm)
    big = W.erdos_renyi_batch(rng, 2, 150, 200, 0.03, (0.5, 1.0), (0.0, 1.0), 4, prm)
    wb = W.concat_batches([small, big], prm)
    solver.set_solver(1e-6, 0)
    K, it, fl = run_gram(torch, solver, wb)
    pi, pj = W.gram_pairs(5)
    ref = C.pairs(wb, pi, pj, tier=1)
    np.testing.assert_allclose(K[pi, pj], ref, rtol=RTOL)
    assert (fl == 0).all() and (K == K.T).all()


@pytest.mark.parametrize("weighted", [False, True])
def test_dense_and_sparse_tile_paths_agree(torch, solver, weighted):
    # sizes that are not multiples of 8 exercise the padded last tile row
    rng = np.random.default_rng(44)
    prm = W.KernelParams(q=0.05, h=0.5, length_scale=0.7)
    wr = (0.3, 1.5) if weighted else (1.0, 1.0)
    X = W.erdos_renyi_batch(rng, 3, 37, 61, 0.5, wr, (0.0, 2.0), 3, prm)
    Y = W.erdos_renyi_batch(rng, 2, 19, 45, 0.15, wr, (0.0, 2.0), 3, prm)
    both = W.concat_batches([X, Y], prm)
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    solver.set_onchip_limit(0)
    try:
        BX = solver.load_batch(X); BY = solver.load_batch(Y, reorder=M.REORDER_NONE)
        pi = np.repeat(np.arange(3), 2).astype(np.int32); pj = np.tile(np.arange(2), 3).astype(np.int32)
        ref = C.pairs(both, pi, pj + 3, tier=0)
        out = {}
        for mode in (M.TILE_SPARSE, M.TILE_SPARSE_GATHER, M.TILE_DENSE, M.TILE_AUTO):
            solver.set_tile_path(mode)
            K, it, fl = run_pairs(torch, solver, BX, BY, pi, pj)
            np.testing.assert_allclose(K, ref, rtol=RTOL)
            assert (fl == 0).all()
            out[mode] = (K, it)
        np.testing.assert_allclose(out[M.TILE_DENSE][0], out[M.TILE_SPARSE][0], rtol=2e-5)
        np.testing.assert_allclose(out[M.TILE_SPARSE_GATHER][0], out[M.TILE_SPARSE][0], rtol=2e-5)
        assert np.abs(out[M.TILE_DENSE][1] - out[M.TILE_SPARSE][1]).max() <= 1
        # constant edge kernel through the dense primitive
        solver.set_edge_kernel_const(0.5)
        solver.set_tile_path(M.TILE_DENSE)
        qi, qj = W.gram_pairs(3)
        Kd, _, _ = run_pairs(torch, solver, BX, BX, qi, qj)
        solver.set_tile_path(M.TILE_SPARSE)
        Ks, _, _ = run_pairs(torch, solver, BX, BX, qi, qj)
        np.testing.assert_allclose(Kd, Ks, rtol=2e-5)
    finally:
        solver.set_tile_path(M.TILE_AUTO)
        solver.set_onchip_limit(16384)


@pytest.mark.parametrize("kind", ["nws", "ba"])
def test_paper_synthetic_sets(torch, solver, kind):
    """The paper's own synthetic families at full size (160 graphs of 96 nodes):
    whole Gram on the device, sampled pairs against the oracle, matrix properties."""
    wb = W.paper_synthetic(kind)
    solver.set_solver(1e-6, 0)
    K, it, fl = run_gram(torch, solver, wb)
    assert np.isfinite(K).all() and (fl == 0).all() and (K == K.T).all()
    pi, pj = W.gram_pairs(wb.n_graphs)
    sel = np.random.default_rng(6).choice(len(pi), 60, replace=False)
    np.testing.assert_allclose(K[pi[sel], pj[sel]], C.pairs(wb, pi[sel], pj[sel], tier=1), rtol=RTOL)
    ev = np.linalg.eigvalsh(K)
    assert ev.min() >= -1e-5 * ev.max()


def test_nodal_similarity_and_normalized_gram(torch, solver):
    """x itself (node-wise similarity) in the caller's vertex numbering, for both
    orientations, both solvers and with reordering on; then K / sqrt(K_ii K_jj)."""
    rng = np.random.default_rng(17)
    prm = W.KernelParams(q=0.05, h=0.4, length_scale=0.6)
    X = W.permute_vertices(W.erdos_renyi_batch(rng, 3, 9, 40, 0.15, (0.3, 1.2), (0.0, 2.0), 3, prm), rng)
    Y = W.permute_vertices(W.erdos_renyi_batch(rng, 3, 30, 80, 0.08, (0.3, 1.2), (0.0, 2.0), 3, prm), rng)
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    BX = solver.load_batch(X); BY = solver.load_batch(Y)
    pi = np.repeat(np.arange(3), 3).astype(np.int32); pj = np.tile(np.arange(3), 3).astype(np.int32)
    sizes = X.sizes()[pi] * Y.sizes()[pj]
    off = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int64)
    refs = [C.pair_nodal(X.graph(int(i)), Y.graph(int(j)), prm.q, prm.h, prm.length_scale) for i, j in zip(pi, pj)]
    try:
        for limit in (16384, 0):
            solver.set_onchip_limit(limit)
            K = torch.zeros(9, dtype=torch.float32, device="cuda")
            x = torch.full((int(sizes.sum()),), float("nan"), dtype=torch.float32, device="cuda")
            solver.pairs_nodal(BX, BY, pi, pj, K, x, off)
            torch.cuda.synchronize()
            xs = x.cpu().numpy().astype(np.float64); Ks = K.cpu().numpy()
            for k, (Kref, xref) in enumerate(refs):
                got = xs[off[k]:off[k] + sizes[k]].reshape(xref.shape)
                np.testing.assert_allclose(got, xref, rtol=RTOL, atol=RTOL * np.abs(xref).max())
                assert Ks[k] == pytest.approx(Kref, rel=RTOL)
            # the other argument order returns the transposed blocks
            K2 = torch.zeros(9, dtype=torch.float32, device="cuda")
            x2 = torch.zeros_like(x)
            solver.pairs_nodal(BY, BX, pj, pi, K2, x2, off)
            torch.cuda.synchronize()
            x2s = x2.cpu().numpy()
            for k, (_, xref) in enumerate(refs):
                got = x2s[off[k]:off[k] + sizes[k]].reshape(xref.shape[::-1]).T
                np.testing.assert_allclose(got, xref, rtol=RTOL, atol=RTOL * np.abs(xref).max())
    finally:
        solver.set_onchip_limit(16384)
    wb = W.config1(12)
    Kg, _, _ = run_gram(torch, solver, wb)
    Kt = torch.tensor(Kg, dtype=torch.float32, device="cuda")
    solver.normalize_gram(12, Kt)
    torch.cuda.synchronize()
    dg = np.sqrt(np.diag(Kg))
    np.testing.assert_allclose(Kt.cpu().numpy(), Kg / np.outer(dg, dg), rtol=1e-5)
    assert np.allclose(np.diag(Kt.cpu().numpy()), 1.0, atol=1e-6)


@pytest.mark.parametrize("cache", [True, False])
def test_small_weighted_pairs_on_both_onchip_solvers(torch, solver, cache):
    """Molecule-sized weighted graphs from two batches, with the matrix entries kept in
    registers (cache) and regenerated every iteration: values and nodal solutions in
    both argument orders, square-exponential and constant edge kernels."""
    rng = np.random.default_rng(23)
    prm = W.KernelParams(q=0.07, h=0.4, length_scale=0.3)
    X = W.molecule_like_batch(rng, 5, 12, 30, prm)
    Y = W.molecule_like_batch(rng, 4, 30, 60, prm)
    for b in (X, Y):
        b.weight = rng.uniform(0.4, 1.6, len(b.weight)).astype(np.float32)
    X = W.permute_vertices(X, rng)
    Y = W.permute_vertices(Y, rng)
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    solver.set_launch(0)
    solver.set_product_cache(cache)
    try:
        BX = solver.load_batch(X); BY = solver.load_batch(Y)
        pi = np.repeat(np.arange(5), 4).astype(np.int32); pj = np.tile(np.arange(4), 5).astype(np.int32)
        sizes = X.sizes()[pi] * Y.sizes()[pj]
        off = np.concatenate([[0], np.cumsum(sizes)[:-1]]).astype(np.int64)
        refs = [C.pair_nodal(X.graph(int(i)), Y.graph(int(j)), prm.q, prm.h, prm.length_scale) for i, j in zip(pi, pj)]
        for (A, B, ai, bi, transposed) in ((BX, BY, pi, pj, False), (BY, BX, pj, pi, True)):
            K = torch.zeros(len(pi), dtype=torch.float32, device="cuda")
            x = torch.full((int(sizes.sum()),), float("nan"), dtype=torch.float32, device="cuda")
            fl = torch.full((len(pi),), -1, dtype=torch.int32, device="cuda")
            solver.pairs_nodal(A, B, ai, bi, K, x, off, None, fl)
            torch.cuda.synchronize()
            xs = x.cpu().numpy().astype(np.float64); Ks = K.cpu().numpy()
            assert (fl.cpu().numpy() == 0).all()
            for k, (Kref, xref) in enumerate(refs):
                got = xs[off[k]:off[k] + sizes[k]]
                got = got.reshape(xref.shape[::-1]).T if transposed else got.reshape(xref.shape)
                np.testing.assert_allclose(got, xref, rtol=RTOL, atol=RTOL * np.abs(xref).max())
                assert Ks[k] == pytest.approx(Kref, rel=RTOL)
        # constant edge kernel on the same weighted graphs: labels all equal in the oracle
        solver.set_edge_kernel_const(1.0)
        Kc, _, flc = run_pairs(torch, solver, BX, BY, pi, pj)
        X0 = W.GraphBatch(X.vtx_off, X.vtx_label, X.edge_off, X.src, X.dst, X.weight,
                          np.zeros_like(X.edge_label), prm)
        Y0 = W.GraphBatch(Y.vtx_off, Y.vtx_label, Y.edge_off, Y.src, Y.dst, Y.weight,
                          np.zeros_like(Y.edge_label), prm)
        refc = [C.pair_nodal(X0.graph(int(i)), Y0.graph(int(j)), prm.q, prm.h, prm.length_scale)[0]
                for i, j in zip(pi, pj)]
        np.testing.assert_allclose(Kc, refc, rtol=RTOL)
        assert (flc == 0).all()
    finally:
        solver.set_product_cache(True)


def test_edge_cases(torch, solver):
    """Empty requests, single graphs, single-vertex and edgeless graphs on both solvers,
    and the largest product size the on-chip solver takes."""
    from mgk_workloads.generators import _assemble
    prm = W.KernelParams(q=0.05, h=0.5, length_scale=1.0)
    solver.configure(prm)
    solver.set_solver(1e-6, 0)
    e = np.zeros(0)
    rng = np.random.default_rng(3)
    big = W.erdos_renyi_batch(rng, 2, 128, 128, 0.03, (0.5, 1.0), (0.0, 1.0), 3, prm)   # N = 16384
    graphs = [(1, [2], [], [], e, e), (5, [0, 1, 2, 0, 1], [], [], e, e), big.graph(0), big.graph(1)]
    wb = _assemble(graphs, prm, "edge")
    B = solver.load_batch(wb)
    K = torch.zeros(1, dtype=torch.float32, device="cuda")
    solver.pairs(B, B, np.zeros(0, np.int32), np.zeros(0, np.int32), K)       # nothing to do
    pi, pj = W.gram_pairs(4)
    ref = C.pairs(wb, pi, pj, tier=1)
    try:
        for limit in (16384, 0):
            solver.set_onchip_limit(limit)
            Kp, it, fl = run_pairs(torch, solver, B, B, pi, pj)
            np.testing.assert_allclose(Kp, ref, rtol=RTOL)
            assert (fl == 0).all()
    finally:
        solver.set_onchip_limit(16384)
    one = solver.load_batch(_assemble(graphs[:1], prm, "one"))
    K1, _, _ = run_gram(torch, solver, _assemble(graphs[:1], prm, "one"))
    assert K1.shape == (1, 1) and K1[0, 0] == pytest.approx(0.0025, rel=1e-6)
    one.free()


def test_pairs_with_index_arrays_on_the_device(torch, solver):
    """mgk_pairs_dev takes the pair indices from device memory; same values, bit for bit, as
    the entry point that takes them from the host, and within tolerance of the oracle."""
    wb = W.config1(24)
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    B = solver.load_batch(wb)
    rng = np.random.default_rng(3)
    pi = rng.integers(0, 24, 200).astype(np.int32)
    pj = rng.integers(0, 24, 200).astype(np.int32)
    K_host, it_host, fl_host = run_pairs(torch, solver, B, B, pi, pj)
    K = torch.full((200,), float("nan"), dtype=torch.float32, device="cuda")
    it = torch.zeros((200,), dtype=torch.int32, device="cuda")
    fl = torch.full((200,), -1, dtype=torch.int32, device="cuda")
    solver.pairs_dev(B, B, torch.from_numpy(pi).cuda(), torch.from_numpy(pj).cuda(), K, it, fl)
    torch.cuda.synchronize()
    assert (K.cpu().numpy().astype(np.float64) == K_host).all()
    assert (it.cpu().numpy() == it_host).all() and (fl.cpu().numpy() == 0).all()
    np.testing.assert_allclose(K_host, C.pairs(wb, pi, pj, tier=1), rtol=RTOL)


def test_owner_computes_kernel_agrees_with_oracle(torch, solver):
    """mgk_set_product_cache(3): every lane owns rows of the system (degree-sorted tiles).
    All pairs of the 100 molecule-like graphs and of the 4 small random graphs (isolated
    vertices, weights), start probabilities and the nodal solution included."""
    solver.set_solver(1e-6, 0)
    solver.set_launch(0)
    solver.set_product_cache(3)
    try:
        wb = W.config1()
        K, it, fl = run_gram(torch, solver, wb)
        pi, pj = W.gram_pairs(100)
        ref = C.pairs(wb, pi, pj, tier=1)
        err = np.abs(K[pi, pj] - ref) / ref
        assert err.max() <= RTOL, (err.max(), int(err.argmax()))
        assert (K == K.T).all() and (fl == 0).all() and (it > 0).all()
        solver.set_product_cache(1)
        K1, it1, _ = run_gram(torch, solver, wb)
        solver.set_product_cache(3)
        assert (it1 == it).all()   # same iteration, same stopping rule
        np.testing.assert_allclose(K, K1, rtol=2e-5)

        wb = W.config0()
        K, it, fl = run_gram(torch, solver, wb)
        pi, pj = W.gram_pairs(4)
        np.testing.assert_allclose(K[pi, pj], O.gram_values(wb, pi, pj), rtol=RTOL)
        assert (fl == 0).all()

        # nodal solution in the caller's numbering, with non-uniform start probabilities
        wb = W.config1(6)
        rng = np.random.default_rng(5)
        sp = np.concatenate([(lambda v: v / v.sum())(rng.uniform(0.2, 1.0, n)) for n in wb.sizes()]).astype(np.float32)
        solver.configure(wb.params)
        B = solver.load_batch(wb, start_prob=sp)
        pi, pj = W.gram_pairs(6)
        sizes = wb.sizes()
        off = np.concatenate([[0], np.cumsum(sizes[pi] * sizes[pj])]).astype(np.int64)
        Kd = torch.zeros(len(pi), dtype=torch.float32, device="cuda")
        xd = torch.full((int(off[-1]),), float("nan"), dtype=torch.float32, device="cuda")
        solver.pairs_nodal(B, B, pi, pj, Kd, xd, off[:-1])
        torch.cuda.synchronize()
        ref = C.pairs(wb, pi, pj, tier=0, start_prob=sp.astype(np.float64))
        np.testing.assert_allclose(Kd.cpu().numpy(), ref, rtol=RTOL)
        xs = xd.cpu().numpy().astype(np.float64)
        for k in (0, 7, len(pi) - 1):
            _, xref = C.pair_nodal(wb.graph(int(pi[k])), wb.graph(int(pj[k])), wb.params.q, wb.params.h,
                                   wb.params.length_scale, tier=0)
            np.testing.assert_allclose(xs[off[k]:off[k + 1]], xref.reshape(-1), rtol=RTOL)
    finally:
        solver.set_product_cache(1)
