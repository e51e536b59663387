"""Host logic of the library on a host-only context (no GPU): validation,
vertex reordering, octile packing, exported symbols."""
import ctypes
import os
import re

import numpy as np
import pytest

import mgk_workloads as W
import paper_1910_06310_amd as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def solver():
    return M.Solver(-1)


def dense_from_batch(b, g):
    n, _lab, s, d, w, e = b.graph(g)
    A = np.zeros((n, n), np.float32); E = np.zeros((n, n), np.float32)
    A[s, d] = w; A[d, s] = w
    E[s, d] = e; E[d, s] = e
    return A, E


def unpack(tiles, n):
    """Expand the packed tiles back to dense A, E in stored vertex order."""
    A = np.zeros((n, n), np.float32); E = np.zeros((n, n), np.float32)
    k = 0
    for tr, tc, bm in zip(tiles["tile_row"], tiles["tile_col"], tiles["bitmap"]):
        for bit in range(64):
            if (int(bm) >> bit) & 1:
                i, j = tr * 8 + bit // 8, tc * 8 + bit % 8
                A[i, j] = tiles["w"][k]; E[i, j] = tiles["e"][k]
                k += 1
    assert k == len(tiles["w"])
    return A, E


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "mgk.h")).read()
    declared = sorted(set(re.findall(r"\b(mgk_[a-z_]+)\s*\(", header)))
    assert declared, "no declarations found"
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_1910_06310_amd", "libmgk.so"))
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(M.EXPORTS) == declared


@pytest.mark.parametrize("reorder", [M.REORDER_NONE, M.REORDER_PBR, M.REORDER_RCM])
def test_pack_unpack_roundtrip_and_permutation(solver, reorder):
    b = W.concat_batches([W.config0(), W.config1(12), W.config2(0.05, 2, 64)])
    B = solver.load_batch(b, reorder=reorder)
    perm = B.permutation()
    st = B.stats()
    assert st["n_graphs"] == b.n_graphs and st["nnz"] == int(b.nnz().sum())
    tiles_total = offdiag_total = 0
    for g in range(b.n_graphs):
        n = b.n_vertices(g)
        p = perm[b.vtx_off[g]:b.vtx_off[g + 1]]
        assert sorted(p.tolist()) == list(range(n))            # bijection
        if reorder == M.REORDER_NONE:
            assert (p == np.arange(n)).all()
        A, E = dense_from_batch(b, g)
        inv = np.empty(n, np.int64); inv[p] = np.arange(n)      # stored -> original
        t = B.get_tiles(g)
        A2, E2 = unpack(t, n)
        np.testing.assert_array_equal(A2, A[np.ix_(inv, inv)])   # exact, both triangles
        np.testing.assert_array_equal(E2, E[np.ix_(inv, inv)])
        # tiles sorted by (row, col), none empty, bit count = packed length
        keys = t["tile_row"].astype(np.int64) * 100000 + t["tile_col"]
        assert (np.diff(keys) > 0).all()
        assert all(int(x) != 0 for x in t["bitmap"])
        assert sum(bin(int(x)).count("1") for x in t["bitmap"]) == len(t["w"])
        # Eq. 3: off-diagonal non-empty tiles = 2 x (connected pairs of 8-blocks)
        _, _, s, d, _, _ = b.graph(g)
        blocks = {(min(p[a] // 8, p[c] // 8), max(p[a] // 8, p[c] // 8))
                  for a, c in zip(s, d) if p[a] // 8 != p[c] // 8}
        offdiag = int((t["tile_row"] != t["tile_col"]).sum())
        assert offdiag == 2 * len(blocks)
        tiles_total += len(t["bitmap"]); offdiag_total += offdiag
    assert st["n_tiles"] == tiles_total and st["n_offdiag_tiles"] == offdiag_total


def test_pbr_does_not_lose_to_natural_order_on_shuffled_molecules(solver):
    # reported, heuristic: on randomly relabelled molecule-like graphs the
    # partition-based order must at least beat the shuffled order clearly
    b = W.permute_vertices(W.config1(40), np.random.default_rng(0))
    nat = solver.load_batch(b, reorder=M.REORDER_NONE).stats()["n_offdiag_tiles"]
    pbr = solver.load_batch(b, reorder=M.REORDER_PBR).stats()["n_offdiag_tiles"]
    rcm = solver.load_batch(b, reorder=M.REORDER_RCM).stats()["n_offdiag_tiles"]
    assert pbr < 0.7 * nat
    assert pbr <= 1.05 * rcm


def _load(solver, n, edges, w=None, e=None, labels=None, start=None):
    edges = np.asarray(edges, np.int32).reshape(-1, 2)
    return solver.load_graphs([0, n], labels if labels is not None else np.zeros(n, np.int32),
                              [0, len(edges)], edges[:, 0], edges[:, 1], w, e, start)


def test_invalid_graphs_are_rejected(solver):
    for kwargs in [
        dict(n=3, edges=[(0, 0)]),                       # self loop
        dict(n=3, edges=[(0, 1), (1, 0)]),               # duplicate edge
        dict(n=3, edges=[(0, 3)]),                       # out of range
        dict(n=3, edges=[(0, 1)], w=[-1.0]),             # negative weight
        dict(n=3, edges=[(0, 1)], w=[0.0]),              # zero weight
        dict(n=3, edges=[(0, 1)], w=[np.nan]),
        dict(n=3, edges=[(0, 1)], e=[np.inf]),
        dict(n=0, edges=[]),                             # empty graph
        dict(n=2, edges=[(0, 1)], start=[np.nan, 0.5]),
    ]:
        with pytest.raises(M.MgkError) as ei:
            _load(solver, **kwargs)
        assert ei.value.status == M.binding.EINVAL, kwargs


def test_parameter_validation_and_host_only_solve(solver):
    for fn, bad in [(solver.set_vertex_kernel_delta, 0.0), (solver.set_vertex_kernel_delta, 1.5),
                    (solver.set_edge_kernel_se, 0.0), (solver.set_edge_kernel_const, 1.1),
                    (solver.set_stop_prob, 0.0), (solver.set_launch, 3), (solver.set_tile_path, 7),
                    (solver.set_onchip_limit, -1)]:
        with pytest.raises(M.MgkError):
            fn(bad)
    with pytest.raises(M.MgkError):
        solver.set_solver(0.0, 10)
    solver.set_solver(1e-6, 0)
    B = _load(solver, 2, [(0, 1)])
    lib = M.load_library()
    st = lib.mgk_gram(solver._h, B._h, ctypes.c_void_p(16), None, None, None)
    assert st == M.binding.ESTATE


def test_single_vertex_and_edgeless_graphs_pack(solver):
    B = solver.load_graphs([0, 1, 4], np.zeros(4, np.int32), [0, 0, 0], [], [])
    st = B.stats()
    assert st["n_tiles"] == 0 and st["nnz"] == 0 and st["n_vertices"] == 4


def test_morton_numbering_of_geometric_graphs():
    """The space-filling-curve ordering (Section IV-A) is a property of the input
    numbering: the same graphs, far fewer non-empty octiles than the random
    numbering, more than PBR finds."""
    import mgk_workloads as W
    from oracle import mgk_oracle as O
    rnd = W.geometric_batch(np.random.default_rng(5), 2, 40, 5.0, 3, W.KernelParams(0.05, 0.5, 0.3), order="random")
    mor = W.geometric_batch(np.random.default_rng(5), 2, 40, 5.0, 3, W.KernelParams(0.05, 0.5, 0.3), order="morton")
    assert O.gram_values(mor, [0], [1])[0] == pytest.approx(O.gram_values(rnd, [0], [1])[0], rel=1e-12)
    s = M.Solver(-1)
    big_r, big_m = W.config3(2, 512, order="random"), W.config3(2, 512, order="morton")
    t_rand = s.load_batch(big_r, reorder=M.REORDER_NONE).stats()["n_offdiag_tiles"]
    t_mort = s.load_batch(big_m, reorder=M.REORDER_NONE).stats()["n_offdiag_tiles"]
    t_pbr = s.load_batch(big_r, reorder=M.REORDER_PBR).stats()["n_offdiag_tiles"]
    assert t_pbr < t_mort < 0.5 * t_rand


def test_offsets_are_validated_before_anything_is_sized_by_them(solver):
    """Offset arrays that decrease in the middle (the last entry is then not a bound for the
    others) and absurd totals are rejected with a status: no write past the arrays they size,
    no exception across the C ABI."""
    lab = np.zeros(150, np.int32)
    # graph 0 claims 100 vertices although the total is 50
    with pytest.raises(M.MgkError) as ei:
        solver.load_graphs([0, 100, 50], lab, [0, 0, 0], [], [])
    assert ei.value.status == 1
    # edge offsets that come back below an earlier one
    src = np.zeros(8, np.int32); dst = np.ones(8, np.int32)
    with pytest.raises(M.MgkError) as ei:
        solver.load_graphs([0, 2, 4], lab, [0, 8, 1], src, dst)
    assert ei.value.status == 1
    # a vertex total no host can hold: refused by the 32-bit limit, not by a failed allocation
    with pytest.raises(M.MgkError) as ei:
        solver.load_graphs([0, 2 ** 40], lab, [0, 0], [], [])
    assert ei.value.status in (1, 5)
    # the context is still usable
    b = W.config0()
    assert solver.load_batch(b).stats()["n_graphs"] == 4


def test_space_filling_curve_order_of_embedded_graphs(solver):
    """mgk_load_graphs_embedded numbers the vertices of graphs that come with coordinates
    along the Morton curve (Section IV-A).  On points in the unit cube the numbering must be
    the one obtained by sorting the interleaved 10-bit cell indices (computed here from the
    definition), the packed form must still be the same graph, and the tile count must
    fall well below that of the random numbering."""
    rng = np.random.default_rng(5)
    b = W.geometric_batch(rng, 3, 300, 12, 4, W.KernelParams(), order="random")
    B = solver.load_graphs_embedded(b.vtx_off, b.vtx_label, b.edge_off, b.src, b.dst, b.coords,
                                    weight=b.weight, edge_label=b.edge_label)
    perm = B.permutation()
    for g in range(3):
        v0, v1 = int(b.vtx_off[g]), int(b.vtx_off[g + 1])
        pts = b.coords[v0:v1].astype(np.float64)
        lo, hi = pts.min(0), pts.max(0)
        cell = np.minimum(((pts - lo) / (hi - lo) * 1024).astype(np.int64), 1023)
        key = np.zeros(len(pts), np.int64)
        for bit in range(10):
            for axis in range(3):
                key |= ((cell[:, axis] >> bit) & 1) << (3 * bit + axis)
        expect = np.empty(len(pts), np.int64)
        expect[np.argsort(key, kind="stable")] = np.arange(len(pts))
        p = perm[v0:v1]
        assert sorted(p) == list(range(len(pts)))
        # cells are computed in float32 there and float64 here: allow the few points that sit
        # on a cell boundary to differ
        assert (p == expect).mean() > 0.97
        A, E = dense_from_batch(b, g)
        Ap, Ep = unpack(B.get_tiles(g), len(pts))
        np.testing.assert_array_equal(Ap[np.ix_(p, p)], A)
        np.testing.assert_array_equal(Ep[np.ix_(p, p)], E)
    random_tiles = solver.load_batch(b, reorder=M.REORDER_NONE).stats()["n_tiles"]
    assert B.stats()["n_tiles"] < 0.5 * random_tiles
    with pytest.raises(M.MgkError):
        solver.load_batch(b, reorder=3)   # the curve order needs coordinates
