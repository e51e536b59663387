"""Pins for the CPU oracle: closed forms of Eq. 1, the random-walk series and
walk enumeration of Appendix A, and the invariants of a valid graph kernel.
None of these re-types the oracle's own assembly loop; each is a different
route to the same number (or a property the number must have)."""
import math
import os

import numpy as np
import pytest

import mgk_workloads as W
from oracle import c_oracle as C
from oracle import mgk_oracle as O

Q = 0.05
GOLD = {}
with open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")) as fh:
    for line in fh:
        if line.startswith("#") or "|" not in line:
            continue
        name, val, _ = [t.strip() for t in line.split("|", 2)]
        GOLD[name] = float(val)


def f32(a):
    """Inputs are float32 at the library boundary; round once so every route sees the same numbers."""
    return np.asarray(a, dtype=np.float32).astype(np.float64)


def G(n, labels, edges, w=None, e=None):
    edges = np.asarray(edges, dtype=np.int64).reshape(-1, 2)
    m = len(edges)
    return (n, np.asarray(labels, dtype=np.int32), edges[:, 0].copy(), edges[:, 1].copy(),
            np.ones(m) if w is None else f32(w),
            np.zeros(m) if e is None else f32(e))


def both(g1, g2, q, h, ls):
    """numpy dense, C dense, C matrix-free: all three must agree."""
    k0 = O.kernel_value(g1, g2, q, h, ls)
    k1, _ = C.pair_nodal(g1, g2, q, h, ls, tier=0)
    k2, _ = C.pair_nodal(g1, g2, q, h, ls, tier=1)
    assert k1 == pytest.approx(k0, rel=1e-12)
    assert k2 == pytest.approx(k0, rel=1e-10)
    return k0


def random_graph(rng, n, prob=0.5, n_labels=3):
    iu, ju = np.triu_indices(n, 1)
    keep = rng.random(len(iu)) < prob
    m = int(keep.sum())
    return (n, rng.integers(0, n_labels, n).astype(np.int32), iu[keep], ju[keep],
            f32(rng.uniform(0.5, 1.5, m)), f32(rng.uniform(0.0, 2.0, m)))


# ---- P1 / P2: systems without edges ---------------------------------------
def test_single_vertex_closed_form():
    g = G(1, [0], [])
    gd = G(1, [1], [])
    assert both(g, g, Q, 0.5, 1.0) == pytest.approx(GOLD["single_vertex_same_label"], rel=1e-14)
    assert both(g, gd, Q, 0.5, 1.0) == pytest.approx(GOLD["single_vertex_diff_label_h0.5"], rel=1e-14)


def test_edgeless_graphs():
    g1 = G(3, [0, 1, 1], [])
    g2 = G(2, [0, 1], [])
    assert both(g1, g2, Q, 0.5, 1.0) == pytest.approx(GOLD["edgeless_3x2_labels"], rel=1e-14)
    _, x = O.kernel_value(g1, g2, Q, 0.5, 1.0, return_nodal=True)
    expect = np.where(np.array([0, 1, 1])[:, None] == np.array([0, 1])[None, :], 1.0, 0.5) * Q * Q
    np.testing.assert_allclose(x, expect, rtol=1e-14)


# ---- P3: regular, uniformly labeled graphs --------------------------------
def _cycle(n, label=0, e=1.0):
    return G(n, [label] * n, [(i, (i + 1) % n) for i in range(n)] if n > 2 else [(0, 1)],
             e=[e] * (n if n > 2 else 1))


def _complete(n, label=0, e=1.0):
    ed = [(i, j) for i in range(n) for j in range(i + 1, n)]
    return G(n, [label] * n, ed, e=[e] * len(ed))


def test_two_triangles_golden():
    t = _cycle(3)
    assert both(t, t, Q, 1.0, 1.0) == pytest.approx(GOLD["two_triangles_unlabeled"], rel=1e-13)


@pytest.mark.parametrize("n1,k1,n2,k2", [(5, 2, 4, 3), (6, 5, 7, 2), (3, 2, 6, 2)])
def test_regular_constant_kernels(n1, k1, n2, k2):
    # all vertex labels differ across the two graphs -> kappa_v == h everywhere;
    # all edges of G carry label e0, all of G' label e1 -> kappa_e == g everywhere.
    h, ls, e0, e1 = 0.4, 0.7, 1.0, 1.5
    g1 = _cycle(n1, 0, e0) if k1 == 2 else _complete(n1, 0, e0)
    g2 = _cycle(n2, 1, e1) if k2 == 2 else _complete(n2, 1, e1)
    gk = math.exp(-(e0 - e1) ** 2 / (2 * ls * ls))
    d1, d2 = k1 + Q, k2 + Q
    c = d1 * d2 * Q * Q / (d1 * d2 / h - k1 * k2 * gk)
    assert both(g1, g2, Q, h, ls) == pytest.approx(c, rel=1e-12)


# ---- P4: two single-edge graphs, 2x2 blocks --------------------------------
def test_single_edge_pair_closed_form():
    w1, w2, e1, e2 = (float(t) for t in f32([0.8, 1.3, 1.1, 1.6]))
    h, ls = 0.35, 0.6
    g1 = G(2, [0, 1], [(0, 1)], w=[w1], e=[e1])
    g2 = G(2, [1, 2], [(0, 1)], w=[w2], e=[e2])
    D = (w1 + Q) * (w2 + Q)
    c = w1 * w2 * math.exp(-(e1 - e2) ** 2 / (2 * ls * ls))
    kv = lambda a, b: 1.0 if a == b else h
    k00, k11 = kv(0, 1), kv(1, 2)     # block {(0,0),(1,1)}
    k01, k10 = kv(0, 2), kv(1, 1)     # block {(0,1),(1,0)}
    rhs = D * Q * Q

    def block(ka, kb):
        det = D * D / (ka * kb) - c * c
        return rhs * (D / kb + c) / det, rhs * (D / ka + c) / det

    x00, x11 = block(k00, k11)
    x01, x10 = block(k01, k10)
    K = 0.25 * (x00 + x11 + x01 + x10)
    assert both(g1, g2, Q, h, ls) == pytest.approx(K, rel=1e-13)
    _, x = O.kernel_value(g1, g2, Q, h, ls, return_nodal=True)
    np.testing.assert_allclose(x, [[x00, x01], [x10, x11]], rtol=1e-13)


# ---- P5 / P6: Appendix A series and explicit walks -------------------------
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_series_equals_direct_solve(seed):
    rng = np.random.default_rng(seed)
    g1 = random_graph(rng, int(rng.integers(3, 7)))
    g2 = random_graph(rng, int(rng.integers(3, 7)))
    h, ls = 0.5, 0.8
    # a larger q keeps the series short; the identity holds for any q > 0
    for q in (0.3, 0.05):
        direct = both(g1, g2, q, h, ls)
        series = O.kernel_series(g1, g2, q, h, ls)
        assert series == pytest.approx(direct, rel=1e-10)


def test_walk_enumeration_equals_series_terms():
    rng = np.random.default_rng(7)
    g1 = random_graph(rng, 4, prob=0.7)
    g2 = random_graph(rng, 3, prob=0.9)
    q, h, ls = 0.2, 0.5, 0.9
    walks = O.kernel_walks(g1, g2, q, h, ls, max_len=4)
    terms = O.series_terms(g1, g2, q, h, ls, n_terms=4)
    np.testing.assert_allclose(walks, terms, rtol=1e-12)
    # and the infinite sum of those terms is the direct solve
    many = O.series_terms(g1, g2, q, h, ls, n_terms=400)
    assert many.sum() == pytest.approx(O.kernel_value(g1, g2, q, h, ls), rel=1e-12)


def test_nonuniform_start_probability():
    rng = np.random.default_rng(11)
    g1 = random_graph(rng, 4, prob=0.7)
    g2 = random_graph(rng, 3, prob=0.9)
    p1 = rng.random(4); p1 /= p1.sum()
    p2 = rng.random(3); p2 /= p2.sum()
    q, h, ls = 0.2, 0.5, 0.9
    walks = O.kernel_walks(g1, g2, q, h, ls, max_len=3, p1=p1, p2=p2)
    terms = O.series_terms(g1, g2, q, h, ls, n_terms=3, p1=p1, p2=p2)
    np.testing.assert_allclose(walks, terms, rtol=1e-12)
    assert O.kernel_series(g1, g2, q, h, ls, p1=p1, p2=p2) == pytest.approx(
        O.kernel_value(g1, g2, q, h, ls, p1=p1, p2=p2), rel=1e-10)


def test_c_oracle_start_probabilities_over_a_batch():
    """The C edition slices a batch-wide array of starting probabilities per graph.  Four
    graphs of different sizes with non-uniform p: every pair, both tiers, against the numpy
    definition, and the explicit walk enumeration of Appendix A (first equation) must give
    the leading terms of each value.  A slice shifted by one vertex changes every number
    here (the sizes differ and no two probabilities are equal)."""
    from mgk_workloads.generators import _assemble
    rng = np.random.default_rng(31)
    sizes = [3, 4, 2, 5]
    graphs = [random_graph(rng, n, prob=0.8) for n in sizes]
    q, h, ls = 0.25, 0.5, 0.9
    wb = _assemble(graphs, W.KernelParams(q=q, h=h, length_scale=ls), "start")
    sp = np.concatenate([(lambda v: v / v.sum())(rng.uniform(0.2, 1.0, n)) for n in sizes])
    off = np.concatenate([[0], np.cumsum(sizes)])
    pi, pj = W.gram_pairs(len(sizes))
    d = C.pairs(wb, pi, pj, tier=0, start_prob=sp)
    m = C.pairs(wb, pi, pj, tier=1, start_prob=sp)
    for k, (i, j) in enumerate(zip(pi, pj)):
        p1, p2 = sp[off[i]:off[i + 1]], sp[off[j]:off[j + 1]]
        gi, gj = wb.graph(int(i)), wb.graph(int(j))
        ref = O.kernel_value(gi, gj, q, h, ls, p1=p1, p2=p2)
        assert d[k] == pytest.approx(ref, rel=1e-12)
        assert m[k] == pytest.approx(ref, rel=1e-10)
        # walks of up to 3 vertices: the first three terms of the series whose sum is K;
        # the rest is positive and bounded by the geometric tail (1 - q/d_max)^2 per step
        walks = O.kernel_walks(gi, gj, q, h, ls, max_len=3, p1=p1, p2=p2)
        assert walks.sum() < d[k]
        terms = O.series_terms(gi, gj, q, h, ls, n_terms=200, p1=p1, p2=p2)
        np.testing.assert_allclose(walks, terms[:3], rtol=1e-12)
        assert terms.sum() == pytest.approx(d[k], rel=1e-9)
    # uniform p is a different number on every pair
    assert np.all(np.abs(C.pairs(wb, pi, pj, tier=0) - d) > 1e-6 * d)


# ---- independent assembly with library Kronecker products ------------------
def test_dense_system_matches_kron_construction():
    rng = np.random.default_rng(3)
    g1 = random_graph(rng, 5)
    g2 = random_graph(rng, 4)
    q, h, ls = Q, 0.5, 0.8
    A1, E1 = O.dense_graph(g1)
    A2, E2 = O.dense_graph(g2)
    d = np.kron(A1.sum(1) + q, A2.sum(1) + q)
    v = np.where(g1[1][:, None] == g2[1][None, :], 1.0, h).reshape(-1)
    Ek = np.exp(-(E1[:, None, :, None] - E2[None, :, None, :]) ** 2 / (2 * ls * ls)).reshape(20, 20)
    S_ref = np.diag(d / v) - np.kron(A1, A2) * Ek
    S, b, px = O.assemble_system(g1, g2, q, h, ls)
    np.testing.assert_allclose(S, S_ref, rtol=1e-14, atol=1e-300)
    np.testing.assert_allclose(b, d * q * q, rtol=1e-14)
    assert O.kernel_value(g1, g2, q, h, ls) == pytest.approx(
        float(px @ np.linalg.solve(S_ref, d * q * q)), rel=1e-12)
    # the matrix-free operators (numpy and C) apply the same S
    u = rng.standard_normal(20)
    np.testing.assert_allclose(O.apply_system(g1, g2, q, h, ls, u), S_ref @ u, rtol=1e-12)
    np.testing.assert_allclose(C.apply(g1, g2, q, h, ls, u), S_ref @ u, rtol=1e-12)


def test_unlabeled_limit_is_random_walk_kernel():
    # h -> 1 and l -> infinity turn Eq. 1 into Eq. 2: (D_x - A_x) x = D_x q_x
    rng = np.random.default_rng(5)
    g1 = random_graph(rng, 6)
    g2 = random_graph(rng, 5)
    A1, _ = O.dense_graph(g1)
    A2, _ = O.dense_graph(g2)
    d = np.kron(A1.sum(1) + Q, A2.sum(1) + Q)
    x = np.linalg.solve(np.diag(d) - np.kron(A1, A2), d * Q * Q)
    k_rw = x.mean()
    assert both(g1, g2, Q, 1.0, 1e9) == pytest.approx(k_rw, rel=1e-10)


def test_zero_length_scale_limit_is_edgeless():
    # distinct edge labels and l -> 0: kappa_e -> 0, only the diagonal remains,
    # x_ii' = kv q^2 regardless of the degrees
    g1 = G(3, [0, 0, 1], [(0, 1), (1, 2)], e=[1.0, 2.0])
    g2 = G(2, [0, 1], [(0, 1)], e=[3.0])
    _, x = O.kernel_value(g1, g2, Q, 0.5, 1e-3, return_nodal=True)
    expect = np.where(np.array([0, 0, 1])[:, None] == np.array([0, 1])[None, :], 1.0, 0.5) * Q * Q
    np.testing.assert_allclose(x, expect, rtol=1e-12)


# ---- P7: kernel invariants --------------------------------------------------
def test_symmetry_and_permutation_invariance():
    b = W.config0()
    prm = b.params
    bp = W.permute_vertices(b, np.random.default_rng(9))
    for i in range(4):
        for j in range(i, 4):
            kij = O.kernel_value(b.graph(i), b.graph(j), prm.q, prm.h, prm.length_scale)
            kji = O.kernel_value(b.graph(j), b.graph(i), prm.q, prm.h, prm.length_scale)
            kpp = O.kernel_value(bp.graph(i), bp.graph(j), prm.q, prm.h, prm.length_scale)
            assert kji == pytest.approx(kij, rel=1e-12)
            assert kpp == pytest.approx(kij, rel=1e-12)


def test_gram_is_psd_and_cauchy_schwarz():
    b = W.config1(16)
    pi, pj = W.gram_pairs(16)
    vals = C.pairs(b, pi, pj, tier=0)
    K = np.zeros((16, 16))
    K[pi, pj] = vals
    K[pj, pi] = vals
    ev = np.linalg.eigvalsh(K)
    assert ev.min() >= -1e-10 * ev.max()
    dg = np.diag(K)
    assert (K * K <= np.outer(dg, dg) * (1 + 1e-12)).all()


# ---- P8: SPD / diagonal dominance -------------------------------------------
def test_system_is_strictly_diagonally_dominant():
    b = W.config0()
    prm = b.params
    S, _, _ = O.assemble_system(b.graph(1), b.graph(2), prm.q, prm.h, prm.length_scale)
    off = np.abs(S).sum(1) - np.abs(np.diag(S))
    assert (np.diag(S) > off).all()
    assert np.allclose(S, S.T, rtol=0, atol=0)
    assert np.diag(S).min() > 0 and (S - np.diag(np.diag(S)) <= 0).all()


def test_plus_sign_reading_of_alg1_is_not_eq1():
    # Alg. 1 prints "+" before the off-diagonal product; Eq. 1 and the appendix have "-".
    # The "+" matrix gives a different kernel value, so the pins above (series, walks,
    # closed forms) discriminate between the two readings.
    b = W.config0()
    prm = b.params
    S, rhs, px = O.assemble_system(b.graph(1), b.graph(2), prm.q, prm.h, prm.length_scale)
    S_plus = 2 * np.diag(np.diag(S)) - S
    k_minus = float(px @ np.linalg.solve(S, rhs))
    k_plus = float(px @ np.linalg.solve(S_plus, rhs))
    assert abs(k_plus - k_minus) > 0.05 * abs(k_minus)
    assert O.kernel_series(b.graph(1), b.graph(2), prm.q, prm.h, prm.length_scale) == pytest.approx(
        k_minus, rel=1e-10)


# ---- P11: the three oracle tiers agree on the benchmark configs -------------
def test_oracle_tiers_agree_on_config0_and_config1():
    b0 = W.config0()
    pi, pj = W.gram_pairs(4)
    ref = O.gram_values(b0, pi, pj)
    np.testing.assert_allclose(C.pairs(b0, pi, pj, tier=0), ref, rtol=1e-12)
    np.testing.assert_allclose(C.pairs(b0, pi, pj, tier=1), ref, rtol=1e-10)
    mf = [O.kernel_value_matrix_free(b0.graph(i), b0.graph(j), b0.params.q, b0.params.h,
                                     b0.params.length_scale) for i, j in zip(pi, pj)]
    np.testing.assert_allclose(mf, ref, rtol=1e-10)

    b1 = W.config1()
    rng = np.random.default_rng(1)
    sel = rng.choice(5050, size=40, replace=False)
    pi, pj = W.gram_pairs(100)
    d = C.pairs(b1, pi[sel], pj[sel], tier=0)
    m = C.pairs(b1, pi[sel], pj[sel], tier=1)
    np.testing.assert_allclose(m, d, rtol=1e-10)
    few = sel[:6]
    np.testing.assert_allclose(O.gram_values(b1, pi[few], pj[few]), d[:6], rtol=1e-12)


def test_c_oracle_rejects_bad_edges():
    g = G(2, [0, 0], [(0, 0)])
    with pytest.raises(RuntimeError):
        C.pair_nodal(g, g, Q, 0.5, 1.0)


def test_c_oracle_nodal_solution_matches_numpy():
    rng = np.random.default_rng(23)
    g1 = random_graph(rng, 7)
    g2 = random_graph(rng, 5)
    k0, x0 = O.kernel_value(g1, g2, Q, 0.5, 0.8, return_nodal=True)
    for tier in (0, 1):
        k1, x1 = C.pair_nodal(g1, g2, Q, 0.5, 0.8, tier=tier)
        assert k1 == pytest.approx(k0, rel=1e-10)
        np.testing.assert_allclose(x1, x0, rtol=1e-9)
    # x of (G', G) is the transpose
    _, xt = O.kernel_value(g2, g1, Q, 0.5, 0.8, return_nodal=True)
    np.testing.assert_allclose(xt.T, x0, rtol=1e-10)


# ---- P12: the other edge base kernels of Appendix B --------------------------
# Each closed form below takes the value of kappa_e from the kernel's textbook
# expression (never from the oracle's own evaluation of it).
WENDLAND_C2 = (1.0, 0.0, -10.0, 20.0, -15.0, 4.0)   # (1 - r)^4 (4 r + 1), expanded


def _wendland(r):
    return (1.0 - r) ** 4 * (4.0 * r + 1.0) if r < 1.0 else 0.0


def test_compact_polynomial_values_and_support():
    spec = O.EdgeKernel("poly", coef=WENDLAND_C2, rho=0.8)
    for d in (0.0, 0.1, 0.37, 0.79, 0.8, 0.81, 5.0):
        assert float(O.edge_kernel(1.0 + d, 1.0, spec)) == pytest.approx(_wendland(d / 0.8), abs=1e-14)
        assert float(O.edge_kernel(1.0, 1.0 + d, spec)) == pytest.approx(_wendland(d / 0.8), abs=1e-14)


@pytest.mark.parametrize("n1,k1,n2,k2", [(5, 2, 4, 3), (3, 2, 6, 2)])
def test_regular_graphs_with_each_edge_kernel(n1, k1, n2, k2):
    """Regular graphs, one label value per graph: kappa_e is one number g and
    K = d d' q^2 / (d d' / h - k k' g), whatever kernel produced g."""
    h, e0, e1 = 0.4, 1.0, 1.5
    d1, d2 = k1 + Q, k2 + Q
    closed = lambda g: d1 * d2 * Q * Q / (d1 * d2 / h - k1 * k2 * g)
    mk = lambda n, k, lab, e: _cycle(n, lab, e) if k == 2 else _complete(n, lab, e)
    # compact polynomial, inside and outside its support
    spec = O.EdgeKernel("poly", coef=WENDLAND_C2, rho=0.8)
    assert both(mk(n1, k1, 0, e0), mk(n2, k2, 1, e1), Q, h, spec) == pytest.approx(closed(_wendland(0.5 / 0.8)), rel=1e-12)
    spec = O.EdgeKernel("poly", coef=WENDLAND_C2, rho=0.4)
    assert both(mk(n1, k1, 0, e0), mk(n2, k2, 1, e1), Q, h, spec) == pytest.approx(closed(0.0), rel=1e-12)
    # Kronecker product of square exponentials over two attributes
    def attr(g, vals):
        n, lab, s, d, w, e = g
        return (n, lab, s, d, w, np.tile(f32(vals), (len(s), 1)))
    a, b = (1.0, 0.25), (1.5, -0.5)
    spec = O.EdgeKernel("kron_se", length_scales=(0.7, 1.3))
    gk = math.exp(-(a[0] - b[0]) ** 2 / (2 * 0.7 ** 2)) * math.exp(-(a[1] - b[1]) ** 2 / (2 * 1.3 ** 2))
    assert both(attr(mk(n1, k1, 0, 0.0), a), attr(mk(n2, k2, 1, 0.0), b), Q, h, spec) == pytest.approx(closed(gk), rel=1e-12)
    # R-convolution over two parts
    spec = O.EdgeKernel("rconv_se", length_scales=(0.9,), dim=2)
    gr = sum(math.exp(-(x - y) ** 2 / (2 * 0.9 ** 2)) for x in a for y in b) / 4.0
    assert both(attr(mk(n1, k1, 0, 0.0), a), attr(mk(n2, k2, 1, 0.0), b), Q, h, spec) == pytest.approx(closed(gr), rel=1e-12)


def test_edge_kernels_reduce_to_each_other():
    """Special cases: a one-attribute Kronecker product and a one-part R-convolution are
    the square exponential; two equal parts give the same R-convolution value as one;
    a polynomial of degree 0 is the constant kernel (the unlabeled limit with c = 1)."""
    rng = np.random.default_rng(12)
    g1, g2 = random_graph(rng, 5), random_graph(rng, 6)
    col = lambda g, reps: g[:5] + (np.repeat(np.asarray(g[5])[:, None], reps, axis=1),)
    ref = both(g1, g2, Q, 0.5, 0.8)
    assert both(col(g1, 1), col(g2, 1), Q, 0.5, O.EdgeKernel("kron_se", length_scales=(0.8,))) == pytest.approx(ref, rel=1e-12)
    assert both(col(g1, 1), col(g2, 1), Q, 0.5, O.EdgeKernel("rconv_se", length_scales=(0.8,), dim=1)) == pytest.approx(ref, rel=1e-12)
    assert both(col(g1, 2), col(g2, 2), Q, 0.5, O.EdgeKernel("rconv_se", length_scales=(0.8,), dim=2)) == pytest.approx(ref, rel=1e-12)
    # a second attribute that is the same on every edge does not change a Kronecker product
    two = lambda g: g[:5] + (np.stack([np.asarray(g[5]), np.full(len(g[5]), 0.3)], axis=1),)
    assert both(two(g1), two(g2), Q, 0.5, O.EdgeKernel("kron_se", length_scales=(0.8, 0.2))) == pytest.approx(ref, rel=1e-12)
    flat = both(g1, g2, Q, 0.5, 1e9)                      # kappa_e == 1
    assert both(g1, g2, Q, 0.5, O.EdgeKernel("poly", coef=(1.0,), rho=1e9)) == pytest.approx(flat, rel=1e-9)


@pytest.mark.parametrize("kind", ["poly", "kron_se", "rconv_se"])
def test_walk_sum_and_series_with_each_edge_kernel(kind):
    """Appendix A: the explicit sum over walk pairs and the matrix series give the
    value of Eq. 1 for any edge kernel; symmetric in its arguments."""
    rng = np.random.default_rng(5)
    g1, g2 = random_graph(rng, 4, 0.6), random_graph(rng, 3, 0.7)
    if kind == "poly":
        spec = O.EdgeKernel("poly", coef=WENDLAND_C2, rho=1.5)
    else:
        D = 2
        ext = lambda g: g[:5] + (f32(rng.uniform(0.0, 2.0, (len(g[2]), D))),)
        g1, g2 = ext(g1), ext(g2)
        spec = (O.EdgeKernel("kron_se", length_scales=(0.6, 1.1)) if kind == "kron_se"
                else O.EdgeKernel("rconv_se", length_scales=(0.7,), dim=D))
    q = 0.4
    K = both(g1, g2, q, 0.5, spec)
    assert O.kernel_series(g1, g2, q, 0.5, spec) == pytest.approx(K, rel=1e-12)
    walks = O.kernel_walks(g1, g2, q, 0.5, spec, 4)
    terms = O.series_terms(g1, g2, q, 0.5, spec, 4)
    np.testing.assert_allclose(walks, terms, rtol=1e-12)
    assert both(g2, g1, q, 0.5, spec) == pytest.approx(K, rel=1e-12)
    assert O.kernel_value_matrix_free(g1, g2, q, 0.5, spec) == pytest.approx(K, rel=1e-10)
