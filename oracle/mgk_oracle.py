"""Plain fp64 CPU oracle for the marginalized graph kernel.  TEST INFRASTRUCTURE.

This file is the checker, not the product: only the tests, the smoke entry and
the CPU-baseline leg of the benchmark may import it.  It shares no code with
the HIP path and never imports it.

What it computes is the definition itself (paper Eq. 1, Section II-B): for two
labeled graphs G, G' the dense N x N system (N = n n')

    S = D_x V_x^{-1} - A_x (.) E_x ,   b = D_x q_x ,   K = p_x^T S^{-1} b

is assembled entry by entry and solved with a library direct solver.  Because
the method in the paper (preconditioned CG, Alg. 1) converges to the unique
solution of this SPD system, the oracle is the definition, not the iteration.

Readings of the paper taken here (each also listed in the design notes):
  * product index of (i, i') is i * n' + i' (Definition 6 prints the first
    operand's size; the block matrix above it fixes the second operand's).
  * d_i = sum_j A_ij + q_i literally (Eq. 1 bullet list), q_i = q on all
    vertices, p_i = 1/n unless start probabilities are given.
  * square-exponential edge kernel exp(-alpha (e-e')^2) (Appendix B) with
    alpha = 1 / (2 l^2) for length scale l.
  * vertex kernel: 1 if labels are equal, else h, 0 < h <= 1.
  * absent edges are decided by A_ij = 0 only.

Second, independent routes to the same number, used to pin the first:
  * ``kernel_series``  - the fixed-point form r = q_x + [(P (x) P') (.) E_x] V_x r,
    K = p_x^T V_x r (Appendix A, matrix form), summed term by term.
  * ``kernel_walks``   - the explicit sum over pairs of equal-length walks
    (Appendix A, first equation), by brute-force enumeration.
  * ``kernel_value_matrix_free`` - S applied edge by edge without forming it,
    CG to a tight tolerance (for sizes where S cannot be stored).
"""
from __future__ import annotations

import itertools
from typing import Optional, Sequence, Tuple

import numpy as np

Graph = Tuple[int, np.ndarray, np.ndarray, np.ndarray, np.ndarray, np.ndarray]
# (n, vertex_label[n], src[m], dst[m], weight[m], edge_label[m]); each undirected edge once


# ---------------------------------------------------------------- base kernels
def vertex_kernel(a, b, h: float):
    """kappa_v: 1 where labels are equal, h elsewhere (range (0, 1], Section II-B)."""
    return np.where(np.asarray(a) == np.asarray(b), 1.0, float(h))


class EdgeKernel:
    """An edge base kernel other than the plain square exponential (the list of
    examples in Appendix B).  Passed wherever the functions below take
    ``length_scale``; a bare number there means the square-exponential kernel.

    kind "poly":     compact polynomial radial basis kernel on scalar labels,
                     sum_i coef[i] r^i for r = |e1 - e2| / rho < 1, and 0 from
                     r = 1 on (compact support).
    kind "kron_se":  Kronecker-product kernel over labels with D attributes,
                     prod_a exp(-(e1_a - e2_a)^2 / (2 l_a^2)), one length
                     scale per attribute.
    kind "rconv_se": R-convolution kernel over labels made of D parts,
                     (1 / D^2) sum_a sum_b exp(-(e1_a - e2_b)^2 / (2 l^2));
                     the factor 1 / D^2 keeps the range inside [0, 1].
    """

    def __init__(self, kind: str, coef=(), rho: float = 1.0, length_scales=(), dim: int = 0):
        if kind not in ("poly", "kron_se", "rconv_se"):
            raise ValueError("unknown edge kernel " + kind)
        self.kind = kind
        self.coef = tuple(float(c) for c in coef)
        self.rho = float(rho)
        self.length_scales = tuple(float(l) for l in length_scales)
        self.dim = int(dim) if dim else (len(self.length_scales) if kind == "kron_se" else 1)


def edge_kernel(e1, e2, length_scale):
    """kappa_e.  Square exponential exp(-alpha (e1 - e2)^2), alpha = 1/(2 l^2), when
    ``length_scale`` is a number; otherwise the kernel an EdgeKernel describes
    (Appendix B).  Labels with attributes carry them on the last axis."""
    a = np.asarray(e1, dtype=np.float64)
    b = np.asarray(e2, dtype=np.float64)
    if not isinstance(length_scale, EdgeKernel):
        alpha = 1.0 / (2.0 * float(length_scale) ** 2)
        d = a - b
        return np.exp(-alpha * d * d)
    spec = length_scale
    if spec.kind == "poly":
        r = np.abs(a - b) / spec.rho
        val = np.zeros_like(r)
        for i, c in enumerate(spec.coef):
            val = val + c * r ** i
        return np.where(r < 1.0, val, 0.0)
    if spec.kind == "kron_se":
        out = 1.0
        for k, l in enumerate(spec.length_scales):
            d = a[..., k] - b[..., k]
            out = out * np.exp(-d * d / (2.0 * l * l))
        return out
    # rconv_se
    (l,) = spec.length_scales
    D = a.shape[-1]
    out = 0.0
    for i in range(D):
        for j in range(D):
            d = a[..., i] - b[..., j]
            out = out + np.exp(-d * d / (2.0 * l * l))
    return out / float(D * D)


# ---------------------------------------------------------------- per-graph matrices
def dense_graph(g: Graph):
    """Symmetric adjacency matrix A and edge-label matrix E (Definitions 4, 5)."""
    n, _lab, src, dst, w, e = g
    e = np.asarray(e, dtype=np.float64)
    A = np.zeros((n, n), dtype=np.float64)
    E = np.zeros((n, n) + e.shape[1:], dtype=np.float64)   # attributes, if any, on the last axis
    for s, d, ww, ee in zip(src, dst, w, e):
        s = int(s); d = int(d)
        if s == d:
            raise ValueError("self loop")
        if A[s, d] != 0.0:
            raise ValueError("duplicate edge")
        A[s, d] = A[d, s] = float(ww)
        E[s, d] = E[d, s] = ee
    return A, E


def degree(A: np.ndarray, q: float) -> np.ndarray:
    """d_i = sum_j A_ij + q_i (Eq. 1, definition of D_x)."""
    return A.sum(axis=1) + q


def start_probability(n: int, p: Optional[np.ndarray]) -> np.ndarray:
    return np.full(n, 1.0 / n) if p is None else np.asarray(p, dtype=np.float64)


# ---------------------------------------------------------------- Eq. 1, dense
def assemble_system(g1: Graph, g2: Graph, q: float, h: float, length_scale: float,
                    p1: Optional[np.ndarray] = None, p2: Optional[np.ndarray] = None):
    """Dense S, right-hand side b = D_x q_x and start vector p_x of Eq. 1."""
    n1, n2 = g1[0], g2[0]
    A1, E1 = dense_graph(g1)
    A2, E2 = dense_graph(g2)
    d1, d2 = degree(A1, q), degree(A2, q)
    N = n1 * n2
    S = np.zeros((N, N), dtype=np.float64)
    for i in range(n1):
        for ip in range(n2):
            row = i * n2 + ip
            kv = float(vertex_kernel(g1[1][i], g2[1][ip], h))
            S[row, row] = d1[i] * d2[ip] / kv
            for j in np.flatnonzero(A1[i]):
                nbr = np.flatnonzero(A2[ip])
                ke = edge_kernel(E1[i, j], E2[ip, nbr], length_scale)
                S[row, j * n2 + nbr] = -A1[i, j] * A2[ip, nbr] * ke
    qx = np.full(N, q * q)
    b = np.kron(d1, d2) * qx
    px = np.kron(start_probability(n1, p1), start_probability(n2, p2))
    return S, b, px


def kernel_value(g1: Graph, g2: Graph, q: float, h: float, length_scale: float,
                 p1=None, p2=None, return_nodal: bool = False):
    """K(G, G') = p_x^T S^{-1} D_x q_x by dense direct solve (Eq. 1).

    The Cholesky factorisation doubles as a check that S is SPD (Section II-B);
    it raises if the assembled matrix is not.
    """
    S, b, px = assemble_system(g1, g2, q, h, length_scale, p1, p2)
    L = np.linalg.cholesky(S)
    y = np.linalg.solve(L, b)
    x = np.linalg.solve(L.T, y)
    K = float(px @ x)
    if return_nodal:
        return K, x.reshape(g1[0], g2[0])
    return K


# ---------------------------------------------------------------- Appendix A, matrix form
def kernel_series(g1: Graph, g2: Graph, q: float, h: float, length_scale: float,
                  p1=None, p2=None, tol: float = 1e-16, max_terms: int = 200000):
    """Sum the fixed-point form term by term:
    r = sum_k T^k q_x, T = [(P (x) P') (.) E_x] V_x, P = D^{-1} A;  K = p_x^T V_x r."""
    n1, n2 = g1[0], g2[0]
    A1, E1 = dense_graph(g1)
    A2, E2 = dense_graph(g2)
    P1 = A1 / degree(A1, q)[:, None]
    P2 = A2 / degree(A2, q)[:, None]
    V = vertex_kernel(np.asarray(g1[1])[:, None], np.asarray(g2[1])[None, :], h)  # n1 x n2
    px = np.outer(start_probability(n1, p1), start_probability(n2, p2))
    # T applied to a vector u (kept as an n1 x n2 array): (T u)_{ii'} =
    #   sum_{j j'} P_ij P'_i'j' kappa_e(E_ij, E'_i'j') V_jj' u_jj'
    edges1 = [(i, j) for i in range(n1) for j in np.flatnonzero(A1[i])]

    def apply_T(u):
        vu = V * u
        out = np.zeros_like(u)
        for (i, j) in edges1:
            for ip in range(n2):
                nbr = np.flatnonzero(A2[ip])
                if len(nbr) == 0:
                    continue
                ke = edge_kernel(E1[i, j], E2[ip, nbr], length_scale)
                out[i, ip] += P1[i, j] * np.sum(P2[ip, nbr] * ke * vu[j, nbr])
        return out

    term = np.full((n1, n2), q * q)
    K = 0.0
    for _ in range(max_terms):
        contrib = float(np.sum(px * V * term))
        K += contrib
        if abs(contrib) <= tol * abs(K):
            break
        term = apply_T(term)
    return K


# ---------------------------------------------------------------- Appendix A, walk sum
def kernel_walks(g1: Graph, g2: Graph, q: float, h: float, length_scale: float,
                 max_len: int, p1=None, p2=None) -> np.ndarray:
    """Partial sums of the random-walk definition: entry l-1 holds the sum over
    all pairs of walks with exactly l vertices (l = 1..max_len).  Transition
    probability P_ij = A_ij / d_i, stopping probability q on every vertex."""
    n1, n2 = g1[0], g2[0]
    A1, E1 = dense_graph(g1)
    A2, E2 = dense_graph(g2)
    d1, d2 = degree(A1, q), degree(A2, q)
    ps1, ps2 = start_probability(n1, p1), start_probability(n2, p2)
    lab1, lab2 = g1[1], g2[1]

    def walks(A, n, length):
        if length == 1:
            return [(v,) for v in range(n)]
        out = []
        for wk in walks(A, n, length - 1):
            for nxt in np.flatnonzero(A[wk[-1]]):
                out.append(wk + (int(nxt),))
        return out

    sums = np.zeros(max_len)
    for length in range(1, max_len + 1):
        total = 0.0
        for w1 in walks(A1, n1, length):
            pr1 = ps1[w1[0]] * q
            for a, b in zip(w1[:-1], w1[1:]):
                pr1 *= A1[a, b] / d1[a]
            for w2 in walks(A2, n2, length):
                pr2 = ps2[w2[0]] * q
                for a, b in zip(w2[:-1], w2[1:]):
                    pr2 *= A2[a, b] / d2[a]
                sim = float(vertex_kernel(lab1[w1[0]], lab2[w2[0]], h))
                for k in range(1, length):
                    sim *= float(vertex_kernel(lab1[w1[k]], lab2[w2[k]], h))
                    sim *= float(edge_kernel(E1[w1[k - 1], w1[k]], E2[w2[k - 1], w2[k]],
                                             length_scale))
                total += pr1 * pr2 * sim
        sums[length - 1] = total
    return sums


def series_terms(g1: Graph, g2: Graph, q: float, h: float, length_scale: float,
                 n_terms: int, p1=None, p2=None) -> np.ndarray:
    """First n_terms terms p_x^T V_x T^k q_x of the matrix series, k = 0..n_terms-1,
    formed with a dense T (tiny graphs only)."""
    n1, n2 = g1[0], g2[0]
    A1, E1 = dense_graph(g1)
    A2, E2 = dense_graph(g2)
    P1 = A1 / degree(A1, q)[:, None]
    P2 = A2 / degree(A2, q)[:, None]
    N = n1 * n2
    T = np.zeros((N, N))
    v = np.zeros(N)
    for i in range(n1):
        for ip in range(n2):
            v[i * n2 + ip] = float(vertex_kernel(g1[1][i], g2[1][ip], h))
    for i in range(n1):
        for ip in range(n2):
            for j in range(n1):
                for jp in range(n2):
                    if A1[i, j] != 0.0 and A2[ip, jp] != 0.0:
                        T[i * n2 + ip, j * n2 + jp] = (
                            P1[i, j] * P2[ip, jp]
                            * float(edge_kernel(E1[i, j], E2[ip, jp], length_scale))
                            * v[j * n2 + jp])
    px = np.kron(start_probability(n1, p1), start_probability(n2, p2))
    term = np.full(N, q * q)
    out = np.zeros(n_terms)
    for k in range(n_terms):
        out[k] = float(px @ (v * term))
        term = T @ term
    return out


# ---------------------------------------------------------------- matrix-free tier
def _directed_edges(g: Graph):
    n, _lab, src, dst, w, e = g
    s = np.concatenate([src, dst]).astype(np.int64)
    d = np.concatenate([dst, src]).astype(np.int64)
    ww = np.concatenate([w, w]).astype(np.float64)
    ee = np.concatenate([e, e], axis=0).astype(np.float64)
    return s, d, ww, ee


def apply_system(g1: Graph, g2: Graph, q: float, h: float, length_scale: float,
                 u: np.ndarray) -> np.ndarray:
    """S u without forming S: diagonal term minus the edge-pair sum (Eq. 1; Alg. 2)."""
    n1, n2 = g1[0], g2[0]
    s1, t1, w1, e1 = _directed_edges(g1)
    s2, t2, w2, e2 = _directed_edges(g2)
    d1 = np.bincount(s1, weights=w1, minlength=n1) + q
    d2 = np.bincount(s2, weights=w2, minlength=n2) + q
    V = vertex_kernel(np.asarray(g1[1])[:, None], np.asarray(g2[1])[None, :], h)
    U = u.reshape(n1, n2)
    out = np.outer(d1, d2) / V * U
    for k in range(len(s1)):
        ke = edge_kernel(e1[k], e2, length_scale)
        contrib = w1[k] * w2 * ke * U[t1[k], t2]
        np.subtract.at(out[s1[k]], s2, contrib)
    return out.reshape(-1)


def kernel_value_matrix_free(g1: Graph, g2: Graph, q: float, h: float, length_scale: float,
                             p1=None, p2=None, rtol: float = 1e-13, max_iter: int = 100000):
    """Same K as ``kernel_value`` by unpreconditioned CG on the matrix-free operator."""
    n1, n2 = g1[0], g2[0]
    s1, _t1, w1, _e1 = _directed_edges(g1)
    s2, _t2, w2, _e2 = _directed_edges(g2)
    d1 = np.bincount(s1, weights=w1, minlength=n1) + q
    d2 = np.bincount(s2, weights=w2, minlength=n2) + q
    b = np.kron(d1, d2) * q * q
    px = np.kron(start_probability(n1, p1), start_probability(n2, p2))
    x = np.zeros_like(b)
    r = b.copy()
    p = r.copy()
    rr = float(r @ r)
    bb = rr
    for _ in range(max_iter):
        if rr <= rtol * rtol * bb:
            break
        a = apply_system(g1, g2, q, h, length_scale, p)
        alpha = rr / float(p @ a)
        x += alpha * p
        r -= alpha * a
        rr_new = float(r @ r)
        p = r + (rr_new / rr) * p
        rr = rr_new
    return float(px @ x)


# ---------------------------------------------------------------- batches
def gram_values(batch, pairs_i: Sequence[int], pairs_j: Sequence[int]) -> np.ndarray:
    """Kernel values for the listed pairs of a GraphBatch-like object exposing
    ``graph(g)`` and ``params`` (q, h, and the edge kernel: length_scale, or
    edge_kernel / poly_coef / poly_rho / length_scales)."""
    prm = batch.params
    spec = edge_kernel_of(prm)
    out = np.zeros(len(pairs_i))
    for k, (i, j) in enumerate(zip(pairs_i, pairs_j)):
        out[k] = kernel_value(batch.graph(int(i)), batch.graph(int(j)), prm.q, prm.h, spec)
    return out


def edge_kernel_of(prm):
    """The ``length_scale`` argument of the functions above for a parameter record."""
    kind = getattr(prm, "edge_kernel", "se")
    if kind == "se":
        return prm.length_scale
    if kind == "poly":
        return EdgeKernel("poly", coef=prm.poly_coef, rho=prm.poly_rho)
    return EdgeKernel(kind, length_scales=prm.length_scales, dim=getattr(prm, "label_dim", 0))
