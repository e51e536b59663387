"""Seeded generators for the five benchmark configurations and the paper's two
synthetic graph families.

A batch of graphs is stored in the flat form the C-ABI loader takes:
``vtx_off[G+1]``, ``vtx_label[sum n]``, ``edge_off[G+1]`` and per-edge
``src < dst`` (vertex ids local to the graph), ``weight`` and ``edge_label``.
Undirected edges are listed once.  Nothing here evaluates a base kernel or
touches the linear system; it only draws graphs.

The paper's real datasets (Section "Real-World Dataset") are not available;
the molecule-like and geometric families stand in for their shapes: bounded
degree trees with a few ring closures for SMILES-derived molecular graphs,
3-D spatial-cutoff graphs with distance labels for protein contact graphs.
The Newman-Watts-Strogatz and Barabasi-Albert families follow the parameters
the paper states for its synthetic benchmark (160 graphs of 96 nodes, k=3
p=0.1, m=6).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Optional, Sequence, Tuple

import numpy as np

SEED_BASE = 19100631


@dataclass
class KernelParams:
    """Hyper-parameters of the marginalized graph kernel for a workload."""

    q: float = 0.05            # stopping probability, same on every vertex
    h: float = 0.5             # vertex delta kernel: 1 if labels equal else h
    length_scale: float = 1.0  # square-exponential edge kernel length scale
    # edge base kernel: "se" (square exponential, length_scale), "poly" (compact polynomial:
    # poly_coef, support radius poly_rho), "kron_se" (product of square exponentials over
    # label_dim attributes, one of length_scales each), "rconv_se" (R-convolution over
    # label_dim parts, length_scales[0])
    edge_kernel: str = "se"
    poly_coef: Tuple[float, ...] = ()
    poly_rho: float = 1.0
    length_scales: Tuple[float, ...] = ()
    label_dim: int = 1


@dataclass
class GraphBatch:
    vtx_off: np.ndarray     # int64 [G+1]
    vtx_label: np.ndarray   # int32 [sum n]
    edge_off: np.ndarray    # int64 [G+1]
    src: np.ndarray         # int32 [sum m], src < dst
    dst: np.ndarray         # int32 [sum m]
    weight: np.ndarray      # float32 [sum m], > 0
    edge_label: np.ndarray  # float32 [sum m]
    params: KernelParams = field(default_factory=KernelParams)
    name: str = ""

    @property
    def n_graphs(self) -> int:
        return len(self.vtx_off) - 1

    def n_vertices(self, g: int) -> int:
        return int(self.vtx_off[g + 1] - self.vtx_off[g])

    def n_edges(self, g: int) -> int:
        return int(self.edge_off[g + 1] - self.edge_off[g])

    def graph(self, g: int):
        """(n, labels, src, dst, weight, edge_label) views of graph ``g``."""
        v0, v1 = int(self.vtx_off[g]), int(self.vtx_off[g + 1])
        e0, e1 = int(self.edge_off[g]), int(self.edge_off[g + 1])
        return (v1 - v0, self.vtx_label[v0:v1], self.src[e0:e1], self.dst[e0:e1],
                self.weight[e0:e1], self.edge_label[e0:e1])

    def sizes(self) -> np.ndarray:
        return np.diff(self.vtx_off).astype(np.int64)

    def nnz(self) -> np.ndarray:
        """Stored nonzeros of the symmetric adjacency matrix (2 per edge)."""
        return 2 * np.diff(self.edge_off).astype(np.int64)

    def subset(self, idx: Sequence[int]) -> "GraphBatch":
        return _assemble([self.graph(int(g)) for g in idx], self.params, self.name)


def _assemble(graphs, params: KernelParams, name: str) -> GraphBatch:
    vtx_off = [0]
    edge_off = [0]
    labels, srcs, dsts, ws, es = [], [], [], [], []
    for (n, lab, s, d, w, e) in graphs:
        vtx_off.append(vtx_off[-1] + int(n))
        edge_off.append(edge_off[-1] + len(s))
        labels.append(np.asarray(lab, dtype=np.int32))
        srcs.append(np.asarray(s, dtype=np.int32))
        dsts.append(np.asarray(d, dtype=np.int32))
        ws.append(np.asarray(w, dtype=np.float32))
        es.append(np.asarray(e, dtype=np.float32))

    def cat(parts, dt):
        return np.concatenate(parts).astype(dt) if parts else np.zeros(0, dt)

    return GraphBatch(
        vtx_off=np.asarray(vtx_off, dtype=np.int64),
        vtx_label=cat(labels, np.int32),
        edge_off=np.asarray(edge_off, dtype=np.int64),
        src=cat(srcs, np.int32), dst=cat(dsts, np.int32),
        weight=cat(ws, np.float32), edge_label=cat(es, np.float32),
        params=params, name=name)


def concat_batches(batches: Sequence[GraphBatch], params: Optional[KernelParams] = None,
                   name: str = "") -> GraphBatch:
    graphs = []
    for b in batches:
        graphs += [b.graph(g) for g in range(b.n_graphs)]
    return _assemble(graphs, params or batches[0].params, name)


def permute_vertices(batch: GraphBatch, rng: np.random.Generator) -> GraphBatch:
    """Relabel the vertices of every graph by a random permutation (edge order
    is shuffled as well).  The kernel value of any pair is unchanged."""
    graphs = []
    for g in range(batch.n_graphs):
        n, lab, s, d, w, e = batch.graph(g)
        perm = rng.permutation(n)          # old id -> new id
        new_lab = np.empty(n, dtype=np.int32)
        new_lab[perm] = lab
        ns, nd = perm[s], perm[d]
        lo, hi = np.minimum(ns, nd), np.maximum(ns, nd)
        order = rng.permutation(len(lo))
        graphs.append((n, new_lab, lo[order], hi[order], w[order], e[order]))
    return _assemble(graphs, batch.params, batch.name + "+perm")


def with_label_attributes(batch: GraphBatch, rng: np.random.Generator, dim: int, spread: float = 0.3,
                          params: Optional[KernelParams] = None) -> GraphBatch:
    """The same graphs with ``dim`` attributes per edge label: attribute 0 is the
    existing label, the others are drawn around it (normal, standard deviation
    ``spread``), as for a bond described by several correlated measurements."""
    base = np.asarray(batch.edge_label, dtype=np.float32).reshape(-1, 1)
    extra = base + rng.normal(0.0, spread, (len(base), dim - 1)).astype(np.float32)
    lab = np.concatenate([base, extra], axis=1).astype(np.float32)
    return GraphBatch(batch.vtx_off, batch.vtx_label, batch.edge_off, batch.src, batch.dst,
                      batch.weight, lab, params or batch.params, batch.name + "+attr%d" % dim)


def gram_pairs(n_graphs: int) -> Tuple[np.ndarray, np.ndarray]:
    """All unordered pairs (i <= j) of a Gram matrix, row-major upper triangle."""
    i, j = np.triu_indices(n_graphs)
    return i.astype(np.int32), j.astype(np.int32)


# --------------------------------------------------------------------------
# families
# --------------------------------------------------------------------------

def _er_graph(rng, n, prob, w_lo, w_hi, e_lo, e_hi, n_vlabels, w_min=0.0):
    iu, ju = np.triu_indices(n, k=1)
    keep = rng.random(len(iu)) < prob
    s, d = iu[keep], ju[keep]
    w = rng.uniform(w_lo, w_hi, size=len(s))
    while True:  # redraw weights that are numerically zero
        bad = w <= w_min
        if not bad.any():
            break
        w[bad] = rng.uniform(w_lo, w_hi, size=int(bad.sum()))
    e = rng.uniform(e_lo, e_hi, size=len(s))
    lab = rng.integers(0, n_vlabels, size=n)
    return (n, lab, s, d, w, e)


def erdos_renyi_batch(rng, n_graphs, n_lo, n_hi, prob, w_range, e_range, n_vlabels,
                      params, name="er", w_min=0.0) -> GraphBatch:
    graphs = []
    for _ in range(n_graphs):
        n = int(rng.integers(n_lo, n_hi + 1))
        graphs.append(_er_graph(rng, n, prob, w_range[0], w_range[1],
                                e_range[0], e_range[1], n_vlabels, w_min))
    return _assemble(graphs, params, name)


_MOL_LABEL_P = np.array([0.55, 0.15, 0.15, 0.10, 0.05])


def _molecule_graph(rng, n):
    """Random tree of maximum degree 4 plus 0-3 ring-closing edges."""
    deg = np.zeros(n, dtype=np.int64)
    adj = set()
    s, d = [], []
    for t in range(1, n):
        cand = np.flatnonzero(deg[:t] < 4)
        u = int(cand[rng.integers(0, len(cand))])
        s.append(u); d.append(t)
        adj.add((u, t))
        deg[u] += 1; deg[t] += 1
    rings = int(rng.integers(0, 4))
    for _ in range(rings):
        for _try in range(100):
            a, b = (int(x) for x in rng.integers(0, n, size=2))
            if a == b:
                continue
            lo, hi = min(a, b), max(a, b)
            if (lo, hi) in adj or deg[lo] >= 4 or deg[hi] >= 4:
                continue
            adj.add((lo, hi)); s.append(lo); d.append(hi)
            deg[lo] += 1; deg[hi] += 1
            break
    m = len(s)
    w = np.ones(m)
    e = np.clip(rng.normal(1.4, 0.1, size=m), 1.0, 1.8)
    lab = rng.choice(5, size=n, p=_MOL_LABEL_P)
    return (n, lab, np.asarray(s), np.asarray(d), w, e)


def molecule_like_batch(rng, n_graphs, n_lo, n_hi, params, name="mol") -> GraphBatch:
    graphs = []
    for _ in range(n_graphs):
        n = int(rng.integers(n_lo, n_hi + 1))
        graphs.append(_molecule_graph(rng, n))
    return _assemble(graphs, params, name)


def _geometric_edges(pts, rc):
    from scipy.spatial import cKDTree
    tree = cKDTree(pts)
    pairs = tree.query_pairs(rc, output_type="ndarray")
    s, d = pairs[:, 0], pairs[:, 1]
    lo, hi = np.minimum(s, d), np.maximum(s, d)
    dist = np.linalg.norm(pts[lo] - pts[hi], axis=1)
    return lo, hi, dist


def morton_rank(pts: np.ndarray, bits: int = 10) -> np.ndarray:
    """Position of each point of the unit cube along the Morton (Z-order) curve:
    the coordinates are quantised to ``bits`` bits and their bits interleaved."""
    q = np.minimum((np.asarray(pts) * (1 << bits)).astype(np.int64), (1 << bits) - 1)
    key = np.zeros(len(q), dtype=np.int64)
    for b in range(bits):
        for axis in range(q.shape[1]):
            key |= ((q[:, axis] >> b) & 1) << (q.shape[1] * b + axis)
    rank = np.empty(len(q), dtype=np.int64)
    rank[np.argsort(key, kind="stable")] = np.arange(len(q))
    return rank


def geometric_batch(rng, n_graphs, n, mean_degree, n_vlabels, params, name="geo",
                    order: str = "random") -> GraphBatch:
    """Points uniform in the unit cube, edge iff distance < r_c.  r_c is
    calibrated once on the first point set so the mean degree is within 0.3 of
    the request, then used for every graph.  weight = exp(-dist), label = dist.
    ``order``: "random" numbers the points in the draw order (no spatial
    locality); "morton" numbers them along the Morton curve through the cube,
    the space-filling-curve ordering for graphs that come with an embedding.
    Both give the same graphs up to the numbering."""
    graphs = []
    coords = []
    rc = (3.0 * mean_degree / (4.0 * np.pi * n)) ** (1.0 / 3.0)
    calibrated = False
    for _ in range(n_graphs):
        pts = rng.random((n, 3))
        if not calibrated:
            for _it in range(60):
                lo, hi, dist = _geometric_edges(pts, rc)
                md = 2.0 * len(lo) / n
                if abs(md - mean_degree) <= 0.3:
                    break
                rc *= (mean_degree / max(md, 1e-9)) ** (1.0 / 3.0)
            calibrated = True
        lo, hi, dist = _geometric_edges(pts, rc)
        lab = rng.integers(0, n_vlabels, size=n)
        if order == "morton":
            rank = morton_rank(pts)
            new_lab = np.empty_like(lab)
            new_lab[rank] = lab
            a, b = rank[lo], rank[hi]
            lab, lo, hi = new_lab, np.minimum(a, b), np.maximum(a, b)
            moved = np.empty_like(pts)
            moved[rank] = pts
            pts = moved
        elif order != "random":
            raise ValueError("order must be random or morton")
        graphs.append((n, lab, lo, hi, np.exp(-dist), dist))
        coords.append(pts.astype(np.float32))
    b = _assemble(graphs, params, name)
    b.cutoff = rc  # type: ignore[attr-defined]
    b.coords = np.concatenate(coords)  # type: ignore[attr-defined]   # [sum n, 3], in the numbering of the batch
    return b


def newman_watts_strogatz_batch(rng, n_graphs, n, k, p, n_vlabels, params, name="nws"):
    """Ring lattice where each vertex joins its k nearest neighbours (k//2 on
    each side, at least one), plus a shortcut per lattice edge with prob. p."""
    half = max(1, k // 2)
    graphs = []
    for _ in range(n_graphs):
        adj = set()
        for u in range(n):
            for t in range(1, half + 1):
                v = (u + t) % n
                adj.add((min(u, v), max(u, v)))
        for (u, v) in sorted(adj):
            if rng.random() < p:
                for _try in range(50):
                    w = int(rng.integers(0, n))
                    key = (min(u, w), max(u, w))
                    if w != u and key not in adj:
                        adj.add(key)
                        break
        ed = np.array(sorted(adj), dtype=np.int64)
        m = len(ed)
        graphs.append((n, rng.integers(0, n_vlabels, size=n), ed[:, 0], ed[:, 1],
                       np.ones(m), rng.uniform(0.0, 1.0, size=m)))
    return _assemble(graphs, params, name)


def barabasi_albert_batch(rng, n_graphs, n, m_attach, n_vlabels, params, name="ba"):
    """Preferential attachment: each new vertex links to m distinct earlier
    vertices drawn with probability proportional to degree."""
    graphs = []
    for _ in range(n_graphs):
        targets = list(range(m_attach))
        repeated: List[int] = []
        s, d = [], []
        for v in range(m_attach, n):
            for t in targets:
                s.append(min(t, v)); d.append(max(t, v))
            repeated.extend(targets)
            repeated.extend([v] * m_attach)
            chosen = set()
            while len(chosen) < m_attach:
                chosen.add(repeated[int(rng.integers(0, len(repeated)))])
            targets = sorted(chosen)
        m = len(s)
        graphs.append((n, rng.integers(0, n_vlabels, size=n), np.asarray(s), np.asarray(d),
                       np.ones(m), rng.uniform(0.0, 1.0, size=m)))
    return _assemble(graphs, params, name)


# --------------------------------------------------------------------------
# the five configurations
# --------------------------------------------------------------------------

def config0() -> GraphBatch:
    """4 Erdos-Renyi graphs of 6-10 vertices, edge prob 0.3, weights U(0.5,1),
    3 vertex labels (h=0.5), edge labels U(1,2) (length scale 1), q=0.05."""
    rng = np.random.default_rng(SEED_BASE + 0)
    return erdos_renyi_batch(rng, 4, 6, 10, 0.3, (0.5, 1.0), (1.0, 2.0), 3,
                             KernelParams(q=0.05, h=0.5, length_scale=1.0), "config0")


def config1(n_graphs: int = 100) -> GraphBatch:
    """100 molecule-like graphs of 10-40 vertices, h=0.3, length scale 0.1."""
    rng = np.random.default_rng(SEED_BASE + 1)
    return molecule_like_batch(rng, n_graphs, 10, 40,
                               KernelParams(q=0.05, h=0.3, length_scale=0.1), "config1")


def config2(density: float, n_graphs: int = 128, n: int = 256) -> GraphBatch:
    """Tile-density sweep: ER graphs with n=256 at one edge density; pair k is
    graphs (2k, 2k+1).  Weights U(0,1) (redrawn below 1e-3), labels U(0,1),
    4 vertex labels, h=0.5, length scale 1."""
    tag = {0.01: 0, 0.05: 1, 0.2: 2, 1.0: 3}.get(density, int(round(density * 1000)) + 10)
    rng = np.random.default_rng(SEED_BASE + 2 + 1000 * tag)
    return erdos_renyi_batch(rng, n_graphs, n, n, density, (0.0, 1.0), (0.0, 1.0), 4,
                             KernelParams(q=0.05, h=0.5, length_scale=1.0),
                             "config2[rho=%g]" % density, w_min=1e-3)


def config3(n_graphs: int = 32, n: int = 2048, order: str = "random") -> GraphBatch:
    """3-D random geometric graphs, mean degree ~12, w=exp(-d), label=d,
    8 vertex labels, h=0.5, length scale 0.05; pair k is graphs (2k, 2k+1).
    ``order`` as in ``geometric_batch`` (the configuration itself uses "random")."""
    rng = np.random.default_rng(SEED_BASE + 3)
    return geometric_batch(rng, n_graphs, n, 12.0, 8,
                           KernelParams(q=0.05, h=0.5, length_scale=0.05), "config3", order)


def config4(n_graphs: int = 2000) -> GraphBatch:
    """Large-batch Gram: molecule-like graphs of 20-60 vertices."""
    rng = np.random.default_rng(SEED_BASE + 4)
    return molecule_like_batch(rng, n_graphs, 20, 60,
                               KernelParams(q=0.05, h=0.3, length_scale=0.1), "config4")


def paper_synthetic(kind: str, n_graphs: int = 160, n: int = 96) -> GraphBatch:
    """The paper's synthetic benchmark sets (Section "Performance Measurement"):
    160 graphs of 96 nodes, Newman-Watts-Strogatz with k=3, p=0.1 ("nws") or
    Barabasi-Albert with m=6 ("ba").  The paper does not state labels or base
    kernels for them: unit weights, 4 uniform vertex labels (h=0.5), edge labels
    U(0,1) with a square-exponential kernel of length scale 1, q=0.05."""
    prm = KernelParams(q=0.05, h=0.5, length_scale=1.0)
    if kind == "nws":
        rng = np.random.default_rng(SEED_BASE + 10)
        return newman_watts_strogatz_batch(rng, n_graphs, n, 3, 0.1, 4, prm, "nws")
    if kind == "ba":
        rng = np.random.default_rng(SEED_BASE + 11)
        return barabasi_albert_batch(rng, n_graphs, n, 6, 4, prm, "ba")
    raise ValueError(kind)
