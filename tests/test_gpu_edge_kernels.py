"""GPU parity for the edge base kernels beyond the square exponential (Appendix B):
compact polynomial, Kronecker product of square exponentials over label attributes,
R-convolution over label parts.  Every solver the kernel is built into is exercised
against the fp64 oracle: register-resident and streaming on chip, sparse and dense
product with vectors in global memory."""
import dataclasses

import numpy as np
import pytest

import mgk_workloads as W
import paper_1910_06310_amd as M
from oracle import c_oracle as C

pytestmark = pytest.mark.gpu
RTOL = 1e-4
WENDLAND_C2 = (1.0, 0.0, -10.0, 20.0, -15.0, 4.0)   # (1 - r)^4 (4 r + 1)


@pytest.fixture(scope="module")
def torch():
    import torch
    return torch


@pytest.fixture(scope="module")
def solver(torch):
    s = M.Solver(0)
    yield s
    s.set_onchip_limit(16384)
    s.set_product_cache(True)
    s.set_tile_path(M.TILE_AUTO)


def pairs_on(torch, solver, wb, pi, pj, onchip=16384, cache=True, tile_path=M.TILE_AUTO, reorder=M.REORDER_PBR):
    solver.configure(wb.params)
    solver.set_solver(1e-6, 0)
    solver.set_launch(0)
    solver.set_onchip_limit(onchip)
    solver.set_product_cache(cache)
    solver.set_tile_path(tile_path)
    B = solver.load_batch(wb, reorder=reorder)
    K = torch.full((len(pi),), float("nan"), dtype=torch.float32, device="cuda")
    fl = torch.full((len(pi),), -1, dtype=torch.int32, device="cuda")
    solver.pairs(B, B, pi, pj, K, None, fl)
    torch.cuda.synchronize()
    assert (fl.cpu().numpy() == 0).all()
    return K.cpu().numpy().astype(np.float64)


def molecules(seed, n_graphs, lo, hi, weighted):
    rng = np.random.default_rng(seed)
    wb = W.molecule_like_batch(rng, n_graphs, lo, hi, W.KernelParams(q=0.06, h=0.4, length_scale=0.2))
    if weighted:
        wb.weight = rng.uniform(0.4, 1.6, len(wb.weight)).astype(np.float32)
    return W.permute_vertices(wb, rng), rng


@pytest.mark.parametrize("weighted", [False, True])
def test_compact_polynomial_all_solvers(torch, solver, weighted):
    wb, rng = molecules(31, 8, 12, 50, weighted)
    # bond-length labels are N(1.4, 0.1): a support radius of 0.25 puts pairs on both sides of it
    wb.params = dataclasses.replace(wb.params, edge_kernel="poly", poly_coef=WENDLAND_C2, poly_rho=0.25)
    pi, pj = W.gram_pairs(8)
    ref = C.pairs(wb, pi, pj, tier=0)
    for kw in (dict(), dict(cache=False), dict(onchip=0, tile_path=M.TILE_SPARSE),
               dict(onchip=0, tile_path=M.TILE_SPARSE_GATHER), dict(onchip=0, tile_path=M.TILE_DENSE)):
        got = pairs_on(torch, solver, wb, pi, pj, **kw)
        np.testing.assert_allclose(got, ref, rtol=RTOL, err_msg=str(kw))
    # graphs with long rows (streaming kernel with atomics, dense tiles)
    prm = W.KernelParams(q=0.1, h=0.5, edge_kernel="poly", poly_coef=WENDLAND_C2, poly_rho=1.2)
    er = W.erdos_renyi_batch(np.random.default_rng(3), 4, 24, 40, 0.6, (0.3, 1.3) if weighted else (1.0, 1.0),
                             (0.0, 2.0), 3, prm)
    pi, pj = W.gram_pairs(4)
    ref = C.pairs(er, pi, pj, tier=1)
    for kw in (dict(), dict(onchip=0, tile_path=M.TILE_SPARSE), dict(onchip=0, tile_path=M.TILE_DENSE)):
        got = pairs_on(torch, solver, er, pi, pj, **kw)
        np.testing.assert_allclose(got, ref, rtol=RTOL, err_msg=str(kw))


def test_polynomial_outside_unit_range_is_rejected(torch, solver):
    with pytest.raises(M.MgkError):
        solver.set_edge_kernel_poly((1.0, 1.0), 1.0)       # 2 at r = 1
    with pytest.raises(M.MgkError):
        solver.set_edge_kernel_poly((0.5, -1.0), 1.0)      # negative beyond r = 0.5
    with pytest.raises(M.MgkError):
        solver.set_edge_kernel_poly(WENDLAND_C2, 0.0)


@pytest.mark.parametrize("kind", ["kron_se", "rconv_se"])
@pytest.mark.parametrize("weighted", [False, True])
def test_attribute_kernels_on_chip_and_in_global_memory(torch, solver, kind, weighted):
    wb, rng = molecules(37, 8, 12, 50, weighted)
    dim = 3
    prm = dataclasses.replace(wb.params, edge_kernel=kind, label_dim=dim,
                              length_scales=(0.15, 0.4, 0.25) if kind == "kron_se" else (0.3,))
    wa = W.with_label_attributes(wb, rng, dim, 0.3, prm)
    pi, pj = W.gram_pairs(8)
    ref = C.pairs(wa, pi, pj, tier=0)
    # register-resident, streaming on chip, both sparse products in global memory
    for kw in (dict(), dict(cache=False), dict(onchip=0), dict(onchip=0, tile_path=M.TILE_SPARSE_GATHER),
               dict(reorder=M.REORDER_NONE)):
        got = pairs_on(torch, solver, wa, pi, pj, **kw)
        np.testing.assert_allclose(got, ref, rtol=RTOL, err_msg=str(kw))
    # larger, denser graphs (rows longer than a lane group): streaming kernel with atomic
    # row sums on chip, the sparse products in global memory
    er = W.erdos_renyi_batch(np.random.default_rng(5), 4, 24, 40, 0.5, (0.3, 1.3) if weighted else (1.0, 1.0),
                             (0.0, 2.0), 3, prm)
    ea = W.with_label_attributes(er, np.random.default_rng(6), dim, 0.5, prm)
    pi, pj = W.gram_pairs(4)
    ref = C.pairs(ea, pi, pj, tier=1)
    for kw in (dict(), dict(onchip=0), dict(onchip=0, tile_path=M.TILE_SPARSE_GATHER)):
        got = pairs_on(torch, solver, ea, pi, pj, **kw)
        np.testing.assert_allclose(got, ref, rtol=RTOL, err_msg=str(kw))


def test_attribute_kernel_needs_matching_batch(torch, solver):
    wb, rng = molecules(41, 3, 10, 20, False)
    solver.configure(wb.params)
    B1 = solver.load_batch(wb)
    solver.set_edge_kernel_kron_se((0.3, 0.3))
    K = torch.zeros(1, dtype=torch.float32, device="cuda")
    with pytest.raises(M.MgkError):
        solver.pairs(B1, B1, [0], [1], K)
    solver.configure(wb.params)


def test_one_attribute_kernels_equal_the_square_exponential(torch, solver):
    wb, rng = molecules(43, 6, 15, 45, True)
    pi, pj = W.gram_pairs(6)
    ref = pairs_on(torch, solver, wb, pi, pj)
    for kind in ("kron_se", "rconv_se"):
        prm = dataclasses.replace(wb.params, edge_kernel=kind, label_dim=1, length_scales=(wb.params.length_scale,))
        got = pairs_on(torch, solver, dataclasses.replace(wb, params=prm), pi, pj)
        np.testing.assert_allclose(got, ref, rtol=2e-6)
