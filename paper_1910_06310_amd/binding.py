"""Thin ctypes binding of the C ABI declared in ``include/mgk.h``.

Argument marshalling only: every step of the solve runs in the HIP library.
torch supplies device memory for the outputs and the stream.  There is no CPU
fallback: if ``libmgk.so`` is missing the import of :func:`load_library` raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libmgk.so")
_lib = None

OK, EINVAL, ENOMEM, EDEVICE, ESTATE, ELIMIT = range(6)
REORDER_NONE, REORDER_PBR, REORDER_RCM = 0, 1, 2
TILE_AUTO, TILE_SPARSE, TILE_DENSE, TILE_SPARSE_GATHER = 0, 1, 2, 3

EXPORTS = [
    "mgk_create", "mgk_destroy", "mgk_last_error",
    "mgk_set_vertex_kernel_delta", "mgk_set_edge_kernel_se", "mgk_set_edge_kernel_const",
    "mgk_set_edge_kernel_poly", "mgk_set_edge_kernel_kron_se", "mgk_set_edge_kernel_rconv_se",
    "mgk_load_graphs_attr",
    "mgk_set_stop_prob", "mgk_set_solver", "mgk_set_tile_path", "mgk_set_launch",
    "mgk_set_onchip_limit", "mgk_set_product_cache", "mgk_set_schedule",
    "mgk_load_graphs", "mgk_load_graphs_embedded", "mgk_free_batch", "mgk_batch_stats", "mgk_batch_permutation",
    "mgk_batch_get_tiles", "mgk_gram", "mgk_pairs", "mgk_pairs_dev", "mgk_pairs_noalloc", "mgk_pairs_nodal", "mgk_normalize_gram", "mgk_launch_log",
]


class MgkError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("mgk status %d: %s" % (status, message))
        self.status = status


def load_library(path: Optional[str] = None):
    """dlopen the HIP library.  torch is imported first so that both share one
    HIP runtime (the stream handle passed across the ABI belongs to it)."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or os.environ.get("MGK_LIBRARY_PATH") or _LIB_PATH
    if not os.path.exists(path):
        raise ImportError(
            "HIP library %s is not built; run `python -m paper_1910_06310_amd.build`" % path)
    import torch  # noqa: F401
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i32, i64, f32 = c.c_void_p, c.c_int32, c.c_int64, c.c_float
    lib.mgk_create.argtypes = [c.POINTER(vp), c.c_int]
    lib.mgk_destroy.argtypes = [vp]
    lib.mgk_destroy.restype = None
    lib.mgk_last_error.argtypes = [vp]
    lib.mgk_last_error.restype = c.c_char_p
    lib.mgk_set_vertex_kernel_delta.argtypes = [vp, f32]
    lib.mgk_set_edge_kernel_se.argtypes = [vp, f32]
    lib.mgk_set_edge_kernel_const.argtypes = [vp, f32]
    lib.mgk_set_edge_kernel_poly.argtypes = [vp, i32, vp, f32]
    lib.mgk_set_edge_kernel_kron_se.argtypes = [vp, i32, vp]
    lib.mgk_set_edge_kernel_rconv_se.argtypes = [vp, i32, f32]
    lib.mgk_load_graphs_attr.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, i32, vp, i32, c.POINTER(vp)]
    lib.mgk_set_stop_prob.argtypes = [vp, f32]
    lib.mgk_set_solver.argtypes = [vp, f32, i32]
    lib.mgk_set_tile_path.argtypes = [vp, i32]
    lib.mgk_set_launch.argtypes = [vp, i32]
    lib.mgk_set_onchip_limit.argtypes = [vp, i32]
    lib.mgk_set_product_cache.argtypes = [vp, i32]
    lib.mgk_set_schedule.argtypes = [vp, i32]
    lib.mgk_load_graphs.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, c.POINTER(vp)]
    lib.mgk_load_graphs_embedded.argtypes = [vp, i32, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, c.POINTER(vp)]
    lib.mgk_free_batch.argtypes = [vp, vp]
    lib.mgk_free_batch.restype = None
    lib.mgk_batch_stats.argtypes = [vp] + [c.POINTER(i64)] * 5
    lib.mgk_batch_permutation.argtypes = [vp, vp]
    lib.mgk_batch_get_tiles.argtypes = [vp, i32, c.POINTER(i32), c.POINTER(i32), vp, vp, vp, vp, vp]
    lib.mgk_gram.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.mgk_pairs.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.mgk_pairs_dev.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.mgk_pairs_noalloc.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp]
    lib.mgk_pairs_nodal.argtypes = [vp, vp, vp, i64, vp, vp, vp, vp, vp, vp, vp, vp]
    lib.mgk_launch_log.argtypes = [vp, vp, i64]
    lib.mgk_normalize_gram.argtypes = [vp, i32, vp, vp]
    for name in EXPORTS:
        fn = getattr(lib, name)
        if name == "mgk_launch_log":
            fn.restype = c.c_int64
        elif name not in ("mgk_destroy", "mgk_free_batch", "mgk_last_error"):
            fn.restype = c.c_int
    _lib = lib
    return lib


def _host(a, dtype):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(a, dtype=dtype)
    return arr, arr.ctypes.data_as(ctypes.c_void_p)


def _dev_ptr(t, dtype_name: str, numel: int):
    import torch
    if t is None:
        return None
    want = getattr(torch, dtype_name)
    if not t.is_cuda or t.dtype != want or not t.is_contiguous() or t.numel() < numel:
        raise ValueError("output must be a contiguous cuda %s tensor with >= %d elements"
                         % (dtype_name, numel))
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return ctypes.c_void_p(s.cuda_stream)


class Batch:
    """A set of graphs packed and resident on the device (mgk_batch)."""

    def __init__(self, solver: "Solver", handle, vtx_off: np.ndarray):
        self._solver = solver
        self._h = handle
        self.vtx_off = vtx_off
        self.n_graphs = len(vtx_off) - 1

    def stats(self) -> dict:
        lib = load_library()
        vals = [ctypes.c_int64(0) for _ in range(5)]
        self._solver._check(lib.mgk_batch_stats(self._h, *[ctypes.byref(v) for v in vals]))
        keys = ["n_graphs", "n_vertices", "nnz", "n_tiles", "n_offdiag_tiles"]
        return {k: int(v.value) for k, v in zip(keys, vals)}

    def permutation(self) -> np.ndarray:
        lib = load_library()
        perm = np.zeros(int(self.vtx_off[-1]), dtype=np.int32)
        self._solver._check(lib.mgk_batch_permutation(self._h, perm.ctypes.data_as(ctypes.c_void_p)))
        return perm

    def get_tiles(self, g: int) -> dict:
        lib = load_library()
        nt, nz = ctypes.c_int32(0), ctypes.c_int32(0)
        self._solver._check(lib.mgk_batch_get_tiles(self._h, g, ctypes.byref(nt), ctypes.byref(nz),
                                                    None, None, None, None, None))
        tr = np.zeros(nt.value, np.int32); tc = np.zeros(nt.value, np.int32)
        bm = np.zeros(nt.value, np.uint64)
        w = np.zeros(nz.value, np.float32); e = np.zeros(nz.value, np.float32)
        p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
        self._solver._check(lib.mgk_batch_get_tiles(self._h, g, ctypes.byref(nt), ctypes.byref(nz),
                                                    p(tr), p(tc), p(bm), p(w), p(e)))
        return {"tile_row": tr, "tile_col": tc, "bitmap": bm, "w": w, "e": e}

    def free(self):
        if self._h is not None and self._solver._h is not None:
            load_library().mgk_free_batch(self._solver._h, self._h)
        self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


class Solver:
    """One mgk_ctx.  Method names follow the C ABI without the ``mgk_`` prefix."""

    def __init__(self, device: int = 0):
        lib = load_library()
        h = ctypes.c_void_p()
        st = lib.mgk_create(ctypes.byref(h), device)
        if st != OK:
            raise MgkError(st, "mgk_create failed (is a HIP device %d visible?)" % device)
        self._h = h
        self.device = device

    def _check(self, st: int):
        if st != OK:
            msg = load_library().mgk_last_error(self._h)
            raise MgkError(st, msg.decode() if msg else "")

    def destroy(self):
        if self._h is not None:
            load_library().mgk_destroy(self._h)
            self._h = None

    def set_vertex_kernel_delta(self, h: float):
        self._check(load_library().mgk_set_vertex_kernel_delta(self._h, h))

    def set_edge_kernel_se(self, length_scale: float):
        self._check(load_library().mgk_set_edge_kernel_se(self._h, length_scale))

    def set_edge_kernel_const(self, c: float):
        self._check(load_library().mgk_set_edge_kernel_const(self._h, c))

    def set_edge_kernel_poly(self, coef, rho: float):
        cf, pcf = _host(coef, np.float32)
        self._check(load_library().mgk_set_edge_kernel_poly(self._h, len(cf), pcf, rho))

    def set_edge_kernel_kron_se(self, length_scales):
        ls, pls = _host(length_scales, np.float32)
        self._check(load_library().mgk_set_edge_kernel_kron_se(self._h, len(ls), pls))

    def set_edge_kernel_rconv_se(self, dim: int, length_scale: float):
        self._check(load_library().mgk_set_edge_kernel_rconv_se(self._h, dim, length_scale))

    def set_stop_prob(self, q: float):
        self._check(load_library().mgk_set_stop_prob(self._h, q))

    def set_solver(self, rtol: float = 1e-6, max_iter: int = 0):
        self._check(load_library().mgk_set_solver(self._h, rtol, max_iter))

    def set_tile_path(self, mode: int):
        self._check(load_library().mgk_set_tile_path(self._h, mode))

    def set_launch(self, waves_per_pair: int = 0):
        self._check(load_library().mgk_set_launch(self._h, waves_per_pair))

    def set_onchip_limit(self, max_product: int = 16384):
        self._check(load_library().mgk_set_onchip_limit(self._h, max_product))

    def set_schedule(self, cost_sorted: bool = True):
        self._check(load_library().mgk_set_schedule(self._h, 1 if cost_sorted else 0))

    def set_product_cache(self, enable=True):
        """False / 0: entries regenerated in every product; True / 1: kept in registers for small
        pairs; 3: the same with the owner-computes kernel where a pair fits it."""
        self._check(load_library().mgk_set_product_cache(self._h, int(enable)))

    def load_graphs(self, vtx_off, vtx_label, edge_off, src, dst, weight=None, edge_label=None,
                    start_prob=None, reorder: int = REORDER_PBR) -> Batch:
        lib = load_library()
        vo, pvo = _host(vtx_off, np.int64)
        vl, pvl = _host(vtx_label, np.int32)
        sp, psp = _host(start_prob, np.float32)
        eo, peo = _host(edge_off, np.int64)
        s, ps = _host(src, np.int32)
        d, pd = _host(dst, np.int32)
        w, pw = _host(weight, np.float32)
        dim = 1
        if edge_label is not None and np.ndim(edge_label) == 2:   # [edges, attributes]
            dim = int(np.shape(edge_label)[1])
        e, pe = _host(None if edge_label is None else np.reshape(edge_label, -1), np.float32)
        h = ctypes.c_void_p()
        self._check(lib.mgk_load_graphs_attr(self._h, len(vo) - 1, pvo, pvl, psp, peo, ps, pd, pw, dim, pe,
                                             reorder, ctypes.byref(h)))
        return Batch(self, h, vo.copy())

    def load_graphs_embedded(self, vtx_off, vtx_label, edge_off, src, dst, coords, weight=None,
                             edge_label=None, start_prob=None) -> Batch:
        """Graphs with vertex coordinates ([sum n, dim]), numbered along the Morton curve."""
        lib = load_library()
        vo, pvo = _host(vtx_off, np.int64)
        vl, pvl = _host(vtx_label, np.int32)
        sp, psp = _host(start_prob, np.float32)
        eo, peo = _host(edge_off, np.int64)
        s, ps = _host(src, np.int32)
        d, pd = _host(dst, np.int32)
        w, pw = _host(weight, np.float32)
        e, pe = _host(edge_label, np.float32)
        xy = np.ascontiguousarray(coords, dtype=np.float32)
        if xy.ndim != 2 or xy.shape[0] != int(vo[-1]):
            raise ValueError("coords must be [total vertices, dim]")
        h = ctypes.c_void_p()
        self._check(lib.mgk_load_graphs_embedded(self._h, len(vo) - 1, pvo, pvl, psp, peo, ps, pd, pw, pe,
                                                 int(xy.shape[1]), xy.ctypes.data_as(ctypes.c_void_p),
                                                 ctypes.byref(h)))
        return Batch(self, h, vo.copy())

    def load_batch(self, batch, reorder: int = REORDER_PBR, start_prob=None) -> Batch:
        """Convenience for objects with the flat arrays as attributes."""
        return self.load_graphs(batch.vtx_off, batch.vtx_label, batch.edge_off, batch.src,
                                batch.dst, batch.weight, batch.edge_label, start_prob, reorder)

    def gram(self, batch: Batch, K, iters=None, flags=None, stream=None):
        G = batch.n_graphs
        self._check(load_library().mgk_gram(
            self._h, batch._h, _dev_ptr(K, "float32", G * G), _dev_ptr(iters, "int32", G * G),
            _dev_ptr(flags, "int32", G * G), _stream_ptr(stream)))

    def pairs(self, X: Batch, Y: Batch, i_idx: Sequence[int], j_idx: Sequence[int], K,
              iters=None, flags=None, stream=None):
        ii, pi = _host(i_idx, np.int32)
        jj, pj = _host(j_idx, np.int32)
        n = len(ii)
        if len(jj) != n:
            raise ValueError("index arrays differ in length")
        self._check(load_library().mgk_pairs(
            self._h, X._h, Y._h, n, pi, pj, _dev_ptr(K, "float32", n),
            _dev_ptr(iters, "int32", n), _dev_ptr(flags, "int32", n), _stream_ptr(stream)))

    def pairs_noalloc(self, X: Batch, Y: Batch, i_idx: Sequence[int], j_idx: Sequence[int], K,
                      iters=None, flags=None, stream=None):
        """As pairs(), without any device allocation inside the library (on-chip pairs only,
        at most 65536 per call)."""
        ii, pi = _host(i_idx, np.int32)
        jj, pj = _host(j_idx, np.int32)
        n = len(ii)
        if len(jj) != n:
            raise ValueError("index arrays differ in length")
        self._check(load_library().mgk_pairs_noalloc(
            self._h, X._h, Y._h, n, pi, pj, _dev_ptr(K, "float32", n),
            _dev_ptr(iters, "int32", n), _dev_ptr(flags, "int32", n), _stream_ptr(stream)))

    def pairs_dev(self, X: Batch, Y: Batch, i_idx, j_idx, K, iters=None, flags=None, stream=None):
        """As pairs(), with the two index arrays as int32 cuda tensors."""
        n = int(i_idx.numel())
        if int(j_idx.numel()) != n:
            raise ValueError("index arrays differ in length")
        self._check(load_library().mgk_pairs_dev(
            self._h, X._h, Y._h, n, _dev_ptr(i_idx, "int32", n), _dev_ptr(j_idx, "int32", n),
            _dev_ptr(K, "float32", n), _dev_ptr(iters, "int32", n), _dev_ptr(flags, "int32", n),
            _stream_ptr(stream)))

    def pairs_nodal(self, X: Batch, Y: Batch, i_idx, j_idx, K, x, x_off, iters=None, flags=None,
                    stream=None):
        """x: flat float32 cuda tensor; x_off[k]: offset of pair k's n x n' block in it."""
        ii, pi = _host(i_idx, np.int32)
        jj, pj = _host(j_idx, np.int32)
        off, po = _host(x_off, np.int64)
        n = len(ii)
        if len(jj) != n or len(off) != n:
            raise ValueError("index arrays differ in length")
        need = 0
        for k in range(n):
            nx = int(X.vtx_off[ii[k] + 1] - X.vtx_off[ii[k]]) * int(Y.vtx_off[jj[k] + 1] - Y.vtx_off[jj[k]])
            need = max(need, int(off[k]) + nx)
        self._check(load_library().mgk_pairs_nodal(
            self._h, X._h, Y._h, n, pi, pj, _dev_ptr(K, "float32", n), _dev_ptr(x, "float32", need), po,
            _dev_ptr(iters, "int32", n), _dev_ptr(flags, "int32", n), _stream_ptr(stream)))

    def launch_log(self) -> str:
        """Kernels the last gram / pairs call enqueued, one line per launch shape."""
        lib = load_library()
        need = int(lib.mgk_launch_log(self._h, None, ctypes.c_int64(0)))
        buf = ctypes.create_string_buffer(max(need, 1))
        lib.mgk_launch_log(self._h, buf, ctypes.c_int64(len(buf)))
        return buf.value.decode()

    def normalize_gram(self, n: int, K, stream=None):
        self._check(load_library().mgk_normalize_gram(self._h, n, _dev_ptr(K, "float32", n * n),
                                                      _stream_ptr(stream)))

    def configure(self, params):
        """Apply q, h and the edge kernel of a workload's parameter record."""
        self.set_stop_prob(params.q)
        self.set_vertex_kernel_delta(params.h)
        kind = getattr(params, "edge_kernel", "se")
        if kind == "se":
            self.set_edge_kernel_se(params.length_scale)
        elif kind == "poly":
            self.set_edge_kernel_poly(params.poly_coef, params.poly_rho)
        elif kind == "kron_se":
            self.set_edge_kernel_kron_se(params.length_scales)
        elif kind == "rconv_se":
            self.set_edge_kernel_rconv_se(params.label_dim, params.length_scales[0])
        else:
            raise ValueError("unknown edge kernel " + str(kind))

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
