"""ctypes access to the C edition of the oracle (``mgk_oracle.c``).  TEST INFRASTRUCTURE.

``build()`` compiles it with gcc; ``pairs()`` evaluates kernel values for a list
of graph pairs of a batch, ``apply()`` returns S u for one pair.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "mgk_oracle.c")
_LIB = os.path.join(_HERE, "libmgk_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99",
                               "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        _lib.mgk_oracle_pairs.restype = ctypes.c_int
        _lib.mgk_oracle_pair_nodal.restype = ctypes.c_int
        _lib.mgk_oracle_apply.restype = ctypes.c_int
        _lib.mgk_oracle_threads.restype = ctypes.c_int
        _lib.mgk_oracle_set_edge_kernel.restype = ctypes.c_int
    return _lib


def _set_edge_kernel(lib, spec) -> float:
    """Put the edge kernel ``spec`` in force (a number = square exponential with that
    length scale; else an object with kind / coef / rho / length_scales, as
    ``mgk_oracle.EdgeKernel``).  Returns the length scale to pass along."""
    if isinstance(spec, (int, float, np.floating)):
        kind, dim, par, ls = 0, 1, [], float(spec)
    elif spec.kind == "poly":
        kind, dim, par, ls = 1, 1, [spec.rho, float(len(spec.coef))] + list(spec.coef), 1.0
    elif spec.kind == "kron_se":
        kind, dim, par, ls = 2, len(spec.length_scales), list(spec.length_scales), 1.0
    elif spec.kind == "rconv_se":
        kind, dim, par, ls = 3, int(spec.dim), list(spec.length_scales), 1.0
    else:
        raise ValueError("unknown edge kernel")
    arr = np.asarray(par + [0.0], dtype=np.float64)
    rc = lib.mgk_oracle_set_edge_kernel(ctypes.c_int32(kind), ctypes.c_int32(dim),
                                        _p(arr, ctypes.c_double), ctypes.c_int32(len(par)))
    if rc != 0:
        raise RuntimeError("mgk_oracle_set_edge_kernel failed with code %d" % rc)
    return ls


def _spec_of(prm):
    """Edge-kernel description of a parameter record (``length_scale`` alone = square
    exponential)."""
    kind = getattr(prm, "edge_kernel", "se")
    if kind == "se":
        return float(prm.length_scale)
    from . import mgk_oracle as O
    if kind == "poly":
        return O.EdgeKernel("poly", coef=prm.poly_coef, rho=prm.poly_rho)
    return O.EdgeKernel(kind, length_scales=prm.length_scales, dim=getattr(prm, "label_dim", 0))


def _p(a, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def threads() -> int:
    return int(_load().mgk_oracle_threads())


def pairs(batch, pi, pj, tier: int = 0, n_threads: int = 0,
          start_prob: Optional[np.ndarray] = None) -> np.ndarray:
    """Kernel values of pairs (pi[k], pj[k]) of ``batch`` (a GraphBatch-like
    object with the flat arrays and ``params``)."""
    lib = _load()
    pi = np.ascontiguousarray(pi, dtype=np.int32)
    pj = np.ascontiguousarray(pj, dtype=np.int32)
    out = np.zeros(len(pi), dtype=np.float64)
    vo = np.ascontiguousarray(batch.vtx_off, dtype=np.int64)
    vl = np.ascontiguousarray(batch.vtx_label, dtype=np.int32)
    eo = np.ascontiguousarray(batch.edge_off, dtype=np.int64)
    s = np.ascontiguousarray(batch.src, dtype=np.int32)
    d = np.ascontiguousarray(batch.dst, dtype=np.int32)
    w = np.ascontiguousarray(batch.weight, dtype=np.float32)
    e = np.ascontiguousarray(batch.edge_label, dtype=np.float32)
    sp = None
    if start_prob is not None:
        sp_arr = np.ascontiguousarray(start_prob, dtype=np.float64)
        sp = _p(sp_arr, ctypes.c_double)
    prm = batch.params
    ls = _set_edge_kernel(lib, _spec_of(prm))
    rc = lib.mgk_oracle_pairs(
        ctypes.c_int32(batch.n_graphs), _p(vo, ctypes.c_int64), _p(vl, ctypes.c_int32), sp,
        _p(eo, ctypes.c_int64), _p(s, ctypes.c_int32), _p(d, ctypes.c_int32),
        _p(w, ctypes.c_float), _p(e, ctypes.c_float),
        ctypes.c_double(prm.q), ctypes.c_double(prm.h), ctypes.c_double(ls),
        ctypes.c_int64(len(pi)), _p(pi, ctypes.c_int32), _p(pj, ctypes.c_int32),
        ctypes.c_int32(tier), ctypes.c_int32(n_threads), _p(out, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("mgk_oracle_pairs failed with code %d" % rc)
    return out


def _graph_args(g):
    n, lab, s, d, w, e = g
    lab = np.ascontiguousarray(lab, dtype=np.int32)
    s = np.ascontiguousarray(s, dtype=np.int32)
    d = np.ascontiguousarray(d, dtype=np.int32)
    w = np.ascontiguousarray(w, dtype=np.float32)
    e = np.ascontiguousarray(e, dtype=np.float32)
    keep = (lab, s, d, w, e)
    args = (ctypes.c_int32(int(n)), _p(lab, ctypes.c_int32), ctypes.c_int32(len(s)),
            _p(s, ctypes.c_int32), _p(d, ctypes.c_int32), _p(w, ctypes.c_float),
            _p(e, ctypes.c_float))
    return args, keep


def pair_nodal(g1, g2, q, h, length_scale, tier: int = 0):
    """(K, x) with x the n x n' nodal solution of Eq. 1 for one pair."""
    lib = _load()
    a1, k1 = _graph_args(g1)
    a2, k2 = _graph_args(g2)
    K = ctypes.c_double(0.0)
    x = np.zeros(int(g1[0]) * int(g2[0]), dtype=np.float64)
    length_scale = _set_edge_kernel(lib, length_scale)
    rc = lib.mgk_oracle_pair_nodal(*a1, *a2, ctypes.c_double(q), ctypes.c_double(h),
                                   ctypes.c_double(length_scale), ctypes.c_int32(tier),
                                   ctypes.byref(K), _p(x, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("mgk_oracle_pair_nodal failed with code %d" % rc)
    return K.value, x.reshape(int(g1[0]), int(g2[0]))


def apply(g1, g2, q, h, length_scale, u: np.ndarray) -> np.ndarray:
    """S u for one pair in fp64 (matrix-free)."""
    lib = _load()
    a1, k1 = _graph_args(g1)
    a2, k2 = _graph_args(g2)
    u = np.ascontiguousarray(u, dtype=np.float64).reshape(-1)
    out = np.zeros_like(u)
    length_scale = _set_edge_kernel(lib, length_scale)
    rc = lib.mgk_oracle_apply(*a1, *a2, ctypes.c_double(q), ctypes.c_double(h),
                              ctypes.c_double(length_scale), _p(u, ctypes.c_double),
                              _p(out, ctypes.c_double))
    if rc != 0:
        raise RuntimeError("mgk_oracle_apply failed with code %d" % rc)
    return out
