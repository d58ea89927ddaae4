"""Build and load the C part of the CPU oracle (test infrastructure only)."""
from __future__ import annotations

import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = [os.path.join(_HERE, "mlip_oracle.c"), os.path.join(_HERE, "rmp_edge.inc"), os.path.join(_HERE, "bond3.inc")]
_SO = os.path.join(_HERE, "libmlip_oracle.so")

c_i32p = ctypes.POINTER(ctypes.c_int32)
c_i64p = ctypes.POINTER(ctypes.c_int64)
c_f64p = ctypes.POINTER(ctypes.c_double)
c_f32p = ctypes.POINTER(ctypes.c_float)


class OrcGraph(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("E", ctypes.c_int64), ("row_ptr", c_i64p),
                ("senders", c_i32p), ("shifts", c_i32p)]


def build(force=False):
    """Compile libmlip_oracle.so with gcc (plain C, OpenMP over rows, no FMA contraction)."""
    stale = force or not os.path.exists(_SO) or any(
        os.path.getmtime(s) > os.path.getmtime(_SO) for s in _SRC)
    if stale:
        cmd = ["gcc", "-O2", "-ftree-vectorize", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-std=c11", "-o", _SO, _SRC[0], "-lm"]
        subprocess.run(cmd, check=True, cwd=_HERE)
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        L.orc_build_brute.restype = ctypes.POINTER(OrcGraph)
        L.orc_build_brute.argtypes = [ctypes.c_int64, c_f64p, c_f64p, ctypes.c_double]
        L.orc_build_cells.restype = ctypes.POINTER(OrcGraph)
        L.orc_build_cells.argtypes = [ctypes.c_int64, c_f64p, c_f64p, ctypes.c_double]
        L.orc_graph_free.restype = None
        L.orc_graph_free.argtypes = [ctypes.POINTER(OrcGraph)]
        L.orc_slab_assign.restype = ctypes.c_int
        L.orc_slab_assign.argtypes = [ctypes.c_int64, c_f64p, c_f64p, ctypes.c_int, c_i32p, c_i32p]
        L.orc_geometry.restype = None
        L.orc_geometry.argtypes = [ctypes.c_int64, c_f64p, c_f64p, c_i64p, c_i32p, c_i32p, c_f64p, c_f64p]
        L.orc_num_threads.restype = ctypes.c_int
        L.orc_set_threads.argtypes = [ctypes.c_int]
        for suf, fp, real in (("f64", c_f64p, ctypes.c_double), ("f32", c_f32p, ctypes.c_float)):
            f = getattr(L, "orc_basis_" + suf)
            f.restype = None
            f.argtypes = [real, real, ctypes.c_int, ctypes.c_int, fp, fp]
            f = getattr(L, "orc_edge_forward_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, c_i64p, c_i32p, fp, real, ctypes.c_int, ctypes.c_int,
                          ctypes.c_int, fp, fp, fp, fp]
            f = getattr(L, "orc_edge_backward_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, ctypes.c_int64, c_i64p, c_i32p, fp, real, ctypes.c_int,
                          ctypes.c_int, ctypes.c_int, fp, fp, fp, fp, fp, fp]
            f = getattr(L, "orc_force_scatter_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, c_i64p, c_i32p, fp, fp, fp]
            f = getattr(L, "orc3_basis_rows_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, fp, real, ctypes.c_int, ctypes.c_int, fp, fp]
            f = getattr(L, "orc3_triplet_forward_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, c_i64p, fp, fp, fp, fp, fp, ctypes.c_int, ctypes.c_int, fp]
            f = getattr(L, "orc3_triplet_backward_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, c_i64p, fp, fp, fp, fp, fp, ctypes.c_int, ctypes.c_int, fp, fp, fp, fp, fp]
            f = getattr(L, "orc3_edge_forward_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, c_i64p, c_i32p, fp, real, ctypes.c_int, ctypes.c_int,
                          ctypes.c_int, fp, fp, c_i64p, fp, fp, fp]
            f = getattr(L, "orc3_edge_backward_" + suf)
            f.restype = None
            f.argtypes = [ctypes.c_int64, ctypes.c_int64, c_i64p, c_i32p, fp, real, ctypes.c_int,
                          ctypes.c_int, ctypes.c_int, fp, fp, c_i64p, fp, fp, fp, fp, fp, fp]
        _lib = L
    return _lib
