"""ctypes binding of libmlip (argument marshalling only; every step runs in the HIP library).

PyTorch supplies device memory (tensors) and the stream; nothing is computed here.
The names mirror include/mlip.h.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# MLIP_LIBRARY selects another build of the same library (timing experiments); the default is the in-tree product build
_LIB_PATH = os.environ.get("MLIP_LIBRARY") or os.path.join(_HERE, "libmlip.so")

MODE_WHOLE, MODE_SLABS = 0, 1
PRECISION_FP32, PRECISION_BF16, PRECISION_FP32_SPLIT = 0, 1, 2
PROF_GROUPS = ("graph", "node", "edge_fwd", "edge_bwd", "ghost", "force", "bond", "triplet_fwd", "triplet_bwd",
               "edge_fwd_lower", "edge_bwd_lower")


class MlipError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"libmlip error {code}: {msg}")
        self.code = code


class _Weights(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("n_species", "F", "L", "K", "p", "precision")] + \
               [(n, ctypes.c_void_p) for n in ("emb", "W1", "W2", "Wm", "Wo", "Wr1", "wr2")]


class _BondWeights(ctypes.Structure):
    _fields_ = [("r_bond", ctypes.c_float), ("A", ctypes.c_int32)] + \
               [(n, ctypes.c_void_p) for n in ("We0", "Wt1", "Wt2", "Wb")]


class _SlabInfo(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("n_owned", "n_pure", "n_border", "n_ghost", "n_local",
                                              "n_edges_owned", "n_edges")] + \
               [(n, ctypes.c_void_p) for n in ("nodes", "markers", "row_ptr", "senders", "owned_sorted")]


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class _Pairs(ctypes.Structure):
    _fields_ = [("n_upper", ctypes.c_int64), ("n_lower", ctypes.c_int64)] + \
               [(n, ctypes.c_void_p) for n in ("u_row_ptr", "u_senders", "u_eid", "u_mirror", "u_d",
                                               "l_row_ptr", "l_senders", "l_slot")]


class _Alloc(ctypes.Structure):
    _fields_ = [("alloc", _ALLOC_FN), ("free", _FREE_FN), ("ctx", ctypes.c_void_p)]


class TorchAllocator:
    """mlip_alloc_t backed by torch tensors: every device block the library uses is a uint8 tensor from torch's
    caching allocator (so torch's memory accounting sees it).  Keeps the blocks alive until the library frees them."""

    def __init__(self):
        self.blocks = {}
        self.bytes_requested = 0
        self.n_alloc = self.n_free = 0
        self._a = _ALLOC_FN(self._alloc)
        self._f = _FREE_FN(self._free)
        self.c = _Alloc(self._a, self._f, None)

    def _alloc(self, nbytes, _ctx):
        try:
            t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device="cuda")
        except Exception:   # out of memory: the library reports MLIP_ENOMEM
            return None
        self.blocks[t.data_ptr()] = t
        self.bytes_requested += int(nbytes)
        self.n_alloc += 1
        return t.data_ptr()

    def _free(self, ptr, _ctx):
        self.n_free += 1
        self.blocks.pop(ptr, None)

    @property
    def bytes_held(self):
        return sum(t.numel() for t in self.blocks.values())


_lib = None


def lib():
    """Load libmlip.so; building it is `python -m paper_2506_02023_amd.build` (or __graft_entry__.build())."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: the HIP library has not been built "
                              "(run __graft_entry__.build()); there is no fallback path")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i64, i32, dbl = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_double
        L.mlip_graph_create.argtypes = [ctypes.POINTER(_Alloc), ctypes.POINTER(vp)]
        L.mlip_graph_invalidate_weights.argtypes = [vp]
        L.mlip_graph_set_skin.argtypes = [vp, dbl]
        L.mlip_graph_skin_stats.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.mlip_forward_static.argtypes = [vp, ctypes.POINTER(_Weights), i32, vp, vp, vp]
        L.mlip_static_scratch_bytes.restype = ctypes.c_size_t
        L.mlip_build_graph.argtypes = [vp, ctypes.POINTER(dbl), vp, i64, dbl, i32, vp, ctypes.POINTER(vp)]
        L.mlip_forward.argtypes = [vp, ctypes.POINTER(_Weights), i32, vp, vp, vp]
        L.mlip_forward_bonds.argtypes = [vp, ctypes.POINTER(_Weights), ctypes.POINTER(_BondWeights), i32, vp, vp, vp]
        L.mlip_graph_bonds.argtypes = [vp, i32, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(i64)]
        L.mlip_graph_destroy.argtypes = [vp]
        L.mlip_graph_destroy.restype = None
        L.mlip_graph_sizes.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.mlip_graph_csr.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(vp), ctypes.POINTER(vp)]
        L.mlip_graph_shifts.argtypes = [vp, vp]
        L.mlip_graph_mirror.argtypes = [vp, ctypes.POINTER(vp)]
        L.mlip_graph_slab_of.argtypes = [vp, ctypes.POINTER(vp), ctypes.POINTER(i32)]
        L.mlip_graph_slab.argtypes = [vp, i32, ctypes.POINTER(_SlabInfo)]
        L.mlip_graph_pairs.argtypes = [vp, i32, ctypes.POINTER(_Pairs)]
        L.mlip_graph_from.argtypes = [vp, i32, i32, ctypes.POINTER(vp), ctypes.POINTER(i64)]
        L.mlip_graph_to.argtypes = [vp, i32, i32, ctypes.POINTER(vp), ctypes.POINTER(i64)]
        L.mlip_profile_enable.argtypes = [vp, i32]
        L.mlip_profile_read.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i64), i32]
        L.mlip_copy_to_host.argtypes = [vp, vp, vp, ctypes.c_size_t]
        L.mlip_last_error.restype = ctypes.c_char_p
        L.mlip_version.restype = ctypes.c_char_p
        _lib = L
    return _lib


def _check(rc):
    if rc != 0:
        raise MlipError(rc, lib().mlip_last_error().decode())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


class Graph:
    """Owner of a mlip_graph_t handle.  By default the handle takes its device memory from torch (TorchAllocator);
    allocator=False leaves allocation to the library (hipMalloc)."""

    def __init__(self, allocator=None):
        self._h = ctypes.c_void_p(None)
        self.allocator = TorchAllocator() if allocator is None else (allocator or None)
        if self.allocator is not None:
            _check(lib().mlip_graph_create(ctypes.byref(self.allocator.c), ctypes.byref(self._h)))

    def set_skin(self, skin):
        """Verlet skin (same length unit as the positions) for repeated builds on this handle; 0 switches it off."""
        if not self._h.value:
            _check(lib().mlip_graph_create(None, ctypes.byref(self._h)))
        _check(lib().mlip_graph_set_skin(self._h, float(skin)))

    def skin_stats(self):
        """(candidate list rebuilds, reuses) since the handle was made."""
        a, b = ctypes.c_int64(), ctypes.c_int64()
        _check(lib().mlip_graph_skin_stats(self._h, ctypes.byref(a), ctypes.byref(b)))
        return a.value, b.value

    def invalidate_weights(self):
        _check(lib().mlip_graph_invalidate_weights(self._h))

    def __del__(self):
        self.destroy()

    def destroy(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().mlip_graph_destroy(self._h)
            self._h = ctypes.c_void_p(None)

    # -- sizes and host copies of the index structures (for parity checks and inspection)
    def sizes(self):
        n, e, p = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int32()
        _check(lib().mlip_graph_sizes(self._h, ctypes.byref(n), ctypes.byref(e), ctypes.byref(p)))
        return n.value, e.value, p.value

    def _host(self, ptr, count, dtype):
        out = np.empty(count, dtype)
        _check(lib().mlip_copy_to_host(self._h, out.ctypes.data_as(ctypes.c_void_p), ctypes.c_void_p(ptr),
                                       out.nbytes))
        return out

    def csr(self):
        """(row_ptr int64 [N+1], senders int32 [E], shifts int32 [E,3], d float32 [E]) as numpy arrays."""
        N, E, _ = self.sizes()
        rp, sd, dd = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
        _check(lib().mlip_graph_csr(self._h, ctypes.byref(rp), ctypes.byref(sd), ctypes.byref(dd)))
        shifts = torch.empty((max(E, 1), 3), dtype=torch.int32, device="cuda")
        _check(lib().mlip_graph_shifts(self._h, ctypes.c_void_p(shifts.data_ptr())))
        torch.cuda.synchronize()
        return (self._host(rp.value, N + 1, np.int64), self._host(sd.value, E, np.int32),
                shifts[:E].cpu().numpy(), self._host(dd.value, E, np.float32))

    def mirror(self):
        """int32 [E]: position of every edge's reverse edge."""
        _, E, _ = self.sizes()
        ptr = ctypes.c_void_p()
        _check(lib().mlip_graph_mirror(self._h, ctypes.byref(ptr)))
        return self._host(ptr.value, E, np.int32)

    def bonds(self, p=-1):
        """(bond_edge int32 [n_bonds], bond_ptr int64 [rows+1]) of the last mlip_forward_bonds: whole graph (p = -1)
        or partition p."""
        rows = self.sizes()[0] if p < 0 else self.slab(p)["n_owned"]
        be, bp, n = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_int64()
        _check(lib().mlip_graph_bonds(self._h, p, ctypes.byref(be), ctypes.byref(bp), ctypes.byref(n)))
        return self._host(be.value, n.value, np.int32), self._host(bp.value, rows + 1, np.int64)

    def pairs(self, p=-1):
        """dict with the upper / lower split of the owned rows' edges of partition p (-1: the whole graph)."""
        rows = self.sizes()[0] if p < 0 else self.slab(p)["n_owned"]
        q = _Pairs()
        _check(lib().mlip_graph_pairs(self._h, p, ctypes.byref(q)))
        nu, nl = q.n_upper, q.n_lower
        d = {"n_upper": nu, "n_lower": nl}
        d["u_row_ptr"] = self._host(q.u_row_ptr, rows + 1, np.int64)
        d["l_row_ptr"] = self._host(q.l_row_ptr, rows + 1, np.int64)
        for k in ("u_senders", "u_eid", "u_mirror"):
            d[k] = self._host(getattr(q, k), nu, np.int32)
        d["u_d"] = self._host(q.u_d, nu, np.float32)
        for k in ("l_senders", "l_slot"):
            d[k] = self._host(getattr(q, k), nl, np.int32)
        return d

    def slab_of(self):
        N, _, _ = self.sizes()
        ptr, ax = ctypes.c_void_p(), ctypes.c_int32()
        _check(lib().mlip_graph_slab_of(self._h, ctypes.byref(ptr), ctypes.byref(ax)))
        return self._host(ptr.value, N, np.int32), ax.value

    def slab(self, p):
        """dict with the counts, nodes, markers, local row_ptr/senders and owned_sorted of partition p."""
        _, _, P = self.sizes()
        info = _SlabInfo()
        _check(lib().mlip_graph_slab(self._h, p, ctypes.byref(info)))
        d = {k: getattr(info, k) for k in ("n_owned", "n_pure", "n_border", "n_ghost", "n_local",
                                           "n_edges_owned", "n_edges")}
        d["nodes"] = self._host(info.nodes, d["n_local"], np.int32)
        d["markers"] = np.ctypeslib.as_array(ctypes.cast(info.markers, ctypes.POINTER(ctypes.c_int64)),
                                             shape=(P + 3,)).copy()
        d["row_ptr"] = self._host(info.row_ptr, d["n_local"] + 1, np.int64)
        d["senders"] = self._host(info.senders, d["n_edges"], np.int32)
        d["owned_sorted"] = self._host(info.owned_sorted, d["n_owned"], np.int32)
        return d

    def _bucket(self, fn, p, q):
        ptr, n = ctypes.c_void_p(), ctypes.c_int64()
        _check(fn(self._h, p, q, ctypes.byref(ptr), ctypes.byref(n)))
        return self._host(ptr.value, n.value, np.int32), ptr.value

    def frm(self, p, q):
        return self._bucket(lib().mlip_graph_from, p, q)[0]

    def to(self, p, q):
        return self._bucket(lib().mlip_graph_to, p, q)[0]

    def bucket_address(self, kind, p, q):
        return self._bucket(lib().mlip_graph_from if kind == "from" else lib().mlip_graph_to, p, q)[1]

    # -- profiling
    def profile_enable(self, on=True):
        _check(lib().mlip_profile_enable(self._h, 1 if on else 0))

    def profile_read(self, reset=True):
        ms = (ctypes.c_float * len(PROF_GROUPS))()
        n = (ctypes.c_int64 * len(PROF_GROUPS))()
        _check(lib().mlip_profile_read(self._h, ms, n, 1 if reset else 0))
        return {k: (ms[i], n[i]) for i, k in enumerate(PROF_GROUPS)}


def mlip_build_graph(positions, cell, species, r_cut, n_slabs=1, graph=None):
    """positions: cuda float64 [N,3]; cell: 3x3 host array (rows = lattice vectors); species: cuda int32 [N]."""
    assert positions.is_cuda and positions.dtype == torch.float64 and positions.is_contiguous()
    assert species.is_cuda and species.dtype == torch.int32 and species.is_contiguous()
    assert positions.dim() == 2 and positions.shape[1] == 3 and species.numel() == positions.shape[0]
    cell_h = np.ascontiguousarray(np.asarray(cell, dtype=np.float64).reshape(9))
    g = graph if graph is not None else Graph()
    _check(lib().mlip_build_graph(ctypes.c_void_p(positions.data_ptr()),
                                  cell_h.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                  ctypes.c_void_p(species.data_ptr()), positions.shape[0], float(r_cut),
                                  int(n_slabs), _stream(), ctypes.byref(g._h)))
    return g


class Weights:
    """Device copies of the model weights plus the POD struct the library takes."""

    def __init__(self, weights, p, K=8, device="cuda", precision=0):
        """precision: 0 = fp32, 1 = bf16 operands for the filter MLP's F x F products (fp32 accumulation),
        2 = those products as split-fp16 triples (fp32-grade results)."""
        self.t = {k: torch.as_tensor(np.ascontiguousarray(weights[k], np.float32)).to(device).contiguous()
                  for k in ("emb", "W1", "W2", "Wm", "Wo", "Wr1", "wr2")}
        S, F = self.t["emb"].shape
        L = self.t["W1"].shape[0]
        self.F, self.L = F, L
        self.c = _Weights(S, F, L, K, p, int(precision), *[self.t[k].data_ptr() for k in
                                               ("emb", "W1", "W2", "Wm", "Wo", "Wr1", "wr2")])


class BondWeights:
    """Device copies of the three-body variant's extra weights plus the POD struct the library takes."""

    def __init__(self, weights, r_bond, A=8, device="cuda"):
        self.t = {k: torch.as_tensor(np.ascontiguousarray(weights[k], np.float32)).to(device).contiguous()
                  for k in ("We0", "Wt1", "Wt2", "Wb")}
        self.c = _BondWeights(float(r_bond), int(A), *[self.t[k].data_ptr() for k in ("We0", "Wt1", "Wt2", "Wb")])


def mlip_forward_bonds(graph, weights, bond_weights, mode=MODE_WHOLE, out=None, want_atom_energy=True):
    """Three-body variant; returns as mlip_forward.  Builds the bond list on first use (one stream synchronisation)."""
    N, _, _ = graph.sizes()
    if out is None:
        energy = torch.empty(1, dtype=torch.float64, device="cuda")
        forces = torch.empty((N, 3), dtype=torch.float32, device="cuda")
        atom_e = torch.empty(N, dtype=torch.float32, device="cuda") if want_atom_energy else None
    else:
        energy, forces, atom_e = out
    _check(lib().mlip_forward_bonds(graph._h, ctypes.byref(weights.c), ctypes.byref(bond_weights.c), int(mode),
                                    ctypes.c_void_p(energy.data_ptr()), ctypes.c_void_p(forces.data_ptr()),
                                    ctypes.c_void_p(atom_e.data_ptr() if atom_e is not None else None)))
    return energy, forces, atom_e


def mlip_forward_static(graph, weights, mode=MODE_WHOLE, out=None, want_atom_energy=True):
    """mlip_forward with the library's fixed workspace (no device allocation inside the call); `out` as mlip_forward."""
    return mlip_forward(graph, weights, mode, out, want_atom_energy, _fn="mlip_forward_static")


def mlip_forward(graph, weights, mode=MODE_WHOLE, out=None, want_atom_energy=True, _fn="mlip_forward"):
    """Returns (energy cuda f64 [1], forces cuda f32 [N,3], atom_energy cuda f32 [N] or None); asynchronous."""
    N, _, _ = graph.sizes()
    if out is None:
        energy = torch.empty(1, dtype=torch.float64, device="cuda")
        forces = torch.empty((N, 3), dtype=torch.float32, device="cuda")
        atom_e = torch.empty(N, dtype=torch.float32, device="cuda") if want_atom_energy else None
    else:
        energy, forces, atom_e = out
    _check(getattr(lib(), _fn)(graph._h, ctypes.byref(weights.c), int(mode), ctypes.c_void_p(energy.data_ptr()),
                              ctypes.c_void_p(forces.data_ptr()),
                              ctypes.c_void_p(atom_e.data_ptr() if atom_e is not None else None)))
    return energy, forces, atom_e
