"""Oracle: periodic radius graph, slab rule and partition index sets.

TEST INFRASTRUCTURE ONLY (see mlip_oracle.c).  The index sets are the paper's
set definitions written out with numpy on the global edge list:

  G_p  = owned_p                      nodes whose slab is p
  H_p  = ghost_p  = { v not in G_p : exists u in G_p with edge u <- v }
         (Graph-Parallel Message Passing, definitions of G'_i and H_i)
  TO_p[q]   = { u in G_p : exists v in G_q, q != p, with edge v <- u }
  FROM_p[q] = TO_q[p]                 ("should be the same array")
  PURE_p    = G_p minus the union of TO_p[.]
  an edge belongs to the partition of its receiving node
  (Distributing Atom Graphs; Alg. "assign_to_partitions"; Alg. "Atom Subgraph Creation")

Readings taken where the printed algorithms are garbled or silent:
  * the node table of assign_to_partitions is indexed by the edge's source
    node and only written when source and destination lie in different
    partitions (otherwise no node could be PURE);
  * a node may be needed by several partitions, so TO is multi-valued;
  * the per-partition node array is PURE | BORDER | FROM[0] | ... | FROM[P-1]
    with BORDER = owned non-pure nodes stored once, all spans in ascending
    global id; markers are the span starts (exclusive prefix sums).
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass, field

import numpy as np

from ._lib import c_f64p, c_i32p, lib


def _p(a, t):
    return a.ctypes.data_as(t)


@dataclass
class Graph:
    N: int
    E: int
    row_ptr: np.ndarray  # int64 [N+1]
    senders: np.ndarray  # int32 [E]
    shifts: np.ndarray   # int32 [E,3]

    @property
    def receivers(self):
        return np.repeat(np.arange(self.N, dtype=np.int32), np.diff(self.row_ptr))


def _take(gp):
    g = gp.contents
    N, E = int(g.N), int(g.E)
    row_ptr = np.ctypeslib.as_array(g.row_ptr, shape=(N + 1,)).copy()
    if E:
        senders = np.ctypeslib.as_array(g.senders, shape=(E,)).copy()
        shifts = np.ctypeslib.as_array(g.shifts, shape=(E, 3)).copy()
    else:
        senders = np.zeros(0, np.int32)
        shifts = np.zeros((0, 3), np.int32)
    lib().orc_graph_free(gp)
    return Graph(N, E, row_ptr, senders, shifts)


def build_graph(positions, cell, r_cut, method="cells"):
    """Edges (i <- j, S) with 0 < |r_j + S.C - r_i| <= r_cut, sorted by (i, j, Sx, Sy, Sz)."""
    pos = np.ascontiguousarray(positions, np.float64)
    C = np.ascontiguousarray(cell, np.float64)
    fn = lib().orc_build_brute if method == "brute" else lib().orc_build_cells
    gp = fn(pos.shape[0], _p(pos, c_f64p), _p(C, c_f64p), float(r_cut))
    if not gp:
        raise ValueError("singular cell or no atoms")
    return _take(gp)


def slab_assign(positions, cell, n_slabs):
    """slab index of every atom and the axis used (vertical-wall rule)."""
    pos = np.ascontiguousarray(positions, np.float64)
    C = np.ascontiguousarray(cell, np.float64)
    out = np.zeros(pos.shape[0], np.int32)
    ax = ctypes.c_int32(0)
    rc = lib().orc_slab_assign(pos.shape[0], _p(pos, c_f64p), _p(C, c_f64p), int(n_slabs),
                               _p(out, c_i32p), ctypes.byref(ax))
    if rc:
        raise ValueError("singular cell")
    return out, int(ax.value)


def geometry(positions, cell, graph):
    """(d [E], rhat [E,3]) in fp64 for the edges of `graph`."""
    pos = np.ascontiguousarray(positions, np.float64)
    C = np.ascontiguousarray(cell, np.float64)
    d = np.zeros(graph.E, np.float64)
    rhat = np.zeros((graph.E, 3), np.float64)
    from ._lib import c_i64p
    lib().orc_geometry(graph.N, _p(pos, c_f64p), _p(C, c_f64p), _p(graph.row_ptr, c_i64p),
                       _p(graph.senders, c_i32p), _p(np.ascontiguousarray(graph.shifts), c_i32p),
                       _p(d, c_f64p), _p(rhat, c_f64p))
    return d, rhat


@dataclass
class Slab:
    p: int
    owned: np.ndarray          # ascending global ids
    pure: np.ndarray
    border: np.ndarray         # owned, non-pure
    ghost: np.ndarray          # FROM[0] | FROM[1] | ... (owner slab ascending, ids ascending)
    to: dict = field(default_factory=dict)     # q -> ascending global ids
    frm: dict = field(default_factory=dict)    # q -> ascending global ids
    nodes: np.ndarray = None   # local -> global: pure | border | ghost
    markers: np.ndarray = None  # [0, |pure|, |pure|+|border|, + cumulative FROM[q] ...]  (P + 3 entries)
    row_ptr: np.ndarray = None  # int64 [n_owned + 1], rows in local order
    senders: np.ndarray = None  # int32 local ids
    edge_ids: np.ndarray = None  # int64 global edge index of every local edge


def partition(graph, slab_of, n_slabs):
    """All index sets and local graphs of the slab partition, from the definitions."""
    P = int(n_slabs)
    recv = graph.receivers
    send = graph.senders
    s_recv = slab_of[recv]
    s_send = slab_of[send]
    slabs = []
    for p in range(P):
        owned = np.flatnonzero(slab_of == p).astype(np.int32)
        slabs.append(Slab(p=p, owned=owned, pure=None, border=None, ghost=None))
    cross = np.flatnonzero(s_recv != s_send)      # only edges that cross a wall define TO / FROM
    c_send, c_ss, c_sr = send[cross], s_send[cross], s_recv[cross]
    for p in range(P):
        sl = slabs[p]
        needed_anywhere = []
        from_p = c_ss == p
        for q in range(P):
            if q == p:
                sl.to[q] = np.zeros(0, np.int32)
                continue
            # u owned by p, some receiver v owned by q
            sl.to[q] = np.unique(c_send[from_p & (c_sr == q)]).astype(np.int32)
            needed_anywhere.append(sl.to[q])
        border = np.unique(np.concatenate(needed_anywhere)) if needed_anywhere else np.zeros(0, np.int32)
        sl.border = border.astype(np.int32)
        sl.pure = np.setdiff1d(sl.owned, sl.border).astype(np.int32)
    for p in range(P):
        sl = slabs[p]
        for q in range(P):
            sl.frm[q] = slabs[q].to[p] if q != p else np.zeros(0, np.int32)
        sl.ghost = (np.concatenate([sl.frm[q] for q in range(P)]) if P > 0 else np.zeros(0)).astype(np.int32)
        sl.nodes = np.concatenate([sl.pure, sl.border, sl.ghost]).astype(np.int32)
        lens = [len(sl.pure), len(sl.border)] + [len(sl.frm[q]) for q in range(P)]
        sl.markers = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
        # local graph: rows = owned nodes in local order, each row = the node's global row
        local_of = np.full(graph.N, -1, np.int64)
        local_of[sl.nodes] = np.arange(len(sl.nodes))
        own_local = sl.nodes[: len(sl.owned)]
        starts = graph.row_ptr[own_local]
        lens_r = graph.row_ptr[own_local + 1] - starts
        sl.row_ptr = np.concatenate([[0], np.cumsum(lens_r)]).astype(np.int64)
        total = int(sl.row_ptr[-1])
        sl.edge_ids = (np.arange(total, dtype=np.int64) - np.repeat(sl.row_ptr[:-1], lens_r)
                       + np.repeat(starts, lens_r))
        sl.senders = local_of[send[sl.edge_ids]].astype(np.int32)
        assert (sl.senders >= 0).all()
    return slabs


def reverse_edges(graph):
    """mirror[e] = index of the edge with sender and receiver swapped and the image shift negated.  It exists for
    every edge: the radius-graph predicate is symmetric (Methods, "Distributing Atom Graphs": atoms within the cutoff
    of each other are joined in both directions)."""
    recv = graph.receivers.astype(np.int64)
    send = graph.senders.astype(np.int64)
    S = graph.shifts.astype(np.int64)
    fwd = np.lexsort((S[:, 2], S[:, 1], S[:, 0], send, recv))          # edges by (receiver, sender, shift)
    rev = np.lexsort((-S[:, 2], -S[:, 1], -S[:, 0], recv, send))       # edges by (sender, receiver, -shift)
    mirror = np.empty(graph.E, np.int64)
    mirror[rev] = fwd
    assert np.array_equal(recv[mirror], send) and np.array_equal(send[mirror], recv)
    assert np.array_equal(S[mirror], -S)
    return mirror


def pair_split(graph, slab=None):
    """Upper / lower split of the edges of a partition's owned rows (slab=None: of the whole graph), by definition:
    the two edges of an edge / reverse-edge pair have the same length, hence the same filter values (the filter of the
    benchmark's message-passing layer is a function of the edge length alone), so one of them, the "upper" one, stands
    for the pair: the one that comes first in the partition's edge list (owned rows in local order, each a copy of
    the atom's global row; rows of ghost atoms come after all owned rows, so an edge from a ghost sender is upper).

    Returns a dict: u_row_ptr, u_senders (local rows), u_eid (position in the partition's list of owned-row edges),
    u_mirror_owned (position of the reverse edge in that list, -1 if it lies in a ghost row), l_row_ptr, l_senders,
    l_slot (index of the pair's upper edge among the upper edges)."""
    mirror = reverse_edges(graph)
    if slab is None:
        n_rows = graph.N
        row_ptr = graph.row_ptr.astype(np.int64)
        edge_ids = np.arange(graph.E, dtype=np.int64)
        senders = graph.senders.astype(np.int64)
    else:
        n_rows = len(slab.owned)
        row_ptr = slab.row_ptr.astype(np.int64)
        edge_ids = slab.edge_ids.astype(np.int64)
        senders = slab.senders.astype(np.int64)
    E_own = len(edge_ids)
    # position of every global edge in this partition's list of owned-row edges (-1: not an owned row's edge)
    pos_of = np.full(graph.E, -1, np.int64)
    pos_of[edge_ids] = np.arange(E_own)
    m_pos = pos_of[mirror[edge_ids]]
    e_pos = np.arange(E_own)
    upper = (m_pos < 0) | (m_pos > e_pos)
    assert not np.any(m_pos == e_pos)
    rows = np.repeat(np.arange(n_rows), np.diff(row_ptr))
    out = {}
    up = np.flatnonzero(upper)
    lo = np.flatnonzero(~upper)
    out["u_row_ptr"] = np.concatenate([[0], np.cumsum(np.bincount(rows[up], minlength=n_rows))]).astype(np.int64)
    out["l_row_ptr"] = np.concatenate([[0], np.cumsum(np.bincount(rows[lo], minlength=n_rows))]).astype(np.int64)
    out["u_senders"] = senders[up].astype(np.int32)
    out["u_eid"] = up.astype(np.int32)
    out["u_mirror_owned"] = m_pos[up].astype(np.int64)
    out["l_senders"] = senders[lo].astype(np.int32)
    index_among_upper = np.full(E_own, -1, np.int64)
    index_among_upper[up] = np.arange(len(up))
    out["l_slot"] = index_among_upper[m_pos[lo]].astype(np.int32)
    assert (out["l_slot"] >= 0).all()
    return out
