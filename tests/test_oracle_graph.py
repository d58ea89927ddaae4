"""Pins for the oracle's neighbour list, slab rule and partition index sets (CPU only)."""
import itertools
import os

import numpy as np
import pytest

import workloads as wl
from oracle import graph as og

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "lattice_shells.txt")


def _shells(lattice):
    rows = []
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        name, _, d2, cnt = line.split()
        if name == lattice:
            rows.append((float(d2), int(cnt)))
    return rows


def _same(a, b):
    return (a.E == b.E and np.array_equal(a.row_ptr, b.row_ptr) and np.array_equal(a.senders, b.senders)
            and np.array_equal(a.shifts, b.shifts))


@pytest.mark.parametrize("method", ["brute", "cells"])
@pytest.mark.parametrize("lattice", ["sc", "fcc", "bcc"])
def test_lattice_shell_counts(lattice, method):
    """Closed form: cumulative coordination numbers of ideal lattices (one atom per primitive cell
    for sc -> every neighbour is a periodic image of the atom itself)."""
    a = 2.0
    basis = {"sc": [[0, 0, 0]], "fcc": [[0, 0, 0], [0, .5, .5], [.5, 0, .5], [.5, .5, 0]],
             "bcc": [[0, 0, 0], [.5, .5, .5]]}[lattice]
    pos = np.array(basis, float) * a
    cell = np.eye(3) * a
    total = 0
    shells = _shells(lattice)
    for k, (d2, cnt) in enumerate(shells):
        total += cnt
        nxt = shells[k + 1][0] if k + 1 < len(shells) else d2 + 0.4
        r_cut = a * np.sqrt(0.5 * (d2 + nxt))     # between this shell and the next
        g = og.build_graph(pos, cell, r_cut, method)
        assert np.all(np.diff(g.row_ptr) == total), (lattice, k)


def test_fcc_benchmark_counts():
    """Un-jittered benchmark lattice: exactly 42 neighbours at r_cut = 5.0, 12 at r_cut = 3.0."""
    pos, cell, _ = wl.fcc_lattice(4, 0.0, 1, seed=1)
    g = og.build_graph(pos, cell, 5.0)
    assert g.E == 42 * len(pos) and np.all(np.diff(g.row_ptr) == 42)
    g = og.build_graph(pos, cell, 3.0)
    assert g.E == 12 * len(pos)


def test_inclusive_cutoff():
    """d == r_cut is an edge (inclusive); the next representable cutoff below is not."""
    pos = np.array([[0.0, 0, 0], [3.0, 0, 0]])
    cell = np.eye(3) * 20.0
    assert og.build_graph(pos, cell, 3.0, "brute").E == 2
    assert og.build_graph(pos, cell, np.nextafter(3.0, 0), "brute").E == 0
    assert og.build_graph(pos, cell, 3.0, "cells").E == 2
    assert og.build_graph(pos, cell, np.nextafter(3.0, 0), "cells").E == 0


@pytest.mark.parametrize("seed", range(8))
def test_cells_equal_brute_triclinic(seed):
    """Cell list == brute force on random triclinic cells, including cells thinner than
    r_cut (several images of one atom, self images) and atoms outside the cell."""
    scale = [2.5, 4.0, 6.0, 9.0, 12.0, 3.0, 7.0, 15.0][seed]
    pos, cell, _ = wl.random_triclinic(14 + 3 * seed, seed, scale=scale, spread=1.0 + 0.4 * seed)
    r_cut = 3.1
    a = og.build_graph(pos, cell, r_cut, "brute")
    b = og.build_graph(pos, cell, r_cut, "cells")
    assert a.E > 0 and _same(a, b)


def test_cells_equal_brute_config0():
    c = wl.make_config(0)
    a = og.build_graph(c["positions"], c["cell"], c["r_cut"], "brute")
    b = og.build_graph(c["positions"], c["cell"], c["r_cut"], "cells")
    assert _same(a, b)
    assert 4536 < a.E < 5400       # 42 N plus part of the 5.09 A shell


def test_edges_match_python_definition():
    """Edge set against the definition evaluated with Python floats (pair by pair, image by image)."""
    pos, cell, _ = wl.random_triclinic(9, 77, scale=4.0)
    r_cut = 2.9
    g = og.build_graph(pos, cell, r_cut, "cells")
    want = []
    rng = range(-4, 5)
    for i in range(len(pos)):
        for j in range(len(pos)):
            for S in itertools.product(rng, rng, rng):
                if i == j and S == (0, 0, 0):
                    continue
                d2 = 0.0
                dl = []
                for k in range(3):
                    sh = (S[0] * cell[0, k] + S[1] * cell[1, k]) + S[2] * cell[2, k]
                    dl.append((pos[j, k] - pos[i, k]) + sh)
                d2 = (dl[0] * dl[0] + dl[1] * dl[1]) + dl[2] * dl[2]
                if d2 <= r_cut * r_cut:
                    want.append((i, j) + S)
    got = [(int(i), int(j), *map(int, s)) for i, j, s in zip(g.receivers, g.senders, g.shifts)]
    assert got == want            # same set, same canonical order


def test_edge_set_symmetry_and_order():
    c = wl.make_config(0)
    g = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    fwd = set(zip(g.receivers.tolist(), g.senders.tolist(), map(tuple, g.shifts.tolist())))
    rev = set((j, i, (-s[0], -s[1], -s[2])) for i, j, s in fwd)
    assert fwd == rev
    keys = np.column_stack([g.receivers, g.senders, g.shifts]).tolist()
    assert keys == sorted(keys)


def test_translation_by_lattice_vector_changes_only_shifts():
    """Moving one atom by a lattice vector keeps its neighbours and moves the shifts by one."""
    c = wl.make_config(0)
    g0 = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    pos = c["positions"].copy()
    pos[10] += c["cell"][0] * 2 - c["cell"][2]
    g1 = og.build_graph(pos, c["cell"], c["r_cut"])
    assert g1.E == g0.E and np.array_equal(np.diff(g0.row_ptr), np.diff(g1.row_ptr))
    assert np.array_equal(np.sort(g0.senders[g0.row_ptr[10]:g0.row_ptr[11]]),
                          np.sort(g1.senders[g1.row_ptr[10]:g1.row_ptr[11]]))


# ---------------------------------------------------------------- slabs / index sets

def test_slab_rule_axis_and_bins():
    pos = np.array([[0.1, 0, 0], [4.9, 1, 1], [5.0, 2, 2], [9.99, 3, 3], [-0.1, 0, 0], [10.0, 0, 0], [25.0, 0, 0]])
    cell = np.diag([10.0, 4.0, 4.0])
    slab, ax = og.slab_assign(pos, cell, 2)
    assert ax == 0
    assert slab.tolist() == [0, 0, 1, 1, 1, 0, 1]
    # ties -> lowest axis; longest vector wins even if listed last
    assert og.slab_assign(pos, np.eye(3) * 7.0, 3)[1] == 0
    assert og.slab_assign(pos, np.diag([3.0, 4.0, 9.0]), 3)[1] == 2


def _sets_by_definition(g, slab_of, P):
    """The paper's definitions as Python set comprehensions."""
    edges = list(zip(g.receivers.tolist(), g.senders.tolist()))
    G = [set(np.flatnonzero(slab_of == p).tolist()) for p in range(P)]
    H = [set(v for (u, v) in edges if u in G[p] and v not in G[p]) for p in range(P)]
    TO = [[set(v for (u, v) in edges if v in G[p] and u in G[q]) if q != p else set() for q in range(P)]
          for p in range(P)]
    return G, H, TO


@pytest.mark.parametrize("P", [1, 2, 3, 8])
@pytest.mark.parametrize("case", ["config0", "triclinic"])
def test_index_sets_against_definitions(case, P):
    if case == "config0":
        c = wl.make_config(0)
        pos, cell = c["positions"], c["cell"]
        r_cut = 5.0
    else:
        pos, cell, _ = wl.random_triclinic(60, 5, scale=9.0)
        r_cut = 3.0
    g = og.build_graph(pos, cell, r_cut)
    slab_of, _ = og.slab_assign(pos, cell, P)
    slabs = og.partition(g, slab_of, P)
    G, H, TO = _sets_by_definition(g, slab_of, P)
    all_owned = []
    n_edges = 0
    for p, sl in enumerate(slabs):
        assert set(sl.owned.tolist()) == G[p] and np.all(np.diff(sl.owned) > 0)
        assert set(sl.ghost.tolist()) == H[p] and len(set(sl.ghost.tolist())) == len(sl.ghost)
        for q in range(P):
            assert set(sl.to[q].tolist()) == TO[p][q]
            assert np.array_equal(sl.to[q], slabs[q].frm[p])          # TO_p[q] and FROM_q[p]: same array
            assert np.all(np.diff(sl.to[q]) > 0)
        border = set().union(*TO[p]) if P > 1 else set()
        assert set(sl.pure.tolist()) == G[p] - border
        assert set(sl.border.tolist()) == border
        # node array and markers
        assert np.array_equal(sl.nodes, np.concatenate([sl.pure, sl.border] + [sl.frm[q] for q in range(P)]))
        assert sl.markers[0] == 0 and sl.markers[-1] == len(sl.nodes) and len(sl.markers) == P + 3
        assert sl.markers[2] == len(sl.owned)
        # local graph: every edge whose receiver is owned, once, in row order
        n_edges += len(sl.edge_ids)
        assert np.array_equal(sl.nodes[sl.senders], g.senders[sl.edge_ids])
        all_owned += sl.owned.tolist()
    assert sorted(all_owned) == list(range(g.N))         # disjoint cover
    assert n_edges == g.E                                # every edge in exactly one partition
    if P == 1:
        assert len(slabs[0].ghost) == 0 and len(slabs[0].pure) == g.N


def test_wide_slabs_talk_to_neighbours_only():
    """Slab width >= r_cut and P >= 3: ghosts come from slabs p-1 and p+1 (periodic) only,
    and lie within one cutoff of the slab (the geometric shell contains the graph-defined ghosts)."""
    pos, cell, _ = wl.fcc_lattice(6, 0.05, 2, seed=3)      # 21.6 A box, 3 slabs of 7.2 A
    P, r_cut = 3, 5.0
    g = og.build_graph(pos, cell, r_cut)
    slab_of, ax = og.slab_assign(pos, cell, P)
    slabs = og.partition(g, slab_of, P)
    Lx = cell[0, 0]
    for p, sl in enumerate(slabs):
        assert len(sl.ghost) > 0
        for q in range(P):
            if q not in ((p - 1) % P, (p + 1) % P):
                assert len(sl.frm[q]) == 0
        x = np.mod(pos[sl.ghost, 0], Lx)
        lo, hi = p * Lx / P, (p + 1) * Lx / P
        dist = np.minimum(np.abs((x - lo + Lx / 2) % Lx - Lx / 2), np.abs((x - hi + Lx / 2) % Lx - Lx / 2))
        assert np.all(dist <= r_cut + 1e-9)


@pytest.mark.parametrize("P", [1, 3])
def test_pair_split_against_a_python_walk(P):
    """reverse_edges and pair_split against plain loops over the edge list of a small triclinic system: every pair of
    owned-row edges has exactly one upper edge (the earlier one), an edge whose reverse edge is not an owned row's
    edge is upper, and a lower edge's slot names its reverse edge among the upper ones."""
    pos, cell, _ = wl.random_triclinic(40, 11, scale=6.0)
    g = og.build_graph(pos, cell, 3.5)
    recv = g.receivers
    table = {(int(recv[e]), int(g.senders[e]), *map(int, g.shifts[e])): e for e in range(g.E)}
    mirror = og.reverse_edges(g)
    for e in range(g.E):
        s = g.shifts[e]
        assert mirror[e] == table[(int(g.senders[e]), int(recv[e]), int(-s[0]), int(-s[1]), int(-s[2]))]
    slab_of, _ = og.slab_assign(pos, cell, P)
    for sl in og.partition(g, slab_of, P):
        q = og.pair_split(g, sl if P > 1 else None)
        edge_ids = sl.edge_ids if P > 1 else np.arange(g.E)
        pos_of = {int(ge): k for k, ge in enumerate(edge_ids)}
        uppers, lowers = [], []
        for k, ge in enumerate(edge_ids):
            m = pos_of.get(int(mirror[ge]), -1)
            (uppers if (m < 0 or m > k) else lowers).append(k)
        assert list(q["u_eid"]) == uppers
        n_ghost_edges = sum(1 for k in uppers if pos_of.get(int(mirror[edge_ids[k]]), -1) < 0)
        assert len(uppers) == (len(edge_ids) - n_ghost_edges) // 2 + n_ghost_edges
        assert len(q["l_slot"]) == len(lowers)
        for t, k in enumerate(lowers):
            upper_of_pair = uppers[q["l_slot"][t]]
            assert edge_ids[upper_of_pair] == mirror[edge_ids[k]]
        # row pointers: the upper / lower edges of every row, in order
        row_ptr = sl.row_ptr if P > 1 else g.row_ptr
        for r in range(len(row_ptr) - 1):
            in_row = [k for k in uppers if row_ptr[r] <= k < row_ptr[r + 1]]
            assert list(q["u_eid"][q["u_row_ptr"][r]: q["u_row_ptr"][r + 1]]) == in_row
            assert q["l_row_ptr"][r + 1] - q["l_row_ptr"][r] == (row_ptr[r + 1] - row_ptr[r]) - len(in_row)
