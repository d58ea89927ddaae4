"""GPU parity: neighbour lists, CSR and partition index sets are bit-exact against the oracle."""
import numpy as np
import pytest

import workloads as wl
from oracle import graph as og

from gpu_util import assert_graph_equal, gpu_graph, oracle_config

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("index", [0, 1])
def test_graph_configs(index):
    c, ref, _ = oracle_config(index)
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"])
    assert_graph_equal(g, ref, c["positions"], c["cell"])


@pytest.mark.parametrize("seed", range(8))
def test_graph_triclinic_small_cells(seed):
    """Random triclinic cells, some thinner than r_cut (multiple and self images), atoms outside the cell."""
    scale = [2.5, 4.0, 6.0, 9.0, 12.0, 3.0, 7.0, 15.0][seed]
    pos, cell, sp = wl.random_triclinic(14 + 3 * seed, seed, scale=scale, spread=1.0 + 0.4 * seed)
    ref = og.build_graph(pos, cell, 3.1)
    g = gpu_graph(pos, cell, sp, 3.1)
    assert_graph_equal(g, ref, pos, cell)


def test_graph_rows_longer_than_staging():
    """More than 96 neighbours per atom: the counting pass cannot park the keys, the second pass fills the rows."""
    c = wl.make_config(0, n=4)
    ref = og.build_graph(c["positions"], c["cell"], 7.0)
    assert np.diff(ref.row_ptr).min() > 96
    g = gpu_graph(c["positions"], c["cell"], c["species"], 7.0)
    assert_graph_equal(g, ref, c["positions"], c["cell"])
    # a mixed case: most rows short, a few long (a dense cluster inside a sparse box)
    rng = np.random.default_rng(5)
    pos = np.concatenate([rng.uniform(0, 40.0, (300, 3)), 20.0 + rng.uniform(0, 3.0, (130, 3))])
    cell = np.eye(3) * 40.0
    sp = np.zeros(len(pos), np.int32)
    ref = og.build_graph(pos, cell, 5.0)
    deg = np.diff(ref.row_ptr)
    assert deg.max() > 96 and np.median(deg) < 96
    g = gpu_graph(pos, cell, sp, 5.0)
    assert_graph_equal(g, ref, pos, cell)


def test_graph_edge_cases():
    import paper_2506_02023_amd as M
    cell = np.eye(3) * 30.0
    # single atom, no neighbours: E = 0
    g = gpu_graph(np.array([[1.0, 2, 3]]), cell, np.array([0]), 5.0)
    assert g.sizes() == (1, 0, 1)
    assert np.array_equal(g.csr()[0], [0, 0])
    # single atom in a tiny cell: only self images
    pos = np.array([[0.3, 0.2, 0.1]])
    small = np.eye(3) * 2.0
    ref = og.build_graph(pos, small, 3.1)
    assert_graph_equal(gpu_graph(pos, small, np.array([0]), 3.1), ref, pos, small)
    # handle reuse: big then small then big again
    c, ref0, _ = oracle_config(0)
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"])
    g = gpu_graph(pos, small, np.array([0]), 3.1, graph=g)
    assert_graph_equal(g, ref, pos, small)
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"], graph=g)
    assert_graph_equal(g, ref0)
    # errors: coincident atoms, singular cell, atom absurdly far away; the handle survives
    two = np.array([[1.0, 1, 1], [1.0, 1, 1]])
    with pytest.raises(M.MlipError) as ei:
        gpu_graph(two, cell, np.array([0, 0]), 5.0)
    assert ei.value.code == -3
    with pytest.raises(M.MlipError) as ei:
        gpu_graph(two + [[0, 0, 0], [1, 0, 0]], np.array([[1.0, 0, 0], [2.0, 0, 0], [0, 0, 1]]), np.array([0, 0]), 5.0)
    assert ei.value.code == -2
    with pytest.raises(M.MlipError) as ei:
        gpu_graph(np.array([[1e6, 0, 0], [1.0, 0, 0]]), cell, np.array([0, 0]), 5.0)
    assert ei.value.code == -2


def _check_partition(pos, cell, sp, r_cut, P):
    ref = og.build_graph(pos, cell, r_cut)
    slab_ref, ax_ref = og.slab_assign(pos, cell, P)
    slabs = og.partition(ref, slab_ref, P)
    g = gpu_graph(pos, cell, sp, r_cut, n_slabs=P)
    assert_graph_equal(g, ref)
    slab_gpu, ax = g.slab_of()
    assert ax == ax_ref and np.array_equal(slab_gpu, slab_ref)
    total_owned_edges = 0
    for p in range(P):
        s, r = g.slab(p), slabs[p]
        assert np.array_equal(s["owned_sorted"], r.owned)
        assert np.array_equal(s["nodes"], r.nodes)
        assert np.array_equal(s["markers"], r.markers)
        assert (s["n_pure"], s["n_border"], s["n_ghost"]) == (len(r.pure), len(r.border), len(r.ghost))
        assert np.array_equal(s["nodes"][: s["n_pure"]], r.pure)
        # owned rows of the local CSR are the oracle's local graph, bit for bit
        no = s["n_owned"]
        assert np.array_equal(s["row_ptr"][: no + 1], r.row_ptr)
        assert np.array_equal(s["senders"][: s["n_edges_owned"]], r.senders)
        total_owned_edges += s["n_edges_owned"]
        # ghost rows: the ghost atom's neighbours that this partition owns, canonical order
        for k in range(0, s["n_ghost"], max(1, s["n_ghost"] // 50)):
            u = s["nodes"][no + k]
            row = ref.senders[ref.row_ptr[u]: ref.row_ptr[u + 1]]
            want = row[slab_ref[row] == p]
            got = s["nodes"][s["senders"][s["row_ptr"][no + k]: s["row_ptr"][no + k + 1]]]
            assert np.array_equal(got, want)
        for q in range(P):
            assert np.array_equal(g.frm(p, q), r.frm[q])
            assert np.array_equal(g.to(p, q), r.to[q])
            assert g.bucket_address("to", p, q) == g.bucket_address("from", q, p)   # literally the same array
    assert total_owned_edges == ref.E


@pytest.mark.parametrize("P", [2, 3, 8])
def test_partition_config0(P):
    c, _, _ = oracle_config(0)
    _check_partition(c["positions"], c["cell"], c["species"], c["r_cut"], P)


@pytest.mark.parametrize("P", [2, 5])
def test_partition_triclinic(P):
    pos, cell, sp = wl.random_triclinic(300, 21, scale=14.0)
    _check_partition(pos, cell, sp, 3.0, P)


def test_partition_maximum_slab_count():
    """64 slabs (the limit) across a 21.6 A box: slabs a third of an Angstrom wide, every owned atom needed by many
    partitions (multi-valued TO), ghosts from dozens of owners."""
    c = wl.make_config(0, n=6)
    _check_partition(c["positions"], c["cell"], c["species"], c["r_cut"], 64)


def test_partition_medium_8_slabs():
    c, _, _ = oracle_config(1)
    _check_partition(c["positions"], c["cell"], c["species"], c["r_cut"], 8)


def test_mirror_index():
    """mirror[e] is the reverse edge: receiver and sender swapped, shift negated; an involution."""
    for pos, cell, sp, rc in [(*wl.random_triclinic(60, 4, scale=5.0)[:3], 3.3),
                              (*[oracle_config(0)[0][k] for k in ("positions", "cell", "species")], 5.0)]:
        g = gpu_graph(pos, cell, sp, rc)
        row_ptr, senders, shifts, _ = g.csr()
        recv = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))
        m = g.mirror()
        assert np.array_equal(m[m], np.arange(len(m)))
        assert np.array_equal(senders[m], recv) and np.array_equal(recv[m], senders)
        assert np.array_equal(shifts[m], -shifts)
        assert not np.any(m == np.arange(len(m)))


def _check_pairs(pos, cell, sp, r_cut, P):
    """The upper / lower split of the owned rows' edges (what the fp32 edge kernels walk) against the oracle's
    definition, bit for bit; where the reverse edge lies in a ghost row (which the oracle's local graph does not hold)
    the index the library gives is checked against the library's own local CSR instead."""
    ref = og.build_graph(pos, cell, r_cut)
    g = gpu_graph(pos, cell, sp, r_cut, n_slabs=P)
    _, _, _, d_all = g.csr()
    if P == 1:
        parts = [(-1, None, ref.row_ptr, np.arange(ref.E))]
    else:
        slab_ref, _ = og.slab_assign(pos, cell, P)
        parts = [(p, sl, sl.row_ptr, sl.edge_ids) for p, sl in enumerate(og.partition(ref, slab_ref, P))]
    for p, sl, row_ptr, edge_ids in parts:
        want = og.pair_split(ref, sl)
        got = g.pairs(p)
        assert got["n_upper"] == len(want["u_eid"]) and got["n_lower"] == len(want["l_slot"])
        for k in ("u_row_ptr", "u_senders", "u_eid", "l_row_ptr", "l_senders", "l_slot"):
            assert np.array_equal(got[k], want[k]), (p, k)
        assert np.array_equal(got["u_d"], d_all[edge_ids[want["u_eid"]]])   # the lengths are copies, not recomputed
        owned = want["u_mirror_owned"] >= 0
        assert np.array_equal(got["u_mirror"][owned], want["u_mirror_owned"][owned])
        if not owned.all():   # reverse edges in ghost rows: behind the owned rows' edges, in the sender's row, from the receiver
            s = g.slab(p)
            m = got["u_mirror"][~owned].astype(np.int64)
            assert (m >= s["n_edges_owned"]).all() and (m < s["n_edges"]).all()
            rows_of_m = np.searchsorted(s["row_ptr"], m, side="right") - 1
            assert np.array_equal(rows_of_m, got["u_senders"][~owned])
            recv_rows = np.repeat(np.arange(len(row_ptr) - 1), np.diff(row_ptr))[want["u_eid"][~owned]]
            assert np.array_equal(s["senders"][m], recv_rows)
            assert len(np.unique(m)) == len(m)


@pytest.mark.parametrize("P", [1, 3, 8])
def test_pair_split_config0(P):
    c, _, _ = oracle_config(0)
    _check_pairs(c["positions"], c["cell"], c["species"], c["r_cut"], P)


@pytest.mark.parametrize("P", [1, 5])
def test_pair_split_triclinic(P):
    pos, cell, sp = wl.random_triclinic(300, 21, scale=14.0)
    _check_pairs(pos, cell, sp, 3.0, P)


def test_pair_split_medium_8_slabs_and_many_slabs():
    c, _, _ = oracle_config(1)
    _check_pairs(c["positions"], c["cell"], c["species"], c["r_cut"], 8)
    c = wl.make_config(0, n=6)
    _check_pairs(c["positions"], c["cell"], c["species"], c["r_cut"], 64)   # thin slabs: most edges come from ghosts
