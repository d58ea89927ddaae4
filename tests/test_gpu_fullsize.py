"""GPU parity at the benchmark's full sizes.

configs[2] (108,000 atoms, 8 slabs): index sets bit-exact, whole-graph and partitioned energy/forces
against the full fp64 oracle.
configs[3] (1,000,188 atoms, the configuration bench.py times, 8 slabs): neighbour list and index
sets bit-exact against the oracle; total energy, every per-atom energy and every force component of
the whole-graph, the 8-slab and the split-fp16 runs against the full fp64 oracle run of the same
million atoms (relative energy error <= 1e-5, force error <= 1e-4 max|F|); as a second, independent
witness, sampled atoms recomputed by the oracle on the atom's own dependency cluster (all atoms within
2 L r_cut, which determines its energy and its force exactly), plus properties that hold at any size.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import graph as og
from oracle import model as om

from gpu_util import E_RTOL, F_RTOL, assert_energy_forces, assert_graph_equal, gpu_energy_forces, gpu_graph

pytestmark = pytest.mark.gpu
WHOLE, SLABS = 0, 1


def _check_sets(g, ref, pos, cell, P):
    slab_ref, ax_ref = og.slab_assign(pos, cell, P)
    slabs = og.partition(ref, slab_ref, P)
    slab_gpu, ax = g.slab_of()
    assert ax == ax_ref and np.array_equal(slab_gpu, slab_ref)
    for p in range(P):
        s, r = g.slab(p), slabs[p]
        assert np.array_equal(s["owned_sorted"], r.owned)
        assert np.array_equal(s["nodes"], r.nodes)                 # PURE | BORDER | FROM[0..P-1]
        assert np.array_equal(s["markers"], r.markers)
        no = s["n_owned"]
        assert np.array_equal(s["row_ptr"][: no + 1], r.row_ptr)
        assert np.array_equal(s["senders"][: s["n_edges_owned"]], r.senders)
        for q in range(P):
            assert np.array_equal(g.frm(p, q), r.frm[q])
            assert np.array_equal(g.to(p, q), r.to[q])
    return slab_ref


def test_config2_partition_equivalence():
    c = wl.make_config(2)
    pos, cell, sp = c["positions"], c["cell"], c["species"]
    ref_g = og.build_graph(pos, cell, c["r_cut"])
    ref = om.energy_forces(pos, cell, sp, c["weights"], ref_g, c["r_cut"], c["K"], c["p"])
    g = gpu_graph(pos, cell, sp, c["r_cut"], n_slabs=8)
    assert_graph_equal(g, ref_g, pos, cell)
    _check_sets(g, ref_g, pos, cell, 8)
    ew, fw, aw = gpu_energy_forces(g, c["weights"], c["p"], WHOLE)
    es, fs, as_ = gpu_energy_forces(g, c["weights"], c["p"], SLABS)
    dw = assert_energy_forces(ew, fw, ref, "configs[2] whole")
    ds = assert_energy_forces(es, fs, ref, "configs[2] 8 slabs")
    e2, f2, _ = gpu_energy_forces(g, c["weights"], c["p"], SLABS, precision=2)   # split-fp16 W2 products, same bounds
    d2 = assert_energy_forces(e2, f2, ref, "configs[2] 8 slabs, split-fp16 products")
    print(f"configs[2] split-fp16 products: dE/E {d2[0]:.2e} dF {d2[1]:.2e}")
    assert abs(es - ew) <= E_RTOL * abs(ew)
    assert np.abs(fs - fw).max() <= F_RTOL * np.abs(fw).max()
    print(f"configs[2]: whole dE/E {dw[0]:.2e} dF {dw[1]:.2e}; slabs dE/E {ds[0]:.2e} dF {ds[1]:.2e}")


def _cluster(pos, cell, centre, radius):
    """All atoms (minimum image) within `radius` of atom `centre`, as a free cluster in a big box."""
    inv = np.linalg.inv(cell)
    d = pos - pos[centre]
    frac = d @ inv
    d = (frac - np.round(frac)) @ cell
    sel = np.flatnonzero((d * d).sum(1) <= radius * radius)
    box = 4.0 * radius
    return sel, d[sel] + box / 2, np.eye(3) * box


def test_config3_million_atoms():
    c = wl.make_config(3)
    pos, cell, sp = c["positions"], c["cell"], c["species"]
    N = len(sp)
    P = 8
    ref_g = og.build_graph(pos, cell, c["r_cut"])
    g = gpu_graph(pos, cell, sp, c["r_cut"], n_slabs=P)
    assert_graph_equal(g, ref_g, pos, cell)
    slab_of = _check_sets(g, ref_g, pos, cell, P)
    ew, fw, aw = gpu_energy_forces(g, c["weights"], c["p"], WHOLE)
    es, fs, as_ = gpu_energy_forces(g, c["weights"], c["p"], SLABS)
    e2, f2, a2 = gpu_energy_forces(g, c["weights"], c["p"], SLABS, precision=2)   # split-fp16 W2 products
    # the same unpartitioned: 45.8 M kept rows do not fit one descriptor's range, so every edge keeps its own filter
    # values there, where in the slabs only the upper edge of a pair does
    e3, f3, a3 = gpu_energy_forces(g, c["weights"], c["p"], WHOLE, precision=2)
    # properties: reductions consistent, zero net force, partitioned == whole
    assert abs(ew - aw.sum()) <= 1e-9 * abs(ew) and abs(es - as_.sum()) <= 1e-9 * abs(es)
    fmax = np.abs(fw).max()
    assert np.abs(fw.sum(0)).max() <= 1e-6 * fmax * np.sqrt(N)
    assert np.abs(fs.sum(0)).max() <= 1e-6 * fmax * np.sqrt(N)
    assert abs(es - ew) <= E_RTOL * abs(ew)
    assert np.abs(fs - fw).max() <= F_RTOL * fmax
    # the full fp64 oracle on the same 1,000,188 atoms: total energy and all forces, every mode
    ref_full = om.energy_forces(pos, cell, sp, c["weights"], ref_g, c["r_cut"], c["K"], c["p"])
    eps_scale = np.abs(ref_full["atom_energy"]).mean()
    for what, e_, f_, a_ in (("whole", ew, fw, aw), ("8 slabs", es, fs, as_), ("8 slabs, split-fp16 products", e2, f2, a2),
                             ("whole, split-fp16 products", e3, f3, a3)):
        de, df = assert_energy_forces(e_, f_, ref_full, "configs[3] " + what)
        da = np.abs(a_ - ref_full["atom_energy"]).max() / eps_scale
        print(f"configs[3] {what} against the full oracle: dE/E {de:.2e}, dF {df:.2e} of max|F|, "
              f"worst atom energy {da:.2e} of mean|eps|")
        assert da <= 1e-4, (what, da)      # a single fp32 atom energy; the 1e-5 bound is on the total
    # sampled atoms: near a slab wall, near the box faces, and in the bulk
    L = c["L"]
    radius = 2 * L * c["r_cut"] + 0.5
    x = np.mod(pos[:, 0], cell[0, 0])
    wall = cell[0, 0] / P * 3
    samples = [int(np.argmin(np.abs(x - wall))), 0, N - 1, int(np.argmax(x)), N // 2 + 17, N // 3]
    worst_e = worst_f = 0.0
    for i in samples:
        sel, cpos, ccell = _cluster(pos, cell, i, radius)
        cg = og.build_graph(cpos, ccell, c["r_cut"])
        ref = om.energy_forces(cpos, ccell, sp[sel], c["weights"], cg, c["r_cut"], c["K"], c["p"])
        k = int(np.flatnonzero(sel == i)[0])
        # the two oracle routes (periodic million-atom run, free cluster) agree on this atom
        assert abs(ref["atom_energy"][k] - ref_full["atom_energy"][i]) <= 1e-9 * eps_scale
        assert np.abs(ref["forces"][k] - ref_full["forces"][i]).max() <= 1e-9 * fmax
        # the cluster graph reproduces the atom's row of the periodic graph
        assert cg.row_ptr[k + 1] - cg.row_ptr[k] == ref_g.row_ptr[i + 1] - ref_g.row_ptr[i]
        for ae, ff in ((aw, fw), (as_, fs), (a2, f2)):
            de = abs(ae[i] - ref["atom_energy"][k]) / max(abs(ref["atom_energy"][k]), np.abs(aw).mean())
            df = np.abs(ff[i] - ref["forces"][k]).max() / fmax
            worst_e, worst_f = max(worst_e, de), max(worst_f, df)
            assert de <= 1e-4, (i, de)          # one fp32 atom energy; the 1e-5 bound is on the total
            assert df <= F_RTOL, (i, df)
    print(f"configs[3]: {len(samples)} sampled atoms, worst atom-energy error {worst_e:.2e}, "
          f"worst force error {worst_f:.2e} of max|F|; E = {ew:.6f}, |E_slabs - E_whole|/|E| = {abs(es - ew) / abs(ew):.1e}")
