"""Pins of the three-body (bond graph) oracle: what the mathematics fixes, not the oracle's own formulas.

Benchmark configuration 4 gives counts (about 12 bonds and 132 triplets per atom); everything else is pinned by
closed forms on the perfect lattice, an independent loop-level re-derivation, finite differences, invariances,
the reduction to the (separately pinned) two-body model, and continuity where a bond crosses the bond cutoff.
"""
import numpy as np
import pytest

import workloads as wl
from oracle import graph as og
from oracle import model as om
from oracle import three_body as tb


def _cfg(n=3, sigma=None, seed=None):
    c = wl.make_config(4, n=n, seed=seed)
    if sigma is not None:
        pos, cell, sp = wl.fcc_lattice(n, sigma, 4, wl.BASE_SEED + 4)
        c["positions"], c["cell"], c["species"] = pos, cell, sp
    return c


def _run(c, pos=None, weights=None, species=None, cell=None, fp32=False):
    pos = c["positions"] if pos is None else pos
    cell = c["cell"] if cell is None else cell
    g = og.build_graph(pos, cell, c["r_cut"])
    return tb.energy_forces3(pos, cell, c["species"] if species is None else species,
                             c["weights"] if weights is None else weights, g, c["r_cut"], c["r_bond"], c["K"], c["p"],
                             fp32=fp32), g


def test_perfect_fcc_counts_and_angles():
    """fcc at a = 3.6: 12 nearest neighbours at a/sqrt(2) = 2.546 < 3.0 < a, so 12 bonds and 12*11 = 132
    ordered triplets per atom; seen from one bond the other 11 make angles of 60 (4x), 90 (2x), 120 (4x)
    and 180 degrees (1x)."""
    c = _cfg(n=3, sigma=0.0)
    g = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    bond_edge, bptr, bond_of_edge = tb.bond_graph(c["positions"], c["cell"], g, c["r_bond"])
    assert np.all(np.diff(bptr) == 12)
    assert len(bond_edge) == 12 * g.N
    assert (bond_of_edge >= 0).sum() == len(bond_edge) and np.array_equal(bond_of_edge[bond_edge], np.arange(len(bond_edge)))
    d, rhat = og.geometry(c["positions"], c["cell"], g)
    assert np.allclose(d[bond_edge], 3.6 / np.sqrt(2))
    assert np.all(d[bond_of_edge < 0] > 3.0)
    for i in (0, 17, g.N - 1):
        r = rhat[bond_edge[bptr[i]:bptr[i + 1]]]
        cosines = np.round(r @ r.T, 6)
        for row in range(12):
            others = np.delete(cosines[row], row)
            vals, counts = np.unique(others, return_counts=True)
            assert dict(zip(vals.tolist(), counts.tolist())) == {-1.0: 1, -0.5: 4, 0.0: 2, 0.5: 4}


def test_jittered_counts_match_the_benchmark_description():
    c = _cfg(n=6)
    r, g = _run(c)
    assert abs(r["n_bonds"] / g.N - 12) < 0.1          # "about 12 bonds per atom"
    assert abs(r["n_triplets"] / g.N - 132) < 2.5      # "about 132 per atom"


def test_angle_basis_is_cos_n_theta():
    theta = np.linspace(0.0, np.pi, 37)
    T = tb.angle_basis(np.cos(theta))
    assert T.shape == (37, 8)
    assert np.allclose(T, np.cos(np.arange(8)[None, :] * theta[:, None]), atol=1e-13)


def test_energy_matches_loop_rederivation():
    """Independent re-derivation: python loops over atoms, bonds and triplets, arccos + cos(n theta) instead of
    the recurrence, one concatenated Linear instead of split products."""
    c = _cfg(n=3)
    r, g = _run(c)
    e = tb.energy3_reference(c["positions"], c["cell"], c["species"], c["weights"], g, c["r_cut"], c["r_bond"], c["K"], c["p"])
    assert abs(e - r["energy"]) <= 1e-11 * abs(e)
    # a triclinic cell with a few atoms, images included
    pos, cell, sp = wl.random_triclinic(9, 3, scale=5.0)
    g = og.build_graph(pos, cell, c["r_cut"])
    r = tb.energy_forces3(pos, cell, sp, c["weights"], g, c["r_cut"], c["r_bond"], c["K"], c["p"])
    e = tb.energy3_reference(pos, cell, sp, c["weights"], g, c["r_cut"], c["r_bond"], c["K"], c["p"])
    assert r["n_triplets"] > 0
    assert abs(e - r["energy"]) <= 1e-11 * abs(e)


def test_forces_are_minus_the_energy_gradient():
    c = _cfg(n=3)
    r, g = _run(c)
    fmax = np.abs(r["forces"]).max()
    rng = np.random.default_rng(1)
    h = 1e-4
    for _ in range(8):
        i, k = int(rng.integers(g.N)), int(rng.integers(3))
        pp = c["positions"].copy()
        pp[i, k] += h
        ep = _run(c, pos=pp)[0]["energy"]
        pp[i, k] -= 2 * h
        em = _run(c, pos=pp)[0]["energy"]
        assert abs(-(ep - em) / (2 * h) - r["forces"][i, k]) <= 1e-6 * fmax
    assert np.abs(r["forces"].sum(0)).max() <= 1e-10 * fmax


def test_without_bond_term_it_is_the_two_body_model():
    """Wb = 0 removes the only path from the bonds to the energy: energy and forces of the (separately pinned)
    two-body oracle must come back, to rounding."""
    c = _cfg(n=3)
    w = dict(c["weights"])
    w["Wb"] = np.zeros_like(w["Wb"])
    r, g = _run(c, weights=w)
    ref = om.energy_forces(c["positions"], c["cell"], c["species"], c["weights"], g, c["r_cut"], c["K"], c["p"])
    assert abs(r["energy"] - ref["energy"]) <= 1e-12 * abs(ref["energy"])
    assert np.abs(r["forces"] - ref["forces"]).max() <= 1e-12 * np.abs(ref["forces"]).max()
    # and the bond term matters when it is there
    r2, _ = _run(c)
    assert abs(r2["energy"] - ref["energy"]) > 1e-3 * abs(ref["energy"])


def test_invariances():
    c = _cfg(n=3)
    r, g = _run(c)
    fmax = np.abs(r["forces"]).max()
    # rigid translation
    r2, _ = _run(c, pos=c["positions"] + np.array([0.37, -1.2, 2.9]))
    assert abs(r2["energy"] - r["energy"]) <= 1e-11 * abs(r["energy"])
    assert np.abs(r2["forces"] - r["forces"]).max() <= 1e-9 * fmax
    # rotation of positions and cell
    q, _ = np.linalg.qr(np.random.default_rng(2).normal(size=(3, 3)))
    if np.linalg.det(q) < 0:
        q[:, 0] = -q[:, 0]
    r3, _ = _run(c, pos=c["positions"] @ q, cell=c["cell"] @ q)
    assert abs(r3["energy"] - r["energy"]) <= 1e-11 * abs(r["energy"])
    assert np.abs(r3["forces"] - r["forces"] @ q).max() <= 1e-9 * fmax
    # permutation of the atoms
    perm = np.random.default_rng(3).permutation(g.N)
    r4, _ = _run(c, pos=c["positions"][perm], species=c["species"][perm])
    assert abs(r4["energy"] - r["energy"]) <= 1e-11 * abs(r["energy"])
    assert np.abs(r4["forces"] - r["forces"][perm]).max() <= 1e-9 * fmax


def test_perfect_single_species_lattice():
    c = _cfg(n=3, sigma=0.0)
    sp = np.zeros_like(c["species"])
    r, _ = _run(c, species=sp)
    assert np.ptp(r["atom_energy"]) <= 1e-12 * abs(r["atom_energy"][0])
    assert np.abs(r["forces"]).max() <= 1e-10


def test_energy_is_smooth_where_a_bond_crosses_the_cutoff():
    """Three atoms in a large box; the third one moves along a line so that its distance to the first crosses
    r_bond.  The bond (and the triplets it takes part in) appears with an envelope that vanishes to second
    order, so energy and forces are continuous there."""
    c = _cfg(n=3)
    cell = np.eye(3) * 40.0
    sp = np.array([0, 1, 2], np.int32)
    base = np.array([[10.0, 10.0, 10.0], [12.4, 10.3, 9.8], [10.0, 10.0, 10.0]])
    direction = np.array([0.6, 0.64, 0.48])
    direction /= np.linalg.norm(direction)

    def at(dist):
        pos = base.copy()
        pos[2] = base[0] + dist * direction
        g = og.build_graph(pos, cell, c["r_cut"])
        r = tb.energy_forces3(pos, cell, sp, c["weights"], g, c["r_cut"], c["r_bond"], c["K"], c["p"])
        return r

    below, above = at(c["r_bond"] - 1e-7), at(c["r_bond"] + 1e-7)
    assert below["n_bonds"] == above["n_bonds"] + 2          # the pair (both directions) is a bond only below
    assert below["n_triplets"] > above["n_triplets"]
    scale = np.abs(below["forces"]).max()
    assert abs(below["energy"] - above["energy"]) <= 1e-6 * scale
    assert np.abs(below["forces"] - above["forces"]).max() <= 1e-5 * scale
    # away from the cutoff the bond does matter
    assert abs(at(2.5)["energy"] - at(2.5 + 1e-7)["energy"]) < 1e-5 and abs(at(2.5)["energy"] - at(3.2)["energy"]) > 1e-4


def test_fp32_mode_within_the_bf16_config_tolerance():
    c = _cfg(n=3)
    r64, _ = _run(c)
    r32, _ = _run(c, fp32=True)
    assert abs(r32["energy"] - r64["energy"]) <= 1e-5 * abs(r64["energy"])
    assert np.abs(r32["forces"] - r64["forces"]).max() <= 1e-4 * np.abs(r64["forces"]).max()


@pytest.mark.parametrize("P", [2, 3])
def test_partitioned_equals_whole(P):
    """The paper's scheme (per-layer border transfers forward, gradient add-backs in reverse) reproduces the
    unpartitioned result; bonds and triplets of an owned centre are local to its partition."""
    c = _cfg(n=4)
    r, g = _run(c)
    slab_of, _ = og.slab_assign(c["positions"], c["cell"], P)
    slabs = og.partition(g, slab_of, P)
    r2 = tb.energy_forces3_slabs(c["positions"], c["cell"], c["species"], c["weights"], g, slabs, slab_of, c["r_cut"],
                                 c["r_bond"], c["K"], c["p"])
    assert abs(r2["energy"] - r["energy"]) <= 1e-12 * abs(r["energy"])
    assert np.abs(r2["forces"] - r["forces"]).max() <= 1e-11 * np.abs(r["forces"]).max()
    assert np.abs(r2["atom_energy"] - r["atom_energy"]).max() <= 1e-12
    # thin triclinic cell: periodic images across the walls, empty rows
    pos, cell, sp = wl.random_triclinic(16, 5, scale=6.0)
    g = og.build_graph(pos, cell, c["r_cut"])
    r = tb.energy_forces3(pos, cell, sp, c["weights"], g, c["r_cut"], c["r_bond"], c["K"], c["p"])
    slab_of, _ = og.slab_assign(pos, cell, P)
    slabs = og.partition(g, slab_of, P)
    r2 = tb.energy_forces3_slabs(pos, cell, sp, c["weights"], g, slabs, slab_of, c["r_cut"], c["r_bond"], c["K"], c["p"])
    assert abs(r2["energy"] - r["energy"]) <= 1e-12 * abs(r["energy"])
    assert np.abs(r2["forces"] - r["forces"]).max() <= 1e-11 * np.abs(r["forces"]).max()
