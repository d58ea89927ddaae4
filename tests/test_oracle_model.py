"""Pins for the oracle's model arithmetic: basis, forward energy, forces, partitioned mode (CPU only)."""
import math

import numpy as np
import pytest

import workloads as wl
from oracle import graph as og
from oracle import model as om

RC, K, P_ENV = 5.0, 8, 6


def _run(c, pos=None, cell=None, species=None, weights=None, fp32=False):
    pos = c["positions"] if pos is None else pos
    cell = c["cell"] if cell is None else cell
    species = c["species"] if species is None else species
    weights = c["weights"] if weights is None else weights
    g = og.build_graph(pos, cell, c["r_cut"])
    return om.energy_forces(pos, cell, species, weights, g, c["r_cut"], c["K"], c["p"], fp32=fp32)


@pytest.fixture(scope="module")
def cfg0():
    return wl.make_config(0)


# ------------------------------------------------------------------ basis and envelope

def test_envelope_limits():
    """u(0) = 1 and u, u', u'' vanish at x = 1 (p = 6: u = 1 - 28 x^6 + 48 x^7 - 21 x^8)."""
    def u(x):  # recovered from b_1: u = b_1 d / sin(pi x)
        d = x * RC
        b, _ = om.basis(d, RC, K, P_ENV)
        return b[0] * d / math.sin(math.pi * x)
    for x in (0.1, 0.37, 0.8, 0.95):
        assert abs(u(x) - (1 - 28 * x**6 + 48 * x**7 - 21 * x**8)) < 1e-12
    assert abs(u(1e-6) - 1.0) < 1e-12
    h = 1e-3
    # u ~ c (1-x)^3 near 1  ->  u(1-h)/h^3 stays bounded, second difference ~ h
    assert abs(u(1 - h)) < 100 * h**3
    assert abs(u(1 - 2 * h) - 2 * u(1 - h)) < 1e3 * h**3


def test_basis_limits_and_cutoff():
    b, db = om.basis(1e-7, RC, K, P_ENV)
    for n in range(1, K + 1):
        assert abs(b[n - 1] - n * math.pi / RC) < 1e-9          # sin(n pi d/rc)/d -> n pi / rc
    b, db = om.basis(RC, RC, K, P_ENV)
    assert np.all(np.abs(b) < 1e-14) and np.all(np.abs(db) < 1e-13)


def test_bare_basis_orthogonality():
    """int_0^rc [sin(n pi d/rc)/d][sin(m pi d/rc)/d] d^2 dd = rc/2 delta_nm; the bare functions
    are recovered by dividing out the envelope."""
    n_q = 4000
    x = (np.arange(n_q) + 0.5) / n_q
    d = x * RC
    u = 1 - 28 * x**6 + 48 * x**7 - 21 * x**8
    B = np.array([om.basis(di, RC, K, P_ENV)[0] for di in d]) / u[:, None]
    gram = (B[:, :, None] * B[:, None, :] * (d**2)[:, None, None]).sum(0) * (RC / n_q)
    assert np.allclose(gram, np.eye(K) * RC / 2, atol=1e-5)


def test_basis_derivative():
    for d in (0.7, 2.3, 3.9, 4.8):
        h = 1e-5
        _, db = om.basis(d, RC, K, P_ENV)
        fd = (om.basis(d + h, RC, K, P_ENV)[0] - om.basis(d - h, RC, K, P_ENV)[0]) / (2 * h)
        assert np.allclose(db, fd, rtol=1e-7, atol=1e-8)


# ------------------------------------------------------------------ forward energy

def _scalar_model(pos, species, W, r_cut, Kn, p):
    """The model of benchmark configuration 0 for a free cluster, written per atom with Python
    floats and math.* only (no shared code, different loop structure: gathers per receiver from a
    dense distance table, recursion over layers)."""
    n = len(pos)
    F = W["emb"].shape[1]
    L = W["W1"].shape[0]
    silu = lambda v: v / (1.0 + math.exp(-v))
    dist = [[math.dist(pos[i], pos[j]) for j in range(n)] for i in range(n)]

    def filt(l, d):
        x = d / r_cut
        u = 1 - (p + 1) * (p + 2) / 2 * x**p + p * (p + 2) * x**(p + 1) - p * (p + 1) / 2 * x**(p + 2)
        b = [math.sin(m * math.pi * x) / d * u for m in range(1, Kn + 1)]
        s = [silu(sum(b[m] * float(W["W1"][l, m, f]) for m in range(Kn))) for f in range(F)]
        return [sum(s[k] * float(W["W2"][l, k, f]) for k in range(F)) for f in range(F)]

    h = [[float(W["emb"][species[i], f]) for f in range(F)] for i in range(n)]
    for l in range(L):
        g = [[sum(h[i][k] * float(W["Wm"][l, k, f]) for k in range(F)) for f in range(F)] for i in range(n)]
        new_h = []
        for i in range(n):
            a = [0.0] * F
            for j in range(n):
                if j != i and dist[i][j] <= r_cut:
                    w = filt(l, dist[i][j])
                    a = [a[f] + w[f] * g[j][f] for f in range(F)]
            q = [sum(a[k] * float(W["Wo"][l, k, f]) for k in range(F)) for f in range(F)]
            new_h.append([h[i][f] + silu(q[f]) for f in range(F)])
        h = new_h
    eps = []
    for i in range(n):
        pre = [sum(h[i][k] * float(W["Wr1"][k, f]) for k in range(F)) for f in range(F)]
        eps.append(sum(silu(pre[f]) * float(W["wr2"][f]) for f in range(F)))
    return eps


def test_forward_against_scalar_python_cluster():
    """Small free cluster in a huge box (no periodic images in range), asymmetric tiny weights."""
    rng = np.random.default_rng(11)
    n, F, L, S, Kn = 7, 5, 2, 3, 4
    pos = rng.random((n, 3)) * 4.0 + 20.0
    species = rng.integers(0, S, n).astype(np.int32)
    W = wl.rmp_weights(S, F, L, seed=5, K=Kn)
    cell = np.eye(3) * 60.0
    g = og.build_graph(pos, cell, 3.0)
    assert g.E > 10
    r = om.energy_forces(pos, cell, species, W, g, 3.0, Kn, 6)
    eps = _scalar_model(pos.tolist(), species.tolist(), W, 3.0, Kn, 6)
    assert np.allclose(r["atom_energy"], eps, rtol=1e-12, atol=1e-13)
    assert abs(r["energy"] - sum(eps)) < 1e-12


def test_zero_layers_closed_form(cfg0):
    """L = 0: E = sum_s count_s * eps(Emb[s]) and all forces vanish."""
    W = {k: (v[:0] if k in ("W1", "W2", "Wm", "Wo") else v) for k, v in cfg0["weights"].items()}
    r = _run(cfg0, weights=W)
    emb = W["emb"].astype(np.float64)
    pre = emb @ W["Wr1"].astype(np.float64)
    eps_s = (pre / (1 + np.exp(-pre))) @ W["wr2"].astype(np.float64)
    want = sum(eps_s[s] for s in cfg0["species"])
    assert abs(r["energy"] - want) < 1e-10
    assert np.all(r["forces"] == 0)


def test_zero_filter_output_gives_same_closed_form(cfg0):
    """W2 = 0 -> messages vanish -> h stays the embedding (SiLU(0) = 0)."""
    W = dict(cfg0["weights"])
    W["W2"] = np.zeros_like(W["W2"])
    r = _run(cfg0, weights=W)
    W0 = {k: (v[:0] if k in ("W1", "W2", "Wm", "Wo") else v) for k, v in cfg0["weights"].items()}
    assert abs(r["energy"] - _run(cfg0, weights=W0)["energy"]) < 1e-10
    assert np.abs(r["forces"]).max() == 0


def test_dimer(cfg0):
    """Two atoms in a 40 A box: E depends on d only, is constant beyond r_cut, and the force is
    -dE/dd along the bond (checked with a numerical derivative of E(d))."""
    W = cfg0["weights"]
    cell = np.eye(3) * 40.0
    sp = np.array([0, 1], np.int32)
    axis = np.array([1.0, 2.0, -0.5]); axis /= np.linalg.norm(axis)

    def E(d):
        pos = np.array([[10.0, 10, 10], [10.0, 10, 10] + axis * d])
        g = og.build_graph(pos, cell, RC)
        return om.energy_forces(pos, cell, sp, W, g, RC, K, P_ENV)
    far = E(5.5)["energy"]
    assert E(7.0)["energy"] == far and np.all(E(6.0)["forces"] == 0)
    assert abs(E(4.9999999)["energy"] - far) < 1e-12      # C^2 approach to the cutoff
    d, h = 2.7, 1e-5
    r = E(d)
    dEdd = (E(d + h)["energy"] - E(d - h)["energy"]) / (2 * h)
    assert np.allclose(r["forces"][1], -dEdd * axis, rtol=1e-7, atol=1e-9)
    assert np.allclose(r["forces"][0], +dEdd * axis, rtol=1e-7, atol=1e-9)


def test_ideal_lattice_identical_atoms():
    """Un-jittered single-species lattice: identical per-atom energies, zero forces."""
    pos, cell, sp = wl.fcc_lattice(3, 0.0, 1, seed=2)
    W = wl.rmp_weights(1, 16, 2, seed=2)
    g = og.build_graph(pos, cell, RC)
    r = om.energy_forces(pos, cell, sp, W, g, RC, K, P_ENV)
    assert np.ptp(r["atom_energy"]) < 1e-12 * max(1.0, abs(r["atom_energy"][0]))
    assert np.abs(r["forces"]).max() < 1e-11


def test_supercell_replication(cfg0):
    """Tiling the jittered box 2x1x1 doubles the energy and replicates the forces."""
    r1 = _run(cfg0)
    pos, cell = cfg0["positions"], cfg0["cell"]
    pos2 = np.concatenate([pos, pos + cell[0]])
    cell2 = cell.copy(); cell2[0] *= 2
    sp2 = np.concatenate([cfg0["species"], cfg0["species"]])
    r2 = _run(cfg0, pos=pos2, cell=cell2, species=sp2)
    assert abs(r2["energy"] - 2 * r1["energy"]) < 1e-10 * abs(r1["energy"])
    assert np.allclose(r2["forces"][: len(pos)], r1["forces"], atol=1e-11)
    assert np.allclose(r2["forces"][len(pos):], r1["forces"], atol=1e-11)


# ------------------------------------------------------------------ forces

def test_forces_finite_differences(cfg0):
    r = _run(cfg0)
    pos = cfg0["positions"]
    h = 1e-4
    rng = np.random.default_rng(0)
    for i, k in zip(rng.integers(0, len(pos), 6), rng.integers(0, 3, 6)):
        pp = pos.copy(); pp[i, k] += h
        pm = pos.copy(); pm[i, k] -= h
        fd = -(_run(cfg0, pos=pp)["energy"] - _run(cfg0, pos=pm)["energy"]) / (2 * h)
        assert abs(fd - r["forces"][i, k]) < 2e-7 * max(1.0, np.abs(r["forces"]).max())


def test_forces_finite_differences_triclinic_small_cell():
    """Cell thinner than 2 r_cut (an atom sees several images of a neighbour and of itself)."""
    pos, cell, sp = wl.random_triclinic(10, 3, scale=4.5)
    W = wl.rmp_weights(4, 8, 2, seed=9)
    c = dict(positions=pos, cell=cell, species=sp, weights=W, r_cut=3.5, K=K, p=P_ENV)
    r = _run(c)
    h = 1e-4
    for i, k in [(0, 0), (3, 1), (9, 2)]:
        pp = pos.copy(); pp[i, k] += h
        pm = pos.copy(); pm[i, k] -= h
        fd = -(_run(c, pos=pp)["energy"] - _run(c, pos=pm)["energy"]) / (2 * h)
        assert abs(fd - r["forces"][i, k]) < 1e-6 * max(1.0, np.abs(r["forces"]).max())


def test_net_force_and_invariances(cfg0):
    r = _run(cfg0)
    fmax = np.abs(r["forces"]).max()
    assert np.abs(r["forces"].sum(0)).max() < 1e-12 * fmax * len(r["forces"])
    # rigid translation
    rt = _run(cfg0, pos=cfg0["positions"] + np.array([0.37, -1.2, 5.5]))
    assert abs(rt["energy"] - r["energy"]) < 1e-11 * abs(r["energy"])
    assert np.allclose(rt["forces"], r["forces"], atol=1e-11 * fmax)
    # rotation of positions and cell together
    a, b = 0.7, -0.4
    Rz = np.array([[math.cos(a), -math.sin(a), 0], [math.sin(a), math.cos(a), 0], [0, 0, 1]])
    Rx = np.array([[1, 0, 0], [0, math.cos(b), -math.sin(b)], [0, math.sin(b), math.cos(b)]])
    R = Rz @ Rx
    rr = _run(cfg0, pos=cfg0["positions"] @ R.T, cell=cfg0["cell"] @ R.T)
    assert abs(rr["energy"] - r["energy"]) < 1e-10 * abs(r["energy"])
    assert np.allclose(rr["forces"], r["forces"] @ R.T, atol=1e-9 * fmax)
    # permutation of atoms
    perm = np.random.default_rng(4).permutation(len(cfg0["species"]))
    rp = _run(cfg0, pos=cfg0["positions"][perm], species=cfg0["species"][perm])
    assert abs(rp["energy"] - r["energy"]) < 1e-11 * abs(r["energy"])
    assert np.allclose(rp["forces"], r["forces"][perm], atol=1e-11 * fmax)


# ------------------------------------------------------------------ partitioned scheme, fp32 mode

@pytest.mark.parametrize("P", [1, 2, 3, 8])
def test_partitioned_equals_whole(cfg0, P):
    c = cfg0
    g = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    whole = om.energy_forces(c["positions"], c["cell"], c["species"], c["weights"], g, c["r_cut"], c["K"], c["p"])
    slab_of, _ = og.slab_assign(c["positions"], c["cell"], P)
    slabs = og.partition(g, slab_of, P)
    part = om.energy_forces_slabs(c["positions"], c["cell"], c["species"], c["weights"], g, slabs, slab_of,
                                  c["r_cut"], c["K"], c["p"])
    assert abs(part["energy"] - whole["energy"]) < 1e-11 * abs(whole["energy"])
    assert np.allclose(part["forces"], whole["forces"], atol=1e-11 * np.abs(whole["forces"]).max())
    assert np.allclose(part["atom_energy"], whole["atom_energy"], atol=1e-12)


def test_fp32_mode_within_tolerance(cfg0):
    """The stated fp32 tolerances (1e-5 relative energy, 1e-4 max|F| per component) are attainable."""
    r64 = _run(cfg0)
    r32 = _run(cfg0, fp32=True)
    assert abs(r32["energy"] - r64["energy"]) <= 1e-5 * abs(r64["energy"])
    assert np.abs(r32["forces"] - r64["forces"]).max() <= 1e-4 * np.abs(r64["forces"]).max()
    assert abs(r64["energy"]) > 0.01 * np.abs(r64["atom_energy"]).sum()      # E is not a near-cancellation
