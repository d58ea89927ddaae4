"""A short constant-energy trajectory on the GPU path, the graph rebuilt at every step as the paper's
molecular-dynamics runs do (Results: the graph is re-created each step).  Forces that are the exact gradient of
the energy conserve E_pot + E_kin under velocity Verlet up to O(dt^2); an inconsistency between the forward and
the hand-written reverse pass (or between partitions) shows up as a drift.  The integrator is three lines of
torch arithmetic in this test; energies and forces come from the library.
"""
import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_slabs,three_body", [(1, False), (3, False), (2, True)])
def test_energy_is_conserved_along_a_trajectory(n_slabs, three_body):
    import torch
    import paper_2506_02023_amd as M
    c = wl.make_config(4 if three_body else 0, n=3)
    w = c["weights"]
    W = M.Weights({k: w[k] for k in ("emb", "W1", "W2", "Wm", "Wo", "Wr1", "wr2")}, c["p"])
    BW = M.BondWeights(w, c["r_bond"], c["A"]) if three_body else None
    pos = torch.as_tensor(c["positions"], device="cuda")
    spec = torch.as_tensor(c["species"], device="cuda")
    rng = np.random.default_rng(0)
    vel = rng.normal(0.0, 0.05, pos.shape)
    vel = torch.as_tensor(vel - vel.mean(0), device="cuda")
    mode = M.MODE_SLABS if n_slabs > 1 else M.MODE_WHOLE
    g = None

    def energy_forces():
        nonlocal g
        g = M.mlip_build_graph(pos, c["cell"], spec, c["r_cut"], n_slabs=n_slabs, graph=g)
        if three_body:
            e, f, _ = M.mlip_forward_bonds(g, W, BW, mode)
        else:
            e, f, _ = M.mlip_forward(g, W, mode)
        return float(e.cpu()[0]), f.double()

    dt = 0.004
    e, f = energy_forces()
    total0 = e + 0.5 * float((vel ** 2).sum())
    totals, pots = [], []
    for _ in range(40):
        vel += 0.5 * dt * f
        pos += dt * vel
        e, f = energy_forces()
        vel += 0.5 * dt * f
        totals.append(e + 0.5 * float((vel ** 2).sum()))
        pots.append(e)
    drift = np.abs(np.array(totals) - total0).max()
    swing = np.ptp(pots)
    print(f"{n_slabs} slab(s), three_body={three_body}: potential energy moved by {swing:.3f}, total drifted by {drift:.2e}")
    assert swing > 0.1                      # the trajectory exchanges a visible amount of energy
    # measured 8e-6 (two-body) and 7e-5 (three-body, larger forces at the same time step) of the swing
    assert drift <= (5e-4 if three_body else 1e-4) * swing


@pytest.mark.parametrize("n_slabs", [1, 3])
def test_verlet_skin_graph_is_bit_identical_to_a_fresh_build(n_slabs):
    """Atoms drift for 60 steps; one handle rebuilds its graph at every step from a candidate list with a 0.1 A skin
    (rebuilt whenever an atom has moved more than 0.05 A since the list was made), another handle searches afresh.
    Neighbour list, lengths, reverse-edge index, slab assignment, index sets, energy and forces must agree bit for
    bit at every step, across several list rebuilds; the first and last graphs are also compared with the oracle."""
    import torch
    import paper_2506_02023_amd as M
    from oracle import graph as og
    from gpu_util import assert_graph_equal
    c = wl.make_config(1, n=6)      # 864 atoms, F = 64, L = 3
    W = M.Weights(c["weights"], c["p"])
    pos = torch.as_tensor(c["positions"], device="cuda")
    spec = torch.as_tensor(c["species"], device="cuda")
    vel = torch.as_tensor(np.random.default_rng(5).normal(0.0, 0.5, pos.shape), device="cuda")
    mode = M.MODE_SLABS if n_slabs > 1 else M.MODE_WHOLE
    gs = M.Graph()
    gs.set_skin(0.1)
    gf = None
    for step in range(60):
        gs = M.mlip_build_graph(pos, c["cell"], spec, c["r_cut"], n_slabs=n_slabs, graph=gs)
        gf = M.mlip_build_graph(pos, c["cell"], spec, c["r_cut"], n_slabs=n_slabs, graph=gf)
        assert gs.sizes() == gf.sizes(), step
        for a, b in zip(gs.csr(), gf.csr()):
            assert np.array_equal(a, b), step
        assert np.array_equal(gs.mirror(), gf.mirror()), step
        assert np.array_equal(gs.slab_of()[0], gf.slab_of()[0]), step
        for p in range(n_slabs if n_slabs > 1 else 0):
            sa, sb = gs.slab(p), gf.slab(p)
            for k in ("nodes", "markers", "row_ptr", "senders", "owned_sorted"):
                assert np.array_equal(sa[k], sb[k]), (step, p, k)
        ra, rb = M.mlip_forward(gs, W, mode), M.mlip_forward(gf, W, mode)
        torch.cuda.synchronize()
        assert float(ra[0].cpu()[0]) == float(rb[0].cpu()[0]), step
        assert torch.equal(ra[1], rb[1]), step
        if step in (0, 59):
            p_now = pos.cpu().numpy()
            assert_graph_equal(gs, og.build_graph(p_now, c["cell"], c["r_cut"]), p_now, c["cell"])
        pos += 0.01 * vel
    builds, reuses = gs.skin_stats()
    print(f"{n_slabs} slab(s): candidate list built {builds} times, reused {reuses} times over 60 steps")
    assert builds >= 3 and reuses >= 40 and builds + reuses == 60
    # a change of the cell, of the atom count or of the cutoff is noticed without being told
    g2 = M.mlip_build_graph(pos[:800].contiguous(), c["cell"], spec[:800].contiguous(), c["r_cut"], n_slabs=n_slabs, graph=gs)
    gf2 = M.mlip_build_graph(pos[:800].contiguous(), c["cell"], spec[:800].contiguous(), c["r_cut"], n_slabs=n_slabs)
    for a, b in zip(g2.csr(), gf2.csr()):
        assert np.array_equal(a, b)
    assert g2.skin_stats()[0] == builds + 1
