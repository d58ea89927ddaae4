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
