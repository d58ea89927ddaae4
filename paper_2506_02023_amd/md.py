"""A few steps of constant-energy molecular dynamics on the synthetic lattice, the graph rebuilt at every step
as in the paper's runs (Results: the graph is re-created each step because atoms move).

    python -m paper_2506_02023_amd.md [--cells 63] [--slabs 8] [--steps 50] [--dt 0.004] [--three-body] [--skin 0.5]

Energies and forces come from the HIP library (mlip_build_graph + mlip_forward per step); the velocity-Verlet update
is three lines of torch arithmetic on the positions and velocities (unit masses, the model's own energy unit).
Prints the time per MD step and how well E_pot + E_kin is conserved, which holds only if the forces are the
gradient of the energy along the trajectory.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--cells", type=int, default=63, help="fcc cells per side (63: the 1,000,188-atom benchmark system)")
    ap.add_argument("--slabs", type=int, default=8)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--dt", type=float, default=0.004)
    ap.add_argument("--skin", type=float, default=0.0,
                    help="Verlet skin in Angstrom: the neighbour list is filtered from a candidate list for r_cut + skin that "
                         "is rebuilt when an atom has moved skin / 2 (0: search at every step)")
    ap.add_argument("--three-body", action="store_true", help="the three-body variant (benchmark configuration 4's model)")
    args = ap.parse_args()

    import numpy as np
    import torch

    import paper_2506_02023_amd as M
    import workloads as wl

    c = wl.make_config(4 if args.three_body else 3, n=args.cells)
    w = c["weights"]
    W = M.Weights(w, c["p"])
    BW = M.BondWeights(w, c["r_bond"], c["A"]) if args.three_body else None
    pos = torch.as_tensor(c["positions"], device="cuda")
    spec = torch.as_tensor(c["species"], device="cuda")
    N = pos.shape[0]
    vel = np.random.default_rng(0).normal(0.0, 0.05, (N, 3))
    vel = torch.as_tensor(vel - vel.mean(0), device="cuda")
    mode = M.MODE_SLABS if args.slabs > 1 else M.MODE_WHOLE
    out = (torch.empty(1, dtype=torch.float64, device="cuda"), torch.empty((N, 3), dtype=torch.float32, device="cuda"), None)
    g = None
    if args.skin > 0:
        g = M.Graph()
        g.set_skin(args.skin)

    def energy_forces():
        nonlocal g
        g = M.mlip_build_graph(pos, c["cell"], spec, c["r_cut"], n_slabs=args.slabs, graph=g)
        if args.three_body:
            M.mlip_forward_bonds(g, W, BW, mode, out=out, want_atom_energy=False)
        else:
            M.mlip_forward(g, W, mode, out=out, want_atom_energy=False)
        return out[0], out[1]

    def total(e):
        return float(e.cpu()[0]) + 0.5 * float((vel ** 2).sum())

    e, f = energy_forces()
    e_first, total_first = float(e.cpu()[0]), total(e)
    pots, totals = [e_first], [total_first]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        vel += (0.5 * args.dt) * f
        pos += args.dt * vel
        e, f = energy_forces()
        vel += (0.5 * args.dt) * f
        pots.append(e.clone())        # read back after the loop: no host synchronisation inside an MD step
        totals.append(0.5 * (vel ** 2).sum())
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / max(args.steps, 1)
    pots = [pots[0]] + [float(p.cpu()[0]) for p in pots[1:]]
    totals = [totals[0]] + [p + float(k.cpu()) for p, k in zip(pots[1:], totals[1:])]
    _, E, _ = g.sizes()
    swing = float(np.ptp(pots))
    drift = float(np.abs(np.array(totals) - total_first).max())
    print(f"{N} atoms, {E} directed edges, {args.slabs} slab(s), {'three-body' if args.three_body else 'two-body'} model")
    print(f"{args.steps} velocity-Verlet steps of dt = {args.dt}: {dt * 1e3:.2f} ms per step "
          f"({N / dt / 1e6:.2f} M atom-steps/s), graph rebuilt every step")
    if args.skin > 0:
        builds, reuses = g.skin_stats()
        print(f"Verlet skin {args.skin}: candidate list built {builds} times, reused {reuses} times")
    print(f"potential energy moved by {swing:.4f}, E_pot + E_kin drifted by at most {drift:.3e} "
          f"({drift / swing:.1e} of the swing)" if swing > 0 else "no motion")


if __name__ == "__main__":
    main()
