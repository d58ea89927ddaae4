"""Scaling sweeps on the synthetic lattices, mirroring the kind of figures the paper reports:
step time against the number of layers (interaction range), the feature width (model size), the density
(neighbours per atom), the number of slabs and the system size (Results: scaling studies).

    python -m paper_2506_02023_amd.sweeps [--which layers,width,density,slabs,size,order] [--steps 5]

`--which order` times configs[3] with the atoms numbered in lattice order and in blocks of B^3 cells (a spatially
blocked numbering keeps the sender rows an XCD gathers closer together); `--order-blocks B` restricts it to one
numbering, so that a counter run (rocprofv3 --pmc) sees one case per process.

One step = mlip_build_graph + mlip_forward (SLABS mode when more than one slab, else WHOLE), inputs resident in
HBM, as in bench.py.  Prints a markdown table per sweep.  Everything runs in the HIP library; this module only
prepares seeded inputs and times.
"""
from __future__ import annotations

import argparse
import os
import sys
import time

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))


def _time_case(pos, cell, species, weights, r_cut, p, n_slabs, steps, warmup=2):
    import torch

    import paper_2506_02023_amd as M
    pos_d = torch.as_tensor(pos, device="cuda")
    spec_d = torch.as_tensor(species, device="cuda")
    W = M.Weights(weights, p)
    N = pos_d.shape[0]
    out = (torch.empty(1, dtype=torch.float64, device="cuda"), torch.empty((N, 3), dtype=torch.float32, device="cuda"), None)
    mode = M.MODE_SLABS if n_slabs > 1 else M.MODE_WHOLE
    g = None
    for it in range(warmup + steps):
        if it == warmup:
            torch.cuda.synchronize()
            g.profile_enable(True)
            g.profile_read(reset=True)
            t0 = time.perf_counter()
        g = M.mlip_build_graph(pos_d, cell, spec_d, r_cut, n_slabs=n_slabs, graph=g)
        M.mlip_forward(g, W, mode, out=out, want_atom_energy=False)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    prof = {k: v[0] / steps for k, v in g.profile_read(reset=True).items()}
    _, E, _ = g.sizes()
    g.destroy()
    return dict(N=N, E=E, ms=dt * 1e3, prof=prof)


def _row(label, r):
    pr = r["prof"]
    return (f"| {label} | {r['N']:,} | {r['E']:,} | {r['E'] / r['N']:.1f} | {r['ms']:.2f} | {r['N'] / r['ms'] / 1e3:.2f} | "
            f"{r['E'] / r['ms'] / 1e6:.3f} | {r['ms'] * 1e3 / r['N']:.4f} | {pr['graph']:.2f} | "
            f"{pr['edge_fwd'] + pr['edge_fwd_lower'] + pr['edge_bwd'] + pr['edge_bwd_lower']:.2f} | {pr['node']:.2f} | {pr['ghost']:.2f} |")


_HEAD = ("| case | atoms | edges | edges/atom | ms/step | M atoms/s | G edges/s | us/atom | graph ms | edge ms | node ms | "
         "ghost ms |\n|---|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|---:|")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--which", default="layers,width,density,slabs,size")
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--cells", type=int, default=40, help="fcc cells per side of the fixed-size sweeps")
    ap.add_argument("--order-blocks", type=int, default=None,
                    help="with --which order: only this numbering (0 = lattice order, B = blocks of B^3 cells)")
    args = ap.parse_args()
    which = set(args.which.split(","))

    import workloads as wl
    seed = wl.BASE_SEED + 3
    n = args.cells

    def lattice(cells, a=wl.A_LAT, sigma=0.15):
        return wl.fcc_lattice(cells, sigma, 8, seed, a=a)

    if "layers" in which:
        print(f"\n### Layers (interaction range), fcc {n}^3, F = 64, 8 slabs\n\n" + _HEAD)
        pos, cell, sp = lattice(n)
        for L in (1, 2, 3, 4, 6):
            print(_row(f"L = {L}", _time_case(pos, cell, sp, wl.rmp_weights(8, 64, L, seed), wl.R_CUT, wl.P_ENVELOPE, 8, args.steps)),
                  flush=True)
    if "width" in which:
        print(f"\n### Feature width (model size), fcc {n}^3, L = 3, 8 slabs\n\n" + _HEAD)
        pos, cell, sp = lattice(n)
        for F in (32, 64):
            print(_row(f"F = {F}", _time_case(pos, cell, sp, wl.rmp_weights(8, F, 3, seed), wl.R_CUT, wl.P_ENVELOPE, 8, args.steps)),
                  flush=True)
    if "density" in which:
        print(f"\n### Density (lattice constant at fixed r_cut = 5.0), fcc {n}^3, F = 64, L = 3, 8 slabs\n\n" + _HEAD)
        for a in (4.4, 4.0, 3.6, 3.3, 3.0):
            pos, cell, sp = lattice(n, a=a, sigma=0.15 * a / wl.A_LAT)
            print(_row(f"a = {a}", _time_case(pos, cell, sp, wl.rmp_weights(8, 64, 3, seed), wl.R_CUT, wl.P_ENVELOPE, 8, args.steps)),
                  flush=True)
    if "slabs" in which:
        print("\n### Number of slabs, configs[3] (fcc 63^3), F = 64, L = 3\n\n" + _HEAD)
        pos, cell, sp = lattice(63)
        for P in (1, 2, 4, 8, 16, 32):
            print(_row(f"P = {P}", _time_case(pos, cell, sp, wl.rmp_weights(8, 64, 3, seed), wl.R_CUT, wl.P_ENVELOPE, P, args.steps)),
                  flush=True)
    if "order" in which:
        import numpy as np
        print("\n### Atom numbering, configs[3] (fcc 63^3), F = 64, L = 3, 8 slabs\n\n" + _HEAD)
        pos, cell, sp = lattice(63)
        idx = np.arange(len(sp))
        ix, iy, iz, b = np.unravel_index(idx, (63, 63, 63, 4))
        for B in ([args.order_blocks] if args.order_blocks is not None else [0, 4, 8, 16]):
            if B:
                key = ((((ix // B) * 100 + (iy // B)) * 100 + (iz // B)) * B + ix % B) * B * B * 4 + ((iy % B) * B + iz % B) * 4 + b
                perm = np.argsort(key, kind="stable")
            else:
                perm = idx
            r = _time_case(np.ascontiguousarray(pos[perm]), cell, np.ascontiguousarray(sp[perm]),
                           wl.rmp_weights(8, 64, 3, seed), wl.R_CUT, wl.P_ENVELOPE, 8, args.steps)
            print(_row("lattice order" if not B else f"blocks of {B}^3 cells", r) +
                  f" edge fwd {r['prof']['edge_fwd'] + r['prof']['edge_fwd_lower']:.2f} / bwd {r['prof']['edge_bwd'] + r['prof']['edge_bwd_lower']:.2f} ms", flush=True)
    if "size" in which:
        print("\n### System size, F = 64, L = 3, 8 slabs\n\n" + _HEAD)
        for cells in (10, 20, 30, 40, 50, 63, 80):
            pos, cell, sp = lattice(cells)
            print(_row(f"fcc {cells}^3", _time_case(pos, cell, sp, wl.rmp_weights(8, 64, 3, seed), wl.R_CUT, wl.P_ENVELOPE, 8,
                                                   args.steps)), flush=True)


if __name__ == "__main__":
    main()
