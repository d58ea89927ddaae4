"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This module only draws random numbers and lays out arrays.  It holds none of
the method's arithmetic (no distances, no basis functions, no partition rule),
so the oracle and the GPU library can both be fed from it without sharing any
code of the method itself.

The structures are jittered fcc lattices (a = 3.6 A, four atoms per cubic
cell) under full periodic boundary conditions; they stand in for the crystal
supercells the paper times (Results section, "alpha-quartz SiO2 supercells"),
which are not available offline.  Atom order is lattice order:
index = ((ix * n + iy) * n + iz) * 4 + basis.
"""
from __future__ import annotations

import numpy as np

A_LAT = 3.6
R_CUT = 5.0
R_BOND = 3.0      # bond-graph cutoff of the three-body configuration
A_ANGLE = 8       # angle basis size of the three-body configuration
K_RADIAL = 8
P_ENVELOPE = 6
BASE_SEED = 2506020230

# n = fcc cells per side, sigma = per-component Gaussian jitter (Angstrom),
# S = species, F = feature width, L = layers, P = slabs of the partitioned run
CONFIGS = {
    0: dict(n=3, sigma=0.10, S=4, F=32, L=2, P=1),
    1: dict(n=20, sigma=0.10, S=4, F=64, L=3, P=1),
    2: dict(n=30, sigma=0.10, S=4, F=64, L=3, P=8),
    3: dict(n=63, sigma=0.15, S=8, F=64, L=3, P=8),
    4: dict(n=37, sigma=0.10, S=4, F=64, L=3, P=1, three_body=True),
}

_FCC_BASIS = np.array(
    [[0.0, 0.0, 0.0], [0.0, 0.5, 0.5], [0.5, 0.0, 0.5], [0.5, 0.5, 0.0]]
)


def fcc_lattice(n, sigma, n_species, seed, a=A_LAT):
    """Return (positions [N,3] f64, cell [3,3] f64 rows = lattice vectors, species [N] i32).

    Positions are lattice sites plus N(0, sigma^2) per Cartesian component and
    are NOT wrapped back into the cell.
    """
    ss = np.random.SeedSequence(seed)
    s_pos, s_spec = ss.spawn(2)
    idx = np.arange(n, dtype=np.float64)
    gx, gy, gz = np.meshgrid(idx, idx, idx, indexing="ij")
    corners = np.stack([gx.ravel(), gy.ravel(), gz.ravel()], axis=1)
    sites = (corners[:, None, :] + _FCC_BASIS[None, :, :]).reshape(-1, 3) * a
    n_atoms = sites.shape[0]
    if sigma > 0.0:
        jitter = np.random.default_rng(s_pos).normal(0.0, sigma, size=(n_atoms, 3))
        positions = sites + jitter
    else:
        positions = sites.copy()
    species = np.random.default_rng(s_spec).integers(
        0, n_species, size=n_atoms, dtype=np.int32
    )
    cell = np.eye(3, dtype=np.float64) * (n * a)
    return np.ascontiguousarray(positions), cell, np.ascontiguousarray(species)


def rmp_weights(n_species, F, L, seed, K=K_RADIAL):
    """Random fp32 weights of the radial message-passing potential.

    All linear maps are stored row-major as [fan_in, fan_out] (y = x @ W) and
    drawn from N(0, 1/fan_in) (variance); the embedding is N(0, 1).  No biases.
    Keys: emb [S,F]; W1 [L,K,F]; W2 [L,F,F]; Wm [L,F,F]; Wo [L,F,F];
    Wr1 [F,F]; wr2 [F].
    """
    rng = np.random.default_rng(np.random.SeedSequence(seed).spawn(3)[2])

    def lin(*shape, fan_in):
        return (rng.normal(0.0, 1.0, size=shape) / np.sqrt(fan_in)).astype(np.float32)

    return dict(
        emb=rng.normal(0.0, 1.0, size=(n_species, F)).astype(np.float32),
        W1=lin(L, K, F, fan_in=K),
        W2=lin(L, F, F, fan_in=F),
        Wm=lin(L, F, F, fan_in=F),
        Wo=lin(L, F, F, fan_in=F),
        Wr1=lin(F, F, fan_in=F),
        wr2=lin(F, fan_in=F),
    )


def three_body_weights(F, L, seed, K=K_RADIAL, A=A_ANGLE):
    """Extra fp32 weights of the three-body variant (bond width Fb = F), same conventions as rmp_weights.

    Keys: We0 [K,F] bond embedding; Wt1 [2F+A,F], Wt2 [F,F] triplet MLP; Wb [L,F,F] bond term of each
    layer's filter.
    """
    rng = np.random.default_rng(np.random.SeedSequence(seed).spawn(4)[3])

    def lin(*shape, fan_in):
        return (rng.normal(0.0, 1.0, size=shape) / np.sqrt(fan_in)).astype(np.float32)

    return dict(We0=lin(K, F, fan_in=K), Wt1=lin(2 * F + A, F, fan_in=2 * F + A), Wt2=lin(F, F, fan_in=F),
                Wb=lin(L, F, F, fan_in=F))


def make_config(index, n=None, seed=None):
    """Inputs of benchmark configuration `index` (0..4).

    `n` overrides the number of fcc cells per side (used for bounded samples of
    the same workload); everything else keeps the configuration's recipe.
    Returns a dict with positions, cell, species, weights and the scalars
    r_cut, K, p, F, L, S, n_slabs.
    """
    cfg = dict(CONFIGS[index])
    if n is not None:
        cfg["n"] = n
    seed = BASE_SEED + index if seed is None else seed
    positions, cell, species = fcc_lattice(cfg["n"], cfg["sigma"], cfg["S"], seed)
    weights = rmp_weights(cfg["S"], cfg["F"], cfg["L"], seed)
    if cfg.get("three_body"):
        weights.update(three_body_weights(cfg["F"], cfg["L"], seed))
    return dict(
        positions=positions, cell=cell, species=species, weights=weights,
        r_cut=R_CUT, K=K_RADIAL, p=P_ENVELOPE, F=cfg["F"], L=cfg["L"], S=cfg["S"],
        n_slabs=cfg["P"], name=f"configs[{index}] fcc {cfg['n']}^3",
        three_body=bool(cfg.get("three_body")), r_bond=R_BOND, A=A_ANGLE,
    )


def random_triclinic(n_atoms, seed, scale=6.0, skew=0.3, spread=1.5):
    """A small random triclinic cell with atoms scattered in and slightly around it."""
    rng = np.random.default_rng(seed)
    cell = np.eye(3) * scale * (0.7 + 0.6 * rng.random(3))
    cell += skew * scale * (rng.random((3, 3)) - 0.5) * (1 - np.eye(3))
    frac = (rng.random((n_atoms, 3)) - 0.5) * spread + 0.5
    positions = frac @ cell
    species = rng.integers(0, 4, size=n_atoms, dtype=np.int32)
    return np.ascontiguousarray(positions), np.ascontiguousarray(cell), species
