"""Oracle: energy and forces of the radial message-passing potential.

TEST INFRASTRUCTURE ONLY.  Two independent drivers over the same per-edge C
routines (mlip_oracle.c / rmp_edge.inc) and numpy matmuls for the per-node
linear maps:

  energy_forces        whole graph, the plain definition
  energy_forces_slabs  the paper's scheme: every slab holds owned + ghost rows,
                       ghost rows are refreshed from their owners before every
                       layer's edge step ("after each graph convolution, we
                       transfer the border node ... features", Graph-Parallel
                       Message Passing) and ghost-row gradients are added back
                       to the owners in the reverse pass (Introduction:
                       intermediates are kept so that backpropagation works
                       through the transfers); energy is summed over owned
                       atoms only.

Model (benchmark configuration 0):
  h0_i = Emb[z_i]
  layer l: g = h Wm_l;  a_i = sum_{e: recv=i} (SiLU(b_e W1_l) W2_l) * g_send(e);
           h_i <- h_i + SiLU(a_i Wo_l)
  eps_i = SiLU(h_i Wr1) . wr2,   E = sum_i eps_i,   F = -dE/dr
No biases.  fp32 mode: geometry in fp64 then rounded; everything after in fp32;
total energy accumulated in fp64.
"""
from __future__ import annotations

import ctypes

import numpy as np

from . import graph as og
from ._lib import c_f32p, c_f64p, c_i32p, c_i64p, lib


def _silu(x):
    return x / (1.0 + np.exp(-x))


def _dsilu(x):
    sg = 1.0 / (1.0 + np.exp(-x))
    return sg * (1.0 + x * (1.0 - sg))


class _Edge:
    """Typed access to the per-edge C routines."""

    def __init__(self, fp32):
        self.dt = np.float32 if fp32 else np.float64
        self.fp = c_f32p if fp32 else c_f64p
        suf = "f32" if fp32 else "f64"
        L = lib()
        self._fwd = getattr(L, "orc_edge_forward_" + suf)
        self._bwd = getattr(L, "orc_edge_backward_" + suf)
        self._fsc = getattr(L, "orc_force_scatter_" + suf)

    def p(self, a):
        assert a.dtype == self.dt and a.flags.c_contiguous
        return a.ctypes.data_as(self.fp)

    def forward(self, row_ptr, senders, d, rc, K, p, W1, W2, g):
        nrows = len(row_ptr) - 1
        F = g.shape[1]
        a = np.zeros((nrows, F), self.dt)
        self._fwd(nrows, row_ptr.ctypes.data_as(c_i64p), senders.ctypes.data_as(c_i32p), self.p(d),
                  rc, K, p, F, self.p(W1), self.p(W2), self.p(g), self.p(a))
        return a

    def backward(self, row_ptr, senders, d, rc, K, p, W1, W2, g, abar, dbar):
        nrows = len(row_ptr) - 1
        nloc, F = g.shape
        gbar = np.zeros((nloc, F), self.dt)
        self._bwd(nrows, nloc, row_ptr.ctypes.data_as(c_i64p), senders.ctypes.data_as(c_i32p), self.p(d),
                  rc, K, p, F, self.p(W1), self.p(W2), self.p(g), self.p(abar), self.p(gbar), self.p(dbar))
        return gbar

    def force_scatter(self, row_ptr, senders, rhat, dbar, nloc):
        nrows = len(row_ptr) - 1
        gp = np.zeros((nloc, 3), self.dt)
        self._fsc(nrows, row_ptr.ctypes.data_as(c_i64p), senders.ctypes.data_as(c_i32p),
                  self.p(rhat), self.p(dbar), self.p(gp))
        return gp


def _cast(weights, dt):
    return {k: np.ascontiguousarray(v, dt) for k, v in weights.items()}


def energy_forces(positions, cell, species, weights, graph, r_cut, K, p, fp32=False):
    """Whole-graph energy, forces [N,3] and per-atom energies."""
    ed = _Edge(fp32)
    dt = ed.dt
    W = _cast(weights, dt)
    L = W["W1"].shape[0]
    d64, rhat64 = og.geometry(positions, cell, graph)
    d = np.ascontiguousarray(d64, dt)
    rhat = np.ascontiguousarray(rhat64, dt)
    rc = float(r_cut)
    h = W["emb"][species].copy()
    gs, as_ = [], []
    for l in range(L):
        g = np.ascontiguousarray(h @ W["Wm"][l])
        a = ed.forward(graph.row_ptr, graph.senders, d, rc, K, p, W["W1"][l], W["W2"][l], g)
        h = h + _silu(a @ W["Wo"][l])
        gs.append(g)
        as_.append(a)
    pre = h @ W["Wr1"]
    eps = _silu(pre) @ W["wr2"]
    energy = float(np.sum(eps.astype(np.float64)))
    # reverse pass
    hbar = (W["wr2"][None, :] * _dsilu(pre)) @ W["Wr1"].T
    dbar = np.zeros(graph.E, dt)
    for l in reversed(range(L)):
        q = as_[l] @ W["Wo"][l]
        abar = np.ascontiguousarray((hbar * _dsilu(q)) @ W["Wo"][l].T)
        gbar = ed.backward(graph.row_ptr, graph.senders, d, rc, K, p, W["W1"][l], W["W2"][l], gs[l], abar, dbar)
        hbar = hbar + gbar @ W["Wm"][l].T
    gradpos = ed.force_scatter(graph.row_ptr, graph.senders, rhat, dbar, graph.N)
    return dict(energy=energy, forces=-gradpos.astype(np.float64), atom_energy=eps.astype(np.float64))


def energy_forces_slabs(positions, cell, species, weights, graph, slabs, slab_of, r_cut, K, p, fp32=False):
    """Same quantities through the partitioned scheme (slabs from oracle.graph.partition)."""
    ed = _Edge(fp32)
    dt = ed.dt
    W = _cast(weights, dt)
    L = W["W1"].shape[0]
    F = W["emb"].shape[1]
    rc = float(r_cut)
    d64, rhat64 = og.geometry(positions, cell, graph)
    P = len(slabs)
    n_own = [len(s.owned) for s in slabs]
    loc = []          # per slab: d, rhat of its own edges
    local_in_owner = np.full(graph.N, -1, np.int64)
    for s in slabs:
        loc.append((np.ascontiguousarray(d64[s.edge_ids], dt), np.ascontiguousarray(rhat64[s.edge_ids], dt)))
        local_in_owner[s.nodes[: len(s.owned)]] = np.arange(len(s.owned))
    h = [W["emb"][species[s.nodes[: n_own[i]]]].copy() for i, s in enumerate(slabs)]
    gs = [[None] * P for _ in range(L)]
    as_ = [[None] * P for _ in range(L)]
    for l in range(L):
        g = []
        for i, s in enumerate(slabs):
            gi = np.zeros((len(s.nodes), F), dt)
            gi[: n_own[i]] = h[i] @ W["Wm"][l]
            g.append(gi)
        for i, s in enumerate(slabs):          # ghost rows <- owner rows
            gh = s.nodes[n_own[i]:]
            for q in range(P):
                sel = np.flatnonzero(slab_of[gh] == q)
                g[i][n_own[i] + sel] = g[q][local_in_owner[gh[sel]]]
        for i, s in enumerate(slabs):
            a = ed.forward(s.row_ptr, s.senders, loc[i][0], rc, K, p, W["W1"][l], W["W2"][l], g[i])
            h[i] = h[i] + _silu(a @ W["Wo"][l])
            gs[l][i] = g[i]
            as_[l][i] = a
    energy = 0.0
    atom_energy = np.zeros(graph.N, np.float64)
    hbar = []
    for i, s in enumerate(slabs):
        pre = h[i] @ W["Wr1"]
        eps = _silu(pre) @ W["wr2"]
        atom_energy[s.nodes[: n_own[i]]] = eps
        energy += float(np.sum(eps.astype(np.float64)))
        hbar.append((W["wr2"][None, :] * _dsilu(pre)) @ W["Wr1"].T)
    dbar = [np.zeros(len(s.edge_ids), dt) for s in slabs]
    for l in reversed(range(L)):
        gbar = []
        for i, s in enumerate(slabs):
            q = as_[l][i] @ W["Wo"][l]
            abar = np.ascontiguousarray((hbar[i] * _dsilu(q)) @ W["Wo"][l].T)
            gbar.append(ed.backward(s.row_ptr, s.senders, loc[i][0], rc, K, p, W["W1"][l], W["W2"][l],
                                    gs[l][i], abar, dbar[i]))
        for i, s in enumerate(slabs):          # ghost-row gradients -> owners
            gh = s.nodes[n_own[i]:]
            for q in range(P):             # ghost ids are distinct, so a plain indexed add is exact
                sel = np.flatnonzero(slab_of[gh] == q)
                gbar[q][local_in_owner[gh[sel]]] += gbar[i][n_own[i] + sel]
        for i in range(P):
            hbar[i] = hbar[i] + gbar[i][: n_own[i]] @ W["Wm"][l].T
    gradpos = np.zeros((graph.N, 3), np.float64)
    for i, s in enumerate(slabs):
        gp = ed.force_scatter(s.row_ptr, s.senders, loc[i][1], dbar[i], len(s.nodes))
        # owned rows and ghost rows both go back to the global atom they stand for
        np.add.at(gradpos, s.nodes, gp.astype(np.float64))
    return dict(energy=energy, forces=-gradpos, atom_energy=atom_energy)


def basis(d, r_cut, K, p):
    """(b [K], db/dd [K]) in fp64 for one distance."""
    b = np.zeros(K)
    db = np.zeros(K)
    lib().orc_basis_f64(float(d), float(r_cut), K, p, b.ctypes.data_as(c_f64p), db.ctypes.data_as(c_f64p))
    return b, db
