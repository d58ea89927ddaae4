"""Oracle: the three-body (bond graph) variant of the radial message-passing potential.

TEST INFRASTRUCTURE ONLY.  Benchmark configuration 4 sketches the model; the paper's counterpart is the
bond (line) graph built over the atom graph (Methods, "Distributing Bond Graphs"; Fig. 1 b-d): its nodes
are the atom-graph edges within a second, smaller cutoff, and two bonds interact when they share their
centre atom.  The reading taken here (each point is a choice the sketch leaves open):

  bonds      the atom-graph edges (i <- j, S) with d <= r_bond, same fp64 predicate as the atom graph,
             numbered in edge order (so the bonds of one centre are contiguous);
  triplets   every ordered pair (b1, b2) of distinct bonds with the same centre i;
  e0_b       = bbond(d_b) We0, the Bessel basis with the polynomial envelope at r_bond, width F_b = F;
  angle      c = rhat_b1 . rhat_b2,  T_n(c) = cos(n theta) for n = 0..A-1 (Chebyshev recurrence), A = 8;
  update     h = [e0_b1, e0_b2, T(c)] Wt1,  S_b1 = sum_{b2 != b1} u_b2 SiLU(h),  m_b1 = S_b1 Wt2,
             e1_b1 = e0_b1 + u_b1 SiLU(m_b1)
             (the sketch's "e_ij += SiLU(sum_k MLP([e_ij, e_ik, basis]))" with MLP = Linear, SiLU, Linear
             and no biases; the second Linear is applied after the sum, which is the same thing);
  envelopes  u_b = u(d_b / r_bond) multiplies every term a bond takes part in, so that the energy stays a
             smooth function of the positions when a bond crosses r_bond;
  atom layers as in the two-body model, the filter of a bonded edge gets the extra term e1_b Wb_l.

Weights on top of the two-body ones: We0 [K, Fb], Wt1 [2 Fb + A, Fb], Wt2 [Fb, Fb], Wb [L, Fb, F].
"""
from __future__ import annotations

import numpy as np

from . import graph as og
from ._lib import c_f32p, c_f64p, c_i32p, c_i64p, lib
from .model import _cast, _dsilu, _silu

A_ANGLE = 8


def _edge_keys(g):
    """(receiver, key) per edge; within a row the key increases in the canonical (sender, Sx, Sy, Sz) order."""
    s = g.shifts.astype(np.int64) + 512
    assert (s >= 0).all() and (s < 1024).all()
    return g.receivers.astype(np.int64), (g.senders.astype(np.int64) << 30) | (s[:, 0] << 20) | (s[:, 1] << 10) | s[:, 2]


def bond_graph(positions, cell, graph, r_bond):
    """Bonds of the atom graph.  Returns (bond_edge int64 [nb] edge index of every bond, ascending;
    bptr int64 [N+1] bonds per centre; bond_of_edge int64 [E], -1 for edges that are no bonds)."""
    gb = og.build_graph(positions, cell, r_bond)           # same predicate, smaller cutoff
    ra, ka = _edge_keys(graph)
    rb, kb = _edge_keys(gb)
    # every bond is an edge: sort both lists together; a bond lands right behind its edge
    tag = np.concatenate([np.zeros(graph.E, np.int8), np.ones(gb.E, np.int8)])
    order = np.lexsort((tag, np.concatenate([ka, kb]), np.concatenate([ra, rb])))
    where = np.flatnonzero(tag[order] == 1)
    bond_edge = order[where - 1].astype(np.int64)
    assert (tag[order[where - 1]] == 0).all()
    assert np.array_equal(ka[bond_edge], kb) and np.array_equal(ra[bond_edge], rb)
    bond_of_edge = np.full(graph.E, -1, np.int64)
    bond_of_edge[bond_edge] = np.arange(len(bond_edge))
    return bond_edge, gb.row_ptr.copy(), bond_of_edge


def angle_basis(c, A=A_ANGLE):
    """cos(n theta), n = 0..A-1, from c = cos(theta), by the recurrence T_{n+1} = 2 c T_n - T_{n-1}."""
    T = [np.ones_like(c), c]
    for _ in range(2, A):
        T.append(2 * c * T[-1] - T[-2])
    return np.stack(T[:A], -1)


class _C:
    def __init__(self, fp32):
        self.dt = np.float32 if fp32 else np.float64
        self.fp = c_f32p if fp32 else c_f64p
        self.suf = "f32" if fp32 else "f64"

    def p(self, a):
        assert a.dtype == self.dt and a.flags.c_contiguous
        return a.ctypes.data_as(self.fp)

    def fn(self, name):
        return getattr(lib(), name + "_" + self.suf)


def _envelope(x, p):
    c0, c1, c2 = (p + 1) * (p + 2) / 2, p * (p + 2), p * (p + 1) / 2
    u = 1 - c0 * x ** p + c1 * x ** (p + 1) - c2 * x ** (p + 2)
    du = -p * c0 * x ** (p - 1) + (p + 1) * c1 * x ** p - (p + 2) * c2 * x ** (p + 1)
    return u, du


def _basis_rows(cc, d, rc, K, p):
    b = np.zeros((len(d), K), cc.dt)
    db = np.zeros((len(d), K), cc.dt)
    cc.fn("orc3_basis_rows")(len(d), cc.p(np.ascontiguousarray(d)), cc.dt(rc), K, p, cc.p(b), cc.p(db))
    return b, db


def energy_forces3(positions, cell, species, weights, graph, r_cut, r_bond, K, p, fp32=False):
    """Whole-graph energy, forces [N,3] and per-atom energies of the three-body variant."""
    cc = _C(fp32)
    dt = cc.dt
    W = _cast(weights, dt)
    L = W["W1"].shape[0]
    Fb = W["We0"].shape[1]
    A = W["Wt1"].shape[0] - 2 * Fb
    N = graph.N
    d64, rhat64 = og.geometry(positions, cell, graph)
    d = np.ascontiguousarray(d64, dt)
    rhat = np.ascontiguousarray(rhat64, dt)
    rp, sd = graph.row_ptr, graph.senders
    ip, i32 = rp.ctypes.data_as(c_i64p), sd.ctypes.data_as(c_i32p)

    # ---- bonds, e0, triplet sum, e1
    bond_edge, bptr, bond_of_edge = bond_graph(positions, cell, graph, r_bond)
    nb = len(bond_edge)
    db_ = np.ascontiguousarray(d[bond_edge])
    rb_hat = np.ascontiguousarray(rhat[bond_edge])
    bb, dbb = _basis_rows(cc, db_, r_bond, K, p)
    u64, du64 = _envelope(db_.astype(np.float64) / r_bond, p)
    u = np.ascontiguousarray(u64, dt)
    e0 = bb @ W["We0"]
    Wta, Wtb, Wtc = W["Wt1"][:Fb], W["Wt1"][Fb:2 * Fb], np.ascontiguousarray(W["Wt1"][2 * Fb:])
    P = np.ascontiguousarray(e0 @ Wta)
    Q = np.ascontiguousarray(e0 @ Wtb)
    S = np.zeros((nb, Fb), dt)
    bp = bptr.ctypes.data_as(c_i64p)
    cc.fn("orc3_triplet_forward")(N, bp, cc.p(rb_hat), cc.p(u), cc.p(P), cc.p(Q), cc.p(Wtc), A, Fb, cc.p(S))
    m = S @ W["Wt2"]
    e1 = e0 + u[:, None] * _silu(m)

    # ---- atom layers
    boe = bond_of_edge.ctypes.data_as(c_i64p)
    h = W["emb"][species].copy()
    gs, as_, wbs = [], [], []
    for l in range(L):
        g = np.ascontiguousarray(h @ W["Wm"][l])
        wb = np.ascontiguousarray(e1 @ W["Wb"][l])
        a = np.zeros((N, g.shape[1]), dt)
        cc.fn("orc3_edge_forward")(N, ip, i32, cc.p(d), dt(r_cut), K, p, g.shape[1], cc.p(W["W1"][l]),
                                   cc.p(W["W2"][l]), boe, cc.p(wb), cc.p(g), cc.p(a))
        h = h + _silu(a @ W["Wo"][l])
        gs.append(g)
        as_.append(a)
        wbs.append(wb)
    pre = h @ W["Wr1"]
    eps = _silu(pre) @ W["wr2"]
    energy = float(np.sum(eps.astype(np.float64)))

    # ---- reverse pass: atom layers
    hbar = (W["wr2"][None, :] * _dsilu(pre)) @ W["Wr1"].T
    dbar = np.zeros(graph.E, dt)                      # dE/dd_e through the radial filters
    e1bar = np.zeros((nb, Fb), dt)
    for l in reversed(range(L)):
        q = as_[l] @ W["Wo"][l]
        abar = np.ascontiguousarray((hbar * _dsilu(q)) @ W["Wo"][l].T)
        gbar = np.zeros_like(gs[l])
        wbbar = np.zeros((nb, gs[l].shape[1]), dt)
        cc.fn("orc3_edge_backward")(N, N, ip, i32, cc.p(d), dt(r_cut), K, p, gs[l].shape[1], cc.p(W["W1"][l]),
                                    cc.p(W["W2"][l]), boe, cc.p(wbs[l]), cc.p(gs[l]), cc.p(abar), cc.p(gbar),
                                    cc.p(dbar), cc.p(wbbar))
        hbar = hbar + gbar @ W["Wm"][l].T
        e1bar += wbbar @ W["Wb"][l].T
    # ---- reverse pass: bond update
    sm = _silu(m)
    ubar = (e1bar * sm).sum(1)                        # e1 = e0 + u SiLU(m)
    mbar = e1bar * u[:, None] * _dsilu(m)
    Sbar = np.ascontiguousarray(mbar @ W["Wt2"].T)
    Pbar = np.zeros((nb, Fb), dt)
    Qbar = np.zeros((nb, Fb), dt)
    ubar_t = np.zeros(nb, dt)
    rbar = np.zeros((nb, 3), dt)
    cc.fn("orc3_triplet_backward")(N, bp, cc.p(rb_hat), cc.p(u), cc.p(P), cc.p(Q), cc.p(Wtc), A, Fb, cc.p(Sbar),
                                   cc.p(Pbar), cc.p(Qbar), cc.p(ubar_t), cc.p(rbar))
    e0bar = e1bar + Pbar @ Wta.T + Qbar @ Wtb.T
    ubar = ubar + ubar_t
    # distance dependence of the bonds: e0 = bbond(d) We0, u = u(d / r_bond)
    dbond = ((e0bar @ W["We0"].T) * dbb).sum(1) + ubar * np.asarray(du64, dt) / dt(r_bond)
    # ---- positions: Delta_e = r_j + S C - r_i;  d = |Delta|, rhat = Delta / d
    gdelta = dbar[:, None].astype(np.float64) * rhat64
    rb64 = rhat64[bond_edge]
    rbar64 = rbar.astype(np.float64)
    gdelta[bond_edge] += dbond[:, None].astype(np.float64) * rb64 + \
        (rbar64 - (rbar64 * rb64).sum(1, keepdims=True) * rb64) / d64[bond_edge][:, None]
    gradpos = np.zeros((N, 3), np.float64)
    np.add.at(gradpos, sd, gdelta)
    np.add.at(gradpos, graph.receivers, -gdelta)
    return dict(energy=energy, forces=-gradpos, atom_energy=eps.astype(np.float64), n_bonds=nb,
                n_triplets=int((np.diff(bptr) * (np.diff(bptr) - 1)).sum()), e1=e1, bond_edge=bond_edge, bptr=bptr)


def energy3_reference(positions, cell, species, weights, graph, r_cut, r_bond, K, p):
    """The same energy written a second time with plain numpy loops over atoms, bonds and triplets
    (no shared routines with energy_forces3 beyond the neighbour list): small systems only."""
    W = {k: np.asarray(v, np.float64) for k, v in weights.items()}
    L = W["W1"].shape[0]
    Fb = W["We0"].shape[1]
    N = graph.N
    recv = graph.receivers
    delta = positions[graph.senders] + graph.shifts @ cell - positions[recv]
    d = np.sqrt((delta ** 2).sum(1))
    rhat = delta / d[:, None]

    def basis(dd, rc):
        n = np.arange(1, K + 1)
        x = dd / rc
        return np.sin(n * np.pi * x) / dd * _envelope(x, p)[0]

    is_bond = d <= r_bond
    e1 = {}
    for i in range(N):
        es = [e for e in range(graph.row_ptr[i], graph.row_ptr[i + 1]) if is_bond[e]]
        e0 = {e: basis(d[e], r_bond) @ W["We0"] for e in es}
        for e in es:
            S = np.zeros(Fb)
            for e2 in es:
                if e2 == e:
                    continue
                c = float(rhat[e] @ rhat[e2])
                theta = np.arccos(np.clip(c, -1.0, 1.0))
                T = np.cos(np.arange(W["Wt1"].shape[0] - 2 * Fb) * theta)
                hvec = np.concatenate([e0[e], e0[e2], T]) @ W["Wt1"]
                S += _envelope(d[e2] / r_bond, p)[0] * _silu(hvec)
            e1[e] = e0[e] + _envelope(d[e] / r_bond, p)[0] * _silu(S @ W["Wt2"])
    h = W["emb"][species].copy()
    for l in range(L):
        g = h @ W["Wm"][l]
        a = np.zeros_like(g)
        for e in range(graph.E):
            w = _silu(basis(d[e], r_cut) @ W["W1"][l]) @ W["W2"][l]
            if is_bond[e]:
                w = w + e1[e] @ W["Wb"][l]
            a[recv[e]] += w * g[graph.senders[e]]
        h = h + _silu(a @ W["Wo"][l])
    return float((_silu(h @ W["Wr1"]) @ W["wr2"]).sum())


def energy_forces3_slabs(positions, cell, species, weights, graph, slabs, slab_of, r_cut, r_bond, K, p):
    """The three-body variant through the partitioned scheme (slabs from oracle.graph.partition), fp64.

    An edge belongs to the partition of its receiver (Distributing Atom Graphs), so all bonds of an owned centre,
    and with them all its triplets, lie inside its partition: the bond update needs no transfer.  The atom layers
    exchange border-node features per layer as in the two-body scheme; in the reverse pass the gradients of ghost
    rows (features and positions, the latter now also through bond vectors that end on a ghost atom) go back to
    the owners."""
    cc = _C(False)
    dt = cc.dt
    W = _cast(weights, dt)
    L = W["W1"].shape[0]
    F = W["emb"].shape[1]
    Fb = W["We0"].shape[1]
    A = W["Wt1"].shape[0] - 2 * Fb
    Wta, Wtb, Wtc = W["Wt1"][:Fb], W["Wt1"][Fb:2 * Fb], np.ascontiguousarray(W["Wt1"][2 * Fb:])
    d64, rhat64 = og.geometry(positions, cell, graph)
    _, _, bond_of_edge_g = bond_graph(positions, cell, graph, r_bond)
    P_ = len(slabs)
    n_own = [len(s.owned) for s in slabs]
    local_in_owner = np.full(graph.N, -1, np.int64)
    for s in slabs:
        local_in_owner[s.nodes[: len(s.owned)]] = np.arange(len(s.owned))

    class Loc:
        pass

    loc = []
    for i, s in enumerate(slabs):
        o = Loc()
        o.d = np.ascontiguousarray(d64[s.edge_ids])
        o.rhat = np.ascontiguousarray(rhat64[s.edge_ids])
        is_bond = bond_of_edge_g[s.edge_ids] >= 0
        o.bond_edge = np.flatnonzero(is_bond).astype(np.int64)          # local edge index of every local bond
        o.boe = np.full(len(s.edge_ids), -1, np.int64)
        o.boe[o.bond_edge] = np.arange(len(o.bond_edge))
        o.bptr = np.concatenate([[0], np.cumsum(is_bond.astype(np.int64))])[s.row_ptr].astype(np.int64)
        o.db = np.ascontiguousarray(o.d[o.bond_edge])
        o.rb = np.ascontiguousarray(o.rhat[o.bond_edge])
        o.bb, o.dbb = _basis_rows(cc, o.db, r_bond, K, p)
        u, du = _envelope(o.db / r_bond, p)
        o.u, o.du = np.ascontiguousarray(u), du
        nb = len(o.bond_edge)
        o.e0 = o.bb @ W["We0"]
        o.P = np.ascontiguousarray(o.e0 @ Wta)
        o.Q = np.ascontiguousarray(o.e0 @ Wtb)
        o.S = np.zeros((nb, Fb))
        cc.fn("orc3_triplet_forward")(n_own[i], o.bptr.ctypes.data_as(c_i64p), cc.p(o.rb), cc.p(o.u), cc.p(o.P),
                                      cc.p(o.Q), cc.p(Wtc), A, Fb, cc.p(o.S))
        o.m = o.S @ W["Wt2"]
        o.e1 = o.e0 + o.u[:, None] * _silu(o.m)
        loc.append(o)

    def edge_args(s):
        return len(s.row_ptr) - 1, s.row_ptr.ctypes.data_as(c_i64p), s.senders.ctypes.data_as(c_i32p)

    h = [W["emb"][species[s.nodes[: n_own[i]]]].copy() for i, s in enumerate(slabs)]
    gs = [[None] * P_ for _ in range(L)]
    as_ = [[None] * P_ for _ in range(L)]
    wbs = [[None] * P_ for _ in range(L)]
    for l in range(L):
        g = []
        for i, s in enumerate(slabs):
            gi = np.zeros((len(s.nodes), F))
            gi[: n_own[i]] = h[i] @ W["Wm"][l]
            g.append(gi)
        for i, s in enumerate(slabs):          # border-node transfer: ghost rows <- owner rows
            gh = s.nodes[n_own[i]:]
            for q in range(P_):
                sel = np.flatnonzero(slab_of[gh] == q)
                g[i][n_own[i] + sel] = g[q][local_in_owner[gh[sel]]]
        for i, s in enumerate(slabs):
            o = loc[i]
            wb = np.ascontiguousarray(o.e1 @ W["Wb"][l])
            a = np.zeros((n_own[i], F))
            nrows, rp, sd = edge_args(s)
            cc.fn("orc3_edge_forward")(nrows, rp, sd, cc.p(o.d), float(r_cut), K, p, F, cc.p(W["W1"][l]), cc.p(W["W2"][l]),
                                       o.boe.ctypes.data_as(c_i64p), cc.p(wb), cc.p(g[i]), cc.p(a))
            h[i] = h[i] + _silu(a @ W["Wo"][l])
            gs[l][i], as_[l][i], wbs[l][i] = g[i], a, wb
    energy = 0.0
    atom_energy = np.zeros(graph.N)
    hbar = []
    for i, s in enumerate(slabs):
        pre = h[i] @ W["Wr1"]
        eps = _silu(pre) @ W["wr2"]
        atom_energy[s.nodes[: n_own[i]]] = eps
        energy += float(eps.sum())
        hbar.append((W["wr2"][None, :] * _dsilu(pre)) @ W["Wr1"].T)
    dbar = [np.zeros(len(s.edge_ids)) for s in slabs]
    e1bar = [np.zeros_like(o.e1) for o in loc]
    for l in reversed(range(L)):
        gbar = []
        for i, s in enumerate(slabs):
            o = loc[i]
            q_ = as_[l][i] @ W["Wo"][l]
            abar = np.ascontiguousarray((hbar[i] * _dsilu(q_)) @ W["Wo"][l].T)
            gb = np.zeros_like(gs[l][i])
            wbbar = np.zeros((len(o.bond_edge), F))
            nrows, rp, sd = edge_args(s)
            cc.fn("orc3_edge_backward")(nrows, len(s.nodes), rp, sd, cc.p(o.d), float(r_cut), K, p, F, cc.p(W["W1"][l]),
                                        cc.p(W["W2"][l]), o.boe.ctypes.data_as(c_i64p), cc.p(wbs[l][i]), cc.p(gs[l][i]),
                                        cc.p(abar), cc.p(gb), cc.p(dbar[i]), cc.p(wbbar))
            gbar.append(gb)
            e1bar[i] += wbbar @ W["Wb"][l].T
        for i, s in enumerate(slabs):          # ghost-row gradients -> owners
            gh = s.nodes[n_own[i]:]
            for q in range(P_):
                sel = np.flatnonzero(slab_of[gh] == q)
                gbar[q][local_in_owner[gh[sel]]] += gbar[i][n_own[i] + sel]
        for i in range(P_):
            hbar[i] = hbar[i] + gbar[i][: n_own[i]] @ W["Wm"][l].T
    gradpos = np.zeros((graph.N, 3))
    for i, s in enumerate(slabs):
        o = loc[i]
        nb = len(o.bond_edge)
        ubar = (e1bar[i] * _silu(o.m)).sum(1)
        mbar = e1bar[i] * o.u[:, None] * _dsilu(o.m)
        Sbar = np.ascontiguousarray(mbar @ W["Wt2"].T)
        Pbar, Qbar = np.zeros((nb, Fb)), np.zeros((nb, Fb))
        ubar_t, rbar = np.zeros(nb), np.zeros((nb, 3))
        cc.fn("orc3_triplet_backward")(n_own[i], o.bptr.ctypes.data_as(c_i64p), cc.p(o.rb), cc.p(o.u), cc.p(o.P), cc.p(o.Q),
                                       cc.p(Wtc), A, Fb, cc.p(Sbar), cc.p(Pbar), cc.p(Qbar), cc.p(ubar_t), cc.p(rbar))
        e0bar = e1bar[i] + Pbar @ Wta.T + Qbar @ Wtb.T
        dbond = ((e0bar @ W["We0"].T) * o.dbb).sum(1) + (ubar + ubar_t) * o.du / r_bond
        gdelta = dbar[i][:, None] * o.rhat
        gdelta[o.bond_edge] += dbond[:, None] * o.rb + (rbar - (rbar * o.rb).sum(1, keepdims=True) * o.rb) / o.db[:, None]
        recv_loc = np.repeat(np.arange(n_own[i]), np.diff(s.row_ptr))
        gp = np.zeros((len(s.nodes), 3))
        np.add.at(gp, s.senders, gdelta)       # owned and ghost senders alike
        np.add.at(gp, recv_loc, -gdelta)
        np.add.at(gradpos, s.nodes, gp)        # ghost rows go back to the atoms they stand for
    return dict(energy=energy, forces=-gradpos, atom_energy=atom_energy)
