"""Helpers for the GPU parity tests: run libmlip through the binding, run the oracle, compare."""
import functools

import numpy as np

import workloads as wl
from oracle import graph as og
from oracle import model as om

E_RTOL = 1e-5      # relative energy error, fp32 path
F_RTOL = 1e-4      # max force-component error relative to max |F| component


def gpu_graph(pos, cell, species, r_cut, n_slabs=1, graph=None):
    import torch
    import paper_2506_02023_amd as M
    tp = torch.as_tensor(np.ascontiguousarray(pos, np.float64), device="cuda")
    ts = torch.as_tensor(np.ascontiguousarray(species, np.int32), device="cuda")
    return M.mlip_build_graph(tp, cell, ts, r_cut, n_slabs=n_slabs, graph=graph)


def gpu_energy_forces(g, weights, p, mode, precision=0):
    import torch
    import paper_2506_02023_amd as M
    W = M.Weights(weights, p, precision=precision)
    e, f, ae = M.mlip_forward(g, W, mode)
    torch.cuda.synchronize()
    return float(e.cpu()[0]), f.cpu().numpy().astype(np.float64), ae.cpu().numpy().astype(np.float64)


@functools.lru_cache(maxsize=4)
def oracle_config(index, n=None):
    """(config dict, oracle graph, oracle fp64 result) -- cached, the medium cases take seconds."""
    c = wl.make_config(index, n=n)
    g = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    r = om.energy_forces(c["positions"], c["cell"], c["species"], c["weights"], g, c["r_cut"], c["K"], c["p"])
    return c, g, r


def assert_graph_equal(gpu, ref, positions=None, cell=None):
    row_ptr, senders, shifts, d = gpu.csr()
    N, E, _ = gpu.sizes()
    assert (N, E) == (ref.N, ref.E)
    assert np.array_equal(row_ptr, ref.row_ptr)
    assert np.array_equal(senders, ref.senders)
    assert np.array_equal(shifts, ref.shifts)
    if positions is not None:
        d64, _ = og.geometry(positions, cell, ref)
        assert np.array_equal(d, d64.astype(np.float32))     # fp64 length rounded once to fp32


def assert_energy_forces(e, f, ref, what=""):
    fmax = np.abs(ref["forces"]).max()
    de = abs(e - ref["energy"]) / abs(ref["energy"])
    df = np.abs(f - ref["forces"]).max() / fmax
    assert de <= E_RTOL, f"{what}: relative energy error {de:.3e}"
    assert df <= F_RTOL, f"{what}: force error {df:.3e} of max|F|"
    return de, df
