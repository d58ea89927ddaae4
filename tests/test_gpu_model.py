"""GPU parity: energy and forces against the fp64 oracle (whole graph and partitioned)."""
import numpy as np
import pytest

import workloads as wl
from oracle import graph as og
from oracle import model as om

from gpu_util import assert_energy_forces, gpu_energy_forces, gpu_graph, oracle_config

pytestmark = pytest.mark.gpu

WHOLE, SLABS = 0, 1


# precision 0: fp32 MFMA; 2: the W2 products as split-fp16 triples, held to the same fp32 bounds
@pytest.mark.parametrize("precision", [0, 2])
@pytest.mark.parametrize("index", [0, 1])
def test_whole_graph_configs(index, precision):
    c, _, ref = oracle_config(index)
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"])
    e, f, ae = gpu_energy_forces(g, c["weights"], c["p"], WHOLE, precision)
    de, df = assert_energy_forces(e, f, ref, f"configs[{index}] whole")
    assert np.abs(ae - ref["atom_energy"]).max() <= 1e-4 * np.abs(ref["atom_energy"]).max()
    print(f"configs[{index}] whole, precision {precision}: dE/E = {de:.2e}, dF/Fmax = {df:.2e}")


@pytest.mark.parametrize("P", [2, 3, 8])
def test_slabs_config0(P):
    c, _, ref = oracle_config(0)
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"], n_slabs=P)
    e, f, ae = gpu_energy_forces(g, c["weights"], c["p"], SLABS)
    assert_energy_forces(e, f, ref, f"configs[0] {P} slabs")
    ew, fw, _ = gpu_energy_forces(g, c["weights"], c["p"], WHOLE)
    assert_energy_forces(ew, fw, ref, "configs[0] whole on a partitioned graph")


@pytest.mark.parametrize("precision", [0, 2])
def test_slabs_medium(precision):
    c, _, ref = oracle_config(1)
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"], n_slabs=8)
    e, f, ae = gpu_energy_forces(g, c["weights"], c["p"], SLABS, precision)
    de, df = assert_energy_forces(e, f, ref, "configs[1] 8 slabs")
    print(f"configs[1] 8 slabs, precision {precision}: dE/E = {de:.2e}, dF/Fmax = {df:.2e}")


def test_triclinic_small_cell_f32_features():
    """F = 32, thin triclinic cell (multiple images), 3 slabs thinner than r_cut."""
    pos, cell, sp = wl.random_triclinic(40, 8, scale=6.0)
    W = wl.rmp_weights(4, 32, 2, seed=3)
    ref_g = og.build_graph(pos, cell, 3.5)
    ref = om.energy_forces(pos, cell, sp, W, ref_g, 3.5, 8, 6)
    g = gpu_graph(pos, cell, sp, 3.5, n_slabs=3)
    for mode in (WHOLE, SLABS):
        e, f, _ = gpu_energy_forces(g, W, 6, mode)
        assert_energy_forces(e, f, ref, f"triclinic mode {mode}")


def test_zero_layers_and_isolated_atoms():
    import paper_2506_02023_amd as M
    c, _, _ = oracle_config(0)
    W0 = {k: (v[:0] if k in ("W1", "W2", "Wm", "Wo") else v) for k, v in c["weights"].items()}
    ref_g = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    ref = om.energy_forces(c["positions"], c["cell"], c["species"], W0, ref_g, c["r_cut"], c["K"], c["p"])
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"])
    e, f, _ = gpu_energy_forces(g, W0, c["p"], WHOLE)
    assert abs(e - ref["energy"]) <= 1e-5 * abs(ref["energy"]) and np.all(f == 0)
    # atoms with no neighbours at all: empty rows everywhere
    pos = np.array([[1.0, 1, 1], [12.0, 12, 12], [22.0, 5, 17]])
    cell = np.eye(3) * 30.0
    sp = np.array([0, 1, 2], np.int32)
    ref_g = og.build_graph(pos, cell, 5.0)
    assert ref_g.E == 0
    ref = om.energy_forces(pos, cell, sp, c["weights"], ref_g, 5.0, 8, 6)
    g = gpu_graph(pos, cell, sp, 5.0)
    e, f, _ = gpu_energy_forces(g, c["weights"], 6, WHOLE)
    assert abs(e - ref["energy"]) <= 1e-5 * abs(ref["energy"]) and np.all(f == 0)
    # species out of range is refused
    g = gpu_graph(pos, cell, np.array([0, 1, 9], np.int32), 5.0)
    with pytest.raises(M.MlipError):
        gpu_energy_forces(g, c["weights"], 6, WHOLE)


@pytest.mark.parametrize("d", [4.9, 4.95])
def test_only_edges_close_to_the_cutoff(d):
    """Three atoms whose only neighbours sit just inside the cutoff, where the envelope and its derivative are tiny:
    the force bound is relative to these tiny forces, so it only holds if the envelope is evaluated without
    cancellation there."""
    c = wl.make_config(1, n=2)
    pos = np.array([[10.0, 10.0, 10.0], [10.0 + d, 10.0, 10.0], [10.0, 10.0 + 0.6 * d, 10.0 + 0.8 * d]])
    cell = np.eye(3) * 30.0
    sp = np.array([0, 1, 2], np.int32)
    ref_g = og.build_graph(pos, cell, c["r_cut"])
    assert ref_g.E == 4
    ref = om.energy_forces(pos, cell, sp, c["weights"], ref_g, c["r_cut"], c["K"], c["p"])
    g = gpu_graph(pos, cell, sp, c["r_cut"])
    e, f, _ = gpu_energy_forces(g, c["weights"], c["p"], WHOLE)
    assert_energy_forces(e, f, ref, f"neighbours at {d}")


@pytest.mark.parametrize("precision", [0, 2])
def test_limits_eight_layers_64_slabs(precision):
    """The largest layer count and slab count the library accepts, whole graph and partitioned."""
    c = wl.make_config(0, n=4)
    w = wl.rmp_weights(4, 32, 8, 91)
    ref_g = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    ref = om.energy_forces(c["positions"], c["cell"], c["species"], w, ref_g, c["r_cut"], c["K"], c["p"])
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"], n_slabs=64)
    e, f, _ = gpu_energy_forces(g, w, c["p"], WHOLE, precision=precision)
    assert_energy_forces(e, f, ref, "L = 8, whole graph")
    es, fs, _ = gpu_energy_forces(g, w, c["p"], SLABS, precision=precision)
    assert_energy_forces(es, fs, ref, "L = 8, 64 slabs")


def test_split_mode_range_violation_is_visible():
    """The split-fp16 mode needs the operands of its products below the fp16 range; weights that push the hidden
    activations of the filter MLP beyond it give a non-finite energy there (and a finite one in fp32 mode)."""
    c, ref_g, _ = oracle_config(0)
    w = dict(c["weights"])
    w["W1"] = w["W1"] * np.float32(3e5)
    g = gpu_graph(c["positions"], c["cell"], c["species"], c["r_cut"])
    e32, _, _ = gpu_energy_forces(g, w, c["p"], WHOLE, precision=0)
    e16, _, _ = gpu_energy_forces(g, w, c["p"], WHOLE, precision=2)
    assert np.isfinite(e32)
    assert not np.isfinite(e16)


def test_more_slabs_than_populated_regions():
    """A cluster at one end of a long cell cut into 8 slabs: most partitions own nothing, some have ghosts only
    on one side.  Two-body and three-body variants, slabs against whole graph and oracle."""
    import torch
    import paper_2506_02023_amd as M
    from oracle import three_body as tb
    c4 = wl.make_config(4, n=3)
    rng = np.random.default_rng(9)
    pos = np.concatenate([rng.uniform(0.5, 9.5, (40, 3)) * np.array([1.0, 0.6, 0.6]), np.array([[41.0, 3.0, 3.0]])])
    cell = np.diag([64.0, 7.0, 7.0])
    sp = rng.integers(0, 4, len(pos)).astype(np.int32)
    ref_g = og.build_graph(pos, cell, 5.0)
    ref = om.energy_forces(pos, cell, sp, c4["weights"], ref_g, 5.0, 8, 6)
    g = gpu_graph(pos, cell, sp, 5.0, n_slabs=8)
    owned = [g.slab(p)["n_owned"] for p in range(8)]
    assert owned.count(0) >= 4
    es, fs, _ = gpu_energy_forces(g, {k: c4["weights"][k] for k in ("emb", "W1", "W2", "Wm", "Wo", "Wr1", "wr2")}, 6, SLABS)
    assert_energy_forces(es, fs, ref, "sparse slabs")
    ref3 = tb.energy_forces3(pos, cell, sp, c4["weights"], ref_g, 5.0, 3.0, 8, 6)
    W = M.Weights({k: c4["weights"][k] for k in ("emb", "W1", "W2", "Wm", "Wo", "Wr1", "wr2")}, 6)
    BW = M.BondWeights(c4["weights"], 3.0, 8)
    e3, f3, _ = M.mlip_forward_bonds(g, W, BW, M.MODE_SLABS)
    torch.cuda.synchronize()
    assert abs(float(e3.cpu()[0]) - ref3["energy"]) <= 1e-4 * abs(ref3["energy"])
    assert np.abs(f3.cpu().numpy() - ref3["forces"]).max() <= 1e-4 * np.abs(ref3["forces"]).max()
