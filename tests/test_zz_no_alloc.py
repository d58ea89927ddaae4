"""mlip_forward_static (the entry point that allocates nothing) against mlip_forward, through the C ABI.

Two calls in a row on the same GPU, the second on a smaller system: the shared static workspace keeps the first
call's contents, so the second call must clear what it needs at zero.  Results are compared with mlip_forward's on
the same handles (every reduction runs in a fixed order, so they are bit-identical, which is within the fp32 bounds
of 1e-5 relative energy error and 1e-4 max|F|), and with the oracle.  Sizes beyond the workspace are rejected.
"""
import numpy as np
import pytest

import workloads as wl

from gpu_util import E_RTOL, F_RTOL, assert_energy_forces, oracle_config

pytestmark = pytest.mark.gpu


def _both(M, g, W, mode):
    import torch
    e0, f0, a0 = M.mlip_forward(g, W, mode)
    torch.cuda.synchronize()
    e0, f0, a0 = float(e0.cpu()[0]), f0.cpu().numpy().astype(np.float64), a0.cpu().numpy().astype(np.float64)
    e1, f1, a1 = M.mlip_forward_static(g, W, mode)
    torch.cuda.synchronize()
    e1, f1, a1 = float(e1.cpu()[0]), f1.cpu().numpy().astype(np.float64), a1.cpu().numpy().astype(np.float64)
    return (e0, f0, a0), (e1, f1, a1)


def test_static_workspace_forward_matches_mlip_forward():
    import torch
    import paper_2506_02023_amd as M
    assert M.lib().mlip_static_scratch_bytes() == 64 << 20
    # first call: configs[1] recipe at 7^3 cells (1,372 atoms, F = 64, L = 3), 3 slabs; second: configs[0] (108 atoms, F = 32)
    for index, n, P in ((1, 7, 3), (0, None, 2)):
        c, ref_g, ref = oracle_config(index, n)
        pos = torch.as_tensor(c["positions"], device="cuda")
        sp = torch.as_tensor(c["species"], device="cuda")
        g = M.mlip_build_graph(pos, c["cell"], sp, c["r_cut"], n_slabs=P)
        for precision in (0, 2):
            W = M.Weights(c["weights"], c["p"], precision=precision)
            for mode in (M.MODE_SLABS, M.MODE_WHOLE):
                (e0, f0, a0), (e1, f1, a1) = _both(M, g, W, mode)
                label = f"configs[{index}] n={n} precision {precision} mode {mode}"
                assert abs(e1 - e0) <= E_RTOL * abs(e0), label
                assert np.abs(f1 - f0).max() <= F_RTOL * np.abs(f0).max(), label
                assert e1 == e0 and np.array_equal(f1, f0) and np.array_equal(a1, a0), label
                assert_energy_forces(e1, f1, ref, label)
        g.destroy()


def test_static_workspace_rejects_what_does_not_fit():
    import torch
    import paper_2506_02023_amd as M
    c = wl.make_config(1, n=12)          # 6,912 atoms, about 311 k edges, L = 3: the kept filter values alone are 159 MB
    pos = torch.as_tensor(c["positions"], device="cuda")
    sp = torch.as_tensor(c["species"], device="cuda")
    g = M.mlip_build_graph(pos, c["cell"], sp, c["r_cut"], n_slabs=2)
    W = M.Weights(c["weights"], c["p"])
    with pytest.raises(M.MlipError) as err:
        M.mlip_forward_static(g, W, M.MODE_WHOLE)
    assert err.value.code == -1 and "static workspace" in str(err.value)
    e, f, _ = M.mlip_forward(g, W, M.MODE_WHOLE)      # the allocating entry point still takes it
    torch.cuda.synchronize()
    assert np.isfinite(float(e.cpu()[0]))
    g.profile_enable(True)
    c0 = wl.make_config(0)
    g0 = M.mlip_build_graph(torch.as_tensor(c0["positions"], device="cuda"), c0["cell"],
                            torch.as_tensor(c0["species"], device="cuda"), c0["r_cut"])
    g0.profile_enable(True)
    with pytest.raises(M.MlipError) as err:
        M.mlip_forward_static(g0, M.Weights(c0["weights"], c0["p"]), M.MODE_WHOLE)
    assert err.value.code == -6
