"""Benchmark: energy + forces throughput of the partitioned hot path on one MI355X.

One step = mlip_build_graph (n_slabs = 8) + mlip_forward in SLABS mode on benchmark
configuration 3 (63^3 fcc cells, 1,000,188 atoms, ~45.8M directed edges, F = 64, L = 3),
i.e. every stage of the path: cell list, CSR, partition, three layers forward with ghost
copies, reverse pass with ghost-gradient add-backs, forces.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3
# Algorithmic flops per directed edge and layer, i.e. of the operation as it is defined:
#   forward: filter MLP, t = b W1 (2 K F) and w = SiLU(t) W2 (2 F F);
#   reverse: pre-activations t = b W1 (2 K F), sbar = wbar W2^T (2 F F), dt/dd contraction through W1 (2 K F);
#            the filter value w_e itself is not recomputed, the forward pass keeps it in HBM (layers >= 1).
# The reverse kernel runs this dense work once per edge / reverse-edge pair (both have the same length), so the
# MFMA units execute half of the reverse figure per directed edge; with fp32 MFMA the edge kernels run on the upper
# edge of every pair only (the forward one then evaluates the filter MLP once per pair too), and memory-bound second
# passes add the lower edges' terms.  A kernel's roofline fraction is taken on what it executes; the rate of the
# operation as defined is reported beside it ("as_defined_tflops").
def flops_fwd_edge(F, K=8):
    return 2 * K * F + 2 * F * F


PEAK_HBM_GBS = 8000.0


def flops_bwd_edge_as_defined(F, K=8):
    return 2 * K * F + 2 * F * F + 2 * K * F


def flops_bwd_edge(F, K=8):
    """Executed per directed edge: the dense work of a pair, shared by its two edges."""
    return flops_bwd_edge_as_defined(F, K) // 2


# HBM bytes per launch (one layer over all 8 slabs) on the default workload, from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE (profiles/edge_traffic_configs3_8slabs.md): KiB x copy-kernel scale (1.9976 for FETCH_SIZE, 1.000 for
# WRITE_SIZE)
TRAFFIC_SOURCE = ("profiled constant, not measured by this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this kernel on "
                  "this workload, profiles/edge_traffic_configs3_8slabs.md")
TRAFFIC_BWD_LAUNCH_BYTES = (6196767 * 1.9976 + 1003909) * 1024         # k_edge_bwd on the upper-edge graphs
TRAFFIC_FWD_LAUNCH_BYTES = (1369693 * 1.9976 + 6367675) * 1024         # k_edge_fwd on the upper-edge graphs
TRAFFIC_FWD_LOWER_LAUNCH_BYTES = (3853592 * 1.9976 + 250047) * 1024    # k_edge_lower, forward
TRAFFIC_BWD_LOWER_LAUNCH_BYTES = (3853695 * 1.9976 + 250047) * 1024    # k_edge_lower, reverse


# fp32 vector peak that applies to this build: 256 CUs x 4 SIMDs x 16 lanes x 2 flop per FMA x 2.4 GHz = 78.6 TFLOP/s.
# (The published 157.3 TFLOP/s counts packed fp32 FMAs, which the library is compiled without.)  It bounds the triplet
# kernels of the three-body variant.
PEAK_FP32_VECTOR_TFLOPS = 78.6


def flops_triplet_fwd(F, A=8):
    """Per ordered triplet: h = P + Q + T(c) Wtc (2 + 2A per feature), SiLU (5), u * SiLU accumulated (2)."""
    return F * (2 + 2 * A + 5 + 2)


def flops_triplet_bwd(F, A=8):
    """Per ordered triplet, each evaluated once: h again (2 + 2A), SiLU and SiLU' (8), hbar = Sbar u SiLU' (2), sums into
    Pbar, Qbar (2), ubar (2), dT/dc Wtc (2A), its product with hbar (2)."""
    return F * (2 + 2 * A + 8 + 2 + 2 + 2 + 2 * A + 2)


def cpu_baseline(cfg_index, n_cells):
    """The oracle, as it stands, timed once on the timed system itself (n_cells = None) or on a smaller box of the
    same recipe."""
    import workloads as wl
    from oracle import _lib as ol
    from oracle import graph as og
    from oracle import model as om
    c = wl.make_config(cfg_index, n=n_cells)
    t0 = time.perf_counter()
    g = og.build_graph(c["positions"], c["cell"], c["r_cut"])
    if c["three_body"]:
        from oracle import three_body as tb
        tb.energy_forces3(c["positions"], c["cell"], c["species"], c["weights"], g, c["r_cut"], c["r_bond"], c["K"], c["p"])
    else:
        om.energy_forces(c["positions"], c["cell"], c["species"], c["weights"], g, c["r_cut"], c["K"], c["p"])
    dt = time.perf_counter() - t0
    n = len(c["species"])
    return {"value": n / dt, "unit": "atoms/s", "cores": int(ol.lib().orc_num_threads()), "kind": "oracle",
            "sample": (f"configs[{cfg_index}] itself" if n_cells is None else
                       f"configs[{cfg_index}] recipe at {n_cells}^3 fcc cells")
                      + f" ({n} atoms, {g.E} directed edges), fp64, graph + energy + forces, one run of {dt:.1f} s"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3)
    ap.add_argument("--cells", type=int, default=None, help="override fcc cells per side (smaller runs)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--cpu-cells", type=int, default=None,
                    help="fcc cells per side of a smaller sample for the oracle timing (default: the timed system itself)")
    ap.add_argument("--no-whole", action="store_true", help="skip the unpartitioned (whole-graph) run of the same system")
    ap.add_argument("--precision", choices=("f32", "f32split", "bf16"), default="f32",
                    help="f32split: the F x F products of the filter MLP as split-fp16 MFMA triples (fp32-grade results); "
                         "bf16: those products with bf16 operands (fp32 accumulation)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (slabs are processed in sequence on one device); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2506_02023_amd as M
    import workloads as wl

    c = wl.make_config(args.config, n=args.cells)
    three_body = c["three_body"]   # configs[4]: whole-graph mode (a secondary workload; the default is configs[3])
    P = 1 if three_body else max(c["n_slabs"], 2)
    torch.cuda.set_device(0)
    pos = torch.as_tensor(c["positions"], device="cuda")
    spec = torch.as_tensor(c["species"], device="cuda")
    W = M.Weights(c["weights"], c["p"], precision={"f32": 0, "bf16": 1, "f32split": 2}[args.precision])
    BW = M.BondWeights(c["weights"], c["r_bond"], c["A"]) if three_body else None
    N = pos.shape[0]
    out = (torch.empty(1, dtype=torch.float64, device="cuda"), torch.empty((N, 3), dtype=torch.float32, device="cuda"),
           None)
    g = None

    def step(mode=None):
        nonlocal g
        g = M.mlip_build_graph(pos, c["cell"], spec, c["r_cut"], n_slabs=P, graph=g)
        if three_body:
            M.mlip_forward_bonds(g, W, BW, M.MODE_WHOLE, out=out, want_atom_energy=False)
        else:
            M.mlip_forward(g, W, M.MODE_SLABS if mode is None else mode, out=out, want_atom_energy=False)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    g.profile_enable(True)
    g.profile_read(reset=True)
    torch.cuda.synchronize()
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # step boundaries, on the library's stream
    t0 = time.perf_counter()
    marks[0].record()
    for k in range(args.steps):
        step()
        marks[k + 1].record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = sorted(marks[k].elapsed_time(marks[k + 1]) for k in range(args.steps))
    prof = g.profile_read(reset=True)
    g.profile_enable(False)
    _, E, _ = g.sizes()
    energy = float(out[0].cpu()[0])
    fsum = out[1].double().sum(0).abs().max().item()

    def timed_variant(weights, n_slabs, mode):
        """The same step with other weights / slab count, outside the headline's timed region."""
        gv = None
        t1 = 0.0
        for it in range(2 + args.steps):
            if it == 2:
                torch.cuda.synchronize()
                t1 = time.perf_counter()
            gv = M.mlip_build_graph(pos, c["cell"], spec, c["r_cut"], n_slabs=n_slabs, graph=gv)
            M.mlip_forward(gv, weights, mode, out=out, want_atom_energy=False)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t1) / args.steps * 1e3
        e = float(out[0].cpu()[0])
        gv.destroy()
        return ms, e

    # for the record (not the headline): the unpartitioned run, and the split-fp16 mode of the headline's step
    whole_ms = split_ms = None
    if not three_body and not args.no_whole:
        whole_ms, energy_whole = timed_variant(W, 1, M.MODE_WHOLE)
    if args.precision == "f32" and not three_body:
        split_ms, energy_split = timed_variant(M.Weights(c["weights"], c["p"], precision=2), P, M.MODE_SLABS)

    ms_step = dt / args.steps * 1e3
    L = c["L"]
    default_workload = args.config == 3 and args.cells is None and args.precision == "f32"   # what the traffic constants were profiled on

    def edge_roofline(group, kernel, flops_edge, traffic, as_defined=None):
        ms, n = prof[group]
        per_launch = E * flops_edge * L * args.steps / max(n, 1)
        avg_ms = ms / max(n, 1)
        ach = per_launch / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0
        r = {"kernel": kernel, "bound": "mfma", "achieved": ach, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
             "frac": ach / PEAK_FP32_MFMA_TFLOPS, "traffic": traffic if default_workload else None,
             "traffic_source": TRAFFIC_SOURCE if default_workload else None,
             "avg_launch_ms": avg_ms, "launches": int(n), "flops_per_launch": per_launch,
             "ms_per_step": ms / args.steps}
        if as_defined is not None:   # rate of the operation as defined (twice the executed work), not a utilisation
            r["as_defined_tflops"] = ach * as_defined / flops_edge
            r["flops_per_edge_layer"] = {"executed": flops_edge, "as_defined": as_defined}
        if args.precision != "f32":
            r["note"] = ("the W2 products run on the 16-bit matrix pipeline; frac is the algorithmic rate against the fp32 "
                         "MFMA peak of the default mode, not a utilisation of the units used")
        return r

    F = c["F"]
    roof_bwd = edge_roofline("edge_bwd", f"k_edge_bwd<{F}> (reverse edge step)", flops_bwd_edge(F),
                             TRAFFIC_BWD_LAUNCH_BYTES, flops_bwd_edge_as_defined(F))
    two_pass = prof["edge_fwd_lower"][1] > 0   # edge kernels on the pairs' upper edges, lower edges in second passes
    if two_pass:
        roof_fwd = edge_roofline("edge_fwd", f"k_edge_fwd<{F}> on the upper-edge graphs (forward edge step, first pass)",
                                 flops_fwd_edge(F) // 2, TRAFFIC_FWD_LAUNCH_BYTES, flops_fwd_edge(F))
        # the operation as defined takes both passes: price it on their summed time
        both_ms = prof["edge_fwd"][0] + prof["edge_fwd_lower"][0]
        roof_fwd["as_defined_tflops"] = E * flops_fwd_edge(F) * L * args.steps / (both_ms * 1e-3) / 1e12
        roof_fwd["as_defined_ms_per_step"] = both_ms / args.steps
    else:
        roof_fwd = edge_roofline("edge_fwd", f"k_edge_fwd<{F}> (forward edge step)", flops_fwd_edge(F),
                                 TRAFFIC_FWD_LAUNCH_BYTES)
    if two_pass:   # the reverse operation as defined takes both of its passes
        both_ms = prof["edge_bwd"][0] + prof["edge_bwd_lower"][0]
        roof_bwd["kernel"] = f"k_edge_bwd<{F}> on the upper-edge graphs (reverse edge step, first pass)"
        roof_bwd["as_defined_tflops"] = E * flops_bwd_edge_as_defined(F) * L * args.steps / (both_ms * 1e-3) / 1e12
        roof_bwd["as_defined_ms_per_step"] = both_ms / args.steps
    roof = roof_fwd if roof_fwd["ms_per_step"] >= roof_bwd["ms_per_step"] else roof_bwd   # the dominant kernel
    roof_lower = {}
    if two_pass:   # bound by their row traffic; compulsory bytes: per lower edge the kept filter values (read once), per
                   # atom the row that is gathered (once if the caches were perfect) and the sum (read, written)
        for group, what, traffic in (("edge_fwd_lower", "forward", TRAFFIC_FWD_LOWER_LAUNCH_BYTES),
                                     ("edge_bwd_lower", "reverse", TRAFFIC_BWD_LOWER_LAUNCH_BYTES)):
            ms, n = prof[group]
            if n == 0:
                continue
            per_launch = E / 2 * F * 4 + N * 3 * F * 4
            avg_ms = ms / n
            ach = per_launch / (avg_ms * 1e-3) / 1e9 if avg_ms > 0 else 0.0
            roof_lower[group] = {"kernel": f"k_edge_lower<{F}> ({what} edge step, second pass: lower edges)", "bound": "hbm",
                                 "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                                 "traffic": traffic if default_workload else None,
                                 "traffic_source": TRAFFIC_SOURCE if default_workload else None,
                                 "avg_launch_ms": avg_ms, "launches": int(n),
                                 "bytes_per_launch": per_launch, "ms_per_step": ms / args.steps}
    roof_trip = {}
    if three_body:
        _, bptr = g.bonds()
        cnt = np.diff(bptr).astype(np.int64)
        n_triplets = int((cnt * (cnt - 1)).sum())
        for group, kernel, fl in (("triplet_fwd", f"k_triplet_fwd<{F}>", flops_triplet_fwd(F)),
                                  ("triplet_bwd", f"k_triplet_bwd<{F}>", flops_triplet_bwd(F))):
            ms, n = prof[group]
            per_launch = n_triplets * fl * args.steps / max(n, 1)
            avg_ms = ms / max(n, 1)
            ach = per_launch / (avg_ms * 1e-3) / 1e12 if avg_ms > 0 else 0.0
            roof_trip[group] = {"kernel": kernel, "bound": "alu", "achieved": ach, "peak": PEAK_FP32_VECTOR_TFLOPS,
                                "unit": "TFLOP/s", "frac": ach / PEAK_FP32_VECTOR_TFLOPS, "traffic": None,
                                "avg_launch_ms": avg_ms, "launches": int(n), "flops_per_launch": per_launch,
                                "ms_per_step": ms / args.steps, "triplets": n_triplets}
        if roof_trip["triplet_bwd"]["ms_per_step"] > roof["ms_per_step"]:
            roof = roof_trip["triplet_bwd"]

    res = {
        "metric": "atoms/s (energy+forces)", "value": N / (dt / args.steps), "unit": "atoms/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_step, "ms_per_step_min": per_step[0],
        "ms_per_step_median": per_step[len(per_step) // 2], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None,
        "dtype": {"f32": "f32", "bf16": "f32 with bf16 operands in the filter MLP's F x F products",
                  "f32split": "f32, the filter MLP's F x F products as split-fp16 MFMA triples"}[args.precision],
        "data": "synthetic",
        "config": {"workload": c["name"] + f", {N} atoms, {E} directed edges, r_cut 5.0, F={c['F']} L={L} K=8, "
                               + (f"three-body variant (bonds within {c['r_bond']}), graph build + whole-graph energy+forces"
                                  if three_body else f"graph build + {P}-slab sequential energy+forces"), "n_slabs": P},
        "edges_per_s": E / (dt / args.steps),
        "us_per_atom_step": ms_step * 1e3 / N,
        "breakdown_ms_per_step": {k: v[0] / args.steps for k, v in prof.items()},
        "energy": energy, "net_force_max_component": fsum,
        "roofline": roof, "roofline_edge_fwd": roof_fwd, "roofline_edge_bwd": roof_bwd,
    }
    for k, v in roof_trip.items():
        res["roofline_" + k] = v
    for k, v in roof_lower.items():
        res["roofline_" + k] = v
    if split_ms is not None:
        res["split_fp16_products"] = {"ms_per_step": split_ms, "value": N / (split_ms * 1e-3), "unit": "atoms/s",
                                      "energy": energy_split,
                                      "note": "MLIP_PRECISION_FP32_SPLIT: same step, W2 products as three fp16 MFMA products "
                                              "of split operands; held to the fp32 bounds by the parity tests"}
    if whole_ms is not None:
        res["whole_graph"] = {"ms_per_step": whole_ms, "value": N / (whole_ms * 1e-3), "unit": "atoms/s",
                              "energy": energy_whole, "rel_energy_difference_to_slabs": abs(energy_whole - energy) / abs(energy),
                              "note": "graph build without partition + unpartitioned energy+forces of the same system"}
    if not args.no_cpu:
        res["cpu_baseline"] = cpu_baseline(args.config, args.cpu_cells if args.cpu_cells else args.cells)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
