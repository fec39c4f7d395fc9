#!/usr/bin/env python3
"""Benchmark: triplets/sec of the interaction-block stack, forward + backward, on one MI355X.

A step is one forward + backward pass of all blocks of the workload over one batch of
synthetic structures (graph construction and basis evaluation happen once, before the timed
region, and are reported separately).  For the force workload (cfg5) a step is energy forward,
backward and the force assembly.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# mfma_f32x3: fp32 GEMMs computed as six bf16 plane products per fp32 product (operands split into three bf16 planes):
# the ceiling of their fp32-equivalent rate is a sixth of the bf16 matrix-core peak
PEAK = {"hbm": (8000.0, "GB/s"), "mfma_f32": (157.3, "TFLOP/s"), "mfma_bf16": (2500.0, "TFLOP/s"),
        "mfma_f32x3": (round(2500.0 / 6.0, 1), "TFLOP/s"), "alu_f32": (78.6, "TFLOP/s")}
ALU_KERNELS = ("tripD_fwd", "tripD_bwd", "tripG_fwd", "trip_bwd_H", "tripG_grad_cos", "tripG_edge")


def measured_traffic(workload, modified):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary of this workload, if any
    (profiles/block_<variant>_<workload>_hbm_traffic.md; counters cannot be read from inside the run).
    Nothing for a run whose flags change the workload: the summaries cover the plain workloads only."""
    path = os.path.join(ROOT, "profiles", "block_%s_%s_hbm_traffic.md" % (workload.dims.variant, workload.name))
    out = {}
    if os.path.exists(path) and not modified:
        for line in open(path):
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            if len(cells) == 5 and cells[1].isdigit():
                out[cells[0]] = (float(cells[2]) + float(cells[3])) * 1024.0
    return out


def sample_system(workload, seed):
    """A bounded sample of the workload for the CPU oracle: fewer structures of the same recipe, or
    (single-structure workloads) a smaller box at the same density and cutoff."""
    import synth
    args = list(workload.system_args)
    if workload.system == "slab":
        args[0] = max(1, args[0] // 2) if workload.dims.variant == "D" else 1
        return synth.slab_adsorbate_positions(*args, seed=seed), "%d of %d structures" % (args[0], workload.system_args[0])
    if workload.system == "box":
        # the oracle keeps 16 KB per triplet and block for its reverse pass: 100 atoms (about 1e6 triplets) for one
        # block, 80 atoms for the three blocks of the force workload
        args[0] = 80 if workload.head_hidden else 100
        return synth.box_positions(*args, seed=seed), "%d-atom box at the same density and cutoff (workload: %d atoms)" % (
            args[0], workload.system_args[0])
    return synth.make_positions(workload, seed), "whole workload"


def cpu_baseline(workload, seed):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    import torch

    import synth
    from oracle import energy as oenergy
    from tests import helpers as H

    dims = workload.dims
    (pos, gptr), what = sample_system(workload, seed)
    g = H.oracle_graph(pos, gptr, dims.cutoff, workload.max_neighbors)
    E, T = len(g["src"]), len(g["idx_kj"])
    m, gup = synth.edge_embeddings(E, dims.emb, seed=seed + 7)
    if dims.variant == "D":
        ob = H.oracle_basis_D(pos, g, dims)
        W_list = [synth.weights_D(dims, seed=100 + b) for b in range(workload.n_blocks)]
        run = lambda: H.oracle_stack_D(g, ob, dims, W_list, m, gup)
    elif workload.head_hidden == 0:
        ob = H.oracle_basis_G(pos, g, dims)
        W_list = [synth.weights_G(dims, seed=100 + b) for b in range(workload.n_blocks)]
        run = lambda: H.oracle_stack_G(g, ob, dims, W_list, m, gup)
    else:
        W_list = [H.t64(synth.weights_G(dims, seed=100 + b)) for b in range(workload.n_blocks)]
        Wh = H.t64(synth.weights_head(dims.emb, workload.head_hidden, seed=99))
        m64 = torch.tensor(m, dtype=torch.float64)
        run = lambda: oenergy.forces(oenergy.energy_G, pos, g["src"], g["dst"], g["idx_kj"], g["idx_ji"], m64, W_list, Wh, dims)
    reps, dt, last = 0, 0.0, None
    while reps < 1 or (dt < 10.0 and reps < 8):      # about 10-30 s of CPU work in total
        t0 = time.perf_counter()
        last = run()
        dt += time.perf_counter() - t0
        reps += 1
    res = {"value": T * workload.n_blocks * reps / dt, "unit": "triplets/s", "cores": torch.get_num_threads(),
           "kind": "oracle",
           "sample": "%s (%d edges, %d triplets), %d blocks fwd+bwd in fp64, %d passes, %.1f s"
                     % (what, E, T, workload.n_blocks, reps, dt)}
    extra = None
    if workload.head_hidden:
        # force workload: the oracle's forces on the sample are also the reference for the library's forces there
        extra = force_check(workload, seed, pos, gptr, m, last, what)
    return res, extra


def force_check(workload, seed, pos, gptr, m, oracle_result, what):
    """The library's energy and forces for the sample structure the oracle has just been timed on (same model:
    blocks, widths, head, bf16 GEMM operands, matrix-core triplet kernels as at full size) against the oracle's."""
    import numpy as np
    import torch

    import paper_2203_09697_amd as gp
    import synth
    from paper_2203_09697_amd.binding_e import ForceModelG
    dims = workload.dims
    _e_ref, f_ref = oracle_result
    ctx = gp.Context(0)
    gp.gp_set_triplet_mfma(ctx, 1)
    dptr = torch.as_tensor(gptr).to("cuda:0")
    e, t = gp.build_graph(ctx, torch.as_tensor(pos).to("cuda:0"), dptr, dims.cutoff, workload.max_neighbors)
    basis = gp.gp_basis_forward(ctx, dims, e, t)
    W_list = [gp.weights_to_device(synth.weights_G(dims, seed=100 + b)) for b in range(workload.n_blocks)]
    Wh = gp.weights_to_device(synth.weights_head(dims.emb, workload.head_hidden, seed=99))
    model = ForceModelG(ctx, dims, W_list, Wh, workload.head_hidden, e, t, basis, dptr)
    en, f = model.energy_and_forces(torch.as_tensor(m).to("cuda:0"))
    torch.cuda.synchronize()
    f = f.cpu().numpy().astype(np.float64)
    return {"sample": what, "n_edges": e["n_edges"], "n_triplets": t["n_triplets"],
            "force_max_abs_error": float(np.abs(f - f_ref).max()), "force_max_abs": float(np.abs(f_ref).max()),
            "force_rel_l2": float(np.linalg.norm(f - f_ref) / np.linalg.norm(f_ref))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4",
                    help="cfg4 (default): the largest single-GPU configuration, 1000 atoms, 3e5 edges, 1e8 triplets, the "
                         "paper's large-model widths; cfg1..cfg3 are the smaller parity cases, cfg5 the force-training step")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--all-kernels", action="store_true", help="list every kernel of the step, not only the ten longest")
    ap.add_argument("--radial-at-target", action="store_true",
                    help="variant-G workloads: radial factor of the triplet basis at the target edge")
    ap.add_argument("--symmetric", action="store_true",
                    help="variant-G workloads: symmetric message passing (second up-projection gathered from the opposite edge)")
    ap.add_argument("--output-blocks", action="store_true",
                    help="variant-D workloads: add an output block (out_emb 256, 3 layers) after every interaction "
                         "block and differentiate the summed energies instead of a random upstream gradient")
    ap.add_argument("--trip-mode", type=int, default=-1, choices=[-1, 0, 1, 2, 3],
                    help="variant-G triplet kernels: -1 the library's own choice, 0 per-edge vector kernels, 1 matrix-core "
                         "kernels per centre atom, 2 the two-kernel forward and whole-atom backward forms, 3 the one-pass "
                         "forward kernel with y evaluated on the vector units")
    ap.add_argument("--f32-gemm", choices=["split", "native"], default="split",
                    help="fp32 GEMMs: operands split into three bf16 planes on the bf16 matrix cores (the library's default), or "
                         "the fp32-operand matrix-core instruction")
    ap.add_argument("--no-side-stream", action="store_true", help="weight-gradient GEMMs on the launch stream")
    ap.add_argument("--calib-copy", action="store_true",
                    help="run one 256 MiB device copy first (known traffic, to scale rocprofv3 byte counters)")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py: this build runs the interaction block on ONE GPU (no sharding, no collectives); "
                 "--gpus %d is not supported" % a.gpus)

    import torch

    import paper_2203_09697_amd as gp
    import synth
    from paper_2203_09697_amd.binding_e import ForceModelG
    from paper_2203_09697_amd.binding_g import StackG
    from paper_2203_09697_amd.stack import StackD

    opts = {k: True for k, on in (("radial_at_target", a.radial_at_target), ("symmetric", a.symmetric)) if on}
    w = synth.get_workload(a.workload, **opts)
    dims = w.dims
    if opts and dims.variant != "G":
        sys.exit("bench.py: --radial-at-target / --symmetric apply to the variant-G workloads (cfg3, cfg4, cfg5)")
    pos, gptr = synth.make_positions(w, a.seed)
    ctx = gp.Context(0)
    if a.trip_mode >= 0:
        gp.gp_set_triplet_mfma(ctx, a.trip_mode)
    if a.no_side_stream:
        gp.gp_set_side_stream(ctx, False)
    if a.f32_gemm == "native":
        gp.gp_set_f32_gemm(ctx, False)
    dpos = torch.as_tensor(pos).to("cuda:0")
    dptr = torch.as_tensor(gptr).to("cuda:0")

    # graph + basis: once per batch, outside the timed region (reported separately)
    gp.build_graph(ctx, dpos, dptr, dims.cutoff, w.max_neighbors)  # warm-up of the graph kernels
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e, t = gp.build_graph(ctx, dpos, dptr, dims.cutoff, w.max_neighbors)
    torch.cuda.synchronize()
    graph_ms = (time.perf_counter() - t0) * 1e3
    t0 = time.perf_counter()
    basis = gp.gp_basis_forward(ctx, dims, e, t)
    torch.cuda.synchronize()
    basis_ms = (time.perf_counter() - t0) * 1e3
    E, T = e["n_edges"], t["n_triplets"]

    m, gup = synth.edge_embeddings(E, dims.emb, seed=a.seed + 7)
    dm, dg = torch.as_tensor(m).to("cuda:0"), torch.as_tensor(gup).to("cuda:0")
    del m, gup
    if dims.variant == "D":
        W_list = [gp.weights_to_device(synth.weights_D(dims, seed=100 + b)) for b in range(w.n_blocks)]
        if a.output_blocks:
            from paper_2203_09697_amd.binding_o import ModelD
            Wo = [gp.weights_to_device(synth.weights_out(dims.emb, 256, dims.num_radial, 3, seed=200 + b))
                  for b in range(w.n_blocks)]
            modelD = ModelD(ctx, dims, W_list, Wo, e, t, basis, dptr)
            gE = torch.ones(len(gptr) - 1, dtype=torch.float32, device="cuda:0")
        else:
            stack = StackD(ctx, dims, W_list, t, basis)
    else:
        W_list = [gp.weights_to_device(synth.weights_G(dims, seed=100 + b)) for b in range(w.n_blocks)]
        if w.head_hidden:
            Wh = gp.weights_to_device(synth.weights_head(dims.emb, w.head_hidden, seed=99))
            model = ForceModelG(ctx, dims, W_list, Wh, w.head_hidden, e, t, basis, dptr)
        else:
            stack = StackG(ctx, dims, W_list, t, basis)

    if a.output_blocks and dims.variant != "D":
        sys.exit("bench.py: --output-blocks is implemented for the variant-D workloads (cfg1, cfg2)")
    if a.output_blocks:
        def step():
            modelD.forward(dm)
            modelD.backward(gE)
    elif w.head_hidden:
        def step():
            model.energy_and_forces(dm)
    else:
        def step():
            stack.forward(dm)
            stack.backward(dg)

    if a.calib_copy:
        src_c = torch.empty(64 * 1024 * 1024, dtype=torch.float32, device="cuda:0").normal_()
        dst_c = torch.empty_like(src_c)
        dst_c.copy_(src_c)
        torch.cuda.synchronize()
        del src_c, dst_c
    for _ in range(a.warmup):
        step()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(a.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ms_per_step = ev0.elapsed_time(ev1) / a.steps
    value = T * w.n_blocks / (ms_per_step * 1e-3)

    # per-kernel durations: the same steps again with every launch bracketed by HIP events, all on
    # one stream (with the side stream on, two kernels overlap and a launch has no duration of its own)
    prof_steps = min(a.steps, 5)
    gp.gp_set_side_stream(ctx, False)
    gp.gp_profile_enable(ctx, True)
    gp.gp_profile_reset(ctx)
    for _ in range(prof_steps):
        step()
    torch.cuda.synchronize()
    prof = gp.gp_profile_collect(ctx)
    gp.gp_profile_enable(ctx, False)
    gp.gp_set_side_stream(ctx, True)
    kernels = []
    for name, d in sorted(prof.items(), key=lambda kv: -kv[1]["ms"]):
        per_launch_ms = d["ms"] / d["launches"]
        if name.startswith("gemm_f32x3"):
            ach, (peak, unit), bound = d["flops"] / (d["ms"] * 1e-3) / 1e12, PEAK["mfma_f32x3"], "mfma"
        elif name.startswith(("gemm_f32", "tripD_mfma")):
            ach, (peak, unit), bound = d["flops"] / (d["ms"] * 1e-3) / 1e12, PEAK["mfma_f32"], "mfma"
        elif name.startswith(("gemm_bf16", "tripG_mfma")):
            ach, (peak, unit), bound = d["flops"] / (d["ms"] * 1e-3) / 1e12, PEAK["mfma_bf16"], "mfma"
        elif name.startswith(ALU_KERNELS):
            ach, (peak, unit), bound = d["flops"] / (d["ms"] * 1e-3) / 1e12, PEAK["alu_f32"], "alu"
        else:
            ach, (peak, unit), bound = d["bytes"] / (d["ms"] * 1e-3) / 1e9, PEAK["hbm"], "hbm"
        kernels.append({"kernel": name, "launches_per_step": d["launches"] / prof_steps, "avg_ms": round(per_launch_ms, 5),
                        "ms_per_step": round(d["ms"] / prof_steps, 4), "bound": bound, "achieved": round(ach, 3),
                        "peak": peak, "unit": unit, "frac": round(ach / peak, 4)})
    # the same fractions against rates measured on this GPU (copy kernel, register-resident MFMA chains)
    mp = gp.gp_measure_peaks(ctx)
    measured = {"hbm": mp["copy_GBps"], "mfma_f32": mp["mfma_f32_TFLOPs"], "mfma_bf16": mp["mfma_bf16_TFLOPs"],
                "mfma_f32x3": mp["mfma_bf16_TFLOPs"] / 6.0}
    for k in kernels:
        key = "hbm" if k["bound"] == "hbm" else ("mfma_bf16" if k["peak"] == PEAK["mfma_bf16"][0] else
                                                  "mfma_f32x3" if k["peak"] == PEAK["mfma_f32x3"][0] else
                                                  "mfma_f32" if k["bound"] == "mfma" else None)
        k["frac_of_measured"] = round(k["achieved"] / measured[key], 4) if key else None
    top = kernels[0]
    traffic = measured_traffic(w, bool(opts) or a.output_blocks or a.trip_mode >= 0 or a.no_side_stream or a.f32_gemm != "split")
    for k in kernels:
        k["traffic"] = traffic.get(k["kernel"])
    roofline = {"kernel": top["kernel"], "bound": top["bound"], "achieved": top["achieved"], "peak": top["peak"],
                "unit": top["unit"], "frac": top["frac"], "frac_of_measured": top["frac_of_measured"], "avg_ms": top["avg_ms"],
                "traffic": top["traffic"]}

    # second roofline entry: the TripletUpdate + TripletAggr kernels of the forward pass taken together (they move the
    # per-triplet data), as effective HBM rate = algorithmic bytes / their time.  Algorithmic bytes of the bilinear form
    # with the accumulator materialised: 12 B per triplet (cos alpha and the two edge indices), the accumulator A as
    # stored, the gathered rows x once and the radial table once; of the Hadamard form with the basis projection fused:
    # 8 B per triplet (cos alpha, source-edge index), x and the radial table once, the aggregate once.
    trip_names = ("tripG_y", "tripG_mfma_fwd", "tripG_pack", "tripG_fused_fwd", "tripG_fwd", "tripD_mfma_fwd", "tripD_fwd")
    tk = [k for k in kernels if k["kernel"] in trip_names]
    roofline_triplet = None
    if tk:
        F, S = dims.int_emb, dims.num_spherical
        if dims.variant == "G":
            a_bytes = 2.0 if any(k["kernel"] in ("tripG_mfma_fwd", "tripG_fused_fwd") for k in tk) else 4.0
            alg = 12.0 * T + E * (4.0 * F + a_bytes * dims.emb_cbf * F + 4.0 * S * dims.emb_cbf)
        else:
            alg = 8.0 * T + E * (4.0 * F + 4.0 * F + 4.0 * S * dims.basis_emb)
        per_block_ms = sum(k["ms_per_step"] for k in tk) / w.n_blocks
        tr = [k["traffic"] for k in tk]
        roofline_triplet = {"kernels": [k["kernel"] for k in tk], "bound": "hbm", "achieved": round(alg / (per_block_ms * 1e-3) / 1e9, 1),
                            "peak": PEAK["hbm"][0], "unit": "GB/s", "frac": round(alg / (per_block_ms * 1e-3) / 1e9 / PEAK["hbm"][0], 4),
                            "algorithmic_bytes": alg, "ms_per_block": round(per_block_ms, 4),
                            "traffic": sum(tr) if all(x is not None for x in tr) else None}

    out = {
        "metric": "triplets/sec (interaction block fwd+bwd), 1 MI355X", "value": value, "unit": "triplets/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_per_step, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": dims.dtype, "data": "synthetic",
        "config": {"workload": "%s: %d structures, N=%d atoms, E=%d edges, T=%d triplets, %d blocks, variant %s, "
                               "emb=%d int_emb=%d%s" % (w.name, len(gptr) - 1, len(pos), E, T, w.n_blocks, dims.variant,
                                                        dims.emb, dims.int_emb, ", energy head + forces" if w.head_hidden else
                                                        ", output block per interaction block" if a.output_blocks else
                                                        (", radial factor at the target edge" if a.radial_at_target else "") +
                                                        (", symmetric messages" if a.symmetric else "")),
                   "cutoff": dims.cutoff, "max_neighbors": w.max_neighbors, "seed": a.seed,
                   "f32_gemm": "three bf16 planes per operand, six products, fp32 accumulation (error as fp32)" if a.f32_gemm == "split"
                               else "fp32-operand matrix-core instruction"},
        "roofline": roofline,
        "roofline_triplet": roofline_triplet,
        "measured_peaks": {k: round(v, 1) for k, v in mp.items()},
        "kernels": kernels if a.all_kernels else kernels[:10],
        "graph_build_ms": round(graph_ms, 3), "basis_ms": round(basis_ms, 3), "wall_ms_per_step": round(wall_ms / a.steps, 4),
    }
    if not a.no_cpu_baseline:
        out["cpu_baseline"], fc = cpu_baseline(w, a.seed)
        if fc is not None:
            out["force_check"] = fc
    print(json.dumps(out))


if __name__ == "__main__":
    main()
