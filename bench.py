"""Benchmark of the fused node-centric equivariant attention forward pass on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole hot path over the scaling-point workload (one box of 10 000 atoms at
0.1 atoms/A^3, cutoff 6 A, L_max = 4, C = 128, H = 8, bf16 features with fp32 accumulation): e2f_build_cells
followed by e2f_attn_forward, inputs already resident in device memory.  Prints one JSON line with whole-job
atoms/s, the roofline figure of the dominant kernel (timed with HIP events on the launch stream by the
library's profiling hooks), the fp64 CPU oracle timed on this host, and the fused-vs-materialized comparison.
"""
import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# MI355X published peaks used for the roofline: fp32 vector 157.3 TFLOP/s
# (256 CUs x 4 SIMDs x 16 lanes x 2 (packed) x 2 (FMA) x 2.4 GHz), bf16 dense MFMA 2.5 PFLOP/s, HBM 8 TB/s.
# This build compiles with packed fp32 switched off, so what its vector code can reach is the plain-FMA figure.
PEAK_ALU_TFLOPS = 157.3
PEAK_ALU_PLAIN_FMA_TFLOPS = 78.6
TOL = {"f32": 1e-4, "bf16": 2e-2}   # relative L2 against the fp64 oracle; one atom's own row: five times that


def flop_model(cfg, N, E):
    """Algorithmic flops of the method (1 MAC = 2 flop; block-diagonal Wigner matrices, no padding counted)."""
    L, C, H, B = cfg["L"], cfg["C"], cfg["H"], cfg["B"]
    n = (L + 1) ** 2
    S2 = sum((2 * l + 1) ** 2 for l in range(L + 1))
    nnzP = sum(1 for lo in range(L + 1) for m in range(-lo, lo + 1)
               for li in (lo - 1, lo, lo + 1) if 0 <= li <= L and not (li == lo and m == 0) and abs(m) <= li) \
        if cfg["lf"] == 1 else n
    f_node = 2 * 5 * n * C * C + 2 * 2 * n * C
    f_edge = 2 * (L + 1) * C + 2 * H * B + 2 * S2 * C + 2 * nnzP * C + 2 * S2 * C + 2 * n * C
    return f_node, f_edge, N * f_node + E * f_edge


TRAFFIC_FILE = "profiles/fused_attention_scaling10k_pmc.txt"
COUNTER_FILE = "profiles/tile_attention_scaling10k_counters.txt"


def read_traffic():
    """HBM bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, if any (the counters
    need a profiler run of their own; this run does not measure them)."""
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if not os.path.exists(path):
        return None
    m = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read())
    return float(m.group(1)) if m else None


def read_counters(kernel_pattern):
    """SQ counters of one kernel from the committed rocprofv3 summary: {counter: mean per dispatch}."""
    path = os.path.join(ROOT, COUNTER_FILE)
    if not os.path.exists(path):
        return {}
    out, on = {}, False
    for line in open(path):
        if line.startswith("#"):
            continue
        if not line.startswith(" "):
            on = kernel_pattern in line
        elif on:
            parts = line.split()
            if parts[0].startswith("SQ_"):
                out[parts[0]] = float(parts[1])
    return out


def atom_errors(got, ref):
    d = np.linalg.norm((got - ref).reshape(ref.shape[0], -1), axis=1)
    r = np.linalg.norm(ref.reshape(ref.shape[0], -1), axis=1)
    return np.where(r > 0, d / np.where(r > 0, r, 1.0), d)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-materialized", action="store_true")
    ap.add_argument("--no-factorized", action="store_true")
    ap.add_argument("--workload", default="scaling", help="scaling | large | small | tiny | box<N>")
    ap.add_argument("--sweep", action="store_true",
                    help="also time the Large-N boxes (20k, 50k, 100k atoms) and fit peak activation bytes against N")
    ap.add_argument("--tp", action="store_true",
                    help="also time the stand-alone EAAS tensor product at the shape of the paper's tensor-product table")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="BYTES",
                    help="also run a plain device copy of this many bytes (reference for HBM counter scaling)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on one GPU only (the path has no multi-GPU code); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2601_16622_amd import binding as B, workloads as W
    B.load()
    assert torch.cuda.is_available(), "bench.py needs the MI355X"

    if args.copy_calibration > 0:
        src = torch.ones(args.copy_calibration // 4, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    wl = W.by_name(args.workload, 0)
    cfg = wl["cfg"]
    P = B.Problem(wl, "cuda:0")
    N = P.N

    def step():
        P.build_cells()
        P.forward()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    B.e2f_profile_begin(P.ctx, args.steps)
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]   # on the launch stream (current)
    t0 = time.perf_counter()
    ev[0].record()
    for i in range(args.steps):
        step()
        ev[i + 1].record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    timed_out = P.out.clone()   # the output of the timed region's last step: checked against the oracle below
    per_call = B.e2f_profile_read(P.ctx, args.steps)
    stage_ms, calls = B.e2f_profile_end(P.ctx)
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    step_ms_median = float(np.median([ev[i].elapsed_time(ev[i + 1]) for i in range(args.steps)]))
    attn_ms_median = float(np.median([c["attention"] for c in per_call])) if per_call else 0.0
    deg, _, _ = P.neighbors()
    E = int(deg.sum())
    f_node, f_edge, f_alg = flop_model(cfg, N, E)

    # forward alone (cells prebuilt), same protocol
    for _ in range(3):
        P.forward()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        P.forward()
    torch.cuda.synchronize()
    fwd_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    attn_ms = stage_ms["attention"]
    bf16 = cfg["dtype"] == "bf16"
    mc_ok = bf16 and cfg["C"] // cfg["H"] == 16 and cfg["L"] >= 1
    if mc_ok and cfg["lf"] == 1 and cfg["C"] in (32, 64, 128, 256) and cfg["B"] <= 16:
        kernel = "k_tile_heads"
    elif mc_ok and cfg["lf"] in (1, 2) and cfg["H"] in (1, 2, 4, 8):
        kernel = "k_fused_mfma"
    elif not bf16 and cfg["C"] // cfg["H"] == 16 and cfg["L"] >= 1 and cfg["lf"] == 1 and cfg["B"] <= 16:
        kernel = "k_tile_f32"
    else:
        kernel = "k_fused_valu"
    # Roofs of the attention kernel from the algorithmic work of the method (per pair: logits, rotate in, re-index,
    # rotate back, weighted accumulate): HBM time of the rows it must touch once, matrix-core time of the dense
    # pieces, plain-ALU time of the rest.  The largest of the three binds; `frac` is that time over the measured one.
    Lm, Cc = cfg["L"], cfg["C"]
    n = (Lm + 1) ** 2
    S2 = sum((2 * l + 1) ** 2 for l in range(Lm + 1))
    f_dense = E * (2 * (Lm + 1) * Cc + 4 * S2 * Cc)
    f_rest = E * f_edge - f_dense
    esz = 2 if bf16 else 4
    hbm_bytes = N * (16 + 2 * (Lm + 1) * Cc * 4 + n * Cc * esz + n * Cc * 4)
    peak_mfma = 2500.0 if bf16 else PEAK_ALU_TFLOPS
    roofs = {"hbm": (hbm_bytes / 8e12, hbm_bytes / 1e9, 8000.0, "GB/s"),
             "mfma": (f_dense / (peak_mfma * 1e12), f_dense / 1e12, peak_mfma, "TFLOP/s"),
             "alu": (f_rest / (PEAK_ALU_TFLOPS * 1e12), f_rest / 1e12, PEAK_ALU_TFLOPS, "TFLOP/s")}
    bound = max(roofs, key=lambda k: roofs[k][0])
    t_roof, work, peak, unit = roofs[bound]
    achieved = work / (attn_ms * 1e-3) if attn_ms > 0 else 0.0
    roofline = {"bound": bound, "kernel": kernel, "achieved": round(achieved, 3), "peak": peak, "unit": unit,
                "frac": round(achieved / peak, 4), "traffic": read_traffic(),
                "traffic_source": TRAFFIC_FILE + " (rocprofv3 FETCH_SIZE + WRITE_SIZE runs; not measured in this run)",
                "kernel_ms": round(attn_ms, 4), "kernel_ms_median": round(attn_ms_median, 4),
                "achieved_is": "the method's per-pair work of the bound (model) over the measured time of the "
                               "attention stage, not executed instructions",
                "pairs_per_launch": E,
                "algorithmic_flops_per_launch": E * f_edge,
                "algorithmic_tflops": round(E * f_edge / (attn_ms * 1e-3) / 1e12, 3) if attn_ms > 0 else 0.0,
                "work_of_bound_per_launch": work * (1e9 if bound == "hbm" else 1e12),
                "roof_ms": {k: round(v[0] * 1e3, 4) for k, v in roofs.items()},
                "stage_ms": {k: round(v, 4) for k, v in stage_ms.items()}}
    if bound == "alu":
        roofline["frac_of_plain_fma_peak"] = round(achieved / PEAK_ALU_PLAIN_FMA_TFLOPS, 4)
    if kernel == "k_tile_heads":
        # what the kernel executes (matrix-core instructions over all candidate slots, masked ones included), from the
        # committed counter summary of the same workload
        sq = read_counters("k_tile_heads<4, false, 8>")
        useful = E * cfg["H"] * (2 * (Lm + 1) * 16 + 3 * n * 16 * 2)
        if sq.get("SQ_INSTS_MFMA"):
            roofline["executed"] = {
                "source": COUNTER_FILE,
                "mfma_instructions": sq["SQ_INSTS_MFMA"], "mfma_flops_issued": sq["SQ_INSTS_MFMA"] * 16384,
                "mfma_flops_useful": useful, "valu_instructions": sq.get("SQ_INSTS_VALU"),
                # SIMD cycles the pipes were busy (the counter file's figures) over the SIMD cycles of this run's
                # kernel time (1024 SIMDs at 2.4 GHz)
                "valu_active_frac": round(sq.get("SQ_ACTIVE_INST_VALU", 0.0) * 4 / (attn_ms * 2.4e6 * 1024), 3),
                "mfma_busy_frac": round(sq.get("SQ_VALU_MFMA_BUSY_CYCLES", 0.0) / (attn_ms * 2.4e6 * 1024), 3)}

    result = {
        "metric": "atoms/sec of fused equivariant attention forward (cells + projections + attention)",
        "value": round(N / (ms_per_step * 1e-3), 1), "unit": "atoms/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median_of_events": round(step_ms_median, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16" if cfg["dtype"] == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: N={N} atoms, E={E} directed pairs, cutoff {cfg['cutoff']} A, "
                               f"L_max={cfg['L']}, C={cfg['C']}, H={cfg['H']}, B={cfg['B']}, lf={cfg['lf']}, "
                               f"{cfg['dtype']} features, fp32 accumulation"},
        "tflops": round(f_alg / (ms_per_step * 1e-3) / 1e12, 3),
        "forward_only_ms": round(fwd_ms, 4),
        "forward_only_atoms_per_s": round(N / (fwd_ms * 1e-3), 1),
        "peak_activation_bytes": P.activation_bytes(),
        "roofline": roofline,
    }

    # the same step replayed from a captured graph (the calls allocate nothing and never synchronise)
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            step()
            side.synchronize()
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.synchronize()
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        g_ms = (time.perf_counter() - t0) * 1e3 / args.steps
        result["graph_replay"] = {"ms_per_step": round(g_ms, 4), "atoms_per_s": round(N / (g_ms * 1e-3), 1)}
        del graph
    except Exception as e:   # noqa: BLE001 - a capture problem must not take the benchmark line away
        result["graph_replay"] = {"error": str(e)[:200]}

    # the paper's own factorized pipeline (node-level products around Algorithm 1) on the same inputs
    try:
        if args.no_factorized:
            raise B.E2fError(0, "skipped")
        out_f = torch.empty_like(P.out)
        for _ in range(3):
            P.forward_factorized(out_f)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        reps = 20
        for _ in range(reps):
            P.forward_factorized(out_f)
        torch.cuda.synchronize()
        fact_ms = (time.perf_counter() - t0) * 1e3 / reps
        result["factorized"] = {"ms": round(fact_ms, 4), "atoms_per_s": round(N / (fact_ms * 1e-3), 1),
                                "workspace_bytes": int(B.e2f_attn_factorized_workspace_bytes(P.ctx, N)),
                                "max_abs_diff_vs_fused": float((out_f - P.out).abs().max())}
    except B.E2fError as e:
        result["factorized"] = {"error": str(e)}

    # neighbour cap (max_neighbors of the paper's model table is 32) and the padded-table form of the call
    if not args.no_factorized:
        def timed(fn, reps=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(reps):
                fn()
            torch.cuda.synchronize()
            return (time.perf_counter() - t0) * 1e3 / reps
        out_c = torch.empty_like(P.out)
        capped = {}
        for K in (32, 64):
            ms = timed(lambda: P.forward_capped(K, out_c))
            capped[str(K)] = {"forward_ms": round(ms, 4), "atoms_per_s": round(N / (ms * 1e-3), 1)}
        table, count = P.neighbor_table(32)
        build_ms = timed(lambda: B.e2f_build_neighbor_table(P.ctx, P.cells, P.pos, 32, table, count), reps=10)
        ms = timed(lambda: P.forward_table(table, out_c), reps=10)
        result["capped"] = capped
        result["table"] = {"K": 32, "build_ms": round(build_ms, 4), "forward_ms": round(ms, 4),
                           "pairs": int(count.sum().item()),
                           "max_abs_diff_vs_capped": float((out_c - P.forward_capped(32, torch.empty_like(P.out))).abs().max())}

        # the same number of atoms at the same density in a periodic box (no surface: about a sixth more pairs)
        Pp = B.Problem(W.by_name("pbox%d" % N, 0))
        try:
            Pp.build_cells()
            deg_p = torch.zeros(N, dtype=torch.int32, device=Pp.device)
            B.e2f_count_neighbors(Pp.ctx, Pp.cells, Pp.pos, deg_p)
            step_ms = timed(lambda: (Pp.build_cells(), Pp.forward()))
            ms = timed(Pp.forward)
            result["periodic"] = {"workload": "pbox%d" % N, "pairs": int(deg_p.sum().item()),
                                  "forward_ms": round(ms, 4), "ms_per_step": round(step_ms, 4),
                                  "atoms_per_s": round(N / (step_ms * 1e-3), 1)}
        finally:
            Pp.close()

        # backward pass of the fused call (positions, q, k, v, h), same workload
        try:
            g_out = torch.randn_like(P.out)
            P.forward()
            bwd_ms = timed(lambda: P.backward(g_out), reps=10)
            bwd_core_ms = timed(lambda: P.backward(g_out, with_h=False), reps=10)
            bwd_w_ms = timed(lambda: P.backward(g_out, with_weights=True), reps=10)
            # the same call right after a forward pass that ran in its workspace (projections and lists are kept)
            P.forward(for_backward=True)
            bwd_saved_ms = timed(lambda: P.backward(g_out, after_forward=True), reps=10)
            result["backward"] = {"ms": round(bwd_ms, 4), "ms_without_grad_h": round(bwd_core_ms, 4),
                                  "ms_with_weight_gradients": round(bwd_w_ms, 4),
                                  "ms_after_forward": round(bwd_saved_ms, 4),
                                  "over_forward": round(bwd_ms / fwd_ms, 2),
                                  "after_forward_over_forward": round(bwd_saved_ms / fwd_ms, 2),
                                  "workspace_bytes": int(B.e2f_attn_backward_workspace_bytes(P.ctx, N)),
                                  "workspace_bytes_with_weight_gradients":
                                      int(B.e2f_attn_backward_weights_workspace_bytes(P.ctx, N))}
        except B.E2fError as e:
            result["backward"] = {"error": str(e)}

        # the logit with the non-linear pair feature (vector-ALU kernel), same workload
        try:
            nl_ms = timed(lambda: P.forward_nonlinear(out_c), reps=5)
            result["nonlinear_score"] = {"forward_ms": round(nl_ms, 4), "atoms_per_s": round(N / (nl_ms * 1e-3), 1),
                                         "workspace_bytes": int(B.e2f_attn_nonlinear_workspace_bytes(P.ctx, N))}
        except B.E2fError as e:
            result["nonlinear_score"] = {"error": str(e)}

    if not args.no_materialized:
        try:
            out_m = torch.empty_like(P.out)
            P.forward_materialized(out_m)
            torch.cuda.synchronize()
            reps = 3
            B.e2f_profile_begin(P.ctx, reps)
            t0 = time.perf_counter()
            for _ in range(reps):
                _, peak = P.forward_materialized(out_m)
            torch.cuda.synchronize()
            mat_ms = (time.perf_counter() - t0) * 1e3 / reps
            # the baseline's kernels alone (HIP events inside the call: node-level kernels + edge kernels, without the
            # allocation of the edge tensors and the host synchronisation between them), and the whole call
            mat_stage, _ = B.e2f_profile_end(P.ctx)
            mat_kernels = mat_stage["prepare"] + mat_stage["attention"]
            result["materialized"] = {"ms_kernels": round(mat_kernels, 3), "ms_call": round(mat_ms, 3),
                                      "ms_alloc_and_sync": round(mat_stage["project"], 3),
                                      "peak_bytes": int(peak) + P.activation_bytes(),
                                      "fused_speedup": round(mat_kernels / fwd_ms, 2),
                                      "fused_speedup_is": "materialized kernels / fused forward (kernels only)",
                                      "memory_ratio": round((peak + P.activation_bytes()) / P.activation_bytes(), 1)}
        except B.E2fError as e:
            result["materialized"] = {"error": str(e)}

    if not args.no_cpu_baseline:
        import oracle
        nbr = oracle.neighbor_list(wl["pos"], wl["seg"], np.float32(cfg["cutoff"]), use_cells=True)
        n_t = min(N, 10_000)
        targets = None if n_t == N else np.random.default_rng(0).choice(N, n_t, replace=False).astype(np.int32)
        t0 = time.perf_counter()
        ref = oracle.attn_forward(cfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], targets=targets, nbr=nbr)
        dt = time.perf_counter() - t0
        # the output of the timed region against what the oracle just computed, over the same targets
        got = timed_out.cpu().numpy().astype(np.float64)
        got = got if targets is None else got[targets]
        per_atom = atom_errors(got, ref)
        tol = TOL["bf16" if bf16 else "f32"]
        parity = {"rel_l2": float(np.linalg.norm(got - ref) / np.linalg.norm(ref)),
                  "max_atom_rel_err": float(per_atom.max()), "worst_atom": int(np.argmax(per_atom)),
                  "targets": int(ref.shape[0]), "tolerance": tol, "atom_tolerance": 5 * tol,
                  "finite": bool(np.isfinite(got).all())}
        parity["ok"] = bool(parity["finite"] and parity["rel_l2"] <= tol and parity["max_atom_rel_err"] <= 5 * tol)
        result["parity"] = parity
        result["cpu_baseline"] = {"value": round(n_t / dt, 1), "unit": "atoms/s", "cores": oracle.num_threads(),
                                  "kind": "oracle",
                                  "sample": f"{n_t} of {N} target atoms of the same workload, fp64 dense-CG route, "
                                            f"{dt:.1f} s wall"}
        # the same oracle on one thread, a smaller sample of targets
        all_threads = oracle.num_threads()
        n_1 = min(N, 400)
        t_1 = np.random.default_rng(1).choice(N, n_1, replace=False).astype(np.int32)
        oracle.set_num_threads(1)
        t0 = time.perf_counter()
        oracle.attn_forward(cfg, wl["pos"], wl["h"], wl["seg"], wl["weights"], targets=t_1, nbr=nbr)
        dt1 = time.perf_counter() - t0
        oracle.set_num_threads(all_threads)
        result["cpu_baseline_1thread"] = {"value": round(n_1 / dt1, 1), "unit": "atoms/s", "cores": 1, "kind": "oracle",
                                          "sample": f"{n_1} of {N} target atoms, {dt1:.1f} s wall"}
    P.close()

    if args.tp:
        # (128x0e+128x1e+128x2e) (x) (1x2e), fp32, 1k..32k products; paper's numbers are from an NVIDIA H20
        paper_ms = {1000: 0.15, 2000: 0.22, 4000: 0.35, 8000: 0.65, 16000: 1.20, 32000: 2.25}
        ctx = B.e2f_create(2, 128, 1, 1, 2, 1.0, "f32")
        rows = []
        for T in sorted(paper_ms):
            ht = torch.randn((T, 9, 128), dtype=torch.float32, device="cuda:0")
            rt = torch.randn((T, 3), dtype=torch.float32, device="cuda:0")
            wt = torch.rand((3, 3), dtype=torch.float32, device="cuda:0") + 0.5
            ot = torch.empty_like(ht)
            for _ in range(10):
                B.e2f_eaas_tensor_product(ctx, ht, rt, wt, ot)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(50):
                B.e2f_eaas_tensor_product(ctx, ht, rt, wt, ot)
            torch.cuda.synchronize()
            ms = (time.perf_counter() - t0) * 1e3 / 50
            nbytes = T * (9 * 128 * 4 * 2 + 12)
            rows.append({"T": T, "ms": round(ms, 4), "GB_per_s": round(nbytes / ms / 1e6, 1),
                         "paper_H20_ms": paper_ms[T]})
        B.e2f_destroy(ctx)
        result["eaas_tensor_product"] = {"shape": "(128x0e+128x1e+128x2e) x (1x2e), fp32", "bound": "hbm",
                                         "peak_GB_per_s": 8000, "rows": rows}

    if args.sweep:
        rows = [{"N": N, "forward_ms": round(fwd_ms, 4), "step_ms": round(ms_per_step, 4),
                 "peak_activation_bytes": result["peak_activation_bytes"], "pairs": E}]
        fcc_rows = []
        # boxes of the Large-N regime, then the FCC-subsample systems of the paper's inference-scaling experiment
        for kind, n_atoms in (("box", 20_000), ("box", 50_000), ("box", 100_000),
                              ("fcc", 1_000), ("fcc", 10_000), ("fcc", 50_000), ("fcc", 100_000)):
            wl2 = W.box(n_atoms, 0) if kind == "box" else W.fcc_subsample(n_atoms, 0)
            P2 = B.Problem(wl2, "cuda:0")
            for _ in range(3):
                P2.build_cells()
                P2.forward()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(10):
                P2.build_cells()
                P2.forward()
            torch.cuda.synchronize()
            step2 = (time.perf_counter() - t0) * 1e2
            t0 = time.perf_counter()
            for _ in range(10):
                P2.forward()
            torch.cuda.synchronize()
            fwd2 = (time.perf_counter() - t0) * 1e2
            deg2, _, _ = P2.neighbors()
            row = {"N": n_atoms, "forward_ms": round(fwd2, 4), "step_ms": round(step2, 4),
                   "peak_activation_bytes": P2.activation_bytes(), "pairs": int(deg2.sum())}
            if kind == "fcc":   # with the model's max_neighbors = 32 as well
                outc = torch.empty_like(P2.out)
                for _ in range(3):
                    P2.forward_capped(32, outc)
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(10):
                    P2.forward_capped(32, outc)
                torch.cuda.synchronize()
                row["forward_capped32_ms"] = round((time.perf_counter() - t0) * 1e2, 4)
                row["atoms_per_s"] = round(n_atoms / (step2 * 1e-3), 1)
                fcc_rows.append(row)
            else:
                rows.append(row)
            P2.close()
            del P2, wl2
        result["fcc_subsample"] = {"rows": fcc_rows, "recipe": "FCC supercell a=3.8 A, N sites drawn without replacement, "
                                                               "cutoff 6 A, no periodic images"}
        xs = np.array([r["N"] for r in rows], dtype=np.float64)
        ys = np.array([r["peak_activation_bytes"] for r in rows], dtype=np.float64)
        slope, icpt = np.polyfit(xs, ys, 1)
        r2 = 1.0 - np.sum((ys - (slope * xs + icpt)) ** 2) / np.sum((ys - ys.mean()) ** 2)
        result["large_n"] = {"rows": rows, "bytes_per_atom": round(float(slope), 2), "intercept_bytes": round(float(icpt), 1),
                             "r2": round(float(r2), 8)}
    print(json.dumps(result))
    if result.get("parity") is not None and not result["parity"]["ok"]:
        print("bench.py: the timed output does not match the oracle: %r" % (result["parity"],), file=sys.stderr)
        sys.exit(1)


if __name__ == "__main__":
    main()
