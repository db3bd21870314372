#!/usr/bin/env python3
"""Benchmark of the exact-kNN hot path on one MI355X.

One "step" = one whole all-pairs kNN (norm prologue + fused distance/selection
kernel + finalize) over the synthetic workload, inputs already resident in HBM.
Prints ONE JSON line: whole-job throughput in pair-distances per second
(top-k included), the roofline of the dominant kernel (fp32 MFMA), and the CPU
oracle timed on a bounded sample of the same workload on this machine's host cores.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 3] [--n N]
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_F32_PEAK_TFLOPS = 157.3      # MI355X published dense fp32 matrix peak
MFMA_BF16_PEAK_TFLOPS = 2500.0    # ... and the dense bf16 one (the split-precision experiment's instruction)
# Vector-ALU ceiling for the fold kernel: its arithmetic is one subtract and one add (or max)
# per coordinate and pair -- single-flop instructions that cannot fuse into FMAs.  The published
# 157.3 TFLOP/s fp32 vector figure is 256 CUs x 4 SIMDs x 32 lanes per clock x 2 flop (FMA) x
# 2.4 GHz; one flop per instruction gives half of it.  (A lone wave issues every 4th cycle, 16
# lanes per clock; two or more waves of a SIMD reach the 32, measured by knn_valu_calibration.)
VALU_F32_PLAIN_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12

# HBM bytes per step of the dominant kernel, measured OFFLINE (two rocprofv3 --pmc runs of this
# script, FETCH_SIZE then WRITE_SIZE, scaled by what the same counters read for a 1 GiB copy
# kernel).  Keyed by (workload, kernel); each entry names the summary under profiles/ that
# holds the run.  Reported per launch next to `achieved`; null for anything not listed.
OFFLINE_TRAFFIC_BYTES_PER_STEP = {
    ("c3_lowrank32_n1048576_d256_k10", "knn_dist_qreg"):
        (3.326e11 + 4.864e11, "profiles/knn_two_phase_c3_panel_pairs.md"),
    ("c3_lowrank32_n1048576_d256_k10", "knn_pairs_qreg"):
        (5.83e12 + 3.01e10, "profiles/knn_c3_registers_resident.md"),
    ("c3_lowrank32_n1048576_d256_k10", "knn_tiles_qreg"):
        (5.85e12 + 1.59e9, "profiles/knn_c3_registers_resident.md"),
    ("paper_table1_n80000_d256_k100_hellinger", "knn_dist_qreg"):
        (1.24e10 + 2.68e10, "profiles/knn_two_phase_table1_shapes.md"),
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", type=int, default=3, help="workload 1..8 (3 = the headline one; 7 = Manhattan on the vector ALUs, "
                         "8 = Kullback-Leibler)")
    ap.add_argument("--n", type=int, default=None, help="shrink the workload (testing only)")
    ap.add_argument("--symmetric", type=int, default=0, help="0 auto, 1 triangle, 2 full square")
    ap.add_argument("--variant", type=int, default=0, help="plan: 0 auto, 1 fused streaming, 3 fused with the query operands in registers, 4 two-phase, "
                         "6 the split-precision (bf16 pieces) experiment")
    ap.add_argument("--no-fused-legs", dest="fused_legs", action="store_false",
                    help="skip the extra timing of the fused plans when the default plan is two-phase")
    ap.add_argument("--block-rows", type=int, default=0, help="symmetric schedule: rows per block")
    ap.add_argument("--oracle-rows", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-select", action="store_true", help="skip the stand-alone selection timing")
    ap.add_argument("--calibrate-contraction", action="store_true",
                    help="instead of a workload: time the contraction-only kernel for both fp32 matrix instructions "
                         "and 16 / 32 / 64 coordinates per LDS step (the evidence behind those two design choices)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch one plain elementwise copy of 1 GiB (for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (the path shards by query rows with no "
              "exchange; no multi-GPU run is part of it). Use --gpus 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_0906_0231_amd import knn_build, knn_search, knn_workspace_bytes, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path to time.", file=sys.stderr)
        return 2
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)

    if args.calibrate_contraction:
        from paper_0906_0231_amd import knn_contraction_calibration
        rows = []
        for shape, name in ((0, "v_mfma_f32_32x32x2_f32"), (1, "v_mfma_f32_16x16x4_f32")):
            for dc in (16, 32, 64):
                knn_contraction_calibration(shape, dc, 256)
                tf, ms = knn_contraction_calibration(shape, dc, 4096)
                rows.append({"instruction": name, "coordinates_per_step": dc, "tflops": tf, "ms": ms,
                             "frac": tf / MFMA_F32_PEAK_TFLOPS, "kernel": f"contract_only<{shape}, {dc}>"})
        print(json.dumps({"contraction_calibration": rows, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                          "workload": "2 workgroups per CU x 4096 tiles of 128 queries x 64 references x 256 coordinates"}))
        return 0

    t0 = time.time()
    w = workloads.config(args.config, n=args.n)
    R = w.R.to(dev)
    Q = R if w.symmetric else R[:w.nq]
    nq, nr, d, k = w.nq, w.n, w.d, w.k
    gen_s = time.time() - t0

    idx = torch.empty((nq, k), dtype=torch.int32, device=dev)
    dist = torch.empty((nq, k), dtype=torch.float32, device=dev)

    def time_plan(symmetric, variant, block_rows, steps, warmup):
        """`warmup` untimed calls, then `steps` calls timed as the ABI promises them -- enqueued
        without waiting, one synchronisation at each end -- then ONE more call with a profile
        record, whose HIP events around the kernels (on the launch stream, inside the library)
        give the dominant kernel's time per launch."""
        ws = torch.empty(knn_workspace_bytes(nq, nr, d, k, w.metric, symmetric=w.symmetric, variant=variant,
                                             schedule=symmetric, block_rows=block_rows),
                         dtype=torch.uint8, device=dev)

        def step(profile):
            if w.symmetric:
                return knn_build(R, k, w.metric, symmetric=symmetric, variant=variant, block_rows=block_rows,
                                 profile=profile, workspace=ws, out=(idx, dist))
            return knn_search(Q, R, k, w.metric, self_offset=w.self_offset, variant=variant,
                              profile=profile, workspace=ws, out=(idx, dist))

        for _ in range(warmup):
            step(False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            res = step(False)
        torch.cuda.synchronize()
        ms_per_step = 1e3 * (time.perf_counter() - t0) / steps
        res = step(True)
        plan, prof = res.plan, res.profile
        kernel = plan.kernel.decode()
        if plan.two_phase == 1:
            # matrix written out, then selected from: the dominant kernel is the one that writes it
            launches = 1
            kern_ms = prof.ms_main - prof.ms_select
        elif plan.two_phase == 2:
            # by pairs of row panels: one distance launch per pair (the library brackets each with
            # events), the selections after it.  G panels: G(G+1)/2 distance launches
            G = int(round((-1.0 + (1.0 + 24.0 * plan.main_launches) ** 0.5) / 6.0))
            launches = G * (G + 1) // 2
            kern_ms = (prof.ms_main - prof.ms_select) / launches
        else:
            launches = max(1, plan.main_launches)
            kern_ms = prof.ms_main / launches
        work_per_launch = 2.0 * d * prof.pairs_computed / launches      # flop (matrix path) or lane operations (fold)
        if plan.plan == 6:
            work_per_launch *= 3.0                                      # three bf16 products per pair and coordinate
        achieved = work_per_launch / (kern_ms * 1e-3) / 1e12
        del ws
        return {"ms_per_step": ms_per_step, "kernel": kernel, "launches": launches, "kern_ms": kern_ms,
                "achieved": achieved, "pairs_computed": int(prof.pairs_computed), "symmetric": int(plan.symmetric),
                "two_phase": int(plan.two_phase), "main_ms": float(prof.ms_main), "select_ms": float(prof.ms_select),
                "workspace_bytes": int(plan.workspace_bytes)}

    t = time_plan(args.symmetric, args.variant, args.block_rows, args.steps, args.warmup)
    ms_per_step = t["ms_per_step"]
    two_phase, symmetric, launches, kern_ms, achieved = t["two_phase"], t["symmetric"], t["launches"], t["kern_ms"], t["achieved"]
    pairs_served = float(nq) * float(nr)
    value = pairs_served / (ms_per_step * 1e-3)
    schedule = {0: "", 1: "two-phase ", 2: "two-phase by panel pairs, "}[two_phase] + ("each pair once" if symmetric else "full square")

    out = {
        "metric": "pair-distances/sec incl. top-k",
        "value": value,
        "unit": "pairs/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "nq": nq, "nr": nr, "d": d, "k": k, "metric": w.metric,
                   "value_counts": "pairs served, nq x nr; the pairs evaluated per step are pairs_computed_per_step",
                   "schedule": schedule,
                   "pairs_computed_per_step": t["pairs_computed"],
                   "main_stage_ms": t["main_ms"],
                   "workspace_bytes": t["workspace_bytes"],
                   "datagen_s": round(gen_s, 2)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_F32_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / MFMA_F32_PEAK_TFLOPS,
                     "traffic": None, "kernel": t["kernel"],
                     "kernel_ms_per_launch": kern_ms, "launches_per_step": launches},
    }
    if two_phase:
        out["config"]["select_rows_ms"] = t["select_ms"]

    # the fp32 matrix rate this machine sustains (matrix instructions only, ~0.25 s), beside the nominal peak
    from paper_0906_0231_amd import knn_mfma_calibration
    knn_mfma_calibration(1 << 16, 2)
    cal_tflops, _ = knn_mfma_calibration(1 << 22, 2)
    out["roofline"]["measured_peak"] = cal_tflops
    out["roofline"]["frac_of_measured_peak"] = achieved / cal_tflops

    if w.metric in ("l1", "linf"):
        from paper_0906_0231_amd import knn_valu_calibration
        knn_valu_calibration(1 << 16, 4)
        valu_tops, _ = knn_valu_calibration(1 << 21, 4)
        out["roofline"].update({"bound": "alu", "peak": VALU_F32_PLAIN_TOPS,
                                "frac": achieved / VALU_F32_PLAIN_TOPS,
                                "unit": "1e12 lane operations/s",
                                "peak_derivation": "256 CU x 4 SIMD x 32 lanes/clk x 2.4 GHz, one flop per "
                                                   "instruction (sub, add|.|): half the published FMA rate",
                                "measured_peak": valu_tops,
                                "frac_of_measured_peak": achieved / valu_tops})

    tkey = (w.name, t["kernel"])
    if tkey in OFFLINE_TRAFFIC_BYTES_PER_STEP and args.variant == 0 and not args.block_rows:
        nbytes, source = OFFLINE_TRAFFIC_BYTES_PER_STEP[tkey]
        out["roofline"]["traffic"] = nbytes / launches
        out["roofline"]["traffic_source"] = ("bytes per launch, FETCH_SIZE + WRITE_SIZE, measured offline "
                                             "(not by this run): " + source)

    if args.variant == 6:
        out["dtype"] = "bf16 pieces of f32 data (2 per operand, 3 products), f32 accumulation, f64 re-pricing"
        out["roofline"].update({"peak": MFMA_BF16_PEAK_TFLOPS, "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                                "counts": "every bf16 piece product executed: 3 x 2 d flop per pair"})
        from paper_0906_0231_amd import knn_mfma_bf16_calibration
        knn_mfma_bf16_calibration(1 << 16, 2)
        bf_tflops, _ = knn_mfma_bf16_calibration(1 << 22, 2)       # ~0.3 s of matrix instructions alone
        out["roofline"]["measured_peak"] = bf_tflops
        out["roofline"]["frac_of_measured_peak"] = achieved / bf_tflops
    if args.fused_legs and args.variant == 0 and w.metric == "sqeuclidean" and d <= 256 and k <= 112:
        # The split-precision experiment (never the default, never `value`): the fused full square on
        # bf16 matrix instructions, used as a filter; fraction of the bf16 peak, every product counted.
        f = time_plan(0, 6, 0, 2, 1)
        out["split_precision_experiment"] = {
            "kernel": f["kernel"], "ms_per_step": f["ms_per_step"], "value": pairs_served / (f["ms_per_step"] * 1e-3),
            "steps": 2, "warmup": 1, "kernel_ms_per_launch": f["kern_ms"], "achieved": f["achieved"],
            "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": f["achieved"] / MFMA_BF16_PEAK_TFLOPS,
            "counts": "3 bf16 products per pair and coordinate", "workspace_bytes": f["workspace_bytes"]}
        from paper_0906_0231_amd import knn_mfma_bf16_calibration
        knn_mfma_bf16_calibration(1 << 16, 2)
        bf_tflops, _ = knn_mfma_bf16_calibration(1 << 22, 2)       # ~0.3 s of bf16 matrix instructions alone
        out["split_precision_experiment"]["measured_peak"] = bf_tflops
        out["split_precision_experiment"]["frac_of_measured_peak"] = f["achieved"] / bf_tflops
        if not two_phase:
            time_plan(args.symmetric, args.variant, args.block_rows, 1, 0)   # the default plan's answer back in idx / dist
    if args.fused_legs and two_phase and w.symmetric and w.metric not in ("l1", "linf"):
        # The default plan keeps distances in the workspace between its two phases.  The fused plans
        # (selection inside the distance kernel, nothing of the matrix stored) under the same clock:
        # each pair once (the tournament of block pairs; d <= 256) and the full square.
        legs = []
        for sym in ((1, 2) if d <= 256 else (2,)):
            f = time_plan(sym, 3, 0, 2, 1)
            legs.append({"schedule": "fused, " + ("each pair once" if f["symmetric"] else "full square"),
                         "kernel": f["kernel"], "ms_per_step": f["ms_per_step"],
                         "value": pairs_served / (f["ms_per_step"] * 1e-3), "steps": 2, "warmup": 1,
                         "kernel_ms_per_launch": f["kern_ms"], "launches_per_step": f["launches"],
                         "achieved": f["achieved"], "frac": f["achieved"] / MFMA_F32_PEAK_TFLOPS,
                         "pairs_computed_per_step": f["pairs_computed"], "workspace_bytes": f["workspace_bytes"]})
        out["fused_plans"] = legs
        # leave the default plan's answer in idx / dist for the parity check below
        time_plan(args.symmetric, args.variant, args.block_rows, 1, 0)

    if not args.no_select:
        # Selection stage on its own (the paper's Phase 2 as stated in Sect. 6: rows of a
        # materialised distance slab): HBM-bound, 4 bytes per element read once.
        from paper_0906_0231_amd import knn_select
        from paper_0906_0231_amd.api import load_library
        sm_rows, sm_cols = 4096, 262144                      # 4 GiB slab
        gsel = torch.Generator(device=dev).manual_seed(workloads.BASE_SEED)
        slab = torch.randn(sm_rows, sm_cols, generator=gsel, device=dev, dtype=torch.float32)
        sws = torch.empty(load_library().knn_select_workspace_bytes(sm_rows, sm_cols, k),
                          dtype=torch.uint8, device=dev)
        sout = (torch.empty((sm_rows, k), dtype=torch.int32, device=dev),
                torch.empty((sm_rows, k), dtype=torch.float32, device=dev))
        knn_select(slab, k, workspace=sws, out=sout)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 10
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            knn_select(slab, k, workspace=sws, out=sout)
        e1.record()
        torch.cuda.synchronize()
        sel_ms = e0.elapsed_time(e1) / reps
        gbs = 4.0 * sm_rows * sm_cols / (sel_ms * 1e-3) / 1e9
        out["selection_stage"] = {"kernel": "select_rows", "bound": "hbm", "achieved": gbs,
                                  "peak": 8000.0, "unit": "GB/s", "frac": gbs / 8000.0,
                                  "workload": f"{sm_rows} x {sm_cols} fp32 slab, k={k}",
                                  "ms": sel_ms, "elements_per_s": sm_rows * sm_cols / (sel_ms * 1e-3)}
        # the read rate this machine sustains on the same slab (loads only), beside the nominal peak
        from paper_0906_0231_amd import knn_read_calibration
        knn_read_calibration(slab.view(-1), sm_cols)
        read_gbs = max(knn_read_calibration(slab.view(-1), sm_cols)[0] for _ in range(3))
        out["selection_stage"]["measured_peak"] = read_gbs
        out["selection_stage"]["frac_of_measured_peak"] = gbs / read_gbs
        del slab, sws, sout

    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.add(src, 1.0, out=dst)       # one elementwise kernel: reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        out["config"]["copy_calibration_bytes_each_way"] = src.numel() * 4
        del src, dst

    if not args.no_cpu_baseline:
        import oracle
        from oracle import compare
        S = args.oracle_rows or max(8, min(nq, int(1.0e9 // max(nr, 1))))
        rng = np.random.default_rng(12345)
        rows = np.unique(np.concatenate([rng.choice(nq, size=min(S, nq), replace=False),
                                         [0, nq - 1]])).astype(np.int64)
        Rh = w.R.numpy()
        t0 = time.perf_counter()
        o_idx, o_dist, o_next = oracle.search(Rh[rows + w.self_offset], Rh, k, w.metric,
                                              self_idx=rows + w.self_offset)
        cpu_s = time.perf_counter() - t0
        rep = compare.check(Rh[rows + w.self_offset], Rh, w.metric, o_idx, o_dist, o_next,
                            idx[rows].cpu().numpy(), dist[rows].cpu().numpy(),
                            self_idx=rows + w.self_offset)
        out["cpu_baseline"] = {"value": len(rows) * float(nr) / cpu_s, "unit": "pairs/s",
                               "cores": oracle.threads(), "kind": "oracle",
                               "sample": f"{len(rows)} query rows x all {nr} references "
                                         f"(fp64 distances + full sort per row), {cpu_s:.1f} s"}
        out["parity"] = {"rows_checked": int(rep.rows), "ok": bool(rep.ok),
                         "max_rel_err": rep.max_rel_err, "rows_set_exempt": rep.rows_set_exempt}
        if not rep.ok:
            # a wrong answer has no throughput
            out["value"] = None
            out["parity"]["failures"] = rep.failures[:5]
            print(json.dumps(out))
            return 1
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
