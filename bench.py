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
# Vector-ALU ceiling for the fold kernel: its arithmetic is one subtract and one add (or max)
# per coordinate and pair -- single-flop instructions that cannot fuse into FMAs.  The published
# 157.3 TFLOP/s fp32 vector figure is 256 CUs x 4 SIMDs x 32 lanes per clock x 2 flop (FMA) x
# 2.4 GHz; one flop per instruction gives half of it.  (A lone wave issues every 4th cycle, 16
# lanes per clock; two or more waves of a SIMD reach the 32, measured by knn_valu_calibration.)
VALU_F32_PLAIN_TOPS = 256 * 4 * 32 * 2.4e9 / 1e12

# HBM/fabric bytes per step of the fused kernel(s), from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE runs of this script scaled by a 1 GiB copy kernel (profiles/knn_c3_registers_resident.md,
# profiles/knn_two_phase_c3_panel_pairs.md, profiles/knn_two_phase_table1_shapes.md).
# Keyed by (workload, schedule); reported per launch next to `achieved`.
MEASURED_TRAFFIC_BYTES_PER_STEP = {
    ("c3_lowrank32_n1048576_d256_k10", "triangle"): 5.83e12 + 3.01e10,
    ("c3_lowrank32_n1048576_d256_k10", "full-square"): 5.85e12 + 1.59e9,
    # knn_dist_qreg, all 136 launches of a step (profiles/knn_two_phase_c3_panel_pairs.md)
    ("c3_lowrank32_n1048576_d256_k10", "two-phase by panel pairs"): 3.195e11 + 4.858e11,
    # knn_dist_qreg alone (profiles/knn_two_phase_table1_shapes.md)
    ("paper_table1_n80000_d256_k100_hellinger", "two-phase triangle"): 1.24e10 + 2.68e10,
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
    ap.add_argument("--variant", type=int, default=0, help="0 auto, 1 streaming, 2 query tile in LDS, 3 query tile in registers, 4 two-phase")
    ap.add_argument("--block-rows", type=int, default=0, help="symmetric schedule: rows per block")
    ap.add_argument("--oracle-rows", type=int, default=None)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-select", action="store_true", help="skip the stand-alone selection timing")
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

    t0 = time.time()
    w = workloads.config(args.config, n=args.n)
    R = w.R.to(dev)
    Q = R if w.symmetric else R[:w.nq]
    nq, nr, d, k = w.nq, w.n, w.d, w.k
    gen_s = time.time() - t0

    ws = torch.empty(knn_workspace_bytes(nq, nr, d, k, w.metric, symmetric=w.symmetric,
                                         variant=args.variant, schedule=args.symmetric,
                                         block_rows=args.block_rows),
                     dtype=torch.uint8, device=dev)
    idx = torch.empty((nq, k), dtype=torch.int32, device=dev)
    dist = torch.empty((nq, k), dtype=torch.float32, device=dev)

    def step(profile):
        if w.symmetric:
            return knn_build(R, k, w.metric, symmetric=args.symmetric, variant=args.variant,
                             block_rows=args.block_rows, profile=profile, workspace=ws,
                             out=(idx, dist))
        return knn_search(Q, R, k, w.metric, self_offset=w.self_offset, variant=args.variant,
                          profile=profile, workspace=ws, out=(idx, dist))

    for _ in range(args.warmup):
        step(False)
    torch.cuda.synchronize()
    main_ms, launches, pairs_computed, symmetric, two_phase, select_ms = [], 1, 0, 0, 0, []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        res = step(True)           # events around the fused kernel, on the launch stream
        main_ms.append(res.profile.ms_main)
        launches = max(1, res.profile.main_launches)
        pairs_computed = res.profile.pairs_computed
        symmetric = res.profile.symmetric
        two_phase = res.profile.two_phase
        select_ms.append(res.profile.ms_select)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = 1e3 * elapsed / args.steps

    pairs_served = float(nq) * float(nr)
    value = pairs_served / (ms_per_step * 1e-3)
    # dominant kernel: the fused tile kernel; algorithmic work = 2*d flop per pair it evaluates
    if two_phase == 1:
        # matrix written out, then selected from: the dominant kernel is the one that writes it
        launches = 1
        kern_ms = float(np.mean(main_ms)) - float(np.mean(select_ms))
    elif two_phase == 2:
        # block by block: one distance launch per pair of row panels (the library brackets each
        # with events), two selections after it.  G panels: G(G+1)/2 + G*G launches in all.
        G = int(round((-1.0 + (1.0 + 24.0 * launches) ** 0.5) / 6.0))
        launches = G * (G + 1) // 2
        kern_ms = (float(np.mean(main_ms)) - float(np.mean(select_ms))) / launches
    else:
        kern_ms = float(np.mean(main_ms)) / launches
    flop_per_launch = 2.0 * d * pairs_computed / launches
    achieved = flop_per_launch / (kern_ms * 1e-3) / 1e12

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
                   "schedule": ("two-phase " if two_phase else "") + ("triangle" if symmetric else "full-square"),
                   "pairs_computed_per_step": pairs_computed,
                   "fused_kernel_ms": float(np.mean(main_ms)),
                   "datagen_s": round(gen_s, 2)},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": MFMA_F32_PEAK_TFLOPS,
                     "unit": "TFLOP/s", "frac": achieved / MFMA_F32_PEAK_TFLOPS,
                     "traffic": None, "kernel": ("knn_dist_qreg" if d <= 256 else "knn_dist_stream") if two_phase else "knn_pairs_qreg" if symmetric else "knn_tiles_qreg" if d <= 256 and args.variant in (0, 3) else "knn_tiles",
                     "kernel_ms_per_launch": kern_ms, "launches_per_step": launches},
    }

    if two_phase == 2:
        out["config"]["schedule"] = "two-phase by panel pairs"
        out["config"]["select_rows_ms"] = float(np.mean(select_ms))
    if two_phase == 1:
        out["config"]["select_rows_ms"] = float(np.mean(select_ms))
        out["config"]["matrix_bytes"] = 4.0 * (float((nq + 127) // 128 * 128) * float((nr + 127) // 128 * 128 + 64))

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
                                "kernel": "knn_fold_dist" if two_phase else "knn_fold",
                                "peak_derivation": "256 CU x 4 SIMD x 32 lanes/clk x 2.4 GHz, one flop per "
                                                   "instruction (sub, add|.|): half the published FMA rate",
                                "measured_peak": valu_tops,
                                "frac_of_measured_peak": achieved / valu_tops})

    tkey = (w.name, out["config"]["schedule"])
    if tkey in MEASURED_TRAFFIC_BYTES_PER_STEP and args.variant in (0, 3, 4) and not args.block_rows:
        out["roofline"]["traffic"] = MEASURED_TRAFFIC_BYTES_PER_STEP[tkey] / launches
        out["roofline"]["traffic_unit"] = "bytes per launch (offline rocprofv3 FETCH_SIZE+WRITE_SIZE)"

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
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
