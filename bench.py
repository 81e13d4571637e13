#!/usr/bin/env python3
"""Benchmark of the KAN layer hot path on one MI355X.

One step = kan_forward + kan_backward (all four gradients) of the 512->512, G=20, k=3 layer on a
batch of 16384 synthetic samples resident in HBM.  Prints one JSON line with the whole-job
throughput in edge-evaluations/s, the roofline position of the dominant kernel (its duration is
measured with HIP events on the launch stream, inside the timed region) and the CPU oracle timed on
the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# algorithmic flops per edge evaluation of each kernel family (K = k+1 window multiply-adds for the
# spline plus one multiply-add for the base term, 2 flops each)
def flops_per_edge(k):
    return 2 * (k + 1) + 2


# HBM-side bytes per launch on the config-3 workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE scaled by a
# 1 GiB copy (profiles/kan_c3_fwd_bwd_hbm_traffic.md): read + written.  Only valid for that workload and these kernels.
MEASURED_TRAFFIC_BYTES_C3 = {
    "forward_lds": 235.3e6 + 33.6e6,
    "dx_lds": 268.5e6 + 33.6e6,
    "dparam_sorted": 469.9e6 + 201.3e6,
}

KERNEL_ROLE = {  # kernel family -> which third of the fwd+bwd work it carries
    "forward_generic": "forward", "dx_generic": "dx", "dparam_generic": "dparam",
    "forward_lds": "forward", "dx_lds": "dx", "dparam_sorted": "dparam", "dparam_walk": "dparam",
    "forward_narrow": "forward", "dx_narrow": "dx", "dparam_narrow": "dparam",
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--dense-baseline", action="store_true",
                    help="also time the dense basis x coefficient GEMM formulation of the forward pass")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy (for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU only: this build has no multi-GPU path (--gpus must be 1)",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2408_11200_amd import binding, roofline, workloads

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        return 2
    binding.load()

    w = {"c2": workloads.config2, "c3": workloads.config3, "c4": workloads.config4}[args.workload]()
    s, p = w.layers[0], w.params[0]
    dev = lambda a: torch.from_numpy(a).cuda()
    x, coef, w_s, w_b, gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
    B = w.B
    y = torch.empty((B, s.n_out), device="cuda")
    out = {"gx": torch.empty((B, s.n_in), device="cuda"), "gcoef": torch.empty_like(coef),
           "gw_s": torch.empty_like(w_s), "gw_b": torch.empty_like(w_b)}
    ws_f = torch.empty(binding.kan_workspace_bytes(s, B, binding.PASS_FORWARD), dtype=torch.uint8, device="cuda")
    ws_b = torch.empty(binding.kan_workspace_bytes(s, B, binding.PASS_BACKWARD), dtype=torch.uint8, device="cuda")

    def step():
        binding.kan_forward(s, x, coef, w_s, w_b, y=y, ws=ws_f)
        binding.kan_backward(s, x, coef, w_s, w_b, gy, out=out, ws=ws_b)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    binding.kan_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    binding.kan_profile_enable(False)
    kt = binding.kan_profile_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    edges = roofline.edge_evals(B, s.n_in, s.n_out)
    value = edges / (ms_per_step * 1e-3)

    # dominant kernel = largest average duration
    avg = {n: tot / max(cnt, 1) for n, (tot, cnt) in kt.items()}
    dom = max(avg, key=avg.get)
    dom_ms = avg[dom]
    if dom in KERNEL_ROLE:
        flops = flops_per_edge(s.k) * edges
        achieved = flops / (dom_ms * 1e-3) / 1e12
    else:
        flops, achieved = None, None
    peak = roofline.MI355X_FP32_VECTOR_FLOPS / 1e12
    rl = {"bound": "alu", "kernel": dom, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
          "frac": (achieved / peak) if achieved else None,
          "traffic": MEASURED_TRAFFIC_BYTES_C3.get(dom) if args.workload == "c3" else None,
          "kernel_ms": dom_ms,
          "peak_unpacked": roofline.MI355X_FP32_VECTOR_FLOPS_UNPACKED / 1e12,
          "frac_unpacked": (achieved / (roofline.MI355X_FP32_VECTOR_FLOPS_UNPACKED / 1e12)) if achieved else None,
          "whole_path_frac": roofline.algorithmic_flops_per_edge(s.k + 1) * value / roofline.MI355X_FP32_VECTOR_FLOPS,
          "kernels_ms": {n: round(v, 4) for n, v in sorted(avg.items())}}

    dense = None
    if args.dense_baseline:
        ws_d = torch.empty(binding.load().kan_dense_baseline_workspace_bytes(binding.kan_desc(s), B), dtype=torch.uint8,
                           device="cuda")
        for _ in range(2):
            binding.kan_dense_baseline_forward(s, x, coef, w_s, w_b, y=y, ws=ws_d)
        torch.cuda.synchronize()
        d0 = time.perf_counter()
        for _ in range(5):
            binding.kan_dense_baseline_forward(s, x, coef, w_s, w_b, y=y, ws=ws_d)
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - d0) * 1e3 / 5
        fwd_ms = sum(v for n, v in avg.items() if KERNEL_ROLE.get(n) == "forward") + avg.get("fold_scale", 0.0)
        dense = {"forward_ms_dense_gemm": dense_ms, "forward_ms_local": fwd_ms,
                 "note": "forward pass only; dense = expand all G+k bases + rocBLAS sgemm"}
        del ws_d

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
        reps = 3
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle.kan_forward(w.x, p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h, s.base_act)
            oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h, s.base_act)
        c1 = time.perf_counter()
        cpu = {"value": reps * edges / (c1 - c0), "unit": "edge-evals/s",
               "cores": oracle.num_threads(), "kind": "oracle",
               "sample": "the whole batch (%d rows), forward + backward, %d repetitions, %.1f s" % (B, reps, c1 - c0)}

    line = {"metric": "KAN layer fwd+bwd edge-evals/sec (B*n_in*n_out)", "value": value, "unit": "edge-evals/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
            "data": "synthetic",
            "config": {"workload": w.name, "B": B, "n_in": s.n_in, "n_out": s.n_out, "G": s.G, "k": s.k,
                       "grid": [s.grid_lo, s.grid_hi], "pass": "forward+backward"},
            "roofline": rl, "cpu_baseline": cpu}
    if dense:
        line["dense_baseline"] = dense
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
