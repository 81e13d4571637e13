#!/usr/bin/env python3
"""Benchmark of the KAN / UKAN layer hot path on one MI355X.

One step = forward + backward (every gradient) of every layer of the workload on one batch of
synthetic samples resident in HBM.  The default workload is the 512->512, G=20, k=3 layer on a batch
of 16384 (the configuration the headline metric is quoted on).  Prints one JSON line with the
whole-job throughput in edge-evaluations/s, the roofline position of the dominant kernel (its
duration is measured with HIP events on the launch stream, inside the timed region) and the CPU
oracle timed on the host cores on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

UKAN_MAX_GROUPS = 160   # table bound handed to the UKAN entry points (x ~ N(0, 10^2), groups of width 1)


# algorithmic flops per edge evaluation of each kernel family (K = k+1 window multiply-adds for the
# spline plus one multiply-add for the base term, 2 flops each)
def flops_per_edge(k):
    return 2 * (k + 1) + 2


# HBM-side bytes per launch on the config-3 workload, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
# scaled by a 1 GiB copy (profiles/kan_c3_fwd_bwd_hbm_traffic.md): read + written.  Only valid for
# that workload and these kernels.
MEASURED_TRAFFIC_BYTES_C3 = {
    "forward_lds": 234.9e6 + 33.6e6,
    "backward_walk": 1105.7e6 + 826.6e6,
}

# kernel family -> which third of the fwd+bwd work it carries ("backward" = dL/dx and the parameter
# gradients in one kernel: two thirds)
KERNEL_ROLE = {
    "forward_generic": "forward", "dx_generic": "dx", "dparam_generic": "dparam",
    "forward_lds": "forward", "forward_pairs": "forward", "forward_rows": "forward", "dparam_walk": "dparam", "backward_walk": "backward",
    "forward_narrow": "forward", "dx_narrow": "dx",
}
ROLE_SHARE = {"forward": 1, "dx": 1, "dparam": 1, "backward": 2}


class KanCase:
    """One bounded-grid layer: kan_forward + kan_backward."""

    def __init__(self, w, torch, binding):
        self.binding, self.w = binding, w
        s, p = w.layers[0], w.params[0]
        dev = lambda a: torch.from_numpy(a).cuda()
        self.s = s
        self.x, self.coef, self.w_s, self.w_b, self.gy = (dev(a) for a in (w.x, p["coef"], p["w_s"], p["w_b"], w.gy))
        B = w.B
        self.y = torch.empty((B, s.n_out), device="cuda")
        self.out = {"gx": torch.empty((B, s.n_in), device="cuda"), "gcoef": torch.empty_like(self.coef),
                    "gw_s": torch.empty_like(self.w_s), "gw_b": torch.empty_like(self.w_b)}
        self.ws_f = torch.empty(binding.kan_workspace_bytes(s, B, binding.PASS_FORWARD), dtype=torch.uint8, device="cuda")
        self.ws_b = torch.empty(binding.kan_workspace_bytes(s, B, binding.PASS_BACKWARD), dtype=torch.uint8, device="cuda")
        self.edges = B * s.n_in * s.n_out
        self.k = s.k
        self.config = {"workload": w.name, "B": B, "n_in": s.n_in, "n_out": s.n_out, "G": s.G, "k": s.k,
                       "grid": [s.grid_lo, s.grid_hi], "pass": "forward+backward"}

    def forward(self):
        self.binding.kan_forward(self.s, self.x, self.coef, self.w_s, self.w_b, y=self.y, ws=self.ws_f)

    def backward(self):
        self.binding.kan_backward(self.s, self.x, self.coef, self.w_s, self.w_b, self.gy, out=self.out, ws=self.ws_b)

    def step(self):
        self.forward()
        self.backward()

    def cpu_baseline(self, oracle):
        w, s, p = self.w, self.s, self.w.params[0]
        inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
        reps = 3
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle.kan_forward(w.x, p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h, s.base_act)
            oracle.kan_backward(w.x, p["coef"], p["w_s"], p["w_b"], w.gy, s.G, s.k, s.grid_lo, inv_h, s.base_act)
        c1 = time.perf_counter()
        return reps * self.edges / (c1 - c0), "the whole batch (%d rows), forward + backward, %d repetitions, %.1f s" % (
            w.B, reps, c1 - c0)


class UkanCase:
    """The UKAN stack: ukan_cg_forward + ukan_cg_backward of every layer.  The incoming gradient of
    each layer is a fixed synthetic tensor (the true chained gradient, rescaled to unit RMS, taken
    once before the timed region), so every step does identical work."""

    def __init__(self, w, torch, binding):
        self.binding, self.w = binding, w
        dev = lambda a: torch.from_numpy(a).cuda()
        mg = UKAN_MAX_GROUPS
        self.P = [{n: dev(a) for n, a in p.items()} for p in w.params]
        self.acts = [dev(w.x)]
        for s, pd in zip(w.layers, self.P):
            self.acts.append(binding.ukan_cg_forward(s, self.acts[-1], pd, mg))
        L = len(w.layers)
        self.gys = [None] * L
        g = dev(w.gy)
        for l in reversed(range(L)):
            self.gys[l] = g
            gx = binding.ukan_cg_backward(w.layers[l], self.acts[l], self.P[l], g, mg, want=["gx"])["gx"]
            g = (gx / gx.pow(2).mean().sqrt()).contiguous()
        self.outs, self.ws_f, self.ws_b = [], [], []
        for l, s in enumerate(w.layers):
            K = s.k + 1
            self.outs.append({
                "gx": torch.empty((w.B, s.n_in), device="cuda"), "gE": torch.empty((s.n_in, s.d_feat), device="cuda"),
                "gW1": torch.empty((s.d_feat + s.d_pe, s.d_hidden), device="cuda"),
                "gb1": torch.empty((s.d_hidden,), device="cuda"),
                "gW2": torch.empty((s.d_hidden, K * s.n_out), device="cuda"),
                "gb2": torch.empty((K * s.n_out,), device="cuda"),
                "gscale": torch.empty((s.n_in, s.n_out), device="cuda")})
            self.ws_f.append(torch.empty(binding.ukan_workspace_bytes(s, w.B, mg, binding.PASS_FORWARD),
                                         dtype=torch.uint8, device="cuda"))
            self.ws_b.append(torch.empty(binding.ukan_workspace_bytes(s, w.B, mg, binding.PASS_BACKWARD),
                                         dtype=torch.uint8, device="cuda"))
        self.edges = sum(w.B * s.n_in * s.n_out for s in w.layers)
        self.k = w.layers[0].k
        self.config = {"workload": w.name, "B": w.B, "widths": [w.layers[0].n_in] + [s.n_out for s in w.layers],
                       "h": w.layers[0].h, "k": self.k, "max_groups": mg, "pass": "forward+backward"}

    def forward(self):
        b, w, mg = self.binding, self.w, UKAN_MAX_GROUPS
        for l, s in enumerate(w.layers):
            b.ukan_cg_forward(s, self.acts[l], self.P[l], mg, y=self.acts[l + 1], ws=self.ws_f[l])

    def backward(self):
        b, w, mg = self.binding, self.w, UKAN_MAX_GROUPS
        for l in reversed(range(len(w.layers))):
            b.ukan_cg_backward(w.layers[l], self.acts[l], self.P[l], self.gys[l], mg, out=self.outs[l], ws=self.ws_b[l])

    def step(self):
        self.forward()
        self.backward()

    def cpu_baseline(self, oracle):
        # first layer only, on a slice of the batch, scaled by its share of the edge evaluations
        w, s, p = self.w, self.w.layers[0], self.w.params[0]
        n = min(w.B, 4096)
        x = w.x[:n]
        inv_h = oracle.inv_h_of_spacing(s.h)
        gy = self.gys[0][:n].cpu().numpy()
        c0 = time.perf_counter()
        oracle.ukan_forward(x, p, s.k, inv_h, s.base_act)
        oracle.ukan_backward(x, p, gy, s.k, inv_h, s.base_act)
        c1 = time.perf_counter()
        return n * s.n_in * s.n_out / (c1 - c0), "first layer (%d->%d), rows 0..%d, forward + backward once, %.1f s" % (
            s.n_in, s.n_out, n - 1, c1 - c0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="c3", choices=["c2", "c3", "c4", "c5", "p"],
                    help="c2..c5: the benchmark configurations; p: the paper's 32->32, N=2^17 shape (see --grid)")
    ap.add_argument("--grid", type=int, default=64, help="grid size G of workload p")
    ap.add_argument("--degree", type=int, default=3, help="spline degree k of workload p (1..3)")
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

    import torch
    from paper_2408_11200_amd import binding, roofline, workloads

    if not torch.cuda.is_available():
        print("no GPU visible", file=sys.stderr)
        return 2
    binding.load()

    if args.workload == "c5":
        case = UkanCase(workloads.config5(), torch, binding)
    else:
        w = {"c2": workloads.config2, "c3": workloads.config3, "c4": workloads.config4,
             "p": lambda: workloads.paper_shape(args.grid, k=args.degree)}[args.workload]()
        case = KanCase(w, torch, binding)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        case.step()
    torch.cuda.synchronize()
    binding.kan_profile_enable(True)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        case.step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    binding.kan_profile_enable(False)
    kt = binding.kan_profile_read()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    edges = case.edges
    value = edges / (ms_per_step * 1e-3)

    # dominant kernel = largest total time per step; its roofline position uses the edge evaluations
    # it processes per step and the multiply-adds the method needs for its share of the pass
    per_step = {n: tot / args.steps for n, (tot, cnt) in kt.items()}
    launches = {n: cnt / args.steps for n, (tot, cnt) in kt.items()}
    dom = max(per_step, key=per_step.get)
    dom_ms = per_step[dom]
    if dom in KERNEL_ROLE:
        flops = flops_per_edge(case.k) * ROLE_SHARE[KERNEL_ROLE[dom]] * edges
        achieved = flops / (dom_ms * 1e-3) / 1e12
    else:
        flops, achieved = None, None
    peak = roofline.MI355X_FP32_VECTOR_FLOPS / 1e12
    # the walk kernels run the window-row multiply-adds on the matrix cores (fp32 MFMA peak = fp32 vector peak)
    bound = "mfma" if dom in ("backward_walk", "dparam_walk") else "alu"
    rl = {"bound": bound, "kernel": dom, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
          "frac": (achieved / peak) if achieved else None,
          "traffic": MEASURED_TRAFFIC_BYTES_C3.get(dom) if args.workload == "c3" else None,
          "kernel_ms": dom_ms / max(launches[dom], 1), "kernel_launches_per_step": launches[dom],
          "peak_unpacked": roofline.MI355X_FP32_VECTOR_FLOPS_UNPACKED / 1e12,
          "frac_unpacked": (achieved / (roofline.MI355X_FP32_VECTOR_FLOPS_UNPACKED / 1e12)) if achieved else None,
          "whole_path_frac": roofline.algorithmic_flops_per_edge(case.k + 1) * value / roofline.MI355X_FP32_VECTOR_FLOPS,
          "kernels_ms_per_step": {n: round(v, 4) for n, v in sorted(per_step.items())}}

    # forward and backward separately (outside the timed region): device events around each pass, 10 repetitions
    def timed(fn, reps=10):
        ts = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            fn()
            e1.record()
            e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        ts.sort()
        return {"median": ts[len(ts) // 2], "min": ts[0]}
    passes = {"forward_ms": timed(case.forward), "backward_ms": timed(case.backward)}

    dense = None
    if args.dense_baseline and isinstance(case, KanCase):
        s = case.s
        ws_d = torch.empty(binding.load().kan_dense_baseline_workspace_bytes(binding.kan_desc(s), case.w.B),
                           dtype=torch.uint8, device="cuda")
        for _ in range(2):
            binding.kan_dense_baseline_forward(s, case.x, case.coef, case.w_s, case.w_b, y=case.y, ws=ws_d)
        torch.cuda.synchronize()
        d0 = time.perf_counter()
        for _ in range(5):
            binding.kan_dense_baseline_forward(s, case.x, case.coef, case.w_s, case.w_b, y=case.y, ws=ws_d)
        torch.cuda.synchronize()
        dense_ms = (time.perf_counter() - d0) * 1e3 / 5
        fwd_ms = sum(v for n, v in per_step.items() if KERNEL_ROLE.get(n) == "forward") + per_step.get("fold_scale", 0.0) / 2
        del ws_d
        ws_d = torch.empty(binding.load().kan_dense_baseline_backward_workspace_bytes(binding.kan_desc(s), case.w.B),
                           dtype=torch.uint8, device="cuda")
        for _ in range(2):
            binding.kan_dense_baseline_backward(s, case.x, case.coef, case.w_s, case.w_b, case.gy, out=case.out, ws=ws_d)
        torch.cuda.synchronize()
        d0 = time.perf_counter()
        for _ in range(5):
            binding.kan_dense_baseline_backward(s, case.x, case.coef, case.w_s, case.w_b, case.gy, out=case.out, ws=ws_d)
        torch.cuda.synchronize()
        dense_bwd_ms = (time.perf_counter() - d0) * 1e3 / 5
        dense = {"forward_ms_dense_gemm": dense_ms, "forward_ms_local": fwd_ms,
                 "backward_ms_dense_gemm": dense_bwd_ms, "backward_ms_local": ms_per_step - fwd_ms,
                 "note": "dense = expand all G+k bases (and their x-derivatives) + rocBLAS sgemm"}
        del ws_d

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        v, sample = case.cpu_baseline(oracle)
        cpu = {"value": v, "unit": "edge-evals/s", "cores": oracle.num_threads(), "kind": "oracle", "sample": sample}

    line = {"metric": "KAN layer fwd+bwd edge-evals/sec (B*n_in*n_out)", "value": value, "unit": "edge-evals/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
            "data": "synthetic", "config": case.config, "roofline": rl, "cpu_baseline": cpu, "passes": passes}
    if dense:
        line["dense_baseline"] = dense
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
