#!/usr/bin/env python3
"""Benchmark of the KAN / UKAN layer hot path on one MI355X.

One step = forward + backward (every gradient) of every layer of the workload on one batch of
synthetic samples resident in HBM.  The default workload is the 512->512, G=20, k=3 layer on a batch
of 16384 (the configuration the headline metric is quoted on).  Prints one JSON line with the
whole-job throughput in edge-evaluations/s, the roofline position of the dominant kernel (its
duration is measured with HIP events on the launch stream) and the CPU oracle timed on the host
cores on a bounded sample of the same workload.

The headline (ms_per_step, value) is timed with the library's launch observer OFF: exactly --steps
steps between two device synchronisations, nothing else on the stream.  The per-kernel split behind
`roofline` comes from a second pass over the same steps with the event-timing observer of the
benchmark library installed (two events per launch, which costs a few microseconds per launch and is
why it is not part of the headline).
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

UKAN_MAX_GROUPS = 160   # table bound handed to the UKAN entry points (x ~ N(0, 10^2), groups of width 1)


# algorithmic flops per edge evaluation of each kernel family (K = k+1 window multiply-adds for the
# spline plus one multiply-add for the base term, 2 flops each)
def flops_per_edge(k):
    return 2 * (k + 1) + 2


# HBM-side bytes per launch of the dominant kernels are not measured here (that takes rocprofv3 counter
# runs): they are read from the tracked summary of those runs, which carries one machine-readable line
#   <!-- bench-traffic {"workload": "c3", "source_commit": "...", "kernels": {family: {"read": bytes, "written": bytes}}} -->
# `traffic` is null when the file, the workload or the kernel family does not match what ran.
TRAFFIC_FILE = os.path.join("profiles", "kan_c3_fwd_bwd_hbm_traffic.md")


def measured_traffic(workload, family):
    try:
        text = open(os.path.join(ROOT, TRAFFIC_FILE)).read()
    except OSError:
        return None, None
    m = re.search(r"<!-- bench-traffic (\{.*\}) -->", text)
    if not m:
        return None, None
    rec = json.loads(m.group(1))
    k = rec.get("kernels", {}).get(family)
    if rec.get("workload") != workload or not k:
        return None, None
    return k["read"] + k["written"], {"file": TRAFFIC_FILE, "source_commit": rec.get("source_commit"),
                                      "read": k["read"], "written": k["written"]}


# kernel family -> which third of the fwd+bwd work it carries ("backward" = dL/dx and the parameter
# gradients in one kernel: two thirds)
KERNEL_ROLE = {
    "forward_generic": "forward", "dx_generic": "dx", "dparam_generic": "dparam",
    "forward_lds": "forward", "forward_pairs": "forward", "forward_lds_rows": "forward", "forward_rows": "forward", "dparam_walk": "dparam", "backward_walk": "backward",
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
                       "grid": [s.grid_lo, s.grid_hi], "pass": "forward+backward",
                       "hand_off": "the backward pass reads the scale-folded table the forward pass left in its workspace"}

    def forward(self):
        self.binding.kan_forward(self.s, self.x, self.coef, self.w_s, self.w_b, y=self.y, ws=self.ws_f)

    def backward(self):
        # the backward pass of a step reads the scale-folded table its forward pass left in ws_f
        self.binding.kan_backward_saved(self.s, self.x, self.coef, self.w_s, self.w_b, self.gy, self.ws_f, out=self.out,
                                        ws=self.ws_b)

    def step(self):
        self.forward()
        self.backward()

    def cpu_baseline(self, oracle, reps=3, rows=None):
        w, s, p = self.w, self.s, self.w.params[0]
        inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
        n = w.B if rows is None else min(rows, w.B)
        x, gy = w.x[:n], w.gy[:n]
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle.kan_forward(x, p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h, s.base_act)
            oracle.kan_backward(x, p["coef"], p["w_s"], p["w_b"], gy, s.G, s.k, s.grid_lo, inv_h, s.base_act)
        c1 = time.perf_counter()
        return reps * n * s.n_in * s.n_out / (c1 - c0), "rows 0..%d of the batch of %d, forward + backward, %d repetitions, %.1f s" % (
            n - 1, w.B, reps, c1 - c0)


    def cpu_baseline_single(self, oracle):
        # about a quarter of a minute on one core: 1.2e9 edge evaluations
        rows = max(1, min(self.w.B, int(1.2e9 / (self.s.n_in * self.s.n_out))))
        return self.cpu_baseline(oracle, reps=1, rows=rows)


class KanStackCase:
    """A stack of bounded-grid layers trained against a target (the small [2,5,1] network): forward through
    every layer, dL/dy of the mean-squared error (one elementwise torch op, host-side glue between the layer
    calls), backward through every layer."""

    def __init__(self, w, torch, binding):
        self.binding, self.w, self.torch = binding, w, torch
        dev = lambda a: torch.from_numpy(a).cuda()
        self.P = [{n: dev(a) for n, a in p.items()} for p in w.params]
        self.target = dev(w.target)
        B = w.B
        self.acts = [dev(w.x)] + [torch.empty((B, s.n_out), device="cuda") for s in w.layers]
        self.gacts = [torch.empty((B, s.n_in), device="cuda") for s in w.layers] + [torch.empty((B, w.layers[-1].n_out), device="cuda")]
        self.outs = [{"gx": self.gacts[l], "gcoef": torch.empty_like(p["coef"]), "gw_s": torch.empty_like(p["w_s"]),
                      "gw_b": torch.empty_like(p["w_b"])} for l, p in enumerate(self.P)]
        self.ws_f = [torch.empty(binding.kan_workspace_bytes(s, B, binding.PASS_FORWARD), dtype=torch.uint8, device="cuda")
                     for s in w.layers]
        self.ws_b = [torch.empty(binding.kan_workspace_bytes(s, B, binding.PASS_BACKWARD), dtype=torch.uint8, device="cuda")
                     for s in w.layers]
        self.edges = sum(B * s.n_in * s.n_out for s in w.layers)
        self.k = w.layers[0].k
        self.config = {"workload": w.name, "B": B, "widths": [w.layers[0].n_in] + [s.n_out for s in w.layers],
                       "G": w.layers[0].G, "k": self.k, "pass": "forward+mse+backward"}

    def forward(self):
        for l, (s, p) in enumerate(zip(self.w.layers, self.P)):
            self.binding.kan_forward(s, self.acts[l], p["coef"], p["w_s"], p["w_b"], y=self.acts[l + 1], ws=self.ws_f[l])

    def backward(self):
        self.torch.sub(self.acts[-1], self.target, out=self.gacts[-1]).mul_(2.0 / self.w.B)
        for l in reversed(range(len(self.w.layers))):
            s, p = self.w.layers[l], self.P[l]
            self.binding.kan_backward_saved(s, self.acts[l], p["coef"], p["w_s"], p["w_b"], self.gacts[l + 1], self.ws_f[l],
                                            out=self.outs[l], ws=self.ws_b[l])

    def step(self):
        self.forward()
        self.backward()

    def cpu_baseline(self, oracle, reps=2000):
        w = self.w
        import numpy as np
        c0 = time.perf_counter()
        for _ in range(reps):
            acts = [w.x]
            for s, p in zip(w.layers, w.params):
                inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
                acts.append(np.float32(oracle.kan_forward(acts[-1], p["coef"], p["w_s"], p["w_b"], s.G, s.k, s.grid_lo, inv_h,
                                                          s.base_act)))
            g = np.float32(2.0 / w.B * (acts[-1].astype(np.float64) - w.target))
            for l in reversed(range(len(w.layers))):
                s, p = w.layers[l], w.params[l]
                inv_h = oracle.inv_h_of(s.grid_lo, s.grid_hi, s.G)
                g = np.float32(oracle.kan_backward(acts[l], p["coef"], p["w_s"], p["w_b"], g, s.G, s.k, s.grid_lo, inv_h,
                                                   s.base_act)["gx"])
        c1 = time.perf_counter()
        return reps * self.edges / (c1 - c0), "the whole batch (%d rows), both layers forward + backward, %d repetitions, %.1f s" % (
            w.B, reps, c1 - c0)


    def cpu_baseline_single(self, oracle):
        return self.cpu_baseline(oracle, reps=500)


class UkanCase:
    """The UKAN stack: ukan_cg_forward_saved + ukan_cg_backward_saved of every layer (the backward pass
    reuses the group span, the CG activations and the coefficient table its forward pass kept).  The
    incoming gradient of each layer is a fixed synthetic tensor (the true chained gradient, rescaled to unit RMS, taken
    once before the timed region), so every step does identical work."""

    def __init__(self, w, torch, binding, read_back=False):
        self.binding, self.w = binding, w
        self.read_back = read_back
        dev = lambda a: torch.from_numpy(a).cuda()
        mg = UKAN_MAX_GROUPS
        self.P = [{n: dev(a) for n, a in p.items()} for p in w.params]
        self.acts = [dev(w.x)]
        for s, pd in zip(w.layers, self.P):
            self.acts.append(binding.ukan_cg_forward(s, self.acts[-1], pd, mg))
        self.flags = torch.zeros(len(w.layers), dtype=torch.int32, device="cuda")
        L = len(w.layers)
        self.gys = [None] * L
        g = dev(w.gy)
        for l in reversed(range(L)):
            self.gys[l] = g
            gx = binding.ukan_cg_backward(w.layers[l], self.acts[l], self.P[l], g, mg, want=["gx"])["gx"]
            g = (gx / gx.pow(2).mean().sqrt()).contiguous()
        self.outs, self.ws_f, self.ws_b = [], [], []
        self.saved = [torch.empty(binding.ukan_saved_bytes(s, mg), dtype=torch.uint8, device="cuda") for s in w.layers]
        self.span = [0] * L
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
                       "h": w.layers[0].h, "k": self.k, "max_groups": mg, "pass": "forward+backward",
                       "group_span": "read back by every forward call (one stream synchronisation per layer)" if read_back
                       else "stated by the caller (the spans of a first synchronising pass): no read-back, overflow flags checked after the run"}
        # the spans every layer needs, from one synchronising pass
        for l, s in enumerate(w.layers):
            _, _, self.span[l] = binding.ukan_cg_forward_saved(s, self.acts[l], self.P[l], mg, saved=self.saved[l],
                                                               y=self.acts[l + 1], ws=self.ws_f[l])

    def forward(self):
        b, w, mg = self.binding, self.w, UKAN_MAX_GROUPS
        for l, s in enumerate(w.layers):
            if self.read_back:
                _, _, self.span[l] = b.ukan_cg_forward_saved(s, self.acts[l], self.P[l], mg, saved=self.saved[l],
                                                             y=self.acts[l + 1], ws=self.ws_f[l])
            else:
                b.ukan_cg_forward_saved_async(s, self.acts[l], self.P[l], mg, self.span[l], self.saved[l],
                                              self.flags[l:l + 1], self.acts[l + 1], self.ws_f[l])

    def backward(self):
        b, w, mg = self.binding, self.w, UKAN_MAX_GROUPS
        for l in reversed(range(len(w.layers))):
            b.ukan_cg_backward_saved(w.layers[l], self.acts[l], self.P[l], self.gys[l], mg, self.saved[l], self.span[l],
                                     out=self.outs[l], ws=self.ws_b[l])

    def step(self):
        self.forward()
        self.backward()

    def cpu_baseline_single(self, oracle):
        return self.cpu_baseline(oracle, rows=512)

    def cpu_baseline(self, oracle, rows=4096):
        # first layer only, on a slice of the batch, scaled by its share of the edge evaluations
        w, s, p = self.w, self.w.layers[0], self.w.params[0]
        n = min(w.B, rows)
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
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="c3", choices=["c1", "c2", "c3", "c4", "c5", "p"],
                    help="c1..c5: the benchmark configurations; p: the paper's 32->32, N=2^17 shape (see --grid)")
    ap.add_argument("--grid", type=int, default=64, help="grid size G of workload p")
    ap.add_argument("--batch", type=int, default=1 << 17, help="batch size of workload p")
    ap.add_argument("--degree", type=int, default=3, help="spline degree k of workload p (1..5)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--profile-steps", type=int, default=10,
                    help="steps of the separate pass that times every kernel with events (0: skip it)")
    ap.add_argument("--dense-baseline", action="store_true",
                    help="also time the dense basis x coefficient GEMM formulation of the forward pass")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step in a HIP graph and time replays")
    ap.add_argument("--ukan-read-back", action="store_true",
                    help="workload c5: use the forward call that reads the group span back (one synchronisation per layer) "
                         "instead of the one that takes the span from the caller")
    ap.add_argument("--ceilings", action="store_true",
                    help="run the instruction-rate microbenchmarks of the benchmark library instead of a workload")
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

    if args.ceilings:
        # one JSON line per microbenchmark and workgroup size; rates per CU and for the 256 CUs of the chip
        for threads in (256, 512, 1024):
            for name, unit, rate, ms in binding.kan_bench_ceilings(threads, 20000 if threads > 256 else 40000):
                print(json.dumps({"ceiling": name, "threads_per_cu": threads, "unit": unit, "per_cu_per_s": rate,
                                  "chip_per_s": 256 * rate, "kernel_ms": ms}))
        return 0

    if args.workload == "c5":
        case = UkanCase(workloads.config5(), torch, binding, read_back=args.ukan_read_back)
    elif args.workload == "c1":
        case = KanStackCase(workloads.config1(), torch, binding)
    else:
        w = {"c2": workloads.config2, "c3": workloads.config3, "c4": workloads.config4,
             "p": lambda: workloads.paper_shape(args.grid, B=args.batch, k=args.degree)}[args.workload]()
        case = KanCase(w, torch, binding)

    if args.copy_calibration:
        src = torch.empty(1 << 28, dtype=torch.float32, device="cuda").normal_()
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # headline: the launch observer is off, nothing but the steps runs between the two synchronisations
    binding.kan_set_launch_observer(None, None)
    for _ in range(args.warmup):
        case.step()
    torch.cuda.synchronize()
    run_step = case.step
    if args.graph:
        if isinstance(case, UkanCase) and case.read_back:
            print("--graph: the UKAN forward call that reads the span back synchronises and cannot be captured", file=sys.stderr)
            return 2
        # the kan_* calls only enqueue kernels on the current stream (no allocation, no memset, no
        # synchronisation), so one step can be captured as it is and replayed
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            case.step()
        run_step = graph.replay
        for _ in range(args.warmup):
            run_step()
        torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run_step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    edges = case.edges
    value = edges / (ms_per_step * 1e-3)

    # per-kernel split: a separate pass with an event pair around every launch
    psteps = max(args.profile_steps, 0)
    kt = {}
    ms_per_step_profiled = None
    if psteps:
        binding.kan_profile_enable(True)
        p0 = time.perf_counter()
        for _ in range(psteps):
            case.step()
        torch.cuda.synchronize()
        ms_per_step_profiled = (time.perf_counter() - p0) * 1e3 / psteps
        binding.kan_profile_enable(False)
        kt = binding.kan_profile_read()

    # dominant kernel = largest total time per step; its roofline position uses the edge evaluations
    # it processes per step and the multiply-adds the method needs for its share of the pass
    per_step = {n: tot / psteps for n, (tot, cnt) in kt.items()}
    launches = {n: cnt / psteps for n, (tot, cnt) in kt.items()}
    dom = max(per_step, key=per_step.get) if per_step else None
    dom_ms = per_step[dom] if dom else None
    # a stack of layers: the figure is meaningful when the dominant kernel family runs once on every layer
    # (then it carries its share of the work of all the edges); otherwise it is left out
    n_layers = len(case.w.layers)
    if dom in KERNEL_ROLE and (isinstance(case, KanCase) or round(launches[dom]) == n_layers):
        flops = flops_per_edge(case.k) * ROLE_SHARE[KERNEL_ROLE[dom]] * edges
        achieved = flops / (dom_ms * 1e-3) / 1e12
    else:
        flops, achieved = None, None
    peak = roofline.MI355X_FP32_VECTOR_FLOPS / 1e12
    # the walk kernels run the window-row multiply-adds on the matrix cores (fp32 MFMA peak = fp32 vector peak)
    bound = "mfma" if dom in ("backward_walk", "dparam_walk") else "alu"
    traffic, traffic_source = measured_traffic(args.workload, dom)
    rl = {"bound": bound, "kernel": dom, "achieved": achieved, "peak": peak, "unit": "TFLOP/s",
          "frac": (achieved / peak) if achieved else None,
          "traffic": traffic, "traffic_source": traffic_source,
          "kernel_ms": (dom_ms / max(launches[dom], 1)) if dom else None,
          "kernel_launches_per_step": launches[dom] if dom else None,
          "profiled_steps": psteps, "ms_per_step_profiled": ms_per_step_profiled,
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
        need = [binding.kan_dense_baseline_workspace_bytes(s, case.w.B, binding.PASS_FORWARD),
                binding.kan_dense_baseline_workspace_bytes(s, case.w.B, binding.PASS_BACKWARD)]
        free_bytes = torch.cuda.mem_get_info()[0]
        if s.k > 3 or max(need) > 0.8 * free_bytes:
            # the baseline materialises all G + k basis values of every (sample, input) pair
            dense = {"workspace_bytes_dense": need, "free_device_bytes": free_bytes,
                     "note": "not run: " + ("degrees 1..3 only" if s.k > 3 else "its workspace does not fit the device")}
    if args.dense_baseline and isinstance(case, KanCase) and dense is None:
        ws_d = torch.empty(binding.kan_dense_baseline_workspace_bytes(s, case.w.B, binding.PASS_FORWARD),
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
        ws_d = torch.empty(binding.kan_dense_baseline_workspace_bytes(s, case.w.B, binding.PASS_BACKWARD),
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
                 "workspace_bytes_dense": [binding.kan_dense_baseline_workspace_bytes(s, case.w.B, binding.PASS_FORWARD),
                                           binding.kan_dense_baseline_workspace_bytes(s, case.w.B, binding.PASS_BACKWARD)],
                 "workspace_bytes_local": [binding.kan_workspace_bytes(s, case.w.B, binding.PASS_FORWARD),
                                           binding.kan_workspace_bytes(s, case.w.B, binding.PASS_BACKWARD)],
                 "note": "dense = expand all G+k bases (and their x-derivatives) + rocBLAS sgemm"}
        del ws_d

    # the oracle as it stands, on all the host threads it takes, then on one thread on a smaller sample
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        v, sample = case.cpu_baseline(oracle)
        cpu = {"value": v, "unit": "edge-evals/s", "cores": oracle.num_threads(), "kind": "oracle", "sample": sample}
        all_threads = oracle.num_threads()
        oracle.set_num_threads(1)
        v1, sample1 = case.cpu_baseline_single(oracle)
        cpu["single_thread"] = {"value": v1, "unit": "edge-evals/s", "cores": oracle.num_threads(), "sample": sample1}
        oracle.set_num_threads(all_threads)

    if isinstance(case, UkanCase) and int(case.flags.abs().sum().item()) != 0:
        print("a UKAN layer needed more groups than the caller stated: results invalid", file=sys.stderr)
        return 1
    line = {"metric": "KAN layer fwd+bwd edge-evals/sec (B*n_in*n_out)", "value": value, "unit": "edge-evals/s",
            "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
            "data": "synthetic", "config": case.config, "roofline": rl, "cpu_baseline": cpu, "passes": passes}
    if args.graph:
        line["config"] = dict(case.config, launch="one HIP graph replay per step")
    if dense:
        line["dense_baseline"] = dense
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
