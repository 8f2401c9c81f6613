#!/usr/bin/env python3
"""Benchmark of the MGRIT-FAS hot path on one MI355X.

One "step" is one pass of the whole path over one synthetic batch: a forward FAS solve of
`--cycles` V-cycles (relaxation, C-point residual + norm, injection, FAS right-hand side, coarse
solve, correction), then the adjoint solve of as many cycles about the computed states (act'
cache, adjoint relaxation and transfers) and the parameter gradient.  Inputs are resident in HBM
before the timed region.  Prints ONE JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg2] [--cycles 2]

The line's top level is the workload the metric is quoted on (cfg2: "run to residual 1e-6").  The other
three benchmark workloads (N = 64, 512, 1024) ride along under `extras.per_config`, each with its step time,
its dominant kernel's roofline fraction, one forward cycle against serial forward propagation on the GPU and
the time to an RMS residual of 1e-6; `--no-per-config` leaves them out.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK = {"fp32_mfma": 157.3, "bf16_mfma": 2500.0,       # TFLOP/s, published dense peaks of MI355X
        "hbm_GBps": 8000.0}
EVENT_PAIR_US = 2.6
METRIC = "layer-steps/sec per FAS cycle + time-to-1e-6 residual vs serial, 1×MI355X"

# Kernel class of the library's launch trace -> how that kernel's row starts in the rocprofv3 tables under
# profiles/ (template arguments as the profiler prints them).
PROFILE_ROW = {
    "dense_step_kernel<float,64,64>": r"dense_step_kernel<float, 64, 64,",
    "dense_step_kernel<float,128,128>": r"dense_step_kernel<float, 128, 128,",
    "dense_step_kernel<bf16,64,64>": r"dense_step_kernel<__bf16, 64, 64,",
    "dense_step_kernel<bf16,128,128>": r"dense_step_kernel<__bf16, 128, 128,",
    "conv_step_kernel<float>": r"conv_step_kernel<float,",
    "conv_step_kernel<bf16>": r"conv_step_kernel<__bf16,",
    "dense_sweep_kernel<float>": r"dense_sweep_kernel<float,",
    "dense_sweep_kernel<bf16>": r"dense_sweep_kernel<__bf16,",
    "dense_ksplit_kernel<float,8>": r"dense_ksplit_kernel<float, (?:false|true), 8[,>]",
    "dense_ksplit_kernel<float,4>": r"dense_ksplit_kernel<float, (?:false|true), 4[,>]",
    "dense_ksplit_kernel<bf16,4>": r"dense_ksplit_kernel<__bf16, (?:false|true), 4[,>]",
    "dense_ksplit_kernel<bf16,8>": r"dense_ksplit_kernel<__bf16, (?:false|true), 8[,>]",
    "conv_sweep_kernel": r"conv_sweep_kernel",
}


def measured_traffic_bytes(workload, kernel_class):
    """HBM bytes per launch of `kernel_class` as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE on the same
    bench command: the two calibrated means (last column, MB) of profiles/<workload>_bench_hbm_traffic.md, read at
    run time.  None if no counter run exists for the workload; an error if the table exists and does not list the
    kernel (the table is stale then)."""
    path = os.path.join(ROOT, "profiles", "%s_bench_hbm_traffic.md" % workload)
    if not os.path.exists(path):
        return None
    pat = re.compile(r"^\|\s*" + PROFILE_ROW[kernel_class])
    tot, cnt = {}, {}
    for line in open(path):
        if pat.match(line):          # several instances of one class (e.g. streaming and plain weight loads): weighted mean
            cells = [c.strip() for c in line.strip().strip("|").split("|")]
            n = float(cells[2])
            tot[cells[1]] = tot.get(cells[1], 0.0) + n * float(cells[-1]) * 1e6
            cnt[cells[1]] = cnt.get(cells[1], 0.0) + n
    if set(tot) != {"FETCH_SIZE", "WRITE_SIZE"}:
        raise RuntimeError("%s has no FETCH_SIZE / WRITE_SIZE rows for %s: re-run the counter passes after a kernel "
                           "change (profiles/README.md)" % (path, kernel_class))
    return tot["FETCH_SIZE"] / cnt["FETCH_SIZE"] + tot["WRITE_SIZE"] / cnt["WRITE_SIZE"]


def layer_steps_per_solve(sizes, m, relax, iters):
    """Layer-step evaluations (one u + h F(u) for the whole batch at one point of one level) that
    a solve of `iters` V-cycles performs -- mirrors the launch schedule exactly."""
    L = len(sizes)
    if L == 1:
        return sizes[0]

    def cyc(l, opening):
        if l == L - 1:
            return sizes[l]
        Nc = sizes[l + 1]
        nF = sizes[l] - Nc           # F-points: (m - 1) per interval and the trailing ones
        n = nF if opening else 0
        if relax == 1:
            n += Nc + nF
        n += Nc                      # C-point residual
        n += Nc                      # FAS right-hand side (coarse step)
        n += cyc(l + 1, True)
        n += nF                      # F-relaxation after the correction
        return n

    return sum(cyc(0, k == 0) for k in range(iters))


class Workbench:
    """Device buffers of one workload and the calls the benchmark times on it."""

    def __init__(self, name, cycles):
        import numpy as np
        import torch
        import mgrit_inputs as I
        import paper_2007_07336_amd as M
        self.np, self.torch, self.I, self.M = np, torch, I, M
        self.name, self.cycles = name, cycles
        dev = self.dev = "cuda:0"
        if name.startswith("mixed"):
            wl = I.mixed(cycles, I.BF16 if name == "mixed_bf16" else I.FP32)
        else:
            wl = I.ALL[name](cycles)
        self.wl = wl
        self.data = data = I.generate(wl)
        self.p = M.problem_from_workload(wl)
        self.sizes, _ = M.mgrit_level_map(self.p)
        self.W = torch.from_numpy(data["W"]).to(dev)
        if wl.dtype == I.BF16:
            self.W = self.W.to(torch.bfloat16)
        self.b = torch.from_numpy(data["b"]).to(dev)
        self.u0 = torch.from_numpy(data["u0"]).to(dev)
        self.U = torch.zeros((wl.N + 1,) + wl.state_shape, dtype=torch.float32, device=dev)
        # mixed stacks (periodic fully connected layers inside a convolution stack) go through the *_mixed entry
        # points with the same arguments plus the fully connected layers' arrays
        self.mixed = wl.fc_period > 0
        self.fc = None
        if self.mixed:
            Wfc = torch.from_numpy(data["Wfc"]).to(dev)
            if wl.dtype == I.BF16:
                Wfc = Wfc.to(torch.bfloat16)
            bfc = torch.from_numpy(data["bfc"]).to(dev)
            self._fc_keep = (Wfc, bfc, torch.zeros(Wfc.shape, dtype=torch.float32, device=dev), torch.zeros_like(bfc))
            self.fc = M.make_fc_layers(wl.fc_period, *self._fc_keep)
        self.ws = torch.empty(self.ws_bytes(self.p, True), dtype=torch.uint8, device=dev)
        self.Lam = torch.zeros_like(self.U)
        self.dW = torch.zeros(self.W.shape, dtype=torch.float32, device=dev)
        self.db = torch.zeros_like(self.b)
        self.lamN = torch.zeros(wl.state_shape, dtype=torch.float32, device=dev)
        if wl.head_classes:               # terminal adjoint of the softmax head from a first forward solve
            self.fwd(self.p, want_hist=False)
            torch.cuda.synchronize()
            self.lamN.copy_(torch.from_numpy(I.terminal_adjoint(wl, data, self.U[-1].cpu().numpy())))
        else:
            rng = np.random.default_rng(1)
            self.lamN.copy_(torch.from_numpy(rng.standard_normal(wl.state_shape).astype(np.float32) / wl.B))

    def ws_bytes(self, pp, adj):
        M = self.M
        if self.mixed:
            return (M.mgrit_adjoint_workspace_bytes_mixed if adj else M.mgrit_workspace_bytes_mixed)(pp, self.wl.fc_period)
        return (M.mgrit_adjoint_workspace_bytes if adj else M.mgrit_workspace_bytes)(pp)

    def fwd(self, pp, W=None, b=None, ws=None, **kw):
        W = self.W if W is None else W
        b = self.b if b is None else b
        ws = self.ws if ws is None else ws
        if self.mixed:
            return self.M.mgrit_fas_forward_mixed(pp, self.fc, W, b, self.u0, self.U, ws, **kw)
        return self.M.mgrit_fas_forward(pp, W, b, self.u0, self.U, ws, **kw)

    def adj(self, pp, **kw):
        if self.mixed:
            return self.M.mgrit_fas_adjoint_mixed(pp, self.fc, self.W, self.b, self.U, self.lamN, self.Lam, self.dW,
                                                  self.db, self.ws, **kw)
        return self.M.mgrit_fas_adjoint(pp, self.W, self.b, self.U, self.lamN, self.Lam, self.dW, self.db, self.ws, **kw)

    def step(self):
        self.fwd(self.p, want_hist=False)
        self.adj(self.p, want_hist=False)

    def problem(self, **kw):
        return self.M.problem_from_workload(self.wl, **kw)

    # ---- timing helpers: medians of `reps` runs after 3 warm-ups
    def timed(self, fn, reps=20):
        torch, np = self.torch, self.np
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a = time.perf_counter()
            fn()
            torch.cuda.synchronize()
            ts.append((time.perf_counter() - a) * 1e3)
        return float(np.median(ts))

    def timed_graph(self, fn, reps=20):
        """The same launches recorded into a HIP graph and replayed (no host launch cost in the timing)."""
        torch = self.torch
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            fn()
            torch.cuda.synchronize()
            with torch.cuda.graph(graph, stream=side):
                fn()
        torch.cuda.synchronize()
        return self.timed(graph.replay, reps)

    # ---- the timed region: W warm-up steps, then exactly K steps between synchronisations
    def run_steps(self, steps, warmup):
        torch = self.torch
        for _ in range(warmup):
            self.step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            self.step()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def step_counts(self):
        wl = self.wl
        solve = layer_steps_per_solve(self.sizes, wl.m, wl.relax, self.cycles)
        # relaxation / residual / right-hand-side / coarse-solve steps of the two solves, then the two passes over all
        # layers that are not part of a FAS cycle: the act' cache (one affine map per layer) and the parameter
        # gradient (one contraction of the same size per layer)
        return {"forward_solve": solve, "adjoint_solve": solve, "act_prime_cache": wl.N, "parameter_gradient": wl.N}

    def roofline(self, steps):
        """Dominant step kernel: the same steps again with the library's HIP-event launch trace on."""
        wl, I, M = self.wl, self.I, self.M
        M.mgrit_trace_begin()
        for _ in range(steps):
            self.step()
        tr = M.mgrit_trace_end()
        self.torch.cuda.synchronize()
        step_classes = {k: v for k, v in tr.items() if k != "dense_grad_kernel"}
        # The dominant kernel is the one with the most kernel time.  The trace brackets every launch with a HIP event
        # pair, which adds EVENT_PAIR_US to the interval of a short launch (bracketed minus rocprofv3 duration of the
        # 5 and 7 us launches of workload 2: 2.6 and 2.8 us), so a class of many short launches would look larger
        # than it is; the ranking takes that off, the figures reported below are the raw bracketed ones.
        dom = max(step_classes, key=lambda k: step_classes[k][0] - step_classes[k][1] * EVENT_PAIR_US * 1e-3)
        ms_tot, launches, units, alg_bytes = step_classes[dom]
        if wl.layer == I.DENSE:
            flops_per_unit = 2.0 * wl.B * wl.q * wl.q
            bytes_per_unit = wl.q * wl.q * (4 if wl.dtype == I.FP32 else 2) + 2 * wl.B * wl.q * 4
        else:
            flops_per_unit = 2.0 * wl.B * wl.Himg * wl.Wimg * wl.C * 9 * wl.C
            bytes_per_unit = 9 * wl.C * wl.C * (4 if wl.dtype == I.FP32 else 2) + 2 * wl.E * 4
        if self.mixed and dom.startswith("dense"):      # the fully connected layers' launches dominate
            flops_per_unit = 2.0 * wl.B * wl.d_fc * wl.d_fc
            bytes_per_unit = wl.d_fc * wl.d_fc * (4 if wl.dtype == I.FP32 else 2) + 2 * wl.E * 4
        peak_mfma = PEAK["fp32_mfma"] if wl.dtype == I.FP32 else PEAK["bf16_mfma"]
        avg_us = ms_tot * 1e3 / launches
        tflops = units * flops_per_unit / (ms_tot * 1e-3) / 1e12
        # algorithmic bytes: the library's launch trace sums, per layer step, weights and bias, the input state, every
        # fused epilogue operand (residual and right-hand-side launches read one or two more states), the act' factor
        # of the adjoint and the output, each once; bytes_per_unit is the bare step (weights, state in, state out)
        gbps = alg_bytes / (ms_tot * 1e-3) / 1e9
        gbps_bare = units * bytes_per_unit / (ms_tot * 1e-3) / 1e9
        # the roof that binds is the one that takes longer for this kernel's flops and algorithmic bytes
        hbm_bound = alg_bytes / (PEAK["hbm_GBps"] * 1e9) > units * flops_per_unit / (peak_mfma * 1e12)
        return {"bound": "hbm" if hbm_bound else "mfma", "kernel": dom,
                "achieved": round(gbps if hbm_bound else tflops, 3),
                "peak": PEAK["hbm_GBps"] if hbm_bound else peak_mfma,
                "unit": "GB/s" if hbm_bound else "TFLOP/s",
                "frac": round(gbps / PEAK["hbm_GBps"] if hbm_bound else tflops / peak_mfma, 5),
                "traffic": measured_traffic_bytes(self.name, dom),
                "launches": launches, "avg_launch_us": round(avg_us, 3),
                "flops_per_launch": units * flops_per_unit / launches,
                "algorithmic_bytes_per_launch": alg_bytes / launches,
                "bare_step_bytes_per_launch": units * bytes_per_unit / launches,
                "hbm_GBps_bare_step": round(gbps_bare, 1),
                "mfma_TFLOPs": round(tflops, 3), "mfma_frac": round(tflops / peak_mfma, 5),
                "hbm_GBps_algorithmic": round(gbps, 1), "hbm_frac": round(gbps / PEAK["hbm_GBps"], 5),
                "all_kernels_ms": {k: round(v[0] / steps, 4) for k, v in tr.items()},
                "all_kernels_launches": {k: v[1] // steps for k, v in tr.items()}}

    def cycle_vs_serial(self, reps_tol=5, reps=20):
        """The second half of the metric: one forward cycle and the forward solve to an RMS residual of 1e-6 against
        serial forward propagation on the GPU through the same step kernel (max_levels = 1)."""
        torch, wl = self.torch, self.wl
        p_tol = self.problem(max_iter=40, tol=1e-6, norm_kind=1)
        self.ws_tol = torch.empty(self.ws_bytes(p_tol, False), dtype=torch.uint8, device=self.dev)
        res = {}

        def solve_tol():
            res["r"] = self.fwd(p_tol, ws=self.ws_tol)
        t_tol = self.timed(solve_tol, reps_tol)
        p_ser = self.problem(max_levels=1)
        t_ser = self.timed(lambda: self.fwd(p_ser, ws=self.ws_tol, want_hist=False), reps)
        p_one = self.problem(max_iter=1)
        t_one = self.timed(lambda: self.fwd(p_one, want_hist=False), reps)
        # the same cycle with F- instead of FCF-relaxation (Alg. 1 step 1 allows either; the workloads prescribe FCF):
        # reported beside it, not used for any other figure
        p_one_f = self.problem(max_iter=1, relax=0)
        t_one_f = self.timed(lambda: self.fwd(p_one_f, want_hist=False), reps)
        return {"forward_1_cycle_ms": round(t_one, 3), "serial_forward_gpu_ms": round(t_ser, 3),
                "cycle_faster_than_serial": bool(t_one < t_ser),
                "forward_1_cycle_with_f_relaxation_ms": round(t_one_f, 3),
                "forward_cycle_layer_steps_per_s":
                    round(layer_steps_per_solve(self.sizes, wl.m, wl.relax, 1) / (t_one * 1e-3), 1),
                "time_to_rms_1e-6_ms": round(t_tol, 3), "cycles_to_rms_1e-6": res["r"][2],
                "final_rms_residual": res["r"][1][-1]}, p_tol, p_ser


def headline(args):
    import numpy as np
    import torch
    import mgrit_inputs as I
    import paper_2007_07336_amd as M
    wb = Workbench(args.workload, args.cycles)
    wl, sizes = wb.wl, wb.sizes
    ms_per_step = wb.run_steps(args.steps, args.warmup)
    counts = wb.step_counts()
    steps_per_step = sum(counts.values())
    value = steps_per_step / (ms_per_step * 1e-3)
    out = {"metric": METRIC, "value": round(value, 1), "unit": "layer-steps/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
           "scaling": "weak", "vs_baseline": None,
           "dtype": "f32" if wl.dtype == I.FP32 else "bf16", "data": "synthetic",
           "config": {"workload": wl.name, "levels": sizes, "m": wl.m, "relax": "FCF" if wl.relax else "F",
                      "step": "forward solve + adjoint solve of %d V-cycles each + parameter gradient" % args.cycles,
                      "cycles_per_solve": args.cycles, "layer_steps_per_step": steps_per_step,
                      "layer_steps_by_part": counts,
                      "fas_cycle_layer_steps_per_s": round((counts["forward_solve"] + counts["adjoint_solve"]) /
                                                           (ms_per_step * 1e-3), 1),
                      "sample_steps_per_s": round(value * wl.B, 1), "adjoint": True},
           "roofline": wb.roofline(args.steps)}

    if not args.no_extras:
        ext, p_tol, p_ser = wb.cycle_vs_serial()
        t_ser_graph = wb.timed_graph(lambda: wb.fwd(p_ser, ws=wb.ws_tol, want_hist=False))
        t_two = wb.timed(lambda: wb.fwd(wb.p, want_hist=False))
        # nested-iteration start against the copy start, on this workload's independent random layers
        # and on the same shapes with parameters that vary smoothly with depth
        nested = {}
        wl_s = I.reduced(wl, smooth_depth=True)
        data_s = I.generate(wl_s)
        W_s = torch.from_numpy(data_s["W"]).to(wb.dev)
        if wl.dtype == I.BF16:
            W_s = W_s.to(torch.bfloat16)
        b_s = torch.from_numpy(data_s["b"]).to(wb.dev)
        for tag, Wx, bx in (("random_layers", wb.W, wb.b), ("smooth_depth", W_s, b_s)):
            for init, iname in ((1, "copy"), (3, "nested")):
                p_i = wb.problem(max_iter=40, tol=1e-6, norm_kind=1, init=init)
                r = {}

                def run():
                    r["r"] = wb.fwd(p_i, Wx, bx, wb.ws_tol)
                t_i = wb.timed(run, 3)
                nested["%s_%s" % (tag, iname)] = {"cycles": r["r"][2], "ms": round(t_i, 3),
                                                  "first_rms_residual": r["r"][1][0]}
        del W_s, b_s
        # gradient of the early-stopped solves against the exact one (Sec. IV-A: two cycles suffice for
        # training): k forward cycles, k adjoint cycles about those states, gradient; the reference is
        # max_levels = 1, i.e. serial forward and backward propagation through the same kernels
        grad_err = {}
        p_ser_a = wb.problem(max_levels=1)
        wb.fwd(p_ser_a, want_hist=False)
        wb.adj(p_ser_a, want_hist=False)
        torch.cuda.synchronize()
        ref_n = float(torch.linalg.vector_norm(wb.dW.double()))
        dW_ref = wb.dW.clone()
        t_ser_train = wb.timed(lambda: (wb.fwd(p_ser_a, want_hist=False), wb.adj(p_ser_a, want_hist=False)), 3)
        for k in (1, 2, 3, 4):
            p_k = wb.problem(max_iter=k)
            wb.fwd(p_k, want_hist=False)
            wb.adj(p_k, want_hist=False)
            torch.cuda.synchronize()
            grad_err[str(k)] = float(torch.linalg.vector_norm((wb.dW - dW_ref).double())) / ref_n
        del dW_ref
        grad_err["serial_forward_backward_gradient_gpu_ms"] = round(t_ser_train, 3)
        out["time_to_tolerance"] = {"rms_residual": 1e-6, "ms": ext["time_to_rms_1e-6_ms"], "cycles": ext["cycles_to_rms_1e-6"],
                                    "serial_forward_gpu_ms": ext["serial_forward_gpu_ms"],
                                    "serial_forward_gpu_graph_replay_ms": round(t_ser_graph, 3)}
        out["extras"] = dict(ext)
        out["extras"].update({"gradient_rel_error_vs_cycles": grad_err, "start_comparison_to_rms_1e-6": nested,
                              "forward_%d_cycles_ms" % args.cycles: round(t_two, 3)})

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wb, args.cycles)
    return out, wb


def cpu_baseline(wb, cycles):
    """The CPU oracle on the host cores, same workload, bounded sample; then the same on one thread."""
    np, I = wb.np, wb.I
    wl, data, sizes = wb.wl, wb.data, wb.sizes
    from oracle import mgrit_oracle as O
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([d.get("num_threads", 1) for d in threadpool_info()] or [1])
    except Exception:
        threadpool_limits = None
        cores = os.cpu_count() or 1
    # bounded sample of about 10-30 s of CPU work: the same workload (widths, hierarchy rules, relaxation,
    # cycle count) cut to its first Ns layers and, if one pass is still too long, to its first Bs samples;
    # if one pass is short it is repeated.  Layer steps are counted as for the GPU, scaled by Bs / B.
    flop_step = 2.0 * wl.E * (wl.q if wl.layer == I.DENSE else 9 * wl.C)       # one layer step, whole batch
    if wb.mixed:
        flop_step += 2.0 * wl.B * wl.d_fc * wl.d_fc / wl.fc_period              # share of the fully connected layers
    budget = 4.0e12 if wl.layer == I.DENSE else 5.0e11                          # flops of oracle work aimed at
    per_layer = 3.2 * 3.0 * cycles
    Ns, unit, Bs = wl.N, wl.m ** (len(sizes) - 1), wl.B
    while Ns > unit and Ns * per_layer * flop_step > budget:
        Ns //= 2
    Ns = max(unit, (Ns // unit) * unit)
    while Bs > 1 and Ns * per_layer * flop_step * Bs / wl.B > budget:
        Bs //= 2
    sizes_s = O.level_sizes(Ns, wl.m, wl.max_levels, wl.min_coarse)
    Ws, bs, u0s = data["W"][:Ns], data["b"][:Ns], data["u0"][:Bs]
    kinds = wl.layer
    if wb.mixed:
        Ws, bs, kinds = I.per_layer_lists(I.reduced(wl, N=Ns), data)
    n_pass = 2 * layer_steps_per_solve(sizes_s, wl.m, wl.relax, cycles) + 2 * Ns   # counted as for the GPU
    sample = ("first %d of %d layers, first %d of %d samples, forward solve of %d cycle(s) + adjoint solve + gradient"
              % (Ns, wl.N, Bs, wl.B, cycles))
    lam_np = wb.lamN.cpu().numpy()[:Bs]

    def one_pass():
        Uo, _, _ = O.fas_forward(Ws, bs, u0s, wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax, cycles, kinds, wl.act)
        O.fas_adjoint(Ws, bs, Uo, lam_np, wl.h, wl.m, wl.max_levels, wl.min_coarse, wl.relax, cycles, kinds, wl.act)

    def run(seconds):
        a = time.perf_counter()
        reps, want = 0, 1
        while reps < want:
            one_pass()
            reps += 1
            if reps == 1:                                          # short pass: repeat it up to about `seconds` in all
                want = int(min(50, max(1, seconds // max(time.perf_counter() - a, 1e-3))))
        dt = time.perf_counter() - a
        return n_pass * reps * (Bs / wl.B) / dt, reps, dt

    v, reps, dt = run(12.0)
    out = {"value": round(v, 1), "unit": "layer-steps/s", "cores": int(cores), "kind": "oracle",
           "sample": sample + ", %d pass(es) of %s (fp64 numpy, %.1f s)" % (reps, wl.name, dt)}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            v1, reps1, dt1 = run(5.0)
        out["single_thread"] = {"value": round(v1, 1), "unit": "layer-steps/s", "cores": 1,
                                "sample": "the same sample, %d pass(es), %.1f s" % (reps1, dt1)}
    return out


def per_config_entry(name, cycles, steps=3, warmup=1):
    """One of the other benchmark workloads, measured like the headline but shorter and without the CPU leg."""
    import mgrit_inputs as I
    wb = Workbench(name, cycles)
    wl = wb.wl
    ms_per_step = wb.run_steps(steps, warmup)
    counts = wb.step_counts()
    rf = wb.roofline(steps)
    ext, _, _ = wb.cycle_vs_serial(reps_tol=3, reps=7)
    entry = {"workload": wl.name, "levels": wb.sizes, "dtype": "f32" if wl.dtype == I.FP32 else "bf16",
             "steps": steps, "warmup": warmup, "ms_per_step": round(ms_per_step, 3),
             "layer_steps_per_s": round(sum(counts.values()) / (ms_per_step * 1e-3), 1),
             "dominant_kernel": rf["kernel"], "bound": rf["bound"], "frac": rf["frac"], "achieved": rf["achieved"],
             "unit": rf["unit"], "mfma_frac": rf["mfma_frac"], "hbm_frac": rf["hbm_frac"],
             "avg_launch_us": rf["avg_launch_us"], "traffic": rf["traffic"],
             "algorithmic_bytes_per_launch": rf["algorithmic_bytes_per_launch"]}
    entry.update(ext)
    return entry


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg5", "mixed", "mixed_bf16"])
    ap.add_argument("--cycles", type=int, default=2, help="V-cycles per forward / adjoint solve (Sec. IV-A: two)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip time-to-tolerance and serial comparisons")
    ap.add_argument("--no-per-config", action="store_true", help="skip the other benchmark workloads under extras.per_config")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    out, wb = headline(args)
    if not args.no_extras and not args.no_per_config and args.workload == "cfg2":
        del wb
        per = {}
        for name in ("cfg3", "cfg4", "cfg5"):
            torch.cuda.empty_cache()
            per[name] = per_config_entry(name, args.cycles)
        out["extras"]["per_config"] = per
    print(json.dumps(out))


if __name__ == "__main__":
    main()
