#!/usr/bin/env python3
"""Benchmark of the multi-adapter LoRA linear layer, forward + backward, on one MI355X.

A step is one pass of the whole path over one packed batch: fwd (down projection, base GEMM with
the fused up projection) then bwd (gradient down projection, base GEMM^T with fused up projection,
dB and dA reductions).  Inputs are synthetic, seeded and resident in HBM before timing starts; the
batch plan is built once outside the timed region (one packed batch shares its plan over every
layer).  Prints ONE JSON line.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3      # MI355X fp32 vector
PEAK_HBM_GBS = 8000.0
COLD_SETS = 3                 # independent (x, dy, y, dx) sets the cold figures rotate over


def measure_ceilings(torch, read_bytes):
    """What this chip sustains, measured here and now with the bench-only kernels of liblobra_ceilings.so: a loop
    of nothing but the GEMM's MFMA (random bf16 operands), and a streaming read / copy - of a buffer as large as
    one activation tensor, read again and again (it stays in the 256 MB infinity cache, like the inputs of the
    warm steps), and of a 1 GiB buffer (which does not)."""
    import ctypes
    path = os.path.join(ROOT, "paper_2509_01193_amd", "liblobra_ceilings.so")
    if not os.path.exists(path):
        raise FileNotFoundError(path + " is missing: build it with `python -m paper_2509_01193_amd.build`")
    L = ctypes.CDLL(path)
    vp = ctypes.c_void_p
    L.lobra_ceiling_mfma.argtypes = [vp, vp, ctypes.c_int, ctypes.c_int, vp]
    L.lobra_ceiling_read.argtypes = [vp, ctypes.c_size_t, vp, ctypes.c_int, vp]
    L.lobra_ceiling_copy.argtypes = [vp, vp, ctypes.c_size_t, ctypes.c_int, vp]
    dev = torch.device("cuda:0")
    st = vp(torch.cuda.current_stream().cuda_stream)
    ncu = torch.cuda.get_device_properties(0).multi_processor_count

    def t_of(fn, reps=5, warm=2):
        for _ in range(warm):
            assert fn() == 0
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            assert fn() == 0
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e-3

    ops = (torch.randn(64 * 64 * 8, device=dev) * 0.5).to(torch.bfloat16)       # 64 KiB of operands
    out = torch.empty(ncu * 256, dtype=torch.float32, device=dev)
    iters = 4000
    sec = t_of(lambda: L.lobra_ceiling_mfma(vp(ops.data_ptr()), vp(out.data_ptr()), ncu, iters, st))
    res = {"mfma_only_measured_tflops": ncu * 4 * iters * 64 * 2.0 * 16 * 16 * 32 / sec / 1e12}
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    wgs = ncu * 8
    n = max(read_bytes // 16 * 16, 64 << 20)
    a = torch.randint(0, 255, (n,), dtype=torch.uint8, device=dev)
    b = torch.empty_like(a)
    big = torch.empty(1 << 30, dtype=torch.uint8, device=dev).random_(0, 255)
    res["stream_read_warm_measured_gbs"] = n / t_of(lambda: L.lobra_ceiling_read(vp(a.data_ptr()), n, vp(sink.data_ptr()), wgs, st), 10, 3) / 1e9
    res["stream_read_cold_measured_gbs"] = (1 << 30) / t_of(lambda: L.lobra_ceiling_read(vp(big.data_ptr()), 1 << 30, vp(sink.data_ptr()), wgs, st), 4, 1) / 1e9
    res["stream_copy_measured_gbs"] = 2.0 * n / t_of(lambda: L.lobra_ceiling_copy(vp(a.data_ptr()), vp(b.data_ptr()), n, wgs, st), 10, 3) / 1e9
    res["stream_buffer_bytes"] = n
    return res


def cpu_baseline(p, budget_rows):
    """The fp64 oracle, as it stands, on a bounded sample of the same workload."""
    import numpy as np
    import oracle
    o = oracle.Oracle(p.x, p.W, p.A, p.B, p.s, p.dy, p.rank_off, p.seg_off, p.seg_task)
    rows = np.linspace(0, p.T - 1, budget_rows).astype(np.int64)
    t0 = time.perf_counter()
    o.y(rows)
    o.dx(rows)
    t_rows = time.perf_counter() - t0
    t0 = time.perf_counter()
    o.grads()
    t_grads = time.perf_counter() - t0
    per_token = t_rows / len(rows) + t_grads / p.T
    cores = int(os.environ.get("OMP_NUM_THREADS", 0)) or len(os.sched_getaffinity(0))
    out = {
        "value": 1.0 / per_token, "unit": "tokens/s", "cores": cores, "kind": "oracle",
        "sample": "y and dx of %d evenly spaced rows (%.2f s) + dA, dB over all %d tokens (%.2f s); "
                  "per-token cost = rows_time/rows + grads_time/T" % (len(rows), t_rows, p.T, t_grads),
    }
    # the same code on one thread (the OpenMP runtime's own switch; the oracle is not touched)
    try:
        import ctypes
        gomp = ctypes.CDLL("libgomp.so.1")
        gomp.omp_set_num_threads(1)
        try:
            rows1 = rows[:: max(1, cores)]
            t0 = time.perf_counter()
            o.y(rows1)
            o.dx(rows1)
            t_rows1 = time.perf_counter() - t0
            if t_grads * cores <= 20.0:
                t0 = time.perf_counter()
                o.grads()
                t_grads1 = time.perf_counter() - t0
                how = "dA, dB (%.2f s)" % t_grads1
            else:   # keep the run short: the full reductions on one thread would take about a minute
                t_grads1 = t_grads * cores
                how = "dA, dB not run on one thread (taken as threads x the time above)"
        finally:
            gomp.omp_set_num_threads(cores)
        out["value_1core"] = 1.0 / (t_rows1 / len(rows1) + t_grads1 / p.T)
        out["sample_1core"] = "%d rows (%.2f s) + %s" % (len(rows1), t_rows1, how)
    except OSError:
        pass
    return out


def read_traffic(workload, key="TRAFFIC_BYTES_PER_LAUNCH"):
    """HBM bytes per launch of a kernel from the committed rocprofv3 --pmc summary."""
    path = os.path.join(ROOT, "profiles", "gemm_%s_pmc.txt" % workload)
    try:
        m = re.search(r"^%s\s*=\s*([0-9.eE+]+)" % key, open(path).read(), re.M)
        return float(m.group(1)) if m else None
    except OSError:
        return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=2, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--order", default="shuffled", choices=["shuffled", "sorted"])
    ap.add_argument("--layout", default="packed", choices=["packed", "padded"],
                    help="padded: every sequence padded to one of --buckets boundaries chosen by "
                         "lobra_dynamic_buckets among multiples of 256 (pad tokens take the base product only); "
                         "`value` then counts the real tokens")
    ap.add_argument("--buckets", type=int, default=8)
    ap.add_argument("--projections", type=int, default=1,
                    help="P > 1: P LoRA linears that read the same x (q/k/v, gate/up) as ONE call - W "
                         "concatenated along d_out, A_t stacked along the rank, B_t compact (desc.n_proj = P) - "
                         "timed against P separate calls and against one call on block-diagonal up factors; "
                         "prints its own JSON line and exits")
    ap.add_argument("--oracle-rows", type=int, default=8192)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-graph", action="store_true",
                    help="time eager launches instead of replays of a HIP graph of one step")
    ap.add_argument("--vendor-gemm", action="store_true",
                    help="context only (the library never calls it): time torch.matmul on the two base products "
                         "of the workload, x @ W and dy @ W^T, next to this library's base-only step; prints its "
                         "own JSON line and exits")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="for rocprofv3 --pmc runs: 2 steps and one plain device copy of x (a kernel of "
                         "known traffic that calibrates FETCH_SIZE / WRITE_SIZE), then exit")
    a = ap.parse_args()
    if a.gpus != 1:
        sys.exit("bench.py measures one GPU: this build has no multi-GPU path (run with --gpus 1)")

    import numpy as np
    import torch
    from paper_2509_01193_amd import binding as bd
    from paper_2509_01193_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py needs a GPU")
    torch.cuda.set_device(0)
    p = wl.make_config(a.config, a.order, fill=(a.layout == "packed"))
    real_tokens, useful, layout_info = p.T, p.useful_flops(), {"layout": "packed"}   # pad tokens are not useful work
    if a.layout == "padded":
        lens = [L for L, _ in p.seqs if L > 0]
        cand = list(range(256, (max(lens) + 255) // 256 * 256 + 1, 256))
        bounds, pad = bd.lobra_dynamic_buckets(lens, cand, a.buckets)
        seqs = [(L, t) for L, t in p.seqs if L > 0]
        p = wl.pad_to_buckets(p, bounds, fill=False)
        # the chunk's segment table from the library's own helper (every sequence padded to its bucket boundary)
        so, stk, T = bd.lobra_padded_segments([L for L, _ in seqs], [t for _, t in seqs], p.n_tasks,
                                              [min(b for b in bounds if b >= L) for L, _ in seqs])
        assert T == p.T == real_tokens + pad
        p.seg_off, p.seg_task = so, stk
        p = p.fill()
        layout_info = {"layout": "padded", "bucket_bounds": bounds, "pad_tokens": pad, "real_tokens": real_tokens}
    t0 = time.perf_counter()
    dp = bd.DeviceProblem(p)
    torch.cuda.synchronize()

    if a.projections > 1:
        P = a.projections
        # (a) the fused call: stacked down factors, compact up factors, desc.n_proj = P
        df = bd.DeviceProblem(wl.fuse_projections(p, P))
        # (b) the same layers as ONE ordinary call on concatenated weights: up factors block-diagonal
        dense = wl.make_custom(p.name + "-dense-x%d" % P, p.dtype, p.d_in, P * p.d_out, P * p.ranks, p.seg_off,
                               p.seg_task, p.seed, s=p.s)
        fro = dense.rank_off
        for t in range(p.n_tasks):
            r = int(p.ranks[t])
            for j in range(P):
                rows = slice(int(fro[t]) + j * r, int(fro[t]) + (j + 1) * r)
                dense.B[rows, : j * p.d_out] = 0
                dense.B[rows, (j + 1) * p.d_out:] = 0
        dd = bd.DeviceProblem(dense)
        # (c) P separate calls
        parts = [dp] + [bd.DeviceProblem(p) for _ in range(P - 1)]

        def t_of(fn):
            for _ in range(a.warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(a.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / a.steps

        def separate():
            for q in parts:
                q.step()
        acc = torch.empty_like(dp.dx)

        def dx_sum():                       # what the caller of separate calls still owes: dx = sum of P partial dx
            torch.add(parts[0].dx, parts[1].dx, out=acc)
            for q in parts[2:]:
                acc.add_(q.dx)
        ms_sep, ms_sum, ms_dense, ms_fused = t_of(separate), t_of(dx_sum), t_of(dd.step), t_of(df.step)
        print(json.dumps({"projection_fusion": True, "projections": P, "workload": p.name,
                          "ms_per_step_fused_call": ms_fused, "ms_per_step_dense_concatenated_call": ms_dense,
                          "ms_per_step_separate_calls": ms_sep, "ms_dx_sum_after_separate_calls": ms_sum,
                          "tokens_per_s_fused": p.T / (ms_fused * 1e-3),
                          "speedup_vs_separate_plus_sum": (ms_sep + ms_sum) / ms_fused}))
        return

    if a.vendor_gemm:
        if p.dtype != "bf16":
            sys.exit("--vendor-gemm: bf16 workloads only")
        base = dp.base_only()
        x, W, dy = base.x, base.W, base.dy
        y, dx = torch.empty_like(dy), torch.empty_like(x)

        def t_of(fn):
            for _ in range(a.warmup):
                fn()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(a.steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / a.steps
        ms_fwd = t_of(lambda: torch.matmul(x, W, out=y))
        ms_bwd = t_of(lambda: torch.matmul(dy, W.t(), out=dx))
        ms_own = t_of(base.step)
        fl = 2.0 * p.T * p.d_in * p.d_out
        print(json.dumps({"vendor_gemm_context": True, "workload": p.name, "T": p.T, "d_in": p.d_in, "d_out": p.d_out,
                          "torch_matmul_x_W_ms": ms_fwd, "torch_matmul_x_W_tflops": fl / ms_fwd / 1e9,
                          "torch_matmul_dy_Wt_ms": ms_bwd, "torch_matmul_dy_Wt_tflops": fl / ms_bwd / 1e9,
                          "this_library_base_only_step_ms": ms_own,
                          "this_library_base_only_tflops": 2 * fl / ms_own / 1e9}))
        return

    if a.pmc_probe:
        dp.step()
        dp.step()
        ref = torch.empty_like(dp.x)
        ref.copy_(dp.x)          # reads and writes x.numel() * 2 bytes
        torch.cuda.synchronize()
        print(json.dumps({"pmc_probe": True, "copy_bytes_each_way": dp.x.numel() * dp.x.element_size()}))
        return

    ceilings = measure_ceilings(torch, p.T * p.d_in * (2 if p.dtype == "bf16" else 4))

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        w0 = time.perf_counter()
        e0.record()
        for _ in range(steps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - w0) * 1e3 / steps
        return wall, e0.elapsed_time(e1) / steps

    ms_wall_eager, ms_ev_eager = timed(dp.step, a.steps, a.warmup)
    # A training loop captures far more than one layer's step in a HIP graph (a whole stack of LoRA linears), so
    # the cost of starting a replay is spread over many kernels.  Here a graph holds `spg` steps (the largest
    # divisor of --steps up to 10) and is replayed steps / spg times: exactly --steps steps are timed.
    spg = max(g for g in range(1, 11) if a.steps % g == 0)

    def step_graph(q, n):
        q.step()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            with torch.cuda.graph(g, stream=side):
                for _ in range(n):
                    q.step()
        torch.cuda.synchronize()
        return g
    if a.no_graph:
        ms_wall, ms_ev = ms_wall_eager, ms_ev_eager
    else:
        side = torch.cuda.Stream()
        wall, ev = timed(step_graph(dp, spg).replay, a.steps // spg, -(-a.warmup // spg))
        ms_wall, ms_ev = wall / spg, ev / spg

    # the same library with no adapters: base GEMM time, for the LoRA overhead figure
    base = dp.base_only()
    if a.no_graph:
        ms_base_wall, ms_base = timed(base.step, a.steps, min(a.warmup, 3))
    else:
        ms_base_wall, ms_base = (t / spg for t in timed(step_graph(base, spg).replay, a.steps // spg, -(-min(a.warmup, 3) // spg)))

    # per-kernel durations from HIP events on the launch stream, over `steps` more passes
    tr = bd.LaunchTrace(dp.plan, 32)

    def traced(problems):
        per = {}
        for i in range(a.steps):
            tr.attach()
            problems[i % len(problems)].step()
            torch.cuda.synchronize()
            for name, ms in tr.durations():
                per.setdefault(name, []).append(ms)
        return {k: {"launches_per_step": len(v) // a.steps, "avg_ms": float(np.mean(v))} for k, v in per.items()}
    kern = traced([dp])

    # the same with inputs that no cache holds: the step rotates over COLD_SETS independent sets of x, dy, y, dx
    # (in a model every layer's activations are new; at workload 2 one set is 0.5 GB, twice the infinity cache)
    sets = [dp] + [dp.clone_io() for _ in range(COLD_SETS - 1)]
    bases = [q.base_only() for q in sets]
    kern_cold = traced(sets)
    tr.close()
    if a.no_graph:
        def rot(qs):
            def f():
                for q in qs:
                    q.step()
            return f
        ms_cold = timed(rot(sets), max(a.steps // COLD_SETS, 1), min(a.warmup, 2))[1] / COLD_SETS
        ms_base_cold = timed(rot(bases), max(a.steps // COLD_SETS, 1), min(a.warmup, 2))[1] / COLD_SETS
    else:
        def rot_graph(qs):
            for q in qs:
                q.step()
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    for q in qs:
                        q.step()
            torch.cuda.synchronize()
            return g
        ms_cold = timed(rot_graph(sets).replay, max(a.steps // COLD_SETS, 1), min(a.warmup, 2))[1] / COLD_SETS
        ms_base_cold = timed(rot_graph(bases).replay, max(a.steps // COLD_SETS, 1), min(a.warmup, 2))[1] / COLD_SETS

    # outside the step: the optimiser update that follows it, and the cost of building a batch plan
    extras = {}
    if p.R_tot:
        cfg = bd.AdamConfig(0.9, 0.999, 1e-8, 0.0)
        f = lambda shape: torch.zeros(shape, dtype=torch.float32, device=dp.dev)
        lr = torch.full((p.n_tasks,), 1e-4, dtype=torch.float32, device=dp.dev)
        stp = torch.ones((p.n_tasks,), dtype=torch.int32, device=dp.dev)
        mA, vA, mB, vB = f(dp.dA.shape), f(dp.dA.shape), f(dp.dB.shape), f(dp.dB.shape)
        wA, wB = dp.A.float(), dp.B.float()
        a2, b2 = dp.A.clone(), dp.B.clone()
        adam = lambda: bd.lobra_mlora_adam_step(dp.plan, cfg, lr, stp, None, dp.dA, dp.dB, wA, wB, mA, vA, mB, vB, a2, b2)
        extras["adam_step_ms"] = timed(adam, 20, 3)[1]
    t1 = time.perf_counter()
    for _ in range(5):
        bd.Plan.for_problem(p).close()
    extras["plan_create_ms"] = (time.perf_counter() - t1) * 1e3 / 5

    cnt = p.task_tokens()
    tok_rank = float((cnt * p.ranks).sum())
    flops = useful
    # dominant kernel: the fused GEMM (two launches per step: y and dx)
    gemm_flops = 0.5 * (4.0 * p.T * p.d_in * p.d_out + 2.0 * tok_rank * (p.d_in + p.d_out))
    gemm_ms = kern.get("gemm", {}).get("avg_ms", float("nan"))
    gemm_ms_cold = kern_cold.get("gemm", {}).get("avg_ms", float("nan"))
    peak = PEAK_BF16_TFLOPS if p.dtype == "bf16" else PEAK_FP32_TFLOPS
    achieved = gemm_flops / (gemm_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma" if p.dtype == "bf16" else "alu", "kernel": "gemm (base product + fused up projection)",
                "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                "traffic": read_traffic("cfg%d" % a.config), "avg_launch_ms": gemm_ms,
                "flops_per_launch": gemm_flops,
                "frac_cold": gemm_flops / (gemm_ms_cold * 1e-3) / 1e12 / peak, "avg_launch_ms_cold": gemm_ms_cold,
                # a loop of nothing but this kernel's MFMA, measured in this process before the timed region
                "mfma_only_measured_tflops": ceilings["mfma_only_measured_tflops"] if p.dtype == "bf16" else None}
    esz = 2 if p.dtype == "bf16" else 4
    skinny = {}
    # each of the two rank-r stages reads x once and dy once per step (algorithmic bytes); `traffic` is
    # the same launch by the HBM-side counters of the committed rocprofv3 --pmc summary
    # (long batches of ranks up to 16: dB is accumulated by the projection's pass over dy, so the reduction's
    #  stage 1 reads x alone)
    sliced = dp.plan.query(bd.Q_SLICED).tolist()
    fused_db = bool(sliced[2])
    for name in ("shrink", "grad_stage1"):
        if name in kern and kern[name]["launches_per_step"] > 0:
            step_bytes = float(esz) * p.T * (p.d_in if (fused_db and name == "grad_stage1") else p.d_in + p.d_out)
            per_launch = step_bytes / kern[name]["launches_per_step"]
            gbs = per_launch / (kern[name]["avg_ms"] * 1e-3) / 1e9
            gbs_cold = per_launch / (kern_cold[name]["avg_ms"] * 1e-3) / 1e9
            skinny[name] = {"bound": "hbm", "achieved": gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                            "frac": gbs / PEAK_HBM_GBS, "avg_launch_ms": kern[name]["avg_ms"],
                            "achieved_cold": gbs_cold, "frac_cold": gbs_cold / PEAK_HBM_GBS,
                            "avg_launch_ms_cold": kern_cold[name]["avg_ms"],
                            # a plain streaming read measured in this process: of a buffer this size that stays
                            # in the infinity cache, and of 1 GiB that does not
                            "stream_read_measured_gbs": ceilings["stream_read_warm_measured_gbs"],
                            "stream_read_cold_measured_gbs": ceilings["stream_read_cold_measured_gbs"],
                            "bytes_per_launch": per_launch,
                            "traffic": read_traffic("cfg%d" % a.config, "TRAFFIC_%s_BYTES_PER_LAUNCH" % name.upper())}
    out = {
        "metric": "multi-LoRA linear fwd+bwd tokens/s", "value": real_tokens / (ms_wall * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms_wall,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": p.dtype, "data": "synthetic",
        "launch": "eager" if a.no_graph else "hip_graph_replay", "steps_per_graph": 1 if a.no_graph else spg,
        "ms_per_step_eager": ms_wall_eager,
        "config": {"workload": p.name, "T": p.T, "d_in": p.d_in, "d_out": p.d_out,
                   "n_tasks": p.n_tasks, "ranks": sorted(set(int(r) for r in p.ranks)),
                   "segments": p.S, "order": a.order, **layout_info},
        "useful_tflops": flops / (ms_wall * 1e-3) / 1e12,
        "pct_of_peak": 100.0 * flops / (ms_wall * 1e-3) / 1e12 / peak,
        "ms_per_step_events": ms_ev, "ms_base_only": ms_base,
        "lora_overhead_pct": 100.0 * (ms_ev - ms_base) / ms_base,
        "ms_per_step_cold": ms_cold, "ms_base_only_cold": ms_base_cold,
        "lora_overhead_pct_cold": 100.0 * (ms_cold - ms_base_cold) / ms_base_cold,
        "tokens_per_s_cold": real_tokens / (ms_cold * 1e-3), "cold_sets": COLD_SETS,
        "ceilings": ceilings, "kernels_cold": kern_cold,
        "kernels": kern, "skinny_hbm": skinny, "extras": extras, "roofline": roofline,
        "rank_r_path": {"projection_slices_in": sliced[0], "projection_slices_out": sliced[1], "dB_fused_into_dy_pass": fused_db},
        "setup_s": time.perf_counter() - t0,
    }
    if not a.no_cpu_baseline:
        rows = a.oracle_rows if a.config == 2 else max(64, int(a.oracle_rows * (4096.0 * 4096) / (p.d_in * p.d_out)))
        out["cpu_baseline"] = cpu_baseline(p, min(rows, p.T))
    print(json.dumps(out))


if __name__ == "__main__":
    main()
