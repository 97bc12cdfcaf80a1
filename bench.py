#!/usr/bin/env python3
"""Benchmark of the batched LQR hot path on one MI355X.

A "step" is one pass of the whole hot path (ttc_lqr_solve: load, setup, reverse symplectic steps,
re-bases, final solve, outputs) over every problem of the workload, inputs resident in HBM.
Prints ONE JSON line: problems/s plus a roofline object for the solve kernel (fp32 MFMA) and the CPU
oracle timed on the host cores on a bounded sample of the same inputs.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config llm_adapter] [--n N] [--rebase-every k]
                    [--path symplectic|doubling|tv|cxt|scan|bwd|rollout|grid|block|cxtbwd]

The headline value is the paper's sequential symplectic product (--path symplectic, the default); the same
inputs are also timed on the squaring path and reported under "other_path".
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix peak (256 CUs x 256 flop/clk x 2.4 GHz)
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "traffic.json")


def source_hash():
    """Identifies the build of the kernels: a hash over the HIP sources and their build script (what a measured traffic figure belongs to)."""
    import hashlib
    h = hashlib.sha256()
    folder = os.path.join(ROOT, "paper_2603_09221_amd", "csrc")
    files = [os.path.join(folder, name) for name in sorted(os.listdir(folder))]
    files.append(os.path.join(ROOT, "paper_2603_09221_amd", "build.py"))   # the compile flags of every unit
    for path in files:
        with open(path, "rb") as f:
            h.update(os.path.basename(path).encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def measured_traffic(workload, path, n):
    """HBM bytes per launch from the rocprofv3 FETCH_SIZE / WRITE_SIZE summaries recorded in profiles/traffic.json
    (bytes per problem x n), or None when no row matches this workload and path or the row was measured on
    another build of the kernels."""
    try:
        with open(TRAFFIC_FILE) as f:
            rows = json.load(f)["rows"]
    except (OSError, ValueError, KeyError):
        return None
    cur = source_hash()
    for r in rows:
        if r.get("workload") == workload and r.get("path") == path and r.get("source_hash") == cur:
            return r["bytes_per_problem"] * n
    return None


def cpu_model():
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("model name"):
                    return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def spread(kernel_ms):
    """Median and 20 / 80 % percentiles of the per-launch durations (the paper reports its timings this way)."""
    import numpy as np
    a = np.asarray(kernel_ms, dtype=np.float64)
    return {"kernel_ms_median": float(np.median(a)), "kernel_ms_p20": float(np.percentile(a, 20)),
            "kernel_ms_p80": float(np.percentile(a, 80))}


def default_groups(T, dtype):
    """The library default: number of groups the T factors are split into (one dense solve each): groups of five
    factors for bfloat16 inputs; for float32 inputs groups of three with at most one group of four."""
    return (T + 4) // 5 if dtype == "bf16" else max((T + 1) // 3, (T * 10 + 33) // 34)


def alg_flops(d, T, groups):
    """Algorithmic flops of one problem (2*M*N*K per product): what the re-based symplectic method
    has to compute, not what the kernel happens to execute.
      setup   R^{-1}B^T factor d^3/3, G = B R^{-1} B^T 3 d^3, A^{-1} 2 d^3, C_K = R^{-1}B^T A^{-T} 2 d^3
      steps   T-1 reverse symplectic steps of 4 products (8 d^3 each), the last factor (Q_0 = 0) 3 products
      re-base one pivoted solve Y1^{-1} Y2 per group (the last one yields P_0): 8/3 d^3 each
      output  K_0 = -C_K P_0: 2 d^3
    """
    return (1.0 / 3 + 3 + 2 + 2 + 8 * (T - 1) + 6 + (8.0 / 3) * groups + 2) * d ** 3


def alg_flops_doubling(d, T):
    """Algorithmic flops of one problem on the long-horizon (squaring) path with Q_T = Q: the schedule
    of ttc_lqr_solve under TTC_FLAG_DOUBLING, counted product by product.
      setup    R^{-1}B^T factor d^3/3, G = B R^{-1} B^T 3 d^3
      squaring 8 products + one solve with d right-hand sides (8/3 d^3); the last one, of which only H
               is needed, 3 products + solve
      apply    P <- H + A^T (I + P G)^{-1} P A: 3 products + solve (free while P = 0)
      last     the same with the gain: 4 products + solve
    """
    f, m, have_p = 1.0 / 3 + 3, T, False
    while m:
        if m & 1:
            if have_p:
                f += 6 + 8.0 / 3
            have_p = True
        m >>= 1
        if m:
            f += (6 if (m == 1 and not have_p) else 16) + 8.0 / 3
    return (f + 8 + 8.0 / 3) * d ** 3


def alg_flops_tv(d, T):
    """Algorithmic flops of one time-heterogeneous problem (ttc_lqr_solve_tv): per step the six products of the
    printed Riccati step (P A, P B, B^T P A, B^T P B, A^T P A, F^T W: 2 d^3 each) and the solve with the positive
    definite S (factor d^3/3, d right-hand sides 2 d^3)."""
    return T * (12 + 7.0 / 3) * d ** 3


def alg_flops_rollout(d, T):
    """Rollout (Alg. 1): the backward recursion of Prop. 3.1 with every gain kept (the per-step work of
    alg_flops_tv), then the forward pass: K_t x, A x + B u and the stage cost per step."""
    return alg_flops_tv(d, T) + T * 8 * d * d


def alg_flops_bwd(d, T):
    """Algorithmic flops of one backward pass (ttc_lqr_backward): T-1 steps of the backward recursion of Prop. 3.1
    (six products and a positive definite solve with d right-hand sides, as alg_flops_tv), the first step's
    S_0 = R + B^T P_1 B (two products) and its solve with two right-hand sides (factor d^3/3); the closed loops, the
    co-states and the outer products are O(T d^2) and not counted."""
    return ((T - 1) * (12 + 7.0 / 3) + 4 + 1.0 / 3) * d ** 3


def alg_flops_cxt(d, r, T):
    """Algorithmic flops of one structured problem (ttc_lqr_solve_cxt): combining the bases (three sums of r
    matrices, 2 r d^2 each), then per step four products (P B, B^T V, S^{-1} F, F^T K: 2 d^3 each) and the
    in-place inverse of S (2 d^3); the diagonal scalings are O(d^2) and not counted."""
    return 6 * r * d * d + T * 10 * d ** 3


def bench_cxt(args):
    """The structured, contextualised layer shape of the paper's language-model runs: d = 16, 16 heads, r = 16
    basis matrices, horizon 8 (the mean of its training horizons); batch 8 x 16 heads x 8192 tokens."""
    import numpy as np
    import torch
    from paper_2603_09221_amd import binding, synth
    from paper_2603_09221_amd.errors import rel_err

    d, r, T = 16, 16, args.horizon or 8
    n = args.n or 8 * 16 * 8192
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()
    b = synth.make_contextual_batch(n, d, r, T, seed=0, device=dev)
    keys = synth.ContextualBatch.PER_PROBLEM + ("Bbasis", "Qbasis", "x0")
    ins = [getattr(b, k) for k in keys]
    out = {"P0": torch.empty((n, d, d), dtype=torch.float32, device=dev),
           "K0": torch.empty((n, d, d), dtype=torch.float32, device=dev),
           "u0": torch.empty((n, d), dtype=torch.float32, device=dev),
           "value": torch.empty((n,), dtype=torch.float32, device=dev),
           "info": torch.empty((n,), dtype=torch.int32, device=dev)}
    stream = torch.cuda.current_stream()
    if args.calib_copy_mib:
        src = torch.ones((args.calib_copy_mib << 18,), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    step = lambda: binding.ttc_lqr_solve_cxt(*ins, T, out=out, stream=stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record(stream)
        step()
        e1.record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    kernel_ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    assert int(out["info"].abs().max()) == 0, "a problem reported numerical breakdown"
    flops_pp = alg_flops_cxt(d, r, T)
    achieved = flops_pp * n / kernel_s / 1e12
    in_bytes = n * (6 * d + 3 * r) * 4 + 2 * r * d * d * 4
    out_bytes = n * (2 * d * d + d + 2) * 4
    res = {
        "metric": "LQR solves/sec (tokens x heads x batch problems) at d=%d, T=%d, structured parameters" % (d, T),
        "value": n / wall, "unit": "problems/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "ttc_layer_d16", "problems": n, "d": d, "m": d, "r": r, "T": T, "input_dtype": "f32",
                   "path": "cxt", "outputs": "P0,K0,u0,value"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                     "traffic": measured_traffic("ttc_layer_d16_T%d" % T, "cxt", n),
                     "kernel": "solve_cxt_kernel", "kernel_ms": kernel_s * 1e3, **spread(kernel_ms),
                     "alg_flops_per_problem": flops_pp,
                     "nominal_TFLOPs_N_T_d3": n * T * d ** 3 / kernel_s / 1e12,
                     "alg_bytes_per_launch": in_bytes + out_bytes,
                     "alg_GBps": (in_bytes + out_bytes) / kernel_s / 1e9},
    }
    if not args.no_cpu:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import lqr_oracle
        cores = min(16, os.cpu_count() or 1)

        def run(sample):
            a = b.take(slice(0, sample)).numpy64()
            chunks = [ix for ix in np.array_split(np.arange(sample), cores * 4) if len(ix)]

            def work(ix):
                r_ = lqr_oracle.contextual_solve(*(x[ix] for x in a[:8]), a[8], a[9], a[10][ix], T)
                return {k: r_[k] for k in ("P0", "K0", "u0", "value")}
            t1 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=cores) as ex:
                parts = list(ex.map(work, chunks))
            return {k: np.concatenate([p_[k] for p_ in parts]) for k in parts[0]}, time.perf_counter() - t1
        pilot = min(n, 4096)
        _, pdt = run(pilot)
        sample = min(n, args.cpu_sample or int(max(pilot, pilot * 15.0 / max(pdt, 1e-3))))
        ref, dt = run(sample)
        errs = {k: float(rel_err(out[k][:sample].cpu().numpy(), ref[k]).max()) for k in ("P0", "K0", "u0", "value")}
        res["cpu_baseline"] = {"value": sample / dt, "unit": "problems/s", "cores": cores, "kind": "oracle",
                               "cpu_model": cpu_model(),
                               "sample": "first %d problems of the same workload, float64 numpy (parameters "
                                         "expanded to dense steps, then Riccati), %.1f s wall" % (sample, dt)}
        res["parity"] = {"sample": sample, "max_rel_err": errs, "tolerance": 1e-4}
    print(json.dumps(res))


def alg_flops_block(C, H, d, r, T):
    """Algorithmic flops of the whole block for one token: the two projections (2 C H d each), the contextualisation
    maps of every head (2 d (5 d + 3 r)), the heads' structured problems; normalisations and activations are O(C)
    and not counted."""
    return 4 * C * H * d + H * (2 * d * (5 * d + 3 * r) + alg_flops_cxt(d, r, T))


def bench_block(args):
    """The whole TTC block at the width of the paper's 7B language-model runs: token features of 4096 numbers, 16
    heads of d = 16, r = 16 basis matrices, horizon 8; 8 x 8192 tokens (the problems of --path cxt, with the layer
    normalisations, projections and contextualisation maps around them)."""
    import numpy as np
    import torch
    from paper_2603_09221_amd import binding, synth
    from paper_2603_09221_amd.errors import rel_err

    C, H, d, r, T = 4096, 16, 16, 16, args.horizon or 8
    n = args.n or 8 * 8192
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lib = binding.load()
    w = synth.make_block_weights(C, H, d, r, seed=0, device=dev)
    x = synth.make_block_input(n, C, seed=0, device=dev)
    bf16 = args.block_dtype == "bf16"   # token features and the two projection matrices stored in bfloat16
    if bf16:
        w["W_in"], w["W_out"] = w["W_in"].bfloat16().contiguous(), w["W_out"].bfloat16().contiguous()
        x = x.bfloat16().contiguous()
    esz = 2 if bf16 else 4
    out = {"x_out": torch.empty_like(x), "info": torch.empty((n, H), dtype=torch.int32, device=dev)}
    blk = binding.make_block(w, n, T)
    ws = torch.empty(lib.ttc_block_workspace_bytes(blk), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    if args.calib_copy_mib:
        src = torch.ones((args.calib_copy_mib << 18,), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    step = lambda: binding.ttc_block_forward(x, w, T, out=out, workspace=ws, stream=stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record(stream)
        step()
        e1.record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    kernel_ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    assert int(out["info"].abs().max()) == 0, "a problem reported numerical breakdown"
    flops_pt = alg_flops_block(C, H, d, r, T)
    achieved = flops_pt * n / kernel_s / 1e12
    alg_bytes = 2 * n * C * esz + 2 * C * H * d * esz
    res = {
        "metric": "TTC block forward tokens/sec at C=%d, %d heads of d=%d, T=%d" % (C, H, d, T),
        "value": n / wall, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "ttc_block_c4096" + ("_bf16" if bf16 else ""), "tokens": n, "C": C, "heads": H, "d": d, "r": r,
                   "T": T, "problems": n * H, "path": "block", "input_dtype": args.block_dtype},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                     "traffic": measured_traffic("ttc_block_c4096%s_T%d" % ("_bf16" if bf16 else "", T), "block", n * H),   # the table's unit is the (token, head) problem
                     "kernel": "ttc_block_forward (7 launches: ln_stats, gemm_ln, cxt_maps, qbasis, solve_cxt, ln_stats, gemm_ln)",
                     "kernel_ms": kernel_s * 1e3, **spread(kernel_ms),
                     "alg_flops_per_token": flops_pt,
                     "alg_flops_split": {"projections": 4 * C * H * d, "maps": H * 2 * d * (5 * d + 3 * r),
                                         "solves": H * alg_flops_cxt(d, r, T)},
                     "alg_bytes_per_launch": alg_bytes, "alg_GBps": alg_bytes / kernel_s / 1e9},
    }
    if not args.no_cpu:
        from concurrent.futures import ThreadPoolExecutor
        from oracle import ttc_block_oracle
        cores = min(16, os.cpu_count() or 1)
        w64 = {k: v.float().cpu().double().numpy() for k, v in w.items()}   # the oracle consumes the stored values

        def run(sample):
            xs = x[:sample].float().cpu().double().numpy()
            chunks = [ix for ix in np.array_split(np.arange(sample), cores * 4) if len(ix)]
            t1 = time.perf_counter()
            with ThreadPoolExecutor(max_workers=cores) as ex:
                parts = list(ex.map(lambda ix: ttc_block_oracle.ttc_block(xs[ix], w64, T)["x_out"], chunks))
            return np.concatenate(parts), time.perf_counter() - t1
        pilot = min(n, 256)
        _, pdt = run(pilot)
        sample = min(n, args.cpu_sample or int(max(pilot, pilot * 15.0 / max(pdt, 1e-3))))
        ref, dt = run(sample)
        err = float(rel_err(out["x_out"][:sample].float().cpu().numpy(), ref).max())
        res["cpu_baseline"] = {"value": sample / dt, "unit": "tokens/s", "cores": cores, "kind": "oracle",
                               "cpu_model": cpu_model(),
                               "sample": "first %d tokens of the same workload, float64 numpy, %.1f s wall" % (sample, dt)}
        res["parity"] = {"sample": sample, "max_rel_err": {"x_out": err}, "tolerance": 2e-2 if bf16 else 1e-4}
    print(json.dumps(res))


def bench_cxt_bwd(args):
    """Backward pass of the structured layer shape (ttc_lqr_backward_cxt): d = 16, r = 16, horizon 8, 8 x 16 heads x 8192
    tokens.  Its arithmetic is the forward pass's recursion once more (on the matrix cores) and a sweep on vectors."""
    import numpy as np
    import torch
    from paper_2603_09221_amd import binding, synth
    from paper_2603_09221_amd.errors import rel_err

    d, r, T = 16, 16, args.horizon or 8
    n = args.n or 8 * 16 * 8192
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    lib = binding.load()
    b = synth.make_contextual_batch(n, d, r, T, seed=0, device=dev)
    keys = synth.ContextualBatch.PER_PROBLEM + ("Bbasis", "Qbasis", "x0")
    ins = [getattr(b, k) for k in keys]
    g = torch.randn((n, d), generator=torch.Generator(device=dev).manual_seed(1), device=dev)
    out = binding.ttc_lqr_backward_cxt(*ins, T, g)          # allocates the outputs once
    prob = binding.make_cxt_problem(*ins, T)
    ws = torch.empty(lib.ttc_lqr_backward_cxt_workspace_bytes(prob), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    if args.calib_copy_mib:
        src = torch.ones((args.calib_copy_mib << 18,), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    step = lambda: binding.ttc_lqr_backward_cxt(*ins, T, g, out=out, workspace=ws, stream=stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record(stream)
        step()
        e1.record(stream)
    torch.cuda.synchronize()
    wall = (time.perf_counter() - t0) / args.steps
    kernel_ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    assert int(out["info"].abs().max()) == 0, "a problem reported numerical breakdown"
    # bytes the path moves by construction: per problem the T + 3 matrices and the dual problem's first control that the
    # solve kernel leaves and the sweep reads, the four trajectories written and read (horizons past 15 only: shorter
    # ones stay in LDS), the three kept matrices written and read, inputs and outputs
    traj = 0 if T <= 15 else 2 * 4 * (T + 1) * d * 4
    path_bytes = n * (2 * (T + 3) * d * d * 4 + 2 * d * 4 + traj + 2 * 3 * d * d * 4 + 2 * (6 * d + 3 * r) * 4 + 2 * (6 * d + 3 * r) * 4)
    achieved = path_bytes / kernel_s / 1e9
    res = {
        "metric": "LQR backward passes/sec at d=%d, T=%d, structured parameters" % (d, T),
        "value": n / wall, "unit": "problems/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "ttc_layer_d16", "problems": n, "d": d, "m": d, "r": r, "T": T, "input_dtype": "f32",
                   "path": "cxtbwd", "outputs": "gsA,gsB,gsQ,gsQf,grinv,glgA,glgB,glgQ,gx0,gBbasis,gQbasis"},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": 8000.0, "unit": "GB/s", "frac": achieved / 8000.0,
                     "traffic": measured_traffic("ttc_layer_d16_T%d" % T, "cxtbwd", n),
                     "kernel": "ttc_lqr_backward_cxt (solve_cxt_kernel, backward_cxt_vec_kernel, cxt_basis_kernel per chunk)",
                     "kernel_ms": kernel_s * 1e3, **spread(kernel_ms),
                     "alg_bytes_per_launch": path_bytes,
                     "alg_flops_per_problem": alg_flops_cxt(d, r, T),
                     "alg_TFLOPs": alg_flops_cxt(d, r, T) * n / kernel_s / 1e12},
    }
    if not args.no_cpu:
        from oracle import lqr_grad_oracle
        sample = min(n, args.cpu_sample or 2048)
        sub = b.take(slice(0, sample))
        t1 = time.perf_counter()
        ref = lqr_grad_oracle.contextual_gradients(*sub.numpy64(), T, g[:sample].cpu().double().numpy())
        dt = time.perf_counter() - t1
        errs = {k: float(rel_err(out[k][:sample].cpu().numpy(), ref[k]).max()) for k in ("gsA", "grinv", "glgA", "glgB", "glgQ", "gx0")}
        res["cpu_baseline"] = {"value": sample / dt, "unit": "problems/s", "cores": 1, "kind": "oracle", "cpu_model": cpu_model(),
                               "sample": "first %d problems of the same workload, float64 numpy, %.1f s wall" % (sample, dt)}
        res["parity"] = {"sample": sample, "max_rel_err": errs, "tolerance": 2e-5}
    print(json.dumps(res))


def bench_grid(args):
    """The paper's solver benchmark grid (App. "Efficiency Benchmark": d = 16, horizon 2^4 .. 2^11 at batch 1024, batch
    2^4 .. 2^13 at horizon 64), forward and backward, time-heterogeneous dense steps: milliseconds per call (median
    of the timed calls) and the paper's nominal rate B T d^3 / time."""
    import numpy as np
    import torch
    from paper_2603_09221_amd import binding, synth

    d = 16
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()
    stream = torch.cuda.current_stream()
    combos = [(1024, 2 ** e) for e in range(4, 12)] + [(2 ** e, 64) for e in range(4, 14) if 2 ** e != 1024]
    rows = []
    for B, T in combos:
        b = synth.make_tv_batch(B, d, d, T, seed=0, device=dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(1)
        g = torch.randn((B, d), generator=gen, dtype=torch.float32, device=dev)
        fwd = binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, b.R, b.x0, stream=stream)
        need = binding.load().ttc_lqr_backward_tv_workspace_bytes(binding.make_tv_problem(b.A, b.B, b.Q, b.R, b.x0))
        ws = torch.empty((max(need, 16),), dtype=torch.uint8, device=dev)
        bwd = binding.ttc_lqr_backward_tv(b.A, b.B, b.Q, b.R, b.x0, g, workspace=ws, stream=stream)

        def med(fn):
            for _ in range(max(args.warmup, 2)):
                fn()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(max(args.steps, 5))]
            for e0, e1 in evs:
                e0.record(stream)
                fn()
                e1.record(stream)
            torch.cuda.synchronize()
            return float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
        f_ms = med(lambda: binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, b.R, b.x0, out=fwd, stream=stream))
        b_ms = med(lambda: binding.ttc_lqr_backward_tv(b.A, b.B, b.Q, b.R, b.x0, g, out=bwd, workspace=ws, stream=stream))
        assert int(fwd["info"].abs().max()) == 0 and int(bwd["info"].abs().max()) == 0
        nominal = B * T * d ** 3 / 1e9   # GFLOP in the paper's unit
        rows.append({"B": B, "T": T, "fwd_ms": f_ms, "bwd_ms": b_ms, "fwd_bwd_ms": f_ms + b_ms,
                     "nominal_TFLOPs_fwd_bwd": nominal / (f_ms + b_ms)})
        del b, fwd, bwd, ws
    print(json.dumps({"metric": "paper solver benchmark grid, d=16, forward + backward, time-heterogeneous dense steps",
                      "unit": "ms per call", "n_gpus": 1, "dtype": "f32", "data": "synthetic", "rows": rows}))


def alg_flops_scan(d, T):
    """Algorithmic flops of one problem on the pairwise path (ttc_lqr_solve_tv_scan): T-1 elements (R^{-1}B^T:
    d^3/3 + 2 d^3, G: 2 d^3), T-1 compositions (eight products and a dense solve with d right-hand sides:
    16 d^3 + 8/3 d^3) and the last step as printed (6 products and a positive definite solve)."""
    return ((T - 1) * (13.0 / 3 + 16 + 8.0 / 3) + 12 + 7.0 / 3) * d ** 3


def bench_scan(args):
    """The small-batch, long-horizon corner of the paper's solver benchmark grid (d = 16, B = 16, T = 2048),
    time-heterogeneous dense parameters, factors composed pairwise over the horizon."""
    import numpy as np
    import torch
    from oracle import lqr_oracle
    from paper_2603_09221_amd import binding, synth
    from paper_2603_09221_amd.errors import rel_err

    d, T = 16, args.horizon or 2048
    n = args.n or 16
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()
    b = synth.make_tv_batch(n, d, d, T, seed=0, device=dev)
    ws = torch.empty((n * T * 3 * d * d * 4,), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()
    if args.calib_copy_mib:
        src = torch.ones((args.calib_copy_mib << 18,), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    out = binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, b.R, b.x0, workspace=ws, stream=stream)
    seq = binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, b.R, b.x0, stream=stream)

    def timed(fn, steps, warmup):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for e0, e1 in evs:
            e0.record(stream)
            fn()
            e1.record(stream)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps, sum(e0.elapsed_time(e1) for e0, e1 in evs) / len(evs) / 1e3
    steps = max(args.steps, 20)
    wall, dev_s = timed(lambda: binding.ttc_lqr_solve_tv_scan(b.A, b.B, b.Q, b.R, b.x0, out=out, workspace=ws,
                                                              stream=stream), steps, max(args.warmup, 3))
    swall, sdev_s = timed(lambda: binding.ttc_lqr_solve_tv(b.A, b.B, b.Q, b.R, b.x0, out=seq, stream=stream), 3, 1)
    assert int(out["info"].abs().max()) == 0
    # every P_t and K_t by the up-sweep and the down-sweep (ttc_lqr_tv_scan_values), and the sequential roll-out's
    # backward part for comparison is the sequential solve above
    need = binding.load().ttc_lqr_tv_scan_values_workspace_bytes(binding.make_tv_problem(b.A, b.B, b.Q, b.R, b.x0))
    wsv = torch.empty((need,), dtype=torch.uint8, device=dev)
    vwall, vdev_s = timed(lambda: binding.ttc_lqr_tv_scan_values(b.A, b.B, b.Q, b.R, b.x0, workspace=wsv, stream=stream),
                          max(3, steps // 4), 2)
    flops_pp = alg_flops_scan(d, T)
    achieved = flops_pp * n / dev_s / 1e12
    rounds = max(0, math.ceil(math.log2(T)))
    in_bytes = n * (T * 4 * d * d + d) * 4
    out_bytes = n * (2 * d * d + d + 2) * 4
    res = {
        "metric": "LQR solves/sec at d=%d, T=%d, batch %d, time-heterogeneous, pairwise product" % (d, T, n),
        "value": n / wall, "unit": "problems/s", "n_gpus": 1, "steps": steps, "warmup": max(args.warmup, 3),
        "ms_per_step": wall * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "paper_grid_d16_B%d_T%d" % (n, T), "problems": n, "d": d, "m": d, "T": T,
                   "input_dtype": "f32", "path": "scan", "outputs": "P0,K0,u0,value"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_MFMA_TFLOPS, "traffic": None,
                     "kernel": "scan_leaf_kernel<16> + %d x scan_combine_kernel<16> + solve_tv_kernel<16> "
                               "(one call; latency-bound: %d dependent launches)" % (rounds, rounds + 2),
                     "kernel_ms": dev_s * 1e3, "alg_flops_per_problem": flops_pp,
                     "nominal_TFLOPs_N_T_d3": n * T * d ** 3 / dev_s / 1e12,
                     "alg_bytes_per_launch": in_bytes + out_bytes,
                     "alg_GBps": (in_bytes + out_bytes) / dev_s / 1e9},
        "other_path": {"path": "sequential (ttc_lqr_solve_tv)", "value": n / swall, "unit": "problems/s",
                       "kernel_ms": sdev_s * 1e3},
        "all_values": {"call": "ttc_lqr_tv_scan_values (every P_t and K_t: up-sweep, down-sweep, gains)",
                       "kernel_ms": vdev_s * 1e3, "launches": 3 + 2 * rounds},
    }
    if not args.no_cpu:
        A, B, Q, R, x0 = b.numpy64()
        t1 = time.perf_counter()
        ref = lqr_oracle.riccati_solve_tv(A, B, Q, R, x0)
        dt = time.perf_counter() - t1
        errs = {k: float(rel_err(out[k].cpu().numpy(), ref[k]).max()) for k in ("P0", "K0", "u0", "value")}
        res["cpu_baseline"] = {"value": n / dt, "unit": "problems/s", "cores": 1, "kind": "oracle",
                               "cpu_model": cpu_model(),
                               "sample": "all %d problems, float64 numpy Riccati, batched over problems in one "
                                         "thread, %.2f s wall" % (n, dt)}
        res["parity"] = {"sample": n, "max_rel_err": errs, "tolerance": 1e-4}
    print(json.dumps(res))


def cpu_baseline(batch, sample, want_seconds=(10.0, 30.0)):
    """The oracle, as it stands, on the host cores: one problem chunk per thread, BLAS single-threaded."""
    import numpy as np
    import torch
    from concurrent.futures import ThreadPoolExecutor
    from oracle import lqr_oracle
    try:
        from threadpoolctl import threadpool_limits
    except Exception:  # pragma: no cover
        threadpool_limits = None
    cores = min(16, os.cpu_count() or 1)
    sub = batch.take(slice(0, sample))
    A, B, Q, R, x0 = sub.numpy64()
    chunks = np.array_split(np.arange(sample), cores * 4)

    def work(ix):
        if len(ix) == 0:
            return None
        if A.ndim == 4:   # time-heterogeneous batch
            r = lqr_oracle.riccati_solve_tv(A[ix], B[ix], Q[ix], R[ix], x0[ix])
        else:
            r = lqr_oracle.riccati_solve(A[ix], B[ix], Q[ix], R[ix], None, x0[ix], sub.T)
        return ix, {k: r[k] for k in ("P0", "K0", "u0", "value")}

    import contextlib
    limit = threadpool_limits(limits=1) if threadpool_limits else contextlib.nullcontext()
    with limit:
        t0 = time.perf_counter()
        with ThreadPoolExecutor(max_workers=cores) as ex:
            parts = [p for p in ex.map(work, chunks) if p is not None]
        dt = time.perf_counter() - t0
    ref = {k: np.concatenate([p[1][k] for p in parts]) for k in ("P0", "K0", "u0", "value")}
    return ref, dt, cores


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--config", default="llm_adapter")
    ap.add_argument("--chunk", type=int, default=None, help="problems per launch (default: the whole workload, or "
                    "the largest power-of-two split whose outputs fit the card)")
    ap.add_argument("--path", default="symplectic", choices=("symplectic", "doubling", "tv", "cxt", "scan", "bwd", "rollout", "grid", "block", "cxtbwd"),
                    help="symplectic: the paper's reverse symplectic iteration with re-basing (headline); "
                         "doubling: the long-horizon path, the same product formed by squaring; "
                         "tv: time-heterogeneous parameters (ttc_lqr_solve_tv) on the configuration's shape, "
                         "every step with its own A, B, Q, R (default 16384 problems); "
                         "cxt: structured, contextualised parameters (ttc_lqr_solve_cxt) at d = 16, r = 16, "
                         "1048576 problems, --config ignored; "
                         "scan: ttc_lqr_solve_tv_scan at d = 16, 16 problems, horizon 2048, --config ignored; "
                         "bwd: the backward pass (ttc_lqr_backward) on the configuration's shape (default up to "
                         "131072 problems); grid: the paper's solver benchmark grid at d = 16, forward and backward "
                         "(prints a table, not a bench line); rollout: ttc_lqr_rollout (all T controls, states and the cost) "
                         "on the configuration's shape (default up to 16384 problems); block: the whole TTC block (ttc_block_forward) at "
                         "4096 features, 16 heads of d = 16, 65536 tokens, --config ignored; cxtbwd: the backward pass of the structured "
                         "problems (ttc_lqr_backward_cxt), d = 16, r = 16, 1048576 problems, --config ignored")
    ap.add_argument("--horizon", type=int, default=None, help="horizon of the cxt (default 8) and scan (default 2048) paths")
    ap.add_argument("--block-dtype", default="f32", choices=("f32", "bf16"),
                    help="--path block: token features and projection matrices in float32 or bfloat16")
    ap.add_argument("--no-extra", action="store_true", help="skip the extra timing of the other path")
    ap.add_argument("--n", type=int, default=None, help="number of problems (default: the whole configuration)")
    ap.add_argument("--rebase-every", type=int, default=0, help="0 = library default")
    ap.add_argument("--cpu-sample", type=int, default=None)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one device-to-device copy of this many MiB (a kernel of known traffic, "
                         "to calibrate rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (problems are independent: a multi-GPU run would split "
              "the batch and exchange nothing). Re-run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    if args.path == "block":
        return bench_block(args)
    if args.path == "cxtbwd":
        return bench_cxt_bwd(args)
    if args.path == "cxt":
        return bench_cxt(args)
    if args.path == "scan":
        return bench_scan(args)
    if args.path == "grid":
        return bench_grid(args)

    import numpy as np
    import torch
    from paper_2603_09221_amd import binding, synth
    from paper_2603_09221_amd.errors import rel_err

    cfg = synth.CONFIGS[args.config]
    path = args.path
    full = synth.config_problems(args.config)
    n = args.n or (min(16384, full) if path in ("tv", "rollout") else min(131072, full) if path == "bwd" else full)
    d, m, T = cfg["d"], cfg["m"], cfg["T"]
    k = args.rebase_every
    groups = math.ceil(T / k) if k else default_groups(T, cfg["dtype"])
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load()

    if path == "tv":
        batch = synth.make_tv_batch(n, d, m, T, seed=0, device=dev, dtype=cfg["dtype"])
        args.no_extra = True
    else:
        batch = synth.make_batch(n, d, m, T, seed=0, device=dev, dtype=cfg["dtype"], rho=cfg["rho"])
    if path in ("bwd", "rollout"):
        args.no_extra = True
    esize = batch.A.element_size()
    # Outputs are held for one chunk of problems at a time (inputs for the whole workload stay resident): a step
    # launches the chunks one after the other on the same stream.  One chunk unless inputs plus outputs of the
    # whole workload would not fit the card.
    out_pp = (4 * d * d + d + 1) * 4 if path == "bwd" else (T * m + (T + 1) * d + 2) * 4 if path == "rollout" else \
        (d * d + m * d + m + 2) * 4
    free_bytes = torch.cuda.mem_get_info(dev)[0]
    chunk = n
    while chunk > 1 and chunk * out_pp > 0.85 * free_bytes:
        chunk = (chunk + 1) // 2
    if args.chunk:
        chunk = min(n, args.chunk)
    nchunks = (n + chunk - 1) // chunk
    f32 = dict(dtype=torch.float32, device=dev)
    if path == "bwd":
        out = {kk: torch.empty((chunk, d, d), **f32) for kk in ("gA", "gB", "gQ", "gR")}
        out["gx0"] = torch.empty((chunk, d), **f32)
        out["info"] = torch.empty((chunk,), dtype=torch.int32, device=dev)
        gen = torch.Generator(device=dev)
        gen.manual_seed(1)
        grad_u0 = torch.randn((n, m), generator=gen, **f32)
    else:
        out = {"P0": torch.empty((chunk, d, d), **f32), "K0": torch.empty((chunk, m, d), **f32),
               "u0": torch.empty((chunk, m), **f32), "value": torch.empty((chunk,), **f32),
               "info": torch.empty((chunk,), dtype=torch.int32, device=dev)}
    dbl = binding.TTC_FLAG_DOUBLING
    main_flags = dbl if path == "doubling" else 0
    if path == "tv":
        ws_bytes = 16
    elif path == "rollout":
        ws_bytes = binding.ttc_lqr_workspace_bytes(
            binding.make_problem(batch.A, batch.B, batch.Q, batch.R, None, batch.x0, T), True)
    elif path == "bwd":
        ws_bytes = binding.load().ttc_lqr_backward_workspace_bytes(
            binding.make_problem(batch.A, batch.B, batch.Q, batch.R, None, batch.x0, T))
    else:
        ws_bytes = max(binding.ttc_lqr_workspace_bytes(
            binding.make_problem(batch.A, batch.B, batch.Q, batch.R, None, batch.x0, T, f, k)) for f in (0, dbl))
    ws = torch.empty((max(ws_bytes, 16),), dtype=torch.uint8, device=dev)
    stream = torch.cuda.current_stream()

    def view(t, lo, hi):
        return {kk: v[:hi - lo] for kk, v in t.items()}

    def launch(flags, lo, hi):
        sub = batch.take(slice(lo, hi))
        o = view(out, lo, hi)
        if path == "tv":
            binding.ttc_lqr_solve_tv(sub.A, sub.B, sub.Q, sub.R, sub.x0, out=o, stream=stream)
        elif path == "bwd":
            binding.ttc_lqr_backward(sub.A, sub.B, sub.Q, sub.R, None, sub.x0, T, grad_u0[lo:hi], out=o, workspace=ws,
                                     stream=stream)
        elif path == "rollout":
            out.update(binding.ttc_lqr_rollout(sub.A, sub.B, sub.Q, sub.R, None, sub.x0, T, workspace=ws, stream=stream))
        else:
            binding.ttc_lqr_solve(sub.A, sub.B, sub.Q, sub.R, None, sub.x0, T, flags=flags, rebase_every=k, out=o,
                                  workspace=ws, stream=stream)

    def timed(flags, steps, warmup):
        """warmup untimed + steps timed passes over the whole workload; (wall s per step, kernel ms per step)"""
        def step():
            for c in range(nchunks):
                launch(flags, c * chunk, min(n, (c + 1) * chunk))
        for _ in range(warmup):
            step()
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        t0 = time.perf_counter()
        for e0, e1 in evs:
            e0.record(stream)      # HIP events on the stream the kernels are launched on
            step()
            e1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        kernel_ms = [e0.elapsed_time(e1) for e0, e1 in evs]   # nchunks kernel launches per step, back to back
        assert int(out["info"].abs().max()) == 0, "a problem reported numerical breakdown"
        return wall / steps, kernel_ms

    if args.calib_copy_mib:
        src = torch.ones((args.calib_copy_mib << 18,), dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        dst.copy_(src)          # reads and writes calib_copy_mib MiB each
        torch.cuda.synchronize()
        del src, dst
    wall_per_step, kernel_ms = timed(main_flags, args.steps, args.warmup)
    avg_kernel_s = sum(kernel_ms) / len(kernel_ms) / 1e3
    ms_per_step = wall_per_step * 1e3
    value = n / wall_per_step

    flops_pp = {"doubling": alg_flops_doubling(d, T), "tv": alg_flops_tv(d, T), "bwd": alg_flops_bwd(d, T),
                "rollout": alg_flops_rollout(d, T)}.get(path) \
        or alg_flops(d, T, groups)
    achieved = flops_pp * n / avg_kernel_s / 1e12
    steps_in = T if path == "tv" else 1          # every step has its own matrices on the tv path
    in_bytes = n * (steps_in * (2 * d * d + d * m + m * m) + d) * esize + (n * m * 4 if path == "bwd" else 0)
    out_bytes = n * out_pp
    kernel_name = {"doubling": "doubling_kernel<%d>", "tv": "solve_tv_kernel<%d>", "bwd": "backward_kernel<%d>",
                   "rollout": "rollout_kernel<%d>"}.get(
        path, "solve_kernel<%d>") % d if d != 16 or path in ("doubling", "bwd", "rollout") else (
        "solve_tv_small_kernel" if path == "tv" else "solve_small_kernel")
    res = {
        "metric": "LQR backward passes/sec (gradients of a loss of u0) at d=%d, T=%d" % (d, T) if path == "bwd" else
                  "LQR rollouts/sec (all controls, states and the cost) at d=%d, T=%d" % (d, T) if path == "rollout" else
                  "LQR solves/sec (tokens x heads x batch problems) at d=%d, T=%d" % (d, T),
        "value": value, "unit": "problems/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": args.config, "problems": n, "d": d, "m": m, "T": T, "input_dtype": cfg["dtype"],
                   "path": path, "rebase_every": None if path != "symplectic" else (k or "default"),
                   "groups": groups if path == "symplectic" else None, "chunks": nchunks,
                   "outputs": "gA,gB,gQ,gR,gx0" if path == "bwd" else "U,X,cost" if path == "rollout" else "P0,K0,u0,value"},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_FP32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_FP32_MFMA_TFLOPS,
                     "traffic": measured_traffic(args.config, path, n),
                     "kernel": kernel_name, "launches_per_step": nchunks,
                     "kernel_ms": avg_kernel_s * 1e3, **spread(kernel_ms),
                     "alg_flops_per_problem": flops_pp,
                     "nominal_TFLOPs_N_T_d3": n * T * d ** 3 / avg_kernel_s / 1e12,
                     "alg_bytes_per_launch": (in_bytes + out_bytes) / nchunks,
                     "alg_GBps": (in_bytes + out_bytes) / avg_kernel_s / 1e9},
    }
    tol = 1e-4 if cfg["dtype"] == "f32" else 2e-2
    sample, ref = 0, None
    if not args.no_cpu and path == "bwd":
        from oracle import lqr_grad_oracle
        sample = min(n, chunk, args.cpu_sample or {16: 4096, 32: 1024, 64: 256, 128: 48}[d])
        launch(0, 0, sample)
        torch.cuda.synchronize()
        sub = batch.take(slice(0, sample))
        A, B, Q, R, x0 = sub.numpy64()
        g64 = grad_u0[:sample].cpu().double().numpy()
        t1 = time.perf_counter()
        ref = lqr_grad_oracle.lqr_gradients(A, B, Q, R, None, x0, T, g64)
        dt = time.perf_counter() - t1
        errs = {kk: float(rel_err(out[kk][:sample].cpu().numpy().reshape(sample, -1), ref[kk].reshape(sample, -1)).max())
                for kk in ("gA", "gB", "gQ", "gR", "gx0")}
        res["cpu_baseline"] = {"value": sample / dt, "unit": "problems/s", "cores": 1, "kind": "oracle",
                               "cpu_model": cpu_model(),
                               "sample": "first %d problems of the same workload, float64 numpy (Thm 3.2: primal and "
                                         "dual LQR), batched over problems in one thread, %.1f s wall" % (sample, dt)}
        res["parity"] = {"sample": sample, "max_rel_err": errs, "tolerance": 2e-5 if cfg["dtype"] == "f32" else 2e-3}
    elif not args.no_cpu and path == "rollout":
        from oracle import lqr_oracle
        sample = min(n, chunk, args.cpu_sample or {16: 8192, 32: 2048, 64: 512, 128: 96}[d])
        launch(0, 0, sample)
        torch.cuda.synchronize()
        A, B, Q, R, x0 = batch.take(slice(0, sample)).numpy64()
        t1 = time.perf_counter()
        ref = dict(zip(("U", "X", "cost"), lqr_oracle.riccati_rollout(A, B, Q, R, None, x0, T)))
        dt = time.perf_counter() - t1
        errs = {kk: float(rel_err(out[kk][:sample].cpu().numpy().reshape(sample, -1),
                                  np.asarray(ref[kk]).reshape(sample, -1)).max()) for kk in ("U", "X", "cost")}
        res["cpu_baseline"] = {"value": sample / dt, "unit": "problems/s", "cores": 1, "kind": "oracle",
                               "cpu_model": cpu_model(),
                               "sample": "first %d problems of the same workload, float64 numpy (Alg. 1), batched "
                                         "over problems in one thread, %.1f s wall" % (sample, dt)}
        res["parity"] = {"sample": sample, "max_rel_err": errs, "tolerance": tol}
    elif not args.no_cpu:
        cores_guess = min(16, os.cpu_count() or 1)
        pilot = min(n, cores_guess * 8)
        _, pilot_dt, _ = cpu_baseline(batch, pilot)             # calibrate: aim at ~15 s of wall-clock
        sample = min(n, chunk, args.cpu_sample or int(max(pilot, pilot * 15.0 / max(pilot_dt, 1e-3))))
        ref, dt, cores = cpu_baseline(batch, sample)
        launch(main_flags, 0, sample)                            # the first chunk again: its outputs are compared
        torch.cuda.synchronize()
        errs = {kk: float(rel_err(out[kk][:sample].cpu().numpy(), ref[kk]).max()) for kk in ("P0", "K0", "u0", "value")}
        res["cpu_baseline"] = {"value": sample / dt, "unit": "problems/s", "cores": cores, "kind": "oracle",
                               "cpu_model": cpu_model(),
                               "sample": "first %d problems of the same workload, float64 numpy Riccati, "
                                         "%.1f s wall" % (sample, dt)}
        res["parity"] = {"sample": sample, "max_rel_err": errs, "tolerance": tol}
    if not args.no_extra:
        # the other path on the same inputs, for comparison (never the headline value)
        other = "doubling" if path == "symplectic" else "symplectic"
        o_wall, o_ms = timed(dbl if other == "doubling" else 0, max(1, min(args.steps, 2)), 1)
        o_kernel = sum(o_ms) / len(o_ms) / 1e3
        o_flops = alg_flops_doubling(d, T) if other == "doubling" else alg_flops(d, T, groups)
        extra = {"path": other, "value": n / o_wall, "unit": "problems/s", "kernel_ms": o_kernel * 1e3,
                 "alg_flops_per_problem": o_flops, "achieved_TFLOPs": o_flops * n / o_kernel / 1e12,
                 "frac_of_peak": o_flops * n / o_kernel / 1e12 / PEAK_FP32_MFMA_TFLOPS}
        if ref is not None:
            launch(dbl if other == "doubling" else 0, 0, sample)
            torch.cuda.synchronize()
            extra["max_rel_err"] = {kk: float(rel_err(out[kk][:sample].cpu().numpy(), ref[kk]).max())
                                    for kk in ("P0", "K0", "u0", "value")}
        res["other_path"] = extra
    print(json.dumps(res))


if __name__ == "__main__":
    main()
