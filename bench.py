#!/usr/bin/env python3
"""NestedFP benchmark on one MI355X.

A *step* is one decode iteration of a random-init Llama-3-8B-shaped linear stack
(32 layers x {qkv, o, gate_up, down}, weights stored once as NestedFP byte planes) at
M tokens: every linear is run in FP16 mode (both planes, on-the-fly reconstruction),
then every linear is run in FP8 mode (per-token activation quantisation + upper plane
only).  The stack is 13.0 GiB of planes, so no weight is served from a cache between
steps.  The decomposition is offline in the paper (Sec. 4.1) and is timed separately.

Prints ONE JSON line: the whole-step algorithmic GB/s as `value`, the roofline of the
dominant kernel (FP16-mode streaming GEMM), the CPU oracle timed on the host cores, and
under `extra` the per-mode numbers, the plain same-family baselines and the
compute-bound (prefill) TFLOP/s of the same linears.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0            # MI355X HBM3E
MFMA_PEAK_TFLOPS = {"fp16": 2500.0, "fp8": 5000.0}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--tokens", type=int, default=16, help="decode batch M (tokens per step)")
    ap.add_argument("--layers", type=int, default=32)
    ap.add_argument("--no-prefill", action="store_true", help="skip the compute-bound extras")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--sweep-70b", action="store_true",
                    help="extra: roofline curve on the Llama-3-70B shapes, M = 1 ... 8192 (configs[3])")
    ap.add_argument("--mode-switch", action="store_true",
                    help="extra: per-step mode switching on the stack at M = 64 and 2048 (configs[4])")
    ap.add_argument("--paper-shapes", action="store_true",
                    help="extra: FP16-mode overhead over the plain FP16 GEMM on the shapes of the "
                         "paper's kernel benchmark, M = 32 ... 2048 step 32")
    ap.add_argument("--switch-demo", action="store_true",
                    help="extra: token-count threshold switching over a synthetic bursty arrival sequence")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a 1 GiB elementwise copy (known traffic) so that rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings can be scaled to bytes")
    return ap.parse_args()


def gemm_bytes(M, N, K, mode):
    """Algorithmic bytes of one GEMM call: planes read + X read + Y written."""
    w = 2 * N * K if mode == "fp16" else N * K
    return w + 2 * M * K + 2 * M * N


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the NestedFP hot path has no "
              "collective; see DESIGN.md for how it would shard); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2506_02024_amd import binding as nfp
    from paper_2506_02024_amd import workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    nfp.lib()                                   # fail loudly if the HIP library is missing

    M = args.tokens
    shapes = workloads.LLAMA3_8B
    names = list(shapes)

    # ---- build the stack: decompose once (offline step, timed on its own) -------------
    t_dec = 0.0
    dec_bytes = 0
    planes, plain_w = [], []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for layer in range(args.layers):
        for j, name in enumerate(names):
            N, K = shapes[name]
            W = workloads.weight_device(N, K, workloads.SIGMA_W_8B, seed=layer * 4 + j)
            up = nfp.PackedPlane(N, K, dev)
            lo = nfp.PackedPlane(N, K, dev)
            if layer == 0:
                nfp.decompose(W, up, lo, check=True)      # warm + applicability check
            e0.record()
            nfp.decompose(W, up, lo, check=False)
            e1.record()
            torch.cuda.synchronize()
            t_dec += e0.elapsed_time(e1) * 1e-3
            dec_bytes += 4 * N * K
            planes.append((name, up, lo))
            plain_w.append(W)
    # reconstruct timing on one layer
    t_rec, rec_bytes = 0.0, 0
    for j, name in enumerate(names):
        N, K = shapes[name]
        _, up, lo = planes[j]
        out = torch.empty((N, K), dtype=torch.float16, device=dev)
        nfp.reconstruct(up, lo, out)
        e0.record()
        nfp.reconstruct(up, lo, out)
        e1.record()
        torch.cuda.synchronize()
        assert torch.equal(out, plain_w[j])
        t_rec += e0.elapsed_time(e1) * 1e-3
        rec_bytes += 4 * N * K
        del out

    X = {name: workloads.act_device(M, shapes[name][1], seed=7 + j) for j, name in enumerate(names)}
    Y = {name: torch.empty((M, shapes[name][0]), dtype=torch.float16, device=dev) for name in names}
    ws_bytes = max(nfp.gemm_workspace_size(M, N, K, m) for (N, K) in shapes.values() for m in (0, 1))
    ws = torch.empty(ws_bytes + 256, dtype=torch.uint8, device=dev)
    # the same call on ONE layer over and over: its planes (48 MB for qkv) stay in the 256 MB
    # memory-side cache, so this is the hot-cache number, not an HBM rate
    hot = {}
    for j, name in enumerate(names[:4] if M <= 64 else []):
        N, K = shapes[name]
        _, up, lo = planes[j]
        t_hot = _time(torch, lambda i: nfp.gemm(X[name], up, lo, nfp.MODE_FP16, out=Y[name], workspace=ws))
        hot[name] = {"us": t_hot * 1e6, "GBps": gemm_bytes(M, N, K, "fp16") / t_hot / 1e9}

    def run_fp16():
        for name, up, lo in planes:
            nfp.gemm(X[name], up, lo, nfp.MODE_FP16, out=Y[name], workspace=ws)

    def run_fp8():
        for name, up, lo in planes:
            nfp.gemm(X[name], up, None, nfp.MODE_FP8, out=Y[name], workspace=ws)

    def run_plain16():
        for (name, _, _), W in zip(planes, plain_w):
            nfp.plain_gemm_fp16(X[name], W, out=Y[name], workspace=ws)

    def run_plain8():
        for name, up, lo in planes:
            nfp.plain_gemm_fp8(X[name], up, 2.0 ** -8, out=Y[name], workspace=ws)

    legs = {"fp16": run_fp16, "fp8": run_fp8, "plain_fp16": run_plain16, "plain_fp8": run_plain8}
    for fn in legs.values():                    # eager warm-up (also sets kernel attributes)
        fn()
    torch.cuda.synchronize()

    replay = {}
    if args.no_graph:
        replay = dict(legs)
    else:
        for key, fn in legs.items():
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn()
            replay[key] = g.replay
    torch.cuda.synchronize()

    n_calls = len(planes)
    step_bytes = {m: sum(gemm_bytes(M, *shapes[name], m) for name, _, _ in planes) for m in ("fp16", "fp8")}
    step_flops = sum(2.0 * M * shapes[name][0] * shapes[name][1] for name, _, _ in planes)

    def step():
        replay["fp16"]()
        replay["fp8"]()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps; per-leg HIP events on the launch stream
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        replay["fp16"]()
        ev[i][1].record()
        replay["fp8"]()
        ev[i][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_fp16 = sum(e[0].elapsed_time(e[1]) for e in ev) * 1e-3 / args.steps
    t_fp8 = sum(e[1].elapsed_time(e[2]) for e in ev) * 1e-3 / args.steps
    ms_per_step = wall / args.steps * 1e3
    value = (step_bytes["fp16"] + step_bytes["fp8"]) / (wall / args.steps) / 1e9

    # plain same-family baselines, same stack, same graphs
    def time_leg(key, reps):
        replay[key]()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            replay[key]()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / reps

    reps = max(3, args.steps // 3)
    t_plain16 = time_leg("plain_fp16", reps)
    t_plain8 = time_leg("plain_fp8", reps)

    extra = {
        "tokens": M,
        "gemm_calls_per_mode": n_calls,
        "fp16_mode": {"ms": t_fp16 * 1e3, "GBps": step_bytes["fp16"] / t_fp16 / 1e9,
                      "TFLOPs": step_flops / t_fp16 / 1e12,
                      "frac_hbm": step_bytes["fp16"] / t_fp16 / 1e9 / HBM_PEAK_GBPS,
                      "vs_plain_fp16": t_plain16 / t_fp16},
        "fp8_mode": {"ms": t_fp8 * 1e3, "GBps": step_bytes["fp8"] / t_fp8 / 1e9,
                     "TFLOPs": step_flops / t_fp8 / 1e12,
                     "frac_hbm": step_bytes["fp8"] / t_fp8 / 1e9 / HBM_PEAK_GBPS,
                     "vs_plain_fp8": t_plain8 / t_fp8},
        "plain_fp16": {"ms": t_plain16 * 1e3, "GBps": step_bytes["fp16"] / t_plain16 / 1e9},
        "plain_fp8": {"ms": t_plain8 * 1e3, "GBps": step_bytes["fp8"] / t_plain8 / 1e9},
        "decompose_offline": {"GBps": dec_bytes / t_dec / 1e9, "ms_total": t_dec * 1e3,
                              "frac_hbm": dec_bytes / t_dec / 1e9 / HBM_PEAK_GBPS},
        "reconstruct": {"GBps": rec_bytes / t_rec / 1e9, "frac_hbm": rec_bytes / t_rec / 1e9 / HBM_PEAK_GBPS},
        "fp16_mode_hot_cache_one_layer": hot,
        "mode_switch": "mode is a per-call argument on the same plane pointers; "
                       "torch.cuda.memory_allocated is constant across the timed region",
    }

    # roofline of the dominant kernel: the FP16-mode streaming GEMM (one launch per linear)
    traffic = read_traffic()
    roofline = {
        "kernel": "small_gemm_kernel<kNestedF16> (FP16-mode streaming GEMM, %d launches/step)" % n_calls,
        "bound": "hbm",
        "achieved": step_bytes["fp16"] / t_fp16 / 1e9,
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": step_bytes["fp16"] / t_fp16 / 1e9 / HBM_PEAK_GBPS,
        "traffic": traffic,
        "avg_launch_us": t_fp16 / n_calls * 1e6,
        "algorithmic_bytes_per_launch": step_bytes["fp16"] / n_calls,
    }

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.float32, device=dev)       # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    if not args.no_prefill:
        del replay, legs
        extra["prefill"] = prefill_extras(torch, nfp, workloads, planes, plain_w, dev)
    if args.mode_switch:
        extra["mode_switch_steps"] = mode_switch_extras(torch, nfp, workloads, planes, dev)
    if args.switch_demo:
        extra["switch_demo"] = switch_demo_extras(torch, nfp, workloads, planes, dev)
    del plain_w, planes
    torch.cuda.empty_cache()
    if args.sweep_70b:
        extra["sweep_70b"] = sweep_extras(torch, nfp, workloads, dev, workloads.LLAMA3_70B.items(),
                                          workloads.SIGMA_W_70B, [1 << i for i in range(14)])
    if args.paper_shapes:
        extra["paper_shapes"] = paper_shape_extras(torch, nfp, workloads, dev)

    cpu = None if args.no_cpu else cpu_baseline(workloads, M)

    line = {
        "metric": "NestedFP GEMM algorithmic GB/s over one decode step (FP16 mode + FP8 mode) "
                  "of a Llama-3-8B-shaped linear stack",
        "value": value,
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16/e4m3 operands, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": "configs[1]: Llama-3-8B-shaped linears qkv/o/gate_up/down x %d layers, "
                               "decode M=%d, FP16 mode then FP8 mode per step" % (args.layers, M),
                   "tokens": M, "layers": args.layers, "hip_graph": not args.no_graph},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "extra": extra,
    }
    print(json.dumps(line))


def read_traffic():
    """HBM bytes per launch of the dominant kernel from the committed counter summary
    (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel); None if absent."""
    path = os.path.join(ROOT, "profiles", "small_gemm_nested_f16_decode_traffic.txt")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch="):
                return float(line.split("=", 1)[1])
    except OSError:
        pass
    return None


def prefill_extras(torch, nfp, workloads, planes, plain_w, dev):
    """Compute-bound regime (configs[2]): the same four linears at M in {512, 2048, 8192}."""
    shapes = workloads.LLAMA3_8B
    out = {}
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    n_layers = len(planes) // 4
    for M in workloads.PREFILL_M:
        row = {}
        for j, name in enumerate(shapes):
            N, K = shapes[name]
            X = workloads.act_device(M, K, seed=70 + j)
            Yb = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = torch.empty(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + 256,
                             dtype=torch.uint8, device=dev)
            flops = 2.0 * M * N * K
            res = {}
            for key in ("fp16", "plain_fp16", "fp8", "plain_fp8"):
                reps = 8 if M >= 2048 else 16

                def call(i):
                    _, up, lo = planes[(i % n_layers) * 4 + j]     # rotate layers: cold weights
                    if key == "fp16":
                        nfp.gemm(X, up, lo, nfp.MODE_FP16, out=Yb, workspace=ws)
                    elif key == "plain_fp16":
                        nfp.plain_gemm_fp16(X, plain_w[(i % n_layers) * 4 + j], out=Yb, workspace=ws)
                    elif key == "fp8":
                        nfp.gemm(X, up, None, nfp.MODE_FP8, out=Yb, workspace=ws)
                    else:
                        nfp.plain_gemm_fp8(X, up, 2.0 ** -8, out=Yb, workspace=ws)

                call(0)
                call(1)
                torch.cuda.synchronize()
                a.record()
                for i in range(reps):
                    call(i)
                b.record()
                torch.cuda.synchronize()
                t = a.elapsed_time(b) * 1e-3 / reps
                peak = MFMA_PEAK_TFLOPS["fp16" if "16" in key else "fp8"]
                res[key] = {"us": t * 1e6, "TFLOPs": flops / t / 1e12, "frac_mfma": flops / t / 1e12 / peak}
            res["fp16_vs_plain"] = res["plain_fp16"]["us"] / res["fp16"]["us"]
            res["fp8_vs_plain"] = res["plain_fp8"]["us"] / res["fp8"]["us"]
            row[name] = res
            del X, Yb, ws
        out["M=%d" % M] = row
    return out


def _time(torch, call, budget_s=0.03, max_reps=64):
    """Seconds per call: two warm-up calls, then enough back-to-back calls for ~budget_s."""
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    call(0)
    torch.cuda.synchronize()
    a.record()
    call(1)
    b.record()
    torch.cuda.synchronize()
    one = max(a.elapsed_time(b) * 1e-3, 1e-6)
    reps = int(min(max_reps, max(3, budget_s / one)))
    a.record()
    for i in range(reps):
        call(2 + i)
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) * 1e-3 / reps


def _layer_copies(torch, nfp, workloads, N, K, sigma, dev, seed0):
    """Enough copies of one layer that neither L2 nor the 256 MB cache can serve the weights."""
    copies = int(min(8, max(2, -(-600e6 // (2 * N * K)))))
    Ws = [workloads.weight_device(N, K, sigma, seed=seed0 + i) for i in range(copies)]
    return Ws, [nfp.decompose(W, check=(i == 0)) for i, W in enumerate(Ws)]


def sweep_extras(torch, nfp, workloads, dev, shapes, sigma, Ms):
    """Roofline curve: both modes and the plain FP16 baseline over M on each shape; the bound of
    a point is max(algorithmic bytes / 8 TB/s, flops / MFMA peak of the mode)."""
    out = {}
    for j, (name, (N, K)) in enumerate(shapes):
        Ws, planes = _layer_copies(torch, nfp, workloads, N, K, sigma, dev, 300 + 10 * j)
        R = len(Ws)
        row = {}
        for M in Ms:
            X = workloads.act_device(M, K, seed=90 + j)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = torch.empty(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + 256,
                             dtype=torch.uint8, device=dev)
            t16 = _time(torch, lambda i: nfp.gemm(X, planes[i % R][0], planes[i % R][1], nfp.MODE_FP16, out=Y, workspace=ws))
            t8 = _time(torch, lambda i: nfp.gemm(X, planes[i % R][0], None, nfp.MODE_FP8, out=Y, workspace=ws))
            tp = _time(torch, lambda i: nfp.plain_gemm_fp16(X, Ws[i % R], out=Y, workspace=ws))
            fl = 2.0 * M * N * K
            lb16 = max(gemm_bytes(M, N, K, "fp16") / (HBM_PEAK_GBPS * 1e9), fl / (MFMA_PEAK_TFLOPS["fp16"] * 1e12))
            lb8 = max(gemm_bytes(M, N, K, "fp8") / (HBM_PEAK_GBPS * 1e9), fl / (MFMA_PEAK_TFLOPS["fp8"] * 1e12))
            row["M=%d" % M] = {
                "fp16_us": t16 * 1e6, "fp8_us": t8 * 1e6, "plain_fp16_us": tp * 1e6,
                "fp16_GBps": gemm_bytes(M, N, K, "fp16") / t16 / 1e9, "fp8_GBps": gemm_bytes(M, N, K, "fp8") / t8 / 1e9,
                "fp16_TFLOPs": fl / t16 / 1e12, "fp8_TFLOPs": fl / t8 / 1e12,
                "fp16_frac_roofline": lb16 / t16, "fp8_frac_roofline": lb8 / t8,
                "fp16_vs_plain": tp / t16}
            del X, Y, ws
        out["%s (%d,%d)" % (name, N, K)] = row
        del Ws, planes
        torch.cuda.empty_cache()
    return out


def paper_shape_extras(torch, nfp, workloads, dev):
    """Sec. 5.2 / App. C of the paper sweep M = 32 ... 2048 in steps of 32 on four (N,K) shapes
    and quote the mean slowdown of FP16 mode against a plain FP16 GEMM; same sweep here."""
    out = {}
    for j, (N, K) in enumerate(workloads.PAPER_KERNEL_SHAPES):
        Ws, planes = _layer_copies(torch, nfp, workloads, N, K, workloads.SIGMA_W_8B, dev, 500 + 10 * j)
        R = len(Ws)
        over = []
        for M in range(32, 2049, 32):
            X = workloads.act_device(M, K, seed=95 + j)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = torch.empty(nfp.gemm_workspace_size(M, N, K, 0) + 256, dtype=torch.uint8, device=dev)
            t16 = _time(torch, lambda i: nfp.gemm(X, planes[i % R][0], planes[i % R][1], nfp.MODE_FP16, out=Y, workspace=ws), 0.01, 16)
            tp = _time(torch, lambda i: nfp.plain_gemm_fp16(X, Ws[i % R], out=Y, workspace=ws), 0.01, 16)
            over.append((M, t16 / tp - 1.0, 2.0 * M * N * K / t16 / 1e12))
            del X, Y, ws
        o = [x[1] for x in over]
        big = [x[1] for x in over if x[0] > 64]
        out["(%d,%d)" % (N, K)] = {
            "mean_overhead": sum(o) / len(o), "min_overhead": min(o), "max_overhead": max(o),
            "mean_overhead_tiled_kernel_M>64": sum(big) / len(big),
            "fp16_TFLOPs_at_M=2048": over[-1][2],
            "overhead_at": {"M=%d" % m: ov for m, ov, _ in over if m in (32, 64, 128, 256, 512, 1024, 2048)}}
        del Ws, planes
        torch.cuda.empty_cache()
    return out


def _run_stack(nfp, planes, X, Y, ws, mode):
    for name, up, lo in planes:
        nfp.gemm(X[name], up, None if mode == nfp.MODE_FP8 else lo, mode, out=Y[name], workspace=ws)


def _stack_buffers(torch, nfp, workloads, M, dev):
    shapes = workloads.LLAMA3_8B
    X = {n: workloads.act_device(M, shapes[n][1], seed=60 + j) for j, n in enumerate(shapes)}
    Y = {n: torch.empty((M, shapes[n][0]), dtype=torch.float16, device=dev) for n in shapes}
    need = max(nfp.gemm_workspace_size(M, N, K, m) for (N, K) in shapes.values() for m in (0, 1))
    return X, Y, torch.empty(need + 256, dtype=torch.uint8, device=dev)


def mode_switch_extras(torch, nfp, workloads, planes, dev):
    """Sec. 5.4: the mode is chosen per iteration.  64 steps over the whole stack, the mode
    flipping every 8 steps, at M = 64 and M = 2048: step time by mode, the first step after a
    flip against the steady state, allocated device memory before and after."""
    out = {}
    for M in (64, 2048):
        X, Y, ws = _stack_buffers(torch, nfp, workloads, M, dev)
        for mode in (nfp.MODE_FP16, nfp.MODE_FP8):
            _run_stack(nfp, planes, X, Y, ws, mode)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(65)]
        modes = []
        ev[0].record()
        for step in range(64):
            mode = nfp.MODE_FP8 if (step // 8) % 2 else nfp.MODE_FP16
            modes.append(mode)
            _run_stack(nfp, planes, X, Y, ws, mode)
            ev[step + 1].record()
        torch.cuda.synchronize()
        t = [ev[i].elapsed_time(ev[i + 1]) for i in range(64)]
        first = [t[i] for i in range(8, 64) if i % 8 == 0]
        steady = {m: [t[i] for i in range(64) if modes[i] == m and i % 8 != 0] for m in (nfp.MODE_FP16, nfp.MODE_FP8)}
        out["M=%d" % M] = {
            "fp16_step_ms": sum(steady[nfp.MODE_FP16]) / len(steady[nfp.MODE_FP16]),
            "fp8_step_ms": sum(steady[nfp.MODE_FP8]) / len(steady[nfp.MODE_FP8]),
            "first_step_after_switch_ms": first,
            "allocated_bytes_before": before, "allocated_bytes_after": torch.cuda.memory_allocated()}
        del X, Y, ws
    return out


def switch_demo_extras(torch, nfp, workloads, planes, dev):
    """Sec. 5.4's policy on a synthetic arrival sequence (the paper's trace is not available):
    a step whose token count reaches 1024 runs in FP8 mode, the others in FP16 mode."""
    import numpy as np

    rng = np.random.default_rng(7)
    choices = np.array([16, 32, 64, 128, 256, 512, 1024, 2048, 4096])
    # mostly small decode steps with bursts of large prefill-heavy steps
    seq = [int(choices[min(8, int(abs(rng.normal(0, 1.6)) + (4 if rng.random() < 0.25 else 0)))]) for _ in range(48)]
    bufs = {M: _stack_buffers(torch, nfp, workloads, M, dev) for M in sorted(set(seq))}
    res = {}
    for policy in ("always_fp16", "always_fp8", "threshold_1024"):
        def mode_of(M):
            if policy == "always_fp16":
                return nfp.MODE_FP16
            if policy == "always_fp8":
                return nfp.MODE_FP8
            return nfp.MODE_FP8 if M >= 1024 else nfp.MODE_FP16
        for M in bufs:                                   # warm every kernel once
            _run_stack(nfp, planes, *bufs[M], mode_of(M))
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for M in seq:
            _run_stack(nfp, planes, *bufs[M], mode_of(M))
        b.record()
        torch.cuda.synchronize()
        res[policy] = {"total_ms": a.elapsed_time(b), "fp8_steps": sum(1 for M in seq if mode_of(M) == nfp.MODE_FP8)}
    res["tokens_per_step"] = seq
    return res


def cpu_baseline(workloads, M):
    """The CPU oracle as it stands, timed on this host's cores: one layer (the four
    linears) in FP16 mode and in FP8 mode at the benchmark's M -- 1/32 of a step."""
    import numpy as np

    import oracle

    shapes = workloads.LLAMA3_8B
    cores = int(os.environ.get("OMP_NUM_THREADS", "0")) or (os.cpu_count() or 1)
    nbytes = 0
    inputs = []
    for j, (name, (N, K)) in enumerate(shapes.items()):
        W = workloads.weight_host(N, K, workloads.SIGMA_W_8B, seed=j)
        Xh = workloads.act_host(M, K, seed=7 + j)
        inputs.append((W, Xh))
    ups = [oracle.decompose(W)[0] for W, _ in inputs]   # offline step, not timed
    t_fp16 = t_fp8 = 0.0
    passes = 0
    while passes < 16 and t_fp16 + t_fp8 < 10.0:        # about 10-20 s of CPU work
        t0 = time.perf_counter()
        for W, Xh in inputs:
            N, K = W.shape
            oracle.gemm_fp16(Xh, W)
            nbytes += 2 * N * K + 2 * M * K + 2 * M * N
        t1 = time.perf_counter()
        for (W, Xh), up in zip(inputs, ups):
            N, K = W.shape
            Xq, s = oracle.quantize_act(Xh)
            oracle.gemm_fp8(Xq, s, up)
            nbytes += N * K + 2 * M * K + 2 * M * N
        t2 = time.perf_counter()
        t_fp16 += t1 - t0
        t_fp8 += t2 - t1
        passes += 1
    return {
        "value": nbytes / (t_fp16 + t_fp8) / 1e9,
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle",
        "sample": "%d pass(es) over one layer of the stack (qkv, o, gate_up, down) at M=%d, FP16 mode "
                  "then FP8 mode, each pass 1/32 of a step; %.1f s FP16 mode, %.1f s FP8 mode"
                  % (passes, M, t_fp16, t_fp8),
    }


if __name__ == "__main__":
    main()
