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
under `extra`: both plane layouts (row-major planes as the format defines them, and the
library's optional packed pre-pack) next to plain FP16 / FP8 GEMMs of the same kernel
family in both layouts, what the chip sustains for a pure read stream and a pure MFMA
loop in the same run, the compute-bound (prefill) table, a subset of the Llama-3-70B
sweep and the mode-alternation run.  Every comparison is timed interleaved, burst by
burst, and reported as the median over the bursts with the spread beside it.
"""
import argparse
import json
import os
import statistics
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
    ap.add_argument("--layout", choices=("packed", "rowmajor"), default="packed",
                    help="plane storage the timed step runs on (the other one is reported under extra)")
    ap.add_argument("--bursts", type=int, default=7, help="repetitions per comparison (median is reported)")
    ap.add_argument("--no-prefill", action="store_true", help="skip the compute-bound extras")
    ap.add_argument("--no-vendor", action="store_true", help="leave the vendor library's GEMMs out of the compute-bound extras")
    ap.add_argument("--no-70b", action="store_true", help="skip the Llama-3-70B subset (configs[3])")
    ap.add_argument("--no-mode-switch", action="store_true", help="skip the mode-alternation run (configs[4])")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying HIP graphs")
    ap.add_argument("--sweep-70b", action="store_true",
                    help="extra: full roofline curve on the Llama-3-70B shapes, M = 1 ... 8192 (configs[3])")
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


def bound_seconds(M, N, K, mode):
    """max(algorithmic bytes / HBM peak, flops / MFMA peak of the mode)."""
    return max(gemm_bytes(M, N, K, mode) / (HBM_PEAK_GBPS * 1e9), 2.0 * M * N * K / (MFMA_PEAK_TFLOPS[mode] * 1e12))


def stats(ts):
    """median / min / max of a list of seconds, in microseconds."""
    return {"us": statistics.median(ts) * 1e6, "min_us": min(ts) * 1e6, "max_us": max(ts) * 1e6, "bursts": len(ts)}


class Timer:
    """Interleaved timing: for every burst, each named call runs `launches` times back to back
    between two events; the kinds alternate burst by burst, so drift (clocks, temperature) hits
    all of them alike.  Returns per kind the list of seconds per launch, one entry per burst."""

    def __init__(self, torch):
        self.torch = torch

    def run(self, calls, launches, bursts, warm=1):
        torch = self.torch
        for _ in range(warm):
            for fn in calls.values():
                fn(0)
        torch.cuda.synchronize()
        out = {k: [] for k in calls}
        pairs = {k: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(bursts)]
                 for k in calls}
        for b in range(bursts):
            for k, fn in calls.items():
                a, e = pairs[k][b]
                a.record()
                for i in range(launches):
                    fn(b * launches + i)
                e.record()
        torch.cuda.synchronize()
        for k in calls:
            out[k] = [a.elapsed_time(e) * 1e-3 / launches for a, e in pairs[k]]
        return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the NestedFP hot path has no "
              "collective: column-parallel layers shard the planes by rows, row-parallel ones by K); --gpus %d is not supported"
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
    timer = Timer(torch)

    M = args.tokens
    L = args.layout
    shapes = workloads.LLAMA3_8B
    names = list(shapes)

    # ---- build the stack: decompose once (the offline step of Sec. 4.1) ------------------
    stack = []                                  # per linear: name, W, row-major planes, packed planes, packed FP16
    for layer in range(args.layers):
        for j, name in enumerate(names):
            N, K = shapes[name]
            W = workloads.weight_device(N, K, workloads.SIGMA_W_8B, seed=layer * 4 + j)
            ent = {"name": name, "W": W}
            for key, packed in (("rowmajor", False), ("packed", True)):
                ent[key] = nfp.decompose(W, packed=packed, check=(layer == 0))     # applicability checked once per shape
            ent["Wp"] = nfp.pack_fp16(W)
            stack.append(ent)
    # decompose / reconstruct rates: one layer's four linears per launch burst, replayed as a HIP
    # graph so that the host's call overhead (larger than the kernels of the small linears) stays
    # out of the measurement; both layouts interleaved
    dec_bytes = rec_bytes = sum(4 * N * K for N, K in shapes.values())
    rec_out = {name: torch.empty(shapes[name], dtype=torch.float16, device=dev) for name in names}

    def dec_leg(key):
        def run():
            for ent in stack[:4]:
                nfp.decompose(ent["W"], ent[key][0], ent[key][1], check=False)
        return run

    def rec_leg(key):
        def run():
            for ent in stack[:4]:
                nfp.reconstruct(ent[key][0], ent[key][1], rec_out[ent["name"]])
        return run

    aux = {"decompose/rowmajor": dec_leg("rowmajor"), "decompose/packed": dec_leg("packed"),
           "reconstruct/rowmajor": rec_leg("rowmajor"), "reconstruct/packed": rec_leg("packed")}
    aux_replay = {}
    for key, fn in aux.items():
        fn()
        torch.cuda.synchronize()
        if args.no_graph:
            aux_replay[key] = fn
        else:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fn()
            aux_replay[key] = g.replay
    for ent in stack[:4]:
        assert torch.equal(rec_out[ent["name"]], ent["W"])
    aux_t = {k: statistics.median(v) for k, v in
             timer.run({k: (lambda i, r=r: r()) for k, r in aux_replay.items()}, 1, args.bursts).items()}
    del aux_replay, rec_out

    X = {name: workloads.act_device(M, shapes[name][1], seed=7 + j) for j, name in enumerate(names)}
    Y = {name: torch.empty((M, shapes[name][0]), dtype=torch.float16, device=dev) for name in names}
    ws_bytes = max(nfp.gemm_workspace_size(M, N, K, m) for (N, K) in shapes.values() for m in (0, 1))
    ws = nfp.new_workspace(ws_bytes + 256, dev)

    def leg(kind, layout):
        def run():
            for ent in stack:
                n = ent["name"]
                if kind == "fp16":
                    up, lo = ent[layout]
                    nfp.gemm(X[n], up, lo, nfp.MODE_FP16, out=Y[n], workspace=ws)
                elif kind == "fp8":
                    nfp.gemm(X[n], ent[layout][0], None, nfp.MODE_FP8, out=Y[n], workspace=ws)
                elif kind == "plain_fp16":
                    nfp.plain_gemm_fp16(X[n], ent["Wp"] if layout == "packed" else ent["W"], out=Y[n], workspace=ws)
                else:
                    nfp.plain_gemm_fp8(X[n], ent[layout][0], 2.0 ** -8, out=Y[n], workspace=ws)
        return run

    legs = {"%s/%s" % (k, l): leg(k, l) for l in ("packed", "rowmajor") for k in ("fp16", "fp8", "plain_fp16", "plain_fp8")}
    # FP8 mode when the producer of X already emits E4M3 codes and scales (activation quantisation fused
    # into the preceding operator, as serving stacks do): the GEMM alone, nestedfp_gemm_fp8_prequantized
    Xq = {name: nfp.quantize_act(X[name]) for name in names}

    def run_prequantized():
        for ent in stack:
            n = ent["name"]
            nfp.gemm_fp8_prequantized(Xq[n][0], Xq[n][1], ent[L][0], out=Y[n], workspace=ws)
    legs["fp8_prequantized/" + L] = run_prequantized
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

    n_calls = len(stack)
    step_bytes = {m: sum(gemm_bytes(M, *shapes[e["name"]], m) for e in stack) for m in ("fp16", "fp8")}
    step_flops = sum(2.0 * M * shapes[e["name"]][0] * shapes[e["name"]][1] for e in stack)

    def step():
        replay["fp16/" + L]()
        replay["fp8/" + L]()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: exactly `steps` steps; per-leg HIP events on the launch stream
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        replay["fp16/" + L]()
        ev[i][1].record()
        replay["fp8/" + L]()
        ev[i][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_fp16 = statistics.median(e[0].elapsed_time(e[1]) for e in ev) * 1e-3
    t_fp8 = statistics.median(e[1].elapsed_time(e[2]) for e in ev) * 1e-3
    ms_per_step = wall / args.steps * 1e3
    value = (step_bytes["fp16"] + step_bytes["fp8"]) / (wall / args.steps) / 1e9

    # all eight legs (NestedFP and plain, both modes, both layouts), interleaved: one graph replay
    # (128 launches) per kind and burst
    burst = timer.run({k: (lambda i, r=r: r()) for k, r in replay.items()}, 1, args.bursts)
    legs_out = {}
    for key, ts in burst.items():
        kind = key.split("/")[0]
        nbytes = step_bytes["fp16" if "16" in kind else "fp8"]
        st = stats(ts)
        legs_out[key] = {"ms": st["us"] * 1e-3, "min_ms": st["min_us"] * 1e-3, "max_ms": st["max_us"] * 1e-3,
                         "GBps": nbytes / (st["us"] * 1e-6) / 1e9, "frac_hbm": nbytes / (st["us"] * 1e-6) / 1e9 / HBM_PEAK_GBPS}
    ratios = {}
    for l in ("packed", "rowmajor"):
        ratios["fp16_vs_plain_fp16/" + l] = legs_out["plain_fp16/" + l]["ms"] / legs_out["fp16/" + l]["ms"]
        ratios["fp8_vs_plain_fp8/" + l] = legs_out["plain_fp8/" + l]["ms"] / legs_out["fp8/" + l]["ms"]

    # the same call on ONE layer over and over: its planes (48 MB for qkv) stay in the 256 MB
    # memory-side cache, so this is the hot-cache number, not an HBM rate
    hot = {}
    if M <= 64:
        calls = {}
        for j, name in enumerate(names):
            up, lo = stack[j][L]
            calls[name] = (lambda i, name=name, up=up, lo=lo: nfp.gemm(X[name], up, lo, nfp.MODE_FP16, out=Y[name], workspace=ws))
        for name, ts in timer.run(calls, 50, 5).items():
            N, K = shapes[name]
            st = stats(ts)
            hot[name] = {"us": st["us"], "GBps": gemm_bytes(M, N, K, "fp16") / (st["us"] * 1e-6) / 1e9}

    achievable = achievable_rates(torch, nfp, workloads, stack, timer, dev)

    extra = {
        "tokens": M,
        "gemm_calls_per_mode": n_calls,
        "timed_layout": L,
        "fp16_mode": {"ms": t_fp16 * 1e3, "GBps": step_bytes["fp16"] / t_fp16 / 1e9,
                      "TFLOPs": step_flops / t_fp16 / 1e12,
                      "frac_hbm": step_bytes["fp16"] / t_fp16 / 1e9 / HBM_PEAK_GBPS,
                      "frac_of_stream_read": step_bytes["fp16"] / t_fp16 / 1e9 / achievable["hbm_GBps"],
                      "frac_of_stream_read_cut_like_the_step": step_bytes["fp16"] / t_fp16 / 1e9 / achievable["hbm_GBps_cut_like_the_step"]},
        "fp8_mode": {"ms": t_fp8 * 1e3, "GBps": step_bytes["fp8"] / t_fp8 / 1e9,
                     "TFLOPs": step_flops / t_fp8 / 1e12,
                     "frac_hbm": step_bytes["fp8"] / t_fp8 / 1e9 / HBM_PEAK_GBPS,
                     "frac_of_stream_read": step_bytes["fp8"] / t_fp8 / 1e9 / achievable["hbm_GBps"],
                     "frac_of_stream_read_cut_like_the_step": step_bytes["fp8"] / t_fp8 / 1e9 / achievable["hbm_GBps_cut_like_the_fp8_step"]},
        "legs_interleaved": legs_out,
        "ratios": ratios,
        "achievable": achievable,
        "decompose_offline": {k: {"GBps": dec_bytes / aux_t["decompose/" + k] / 1e9,
                                  "frac_hbm": dec_bytes / aux_t["decompose/" + k] / 1e9 / HBM_PEAK_GBPS}
                              for k in ("rowmajor", "packed")},
        "reconstruct": {k: {"GBps": rec_bytes / aux_t["reconstruct/" + k] / 1e9,
                            "frac_hbm": rec_bytes / aux_t["reconstruct/" + k] / 1e9 / HBM_PEAK_GBPS}
                        for k in ("rowmajor", "packed")},
        "fp16_mode_hot_cache_one_layer": hot,
    }

    # roofline of the dominant kernel: the FP16-mode streaming GEMM (one launch per linear)
    traffic = read_traffic()
    roofline = {
        "kernel": "small_gemm_kernel, NestedFP16 over %s planes (FP16-mode streaming GEMM, %d launches/step)" % (L, n_calls),
        "bound": "hbm",
        "achieved": step_bytes["fp16"] / t_fp16 / 1e9,
        "peak": HBM_PEAK_GBPS,
        "unit": "GB/s",
        "frac": step_bytes["fp16"] / t_fp16 / 1e9 / HBM_PEAK_GBPS,
        "traffic": traffic,
        "avg_launch_us": t_fp16 / n_calls * 1e6,
        "algorithmic_bytes_per_launch": step_bytes["fp16"] / n_calls,
        "frac_of_stream_read_same_run": step_bytes["fp16"] / t_fp16 / 1e9 / achievable["hbm_GBps"],
        "frac_of_best_read_same_run": step_bytes["fp16"] / t_fp16 / 1e9 / max(achievable["hbm_GBps"], achievable["hbm_GBps_few_waves"]),
        "frac_of_stream_read_cut_like_the_step": step_bytes["fp16"] / t_fp16 / 1e9 / achievable["hbm_GBps_cut_like_the_step"],
    }

    if args.calibrate_copy:
        src = torch.ones(256 << 20, dtype=torch.float32, device=dev)       # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst
    del replay, legs
    if not args.no_prefill:
        extra["prefill"] = prefill_extras(torch, nfp, workloads, stack, timer, dev, args.bursts, vendor=not args.no_vendor)
    if not args.no_mode_switch:
        extra["mode_switch_steps"] = mode_switch_extras(torch, nfp, workloads, stack, L, dev)
    if args.switch_demo:
        extra["switch_demo"] = switch_demo_extras(torch, nfp, workloads, stack, L, dev)
    del stack
    torch.cuda.empty_cache()
    if not args.no_70b and not args.sweep_70b:
        sub = [(n, workloads.LLAMA3_70B[n]) for n in ("qkv", "gate_up")]
        extra["llama70b_subset"] = sweep_extras(torch, nfp, workloads, timer, dev, sub, workloads.SIGMA_W_70B,
                                                [1, 16, 64, 512, 8192], args.bursts)
    if args.sweep_70b:
        extra["sweep_70b"] = sweep_extras(torch, nfp, workloads, timer, dev, list(workloads.LLAMA3_70B.items()),
                                          workloads.SIGMA_W_70B, [1 << i for i in range(14)], 5)
    if args.paper_shapes:
        extra["paper_shapes"] = paper_shape_extras(torch, nfp, workloads, timer, dev)

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
                               "decode M=%d, FP16 mode then FP8 mode per step, %s planes" % (args.layers, M, L),
                   "tokens": M, "layers": args.layers, "hip_graph": not args.no_graph, "plane_layout": L},
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


def achievable_rates(torch, nfp, workloads, stack, timer, dev):
    """What this chip sustains, in this run, for the two resources the GEMMs are bound by: a pure
    read stream (1 GiB buffers rotated so that no cache serves them) and a loop of nothing but
    MFMAs on operands with the workload's bit patterns (weights of the stack / their upper plane
    against Gaussian activations / their E4M3 codes)."""
    bufs = [torch.empty(1 << 30, dtype=torch.uint8, device=dev) for _ in range(4)]
    for i, b in enumerate(bufs):
        b.view(torch.int32).random_(0, 1 << 30)
    ts = timer.run({"read": lambda i: nfp.probe_stream_read(bufs[i % 4])}, 8, 5)["read"]
    hbm = (1 << 30) / statistics.median(ts) / 1e9
    ts = timer.run({"read": lambda i: nfp.probe_stream_read(bufs[i % 4], sparse=True)}, 8, 5)["read"]
    hbm_sparse = (1 << 30) / statistics.median(ts) / 1e9
    del bufs
    # the same read stream cut like the decode step: one launch per linear over that linear's FP16
    # weights (2NK bytes, what FP16 mode streams), all launches of the stack in one graph
    # and over that linear's upper plane alone (NK bytes, what FP8 mode streams)
    sink = torch.zeros(1, dtype=torch.int32, device=dev)
    cut = {}
    for key, field in (("fp16", "W"), ("fp8", "rowmajor")):
        reads = [e[field] if key == "fp16" else e[field][0] for e in stack]
        reads = [w for w in reads if (w.numel() * w.element_size()) % 65536 == 0]

        def read_stack():
            for w in reads:
                nfp.probe_stream_read(w, sink)
        read_stack()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            read_stack()
        ts = timer.run({"read": lambda i: g.replay()}, 1, 5)["read"]
        cut[key] = sum(w.numel() * w.element_size() for w in reads) / statistics.median(ts) / 1e9
        n_reads = len(reads)
        del g
    # operand blocks: 8 x 8 KB = weights, activations, weights, ... (see nestedfp_probe_mfma)
    w16 = stack[0]["W"].reshape(-1)[:16384].view(torch.uint8)
    x16 = workloads.act_device(4, 4096, seed=3).reshape(-1)[:16384].view(torch.uint8)
    ops16 = torch.cat([w16[i * 8192:(i + 1) * 8192] if s == 0 else x16[i * 8192:(i + 1) * 8192]
                       for i in range(4) for s in (0, 1)]).contiguous()
    up = stack[0]["rowmajor"][0].reshape(-1)[:32768]
    xq, _ = nfp.quantize_act(workloads.act_device(8, 4096, seed=4))
    xq = xq.reshape(-1)[:32768]
    ops8 = torch.cat([up[i * 8192:(i + 1) * 8192] if s == 0 else xq[i * 8192:(i + 1) * 8192]
                      for i in range(4) for s in (0, 1)]).contiguous()
    out = {"hbm_GBps": hbm, "hbm_frac_of_peak": hbm / HBM_PEAK_GBPS,
           "hbm_probe": "read-only kernel, 8 x 128-bit loads per lane, 1 GiB per launch, 4 buffers rotated",
           "hbm_GBps_few_waves": hbm_sparse,
           "hbm_probe_few_waves": "16 x 128-bit loads per lane, at most 8 waves per CU, 1 GiB per launch: the highest read rate "
                                  "any kernel reached here",
           "hbm_GBps_cut_like_the_step": cut["fp16"],
           "hbm_GBps_cut_like_the_fp8_step": cut["fp8"],
           "hbm_probe_cut_like_the_step": "the same kernel, one launch per linear of the stack over its 2NK bytes of FP16 weights "
                                          "(FP8 step: its NK bytes of upper plane), %d launches replayed as one graph" % n_reads}
    for key, ops, fp8 in (("fp16", ops16, 0), ("fp8", ops8, 1)):
        iters = 4000
        flops = [0.0]

        def call(i, ops=ops, fp8=fp8):
            flops[0] = nfp.probe_mfma(ops, fp8, iters)
        ts = timer.run({"m": call}, 4, 5)["m"]
        tf = flops[0] / statistics.median(ts) / 1e12
        out["mfma_%s_TFLOPs" % key] = tf
        out["mfma_%s_frac_of_peak" % key] = tf / MFMA_PEAK_TFLOPS[key]
    out["mfma_probe"] = "nothing but MFMAs (16x16x32 f16 / 16x16x128 f8f6f4), 16 waves per CU, operands with the workload's bit patterns"
    return out


def prefill_extras(torch, nfp, workloads, stack, timer, dev, bursts, vendor=True):
    """Compute-bound regime (configs[2]): the same four linears at M in {512, 2048, 8192}; both
    modes, both plane layouts and the plain baselines, interleaved; layers rotated so that the
    weights are cold.  With `vendor`, the vendor library's GEMMs (torch.mm and torch._scaled_mm,
    i.e. hipBLASLt) run in the same interleaving on the same operands, as context for what this
    chip sustains: they are no part of the path, and the FP8 one reads the row-major upper plane
    as the E4M3 tensor it is, activations quantised beforehand, unit scales."""
    shapes = workloads.LLAMA3_8B
    out = {}
    n_layers = len(stack) // 4
    for M in workloads.PREFILL_M:
        row = {}
        for j, name in enumerate(shapes):
            N, K = shapes[name]
            X = workloads.act_device(M, K, seed=70 + j)
            Yb = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = nfp.new_workspace(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + 256, dev)
            flops = 2.0 * M * N * K
            Xq, sq = nfp.quantize_act(X)

            def ent(i):
                return stack[(i % n_layers) * 4 + j]
            calls = {
                "fp16/packed": lambda i: nfp.gemm(X, *ent(i)["packed"], nfp.MODE_FP16, out=Yb, workspace=ws),
                "plain_fp16/packed": lambda i: nfp.plain_gemm_fp16(X, ent(i)["Wp"], out=Yb, workspace=ws),
                "fp16/rowmajor": lambda i: nfp.gemm(X, *ent(i)["rowmajor"], nfp.MODE_FP16, out=Yb, workspace=ws),
                "plain_fp16/rowmajor": lambda i: nfp.plain_gemm_fp16(X, ent(i)["W"], out=Yb, workspace=ws),
                "fp8/packed": lambda i: nfp.gemm(X, ent(i)["packed"][0], None, nfp.MODE_FP8, out=Yb, workspace=ws),
                "plain_fp8/packed": lambda i: nfp.plain_gemm_fp8(X, ent(i)["packed"][0], 2.0 ** -8, out=Yb, workspace=ws),
                "fp8/rowmajor": lambda i: nfp.gemm(X, ent(i)["rowmajor"][0], None, nfp.MODE_FP8, out=Yb, workspace=ws),
                "plain_fp8/rowmajor": lambda i: nfp.plain_gemm_fp8(X, ent(i)["rowmajor"][0], 2.0 ** -8, out=Yb, workspace=ws),
                # the FP8-mode GEMM launch alone: activations quantised beforehand (outside the timing)
                "fp8_prequantized/packed": lambda i: nfp.gemm_fp8_prequantized(Xq, sq, ent(i)["packed"][0], out=Yb, workspace=ws),
            }
            if vendor:
                calls["vendor_fp16/rowmajor"] = lambda i: torch.mm(X, ent(i)["W"].t(), out=Yb)
                try:
                    one = torch.ones((), dtype=torch.float32, device=dev)
                    Xq8 = Xq.view(torch.float8_e4m3fn)

                    def vendor_fp8(i):
                        torch._scaled_mm(Xq8, ent(i)["rowmajor"][0].view(torch.float8_e4m3fn).t(), scale_a=one, scale_b=one,
                                         out_dtype=torch.float16)
                    vendor_fp8(0)
                    calls["vendor_fp8/rowmajor"] = vendor_fp8
                except Exception:                       # noqa: BLE001 - context only: left out where the library refuses
                    pass
            launches = 50 if M <= 2048 else 20
            res = {}
            for key, ts in timer.run(calls, launches, bursts).items():
                st = stats(ts)
                mode = "fp16" if "16" in key else "fp8"
                t = st["us"] * 1e-6
                st.update({"TFLOPs": flops / t / 1e12, "frac_mfma": flops / t / 1e12 / MFMA_PEAK_TFLOPS[mode],
                           "frac_of_bound": bound_seconds(M, N, K, mode) / t})
                res[key] = st
            for l in ("packed", "rowmajor"):
                res["fp16_vs_plain/" + l] = res["plain_fp16/" + l]["us"] / res["fp16/" + l]["us"]
                res["fp8_vs_plain/" + l] = res["plain_fp8/" + l]["us"] / res["fp8/" + l]["us"]
            row[name] = res
            del X, Yb, ws, Xq, sq
        out["M=%d" % M] = row
    return out


def _layer_copies(torch, nfp, workloads, N, K, sigma, dev, seed0):
    """Enough copies of one layer that neither L2 nor the 256 MB cache can serve the weights."""
    copies = int(min(8, max(2, -(-600e6 // (2 * N * K)))))
    Ws = [workloads.weight_device(N, K, sigma, seed=seed0 + i) for i in range(copies)]
    return Ws, [nfp.decompose(W, check=(i == 0), packed=True) for i, W in enumerate(Ws)], \
        [nfp.decompose(W, check=False) for W in Ws]


def sweep_extras(torch, nfp, workloads, timer, dev, shapes, sigma, Ms, bursts):
    """Roofline curve (configs[3]): both modes over packed and row-major planes and the plain FP16
    baselines over M on each shape; the bound of a point is max(algorithmic bytes / 8 TB/s, flops /
    MFMA peak of the mode)."""
    out = {}
    for j, (name, (N, K)) in enumerate(shapes):
        Ws, packed, rowmajor = _layer_copies(torch, nfp, workloads, N, K, sigma, dev, 300 + 10 * j)
        Wps = [nfp.pack_fp16(W) for W in Ws]
        R = len(Ws)
        row = {}
        for M in Ms:
            X = workloads.act_device(M, K, seed=90 + j)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = nfp.new_workspace(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + 256, dev)
            calls = {
                "fp16/packed": lambda i: nfp.gemm(X, packed[i % R][0], packed[i % R][1], nfp.MODE_FP16, out=Y, workspace=ws),
                "plain_fp16/packed": lambda i: nfp.plain_gemm_fp16(X, Wps[i % R], out=Y, workspace=ws),
                "fp16/rowmajor": lambda i: nfp.gemm(X, rowmajor[i % R][0], rowmajor[i % R][1], nfp.MODE_FP16, out=Y, workspace=ws),
                "plain_fp16/rowmajor": lambda i: nfp.plain_gemm_fp16(X, Ws[i % R], out=Y, workspace=ws),
                "fp8/packed": lambda i: nfp.gemm(X, packed[i % R][0], None, nfp.MODE_FP8, out=Y, workspace=ws),
                "fp8/rowmajor": lambda i: nfp.gemm(X, rowmajor[i % R][0], None, nfp.MODE_FP8, out=Y, workspace=ws),
            }
            t_guess = max(bound_seconds(M, N, K, "fp16") * 2.5, 20e-6)
            launches = int(min(50, max(5, 0.05 / t_guess)))
            res = {}
            fl = 2.0 * M * N * K
            for key, ts in timer.run(calls, launches, bursts).items():
                st = stats(ts)
                mode = "fp16" if "16" in key else "fp8"
                t = st["us"] * 1e-6
                st.update({"GBps": gemm_bytes(M, N, K, mode) / t / 1e9, "TFLOPs": fl / t / 1e12,
                           "frac_roofline": bound_seconds(M, N, K, mode) / t})
                res[key] = st
            res["fp16_vs_plain/packed"] = res["plain_fp16/packed"]["us"] / res["fp16/packed"]["us"]
            res["fp16_vs_plain/rowmajor"] = res["plain_fp16/rowmajor"]["us"] / res["fp16/rowmajor"]["us"]
            row["M=%d" % M] = res
            del X, Y, ws
        out["%s (%d,%d)" % (name, N, K)] = row
        del Ws, packed, rowmajor, Wps
        torch.cuda.empty_cache()
    return out


def paper_shape_extras(torch, nfp, workloads, timer, dev):
    """Sec. 5.2 / App. C of the paper sweep M = 32 ... 2048 in steps of 32 on four (N,K) shapes
    and quote the mean slowdown of FP16 mode against a plain FP16 GEMM; same sweep here, against
    the plain GEMM on packed FP16 weights (same kernel minus the reconstruction) and on row-major ones."""
    out = {}
    for j, (N, K) in enumerate(workloads.PAPER_KERNEL_SHAPES):
        Ws, packed, rowmajor = _layer_copies(torch, nfp, workloads, N, K, workloads.SIGMA_W_8B, dev, 500 + 10 * j)
        Wps = [nfp.pack_fp16(W) for W in Ws]
        R = len(Ws)
        over = []
        for M in range(32, 2049, 32):
            X = workloads.act_device(M, K, seed=95 + j)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            ws = nfp.new_workspace(nfp.gemm_workspace_size(M, N, K, 0) + 256, dev)
            calls = {
                "fp16": lambda i: nfp.gemm(X, packed[i % R][0], packed[i % R][1], nfp.MODE_FP16, out=Y, workspace=ws),
                "plain_packed": lambda i: nfp.plain_gemm_fp16(X, Wps[i % R], out=Y, workspace=ws),
                "fp16_rowmajor": lambda i: nfp.gemm(X, rowmajor[i % R][0], rowmajor[i % R][1], nfp.MODE_FP16, out=Y, workspace=ws),
                "plain_rowmajor": lambda i: nfp.plain_gemm_fp16(X, Ws[i % R], out=Y, workspace=ws),
            }
            r = {k: statistics.median(v) for k, v in timer.run(calls, 8, 3).items()}
            over.append((M, r["fp16"] / r["plain_packed"] - 1.0, r["fp16_rowmajor"] / r["plain_rowmajor"] - 1.0,
                         2.0 * M * N * K / r["fp16"] / 1e12))
            del X, Y, ws
        o = [x[1] for x in over]
        o2 = [x[2] for x in over]
        out["(%d,%d)" % (N, K)] = {
            "mean_overhead_vs_plain_packed": sum(o) / len(o), "min": min(o), "max": max(o),
            "mean_overhead_rowmajor_vs_plain_rowmajor": sum(o2) / len(o2),
            "fp16_TFLOPs_at_M=2048": over[-1][3],
            "overhead_at": {"M=%d" % m: ov for m, ov, _, _ in over if m in (32, 64, 128, 256, 512, 1024, 2048)}}
        del Ws, packed, rowmajor, Wps
        torch.cuda.empty_cache()
    return out


def _run_stack(nfp, stack, layout, X, Y, ws, mode):
    for ent in stack:
        up, lo = ent[layout]
        n = ent["name"]
        nfp.gemm(X[n], up, None if mode == nfp.MODE_FP8 else lo, mode, out=Y[n], workspace=ws)


def _stack_buffers(torch, nfp, workloads, M, dev):
    shapes = workloads.LLAMA3_8B
    X = {n: workloads.act_device(M, shapes[n][1], seed=60 + j) for j, n in enumerate(shapes)}
    Y = {n: torch.empty((M, shapes[n][0]), dtype=torch.float16, device=dev) for n in shapes}
    need = max(nfp.gemm_workspace_size(M, N, K, m) for (N, K) in shapes.values() for m in (0, 1))
    return X, Y, nfp.new_workspace(need + 256, dev)


def mode_switch_extras(torch, nfp, workloads, stack, layout, dev):
    """Sec. 5.4: the mode is chosen per iteration (configs[4]).  64 steps over the whole stack, the
    mode flipping every 8 steps, at M = 64 and M = 2048: step time by mode, the first step after a
    flip against the steady state, allocated device memory before and after."""
    out = {"plane_layout": layout}
    for M in (64, 2048):
        X, Y, ws = _stack_buffers(torch, nfp, workloads, M, dev)
        for mode in (nfp.MODE_FP16, nfp.MODE_FP8):
            _run_stack(nfp, stack, layout, X, Y, ws, mode)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(65)]
        modes = []
        ev[0].record()
        for step in range(64):
            mode = nfp.MODE_FP8 if (step // 8) % 2 else nfp.MODE_FP16
            modes.append(mode)
            _run_stack(nfp, stack, layout, X, Y, ws, mode)
            ev[step + 1].record()
        torch.cuda.synchronize()
        t = [ev[i].elapsed_time(ev[i + 1]) for i in range(64)]
        first = {m: [t[i] for i in range(8, 64) if i % 8 == 0 and modes[i] == m] for m in (nfp.MODE_FP16, nfp.MODE_FP8)}
        steady = {m: [t[i] for i in range(64) if modes[i] == m and i % 8 != 0] for m in (nfp.MODE_FP16, nfp.MODE_FP8)}
        out["M=%d" % M] = {
            "fp16_step_ms": statistics.median(steady[nfp.MODE_FP16]),
            "fp8_step_ms": statistics.median(steady[nfp.MODE_FP8]),
            "first_fp16_step_after_switch_ms": statistics.median(first[nfp.MODE_FP16]),
            "first_fp8_step_after_switch_ms": statistics.median(first[nfp.MODE_FP8]),
            "allocated_bytes_before": before, "allocated_bytes_after": torch.cuda.memory_allocated()}
        del X, Y, ws
    return out


def switch_demo_extras(torch, nfp, workloads, stack, layout, dev):
    """Sec. 5.4's policy on a synthetic arrival sequence (the paper's trace is not available):
    a step whose token count exceeds 1024 runs in FP8 mode, the others in FP16 mode."""
    import numpy as np

    rng = np.random.default_rng(7)
    choices = np.array([16, 32, 64, 128, 256, 512, 1024, 2048, 4096])
    # mostly small decode steps with bursts of large prefill-heavy steps
    # (a burst is 1024 tokens or more: the policy's threshold is crossed by about one step in six)
    seq = [int(choices[min(8, int(abs(rng.normal(0, 1.6)) + (6 if rng.random() < 0.25 else 0)))]) for _ in range(48)]
    bufs = {M: _stack_buffers(torch, nfp, workloads, M, dev) for M in sorted(set(seq))}
    res = {}
    for policy in ("always_fp16", "always_fp8", "threshold_1024"):
        def mode_of(M):
            if policy == "always_fp16":
                return nfp.MODE_FP16
            if policy == "always_fp8":
                return nfp.MODE_FP8
            return nfp.select_mode(M, 1024)
        for M in bufs:                                   # warm every kernel once
            _run_stack(nfp, stack, layout, *bufs[M], mode_of(M))
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for M in seq:
            _run_stack(nfp, stack, layout, *bufs[M], mode_of(M))
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
    # the upper planes for the FP8 leg: the offline step, not timed (row blocks on a few threads:
    # ctypes releases the interpreter lock during the oracle call)
    from concurrent.futures import ThreadPoolExecutor

    def upper_of(W):
        blocks = [W[i:i + 256] for i in range(0, W.shape[0], 256)]
        with ThreadPoolExecutor(max_workers=min(16, cores)) as pool:
            return np.concatenate(list(pool.map(lambda b: oracle.decompose(b)[0], blocks)))
    ups = [upper_of(W) for W, _ in inputs]
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
