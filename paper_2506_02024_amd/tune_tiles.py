"""Measures the launch shapes of the GEMM kernels on this machine and writes the tables of tuned
choices that the library compiles in (csrc/tuned_tiles.inc for the tiled kernels,
csrc/tuned_small.inc for the streaming kernel).

    python -m paper_2506_02024_amd.tune_tiles [--out PATH] [--out-small PATH] [--shapes N,K ...] [--margin 0.03]

The tiled kernels pick tile shape, K split and pipeline depth from a small cost model.  The model is
within a few per cent of the best choice on average, but off by 10-30 % at some points of the
ridge between the memory-bound and the compute-bound regime (M = 128 ... 512).  This script times
every legal choice through the tuning knobs -- on the layer shapes of the models the paper evaluates
(Sec. 5.1: Llama 3.1 8B / 70B, Mistral Nemo, Phi-4, Mistral Small), at M = 32 ... 8192, for the three
classes of weights (FP16 row-major, FP16 through registers = NestedFP planes, E4M3) -- and records a
choice only where it beats the model's by more than the margin.  At M = 32 and 64 the layers that
the library routes to its 64-token tiles are timed over the K split alone (on the others the knobs
change nothing and nothing is recorded).  Other shapes keep the model.
The streaming kernel (decode batches) is timed at M = 16 over its K-steps per wave, grid-level K
split and tiles per workgroup, as graph replays over the rotated copies; an entry serves batches of up
to 16 tokens.
Rebuild the library after running it.
"""
import argparse
import os
import statistics
import sys
import time


# (N, K) of qkv / o / gate_up / down
MODEL_SHAPES = {
    "llama-3.1-8b": [(6144, 4096), (4096, 4096), (28672, 4096), (4096, 14336)],
    "llama-3.1-70b": [(10240, 8192), (8192, 8192), (57344, 8192), (8192, 28672)],
    "mistral-nemo-12b": [(6144, 5120), (5120, 4096), (28672, 5120), (5120, 14336)],
    "phi-4-14b": [(7680, 5120), (5120, 5120), (35840, 5120), (5120, 17920)],
    "mistral-small-24b": [(6144, 5120), (5120, 4096), (65536, 5120), (5120, 32768)],
}
M_POINTS = (32, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 1536, 2048, 4096, 8192)  # 32, 64: the 64-token tiles, where only the K split is open;
# 4096, 8192: no K split (the chip is full)
TILES = ((256, 256), (256, 128), (128, 256), (128, 128))
SPLITS = (1, 2, 3, 4, 6, 8)
KNOBS = ("large_bm", "large_bn", "large_split", "large_deep")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "tuned_tiles.inc"))
    ap.add_argument("--out-small", default=os.path.join(os.path.dirname(os.path.abspath(__file__)), "csrc", "tuned_small.inc"))
    ap.add_argument("--skip-tiled", action="store_true")
    ap.add_argument("--skip-small", action="store_true")
    ap.add_argument("--shapes", nargs="*", default=None, help="N,K pairs instead of the built-in model shapes")
    ap.add_argument("--margin", type=float, default=0.03)
    ap.add_argument("--m-points", nargs="*", type=int, default=None,
                    help="batch sizes of the tiled section instead of the built-in list (to re-time a part of the table)")
    ap.add_argument("--log", default=None, help="write every timing as JSON lines")
    args = ap.parse_args()

    import torch
    from . import binding as nfp, workloads

    dev = torch.device("cuda:0")
    if args.shapes:
        shapes = [tuple(int(v) for v in s.split(",")) for s in args.shapes]
    else:
        shapes = sorted({s for v in MODEL_SHAPES.values() for s in v})
    log = open(args.log, "w") if args.log else None

    def timeit(fns, launches=8, bursts=3):
        # fns: the same call on different copies of the weights, taken in turn so that no copy is
        # still in the memory-side cache when its turn comes again
        launches = max(launches, len(fns))
        for f in fns:
            f()
        torch.cuda.synchronize()
        ts = []
        for _ in range(bursts):
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for i in range(launches):
                fns[i % len(fns)]()
            e.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(e) * 1e3 / launches)
        return statistics.median(ts)

    def time_graph(fns, reps=3):
        # one graph over all copies: what a decode step looks like to the hardware
        for f in fns:
            f()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for f in fns:
                f()
        g.replay()
        torch.cuda.synchronize()
        ts = []
        for _ in range(reps):
            a, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            g.replay()
            e.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(e) * 1e3 / len(fns))
        return statistics.median(ts)

    t0 = time.time()
    small_rows = []
    SMALL_KNOBS = ("small_spw", "small_split", "small_tiles")
    for N, K in ([] if args.skip_small else shapes):
        copies = max(4, min(24, -(-1_200_000_000 // (N * K))))
        Ws = [workloads.weight_device(N, K, 0.02, seed=i) for i in range(copies)]
        planes = [nfp.decompose(W, packed=True) for W in Ws]
        M = 16
        X = workloads.act_device(M, K, seed=2)
        Y = torch.empty((M, N), dtype=torch.float16, device=dev)
        ws = nfp.new_workspace(8 * M * N * 4 + M * K + 4 * M + (1 << 20), dev)
        calls = {
            0: [lambda W=W: nfp.plain_gemm_fp16(X, W, out=Y, workspace=ws) for W in Ws],
            1: [lambda p=p: nfp.gemm(X, p[0], p[1], nfp.MODE_FP16, out=Y, workspace=ws) for p in planes],
            2: [lambda p=p: nfp.gemm(X, p[0], None, nfp.MODE_FP8, out=Y, workspace=ws) for p in planes],
        }
        for cls, fns in calls.items():
            nfp.tune("tuned_table", 0)
            try:
                t_rule = time_graph(fns)
                best = (t_rule, None)
                for spw in ((2, 4, 8) if cls == 0 else (2, 4)):
                    for sp in SPLITS:
                        for tiles in (1, 2, 3, 4, 5, 6, 8, 10, 12):
                            for k, v in zip(SMALL_KNOBS, (spw, sp, tiles)):
                                nfp.tune(k, v)
                            try:
                                t = time_graph(fns, reps=2)
                            finally:
                                for k in SMALL_KNOBS:
                                    nfp.tune(k, -1)
                            if log:
                                log.write('{"small": 1, "N": %d, "K": %d, "cls": %d, "spw": %d, "split": %d, "tiles": %d, "us": %.2f, "rule_us": %.2f}\n'
                                          % (N, K, cls, spw, sp, tiles, t, t_rule))
                            if t < best[0]:
                                best = (t, (spw, sp, tiles))
                if best[1] is not None and best[0] < t_rule * (1.0 - args.margin):
                    for k, v in zip(SMALL_KNOBS, best[1]):
                        nfp.tune(k, v)
                    try:
                        t_best = time_graph(fns, reps=5)
                    finally:
                        for k in SMALL_KNOBS:
                            nfp.tune(k, -1)
                    t_again = time_graph(fns, reps=5)
                    if t_best < t_again * (1.0 - args.margin):
                        small_rows.append((cls, N, K) + best[1] + (t_best, t_again))
            finally:
                nfp.tune("tuned_table", -1)
        print("streaming N=%d K=%d  %.0f s, %d entries" % (N, K, time.time() - t0, len(small_rows)), flush=True)
        del X, Y, ws, calls, Ws, planes
        torch.cuda.empty_cache()
    if not args.skip_small:
        with open(args.out_small, "w") as f:
            f.write("// Launch shapes of the streaming GEMM kernel that beat its built-in rules by more than %.0f %% when timed\n" % (100 * args.margin))
            f.write("// at 16 tokens on an MI355X; written by paper_2506_02024_amd/tune_tiles.py, which says how.\n")
            f.write("// weight class (0 FP16 row-major, 1 FP16 through registers, 2 E4M3), N, K,\n")
            f.write("// K-steps per wave, grid-level K split, tiles per workgroup   // microseconds: tuned, rules\n")
            for r in sorted(small_rows):
                f.write("{%d, %d, %d, %d, %d, %d},   // %.1f, %.1f\n" % r)
        print("wrote %d entries to %s" % (len(small_rows), args.out_small))

    rows = []
    for N, K in ([] if args.skip_tiled else shapes):
        # enough copies that even the E4M3 plane alone (N*K bytes per call) cycles through more than
        # four times the 256 MB memory-side cache
        copies = max(2, min(64, -(-1_200_000_000 // (N * K))))
        Ws = [workloads.weight_device(N, K, 0.02, seed=i) for i in range(copies)]
        planes = [nfp.decompose(W, packed=True) for W in Ws]
        for M in (args.m_points or M_POINTS):
            X = workloads.act_device(M, K, seed=2)
            Y = torch.empty((M, N), dtype=torch.float16, device=dev)
            # room for any split that is tried (up to 8 below 4096 tokens, the built-in choice above)
            need = (8 if M < 4096 else 0) * M * N * 4 + M * K + 4 * M
            for table in (-1, 0):                       # with and without the table that is compiled in now
                nfp.tune("tuned_table", table)
                need = max(need, max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)))
            nfp.tune("tuned_table", -1)
            ws = nfp.new_workspace(need + (1 << 20), dev)
            calls = {
                0: [lambda W=W: nfp.plain_gemm_fp16(X, W, out=Y, workspace=ws) for W in Ws],
                1: [lambda p=p: nfp.gemm(X, p[0], p[1], nfp.MODE_FP16, out=Y, workspace=ws) for p in planes],
                2: [lambda p=p: nfp.gemm(X, p[0], None, nfp.MODE_FP8, out=Y, workspace=ws) for p in planes],
            }
            for cls, fns in calls.items():
                nfp.tune("tuned_table", 0)
                try:
                    t_model = timeit(fns)
                    best = (t_model, None)
                    kt = (K if cls == 2 else 2 * K) // 128
                    # (the 64-token tiles also compete at 128 and 256 tokens, as two and four token tiles)
                    for bm, bn in (((64, 128),) if M <= 64 else (TILES + ((64, 128),) if M <= 256 else TILES)):
                        for sp in (SPLITS if M < 4096 else (1,)):
                            if sp > 1 and sp > kt // 4:
                                continue
                            for deep in ((0,) if (bm, bn) == (256, 256) or bm == 64 or (cls == 1 and bm != 128) else (0, 1)):
                                for k, v in zip(KNOBS, (bm, bn, sp, deep)):
                                    nfp.tune(k, v)
                                try:
                                    t = timeit(fns)
                                finally:
                                    for k in KNOBS:
                                        nfp.tune(k, -1)
                                if log:
                                    log.write('{"N": %d, "K": %d, "M": %d, "cls": %d, "bm": %d, "bn": %d, "split": %d, "deep": %d, "us": %.2f, "model_us": %.2f}\n'
                                              % (N, K, M, cls, bm, bn, sp, deep, t, t_model))
                                if t < best[0]:
                                    best = (t, (bm, bn, sp, deep))
                finally:
                    nfp.tune("tuned_table", -1)
                if best[1] is not None and best[0] < t_model * (1.0 - args.margin):
                    # confirm against the model's choice once more, interleaved, before recording
                    for k, v in zip(KNOBS, best[1]):
                        nfp.tune(k, v)
                    try:
                        t_best = timeit(fns, bursts=5)
                    finally:
                        for k in KNOBS:
                            nfp.tune(k, -1)
                    nfp.tune("tuned_table", 0)
                    try:
                        t_again = timeit(fns, bursts=5)
                    finally:
                        nfp.tune("tuned_table", -1)
                    if t_best < t_again * (1.0 - args.margin):
                        rows.append((cls, N, K, M) + best[1] + (t_best, t_again))
            print("N=%d K=%d M=%d  %.0f s, %d entries" % (N, K, M, time.time() - t0, len(rows)), flush=True)
            del X, Y, ws, calls
        del Ws, planes
        torch.cuda.empty_cache()

    if args.skip_tiled:
        return 0
    with open(args.out, "w") as f:
        f.write("// Launch shapes of the tiled GEMM kernels that beat the cost model's choice by more than %.0f %% when\n" % (100 * args.margin))
        f.write("// timed on an MI355X; written by paper_2506_02024_amd/tune_tiles.py, which says how.\n")
        f.write("// weight class (0 FP16 row-major, 1 FP16 through registers, 2 E4M3), N, K, tokens tuned at,\n")
        f.write("// tile tokens, tile weight rows, K split, deeper pipeline   // microseconds: tuned, model's choice\n")
        for r in sorted(rows):
            f.write("{%d, %d, %d, %d, %d, %d, %d, %d},   // %.1f, %.1f\n" % r)
    print("wrote %d entries to %s" % (len(rows), args.out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
