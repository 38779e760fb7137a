"""GPU parity: both GEMM modes against the fp64 oracle, the plain baselines, edge cases."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_02024_amd import workloads
from helpers import assert_gemm_close, assert_plane_equal, bits, decompose_ref, structured_sample, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nfp():
    from paper_2506_02024_amd import binding

    return binding


def run_both_modes(nfp, X, W, what, check_plain=True, layouts=(False, True)):
    """Runs decompose + FP16 mode + FP8 mode on the GPU, over row-major planes and over packed
    ones, and checks all of it against the oracle."""
    Xd, Wd = to_dev(X), to_dev(W)
    up_ref, lo_ref, bad = oracle.decompose(W)
    assert bad == 0
    ref16 = oracle.gemm_fp16(X, W)
    Xq, s = oracle.quantize_act(X)
    ref8 = oracle.gemm_fp8(Xq, s, up_ref)
    outs = {}
    for packed in layouts:
        tag = "%s, %s planes" % (what, "packed" if packed else "row-major")
        up, lo = nfp.decompose(Wd, packed=packed)
        assert_plane_equal(up, up_ref)
        assert_plane_equal(lo, lo_ref)
        y16 = nfp.gemm(Xd, up, lo, nfp.MODE_FP16)
        assert_gemm_close(y16.cpu().numpy(), ref16, tag + " FP16 mode")
        # FP8 mode: lower plane is not passed at all
        y8 = nfp.gemm(Xd, up, None, nfp.MODE_FP8)
        assert_gemm_close(y8.cpu().numpy(), ref8, tag + " FP8 mode")
        if check_plain:
            yp8 = nfp.plain_gemm_fp8(Xd, up, 2.0 ** -8)
            assert np.array_equal(bits(yp8), bits(y8)), tag + ": FP8 mode differs from the plain fp8 GEMM"
        outs[packed] = (y16, y8, up, lo)
    if len(outs) == 2:
        # the launch shape is chosen by the kind of weights, not by their storage order, and a
        # lane holds the same 16 columns either way: same bits
        assert np.array_equal(bits(outs[False][0]), bits(outs[True][0])), what + ": FP16 mode differs between the layouts"
        assert np.array_equal(bits(outs[False][1]), bits(outs[True][1])), what + ": FP8 mode differs between the layouts"
    if check_plain:
        if True in outs:
            # FP16 weights in packed storage go through the kernel of FP16 mode minus the merge, in
            # the launch shape chosen for it: bit-identical with no knob pinned
            yp = nfp.plain_gemm_fp16(Xd, nfp.pack_fp16(Wd))
            assert np.array_equal(bits(yp), bits(outs[True][0])), what + ": FP16 mode differs from the plain GEMM on packed FP16"
        # row-major FP16 weights take kernels of their own; with the same launch shape for both
        # (tile shape and K split of the tiled ones, K-steps per wave of the streaming ones) the
        # sums run in the same order
        pins = {"large_bm": 128, "large_bn": 256, "large_split": 2, "small_spw": 4}
        for k, v in pins.items():
            nfp.tune(k, v)
        try:
            yp = nfp.plain_gemm_fp16(Xd, Wd)
            any_layout = next(iter(outs.values()))
            yn = nfp.gemm(Xd, any_layout[2], any_layout[3], nfp.MODE_FP16)
        finally:
            for k in pins:
                nfp.tune(k, -1)
        assert np.array_equal(bits(yp), bits(yn)), what + ": FP16 mode differs from the plain fp16 GEMM"
        assert_gemm_close(yn.cpu().numpy(), ref16, what + " FP16 mode, pinned launch shape")
    first = next(iter(outs.values()))
    return first[0], first[1]


def test_config1_single_linear(nfp):
    # W [1024,1024] sigma 0.02, X [16,1024] sigma 1
    W = workloads.weight_host(1024, 1024, workloads.SIGMA_W_8B, seed=0)
    X = workloads.act_host(16, 1024, seed=0)
    run_both_modes(nfp, X, W, "config 1")


@pytest.mark.parametrize("M", [1, 2, 3, 4, 5, 8, 15, 16, 17, 31, 32, 33, 48, 63, 64])
def test_decode_sized_batches(nfp, M):
    # several 16-row weight tiles, a ragged N tail and a K that is not a multiple of 64 / 128
    N, K = 16 * 9 + 8, 64 * 5 + 16
    W = workloads.weight_host(N, K, seed=M)
    X = workloads.act_host(M, K, seed=M)
    run_both_modes(nfp, X, W, "M=%d" % M)


@pytest.mark.parametrize("N,K", [(4, 16), (16, 16), (20, 32), (1, 4096), (257, 2048), (6, 144),
                                 (48, 8256), (20, 14352), (300, 28672)])
def test_decode_odd_layer_shapes(nfp, N, K):
    W = workloads.weight_host(N, K, seed=N)
    X = workloads.act_host(4, K, seed=K)
    run_both_modes(nfp, X, W, "N=%d K=%d" % (N, K))


@pytest.mark.parametrize("M", [16, 64, 300])
def test_replayed_graph_on_a_side_stream_equals_eager_calls(nfp, M):
    # both modes captured into one HIP graph on a non-default stream (streaming kernel with its
    # split reduction, 64-token tiles, tiled kernels, activation quantisation): every replay, with
    # eager work and new activations in between, must give what the eager calls give
    N, K = 16384 + 72, 1024 + 64
    W = workloads.weight_host(N, K, seed=M)
    up, lo = nfp.decompose(to_dev(W), packed=(M != 64))
    X = to_dev(workloads.act_host(M, K, seed=M + 1))
    Y16 = torch.empty((M, N), dtype=torch.float16, device="cuda:0")
    Y8 = torch.empty_like(Y16)
    ws = nfp.new_workspace(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + 256, "cuda:0")

    def both():
        nfp.gemm(X, up, lo, nfp.MODE_FP16, out=Y16, workspace=ws)
        nfp.gemm(X, up, None, nfp.MODE_FP8, out=Y8, workspace=ws)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        both()                                         # warm-up outside the capture
    side.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=side):
        both()
    for rep in range(3):
        X.copy_(to_dev(workloads.act_host(M, K, seed=100 * M + rep)))     # eager work between the replays
        both()
        torch.cuda.synchronize()
        want16, want8 = Y16.clone(), Y8.clone()
        Y16.zero_()
        Y8.zero_()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Y16, want16) and torch.equal(Y8, want8), "replay %d" % rep
    assert_gemm_close(Y16.cpu().numpy(), oracle.gemm_fp16(X.cpu().numpy(), W), "graph replay, FP16 mode")


def test_calls_on_two_streams_do_not_interfere(nfp):
    # the library holds no device state of its own: two streams, each with its own workspace and output,
    # run different problems at the same time and get what they get alone
    probs = []
    for j, (M, N, K) in enumerate([(16, 4096 + 8, 14336), (200, 2048 + 24, 1024)]):
        W = workloads.weight_host(N, K, seed=60 + j)
        up, lo = nfp.decompose(to_dev(W), packed=(j == 0))
        X = to_dev(workloads.act_host(M, K, seed=70 + j))
        ws = nfp.new_workspace(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + 256, "cuda:0")
        alone = (nfp.gemm(X, up, lo, nfp.MODE_FP16, workspace=ws).clone(), nfp.gemm(X, up, None, nfp.MODE_FP8, workspace=ws).clone())
        outs = (torch.empty_like(alone[0]), torch.empty_like(alone[1]))
        probs.append((X, up, lo, ws, alone, outs, torch.cuda.Stream()))
    torch.cuda.synchronize()
    for rep in range(8):
        for X, up, lo, ws, alone, outs, st in probs:
            with torch.cuda.stream(st):
                nfp.gemm(X, up, lo, nfp.MODE_FP16, out=outs[0], workspace=ws)
                nfp.gemm(X, up, None, nfp.MODE_FP8, out=outs[1], workspace=ws)
    torch.cuda.synchronize()
    for X, up, lo, ws, alone, outs, st in probs:
        assert torch.equal(outs[0], alone[0]) and torch.equal(outs[1], alone[1])


def test_calls_from_two_host_threads(nfp):
    # the entry points may be called from several host threads at once (own stream, own workspace,
    # nobody changing a tuning knob meanwhile): each thread gets what it gets alone
    import threading

    probs = []
    for j, (M, N, K) in enumerate([(16, 2048 + 8, 4096), (130, 1024 + 24, 2048)]):
        W = workloads.weight_host(N, K, seed=80 + j)
        up, lo = nfp.decompose(to_dev(W), packed=(j == 1))
        X = to_dev(workloads.act_host(M, K, seed=90 + j))
        ws = nfp.new_workspace(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + 256, "cuda:0")
        alone = (nfp.gemm(X, up, lo, nfp.MODE_FP16, workspace=ws).clone(), nfp.gemm(X, up, None, nfp.MODE_FP8, workspace=ws).clone())
        probs.append((X, up, lo, ws, alone, torch.cuda.Stream()))
    torch.cuda.synchronize()
    errors = []

    def work(X, up, lo, ws, alone, st):
        try:
            with torch.cuda.stream(st):
                out16, out8 = torch.empty_like(alone[0]), torch.empty_like(alone[1])
                for rep in range(40):
                    nfp.gemm(X, up, lo, nfp.MODE_FP16, out=out16, workspace=ws)
                    nfp.gemm(X, up, None, nfp.MODE_FP8, out=out8, workspace=ws)
                st.synchronize()
                if not (torch.equal(out16, alone[0]) and torch.equal(out8, alone[1])):
                    errors.append("results differ")
        except Exception as e:                          # noqa: BLE001 - reported below
            errors.append(repr(e))

    threads = [threading.Thread(target=work, args=pr) for pr in probs]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    torch.cuda.synchronize()
    assert not errors, errors


@pytest.mark.parametrize("seed", range(6))
def test_random_shapes_against_the_oracle(nfp, seed):
    # eight seeded problems per case: M in 1 ... 300 (all kernel families and the batch sizes where the
    # built-in choice moves between them), N in 1 ... 700, K any multiple of 16 up to 3072, both
    # modes, both plane layouts, the plain baselines -- everything run_both_modes checks
    rng = np.random.default_rng(1000 + seed)
    for _ in range(8):
        M = int(rng.choice([1, 2, 7, 16, 17, 24, 31, 32, 33, 47, 48, 64, 65, 100, 128, 129, 200, 256, 257, 300]))
        N = int(rng.integers(1, 701))
        K = 16 * int(rng.integers(1, 193))
        W = workloads.weight_host(N, K, seed=int(rng.integers(1 << 30)))
        X = workloads.act_host(M, K, seed=int(rng.integers(1 << 30)))
        run_both_modes(nfp, X, W, "random M=%d N=%d K=%d" % (M, N, K))


def test_empty_batch_and_empty_layer(nfp):
    # M = 0 and N = 0 are legal and launch nothing: the output keeps what it held
    K = 64
    W = workloads.weight_host(32, K, seed=5)
    up, lo = nfp.decompose(to_dev(W))
    X0 = torch.empty((0, K), dtype=torch.float16, device="cuda:0")
    for mode in (nfp.MODE_FP16, nfp.MODE_FP8):
        y = nfp.gemm(X0, up, lo if mode == nfp.MODE_FP16 else None, mode)
        assert tuple(y.shape) == (0, 32)
    assert tuple(nfp.plain_gemm_fp16(X0, to_dev(W)).shape) == (0, 32)
    assert nfp.gemm_workspace_size(0, 32, K, nfp.MODE_FP16) == 0 and nfp.gemm_workspace_size(0, 32, K, nfp.MODE_FP8) == 0
    W0 = torch.empty((0, K), dtype=torch.float16, device="cuda:0")
    up0, lo0 = nfp.decompose(W0)
    X = to_dev(workloads.act_host(3, K, seed=6))
    assert tuple(nfp.gemm(X, up0, lo0, nfp.MODE_FP16).shape) == (3, 0)
    assert tuple(nfp.gemm(X, up0, None, nfp.MODE_FP8).shape) == (3, 0)


@pytest.mark.parametrize("knobs", [
    {"small_split": 1, "small_tiles": 1},
    {"small_split": 1, "small_tiles": 2, "small_spw": 2},
    {"small_split": 3, "small_tiles": 3},
    {"small_split": 2, "small_tiles": 8, "small_spw": 4},
    {"small_split": 5, "small_tiles": 5, "small_spw": 2},
    {"small_split": 33, "small_tiles": 7},
])
def test_decode_launch_shapes(nfp, knobs):
    # every combination of K-steps per wave, grid-level K split and tiles per workgroup
    # (odd and even, more than the layer has) gives the same answer
    W = workloads.weight_host(304, 2048 + 64, seed=21)
    try:
        for M in (16, 40):
            for k, v in knobs.items():                 # (the plain-GEMM comparison inside resets the knobs it pins)
                nfp.tune(k, v)
            run_both_modes(nfp, workloads.act_host(M, 2048 + 64, seed=21 + M), W, "%s M=%d" % (knobs, M))
    finally:
        for k in knobs:
            nfp.tune(k, -1)


@pytest.mark.parametrize("M,N,K", [
    (65, 128, 64), (128, 128, 128), (200, 264, 208), (300, 520, 1040), (512, 1024, 1024),
    (257, 129, 4096), (1024, 300, 528),
])
def test_prefill_sized_batches(nfp, M, N, K):
    W = workloads.weight_host(N, K, seed=M + N)
    X = workloads.act_host(M, K, seed=K)
    run_both_modes(nfp, X, W, "M=%d N=%d K=%d" % (M, N, K))


@pytest.mark.parametrize("knobs", [
    {"large_bm": 256, "large_split": 1},
    {"large_bm": 128, "large_split": 1},
    {"large_bm": 256, "large_split": 3},
    {"large_bm": 128, "large_split": 5},
    {"large_bm": 256, "large_bn": 128, "large_split": 1},
    {"large_bm": 128, "large_bn": 256, "large_split": 1},
    {"large_bm": 256, "large_bn": 128, "large_split": 2},
    {"large_bm": 128, "large_bn": 256, "large_split": 3},
    {"large_bm": 64, "large_split": 1},       # 64 x 128 tiles: NestedFP16 only, the other kinds ignore it
    {"large_bm": 64, "large_split": 4},
    {"small_max_m": 0},                       # route a decode-sized batch through the tiled kernel
    # the deeper load pipelines of the tiles below 256 x 256 (three or four LDS stages, eight token stages)
    {"large_deep": 1, "large_bm": 128, "large_bn": 128, "large_split": 1},
    {"large_deep": 1, "large_bm": 128, "large_bn": 128, "large_split": 3},
    {"large_deep": 1, "large_bm": 256, "large_bn": 128, "large_split": 1},
    {"large_deep": 1, "large_bm": 128, "large_bn": 256, "large_split": 2},
    {"large_deep": 1, "large_bm": 128, "large_bn": 256, "large_split": 8},
    {"large_deep": 0, "large_bm": 128, "large_bn": 128, "large_split": 1},
])
def test_prefill_launch_shapes(nfp, knobs):
    W = workloads.weight_host(520, 1040, seed=31)
    try:
        for M in (24, 300, 777):
            for k, v in knobs.items():                 # (the plain-GEMM comparison inside resets the knobs it pins)
                nfp.tune(k, v)
            X = workloads.act_host(M, 1040, seed=M)
            run_both_modes(nfp, X, W, "%s M=%d" % (knobs, M))
    finally:
        for k in knobs:
            nfp.tune(k, -1)


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_random_shapes_and_launch_shapes(nfp, seed):
    # seeded random problem sizes (ragged in every dimension) under random tile shapes and K
    # splits, both modes against the oracle
    rng = np.random.default_rng(seed)
    for case in range(12):
        M = int(rng.choice([rng.integers(1, 65), rng.integers(65, 300), rng.integers(300, 700)]))
        N = int(rng.choice([rng.integers(1, 65), rng.integers(65, 600), rng.integers(600, 1100)]))
        K = 16 * int(rng.choice([rng.integers(1, 9), rng.integers(9, 70), rng.integers(70, 120)]))
        knobs = {}
        if rng.random() < 0.75:
            knobs = {"large_bm": int(rng.choice([64, 128, 256])), "large_bn": int(rng.choice([128, 256])),
                     "large_split": int(rng.choice([1, 1, 2, 3, 5]))}
        W = workloads.weight_host(N, K, seed=100 * seed + case)
        X = workloads.act_host(M, K, seed=100 * seed + case + 50)
        for k, v in knobs.items():
            nfp.tune(k, v)
        try:
            run_both_modes(nfp, X, W, "seed %d case %d M=%d N=%d K=%d %s" % (seed, case, M, N, K, knobs),
                           check_plain=False)
        finally:
            for k in knobs:
                nfp.tune(k, -1)


@pytest.mark.parametrize("M", [49, 57, 64])
def test_tiled_route_of_49_to_64_tokens(nfp, M):
    # from 49 tokens on, FP16 mode leaves the streaming kernel for 64-token tiles split along K
    # (on all but the smallest layers): default routing, ragged N, against the oracle
    N, K = 4100 + 24, 1024 + 48
    W = workloads.weight_host(N, K, seed=410)
    X = workloads.act_host(M, K, seed=411)
    run_both_modes(nfp, X, W, "M=%d" % M, check_plain=False)


@pytest.mark.parametrize("M,N,K", [(50, 16384 + 40, 256 + 16), (35, 16384 + 8, 192), (64, 264, 14336 + 80)])
def test_fp8_mode_tiled_route_of_33_to_64_tokens(nfp, M, N, K):
    # FP8 mode takes 64-token tiles (E4M3 blocks through registers) on wide layers and on layers
    # with a long K: default routing, ragged N and K, against the oracle
    W = workloads.weight_host(N, K, seed=420)
    X = workloads.act_host(M, K, seed=421)
    run_both_modes(nfp, X, W, "M=%d N=%d K=%d" % (M, N, K), check_plain=False)


@pytest.mark.parametrize("M,N,K,bm,bn", [(300, 1100, 512, 128, 128), (300, 600, 256, 128, 128), (700, 2300, 384, 256, 256),
                                         (1000, 3000, 192, 128, 256), (520, 1160, 640, 256, 128)])
def test_xcd_grouped_tile_order_changes_nothing(nfp, M, N, K, bm, bn):
    # 2 .. 8 token tiles per weight tile: the workgroups take their tiles grouped by XCD (all token
    # tiles of a weight tile on one XCD; the last tiles_n % 8 weight tiles in launch order).  Every
    # tile is still computed exactly once: same bits as with the plain launch order, all kinds
    W = workloads.weight_host(N, K, seed=430)
    X = workloads.act_host(M, K, seed=431)
    Xd, Wd = to_dev(X), to_dev(W)
    up, lo = nfp.decompose(Wd, packed=(bm == 256))
    pins = {"large_bm": bm, "large_bn": bn, "large_split": 1}
    outs = {}
    for order in (0, -1):
        for k, v in pins.items():
            nfp.tune(k, v)
        nfp.tune("large_xcd_map", order)
        try:
            outs[order] = (bits(nfp.gemm(Xd, up, lo, nfp.MODE_FP16)), bits(nfp.plain_gemm_fp16(Xd, Wd)),
                           bits(nfp.gemm(Xd, up, None, nfp.MODE_FP8)))
        finally:
            for k in pins:
                nfp.tune(k, -1)
            nfp.tune("large_xcd_map", -1)
    for a, b in zip(outs[0], outs[-1]):
        assert np.array_equal(a, b)
    assert_gemm_close(outs[-1][0].view(np.float16), oracle.gemm_fp16(X, W), "grouped tile order, FP16 mode")


def test_one_hot_tokens_return_weights_exactly(nfp):
    # FP16 mode with one-hot rows returns the reconstructed weights themselves: checks the
    # operand layout, the transposition and Alg. 1 bit-exactly inside the GEMM kernels
    N, K = 200, 192
    W = workloads.weight_host(N, K, seed=77)
    X = np.zeros((K, K), np.float16)
    X[np.arange(K), np.arange(K)] = 1.0
    Wd = to_dev(W)
    up, lo = nfp.decompose(Wd)
    for M in (16, 64, K):                      # streaming and tiled kernels
        y = nfp.gemm(to_dev(X[:M]), up, lo, nfp.MODE_FP16)
        assert np.array_equal(bits(y), np.ascontiguousarray(W[:, :M].T).view(np.uint16)), M
    # FP8 mode: 448 on the diagonal gives scale 1; output = e4m3(upper) * 448 * 2^-8, exact in fp16
    X8 = (X * np.float16(448.0)).astype(np.float16)
    up_ref, _, _ = oracle.decompose(W)
    dec = torch.from_numpy(up_ref).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    want = (dec.T * 448.0 * 2.0 ** -8).astype(np.float16)
    for M in (16, 64, K):
        y = nfp.gemm(to_dev(X8[:M]), up, None, nfp.MODE_FP8).cpu().numpy()
        # equal as numbers: a weight that rounds to -0 in E4M3 gives -0 in the oracle's product
        # and +0 from an fp32 accumulator that starts at +0
        assert np.array_equal(y, want[:M]), M


def test_fp8_mode_never_reads_the_lower_plane(nfp):
    W = workloads.weight_host(256, 512, seed=5)
    Wd = to_dev(W)
    for packed in (False, True):
        up, lo = nfp.decompose(Wd, packed=packed)
        for M in (8, 200):
            X = to_dev(workloads.act_host(M, 512, seed=6))
            a = nfp.gemm(X, up, None, nfp.MODE_FP8)
            junk = nfp.PackedPlane(lo.N, lo.K, data=torch.full_like(lo.data, 0xAB)) if packed else torch.full_like(lo, 0xAB)
            b = nfp.gemm(X, up, junk, nfp.MODE_FP8)
            assert np.array_equal(bits(a), bits(b))
        with pytest.raises(nfp.NestedFPError):
            nfp.gemm(X, up, None, nfp.MODE_FP16)


def test_static_activation_scale_and_prequantized_entry(nfp):
    W = workloads.weight_host(96, 256, seed=8)
    X = workloads.act_host(12, 256, seed=8)
    Wd, Xd = to_dev(W), to_dev(X)
    up, lo = nfp.decompose(Wd)
    up_ref, _, _ = oracle.decompose(W)
    sc = torch.tensor([0.03125], dtype=torch.float32, device="cuda:0")
    y = nfp.gemm(Xd, up, None, nfp.MODE_FP8, act_scale=sc)
    Xq, s = oracle.quantize_act(X, static_scale=0.03125)
    assert_gemm_close(y.cpu().numpy(), oracle.gemm_fp8(Xq, s, up_ref), "static scale")
    Xq_d, s_d = nfp.quantize_act(Xd)
    y2 = nfp.gemm_fp8_prequantized(Xq_d, s_d, up)
    y3 = nfp.gemm(Xd, up, None, nfp.MODE_FP8)
    assert np.array_equal(bits(y2), bits(y3))
    y4 = nfp.gemm_fp8_prequantized(Xq_d, s_d, nfp.pack_plane(up))
    assert np.array_equal(bits(y4), bits(y3))


def test_strided_activations_and_output(nfp):
    N, K, M = 144, 320, 20
    W = workloads.weight_host(N, K, seed=3)
    Xbig = workloads.act_host(M, K + 64, seed=3)
    Wd = to_dev(W)
    up, lo = nfp.decompose(Wd)
    Xd = to_dev(Xbig)[:, :K]
    out = torch.full((M, N + 16), 7.0, dtype=torch.float16, device="cuda:0")
    nfp.gemm(Xd, up, lo, nfp.MODE_FP16, out=out[:, :N])
    ref = oracle.gemm_fp16(Xbig[:, :K], W)
    got = out.cpu().numpy()
    assert_gemm_close(got[:, :N], ref, "strided")
    assert np.all(got[:, N:] == np.float16(7.0))


def test_results_are_deterministic(nfp):
    W = workloads.weight_host(1024, 4096, seed=4)
    Wd = to_dev(W)
    up, lo = nfp.decompose(Wd)
    for M in (16, 384):
        X = to_dev(workloads.act_host(M, 4096, seed=4))
        for mode in (nfp.MODE_FP16, nfp.MODE_FP8):
            a = bits(nfp.gemm(X, up, lo, mode))
            b = bits(nfp.gemm(X, up, lo, mode))
            assert np.array_equal(a, b)


def test_mode_switch_keeps_planes_and_memory(nfp):
    # per-step mode switching: same plane pointers, no allocation growth, planes unchanged
    layers = []
    for i in range(4):
        W = to_dev(workloads.weight_host(512, 1024, seed=40 + i))
        layers.append(nfp.decompose(W))
        del W
    X = to_dev(workloads.act_host(64, 1024, seed=50))
    out = torch.empty((64, 512), dtype=torch.float16, device="cuda:0")
    ws = nfp.new_workspace(max(nfp.gemm_workspace_size(64, 512, 1024, m) for m in (0, 1)), "cuda:0")
    snap = [(u.clone(), l.clone()) for u, l in layers]
    ptrs = [(u.data_ptr(), l.data_ptr()) for u, l in layers]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for step in range(32):
        mode = nfp.MODE_FP8 if (step // 8) % 2 else nfp.MODE_FP16
        for u, l in layers:
            nfp.gemm(X, u, None if mode == nfp.MODE_FP8 else l, mode, out=out, workspace=ws)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert ptrs == [(u.data_ptr(), l.data_ptr()) for u, l in layers]
    for (u, l), (su, sl) in zip(layers, snap):
        assert torch.equal(u, su) and torch.equal(l, sl)


@pytest.mark.parametrize("name,M", [("qkv", 16), ("down", 4), ("o", 64), ("gate_up", 1)])
def test_llama8b_decode_shapes_full_output(nfp, name, M):
    N, K = workloads.LLAMA3_8B[name]
    W = workloads.weight_host(N, K, seed=N % 97)
    X = workloads.act_host(M, K, seed=M)
    run_both_modes(nfp, X, W, "%s M=%d" % (name, M), check_plain=(name != "gate_up"))


def _full_size_check(nfp, N, K, Ms, sigma, tag, seed, pin_sets=None):
    """Full-size launches in the built-in launch shapes (what bench.py times), both plane layouts.
    Planes: every byte against the oracle.  Both GEMM modes: against the oracle on a structured
    sample of at least 2^15 outputs per batch size -- complete rows, complete columns and the
    first and last row / column of the tile bands (helpers.structured_sample); the whole output
    of FP16 mode bit for bit against the plain FP16 GEMM on packed weights (same kernel minus
    Alg. 1) and, under pinned launch shapes, against the plain GEMM on row-major weights."""
    Wd = workloads.weight_device(N, K, sigma, seed=seed)
    W = Wd.cpu().numpy()
    up_ref, lo_ref, bad = decompose_ref(W)
    assert bad == 0
    planes = {}
    for packed in (False, True):
        up, lo = nfp.decompose(Wd, packed=packed)
        if packed:
            assert np.array_equal(up.unpack().cpu().numpy(), up_ref) and np.array_equal(lo.unpack().cpu().numpy(), lo_ref)
        else:
            assert np.array_equal(up.cpu().numpy(), up_ref) and np.array_equal(lo.cpu().numpy(), lo_ref)
        planes[packed] = (up, lo)
    Wp = nfp.pack_fp16(Wd)
    for M in Ms:
        print("  %s M=%d" % (tag, M), flush=True)
        Xd = workloads.act_device(M, K, seed=seed + 1 + M)
        X = Xd.cpu().numpy()
        Xq, sc = oracle.quantize_act(X)
        y16 = {p: nfp.gemm(Xd, planes[p][0], planes[p][1], nfp.MODE_FP16) for p in planes}
        y8 = {p: nfp.gemm(Xd, planes[p][0], None, nfp.MODE_FP8) for p in planes}
        assert torch.equal(y16[False], y16[True]) and torch.equal(y8[False], y8[True]), tag + ": layouts differ"
        assert torch.equal(nfp.plain_gemm_fp16(Xd, Wp), y16[True]), tag + ": FP16 mode differs from plain FP16 on packed weights"
        for pins in (pin_sets(M) if pin_sets else []):
            for k, v in pins.items():
                nfp.tune(k, v)
            try:
                assert torch.equal(nfp.gemm(Xd, planes[False][0], planes[False][1], nfp.MODE_FP16), nfp.plain_gemm_fp16(Xd, Wd)), \
                    tag + ": FP16 mode differs from plain fp16 under %s" % pins
            finally:
                for k in pins:
                    nfp.tune(k, -1)
        got16, got8 = y16[False].cpu().numpy(), y8[False].cpu().numpy()
        total = 0
        for rows, cols in structured_sample(M, N, seed=seed + M):
            Xs, Ws = X[rows], W[cols]
            assert_gemm_close(got16[np.ix_(rows, cols)], oracle.gemm_fp16(Xs, Ws), "%s M=%d FP16 mode" % (tag, M))
            assert_gemm_close(got8[np.ix_(rows, cols)], oracle.gemm_fp8(Xq[rows], sc[rows], up_ref[cols]),
                              "%s M=%d FP8 mode" % (tag, M))
            total += len(rows) * len(cols)
        assert total >= min(1 << 15, M * N)


def _default_pins(M):
    if M <= 64:
        pins = [{"small_max_m": 64, "small_spw": 4}]
        if M > 32:
            pins.append({"small_max_m": 0, "large_bm": 64, "large_split": 4})     # 64-token tiles of the tiled kernels
        return pins
    return [{"large_bm": 256, "large_bn": 256, "large_split": 1}]


@pytest.mark.parametrize("name", ["qkv", "o", "gate_up", "down"])
def test_llama8b_shapes_structured_sample(nfp, name):
    # configs[1] and configs[2]: decode and prefill batch sizes on the 8B linears
    N, K = workloads.LLAMA3_8B[name]
    _full_size_check(nfp, N, K, [1, 16, 64, 512, 2048, 8192], workloads.SIGMA_W_8B, "8B " + name, seed=N % 97,
                     pin_sets=_default_pins)


@pytest.mark.parametrize("name", ["qkv", "o", "gate_up", "down"])
def test_llama70b_shapes_structured_sample(nfp, name):
    # configs[3]: the unsharded 70B linears on one GPU, sigma 0.015, decode to prefill
    N, K = workloads.LLAMA3_70B[name]
    _full_size_check(nfp, N, K, [1, 2, 16, 64, 128, 512, 2048, 8192], workloads.SIGMA_W_70B, "70B " + name, seed=70 + N % 89,
                     pin_sets=_default_pins)


@pytest.mark.parametrize("N,K,Ms", [(4096, 4096, [17, 24, 33, 48, 100, 128, 200, 256]), (6144, 4096, [20, 40, 96, 250]),
                                    (5120, 14336, [12, 17, 32, 40, 128])])
def test_batches_between_the_kernel_families_structured_sample(nfp, N, K, Ms):
    # 17 ... 256 tokens: where the built-in choice moves from the streaming kernel to the 64-token tiles
    # (by class and layer size) and where the table of timed launch shapes puts 64-token tiles under
    # batches of 128 and 256 tokens on small layers
    _full_size_check(nfp, N, K, Ms, workloads.SIGMA_W_8B, "N=%d K=%d" % (N, K), seed=N % 83, pin_sets=_default_pins)


@pytest.mark.parametrize("N,K,M", [(40, 32, 70000), (256, 65536, 8), (264, 65536 + 16, 70), (1000, 16, 1000), (4096, 4096, 20000)])
def test_extreme_aspect_ratios_sampled(nfp, N, K, M):
    # tens of thousands of tokens on a sliver of a layer, the longest rows, the shortest K, a prefill
    # of 20000 tokens
    _full_size_check(nfp, N, K, [M], workloads.SIGMA_W_8B, "N=%d K=%d" % (N, K), seed=N % 97 + M % 89, pin_sets=_default_pins)


def test_vocabulary_sized_layer_sampled(nfp):
    # a Llama-3 output projection (128256 x 4096): half a billion weights, a row count that is no
    # multiple of any tile, 8-tile groups of the XCD order plus a tail
    _full_size_check(nfp, 128256, 4096, [4, 130], workloads.SIGMA_W_8B, "lm_head", seed=128)


@pytest.mark.parametrize("N,K,Ms", [(28672, 5120, [96]), (65536, 5120, [1024]), (35840, 5120, [32])])
def test_paper_kernel_benchmark_shapes_sampled(nfp, N, K, Ms):
    # the (N, K) shapes of Sec. 5.2 / Fig. 6, M inside its 32..2048 sweep
    _full_size_check(nfp, N, K, Ms, workloads.SIGMA_W_8B, "N=%d K=%d" % (N, K), seed=N % 89, pin_sets=_default_pins)


@pytest.mark.parametrize("M,N,K,split", [(16, 4096, 4096, -1), (1, 6144, 4096, -1), (5, 304, 2048 + 64, 1),
                                         (16, 520, 528, 1), (13, 272, 4096 + 16, 1)])
def test_fused_activation_quantisation_equals_the_two_kernel_path(nfp, M, N, K, split):
    # decode batches whose K fits one workgroup pass can quantise the activations inside the GEMM
    # kernel (knob small_fuse_quant); the result must be bit-identical to quantise-then-multiply and match the oracle
    W = workloads.weight_host(N, K, seed=N + K)
    X = workloads.act_host(M, K, seed=M + K)
    X[0, :] = 0                                        # an all-zero token: scale 1
    Xd = to_dev(X)
    up, _ = nfp.decompose(to_dev(W), packed=True)      # the fused kind exists for packed planes
    sc = torch.tensor([0.0123], dtype=torch.float32, device="cuda:0")
    nfp.tune("small_split", split)
    nfp.tune("small_fuse_quant", 1)
    try:
        fused = bits(nfp.gemm(Xd, up, None, nfp.MODE_FP8))
        fused_static = bits(nfp.gemm(Xd, up, None, nfp.MODE_FP8, act_scale=sc))
        nfp.tune("small_fuse_quant", 0)
        plain = bits(nfp.gemm(Xd, up, None, nfp.MODE_FP8))
        plain_static = bits(nfp.gemm(Xd, up, None, nfp.MODE_FP8, act_scale=sc))
        Xq_d, s_d = nfp.quantize_act(Xd)
        pre = bits(nfp.gemm_fp8_prequantized(Xq_d, s_d, up))
    finally:
        nfp.tune("small_fuse_quant", -1)
        nfp.tune("small_split", -1)
    assert np.array_equal(fused, plain) and np.array_equal(fused, pre)
    assert np.array_equal(fused_static, plain_static)
    Xq, s = oracle.quantize_act(X)
    up_ref, _, _ = oracle.decompose(W)
    assert_gemm_close(fused.view(np.float16), oracle.gemm_fp8(Xq, s, up_ref), "fused FP8 mode")



@pytest.mark.parametrize("M", [4, 40, 200])
def test_memory_outside_the_matrix_never_reaches_the_result(nfp, M):
    # K = 1040 is no multiple of the kernels' 64- and 128-column steps, so the last step of a row
    # runs past K: into the next row, or into the gap of a strided matrix.  Exception layers may
    # hold Inf / NaN there (Sec. 4.1 "Handling Exception Layers"), and E4M3 weights passed to the
    # plain FP8 GEMM may hold NaN codes; neither may touch the other rows' outputs.
    N, K, ld = 80, 1040, 1104
    big = workloads.weight_host(N, ld, seed=11)
    big[:, K:] = np.float16(np.nan)                     # the gap columns of the strided matrix
    big[17, 0] = np.float16(np.inf)                     # head of the row after row 16
    big[33, 0:64] = np.float16(np.nan)
    X = workloads.act_host(M, K, seed=12)
    Xd = to_dev(X)
    Wd = to_dev(big)[:, :K]
    assert Wd.stride(0) == ld
    y = nfp.plain_gemm_fp16(Xd, Wd).cpu().numpy()
    ref = oracle.gemm_fp16(X, np.ascontiguousarray(big[:, :K]))
    clean = np.array([n for n in range(N) if n not in (17, 33)])
    assert_gemm_close(y[:, clean], ref[:, clean], "plain FP16, strided W with NaN gaps, M=%d" % M)
    assert not np.isfinite(y[:, [17, 33]]).any()        # the rows that do hold Inf / NaN say so
    # E4M3 weights: a whole 16-row tile of NaN codes next to clean tiles, both storage orders
    rng = np.random.default_rng(5)
    Wq = rng.integers(0, 0x78, size=(48, K), dtype=np.uint8)          # finite codes
    dirty = Wq.copy()
    dirty[16:32, :] = 0x7F
    for packed in (False, True):
        a, b = to_dev(Wq), to_dev(dirty)
        if packed:
            a, b = nfp.pack_plane(a), nfp.pack_plane(b)
        ya = nfp.plain_gemm_fp8(Xd, a, 2.0 ** -8).cpu().numpy()
        yb = nfp.plain_gemm_fp8(Xd, b, 2.0 ** -8).cpu().numpy()
        keep = np.r_[0:16, 32:48]
        assert np.isfinite(ya).all()
        assert np.array_equal(ya[:, keep].view(np.uint16), yb[:, keep].view(np.uint16)), "packed=%s" % packed
        assert np.isnan(yb[:, 16:32]).all()


@pytest.mark.parametrize("M,N,K,knobs", [(16, 4096 + 8, 14336, {}), (4, 300, 28672, {}),
                                         (16, 520, 4096, {"small_split": 4, "small_tiles": 2}),
                                         (40, 304, 2048 + 64, {"small_split": 3, "small_tiles": 3}),
                                         (7, 1027, 1024, {"small_split": 8, "small_tiles": 5, "small_spw": 2})])
def test_split_k_finished_by_the_last_workgroup_equals_the_reduction_launch(nfp, M, N, K, knobs):
    # a grid-level K split is summed by the last workgroup of each tile column to arrive, in slice
    # order; the stand-alone reduction launch (knob fused_reduce = 0) gives the same bits, the
    # arrival counters are back at zero afterwards, and the result matches the oracle
    W = workloads.weight_host(N, K, seed=N)
    X = workloads.act_host(M, K, seed=K)
    Wd, Xd = to_dev(W), to_dev(X)
    ws = nfp.new_workspace(max(nfp.gemm_workspace_size(M, N, K, m) for m in (0, 1)) + (64 << 20), "cuda:0")
    for k, v in knobs.items():
        nfp.tune(k, v)
    try:
        for packed in (False, True):
            up, lo = nfp.decompose(Wd, packed=packed)
            outs = {}
            for fused in (-1, 0):
                nfp.tune("fused_reduce", fused)
                outs[fused] = [bits(nfp.gemm(Xd, up, lo, nfp.MODE_FP16, workspace=ws)),
                               bits(nfp.gemm(Xd, up, None, nfp.MODE_FP8, workspace=ws)),
                               bits(nfp.gemm(Xd, up, lo, nfp.MODE_FP16, workspace=ws))]     # a second call on the same counters
            nfp.tune("fused_reduce", -1)
            for a, b in zip(outs[-1], outs[0]):
                assert np.array_equal(a, b)
            assert int(ws[:nfp.WORKSPACE_COUNTER_BYTES].count_nonzero()) == 0
            assert_gemm_close(outs[-1][0].view(np.float16), oracle.gemm_fp16(X, W), "fused split-K, FP16 mode")
    finally:
        nfp.tune("fused_reduce", -1)
        for k in knobs:
            nfp.tune(k, -1)


@pytest.mark.parametrize("M,N,K,shapes", [
    (256, 2048, 1024, [{"large_bm": 128, "large_bn": 128, "large_split": 1}, {"large_bm": 128, "large_bn": 128, "large_split": 2},
                       {"large_bm": 256, "large_bn": 256, "large_split": 4}, {"large_bm": 128, "large_bn": 256, "large_split": 1, "large_deep": 1},
                       {"large_bm": 256, "large_bn": 128, "large_split": 3}]),
    (16, 16384, 1024, [{"small_split": 1}, {"small_split": 2}, {"small_split": 4, "fused_reduce": 0}, {"small_split": 8, "small_spw": 2}]),
    (64, 8192, 2048, [{"small_split": 1}, {"small_split": 2}, {"small_max_m": 32, "large_split": 1}, {"small_max_m": 32, "large_split": 4}])])
def test_fp8_mode_scales_and_rounds_alike_in_every_launch_shape(nfp, M, N, K, shapes):
    # Operands whose E4M3 codes are small integers: every partial sum is an integer below 2^24, so the
    # FP32 accumulation is exact in any order and any K split, and the output is pinned to one
    # definition -- the FP32 sum times the FP32 scale, rounded to FP32, then to FP16 -- that every
    # kernel and the split-K reduction must follow bit for bit (a product fused with the conversion
    # rounds once and differs in about one output in 10^4)
    rng = np.random.default_rng(M + N)
    kw = rng.integers(-15, 16, size=(N, K))
    jx = rng.integers(-15, 16, size=(M, K))
    s_act = np.float32(0.37)
    W = (kw / 256.0).astype(np.float16)
    X = (jx * np.float64(s_act)).astype(np.float16)
    Wd, Xd = to_dev(W), to_dev(X)
    sc = torch.tensor([float(s_act)], dtype=torch.float32, device="cuda:0")
    acc = (jx @ kw.T).astype(np.float32)
    assert np.abs(jx @ kw.T).max() < 2 ** 24
    want = (acc * (s_act * np.float32(2.0 ** -8))).astype(np.float32).astype(np.float16).view(np.uint16)
    for packed in (False, True):
        up, _ = nfp.decompose(Wd, packed=packed)
        for knobs in shapes:
            for k, v in knobs.items():
                nfp.tune(k, v)
            try:
                got = bits(nfp.gemm(Xd, up, None, nfp.MODE_FP8, act_scale=sc))
            finally:
                for k in knobs:
                    nfp.tune(k, -1)
            assert np.array_equal(got, want), "%s, packed=%s: %d outputs differ" % (knobs, packed, int((got != want).sum()))


@pytest.mark.parametrize("bm,bn", [(128, 128), (256, 128), (128, 256)])
def test_deeper_load_pipelines_change_nothing(nfp, bm, bn):
    # three / four LDS stages (tiled kernels) and eight token stages (register-path kernels): the
    # same sums in the same order, so the same bits as the two-stage pipelines, on a K long enough
    # to go round the rings several times and a K of a single tile
    for M, N, K in ((300, 520, 2064), (129, 260, 64), (513, 1030, 4096)):
        W = workloads.weight_host(N, K, seed=K)
        Xd, Wd = to_dev(workloads.act_host(M, K, seed=M)), to_dev(W)
        planes = {p: nfp.decompose(Wd, packed=p) for p in (False, True)}
        Wp = nfp.pack_fp16(Wd)
        outs = {}
        for deep in (0, 1):
            for k, v in {"large_bm": bm, "large_bn": bn, "large_split": 1, "large_deep": deep}.items():
                nfp.tune(k, v)
            try:
                outs[deep] = [bits(nfp.gemm(Xd, planes[p][0], planes[p][1], nfp.MODE_FP16)) for p in planes] + \
                             [bits(nfp.gemm(Xd, planes[p][0], None, nfp.MODE_FP8)) for p in planes] + \
                             [bits(nfp.plain_gemm_fp16(Xd, Wd)), bits(nfp.plain_gemm_fp16(Xd, Wp))]
            finally:
                for k in ("large_bm", "large_bn", "large_split", "large_deep"):
                    nfp.tune(k, -1)
        for a, b in zip(outs[0], outs[1]):
            assert np.array_equal(a, b), (bm, bn, M, N, K)
        assert_gemm_close(outs[1][0].view(np.float16), oracle.gemm_fp16(Xd.cpu().numpy(), W), "deep pipelines")
