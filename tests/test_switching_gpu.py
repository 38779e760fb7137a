"""GPU parity: per-iteration mode switching on real layer shapes (Sec. 5.4) -- the same planes
serve both modes, a switch moves no data and allocates nothing, and the outputs on both sides of
every switch match the oracle; the load-aware threshold policy picks the mode per step."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_02024_amd import workloads
from helpers import assert_gemm_close, decompose_ref

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def nfp():
    from paper_2506_02024_amd import binding

    return binding


def _sample(M, N, seed):
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([[0, M - 1], rng.choice(M, size=min(M, 6), replace=False)]))
    cols = np.unique(np.concatenate([[0, N - 1], rng.choice(N, size=min(N, 510), replace=False)]))
    return rows, cols


class _Stack:
    """`layers` x {qkv, o, gate_up, down} of the 8B shapes, decomposed once; host copies of the
    sampled weight rows and their oracle planes for checking outputs."""

    def __init__(self, nfp, layers, packed, shapes=workloads.LLAMA3_8B, sigma=workloads.SIGMA_W_8B):
        self.linears = []
        for layer in range(layers):
            for j, (name, (N, K)) in enumerate(shapes.items()):
                Wd = workloads.weight_device(N, K, sigma, seed=900 + 4 * layer + j)
                up, lo = nfp.decompose(Wd, packed=packed)
                cols = _sample(4, N, seed=layer * 4 + j)[1]
                Ws = Wd[torch.from_numpy(cols).cuda()].cpu().numpy()
                up_s, _, bad = decompose_ref(Ws)
                assert bad == 0
                self.linears.append(dict(name=name, N=N, K=K, up=up, lo=lo, cols=cols, Ws=Ws, up_s=up_s))
                del Wd

    def check(self, nfp, lin, X_host, Xq_sc, y, mode, rows, what):
        got = y[torch.from_numpy(rows).cuda()][:, torch.from_numpy(lin["cols"]).cuda()].cpu().numpy()
        if mode == nfp.MODE_FP16:
            ref = oracle.gemm_fp16(X_host[rows], lin["Ws"])
        else:
            Xq, sc = Xq_sc
            ref = oracle.gemm_fp8(Xq[rows], sc[rows], lin["up_s"])
        assert_gemm_close(got, ref, what)


@pytest.mark.parametrize("M,packed", [(64, True), (64, False), (2048, True), (2048, False)])
def test_mode_alternation_on_8b_layer_shapes(nfp, M, packed):
    # configs[4] on two layers of the stack: the mode flips every 8 steps; the steps next to each
    # flip are checked against the oracle, the planes and the allocator are not touched
    stack = _Stack(nfp, 2, packed)
    shapes = workloads.LLAMA3_8B
    X = {n: workloads.act_device(M, shapes[n][1], seed=60 + j) for j, n in enumerate(shapes)}
    Xh = {n: X[n].cpu().numpy() for n in X}
    Xq = {n: oracle.quantize_act(Xh[n]) for n in X}
    Y = {n: torch.empty((M, shapes[n][0]), dtype=torch.float16, device="cuda:0") for n in shapes}
    ws = nfp.new_workspace(max(nfp.gemm_workspace_size(M, N, K, m) for (N, K) in shapes.values() for m in (0, 1)), "cuda:0")
    raw = lambda p: p.data if hasattr(p, "unpack") else p
    snap = [(raw(l["up"]).clone(), raw(l["lo"]).clone()) for l in stack.linears]
    ptrs = [(l["up"].data_ptr(), l["lo"].data_ptr()) for l in stack.linears]
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    checked = 0
    for step in range(32):
        mode = nfp.MODE_FP8 if (step // 8) % 2 else nfp.MODE_FP16
        near_flip = step % 8 in (0, 7)
        for i, lin in enumerate(stack.linears):
            n = lin["name"]
            nfp.gemm(X[n], lin["up"], None if mode == nfp.MODE_FP8 else lin["lo"], mode, out=Y[n], workspace=ws)
            if near_flip and (i + step) % 4 == 0:          # two linears per checked step, rotating over the shapes
                rows = _sample(M, lin["N"], seed=step)[0]
                stack.check(nfp, lin, Xh[n], Xq[n], Y[n], mode, rows, "step %d %s mode %d" % (step, n, mode))
                checked += 1
    torch.cuda.synchronize()
    assert checked >= 16
    assert torch.cuda.memory_allocated() == before
    assert ptrs == [(l["up"].data_ptr(), l["lo"].data_ptr()) for l in stack.linears]
    for l, (su, sl) in zip(stack.linears, snap):
        assert torch.equal(raw(l["up"]), su) and torch.equal(raw(l["lo"]), sl)


def test_threshold_policy_over_a_bursty_arrival_sequence(nfp):
    # Sec. 5.4: FP8 mode iff the iteration's token count exceeds 1024.  A seeded synthetic arrival
    # sequence (the paper's trace is not available) over a small stack: the mode chosen per step,
    # and the outputs of every step against the oracle
    assert [nfp.select_mode(t) for t in (1, 1023, 1024, 1025, 8192)] == [0, 0, 0, 1, 1]
    assert nfp.select_mode(300, threshold=256) == nfp.MODE_FP8 and nfp.select_mode(256, threshold=256) == nfp.MODE_FP16
    shapes = {"a": (1536, 1024), "b": (1024, 1536 + 64)}
    stack = _Stack(nfp, 2, packed=False, shapes=shapes)
    rng = np.random.default_rng(11)
    choices = np.array([16, 48, 64, 200, 512, 1024, 1025, 1500, 2048])
    seq = [int(choices[min(8, int(abs(rng.normal(0, 2.0)) + (4 if rng.random() < 0.3 else 0)))]) for _ in range(24)]
    seq[3], seq[4] = 1024, 1025                           # both sides of the threshold
    fp8_steps = 0
    for step, tokens in enumerate(seq):
        mode = nfp.select_mode(tokens)
        assert mode == (nfp.MODE_FP8 if tokens > 1024 else nfp.MODE_FP16)
        fp8_steps += mode == nfp.MODE_FP8
        for lin in stack.linears:
            Xd = workloads.act_device(tokens, lin["K"], seed=step)
            Xh = Xd.cpu().numpy()
            y = nfp.gemm(Xd, lin["up"], None if mode == nfp.MODE_FP8 else lin["lo"], mode)
            rows = _sample(tokens, lin["N"], seed=step)[0]
            stack.check(nfp, lin, Xh, oracle.quantize_act(Xh) if mode == nfp.MODE_FP8 else None, y, mode, rows,
                        "step %d tokens %d" % (step, tokens))
    assert 0 < fp8_steps < len(seq)
