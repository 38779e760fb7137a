"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

Holds shapes and random-number recipes only -- none of the method's arithmetic.
The paper measures its kernels on the linear-layer *shapes* of public models
(Sec. 5.2) and reports weight ranges of real checkpoints (Sec. 4.1, Fig. 3b:
Llama 3.1 8B weights lie within +-0.92).  No checkpoint is available here, so
Gaussian weights far inside the format's range stand in for them, and Gaussian
activations for the token batch.
"""
import numpy as np

# (N, K) of the four linears of one decoder layer, fused as serving stacks run them.
LLAMA3_8B = {
    "qkv": (6144, 4096),
    "o": (4096, 4096),
    "gate_up": (28672, 4096),
    "down": (4096, 14336),
}
LLAMA3_70B = {
    "qkv": (10240, 8192),
    "o": (8192, 8192),
    "gate_up": (57344, 8192),
    "down": (8192, 28672),
}
# The kernel-benchmark shapes of Sec. 5.2 (Fig. 6), M swept 32..2048 in steps of 32.
PAPER_KERNEL_SHAPES = [(28672, 4096), (28672, 5120), (35840, 5120), (65536, 5120)]

SIGMA_W_8B = 0.02
SIGMA_W_70B = 0.015
DECODE_M = (1, 4, 16, 64)
PREFILL_M = (512, 2048, 8192)


def weight_host(N, K, sigma=SIGMA_W_8B, seed=0):
    """[N,K] float16 Gaussian weights on the host (numpy)."""
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((N, K), dtype=np.float32) * np.float32(sigma)).astype(np.float16)


def act_host(M, K, seed=1, sigma=1.0):
    """[M,K] float16 Gaussian activations on the host (numpy)."""
    rng = np.random.default_rng(1000003 + seed)
    return (rng.standard_normal((M, K), dtype=np.float32) * np.float32(sigma)).astype(np.float16)


def weight_device(N, K, sigma=SIGMA_W_8B, seed=0, device="cuda:0"):
    """[N,K] float16 Gaussian weights generated on the device (torch's seeded generator).

    Used where the host recipe would take minutes (multi-GiB stacks); callers that
    need the same values on the host copy them back."""
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(seed)
    w = torch.empty((N, K), dtype=torch.float16, device=device)
    w.normal_(0.0, sigma, generator=g)
    return w


def act_device(M, K, seed=1, sigma=1.0, device="cuda:0"):
    import torch

    g = torch.Generator(device=device)
    g.manual_seed(1000003 + seed)
    x = torch.empty((M, K), dtype=torch.float16, device=device)
    x.normal_(0.0, sigma, generator=g)
    return x


def all_fp16_words():
    """Every FP16 bit pattern, 0x0000..0xFFFF, as uint16."""
    return np.arange(65536, dtype=np.uint32).astype(np.uint16)


def sample_indices(M, N, rows, cols, seed=0):
    """Seeded sample of output rows/cols for spot checks of large outputs."""
    rng = np.random.default_rng(7919 + seed)
    r = np.sort(rng.choice(M, size=min(rows, M), replace=False))
    c = np.sort(rng.choice(N, size=min(cols, N), replace=False))
    return r, c
