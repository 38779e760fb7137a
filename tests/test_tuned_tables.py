"""The tables of timed launch shapes that the library compiles in must only hold launch shapes the
kernels exist for (they are generated files: paper_2506_02024_amd/tune_tiles.py)."""
import os
import re

CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2506_02024_amd", "csrc")
ROW = re.compile(r"^\{([-0-9, ]+)\},")


def rows(name):
    out = []
    for line in open(os.path.join(CSRC, name)):
        m = ROW.match(line.strip())
        if m:
            out.append(tuple(int(v) for v in m.group(1).split(",")))
    return out


def test_tiled_kernel_table_holds_legal_launch_shapes():
    seen = set()
    for cls, N, K, M, tm, tn, split, deep in rows("tuned_tiles.inc"):
        assert cls in (0, 1, 2)
        assert N > 0 and K > 0 and K % 16 == 0
        assert M in (32, 64, 96, 128, 192, 256, 384, 512, 768, 1024, 1536, 2048, 4096, 8192)
        assert (tm, tn) in ((64, 128), (128, 128), (128, 256), (256, 128), (256, 256))
        assert split in (1, 2, 3, 4, 6, 8)
        if tm == 64:
            assert M <= 256 and deep == 0                 # 64-token tiles: no deeper pipeline
        else:
            assert M > 64                                 # batches of up to 64 tokens take 64-token tiles only
        if deep:
            assert (tm, tn) != (256, 256) and (cls != 1 or tm == 128)   # smaller tiles; the register path on 128 tokens only
        kt = (K if cls == 2 else 2 * K) // 128
        assert split == 1 or split <= kt // 4
        assert (cls, N, K, M) not in seen                 # one entry per problem
        seen.add((cls, N, K, M))


def test_streaming_kernel_table_holds_legal_launch_shapes():
    seen = set()
    for cls, N, K, spw, split, tiles in rows("tuned_small.inc"):
        assert cls in (0, 1, 2)
        assert N > 0 and K > 0 and K % 16 == 0
        assert spw in ((2, 4, 8) if cls == 0 else (2, 4))
        assert split in (1, 2, 3, 4, 6, 8)
        assert 1 <= tiles <= 16
        assert (cls, N, K) not in seen
        seen.add((cls, N, K))
