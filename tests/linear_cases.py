"""Shard shapes (M, Nn, K) that reach every variant of the linear layer's kernels:
each instantiated (batch-tile rows, workgroup columns) of the weight-streaming
kernel, with and without a K split, with one and with several batch tiles, and
the tiled kernel; all with ragged edges.  The CPU suite checks, through the
library's launch query, that every shape still lands on the variant named here
and that no instantiated variant is left out; the GPU suite runs them against the
oracle."""

# (M, Nn, K, tile_rows, tile_cols, split?)      tiled kernel: rows = cols = 256
CASES = [
    (1, 208, 256, 32, 32, False),
    (7, 208, 2048, 32, 32, True),
    (1, 28680, 1088, 32, 128, False),
    (16, 9000, 3072, 32, 128, True),
    (65, 208, 256, 64, 32, False),
    (65, 208, 2048, 64, 32, True),
    (65, 4104, 256, 64, 64, False),
    (65, 528, 4096, 64, 64, True),
    (65, 9000, 1088, 64, 128, False),
    (130, 2056, 4096, 64, 128, True),
    (200, 9000, 512, 96, 128, False),
    (130, 3080, 3072, 96, 128, True),
    (777, 208, 4096, 128, 32, True),
    (200, 7000, 256, 128, 64, False),
    (200, 2056, 2048, 128, 64, True),
    (300, 9000, 512, 128, 128, False),
    (200, 4104, 3072, 128, 128, True),
    (1000, 4104, 256, 192, 128, False),
    (130, 4104, 6144, 192, 128, True),
    (777, 7000, 256, 256, 128, False),
    (200, 4104, 8320, 256, 128, True),
    (520, 19000, 256, 256, 256, False),
]

# every (rows, cols) the library instantiates; (256, 256) is the tiled kernel
VARIANTS = {(32, 32), (32, 128), (64, 32), (64, 64), (64, 128), (96, 128), (128, 32), (128, 64), (128, 128),
            (192, 128), (256, 128), (256, 256)}
