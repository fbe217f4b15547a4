"""Shard shapes (M, Nn, K) that reach every variant of the linear layer's kernels:
each instantiated (batch-tile rows, workgroup columns) of the weight-streaming
kernel, with and without a K split, with one and with several batch tiles, the
decode kernel's (row blocks, wavefronts per K range) pairs and the tiled kernel;
all with ragged edges.  The CPU suite checks, through the
library's launch query, that every shape still lands on the variant named here
and that no instantiated variant is left out; the GPU suite runs them against the
oracle."""

# (M, Nn, K, tile_rows, tile_cols, split?, k_waves, tiled?)
# tiled kernel: 256 x 256, 256 x 192, 256 x 128, 128 x 192 or 128 x 128; decode kernel: rows = 16, k_waves = wavefronts sharing K
CASES = [
    (1, 208, 256, 32, 32, False, 1, False),
    (7, 208, 2048, 16, 16, False, 2, False),
    (1, 28680, 1088, 32, 128, False, 1, False),
    (16, 9000, 3072, 32, 128, True, 1, False),
    (65, 208, 256, 64, 32, False, 1, False),
    (65, 208, 2048, 64, 32, True, 1, False),
    (65, 4104, 256, 64, 64, False, 1, False),
    (65, 528, 4096, 64, 64, True, 1, False),
    (65, 9000, 1088, 64, 128, False, 1, False),
    (130, 2056, 4096, 64, 128, True, 1, False),
    (200, 9000, 512, 96, 128, False, 1, False),
    (130, 3080, 3072, 96, 128, True, 1, False),
    (777, 208, 4096, 128, 32, True, 1, False),
    (200, 7000, 256, 128, 64, False, 1, False),
    (200, 2056, 2048, 128, 64, True, 1, False),
    (300, 9000, 512, 128, 128, False, 1, False),
    (200, 4104, 3072, 128, 128, True, 1, False),
    (1000, 4000, 256, 128, 128, False, 1, True),
    (1000, 4104, 256, 128, 192, False, 1, True),
    (640, 8200, 320, 128, 192, False, 1, True),
    (130, 4104, 6144, 192, 128, True, 1, False),
    (200, 17008, 256, 256, 128, False, 1, False),
    (600, 5000, 320, 128, 128, False, 1, True),
    (777, 7000, 256, 256, 128, False, 1, True),
    (256, 28680, 320, 256, 128, False, 1, True),
    (200, 4104, 8320, 256, 128, True, 1, False),
    (520, 20008, 256, 256, 256, False, 1, True),
    (520, 11008, 256, 256, 192, False, 1, True),
    (1030, 8008, 320, 256, 192, False, 1, True),
    (3, 104, 1600, 16, 16, False, 2, False),
    (1, 184, 1600, 16, 16, False, 4, False),
    (3, 944, 8192, 16, 16, True, 2, False),
    (3, 904, 11904, 16, 16, True, 4, False),
    (3, 584, 2048, 16, 16, False, 2, False),
    (7, 2104, 3392, 16, 16, False, 4, False),
    (1, 904, 12352, 16, 16, True, 4, False),
    (17, 208, 2048, 32, 32, True, 1, False),
    (1, 4984, 3392, 16, 32, False, 4, False),
    (1, 1744, 16384, 16, 32, True, 4, False),
    (1, 104, 4096, 32, 32, True, 1, False),
    (1, 344, 3392, 16, 16, False, 4, False),
    (5, 1264, 3392, 16, 16, False, 4, False),
    (1, 224, 7424, 32, 32, True, 1, False),
    (3, 1384, 7424, 16, 16, True, 4, False),
]

# every (rows, cols, k_waves, tiled) the library instantiates
VARIANTS = {(16, 16, 2, False), (16, 16, 4, False), (16, 32, 4, False)} | {(r, c, 1, False) for r, c in {
    (32, 32), (32, 128), (64, 32), (64, 64), (64, 128), (96, 128), (128, 32), (128, 64), (128, 128), (192, 128),
    (256, 128)}} | {(256, 256, 1, True), (256, 192, 1, True), (256, 128, 1, True), (128, 192, 1, True), (128, 128, 1, True)}
