"""Pins of the shard-selecting linear layer's oracle."""
import numpy as np
import pytest

from oracle import shard_linear as osl
from workload import SplitMix64


def test_bf16_decoding_known_patterns():
    got = osl.bf16_to_f64(np.array([0x3F80, 0xC000, 0x3FC0, 0x0000, 0x8000, 0x4049, 0x0080, 0x7F80], np.uint16))
    assert got[:5].tolist() == [1.0, -2.0, 1.5, 0.0, -0.0]
    assert got[5] == 3.140625                                  # 0x4049 = pi truncated to bfloat16
    assert got[6] == 2.0 ** -126 and np.isinf(got[7])
    assert osl.f16_to_f64(np.array([0x3C00, 0xC000, 0x3555], np.uint16)).tolist()[:2] == [1.0, -2.0]


def test_first_half_and_first_quarter_for_rank_zero():
    """Sec. 3.2.1: under TP2 the first GPU of a group uses the first half of a
    weight matrix, under TP4 the first quarter."""
    assert osl.shard_bounds(4096, 2, 0) == (0, 2048)
    assert osl.shard_bounds(4096, 4, 0) == (0, 1024)
    assert osl.shard_bounds(4096, 4, 3) == (3072, 4096)
    with pytest.raises(ValueError):
        osl.shard_bounds(10, 4, 0)
    with pytest.raises(ValueError):
        osl.shard_bounds(8, 4, 4)


def test_hand_computed_example():
    X = np.array([[1.0, 2.0, 3.0, 4.0]])
    W = np.array([[1.0, 0.0, 0.0, 0.0],
                  [0.0, 1.0, 0.0, 0.0],
                  [1.0, 1.0, 1.0, 1.0],
                  [0.0, 0.0, 2.0, -1.0]])
    y, a = osl.shard_linear(X, W, 2, 1, "out")                 # rows 2..3 of W
    assert y.tolist() == [[10.0, 2.0]] and a.tolist() == [[10.0, 10.0]]
    y, _ = osl.shard_linear(X[:, 2:], W, 2, 1, "in")           # columns 2..3 of W, X's second half
    assert y.tolist() == [[0.0, 0.0, 7.0, 2.0]]
    y, _ = osl.shard_linear(X[:, :2], W, 2, 0, "in")
    assert y.tolist() == [[1.0, 2.0, 3.0, 0.0]]


@pytest.mark.parametrize("tp", [1, 2, 4, 8])
def test_shards_tile_the_full_product(tp):
    """Tensor-parallel identities against the product with the FULL matrix:
    output shards concatenate to it, input shards sum to it.  A shard that is
    shifted, overlapping or cut along the wrong axis breaks one of them."""
    rng = SplitMix64(50 + tp)
    M, n_out, n_in = 5, 24, 16
    X = np.round(rng.uniform(M * n_in).reshape(M, n_in) * 8 - 4)
    W = np.round(rng.uniform(n_out * n_in).reshape(n_out, n_in) * 8 - 4)
    full = np.zeros((M, n_out))
    for i in range(M):                                          # plain triple loop, no library call
        for j in range(n_out):
            full[i, j] = sum(X[i, k] * W[j, k] for k in range(n_in))
    cat = np.concatenate([osl.shard_linear(X, W, tp, r, "out")[0] for r in range(tp)], axis=1)
    assert np.array_equal(cat, full)
    per = n_in // tp
    tot = sum(osl.shard_linear(X[:, r * per:(r + 1) * per], W, tp, r, "in")[0] for r in range(tp))
    assert np.array_equal(tot, full)


def test_tolerance_covers_fp32_accumulation_in_any_order():
    rng = SplitMix64(3)
    k = 4096
    x = (rng.uniform(k) - 0.5)
    w = (rng.uniform(k) - 0.5)
    xb = osl.bf16_to_f64(((x.astype(np.float32).view(np.uint32)) >> 16).astype(np.uint16))
    wb = osl.bf16_to_f64(((w.astype(np.float32).view(np.uint32)) >> 16).astype(np.uint16))
    exact = float(np.dot(xb, wb))
    bound = float(np.dot(np.abs(xb), np.abs(wb)))
    tol = float(osl.tolerance(np.array(exact), np.array(bound), k))
    for order in (np.arange(k), np.arange(k)[::-1], rng.permutation(k)):
        acc = np.float32(0)
        for i in order:
            acc = np.float32(acc + np.float32(xb[i]) * np.float32(wb[i]))
        assert abs(float(acc) - exact) <= tol
    assert tol < 0.02 * bound                                   # and it is not vacuous
