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


def test_tolerance_hand_value_and_what_it_rejects():
    """The worst-case bound on a case small enough for mental arithmetic: y = 1, sum |x w| = 2, k = 256,
    bfloat16 output.  fp32 accumulation: 256 * 2^-23 * 2 = 2^-14; rounding: 2^-8 of (1 + 2^-14);
    together 2^-8 + 2^-14 + 2^-22.  At a short reduction it is therefore tight enough that an error of
    two output ulps (2 * 2^-7 for y = 1) fails, while half an ulp passes."""
    tol = float(osl.tolerance(np.array(1.0), np.array(2.0), 256))
    assert tol == 2.0 ** -8 + 2.0 ** -14 + 2.0 ** -22
    assert 0.5 * 2.0 ** -7 <= tol < 2 * 2.0 ** -7
    # float16 keeps three more bits: the rounding term shrinks by 8, the accumulation term stays
    assert float(osl.tolerance(np.array(1.0), np.array(2.0), 256, out_bits=11)) == 2.0 ** -11 + 2.0 ** -14 + 2.0 ** -25
    with pytest.raises(ValueError):
        osl.shard_bounds(16, 0, 0)


def test_round_to_bits_hand_values_and_ties_to_even():
    """bfloat16 keeps 8 significant bits: integers in [256, 512) are 2 apart, so
    257 and 259 are exact ties; float16 keeps 11: integers in [2048, 4096)."""
    got = osl.round_to_bits(np.array([1.0, 257.0, 258.0, 259.0, -0.0, 1e40, 65520.0, 1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8]), "bf16")
    assert got.tolist() == [0x3F80, 0x4380, 0x4381, 0x4382, 0x8000, 0x7F80, 0x4780, 0x3F80, 0x3F82]
    got = osl.round_to_bits(np.array([1.0, 2049.0, 2051.0, 65519.0, 65520.0, 2.0 ** -25, 3 * 2.0 ** -25, -2.0 ** -14]), "f16")
    assert got.tolist() == [0x3C00, 0x6800, 0x6802, 0x7BFF, 0x7C00, 0x0000, 0x0002, 0x8400]


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_round_to_bits_is_the_nearest_value_on_every_interval(fmt):
    """Every finite value of the format rounds to itself; every midpoint between
    two neighbours rounds to the one with the even pattern; points a quarter of
    the way round to the nearer neighbour.  (Exhaustive over all positive patterns.)"""
    decode = osl.bf16_to_f64 if fmt == "bf16" else osl.f16_to_f64
    top = 0x7F80 if fmt == "bf16" else 0x7C00                 # pattern of +infinity
    pats = np.arange(0, top, dtype=np.uint16)
    vals = decode(pats)
    assert np.array_equal(osl.round_to_bits(vals, fmt), pats)
    assert np.array_equal(osl.round_to_bits(-vals, fmt), pats | np.uint16(0x8000))
    lo, hi = vals[:-1], vals[1:]
    mid = (lo + hi) / 2                                         # exact in float64
    even = np.where(pats[:-1] % 2 == 0, pats[:-1], pats[1:])
    assert np.array_equal(osl.round_to_bits(mid, fmt), even)
    assert np.array_equal(osl.round_to_bits(lo + (hi - lo) / 4, fmt), pats[:-1])
    assert np.array_equal(osl.round_to_bits(lo + 3 * (hi - lo) / 4, fmt), pats[1:])
    assert np.array_equal(osl.ulp(lo, fmt), hi - lo)


def test_round_to_bits_agrees_with_library_conversions():
    """float16: NumPy's own float64 -> float16 conversion.  bfloat16: the input
    generator's float32 -> bfloat16 routine (separate code) on float32 values."""
    from workload.linear import f32_to_bf16_bits
    rng = SplitMix64(8)
    y = (rng.uniform(200000) - 0.5) * np.exp((rng.uniform(200000) - 0.5) * 40)
    with np.errstate(over="ignore"):
        assert np.array_equal(osl.round_to_bits(y, "f16"), y.astype(np.float16).view(np.uint16))
    y32 = y.astype(np.float32)
    assert np.array_equal(osl.round_to_bits(y32.astype(np.float64), "bf16"), f32_to_bf16_bits(y32))


@pytest.mark.parametrize("k", [256, 4096, 14336])
@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_tight_tolerance_admits_fp32_accumulation_and_rejects_a_dropped_product(k, fmt):
    """fp32 accumulation simulated on the CPU in three orders (forward, backward,
    64-wide slabs whose partial sums are then added), rounded once: always
    inside the tight tolerance.  The same sums with ONE product left out, or with
    a 64-wide slab left out: outside it for nearly every output, while the
    worst-case tolerance lets most of them pass at long reductions (a dropped
    product from 4096 terms on, a dropped slab at 14336)."""
    from workload.linear import linear_inputs
    n = 200
    Xh, Wh = linear_inputs(21 + k, 1, n, k, dtype=fmt)
    decode = osl.bf16_to_f64 if fmt == "bf16" else osl.f16_to_f64
    X, W = decode(Xh), decode(Wh)
    want, bound = osl.shard_linear(X, W, 1, 0, "out")
    norm = osl.product_norm(X, W, 1, 0, "out")
    tight = osl.tight_tolerance(want, norm, k, fmt)
    loose = osl.tolerance(want, bound, k, out_bits=8 if fmt == "bf16" else 11)
    assert np.all(tight < loose)
    prod = (X.astype(np.float32) * W.astype(np.float32))          # [n][k], each product exact in fp32
    assert np.array_equal(prod.astype(np.float64), X * W)

    def rounded(sums32):
        return decode(osl.round_to_bits(sums32.astype(np.float64), fmt))

    orders = [np.cumsum(prod, axis=1, dtype=np.float32)[:, -1],
              np.cumsum(prod[:, ::-1], axis=1, dtype=np.float32)[:, -1],
              np.cumsum(np.cumsum(prod.reshape(n, k // 64, 64), axis=2, dtype=np.float32)[:, :, -1], axis=1,
                        dtype=np.float32)[:, -1]]
    for s32 in orders:
        assert np.all(np.abs(rounded(s32) - want[0]) <= tight[0])
    i = int(np.argmin(np.abs(np.abs(X[0]) - 1.0)))                               # an activation of typical size
    one_less = np.cumsum(np.delete(prod, i, axis=1), axis=1, dtype=np.float32)[:, -1]   # product i dropped
    slab_less = np.cumsum(prod[:, 64:], axis=1, dtype=np.float32)[:, -1]        # slab 0 dropped
    big = np.abs(prod[:, i]) > 0.5 * np.abs(prod).mean()                         # outputs whose dropped product is of typical size
    assert big.sum() > n // 3
    caught_one = np.abs(rounded(one_less) - want[0]) > tight[0]
    caught_slab = np.abs(rounded(slab_less) - want[0]) > tight[0]
    assert caught_one[big].mean() > 0.9 and caught_slab.mean() > 0.95
    if k >= 4096:                                   # the worst-case bound alone lets these mistakes through
        assert (np.abs(rounded(one_less) - want[0]) > loose[0])[big].mean() < 0.5
    if k == 14336:
        assert (np.abs(rounded(slab_less) - want[0]) > loose[0]).mean() < 0.5


@pytest.mark.parametrize("fmt", ["bf16", "f16"])
def test_integer_inputs_are_exact_small_integers(fmt):
    from workload.linear import linear_inputs_int
    Xh, Wh = linear_inputs_int(4, 3, 40, 128, dtype=fmt)
    decode = osl.bf16_to_f64 if fmt == "bf16" else osl.f16_to_f64
    for a in (decode(Xh), decode(Wh)):
        assert np.array_equal(a, np.rint(a)) and np.abs(a).max() == 8 and len(np.unique(a)) == 17
    y, _ = osl.shard_linear(decode(Xh), decode(Wh), 1, 0, "out")
    assert np.array_equal(y, np.rint(y))                        # so the exact result is an integer
