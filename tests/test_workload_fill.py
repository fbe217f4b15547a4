"""The host C twin of the stateless pool fill equals the NumPy definition, and
the layer-by-layer comparer the large GPU configurations rely on really looks
at every byte (a wrong byte planted on the CPU, anywhere, is reported)."""
import numpy as np
import pytest

from workload import fill_words, fill_words_fast, make_case


@pytest.mark.parametrize("seed,start,count", [(0, 0, 1000), (5, 12345678901, 4097), (2 ** 63 + 5, 2 ** 40, 10), (7, 3, 0)])
def test_c_fill_equals_numpy_fill(seed, start, count):
    assert np.array_equal(fill_words(seed, start, count), fill_words_fast(seed, start, count))
    out = np.empty(count, dtype="<u8")
    assert fill_words_fast(seed, start, count, out) is out
    with pytest.raises(ValueError):
        fill_words_fast(seed, start, count + 1, out)


def test_layer_comparer_accepts_the_oracle_result_and_finds_one_wrong_byte():
    import torch
    from gpu_util import compare_every_layer, host_layers, oracle_slots
    from oracle import kvmig as orc
    case = make_case("c1")[1]
    sh = case.shape
    es, ed = oracle_slots(case)
    so, do, w = orc.route(sh.H, case.Ns, case.rs, case.Nd, case.rd)
    want = host_layers(case, "dst", range(sh.L)).copy()
    orc.migrate(host_layers(case, "src", range(sh.L)), want, es, ed, so, do, w)
    pool = torch.from_numpy(want.view(np.uint8).reshape(-1).copy())
    assert compare_every_layer(case, pool, es, ed, workers=3) > 0
    assert compare_every_layer(case, pool, es, ed, workers=2, direct=True) > 0
    layer_bytes = pool.numel() // sh.L
    for pos in (0, 5 * layer_bytes + 12345, pool.numel() - 1):
        pool[pos] ^= 0x40
        with pytest.raises(AssertionError) as ei:
            compare_every_layer(case, pool, es, ed, workers=3)
        assert str(pos // layer_bytes) in str(ei.value)
        pool[pos] ^= 0x40
    compare_every_layer(case, pool, es, ed, workers=3)
