"""The synthetic input generator: shapes, padding layout, determinism, skew."""
import numpy as np
import pytest

from paper_2204_04179_amd import workloads as wl


@pytest.mark.parametrize("name", ["tiny", "kt", "news", "kt_multi", "stress"])
def test_ids_shape_range_and_determinism(name):
    w = wl.get(name)
    a = wl.ids(w)
    assert a.shape == (w.B, w.L) and a.dtype == np.int32
    assert a.min() >= 0 and a.max() < w.N
    np.testing.assert_array_equal(a, wl.ids(w))
    if w.K > 1:
        assert np.any(a != wl.ids(w, step=1))
    if w.padding is None:
        assert np.all(a != 0)


def test_padding_layouts():
    t = wl.ids(wl.get("tiny"))
    assert np.all(t[:, -3:] == 0) and np.all(t[:, :-3] != 0)
    k = wl.ids(wl.get("kt"))
    lens = (k != 0).sum(1)
    assert lens.min() >= 20 and lens.max() <= 100
    for row, n in zip(k, lens):           # padding is a suffix
        assert np.all(row[:n] != 0) and np.all(row[n:] == 0)


def test_zipf_skew_and_boost_ratio_band():
    # batch-level interactions / unique items lands in the paper's ~4x regime
    for name, lo, hi in (("kt", 2.0, 3.2), ("news", 3.5, 5.5), ("kt_multi", 3.5, 5.5), ("stress", 3.0, 4.6)):
        a = wl.ids(wl.get(name)).ravel()
        v = a[a != 0]
        r = v.size / np.unique(v).size
        assert lo < r < hi, (name, r)
    w = wl.get("stress")
    c = np.bincount(wl.ids(w).ravel(), minlength=w.N)
    assert c[wl.rank_to_id(w)[0]] == c.max()       # rank 1 is the most frequent item


def test_tensor_draws():
    w = wl.get("tiny")
    X, W, dH = wl.features(w), wl.weights(w), wl.upstream_grad(w)
    assert X.shape == (100, 64) and X.dtype == np.float32
    assert W.shape == (64, 32) and abs(W.std() - 1 / 8) < 0.02
    assert dH.shape == (64, 32) and dH.dtype == np.float32
    w = wl.get("kt")
    W = wl.weights(w)
    assert W.dtype == np.uint16 and W.shape == (768, 256)
    assert abs(wl.bf16_bits_to_f32(W).std() - 768 ** -0.5) < 2e-3


def test_bf16_rounding_is_nearest_even():
    f = np.array([1.0, 1.00390625, 1.01171875, -2.5, 3.0e38, 1.0 + 2 ** -8 + 2 ** -20], np.float32)
    b = wl.f32_to_bf16_bits(f)
    back = wl.bf16_bits_to_f32(b)
    # 1 + 2^-8 is a tie between 1 and 1 + 2^-7 -> even mantissa (1.0);
    # 1 + 3*2^-8 is a tie between 1+2^-7 and 1+2^-6 -> even (1+2^-6)
    assert back[0] == 1.0 and back[1] == 1.0 and back[2] == 1.015625 and back[3] == -2.5
    assert back[5] == 1.0078125
    assert np.all(np.abs(back[:4] - f[:4]) <= np.abs(f[:4]) * 2 ** -8)
