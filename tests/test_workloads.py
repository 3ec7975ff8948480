"""The synthetic input recipes: reproducible, and shaped as stated."""
import numpy as np

import workloads as W


def test_lens_are_reproducible_and_layer_dependent():
    for name, w in W.WORKLOADS.items():
        a, b = W.lens(name, seed=0, layer=3), W.lens(name, seed=0, layer=3)
        assert a.dtype == np.int32 and a.shape == (w.B, w.Hkv) and np.array_equal(a, b)
        assert not np.array_equal(a, W.lens(name, seed=0, layer=4))
        assert not np.array_equal(a, W.lens(name, seed=1, layer=3))


def test_tiny_matches_its_recorded_draw():
    # guards the generator itself (a change here silently changes every workload)
    assert W.lens("tiny").tolist() == [[82, 76, 96, 128], [49, 7, 63, 20]]


def test_shapes_of_the_distributions():
    l2 = np.concatenate([W.lens("llama70b", layer=i).ravel() for i in range(32)])
    assert l2.min() >= 16 and l2.max() <= 8192 and 950 < l2.mean() < 1100
    ratios = [W.lens("llama70b", layer=i).max() / W.lens("llama70b", layer=i).min() for i in range(32)]
    assert 12 < np.median(ratios) < 35                     # "max/min ratio ~20x"
    l3 = W.lens("mistral24b")
    heavy, light = l3[:, [2, 5]].mean(), np.delete(l3, [2, 5], axis=1).mean()
    assert 6 < heavy / light < 11 and l3.max() <= 16384
    l4 = W.lens("faircopy")
    assert np.all(l4[:32, 1] == 0) and np.all(l4[32:, 1] > 0) and np.all(l4[:, 0] > 0)
    l5 = np.concatenate([W.lens("stress", layer=i).ravel() for i in range(80)])
    assert l5.min() == 32 and l5.max() == 32768 and 130 < l5.mean() < 175   # E[len] = 152
    top = np.sort(W.lens("stress").ravel())[::-1]
    assert top[:32].sum() > 0.25 * top.sum()               # a few heads carry much of a layer


def test_offsets_pack_densely_in_pair_order():
    lens = np.array([[3, 0], [5, 2]], np.int32)
    off, total = W.packed_offsets(lens)
    assert off.tolist() == [[0, 3], [3, 8]] and total == 10
    off, total = W.packed_offsets(lens, gap_rows=2)
    assert off.tolist() == [[0, 5], [7, 14]] and total == 18


def test_qkv_bits_are_reproducible():
    w = W.WORKLOADS["llama70b"]
    q1, k1, v1 = W.make_qkv(w, 100, seed=0, layer=1)
    q2, k2, v2 = W.make_qkv(w, 100, seed=0, layer=1)
    assert q1.shape == (16, 64, 128) and k1.shape == (100, 128)
    assert (q1 == q2).all() and (k1 == k2).all() and (v1 == v2).all()
    assert W.to_numpy_bits(k1).dtype == np.uint16
    assert W.algorithmic_bytes(w, np.array([[10]])) == 2 * 10 * 128 * 2 + 16 * 64 * 128 * (2 + 4)
