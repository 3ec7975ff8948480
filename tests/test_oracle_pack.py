"""Pins of the pack / append oracle: hand-made cases, the identity selection, attention over the
packed cache against attention written directly on the dense cache, and the input generator."""
import numpy as np
import pytest

import workloads as W
from oracle import attention as OA
from oracle import pack as PK


def test_hand_made_pack_and_append():
    B, Hkv, T, D = 1, 2, 4, 2
    kd = np.arange(B * Hkv * T * D, dtype=np.uint16).reshape(B, Hkv, T, D)          # k_dense[0][h][t] = [8h+2t, 8h+2t+1]
    vd = kd + 100
    keep_ptr = np.array([0, 2, 5], np.int64)
    keep_t = np.array([3, 0, 1, 2, 3], np.int32)                                  # pair 0 keeps t=3 then t=0
    off = np.array([1, 4], np.int64)                                              # row 0 and row 3 belong to no pair
    k = np.full((8, D), 999, np.uint16)
    v = np.full((8, D), 999, np.uint16)
    PK.pack(kd, vd, keep_ptr, keep_t, off, k, v)
    assert k.tolist() == [[999, 999], [6, 7], [0, 1], [999, 999], [10, 11], [12, 13], [14, 15], [999, 999]]
    assert (v[[1, 2, 4, 5, 6]] == k[[1, 2, 4, 5, 6]] + 100).all() and (v[[0, 3, 7]] == 999).all()
    lens = np.array([2, 3], np.int32)
    cap = np.array([2, 4], np.int32)                                              # pair 0 is full
    kn = np.array([[[50, 51], [60, 61]]], np.uint16)
    full = PK.append(k, v, kn, kn + 1, off, lens, cap)
    assert full == 1 and lens.tolist() == [2, 4]
    assert k[7].tolist() == [60, 61] and v[7].tolist() == [61, 62] and k[3].tolist() == [999, 999]
    with pytest.raises(ValueError):
        PK.pack(kd, vd, keep_ptr, np.array([4, 0, 1, 2, 3], np.int32), off, k, v)


def test_keeping_everything_reproduces_the_dense_cache():
    rng = np.random.default_rng(0)
    B, Hkv, T, D = 2, 3, 7, 4
    kd = rng.integers(0, 60000, size=(B, Hkv, T, D)).astype(np.uint16)
    vd = rng.integers(0, 60000, size=(B, Hkv, T, D)).astype(np.uint16)
    keep_ptr = np.arange(B * Hkv + 1, dtype=np.int64) * T
    keep_t = np.tile(np.arange(T, dtype=np.int32), B * Hkv)
    k = np.zeros((B * Hkv * T, D), np.uint16)
    v = np.zeros_like(k)
    PK.pack(kd, vd, keep_ptr, keep_t, keep_ptr[:-1], k, v)
    assert (k == kd.reshape(-1, D)).all() and (v == vd.reshape(-1, D)).all()


def test_attention_over_the_packed_cache_is_attention_over_the_kept_tokens():
    rng = np.random.default_rng(1)
    B, Hkv, G, T, D = 2, 2, 2, 40, 8
    lens = rng.integers(0, 30, size=(B, Hkv)).astype(np.int32)
    keep_ptr, keep_t = W.keep_lists(lens, T, seed=3, recent=4)
    kd, vd = rng.normal(size=(B, Hkv, T, D)), rng.normal(size=(B, Hkv, T, D))
    q = rng.normal(size=(B, Hkv * G, D))
    off, total = W.packed_offsets(lens, gap_rows=2)
    k, v = np.zeros((total, D)), np.zeros((total, D))
    PK.pack(kd, vd, keep_ptr, keep_t, off.reshape(-1), k, v)
    out, lse = OA.attention(q.astype(np.float32), k.astype(np.float32), v.astype(np.float32), off, lens, 0.3)
    kd32, vd32 = kd.astype(np.float32).astype(np.float64), vd.astype(np.float32).astype(np.float64)
    q32 = q.astype(np.float32).astype(np.float64)
    for b in range(B):
        for hq in range(Hkv * G):
            h = hq // G
            p = b * Hkv + h
            mask = np.zeros(T, bool)
            mask[keep_t[keep_ptr[p]:keep_ptr[p + 1]]] = True
            if not mask.any():
                assert (out[b, hq] == 0).all()
                continue
            s = (kd32[b, h] @ q32[b, hq]) * 0.3
            wgt = np.where(mask, np.exp(s - s[mask].max()), 0.0)
            ref = (wgt[:, None] * vd32[b, h]).sum(0) / wgt.sum()
            assert np.abs(out[b, hq] - ref).max() < 1e-12


def test_keep_lists_have_the_stated_structure():
    lens = np.array([[0, 5, 40], [64, 33, 1]], np.int32)
    keep_ptr, keep_t = W.keep_lists(lens, 64, seed=1, recent=32)
    assert keep_ptr.tolist() == [0, 0, 5, 45, 109, 142, 143] and keep_t.dtype == np.int32
    for p, n in enumerate(lens.reshape(-1)):
        t = keep_t[keep_ptr[p]:keep_ptr[p + 1]]
        assert len(set(t.tolist())) == n and (np.diff(t) > 0).all() and (t >= 0).all() and (t < 64).all()
        tail = min(n, 32)
        assert t[n - tail:].tolist() == list(range(64 - tail, 64))
    a = W.keep_lists(lens, 64, seed=1)[1]
    assert (a == keep_t).all() and (W.keep_lists(lens, 64, seed=2)[1] != keep_t).any()
    with pytest.raises(ValueError):
        W.keep_lists(np.array([[65]]), 64)
