"""Pins of the fp64 attention oracle against things other than itself.

The paper prints no worked numeric example of attention, so the pins are closed
forms, invariants, brute force on tiny inputs, and a library routine on the
special case that reduces to dense attention.  Each test is chosen so that a
plausible slip in the oracle (a dropped scale, a wrong head-group index, a
transposed operand, a missing max subtraction, an off-by-one in the row range)
makes it fail.
"""
import math

import numpy as np
import pytest

import workloads as W
from oracle import attention as OA


def bf16_bits(x):
    """float32 array -> bf16 bit patterns (round to nearest even), as uint16."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return r.astype(np.uint16)


def bf16_to_f64(bits):
    return (bits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def brute(q, k, v, off, lens, scale):
    """Independent dense-numpy evaluation, one (b, hq) at a time."""
    B, Hq, D = q.shape
    Hkv = lens.shape[1]
    G = Hq // Hkv
    out = np.zeros((B, Hq, D))
    lse = np.full((B, Hq), -np.inf)
    for b in range(B):
        for hq in range(Hq):
            h = hq // G
            n = int(lens[b, h])
            if n == 0:
                continue
            Kb = k[off[b, h]: off[b, h] + n]
            Vb = v[off[b, h]: off[b, h] + n]
            s = (Kb @ q[b, hq]) * scale
            w = np.exp(s - s.max())
            out[b, hq] = (w[:, None] * Vb).sum(0) / w.sum()
            lse[b, hq] = s.max() + np.log(w.sum())
    return out, lse


def rand_case(rng, B, Hq, Hkv, D, max_len, min_len=0):
    lens = rng.integers(min_len, max_len + 1, size=(B, Hkv)).astype(np.int32)
    off, total = W.packed_offsets(lens, gap_rows=1)
    q = rng.standard_normal((B, Hq, D))
    k = rng.standard_normal((max(total, 1), D))
    v = rng.standard_normal((max(total, 1), D))
    return q, k, v, off, lens


def test_brute_force_tiny_shapes():
    rng = np.random.default_rng(1)
    for _ in range(40):
        Hkv = int(rng.integers(1, 4))
        G = int(rng.integers(1, 4))
        D = int(rng.integers(1, 5))
        B = int(rng.integers(1, 3))
        q, k, v, off, lens = rand_case(rng, B, Hkv * G, Hkv, D, 8)
        scale = float(rng.uniform(0.1, 2.0))
        o, l = OA.attention(q, k, v, off, lens, scale)
        ro, rl = brute(q, k, v, off, lens, scale)
        assert np.allclose(o, ro, rtol=0, atol=1e-12)
        assert np.array_equal(np.isinf(l), np.isinf(rl))
        fin = np.isfinite(rl)
        assert np.allclose(l[fin], rl[fin], rtol=0, atol=1e-12)


def test_brute_force_tiny_workload_f32_and_bf16():
    w = W.WORKLOADS["tiny"]
    lens = W.lens("tiny", seed=0)
    off, total = W.packed_offsets(lens)
    q, k, v = W.make_qkv(w, total, seed=0)
    qn, kn, vn = (W.to_numpy_bits(t) for t in (q, k, v))
    assert qn.dtype == np.float32
    o, l = OA.attention(qn, kn, vn, off, lens, w.scale)
    ro, rl = brute(qn.astype(np.float64), kn.astype(np.float64), vn.astype(np.float64), off, lens, w.scale)
    assert np.abs(o - ro).max() < 1e-12 and np.abs(l - rl).max() < 1e-12
    # same data rounded to bf16: the oracle must widen the 16-bit patterns exactly
    qb, kb, vb = bf16_bits(qn), bf16_bits(kn), bf16_bits(vn)
    o2, l2 = OA.attention(qb, kb, vb, off, lens, w.scale)
    ro2, rl2 = brute(bf16_to_f64(qb), bf16_to_f64(kb), bf16_to_f64(vb), off, lens, w.scale)
    assert np.abs(o2 - ro2).max() < 1e-12 and np.abs(l2 - rl2).max() < 1e-12
    assert np.abs(o2 - o).max() > 1e-6   # bf16 rounding is visible, so the path was exercised


def test_equal_lengths_reduce_to_library_sdpa():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(2)
    B, Hkv, G, D, L = 3, 2, 4, 16, 37
    lens = np.full((B, Hkv), L, dtype=np.int32)
    off, total = W.packed_offsets(lens)
    q = rng.standard_normal((B, Hkv * G, D))
    k = rng.standard_normal((total, D))
    v = rng.standard_normal((total, D))
    scale = 0.3
    o, _ = OA.attention(q, k, v, off, lens, scale)
    kt = torch.from_numpy(k).reshape(B, Hkv, L, D).repeat_interleave(G, dim=1)
    vt = torch.from_numpy(v).reshape(B, Hkv, L, D).repeat_interleave(G, dim=1)
    qt = torch.from_numpy(q).reshape(B, Hkv * G, 1, D)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, scale=scale)
    assert np.abs(ref.reshape(B, Hkv * G, D).numpy() - o).max() < 1e-10


def test_rational_closed_form():
    # q = e_0, K_t = (ln a_t / scale) e_0  =>  s_t = ln a_t, weights a_t / sum a.
    a = np.array([1.0, 3.0, 4.0, 8.0])
    scale = 0.5
    D = 3
    k = np.zeros((4, D))
    k[:, 0] = np.log(a) / scale
    v = np.array([[16.0, 0.0, -16.0], [0.0, 16.0, 16.0], [32.0, -16.0, 0.0], [-8.0, 8.0, 4.0]])
    q = np.zeros((1, 1, D))
    q[0, 0, 0] = 1.0
    o, l = OA.attention(q, k, v, np.zeros((1, 1), np.int64), np.array([[4]], np.int32), scale)
    want = np.array([16 * 1 + 0 * 3 + 32 * 4 - 8 * 8, 0 + 16 * 3 - 16 * 4 + 8 * 8, -16 + 16 * 3 + 0 + 4 * 8]) / 16.0
    assert np.allclose(o[0, 0], want, atol=1e-13)
    assert abs(l[0, 0] - math.log(16.0)) < 1e-13


def test_length_one_returns_that_value_row_exactly():
    rng = np.random.default_rng(3)
    B, Hkv, G, D = 2, 3, 2, 8
    lens = np.ones((B, Hkv), dtype=np.int32)
    off, total = W.packed_offsets(lens, gap_rows=2)
    q = rng.standard_normal((B, Hkv * G, D)).astype(np.float32)
    k = rng.standard_normal((total, D)).astype(np.float32)
    v = rng.standard_normal((total, D)).astype(np.float32)
    o, l = OA.attention(q, k, v, off, lens, 0.7)
    for b in range(B):
        for hq in range(Hkv * G):
            r = off[b, hq // G]
            assert np.array_equal(o[b, hq], v[r].astype(np.float64))
            s0 = 0.7 * float(q[b, hq].astype(np.float64) @ k[r].astype(np.float64))
            assert abs(l[b, hq] - s0) < 1e-13


def test_zero_query_gives_mean_of_values():
    rng = np.random.default_rng(4)
    q, k, v, off, lens = rand_case(rng, 2, 4, 2, 6, 20, min_len=1)
    q[:] = 0.0
    o, l = OA.attention(q, k, v, off, lens, 1.0)
    for b in range(2):
        for hq in range(4):
            h = hq // 2
            n = lens[b, h]
            assert np.allclose(o[b, hq], v[off[b, h]: off[b, h] + n].mean(0), atol=1e-13)
            assert abs(l[b, hq] - math.log(n)) < 1e-13


def test_empty_head_is_zero_with_minus_inf_lse():
    rng = np.random.default_rng(5)
    q, k, v, off, lens = rand_case(rng, 2, 4, 2, 4, 5, min_len=1)
    lens[1, 0] = 0
    o, l = OA.attention(q, k, v, off, lens, 1.0)
    assert np.all(o[1, 0:2] == 0.0) and np.all(np.isneginf(l[1, 0:2]))
    assert np.all(np.isfinite(l[1, 2:4])) and np.all(np.isfinite(l[0]))


def test_output_inside_value_range_per_coordinate():
    rng = np.random.default_rng(6)
    q, k, v, off, lens = rand_case(rng, 3, 6, 3, 5, 30, min_len=1)
    o, _ = OA.attention(q, k, v, off, lens, 0.9)
    for b in range(3):
        for hq in range(6):
            h = hq // 2
            Vb = v[off[b, h]: off[b, h] + lens[b, h]]
            assert np.all(o[b, hq] >= Vb.min(0) - 1e-12) and np.all(o[b, hq] <= Vb.max(0) + 1e-12)


def test_weights_sum_to_one_via_constant_value_column():
    # a V column that is constant c must come out as exactly c (up to rounding): sum w / l = 1
    rng = np.random.default_rng(7)
    q, k, v, off, lens = rand_case(rng, 2, 4, 2, 4, 50, min_len=1)
    v[:, 2] = 3.25
    o, _ = OA.attention(q, k, v, off, lens, 1.3)
    assert np.abs(o[:, :, 2] - 3.25).max() < 1e-14


def test_token_permutation_and_duplication():
    rng = np.random.default_rng(8)
    B, Hq, Hkv, D = 1, 2, 1, 5
    n = 17
    q = rng.standard_normal((B, Hq, D))
    k = rng.standard_normal((n, D))
    v = rng.standard_normal((n, D))
    off = np.zeros((1, 1), np.int64)
    o, l = OA.attention(q, k, v, off, np.array([[n]], np.int32), 0.8)
    perm = rng.permutation(n)
    o2, l2 = OA.attention(q, k[perm], v[perm], off, np.array([[n]], np.int32), 0.8)
    assert np.abs(o - o2).max() < 1e-13 and np.abs(l - l2).max() < 1e-13
    k3, v3 = np.repeat(k, 2, axis=0), np.repeat(v, 2, axis=0)
    o3, l3 = OA.attention(q, k3, v3, off, np.array([[2 * n]], np.int32), 0.8)
    assert np.abs(o - o3).max() < 1e-13 and np.abs(l3 - l - math.log(2.0)).max() < 1e-13


def test_score_shift_leaves_output_and_moves_lse():
    rng = np.random.default_rng(9)
    D, n, scale, c = 6, 23, 0.6, 40.0
    q = rng.standard_normal((1, 1, D))
    k = rng.standard_normal((n, D))
    v = rng.standard_normal((n, D))
    off = np.zeros((1, 1), np.int64)
    ln = np.array([[n]], np.int32)
    o, l = OA.attention(q, k, v, off, ln, scale)
    k2 = k + c * q[0, 0] / (scale * float(q[0, 0] @ q[0, 0]))
    o2, l2 = OA.attention(q, k2, v, off, ln, scale)
    assert np.abs(o - o2).max() < 1e-11 and abs(l2[0, 0] - l[0, 0] - c) < 1e-11


def test_dominant_token_and_no_overflow():
    rng = np.random.default_rng(10)
    D, n = 4, 9
    q = rng.standard_normal((1, 1, D))
    k = rng.standard_normal((n, D)) * 0.01
    v = rng.standard_normal((n, D))
    k[5] = 400.0 * q[0, 0] / float(q[0, 0] @ q[0, 0])      # score +400
    k[2] = -400.0 * q[0, 0] / float(q[0, 0] @ q[0, 0])     # score -400
    o, l = OA.attention(q, k, v, np.zeros((1, 1), np.int64), np.array([[n]], np.int32), 1.0)
    assert np.all(np.isfinite(o)) and np.isfinite(l[0, 0])
    assert np.allclose(o[0, 0], v[5], rtol=0, atol=1e-15)
    assert abs(l[0, 0] - 400.0) < 1e-12


def test_gqa_group_mapping():
    rng = np.random.default_rng(11)
    B, Hkv, G, D = 1, 3, 4, 4
    q, k, v, off, lens = rand_case(rng, B, Hkv * G, Hkv, D, 12, min_len=2)
    q[0, 5] = q[0, 6]                     # heads 5 and 6 are in group 1: same KV, same q
    q[0, 3] = q[0, 4]                     # heads 3 (group 0) and 4 (group 1): same q, other KV
    o, _ = OA.attention(q, k, v, off, lens, 1.0)
    assert np.array_equal(o[0, 5], o[0, 6])
    assert np.abs(o[0, 3] - o[0, 4]).max() > 1e-6
    # head hq must read KV head hq // G: compare against a single-head call on that slice
    for hq in range(Hkv * G):
        h = hq // G
        sl = slice(off[0, h], off[0, h] + lens[0, h])
        o1, _ = OA.attention(q[:, hq:hq + 1], k[sl], v[sl], np.zeros((1, 1), np.int64),
                             np.array([[lens[0, h]]], np.int32), 1.0)
        assert np.abs(o1[0, 0] - o[0, hq]).max() < 1e-13


def test_row_range_is_exact_neighbours_do_not_leak():
    rng = np.random.default_rng(12)
    q, k, v, off, lens = rand_case(rng, 2, 2, 2, 3, 9, min_len=1)
    o, l = OA.attention(q, k, v, off, lens, 1.0)
    # poison every row that no head owns; results must not move
    owned = np.zeros(k.shape[0], bool)
    for b in range(2):
        for h in range(2):
            owned[off[b, h]: off[b, h] + lens[b, h]] = True
    k2, v2 = k.copy(), v.copy()
    k2[~owned] = 1e6
    v2[~owned] = -1e6
    o2, l2 = OA.attention(q, k2, v2, off, lens, 1.0)
    assert np.array_equal(o, o2) and np.array_equal(l, l2)
    # growing one head by one row must change only that head's outputs
    lens3 = lens.copy()
    lens3[0, 0] += 1          # the gap row after head (0,0) becomes part of it
    o3, _ = OA.attention(q, k, v, off, lens3, 1.0)
    assert np.abs(o3[0, 0] - o[0, 0]).max() > 0
    assert np.array_equal(o3[0, 1], o[0, 1]) and np.array_equal(o3[1], o[1])


def test_chunked_and_merged_equals_unchunked():
    rng = np.random.default_rng(13)
    for _ in range(20):
        D = int(rng.integers(1, 9))
        n = int(rng.integers(1, 60))
        q = rng.standard_normal((1, 2, D)) * 3.0
        k = rng.standard_normal((n + 4, D))
        v = rng.standard_normal((n + 4, D))
        off = np.array([[2]], np.int64)
        o, l = OA.attention(q, k, v, off, np.array([[n]], np.int32), 0.9)
        cuts = np.sort(rng.integers(0, n + 1, size=int(rng.integers(0, 5))))
        edges = [0, *cuts.tolist(), n]
        for hq in range(2):
            parts = [OA.attention_chunk(q, k, v, 0, hq, 2 + a, b - a, 0.9) for a, b in zip(edges[:-1], edges[1:])]
            mo, ml = OA.merge_chunks(parts)
            assert np.abs(mo - o[0, hq]).max() < 1e-12 and abs(ml - l[0, hq]) < 1e-12


def test_selection_computes_only_listed_outputs():
    rng = np.random.default_rng(14)
    q, k, v, off, lens = rand_case(rng, 2, 4, 2, 3, 9, min_len=1)
    o, l = OA.attention(q, k, v, off, lens, 1.0)
    sel = np.array([5, 0, 6], np.int32)
    o2, l2 = OA.attention(q, k, v, off, lens, 1.0, sel=sel)
    flat, flat2 = o.reshape(8, -1), o2.reshape(8, -1)
    assert np.array_equal(flat[sel], flat2[sel]) and np.array_equal(l.reshape(-1)[sel], l2.reshape(-1)[sel])
    rest = np.setdiff1d(np.arange(8), sel)
    assert np.all(np.isnan(flat2[rest]))


def test_rejects_rows_past_the_buffer():
    q = np.zeros((1, 1, 2))
    k = np.zeros((3, 2))
    with pytest.raises(ValueError):
        OA.attention(q, k, k, np.array([[2]], np.int64), np.array([[2]], np.int32), 1.0)


# ---- several new tokens per sequence --------------------------------------------------------
def test_multi_token_queries_are_single_token_queries_over_shorter_caches():
    """New token i of q_len sees everything but the new tokens after it: the same as the single-token
    oracle (pinned above) run with every length reduced by q_len-1-i."""
    rng = np.random.default_rng(21)
    B, Hkv, G, D, QL = 3, 2, 2, 8, 3
    lens = rng.integers(0, 25, size=(B, Hkv)).astype(np.int32)
    lens[0, 0], lens[1, 1] = 1, 2                      # shorter than q_len: early tokens see nothing
    off = np.arange(B * Hkv, dtype=np.int64).reshape(B, Hkv) * 30
    k = rng.normal(size=(B * Hkv * 30, D))
    v = rng.normal(size=(B * Hkv * 30, D))
    q = rng.normal(size=(B, QL, Hkv * G, D))
    out, lse = OA.attention_multi(q, k, v, off, lens, 0.4)
    assert out.shape == (B, QL, Hkv * G, D) and lse.shape == (B, QL, Hkv * G)
    for i in range(QL):
        ro, rl = OA.attention(np.ascontiguousarray(q[:, i]), k, v, off, np.maximum(lens - (QL - 1 - i), 0), 0.4)
        assert np.array_equal(out[:, i], ro) and np.array_equal(lse[:, i], rl)
    assert (out[0, 0, 0:G] == 0).all() and np.isneginf(lse[0, 0, 0:G]).all()     # len 1, first of 3 new tokens
    o1, l1 = OA.attention_multi(np.ascontiguousarray(q[:, :1]), k, v, off, lens, 0.4)
    ro, rl = OA.attention(np.ascontiguousarray(q[:, 0]), k, v, off, lens, 0.4)
    assert np.array_equal(o1[:, 0], ro) and np.array_equal(l1[:, 0], rl)        # q_len = 1 is the plain path
    with pytest.raises(ValueError):
        OA.attention_multi(q[:, 0], k, v, off, lens, 0.4)


def test_multi_token_queries_reduce_to_library_sdpa_with_an_explicit_mask():
    """Equal lengths L: the q_len new tokens' rows are the last q_len of every head, and new token i may look at
    key j exactly when j <= L - q_len + i.  That mask is written out here as a boolean matrix, entry by entry,
    and handed to the library routine; an off-by-one in the oracle's visibility rule shows as a large error."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(33)
    for B, Hkv, G, D, L, QL in ((2, 2, 3, 8, 19, 4), (1, 1, 1, 4, 5, 5), (2, 3, 2, 16, 40, 2), (1, 2, 4, 8, 3, 6)):
        lens = np.full((B, Hkv), L, dtype=np.int32)
        off, total = W.packed_offsets(lens)
        q = rng.standard_normal((B, QL, Hkv * G, D))
        k = rng.standard_normal((total, D))
        v = rng.standard_normal((total, D))
        scale = 0.37
        out, lse = OA.attention_multi(q, k, v, off, lens, scale)
        mask = torch.zeros((QL, L), dtype=torch.bool)
        for i in range(QL):
            for j in range(L):
                mask[i, j] = j <= L - QL + i              # key j is not one of the new tokens after token i
        kt = torch.from_numpy(k).reshape(B, Hkv, L, D).repeat_interleave(G, dim=1)
        vt = torch.from_numpy(v).reshape(B, Hkv, L, D).repeat_interleave(G, dim=1)
        qt = torch.from_numpy(q).permute(0, 2, 1, 3)      # [B, Hq, QL, D]
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask, scale=scale)
        ref = ref.permute(0, 2, 1, 3).numpy()
        seen = mask.any(dim=1).numpy()                    # a new token that sees no key at all: out 0, lse -inf
        for i in range(QL):
            if seen[i]:
                assert np.abs(out[:, i] - ref[:, i]).max() < 1e-10
                s = torch.einsum("bhd,bhjd->bhj", qt[:, :, i], kt) * scale
                want = torch.logsumexp(s.masked_fill(~mask[i], float("-inf")), dim=-1).numpy()
                assert np.abs(lse[:, i] - want).max() < 1e-10
            else:
                assert (out[:, i] == 0).all() and np.isneginf(lse[:, i]).all()
        assert not seen.all() or QL <= L


# ---- a cache stored as 8-bit floats ------------------------------------------------------------
def test_e4m3_decoding_against_an_independent_converter_and_known_values():
    torch = pytest.importorskip("torch")
    codes = np.arange(256, dtype=np.uint8)
    got = OA.decode_e4m3fn(codes)
    ref = torch.arange(256, dtype=torch.uint8).view(torch.float8_e4m3fn).double().numpy()
    assert np.array_equal(np.isnan(got), np.isnan(ref)) and np.array_equal(got[~np.isnan(got)], ref[~np.isnan(ref)])
    assert got[0x38] == 1.0 and got[0x7e] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x08] == 2.0 ** -6
    assert got[0xb8] == -1.0 and got[0x00] == 0.0 and np.signbit(got[0x80]) and np.isnan(got[[0x7f, 0xff]]).all()
    assert (np.diff(got[:0x7f]) > 0).all()                 # the positive codes are ordered like their values
    with pytest.raises(TypeError):
        OA.decode_e4m3fn(np.arange(4))


def test_kv8_attention_is_attention_over_the_dequantised_cache():
    rng = np.random.default_rng(31)
    B, Hkv, G, D = 2, 2, 2, 8
    lens = rng.integers(0, 20, size=(B, Hkv)).astype(np.int32)
    off = np.arange(B * Hkv, dtype=np.int64).reshape(B, Hkv) * 24
    k8 = rng.integers(0, 0x78, size=(B * Hkv * 24, D)).astype(np.uint8)      # finite codes only
    v8 = (rng.integers(0, 0x78, size=(B * Hkv * 24, D)) | (rng.integers(0, 2, size=(B * Hkv * 24, D)) << 7)).astype(np.uint8)
    qf = rng.normal(size=(B, Hkv * G, D)).astype(np.float32)
    qbits = (qf.view(np.uint32) >> 16).astype(np.uint16)                     # truncated to bf16: any bf16 will do
    out, lse = OA.attention_kv8(qbits, k8, v8, off, lens, 0.3, 0.5, 0.25)
    q64 = (qbits.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    for b in range(B):
        for hq in range(Hkv * G):
            h = hq // G
            n, r0 = int(lens[b, h]), int(off[b, h])
            if n == 0:
                assert (out[b, hq] == 0).all() and np.isneginf(lse[b, hq])
                continue
            kk = OA.decode_e4m3fn(k8[r0:r0 + n]) * 0.5
            vv = OA.decode_e4m3fn(v8[r0:r0 + n]) * 0.25
            s = kk @ q64[b, hq] * 0.3
            w = np.exp(s - s.max())
            assert np.abs(out[b, hq] - (w @ vv) / w.sum()).max() < 1e-12
            assert abs(lse[b, hq] - (s.max() + np.log(w.sum()))) < 1e-12
    # scaling K by 2 and halving the score scale changes nothing; scaling V scales the output
    o2, l2 = OA.attention_kv8(qbits, k8, v8, off, lens, 0.15, 1.0, 0.5)
    live = lens.repeat(G, axis=1) > 0
    assert np.allclose(o2[live], 2 * out[live], rtol=1e-12, atol=0) and np.allclose(l2[live], lse[live], rtol=1e-12, atol=1e-12)


def test_e4m3_decoder_against_the_hand_decoded_fixture():
    """tests/golden/e4m3_codes.txt: codes decoded by hand from the format's definition."""
    import math
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "e4m3_codes.txt")
    n = 0
    for line in open(path):
        if not line.strip() or line.startswith("#"):
            continue
        code, value = [f.strip() for f in line.split("|")]
        got = float(OA.decode_e4m3fn(np.array([int(code, 16)], dtype=np.uint8))[0])
        want = float(value)
        if math.isnan(want):
            assert math.isnan(got), line
        else:
            assert got == want and math.copysign(1.0, got) == math.copysign(1.0, want), line
        n += 1
    assert n == 16


def test_kv8_scales_per_head_reduce_to_the_plain_oracle_on_scaled_rows():
    """A scale per KV head is the per-tensor oracle applied to K and V whose rows were scaled head by head: equal
    scales give the per-tensor result, and doubling one head's V scale doubles exactly that head's outputs."""
    rng = np.random.default_rng(3)
    B, Hkv, G, D = 2, 3, 2, 16
    lens = rng.integers(1, 30, size=(B, Hkv)).astype(np.int32)
    off, total = W.packed_offsets(lens, gap_rows=1)
    k8 = rng.integers(0, 0x7e, size=(total, D)).astype(np.uint8) | (rng.integers(0, 2, size=(total, D)).astype(np.uint8) << 7)
    v8 = rng.integers(0, 0x7e, size=(total, D)).astype(np.uint8) | (rng.integers(0, 2, size=(total, D)).astype(np.uint8) << 7)
    import torch
    q = W.to_numpy_bits(torch.randn((B, Hkv * G, D), generator=torch.Generator().manual_seed(1)).to(torch.bfloat16))
    o1, l1 = OA.attention_kv8(q, k8, v8, off, lens, 0.3, 0.01, 0.02)
    o2, l2 = OA.attention_kv8(q, k8, v8, off, lens, 0.3, [0.01] * Hkv, [0.02] * Hkv)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)
    o3, l3 = OA.attention_kv8(q, k8, v8, off, lens, 0.3, [0.01] * Hkv, [0.02, 0.04, 0.02])
    assert np.array_equal(l3, l1)
    assert np.allclose(o3[:, 2:4], 2 * o1[:, 2:4], rtol=1e-14, atol=0) and np.array_equal(o3[:, :2], o1[:, :2])
    # a K scale per head is a softmax scale per head: against the definition written out for one output
    ks = [0.01, 0.03, 0.02]
    o4, l4 = OA.attention_kv8(q, k8, v8, off, lens, 0.3, ks, 0.02)
    b, h, g = 1, 1, 1
    r0, n = int(off[b, h]), int(lens[b, h])
    qv = (q[b, h * G + g].astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    s = 0.3 * ks[h] * OA.decode_e4m3fn(k8[r0:r0 + n]) @ qv
    w_ = np.exp(s - s.max())
    ref = (w_ / w_.sum()) @ (0.02 * OA.decode_e4m3fn(v8[r0:r0 + n]))
    assert np.allclose(o4[b, h * G + g], ref, rtol=1e-12, atol=1e-15) and abs(l4[b, h * G + g] - (s.max() + np.log(w_.sum()))) < 1e-12
