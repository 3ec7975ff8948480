"""GPU parity: the HIP path, called through the C ABI, against the fp64 oracle on the same
seeded inputs, element by element.  Bars: max-abs-error 1e-5 (fp32 inputs), 1e-2 (bf16
inputs); log-sum-exp to the same bars."""
import numpy as np
import pytest

import workloads as W
from oracle import attention as OA

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _F():
    import paper_2502_15804_amd as F
    return F


def make_case(B, Hq, Hkv, D, dtype, lens, seed, gap_rows=0):
    w = W.Workload("case", B, Hq, Hkv, D, dtype, 1, 1e-5 if dtype == "f32" else 1e-2, "")
    off, total = W.packed_offsets(lens, gap_rows=gap_rows)
    q, k, v = W.make_qkv(w, total + 8, seed=seed)
    return w, off, q, k, v


def run_hip(w, q, k, v, off, lens, policy=3, n_slots=256, out_dtype=None, poison=True, calls=1, bf16_on_valu=False,
            **params):
    from paper_2502_15804_amd.runtime import DecodeLayer
    F = _F()
    p = F.fairkv_default_params(256, policy=policy, n_slots=n_slots, **params)
    layer = DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, w.scale, params=p, out_dtype=out_dtype,
                        bf16_on_valu=bf16_on_valu)
    for _ in range(calls):      # a second call finds the workspace as the first left it
        counters = F.fairkv_workspace_counter_bytes(lens.size)              # the first region of the workspace
        if poison:
            layer.out.fill_(float("nan"))
            layer.lse.fill_(float("nan"))
            layer.workspace[counters:].fill_(0xFF)                          # nothing but the counters carries state
        layer.run()
        torch.cuda.synchronize()
        assert int(layer.workspace[:counters].count_nonzero().item()) == 0   # every completed call leaves them zero
    return layer.out.float().cpu().numpy().astype(np.float64), layer.lse.cpu().numpy().astype(np.float64), layer


def check(w, q, k, v, off, lens, tol=None, **kw):
    tol = tol or w.tol
    out, lse, layer = run_hip(w, q, k, v, off, lens, **kw)
    ro, rl = OA.attention(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, w.scale)
    assert np.isfinite(out).all()
    err = np.abs(out - ro).max()
    assert err <= tol, f"max abs err {err:.3e} > {tol}"
    empty = np.isneginf(rl)
    assert np.array_equal(np.isneginf(lse), empty)
    if (~empty).any():
        lerr = np.abs(lse[~empty] - rl[~empty]).max()
        assert lerr <= tol, f"lse err {lerr:.3e}"
    return err, layer


def test_tiny_workload_fp32():
    w = W.WORKLOADS["tiny"]
    lens = W.lens("tiny", seed=0)
    off, total = W.packed_offsets(lens)
    q, k, v = W.make_qkv(w, total, seed=0)
    for policy in (0, 1, 2, 3):
        check(w, q, k, v, off, lens, policy=policy)
    # force splitting even of these short heads: chunks of 16 tokens
    for policy in (2, 3):
        err, layer = check(w, q, k, v, off, lens, policy=policy, tile=16, min_chunk=16, n_slots=64, oversub=1,
                           overhead_tokens=0, calls=2)
        assert layer.plan.n_items > 8


@pytest.mark.parametrize("dtype,D,G", [("bf16", 128, 8), ("bf16", 128, 4), ("bf16", 128, 2), ("bf16", 128, 1),
                                       ("bf16", 64, 8), ("bf16", 64, 2), ("f32", 64, 2), ("f32", 64, 8),
                                       ("f32", 128, 4), ("f32", 128, 1)])
def test_shapes_with_ragged_tails_and_chunks(dtype, D, G):
    rng = np.random.default_rng(D * 10 + G)
    B, Hkv = 3, 2
    lens = rng.integers(1, 900, size=(B, Hkv)).astype(np.int32)
    lens[0, 0] = 1            # a single token
    lens[1, 1] = 0            # an empty head
    lens[2, 0] = 64 * 7       # whole tiles exactly
    lens[2, 1] = 64 * 5 + 1   # one token into a new tile
    w, off, q, k, v = make_case(B, Hkv * G, Hkv, D, dtype, lens, seed=G, gap_rows=3)
    for policy, n_slots in ((0, 16), (2, 16), (3, 16), (3, 3), (1, 300)):
        check(w, q, k, v, off, lens, policy=policy, n_slots=n_slots, oversub=2, min_chunk=64, calls=2)


def test_chunked_equals_unchunked_on_the_gpu():
    # same inputs through one item per pair and through many chunks: both within the bar,
    # and close to each other.  The merge is exact in real arithmetic; what differs is the
    # rounding of the softmax weights to bf16 (relative 2^-9) against different running maxima.
    rng = np.random.default_rng(3)
    lens = rng.integers(200, 3000, size=(2, 2)).astype(np.int32)
    w, off, q, k, v = make_case(2, 16, 2, 128, "bf16", lens, seed=5)
    o1, l1, _ = run_hip(w, q, k, v, off, lens, policy=0)
    o2, l2, layer = run_hip(w, q, k, v, off, lens, policy=3, n_slots=64, min_chunk=64, overhead_tokens=0)
    assert layer.plan.n_items > 16
    assert np.abs(o1 - o2).max() < 2e-3 and np.abs(l1 - l2).max() < 2e-3
    ro, rl = OA.attention(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, w.scale)
    assert np.abs(o1 - ro).max() <= w.tol and np.abs(o2 - ro).max() <= w.tol


@pytest.mark.parametrize("D,G", [(128, 8), (128, 4), (64, 2)])
def test_bf16_cache_on_the_vector_alu_kernel(D, G):
    # FAIRKV_BF16_VALU: the same bf16 buffers and plan through the kernel that fp16 / fp32 caches use.  It keeps
    # the softmax weights in fp32, so it sits much closer to the oracle than the matrix-core kernel's bar, and the
    # two kernels, which share only the hand-over, agree with each other to the rounding of the weights to bf16.
    rng = np.random.default_rng(40 + G)
    lens = rng.integers(0, 1500, size=(3, 2)).astype(np.int32)
    lens[0, 1] = 1
    w, off, q, k, v = make_case(3, 2 * G, 2, D, "bf16", lens, seed=9, gap_rows=1)
    for policy, n_slots in ((0, 16), (3, 16), (3, 5)):
        err, _ = check(w, q, k, v, off, lens, tol=2e-5, policy=policy, n_slots=n_slots, min_chunk=64, bf16_on_valu=True)
    o1, l1, _ = run_hip(w, q, k, v, off, lens, n_slots=16, min_chunk=64, bf16_on_valu=True)
    o2, l2, _ = run_hip(w, q, k, v, off, lens, n_slots=16, min_chunk=64)
    assert np.abs(o1 - o2).max() < 4e-3
    keep = ~np.isneginf(l1)
    assert np.array_equal(keep, ~np.isneginf(l2)) and np.abs(l1[keep] - l2[keep]).max() < 4e-3


def test_all_heads_empty():
    lens = np.zeros((2, 2), np.int32)
    w, off, q, k, v = make_case(2, 8, 2, 128, "bf16", lens, seed=1)
    out, lse, layer = run_hip(w, q, k, v, off, lens)
    assert layer.plan.n_items == 4 and (out == 0).all() and np.isneginf(lse).all()


def test_length_one_returns_the_value_row_exactly():
    lens = np.ones((2, 4), np.int32)
    w, off, q, k, v = make_case(2, 8, 4, 64, "f32", lens, seed=2, gap_rows=1)
    out, lse, _ = run_hip(w, q, k, v, off, lens)
    vn = v.numpy().astype(np.float64)
    for b in range(2):
        for hq in range(8):
            assert np.array_equal(out[b, hq], vn[off[b, hq // 2]])


def test_large_scores_do_not_overflow():
    lens = np.array([[300]], np.int32)
    w, off, q, k, v = make_case(1, 8, 1, 128, "f32", lens, seed=3)
    k = k * 8.0      # scores of order +-100
    check(w, q, k, v, off, lens, tol=2e-5, policy=3, n_slots=4, min_chunk=64)


def test_rows_outside_the_heads_are_never_read():
    rng = np.random.default_rng(7)
    lens = rng.integers(1, 300, size=(2, 2)).astype(np.int32)
    w, off, q, k, v = make_case(2, 8, 2, 128, "bf16", lens, seed=4, gap_rows=2)
    owned = np.zeros(k.shape[0], bool)
    for b in range(2):
        for h in range(2):
            owned[off[b, h]: off[b, h] + lens[b, h]] = True
    k2, v2 = k.clone(), v.clone()
    k2[torch.from_numpy(~owned)] = float("inf")
    v2[torch.from_numpy(~owned)] = float("nan")
    o1, l1, _ = run_hip(w, q, k, v, off, lens, n_slots=8, min_chunk=64)
    o2, l2, _ = run_hip(w, q, k2, v2, off, lens, n_slots=8, min_chunk=64)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


def test_bf16_output_rounding():
    lens = np.array([[500, 77]], np.int32)
    w, off, q, k, v = make_case(1, 8, 2, 128, "bf16", lens, seed=6)
    o32, _, _ = run_hip(w, q, k, v, off, lens, n_slots=4, min_chunk=64)
    o16, _, _ = run_hip(w, q, k, v, off, lens, n_slots=4, min_chunk=64, out_dtype=torch.bfloat16)
    want = torch.from_numpy(o32.astype(np.float32)).to(torch.bfloat16).float().numpy()
    assert np.array_equal(o16.astype(np.float32), want)


def test_runs_are_bit_reproducible():
    lens = W.lens("llama70b", layer=1)[:4]
    w, off, q, k, v = make_case(4, 64, 8, 128, "bf16", lens, seed=8)
    o1, l1, _ = run_hip(w, q, k, v, off, lens)
    o2, l2, _ = run_hip(w, q, k, v, off, lens)
    assert np.array_equal(o1, o2) and np.array_equal(l1, l2)


@pytest.mark.parametrize("name", ["llama70b", "mistral24b", "faircopy", "stress"])
def test_full_size_workloads_every_output(name):
    """Full sizes, the launch configuration the benchmark times (default parameters for the
    device's compute-unit count), every output element against the oracle."""
    from paper_2502_15804_amd.runtime import DecodeLayer
    w = W.WORKLOADS[name]
    for layer_idx in (0, w.n_layers - 1):
        lens = W.lens(name, seed=0, layer=layer_idx)
        off, total = W.packed_offsets(lens)
        q, k, v = W.make_qkv(w, total, seed=0, layer=layer_idx)
        layer = DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, w.scale)
        layer.out.fill_(float("nan"))
        layer.run()
        torch.cuda.synchronize()
        out = layer.out.cpu().numpy().astype(np.float64)
        lse = layer.lse.cpu().numpy().astype(np.float64)
        ro, rl = OA.attention(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, w.scale)
        err = np.abs(out - ro).max()
        print(f"{name} layer {layer_idx}: items={layer.plan.n_items} max_abs_err={err:.3e}")
        assert err <= w.tol, f"{name} layer {layer_idx}: max abs err {err:.3e}"
        fin = np.isfinite(rl)
        assert np.array_equal(np.isneginf(lse), ~fin) and np.abs(lse[fin] - rl[fin]).max() <= w.tol
        for policy in ((0, 2) if layer_idx == 0 else ()):
            p = _F().fairkv_default_params(256, policy=policy)
            naive = DecodeLayer(layer.q, layer.k, layer.v, off, lens, w.scale, params=p)
            naive.run()
            torch.cuda.synchronize()
            assert np.abs(naive.out.cpu().numpy().astype(np.float64) - ro).max() <= w.tol


def test_slot_lists_longer_than_the_item_table():
    # 200 pairs on 2 slots: 100 items per slot, so the kernel walks its list in more than one table fill
    rng = np.random.default_rng(21)
    B, Hkv, G = 25, 8, 4
    lens = rng.integers(0, 90, size=(B, Hkv)).astype(np.int32)
    w, off, q, k, v = make_case(B, Hkv * G, Hkv, 128, "bf16", lens, seed=9, gap_rows=1)
    for policy in (0, 3):
        err, layer = check(w, q, k, v, off, lens, policy=policy, n_slots=2, calls=2)
        assert np.diff(layer.plan.slot_ptr).max() > 64


def test_many_cut_pieces_per_slot_and_per_pair():
    # equal split over few slots: every slot holds many pieces of cut pairs (more than the pending
    # buffer), and the long pair is in more pieces than one merge batch
    lens = np.array([[9000, 700, 40], [33, 2500, 1]], np.int32)
    w, off, q, k, v = make_case(2, 24, 3, 128, "bf16", lens, seed=10)
    err, layer = check(w, q, k, v, off, lens, policy=2, n_slots=3, oversub=6, min_chunk=64, calls=2)
    assert int(layer.plan.items["n_chunks"].max()) > 8 and layer.plan.n_items > 20
    err, layer = check(w, q, k, v, off, lens, policy=3, n_slots=40, min_chunk=32, overhead_tokens=0, calls=2)
    assert int(layer.plan.items["n_chunks"].max()) > 8
    # the cap on pieces per pair (eq. 3) leaves one very long last piece
    err, layer = check(w, q, k, v, off, lens, policy=3, n_slots=40, min_chunk=32, overhead_tokens=0, max_split=3)
    assert int(layer.plan.items["n_chunks"].max()) == 3


def test_longest_supported_head_and_most_slots():
    rng = np.random.default_rng(22)
    lens = rng.integers(1, 400, size=(4, 8)).astype(np.int32)
    lens[1, 3] = 32768
    w, off, q, k, v = make_case(4, 64, 8, 128, "bf16", lens, seed=11)
    for n_slots in (256, 320):
        err, layer = check(w, q, k, v, off, lens, policy=3, n_slots=n_slots)
    assert err < 5e-3


def test_hip_graph_replays_match_eager():
    from paper_2502_15804_amd.runtime import DecodeLayer
    w = W.WORKLOADS["llama70b"]
    lens = W.lens("llama70b", layer=2)[:4]
    small = W.Workload("g", 4, w.Hq, w.Hkv, w.D, w.dtype, 1, w.tol, "")
    off, total = W.packed_offsets(lens)
    q, k, v = W.make_qkv(small, total, seed=3)
    layer = DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, small.scale)
    layer.run()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        layer.run()
    kn, vn = W.to_numpy_bits(k), W.to_numpy_bits(v)
    for rep in range(3):
        # eager work and a new query between the replays
        qr = (torch.randn(q.shape, generator=torch.Generator().manual_seed(100 + rep)) * (1 + rep)).to(torch.bfloat16)
        layer.q.copy_(qr.cuda())
        layer.out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = layer.out.cpu().numpy().astype(np.float64)
        ro, _ = OA.attention(W.to_numpy_bits(qr), kn, vn, off, lens, small.scale)
        assert np.abs(got - ro).max() <= small.tol, rep
        layer.run()                      # the same step eagerly: bit-identical to the replay
        torch.cuda.synchronize()
        assert np.array_equal(layer.out.cpu().numpy().astype(np.float64), got)


def test_layers_sharing_one_workspace_on_one_stream():
    from paper_2502_15804_amd.runtime import DecodeLayer
    F = _F()
    w = W.WORKLOADS["mistral24b"]
    small = W.Workload("s", 6, w.Hq, w.Hkv, w.D, w.dtype, 1, w.tol, "")
    cases, need = [], 0
    for li in range(3):
        lens = W.lens("mistral24b", layer=li)[:6]
        off, total = W.packed_offsets(lens)
        q, k, v = W.make_qkv(small, total, seed=li)
        plan = F.fairkv_plan(lens, off, 6, small.Hkv, F.fairkv_default_params(256))
        need = max(need, F.fairkv_workspace_bytes(plan.n_parts, 6 * small.Hkv, small.G, small.D))
        cases.append((lens, off, q, k, v))
    ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
    layers = [DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, small.scale, workspace=ws, want_lse=False)
              for lens, off, q, k, v in cases]
    for _ in range(2):
        for l in layers:
            l.run()                        # back to back, no synchronisation in between
    torch.cuda.synchronize()
    for l, (lens, off, q, k, v) in zip(layers, cases):
        ro, _ = OA.attention(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, small.scale)
        assert np.abs(l.out.cpu().numpy().astype(np.float64) - ro).max() <= small.tol


# ---- several new tokens per sequence (fairkv_decode_attn_multi) ---------------------------------
@pytest.mark.parametrize("D,G,QL", [(128, 8, 2), (128, 4, 4), (128, 4, 2), (128, 2, 2), (128, 1, 4), (128, 2, 8),
                                    (128, 1, 16), (64, 8, 2), (64, 2, 4), (64, 1, 2)])
def test_several_new_tokens_per_sequence(D, G, QL):
    F = _F()
    from paper_2502_15804_amd.runtime import DecodeLayer
    rng = np.random.default_rng(1000 * D + 10 * G + QL)
    B, Hkv = 3, 2
    lens = rng.integers(QL, 700, size=(B, Hkv)).astype(np.int32)
    lens[0, 0] = max(QL - 1, 1)      # shorter than the draft: the first new tokens see nothing or little
    lens[1, 1] = 0                   # an empty head
    lens[2, 0] = 64 * 5              # the last tile of the last chunk is full
    lens[2, 1] = 64 * 3 + 1
    w = W.Workload("case", B, Hkv * G, Hkv, D, "bf16", 1, 1e-2, "")
    off, total = W.packed_offsets(lens, gap_rows=2)
    g = torch.Generator().manual_seed(G * 100 + QL)
    q = torch.randn((B, QL, Hkv * G, D), generator=g).to(torch.bfloat16)
    _, k, v = W.make_qkv(w, total + 8, seed=QL)
    ro, rl = OA.attention_multi(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, w.scale)
    for policy, n_slots, mc in ((3, 16, 32), (0, 16, 32), (3, 5, 16), (3, 300, 16), (2, 40, 64)):
        p = F.fairkv_default_params(256, policy=policy, n_slots=n_slots, min_chunk=mc, oversub=2)
        layer = DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, w.scale, params=p)
        it = layer.plan.items
        short_tail = ((it["n_chunks"] > 1) & (it["chunk"] == it["n_chunks"] - 1) & (it["tok_count"] < QL - 1)).any()
        if short_tail:               # equal shares can leave a last chunk shorter than the rows to hide: refused
            assert policy == 2
            with pytest.raises(F.FairKVError) as e:
                layer.run()
            assert e.value.code == F.FAIRKV_EINVAL
            continue
        for _ in range(2):           # the second call finds the counters the first one left
            layer.out.fill_(float("nan"))
            layer.lse.fill_(float("nan"))
            layer.run()
            torch.cuda.synchronize()
        out = layer.out.cpu().numpy().astype(np.float64)
        lse = layer.lse.cpu().numpy().astype(np.float64)
        assert out.shape == ro.shape and np.isfinite(out).all()
        assert np.abs(out - ro).max() <= w.tol, (policy, n_slots, np.abs(out - ro).max())
        empty = np.isneginf(rl)
        assert (np.isneginf(lse) == empty).all() and (out[empty] == 0).all()
        assert np.abs(lse[~empty] - rl[~empty]).max() <= w.tol


def test_several_new_tokens_argument_checks():
    F = _F()
    from paper_2502_15804_amd.runtime import DecodeLayer
    lens = np.full((1, 1), 40, np.int32)
    off, total = W.packed_offsets(lens)
    w = W.Workload("case", 1, 8, 1, 128, "bf16", 1, 1e-2, "")
    _, k, v = W.make_qkv(w, total, seed=0)
    q = torch.randn((1, 3, 8, 128)).to(torch.bfloat16)            # 8 heads x 3 tokens = 24 columns: not a supported count
    with pytest.raises(F.FairKVError) as e:
        DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, w.scale).run()
    assert e.value.code == F.FAIRKV_EUNSUPPORTED
    w32 = W.Workload("case", 1, 2, 1, 64, "f32", 1, 1e-5, "")
    _, k32, v32 = W.make_qkv(w32, total, seed=0)
    with pytest.raises(F.FairKVError) as e:                       # fp32 inputs take the single-token path only
        DecodeLayer(torch.randn((1, 2, 2, 64)).cuda(), k32.cuda(), v32.cuda(), off, lens, w32.scale).run()
    assert e.value.code == F.FAIRKV_EUNSUPPORTED


def test_pairs_cut_into_very_many_pieces_are_merged_in_two_levels():
    """Long heads, few of them, many slots: pairs in 32 ... 80 pieces, merged group by group.  Several
    calls in a row on one workspace: every counter is back at zero after each."""
    F = _F()
    rng = np.random.default_rng(11)
    for B, Hkv, G, n_slots, lens_ in ((1, 2, 8, 256, [[16384, 3000]]), (2, 1, 4, 160, [[9000], [700]]),
                                      (1, 3, 2, 256, [[2049, 17, 12000]])):
        lens = np.array(lens_, np.int32)
        w, off, q, k, v = make_case(B, Hkv * G, Hkv, 128, "bf16", lens, seed=int(rng.integers(1 << 20)), gap_rows=1)
        err, layer = check(w, q, k, v, off, lens, policy=3, n_slots=n_slots, min_chunk=32, overhead_tokens=16, calls=3)
        assert layer.plan.items["n_chunks"].max() >= 32
        assert int(layer.workspace[:F.fairkv_workspace_counter_bytes(B * Hkv)].count_nonzero().item()) == 0
    # equal shares with a tiny cap on the counter index: the pair falls back to one level
    lens = np.array([[5000, 5000, 5000]], np.int32)
    w, off, q, k, v = make_case(1, 6, 3, 64, "bf16", lens, seed=5)
    err, layer = check(w, q, k, v, off, lens, policy=2, n_slots=64, min_chunk=32, oversub=4, calls=2)
    assert layer.plan.items["n_chunks"].max() > 8


# ---- a cache stored as 8-bit floats ---------------------------------------------------------------
def _kv8_case(B, Hkv, G, lens, seed, q_len=1, gap_rows=2, D=128):
    w = W.Workload("case", B, Hkv * G, Hkv, D, "bf16", 1, 1e-2, "")
    off, total = W.packed_offsets(lens, gap_rows=gap_rows)
    k_scale, v_scale = 0.0173, 0.0291                 # not powers of two: a scale applied to the wrong side shows
    k8, v8 = W.make_kv8(w, total + 8, k_scale, v_scale, seed=seed)
    g = torch.Generator().manual_seed(seed + 77)
    shape = (B, q_len, Hkv * G, D) if q_len > 1 else (B, Hkv * G, D)
    q = torch.randn(shape, generator=g).to(torch.bfloat16)
    return w, off, q, k8, v8, k_scale, v_scale


def _kv8_check(w, off, lens, q, k8, v8, k_scale, v_scale, out_dtype=None, **params):
    F = _F()
    from paper_2502_15804_amd.runtime import DecodeLayer
    ro, rl = OA.attention_kv8(W.to_numpy_bits(q), k8.numpy(), v8.numpy(), off, lens, w.scale, k_scale, v_scale)
    p = F.fairkv_default_params(256, **params)
    layer = DecodeLayer(q.cuda(), k8.cuda(), v8.cuda(), off, lens, w.scale, params=p, out_dtype=out_dtype,
                        k_scale=k_scale, v_scale=v_scale)
    for _ in range(2):
        layer.out.fill_(float("nan"))
        layer.lse.fill_(float("nan"))
        counters = F.fairkv_workspace_counter_bytes(lens.size)
        layer.workspace[counters:].fill_(0xFF)
        layer.run()
        torch.cuda.synchronize()
        assert int(layer.workspace[:counters].count_nonzero().item()) == 0
    out = layer.out.float().cpu().numpy().astype(np.float64)
    lse = layer.lse.cpu().numpy().astype(np.float64)
    assert out.shape == ro.shape and np.isfinite(out).all()
    err = np.abs(out - ro).max()
    assert err <= w.tol, f"max abs err {err:.3e}"
    empty = np.isneginf(rl)
    assert (np.isneginf(lse) == empty).all() and (out[empty] == 0).all()
    if (~empty).any():
        assert np.abs(lse[~empty] - rl[~empty]).max() <= w.tol
    return layer


@pytest.mark.parametrize("G,D", [(8, 128), (4, 128), (2, 128), (1, 128), (8, 64), (2, 64), (1, 64)])
def test_kv8_shapes_with_ragged_tails_and_chunks(G, D):
    rng = np.random.default_rng(800 + G + D)
    B, Hkv = 3, 2
    lens = rng.integers(1, 900, size=(B, Hkv)).astype(np.int32)
    lens[0, 0] = 1                    # a single row
    lens[0, 1] = 31                   # one row short of a 32-token step
    lens[1, 0] = 0                    # an empty head
    lens[1, 1] = 32 * 4 * 3           # whole steps for every wave
    lens[2, 0] = 33
    case = _kv8_case(B, Hkv, G, lens, seed=G, D=D)
    w, off, q, k8, v8, ks, vs = case
    for policy, n_slots, mc in ((3, 16, 32), (0, 16, 32), (3, 5, 16), (3, 300, 16), (2, 40, 64)):
        _kv8_check(w, off, lens, q, k8, v8, ks, vs, policy=policy, n_slots=n_slots, min_chunk=mc, oversub=2)


def test_kv8_length_one_returns_the_scaled_value_row():
    lens = np.ones((2, 2), np.int32)
    w, off, q, k8, v8, ks, vs = _kv8_case(2, 2, 4, lens, seed=5)
    layer = _kv8_check(w, off, lens, q, k8, v8, ks, vs)
    out = layer.out.cpu().numpy()
    want = v8.view(torch.float8_e4m3fn).float().numpy() * np.float32(vs)
    for b in range(2):
        for h in range(2):
            for g in range(4):
                assert np.array_equal(out[b, h * 4 + g], want[off[b, h]])     # one weight of exactly 1, one product


@pytest.mark.parametrize("G,QL,D", [(8, 2, 128), (4, 4, 128), (1, 16, 128), (4, 2, 64)])
def test_kv8_several_new_tokens(G, QL, D):
    rng = np.random.default_rng(900 + G)
    B, Hkv = 2, 2
    lens = rng.integers(QL, 600, size=(B, Hkv)).astype(np.int32)
    lens[0, 0] = max(QL - 1, 1)
    lens[1, 1] = 64 * 4 + 1
    w, off, q, k8, v8, ks, vs = _kv8_case(B, Hkv, G, lens, seed=G + QL, q_len=QL, D=D)
    for policy, n_slots, mc in ((3, 16, 32), (3, 300, 16), (0, 4, 32)):
        _kv8_check(w, off, lens, q, k8, v8, ks, vs, policy=policy, n_slots=n_slots, min_chunk=mc, oversub=2)


def test_kv8_full_size_headline_workload():
    w = W.WORKLOADS["llama70b"]
    lens = W.lens("llama70b")
    off, total = W.packed_offsets(lens)
    ks, vs = 0.02, 0.03
    k8, v8 = W.make_kv8(w, total, ks, vs, seed=3)
    q, _, _ = W.make_qkv(w, 1, seed=3)
    _kv8_check(w, off, lens, q, k8, v8, ks, vs, out_dtype=torch.bfloat16)


def test_kv8_argument_checks():
    F = _F()
    from paper_2502_15804_amd.runtime import DecodeLayer
    lens = np.full((1, 1), 40, np.int32)
    off, total = W.packed_offsets(lens)
    q = torch.randn((1, 8, 32)).to(torch.bfloat16)                # head_dim 32 is not built
    k8 = torch.zeros((total, 32), dtype=torch.uint8)
    with pytest.raises(F.FairKVError) as e:
        DecodeLayer(q.cuda(), k8.cuda(), k8.cuda(), off, lens, 0.125).run()
    assert e.value.code == F.FAIRKV_EUNSUPPORTED
    q = torch.randn((1, 8, 128)).to(torch.bfloat16)
    k8 = torch.zeros((total, 128), dtype=torch.uint8)
    with pytest.raises(F.FairKVError) as e:
        DecodeLayer(q.cuda(), k8.cuda(), k8.cuda(), off, lens, 0.125, k_scale=float("inf")).run()
    assert e.value.code == F.FAIRKV_EINVAL


# ---- many small random configurations --------------------------------------------------------------
@pytest.mark.parametrize("seed", range(24))
def test_random_small_configurations(seed):
    """Shapes, budgets, policies, slot counts, storage and the number of new tokens drawn at random (valid
    inputs only): the element-by-element bar holds for every draw."""
    F = _F()
    from paper_2502_15804_amd.runtime import DecodeLayer
    rng = np.random.default_rng(4000 + seed)
    D = int(rng.choice([64, 128]))
    G = int(rng.choice([1, 2, 4, 8]))
    QL = int(rng.choice([q for q in (1, 1, 2, 4, 8, 16) if G * q <= 16]))
    kv8 = bool(rng.integers(0, 2))
    B, Hkv = int(rng.integers(1, 5)), int(rng.integers(1, 4))
    kind = int(rng.integers(0, 3))
    if kind == 0:                                  # mostly short, a few long
        lens = rng.integers(0, 80, size=(B, Hkv))
        lens[rng.integers(0, B), rng.integers(0, Hkv)] = int(rng.integers(500, 3000))
    elif kind == 1:                                # around whole tiles and steps
        lens = rng.choice([15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257], size=(B, Hkv))
    else:
        lens = rng.integers(0, 700, size=(B, Hkv))
    lens = np.maximum(lens, QL - 1 if rng.integers(0, 2) else 0).astype(np.int32)
    policy = int(rng.choice([0, 1, 2, 3, 3, 3]))
    n_slots = int(rng.choice([1, 3, 17, 64, 256, 320]))
    tile = int(rng.choice([16, 32]))
    params = dict(policy=policy, n_slots=n_slots, tile=tile, min_chunk=tile * int(rng.integers(1, 5)),
                  oversub=int(rng.integers(1, 4)), overhead_tokens=int(rng.choice([0, 16, 128, 256])),
                  max_split=int(rng.choice([2, 8, 256])))
    w = W.Workload("case", B, Hkv * G, Hkv, D, "bf16", 1, 1e-2, "")
    off, total = W.packed_offsets(lens, gap_rows=int(rng.integers(0, 4)))
    g = torch.Generator().manual_seed(seed)
    shape = (B, QL, Hkv * G, D) if QL > 1 else (B, Hkv * G, D)
    q = torch.randn(shape, generator=g).to(torch.bfloat16)
    ks, vs = (0.019, 0.023) if kv8 else (1.0, 1.0)
    if kv8:
        k, v = W.make_kv8(w, total + 4, ks, vs, seed=seed)
        ro, rl = OA.attention_kv8(W.to_numpy_bits(q), k.numpy(), v.numpy(), off, lens, w.scale, ks, vs)
    else:
        _, k, v = W.make_qkv(w, total + 4, seed=seed)
        fn = OA.attention_multi if QL > 1 else OA.attention
        ro, rl = fn(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, w.scale)
    layer = DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, w.scale, params=F.fairkv_default_params(256, **params),
                        k_scale=ks, v_scale=vs)
    it = layer.plan.items
    if QL > 1 and ((it["n_chunks"] > 1) & (it["chunk"] == it["n_chunks"] - 1) & (it["tok_count"] < QL - 1)).any():
        with pytest.raises(F.FairKVError):          # a last chunk shorter than the rows to hide: refused
            layer.run()
        return
    for _ in range(2):
        layer.out.fill_(float("nan"))
        layer.lse.fill_(float("nan"))
        layer.run()
        torch.cuda.synchronize()
    out = layer.out.cpu().numpy().astype(np.float64)
    lse = layer.lse.cpu().numpy().astype(np.float64)
    what = dict(D=D, G=G, QL=QL, kv8=kv8, B=B, Hkv=Hkv, **params)
    assert np.isfinite(out).all(), what
    assert np.abs(out - ro).max() <= w.tol, (what, np.abs(out - ro).max())
    empty = np.isneginf(rl)
    assert (np.isneginf(lse) == empty).all() and (out[empty] == 0).all(), what
    if (~empty).any():
        assert np.abs(lse[~empty] - rl[~empty]).max() <= w.tol, what


def test_kv8_with_a_scale_per_kv_head():
    F = _F()
    from paper_2502_15804_amd.runtime import DecodeLayer
    rng = np.random.default_rng(77)
    B, Hkv, G = 3, 4, 2
    lens = rng.integers(0, 500, size=(B, Hkv)).astype(np.int32)
    w, off, q, k8, v8, ks, vs = _kv8_case(B, Hkv, G, lens, seed=21)
    ks_h = [ks, ks * 1.7, ks * 0.6, ks * 1.1]            # the same bytes, read with a scale of its own per head
    vs_h = [vs * 0.8, vs, vs * 2.5, vs * 1.3]
    ro, rl = OA.attention_kv8(W.to_numpy_bits(q), k8.numpy(), v8.numpy(), off, lens, w.scale, ks_h, vs_h)
    for n_slots in (16, 256):
        layer = DecodeLayer(q.cuda(), k8.cuda(), v8.cuda(), off, lens, w.scale, k_scale=ks_h, v_scale=vs_h,
                            params=F.fairkv_default_params(256, n_slots=n_slots, min_chunk=32))
        layer.out.fill_(float("nan"))
        layer.run()
        torch.cuda.synchronize()
        out, lse = layer.out.cpu().numpy().astype(np.float64), layer.lse.cpu().numpy().astype(np.float64)
        assert np.isfinite(out).all() and np.abs(out - ro).max() <= w.tol
        empty = np.isneginf(rl)
        assert (np.isneginf(lse) == empty).all() and np.abs(lse[~empty] - rl[~empty]).max() <= w.tol
    k9 = torch.zeros((8, 128), dtype=torch.uint8).cuda()
    with pytest.raises(F.FairKVError) as e:              # more KV heads than scales fit in the kernel arguments
        DecodeLayer(torch.zeros((1, 9, 128), dtype=torch.bfloat16).cuda(), k9, k9, np.zeros((1, 9), np.int64),
                    np.zeros((1, 9), np.int32), 0.1, k_scale=[1.0] * 9, v_scale=[1.0] * 9).run()
    assert e.value.code == F.FAIRKV_EUNSUPPORTED


def test_stream_probe_runs_in_every_shape_it_offers():
    # the measurement aid: nothing to compare, but every instantiation must launch, stay inside the buffers
    # (the sizes below leave a ragged rest that it must not touch) and finish
    F = _F()
    k = torch.zeros(3 * (1 << 20) + 4096 + 16, dtype=torch.uint8, device="cuda")
    v = torch.zeros_like(k)
    sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
    for waves in (4, 8, 16):
        for stages in (2, 3, 4):
            for kib in (2, 4, 8):
                for n_wg in (7, 256, 1024):
                    if waves * stages * 2 * kib > 160:
                        with pytest.raises(F.FairKVError) as e:
                            F.fairkv_stream_probe(k, v, n_wg, sink, shape=(waves, stages, kib))
                        assert e.value.code == F.FAIRKV_EUNSUPPORTED
                    else:
                        F.fairkv_stream_probe(k, v, n_wg, sink, shape=(waves, stages, kib))
    F.fairkv_stream_probe(k, v, 256, sink)
    torch.cuda.synchronize()
    assert int(sink.count_nonzero().item()) == 0


def test_workspace_reset_recovers_a_workspace_with_stale_counters():
    # what a launch that died mid-way leaves behind: counters that are not zero.  After fairkv_workspace_reset the
    # next call is right again; the rest of the workspace may hold anything.
    F = _F()
    from paper_2502_15804_amd.runtime import DecodeLayer
    rng = np.random.default_rng(77)
    lens = rng.integers(100, 2500, size=(2, 4)).astype(np.int32)
    w, off, q, k, v = make_case(2, 16, 4, 128, "bf16", lens, seed=3)
    p = F.fairkv_default_params(256, n_slots=24, min_chunk=64)
    layer = DecodeLayer(q.cuda(), k.cuda(), v.cuda(), off, lens, w.scale, params=p)
    assert layer.plan.n_items > 8
    layer.workspace.fill_(0x5A)
    F.fairkv_workspace_reset(layer.workspace, lens.size)
    layer.run()
    torch.cuda.synchronize()
    counters = F.fairkv_workspace_counter_bytes(lens.size)
    assert int(layer.workspace[:counters].count_nonzero().item()) == 0
    ro, rl = OA.attention(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, w.scale)
    assert np.abs(layer.out.float().cpu().numpy() - ro).max() <= w.tol
    assert np.abs(layer.lse.cpu().numpy() - rl).max() <= w.tol
    small = torch.zeros(16, dtype=torch.uint8, device="cuda")
    with pytest.raises(F.FairKVError) as e:
        F.fairkv_workspace_reset(small, lens.size)
    assert e.value.code == F.FAIRKV_EWORKSPACE
