"""fairkv_pack / fairkv_append / fairkv_plan_grow: host logic on the CPU, kernels on the GPU against
the oracle, byte for byte."""
import ctypes

import numpy as np
import pytest

import paper_2502_15804_amd as F
import workloads as W
from oracle import pack as PK
from oracle import planner as OP


def test_plan_grow_matches_the_oracle_and_keeps_the_plan_valid():
    rng = np.random.default_rng(0)
    for _ in range(40):
        B, Hkv = int(rng.integers(1, 6)), int(rng.integers(1, 5))
        lens = rng.integers(0, 400, size=B * Hkv).astype(np.int32)
        slack = rng.integers(0, 3, size=B * Hkv).astype(np.int32)
        cap = lens + slack
        off = np.concatenate([[0], np.cumsum(cap.astype(np.int64))[:-1]])
        p = F.fairkv_default_params(int(rng.integers(1, 40)), policy=int(rng.integers(0, 4)), min_chunk=32)
        plan = F.fairkv_plan(lens, off, B, Hkv, p)
        ref_items, *_ = OP.plan(lens, off, B, Hkv, OP.Params(n_slots=p.n_slots, tile=p.tile, min_chunk=p.min_chunk,
                                                            max_split=p.max_split, oversub=p.oversub,
                                                            overhead_tokens=p.overhead_tokens, policy=p.policy,
                                                            short_overhead_tokens=p.short_overhead_tokens))
        items, l_lib, l_ref = plan.items.copy(), lens.copy(), [int(x) for x in lens]
        for step in range(3):
            F.fairkv_plan_grow(items, B, Hkv, l_lib, cap)
            ref_items = OP.grow(ref_items, l_ref, [int(x) for x in cap], Hkv)
            got = [tuple(int(x) for x in r) for r in items]
            assert got == [(i.row, i.tok_count, i.b, i.h, i.chunk, i.n_chunks, i.part) for i in ref_items]
            assert l_lib.tolist() == l_ref == np.minimum(lens + step + 1, cap).tolist()
            # still a partition of every pair's rows
            for pr in range(B * Hkv):
                mine = sorted((r for r in got if r[2] * Hkv + r[3] == pr), key=lambda r: r[4])
                assert sum(r[1] for r in mine) == l_lib[pr]
                row = int(off[pr])
                for r in mine:
                    assert r[1] == 0 or r[0] == row
                    row += r[1]


def test_plan_grow_argument_checks():
    items = np.zeros(2, dtype=F.ITEM_DTYPE)
    items["n_chunks"] = 1
    lens, cap = np.zeros(1, np.int32), np.ones(1, np.int32)
    with pytest.raises(F.FairKVError):
        F.fairkv_plan_grow(items, 1, 1, lens, cap)          # two last chunks for one pair
    with pytest.raises(ValueError):
        F.fairkv_plan_grow(items[:1], 2, 1, lens, cap)
    with pytest.raises(TypeError):
        F.fairkv_plan_grow(items[:1], 1, 1, lens.astype(np.int64), cap)


def test_pack_and_append_reject_bad_arguments_without_a_gpu():
    L = F.lib()
    null = ctypes.c_void_p(None)
    one = ctypes.c_void_p(16)
    assert L.fairkv_pack(null, one, 1, 1, 1, 128, 0, one, one, one, one, one, 1, one, one, 1, null, null) == F.FAIRKV_EINVAL
    assert L.fairkv_pack(one, one, 1, 1, 1, 128, 0, one, one, one, one, one, 0, one, one, 1, null, null) == F.FAIRKV_EINVAL
    assert L.fairkv_pack(one, one, 1, 1, 1, 96, 0, one, one, one, one, one, 1, one, one, 1, null, null) == F.FAIRKV_EUNSUPPORTED
    assert L.fairkv_pack(ctypes.c_void_p(8), one, 1, 1, 1, 128, 0, one, one, one, one, one, 1, one, one, 1, null, null) == F.FAIRKV_EINVAL
    assert L.fairkv_append(one, one, 1, 1, 128, 3, one, one, one, one, one, 1, null, null) == F.FAIRKV_EUNSUPPORTED
    assert L.fairkv_append(one, null, 1, 1, 128, 0, one, one, one, one, one, 1, null, null) == F.FAIRKV_EINVAL
    assert L.fairkv_append(one, one, 0, 1, 128, 0, one, one, one, one, one, 1, null, null) == F.FAIRKV_EINVAL


# ---- GPU -------------------------------------------------------------------------------------
def _bits(t):
    import torch
    if t.dtype == torch.uint8:
        return t.cpu().numpy()
    return t.view(torch.int16).cpu().numpy().view(np.uint16) if t.dtype == torch.bfloat16 else \
        t.view(torch.int32).cpu().numpy().view(np.uint32)


def _case(B, Hkv, T, D, dtype, lens, gap, seed, n_slots, policy=3):
    import torch
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    g = torch.Generator().manual_seed(seed)
    if dtype == "u8":                                       # a cache of 8-bit floats: any bytes will do here
        kd = torch.randint(0, 256, (B, Hkv, T, D), generator=g, dtype=torch.uint8)
        vd = torch.randint(0, 256, (B, Hkv, T, D), generator=g, dtype=torch.uint8)
    else:
        kd = torch.randn((B, Hkv, T, D), generator=g).to(tdt)
        vd = torch.randn((B, Hkv, T, D), generator=g).to(tdt)
    keep_ptr, keep_t = W.keep_lists(lens, T, seed=seed, recent=8)
    off, total = W.packed_offsets(lens, gap_rows=gap)
    p = F.fairkv_default_params(n_slots, policy=policy, overhead_tokens=16, min_chunk=32)
    plan = F.fairkv_plan(lens, off, B, Hkv, p)
    return kd, vd, keep_ptr, keep_t, off, total, plan


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("bf16", 64), ("f32", 64), ("f32", 128), ("u8", 128)])
def test_pack_matches_the_oracle_byte_for_byte(dtype, D):
    import torch
    rng = np.random.default_rng(D)
    B, Hkv, T = 3, 4, 700
    lens = rng.integers(0, 600, size=(B, Hkv)).astype(np.int32)
    lens[0, 0], lens[1, 1], lens[2, 2] = 0, 1, T            # empty, single, everything
    for n_slots, policy, gap in ((64, 3, 3), (7, 0, 0), (300, 2, 5)):
        kd, vd, keep_ptr, keep_t, off, total, plan = _case(B, Hkv, T, D, dtype, lens, gap, seed=D + gap, n_slots=n_slots,
                                                            policy=policy)
        k = torch.full((total + 4, D), 7, dtype=kd.dtype, device="cuda")
        v = torch.full((total + 4, D), 9, dtype=kd.dtype, device="cuda")
        rk, rv = _bits(k).copy(), _bits(v).copy()
        PK.pack(_bits(kd), _bits(vd), keep_ptr, keep_t, off.reshape(-1), rk, rv)
        bad = torch.zeros(1, dtype=torch.int32, device="cuda")
        F.fairkv_pack(kd.cuda(), vd.cuda(), torch.from_numpy(keep_ptr).cuda(), torch.from_numpy(keep_t).cuda(),
                      torch.from_numpy(off.reshape(-1)).cuda(), torch.from_numpy(plan.items.view(np.uint8).copy()).cuda(),
                      torch.from_numpy(plan.slot_ptr).cuda(), k, v, bad)
        torch.cuda.synchronize()
        assert int(bad.item()) == 0
        assert (_bits(k) == rk).all() and (_bits(v) == rv).all()


@pytest.mark.gpu
def test_pack_skips_what_points_outside_and_counts_it():
    import torch
    B, Hkv, T, D = 1, 2, 50, 128
    lens = np.array([[20, 30]], np.int32)
    kd, vd, keep_ptr, keep_t, off, total, plan = _case(B, Hkv, T, D, "bf16", lens, 0, seed=1, n_slots=4)
    keep_t = keep_t.copy()
    keep_t[3], keep_t[25] = T, -1                               # two rows name tokens the dense cache does not have
    items = plan.items.copy()
    extra = np.zeros(2, dtype=F.ITEM_DTYPE)
    extra[0] = (total - 1, 5, 0, 1, 0, 1, 0)                    # runs past the packed rows
    extra[1] = (0, 4, 0, 7, 0, 1, 0)                            # no such head
    items = np.concatenate([items, extra])
    slot_ptr = plan.slot_ptr.copy()
    slot_ptr[-1] += 2
    k = torch.zeros((total, D), dtype=torch.bfloat16, device="cuda")
    v = torch.zeros_like(k)
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")
    F.fairkv_pack(kd.cuda(), vd.cuda(), torch.from_numpy(keep_ptr).cuda(), torch.from_numpy(keep_t).cuda(),
                  torch.from_numpy(off.reshape(-1)).cuda(), torch.from_numpy(items.view(np.uint8).copy()).cuda(),
                  torch.from_numpy(slot_ptr).cuda(), k, v, bad)
    torch.cuda.synchronize()
    assert int(bad.item()) == 4
    good = np.ones(total, bool)
    good[[3, 25]] = False
    rk, rv = np.zeros((total, D), np.uint16), np.zeros((total, D), np.uint16)
    kt2 = keep_t.copy()
    kt2[[3, 25]] = 0
    PK.pack(_bits(kd), _bits(vd), keep_ptr, kt2, off.reshape(-1), rk, rv)
    assert (_bits(k)[good] == rk[good]).all() and (_bits(k)[~good] == 0).all() and (_bits(v)[good] == rv[good]).all()


@pytest.mark.gpu
@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_append_then_attend_over_the_grown_cache(dtype, D):
    import torch
    from oracle import attention as OA
    from paper_2502_15804_amd.runtime import DecodeLayer
    rng = np.random.default_rng(5)
    B, Hkv, G, steps = 4, 2, 2, 3
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    lens = rng.integers(0, 300, size=(B, Hkv)).astype(np.int32)
    lens[0, 0] = 0
    cap = (lens + rng.integers(1, steps + 2, size=(B, Hkv))).astype(np.int32)     # some pairs run out of room
    off, total = W.packed_offsets(cap)
    w = W.Workload("case", B, Hkv * G, Hkv, D, dtype, 1, 1e-5 if dtype == "f32" else 1e-2, "")
    q, k, v = W.make_qkv(w, total, seed=2)
    k, v = k.cuda(), v.cuda()
    rk, rv = _bits(k).copy(), _bits(v).copy()
    l_dev = torch.from_numpy(lens.reshape(-1).copy()).cuda()
    l_ref = lens.reshape(-1).copy()
    off_d, cap_d = torch.from_numpy(off.reshape(-1)).cuda(), torch.from_numpy(cap.reshape(-1)).cuda()
    full = torch.zeros(1, dtype=torch.int32, device="cuda")
    plan = F.fairkv_plan(lens, off, B, Hkv, F.fairkv_default_params(24, min_chunk=32))
    items, l_plan = plan.items.copy(), lens.reshape(-1).copy()
    n_full = 0
    for s in range(steps):
        g = torch.Generator().manual_seed(100 + s)
        kn, vn = torch.randn((B, Hkv, D), generator=g).to(tdt), torch.randn((B, Hkv, D), generator=g).to(tdt)
        F.fairkv_append(kn.cuda(), vn.cuda(), off_d, l_dev, cap_d, k, v, full)
        n_full += PK.append(rk, rv, _bits(kn), _bits(vn), off.reshape(-1), l_ref, cap.reshape(-1))
        F.fairkv_plan_grow(items, B, Hkv, l_plan, cap.reshape(-1))
    torch.cuda.synchronize()
    assert l_dev.cpu().numpy().tolist() == l_ref.tolist() == l_plan.tolist() and int(full.item()) == n_full > 0
    assert (_bits(k) == rk).all() and (_bits(v) == rv).all()
    # decode over the grown cache with the grown plan
    layer = DecodeLayer(q.cuda(), k, v, off, lens, w.scale, params=F.fairkv_default_params(24, min_chunk=32))
    assert (layer.plan.items == plan.items).all()
    layer.plan.items[:] = items
    layer.items_d.copy_(torch.from_numpy(items.view(np.uint8).copy()))
    out, lse = layer.run()
    torch.cuda.synchronize()
    ro, rl = OA.attention(W.to_numpy_bits(q), W.to_numpy_bits(k.cpu()), W.to_numpy_bits(v.cpu()), off, l_ref.reshape(B, Hkv),
                          w.scale)
    assert np.abs(out.float().cpu().numpy() - ro).max() <= w.tol


@pytest.mark.gpu
def test_cache_of_8bit_floats_packed_grown_and_attended():
    """The whole chain on E4M3 bytes: gather the kept tokens, append one decode step's rows, attend."""
    import torch
    from oracle import attention as OA
    from paper_2502_15804_amd.runtime import DecodeLayer
    rng = np.random.default_rng(11)
    B, Hkv, G, T, D = 3, 2, 4, 400, 128
    ks, vs = 0.021, 0.017
    lens = rng.integers(1, 350, size=(B, Hkv)).astype(np.int32)
    cap = (lens + 1).astype(np.int32)
    off, total = W.packed_offsets(cap)
    w = W.Workload("case", B, Hkv * G, Hkv, D, "bf16", 1, 1e-2, "")
    dense = W.Workload("dense", 1, 1, 1, D, "bf16", 1, 1e-2, "")
    kd, vd = (t.view(B, Hkv, T, D) for t in W.make_kv8(dense, B * Hkv * T, ks, vs, seed=4))
    kn, vn = (t.view(B, Hkv, D) for t in W.make_kv8(dense, B * Hkv, ks, vs, seed=5))
    keep_ptr, keep_t = W.keep_lists(lens, T, seed=3, recent=8)
    plan = F.fairkv_plan(lens, off, B, Hkv, F.fairkv_default_params(16, min_chunk=32))
    k = torch.zeros((total, D), dtype=torch.uint8, device="cuda")
    v = torch.zeros((total, D), dtype=torch.uint8, device="cuda")
    rk, rv = np.zeros((total, D), np.uint8), np.zeros((total, D), np.uint8)
    l_ref = lens.reshape(-1).copy()
    PK.pack(kd.numpy(), vd.numpy(), keep_ptr, keep_t, off.reshape(-1), rk, rv)
    PK.append(rk, rv, kn.numpy(), vn.numpy(), off.reshape(-1), l_ref, cap.reshape(-1))
    off_d = torch.from_numpy(off.reshape(-1)).cuda()
    l_dev = torch.from_numpy(lens.reshape(-1).copy()).cuda()
    F.fairkv_pack(kd.cuda(), vd.cuda(), torch.from_numpy(keep_ptr).cuda(), torch.from_numpy(keep_t).cuda(), off_d,
                  torch.from_numpy(plan.items.view(np.uint8).copy()).cuda(), torch.from_numpy(plan.slot_ptr).cuda(), k, v)
    F.fairkv_append(kn.cuda(), vn.cuda(), off_d, l_dev, torch.from_numpy(cap.reshape(-1)).cuda(), k, v)
    torch.cuda.synchronize()
    assert (k.cpu().numpy() == rk).all() and (v.cpu().numpy() == rv).all() and l_dev.cpu().numpy().tolist() == l_ref.tolist()
    g = torch.Generator().manual_seed(9)
    q = torch.randn((B, Hkv * G, D), generator=g).to(torch.bfloat16)
    grown = l_ref.reshape(B, Hkv)
    layer = DecodeLayer(q.cuda(), k, v, off, grown, w.scale, k_scale=ks, v_scale=vs)
    out, lse = layer.run()
    torch.cuda.synchronize()
    ro, rl = OA.attention_kv8(W.to_numpy_bits(q), rk, rv, off, grown, w.scale, ks, vs)
    assert np.abs(out.float().cpu().numpy() - ro).max() <= w.tol and np.abs(lse.cpu().numpy() - rl).max() <= w.tol
