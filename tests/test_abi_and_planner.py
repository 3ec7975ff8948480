"""CPU-side checks of the C ABI: the library loads, exports what the header declares,
plans bit-exactly like the oracle planner, and rejects bad arguments before touching
the GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads as W
from oracle import planner as OP

import paper_2502_15804_amd as F
from paper_2502_15804_amd import build as fbuild

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(F.LIB_PATH):
        fbuild.build()


def test_library_exports_every_declared_symbol():
    hdr = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include")))
                  if h.endswith(".h"))
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(fairkv_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(F.EXPORTS)
    L = F.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert F.fairkv_version() >= 100
    assert F.strerror(0) == "ok" and "workspace" in F.strerror(F.FAIRKV_EWORKSPACE)


def test_struct_layouts_match_the_header():
    assert ctypes.sizeof(F.fairkv_item) == 32
    assert ctypes.sizeof(F.fairkv_plan_params) == 32
    assert ctypes.sizeof(F.fairkv_plan_summary) == 32
    p = F.fairkv_default_params(256)
    assert (p.n_slots, p.tile, p.min_chunk, p.max_split, p.oversub, p.overhead_tokens, p.policy, p.short_overhead_tokens) == \
        (256, 16, 32, 256, 2, 160, F.FAIRKV_POLICY_FAIR, 48)
    assert F.FAIRKV_SHORT_PAIR_TOKENS == OP.SHORT_PAIR_TOKENS == 96
    d = OP.Params()
    assert (d.n_slots, d.tile, d.min_chunk, d.max_split, d.oversub, d.overhead_tokens, d.policy) == \
        (256, 16, 32, 256, 2, 160, OP.POLICY_FAIR)


def _same_as_oracle(lens, B, Hkv, offs=None, **kw):
    lens = np.asarray(lens).reshape(B, Hkv)
    if offs is None:
        offs = W.packed_offsets(lens, gap_rows=1)[0]
    kw.setdefault("short_overhead_tokens", int(F.fairkv_default_params(1).short_overhead_tokens))   # the library's default
    op = OP.Params(**kw)
    o_items, o_slot_ptr, o_part_base, o_sum = OP.plan(lens.reshape(-1), np.asarray(offs).reshape(-1), B, Hkv, op)
    p = F.fairkv_default_params(1, **kw)
    plan = F.fairkv_plan(lens, offs, B, Hkv, p)
    got = [tuple(int(x) for x in rec) for rec in plan.items.tolist()]
    assert got == [it.astuple() for it in o_items]
    assert plan.slot_ptr.tolist() == o_slot_ptr
    assert plan.part_base.tolist() == o_part_base
    s = plan.summary
    assert (s.total_tokens, s.max_slot_load, s.min_slot_load, s.n_items, s.n_parts) == \
        (o_sum.total_tokens, o_sum.max_slot_load, o_sum.min_slot_load, o_sum.n_items, o_sum.n_parts)
    assert plan.slot_loads().max() == o_sum.max_slot_load


@pytest.mark.parametrize("name", list(W.WORKLOADS))
@pytest.mark.parametrize("policy", [0, 1, 2, 3])
def test_plan_is_bit_exact_on_the_workloads(name, policy):
    w = W.WORKLOADS[name]
    for layer in range(2):
        _same_as_oracle(W.lens(name, layer=layer), w.B, w.Hkv, n_slots=256, policy=policy)


def test_plan_is_bit_exact_on_random_cases():
    rng = np.random.default_rng(42)
    for _ in range(1200):
        B, Hkv = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        lens = rng.integers(0, 5001, size=(B, Hkv)).astype(np.int32)
        short = rng.random((B, Hkv)) < 0.3           # short pairs: at most 96 tokens, with a fixed cost of their own
        lens[short] = rng.integers(1, 130, size=int(short.sum()))
        lens[rng.random((B, Hkv)) < 0.1] = 0
        if rng.random() < 0.2:
            lens = (lens // 512) * 512          # many exact ties
        tile = int(rng.choice([1, 8, 16, 64, 128]))
        _same_as_oracle(lens, B, Hkv, n_slots=int(rng.integers(1, 65)), tile=tile,
                        min_chunk=tile * int(rng.integers(1, 9)), max_split=int(rng.integers(1, 40)),
                        oversub=int(rng.integers(1, 5)), overhead_tokens=int(rng.integers(0, 200)),
                        short_overhead_tokens=int(rng.choice([0, 0, 16, 48, 150])), policy=int(rng.integers(0, 4)))


def test_plan_sizing_call_and_capacity_error():
    lens = np.array([[1000, 0], [300, 4000]], np.int32)
    off = np.array([[0, 1000], [1000, 1300]], np.int64)
    p = F.fairkv_default_params(4)
    s = F.fairkv_plan_summary()
    L = F.lib()
    rc = L.fairkv_plan(lens.ctypes.data, off.ctypes.data, 2, 2, ctypes.byref(p), None, 0, None, None, ctypes.byref(s))
    assert rc == F.FAIRKV_ECAP and s.n_items > 4 and s.total_tokens == 5300
    items = np.zeros(s.n_items, dtype=F.ITEM_DTYPE)
    small = np.full(2, -7, dtype=F.ITEM_DTYPE)
    rc = L.fairkv_plan(lens.ctypes.data, off.ctypes.data, 2, 2, ctypes.byref(p), small.ctypes.data, 2, None, None,
                       ctypes.byref(s))
    assert rc == F.FAIRKV_ECAP and (small["b"] == -7).all()          # nothing written
    rc = L.fairkv_plan(lens.ctypes.data, off.ctypes.data, 2, 2, ctypes.byref(p), items.ctypes.data, items.size,
                       None, None, ctypes.byref(s))
    assert rc == F.FAIRKV_OK and int(items["tok_count"].sum()) == 5300


def test_plan_all_empty_pairs():
    plan = F.fairkv_plan(np.zeros((3, 2), np.int32), np.zeros((3, 2), np.int64), 3, 2, F.fairkv_default_params(8))
    # every empty pair gets one empty item, so that its zero output is written by somebody
    assert plan.n_items == 6 and plan.n_parts == 6 and plan.part_base.tolist() == list(range(7))
    assert (plan.items["tok_count"] == 0).all() and plan.summary.total_tokens == 0


@pytest.mark.parametrize("bad", [dict(n_slots=0), dict(tile=0), dict(min_chunk=100), dict(max_split=0),
                                 dict(oversub=0), dict(overhead_tokens=-1), dict(policy=4), dict(short_overhead_tokens=-1),
                                 dict(min_chunk=0)])
def test_plan_rejects_bad_parameters(bad):
    p = F.fairkv_default_params(4, **bad)
    with pytest.raises(F.FairKVError) as e:
        F.fairkv_plan(np.ones((1, 1), np.int32), np.zeros((1, 1), np.int64), 1, 1, p)
    assert e.value.code == F.FAIRKV_EINVAL


def test_plan_rejects_bad_inputs():
    L = F.lib()
    p = F.fairkv_default_params(4)
    s = F.fairkv_plan_summary()
    bad = np.array([5, -1], np.int32)
    good = np.array([5, 1], np.int32)
    off = np.array([0, 5], np.int64)
    neg = np.array([0, -5], np.int64)
    lp, op = good.ctypes.data, off.ctypes.data
    assert L.fairkv_plan(bad.ctypes.data, op, 2, 1, ctypes.byref(p), None, 0, None, None, ctypes.byref(s)) == F.FAIRKV_EINVAL
    assert L.fairkv_plan(lp, neg.ctypes.data, 2, 1, ctypes.byref(p), None, 0, None, None, ctypes.byref(s)) == F.FAIRKV_EINVAL
    assert L.fairkv_plan(None, op, 2, 1, ctypes.byref(p), None, 0, None, None, ctypes.byref(s)) == F.FAIRKV_EINVAL
    assert L.fairkv_plan(lp, None, 2, 1, ctypes.byref(p), None, 0, None, None, ctypes.byref(s)) == F.FAIRKV_EINVAL
    assert L.fairkv_plan(lp, op, 0, 1, ctypes.byref(p), None, 0, None, None, ctypes.byref(s)) == F.FAIRKV_EINVAL
    assert L.fairkv_plan(lp, op, 2, 1, ctypes.byref(p), None, 4, None, None, ctypes.byref(s)) == F.FAIRKV_EINVAL
    assert L.fairkv_plan(lp, op, 2, 1, ctypes.byref(p), None, 0, None, None, None) == F.FAIRKV_EINVAL
    assert L.fairkv_plan(lp, op, 2, 1, ctypes.byref(p), None, 0, None, None, ctypes.byref(s)) == F.FAIRKV_ECAP
    with pytest.raises(F.FairKVError):
        F.fairkv_default_params(0)


def test_workspace_bytes():
    need = F.fairkv_workspace_bytes(10, 6, 8, 128)
    assert need >= 10 * 8 * 130 * 4 + 6 * 4 and need % 256 == 0
    assert F.fairkv_workspace_bytes(-1, 6, 8, 128) == 0 and F.fairkv_workspace_bytes(1, 6, 0, 128) == 0
    assert F.fairkv_workspace_bytes(1, 0, 8, 128) == 0


def test_decode_attn_validates_before_any_launch():
    """Every rejected call returns before the first HIP call, so this runs without a GPU.
    The pointers are never dereferenced on the host."""
    L = F.lib()
    fake = ctypes.c_void_p(0x1000)

    good_sp = np.array([0, 1], np.int32)
    good_item = np.zeros(1, F.ITEM_DTYPE)
    good_item["tok_count"], good_item["n_chunks"] = 5, 1

    def item(**kw):
        it = good_item.copy()
        for k_, v_ in kw.items():
            it[k_] = v_
        return it

    def call(q=fake, k=fake, v=fake, items=fake, ih=good_item, n_items=1, sp=good_sp, n_slots=1, n_parts=1, ws=fake,
             ws_bytes=1 << 30, out=fake, lse=None, B=1, Hq=8, Hkv=1, D=128, idt=0, odt=1, scale=0.1, n_rows=5):
        spp = sp.ctypes.data if sp is not None else None
        ihp = ih.ctypes.data if ih is not None else None
        return L.fairkv_decode_attn(q, k, v, n_rows, items, ihp, n_items, spp, n_slots, n_parts, ws, ws_bytes, out, lse,
                                    B, Hq, Hkv, D, idt, odt, scale, None)

    assert call(ih=None) == F.FAIRKV_EINVAL
    for bad in (item(b=1), item(h=-1), item(row=-3), item(tok_count=-1), item(n_chunks=0), item(chunk=1),
                item(part=1), item(n_chunks=2, chunk=1, part=0), item(n_chunks=2)):
        assert call(ih=bad) == F.FAIRKV_EINVAL, bad

    assert call(n_rows=4) == F.FAIRKV_EINVAL                       # the item's rows run past the end of K and V
    assert call(ih=item(row=1)) == F.FAIRKV_EINVAL
    assert call(q=None) == F.FAIRKV_EINVAL
    assert call(out=None) == F.FAIRKV_EINVAL
    assert call(items=None) == F.FAIRKV_EINVAL
    assert call(sp=None) == F.FAIRKV_EINVAL
    assert call(B=0) == F.FAIRKV_EINVAL
    assert call(n_slots=0) == F.FAIRKV_EINVAL
    assert call(sp=np.array([0, 2], np.int32)) == F.FAIRKV_EINVAL   # slot pointer does not end at n_items
    assert call(sp=np.array([1, 1], np.int32)) == F.FAIRKV_EINVAL
    big = np.zeros(322, np.int32); big[-1] = 1
    assert call(sp=big, n_slots=321, ws_bytes=16) == F.FAIRKV_EWORKSPACE   # more slots than workgroups: accepted as far as
                                                                           # the workspace check (slots then share workgroups)
    # a cut pair must come with all its pieces, each once, in consecutive partial slots
    two = np.zeros(2, F.ITEM_DTYPE)
    two["tok_count"], two["n_chunks"] = 2, 2
    two["row"], two["chunk"], two["part"] = [0, 2], [0, 1], [0, 1]
    sp2 = np.array([0, 2], np.int32)
    assert call(ih=two, n_items=2, sp=sp2, n_parts=2, ws_bytes=16) == F.FAIRKV_EWORKSPACE      # a whole pair in two pieces
    half = two[:1].copy()
    assert call(ih=half, n_parts=2) == F.FAIRKV_EINVAL                                           # its second piece is missing
    twice = two.copy(); twice["chunk"], twice["part"] = [0, 0], [0, 0]
    assert call(ih=twice, n_items=2, sp=sp2, n_parts=2) == F.FAIRKV_EINVAL                       # the first piece twice
    three = np.concatenate([two, two[1:]])
    assert call(ih=three, n_items=3, sp=np.array([0, 3], np.int32), n_parts=3) == F.FAIRKV_EINVAL   # a piece too many
    assert call(n_items=0) == F.FAIRKV_EINVAL                      # every pair has at least one item
    assert call(Hq=7, Hkv=2) == F.FAIRKV_EINVAL
    assert call(n_parts=0) == F.FAIRKV_EINVAL                      # fewer parts than items
    assert call(scale=float("nan")) == F.FAIRKV_EINVAL
    assert call(k=ctypes.c_void_p(0x1008)) == F.FAIRKV_EINVAL      # misaligned rows
    assert call(D=96) == F.FAIRKV_EUNSUPPORTED
    assert call(Hq=3, Hkv=1) == F.FAIRKV_EUNSUPPORTED
    assert call(idt=5) == F.FAIRKV_EUNSUPPORTED
    assert call(odt=2) == F.FAIRKV_EUNSUPPORTED
    assert call(ws_bytes=16) == F.FAIRKV_EWORKSPACE
    assert call(ws=None) == F.FAIRKV_EWORKSPACE


def test_decode_attn_kv8_and_multi_validate_before_any_launch():
    """The entry points for 8-bit caches and for several new tokens reject bad calls on the host as well."""
    L = F.lib()
    fake = ctypes.c_void_p(0x1000)
    sp = np.array([0, 1], np.int32)
    it = np.zeros(1, F.ITEM_DTYPE)
    it["tok_count"], it["n_chunks"] = 5, 1

    def kv8(q=fake, ks=0.02, vs=0.03, D=128, q_len=1, Hq=8, odt=1, ws_bytes=1 << 30, n_rows=5):
        return L.fairkv_decode_attn_kv8(q, fake, fake, n_rows, ks, vs, fake, it.ctypes.data, 1, sp.ctypes.data, 1, 1, fake,
                                        ws_bytes, fake, None, 1, q_len, Hq, 1, D, odt, 0.1, None)

    assert kv8(ks=float("nan")) == F.FAIRKV_EINVAL
    assert kv8(vs=float("inf")) == F.FAIRKV_EINVAL
    assert kv8(q=None) == F.FAIRKV_EINVAL
    assert kv8(n_rows=4) == F.FAIRKV_EINVAL
    assert kv8(D=32) == F.FAIRKV_EUNSUPPORTED
    assert kv8(odt=2) == F.FAIRKV_EUNSUPPORTED
    assert kv8(q_len=3) == F.FAIRKV_EUNSUPPORTED                   # 8 heads x 3 tokens: not a supported column count
    assert kv8(q_len=0) == F.FAIRKV_EINVAL
    assert kv8(ws_bytes=16) == F.FAIRKV_EWORKSPACE

    def multi(q_len=2, idt=0, Hq=8, tok=5, n_chunks=1, chunk=0, part=0, n_parts=1):
        it2 = it.copy()
        it2["tok_count"], it2["n_chunks"], it2["chunk"], it2["part"] = tok, n_chunks, chunk, part
        return L.fairkv_decode_attn_multi(fake, fake, fake, 5, fake, it2.ctypes.data, 1, sp.ctypes.data, 1, n_parts, fake,
                                          1 << 30, fake, None, 1, q_len, Hq, 1, 128, idt, 1, 0.1, None)

    assert multi(idt=1) == F.FAIRKV_EUNSUPPORTED                   # fp32 inputs take the single-token path only
    assert multi(q_len=4) == F.FAIRKV_EUNSUPPORTED                 # 32 columns
    assert multi(q_len=4, Hq=4, tok=2, n_chunks=2, chunk=1, part=1, n_parts=2) == F.FAIRKV_EINVAL   # last chunk shorter than q_len - 1


def test_decode_attn_kv8_per_head_validates_before_any_launch():
    L = F.lib()
    fake = ctypes.c_void_p(0x1000)
    sp = np.array([0, 1], np.int32)
    it = np.zeros(1, F.ITEM_DTYPE)
    it["tok_count"], it["n_chunks"] = 5, 1

    def call(ks, vs, Hkv=2, Hq=8, D=128):
        kp = ks.ctypes.data if ks is not None else None
        vp = vs.ctypes.data if vs is not None else None
        return L.fairkv_decode_attn_kv8_per_head(fake, fake, fake, 5, kp, vp, fake, it.ctypes.data, 1, sp.ctypes.data, 1, 1,
                                                 fake, 16, fake, None, 1, 1, Hq, Hkv, D, 1, 0.1, None)

    one = np.ones(16, np.float32)
    assert call(None, one) == F.FAIRKV_EINVAL
    assert call(one, None) == F.FAIRKV_EINVAL
    assert call(one, one, Hkv=9, Hq=9) == F.FAIRKV_EUNSUPPORTED              # more KV heads than scales fit
    bad = one.copy(); bad[1] = np.nan
    assert call(bad, one) == F.FAIRKV_EINVAL
    bad[1] = np.inf
    assert call(one, bad) == F.FAIRKV_EINVAL
    assert call(one, one) == F.FAIRKV_EWORKSPACE                             # everything else valid: the 16-byte workspace is too small


def test_static_and_trace_entry_points_validate_before_any_launch():
    L = F.lib()
    fake = ctypes.c_void_p(0x1000)
    sp = np.array([0, 1], np.int32)
    it = np.zeros(1, F.ITEM_DTYPE)
    it["tok_count"], it["n_chunks"] = 5, 1

    def static(n_parts=1, B=1, Hq=8, Hkv=1, q_len=1, D=128, q=fake, n_rows=5):
        return L.fairkv_decode_attn_static(q, fake, fake, n_rows, fake, it.ctypes.data, 1, sp.ctypes.data, 1, n_parts, fake,
                                           None, B, q_len, Hq, Hkv, D, 0, 1, 0.1, None)

    # the built-in workspace has a stated size: plans that need more are refused, whatever else they are
    assert F.fairkv_workspace_bytes(1500, 128, 8, 128) <= F.FAIRKV_STATIC_WORKSPACE_BYTES
    assert static(n_parts=4000) == F.FAIRKV_EWORKSPACE
    assert static(n_parts=(8 << 20) // 256 + 1) == F.FAIRKV_EWORKSPACE
    assert static(n_parts=1000, B=1 << 20, Hkv=1, Hq=8) == F.FAIRKV_EWORKSPACE       # the counters alone fill it
    assert static(q=None) == F.FAIRKV_EINVAL
    assert static(n_rows=4) == F.FAIRKV_EINVAL
    assert static(Hq=7, Hkv=2) == F.FAIRKV_EINVAL
    assert static(D=96) == F.FAIRKV_EUNSUPPORTED
    assert static(q_len=3) == F.FAIRKV_EUNSUPPORTED

    def trace(tr=fake, tr_bytes=1 << 20, D=128, Hq=8, n_slots=1, ws_bytes=16):
        spp = np.zeros(n_slots + 1, np.int32)
        spp[-1] = 1
        return L.fairkv_decode_attn_trace(fake, fake, fake, 5, fake, it.ctypes.data, 1, spp.ctypes.data, n_slots, 1, fake,
                                          ws_bytes, fake, None, 1, Hq, 1, D, 0.1, tr, tr_bytes, None)

    assert trace(tr=None) == F.FAIRKV_EINVAL
    assert trace(tr_bytes=64) == F.FAIRKV_EINVAL                 # room for half a workgroup's stamps
    assert trace(D=64) == F.FAIRKV_EUNSUPPORTED
    assert trace(Hq=2) == F.FAIRKV_EUNSUPPORTED
    assert trace(n_slots=321) == F.FAIRKV_EUNSUPPORTED
    assert trace() == F.FAIRKV_EWORKSPACE                        # everything else valid: the 16-byte workspace is too small


def test_stream_probe_shape_refuses_what_it_does_not_have():
    L = F.lib()
    fake = ctypes.c_void_p(0x1000)

    def probe(k=fake, waves=4, stages=2, kib=4, n_wg=256, nbytes=1 << 24):
        return L.fairkv_stream_probe_shape(k, fake, nbytes, n_wg, waves, stages, kib, fake, None)

    assert probe(k=None) == F.FAIRKV_EINVAL
    assert probe(k=ctypes.c_void_p(0x1008)) == F.FAIRKV_EINVAL          # not 16-byte aligned
    assert probe(n_wg=0) == F.FAIRKV_EINVAL
    assert probe(nbytes=-1) == F.FAIRKV_EINVAL
    for bad in (dict(waves=5), dict(waves=32), dict(stages=1), dict(stages=5), dict(kib=3), dict(kib=16), dict(kib=0),
                dict(waves=16, stages=4, kib=8), dict(waves=8, stages=3, kib=8)):      # the last two: rings beyond 160 KB
        assert probe(**bad) == F.FAIRKV_EUNSUPPORTED, bad


def test_workspace_reset_validates_before_any_launch():
    L = F.lib()
    fake = ctypes.c_void_p(0x1000)
    need = F.fairkv_workspace_counter_bytes(128)
    assert L.fairkv_workspace_reset(None, need, 128, None) == F.FAIRKV_EINVAL
    assert L.fairkv_workspace_reset(ctypes.c_void_p(0x1004), need, 128, None) == F.FAIRKV_EINVAL
    assert L.fairkv_workspace_reset(fake, need, 0, None) == F.FAIRKV_EINVAL
    assert L.fairkv_workspace_reset(fake, need - 1, 128, None) == F.FAIRKV_EWORKSPACE
