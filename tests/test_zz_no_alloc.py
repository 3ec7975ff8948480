"""fairkv_decode_attn_static (the entry point that allocates nothing: its workspace is a device array inside the
library) against fairkv_decode_attn_multi with a caller's workspace: same kernels, so the outputs must be the
same bits, and both within the parity bar of the oracle.  Two calls in a row, the second with a smaller input
(the array keeps whatever the first call left: its arrival counters must be zero again)."""
import ctypes

import numpy as np
import pytest

import workloads as W
from oracle import attention as OA

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _case(name, rows, layer, q_len=1, **params):
    import paper_2502_15804_amd as F
    w0 = W.WORKLOADS[name]
    lens = W.lens(name, layer=layer)[:rows]
    w = W.Workload("case", rows, w0.Hq, w0.Hkv, w0.D, w0.dtype, 1, w0.tol, "")
    off, total = W.packed_offsets(lens, gap_rows=1)
    q, k, v = W.make_qkv(w, total + 4, seed=40 + layer)
    if q_len > 1:
        g = torch.Generator().manual_seed(layer)
        q = torch.randn((rows, q_len, w.Hq, w.D), generator=g).to(torch.bfloat16)
    plan = F.fairkv_plan(lens, off, rows, w.Hkv, F.fairkv_default_params(256, **params))
    return w, lens, off, q, k, v, plan


def _call(static, w, q, k, v, plan, out, lse, workspace=None):
    import paper_2502_15804_amd as F
    L = F.lib()
    vp = ctypes.c_void_p
    q_len = q.shape[1] if q.dim() == 4 else 1
    items_d = torch.from_numpy(plan.items.view(np.uint8).copy()).cuda()
    head = (vp(q.data_ptr()), vp(k.data_ptr()), vp(v.data_ptr()), k.shape[0], vp(items_d.data_ptr()), plan.items.ctypes.data,
            plan.n_items, plan.slot_ptr.ctypes.data, plan.n_slots, plan.n_parts)
    tail = (vp(out.data_ptr()), vp(lse.data_ptr()), q.shape[0], q_len, w.Hq, w.Hkv, w.D, F.FAIRKV_BF16, F.FAIRKV_F32,
            float(w.scale), vp(torch.cuda.current_stream().cuda_stream))
    if static:
        rc = L.fairkv_decode_attn_static(*head, *tail)
    else:
        rc = L.fairkv_decode_attn_multi(*head, vp(workspace.data_ptr()), workspace.numel(), *tail)
    torch.cuda.synchronize()
    return rc


def test_static_workspace_entry_point_matches_the_one_with_a_callers_workspace():
    import paper_2502_15804_amd as F
    # first a full headline layer (every pair cut, 380 partial slots), then a smaller one with two new tokens per
    # sequence and a pair in more than 32 pieces (two-level merge): different sizes, different offsets in the array
    cases = [_case("llama70b", 16, 0), _case("mistral24b", 3, 1, q_len=2, min_chunk=32, overhead_tokens=0),
             _case("llama70b", 5, 2)]
    assert int(cases[1][6].items["n_chunks"].max()) >= 32
    for w, lens, off, q, k, v, plan in cases:
        qd, kd, vd = q.cuda(), k.cuda(), v.cuda()
        q_len = q.shape[1] if q.dim() == 4 else 1
        need = F.fairkv_workspace_bytes(plan.n_parts, lens.size, w.G * q_len, w.D)
        assert need <= F.FAIRKV_STATIC_WORKSPACE_BYTES
        ws = torch.zeros(need, dtype=torch.uint8, device="cuda")
        out_a = torch.full(tuple(q.shape), float("nan"), dtype=torch.float32, device="cuda")
        lse_a = torch.full(tuple(q.shape[:-1]), float("nan"), dtype=torch.float32, device="cuda")
        out_b, lse_b = out_a.clone(), lse_a.clone()
        assert _call(False, w, qd, kd, vd, plan, out_a, lse_a, ws) == F.FAIRKV_OK
        for rep in range(2):                       # twice: the second call finds what the first left in the array
            out_b.fill_(float("nan"))
            lse_b.fill_(float("nan"))
            assert _call(True, w, qd, kd, vd, plan, out_b, lse_b) == F.FAIRKV_OK
            assert torch.equal(out_a, out_b) and torch.equal(lse_a, lse_b), rep
        fn = OA.attention_multi if q_len > 1 else OA.attention
        ro, rl = fn(W.to_numpy_bits(q), W.to_numpy_bits(k), W.to_numpy_bits(v), off, lens, w.scale)
        got, gl = out_b.cpu().numpy().astype(np.float64), lse_b.cpu().numpy().astype(np.float64)
        assert np.abs(got - ro).max() <= w.tol
        fin = np.isfinite(rl)
        assert np.array_equal(np.isneginf(gl), ~fin) and np.abs(gl[fin] - rl[fin]).max() <= w.tol


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    import paper_2502_15804_amd as F
    w, lens, off, q, k, v, plan = _case("stress", 128, 0, n_slots=320, min_chunk=16, overhead_tokens=0, tile=16)
    big = W.Workload("big", 128, w.Hq, w.Hkv, w.D, w.dtype, 1, w.tol, "")
    need = F.fairkv_workspace_bytes(plan.n_parts, lens.size, w.G * 2, w.D)      # two new tokens: 16 columns
    assert need > F.FAIRKV_STATIC_WORKSPACE_BYTES
    q2 = torch.zeros((128, 2, w.Hq, w.D), dtype=torch.bfloat16, device="cuda")
    out = torch.full(tuple(q2.shape), 7.0, dtype=torch.float32, device="cuda")
    lse = torch.full(tuple(q2.shape[:-1]), 7.0, dtype=torch.float32, device="cuda")
    assert _call(True, big, q2, k.cuda(), v.cuda(), plan, out, lse) == F.FAIRKV_EWORKSPACE
    assert bool((out == 7.0).all()) and bool((lse == 7.0).all())               # refused: nothing was written
