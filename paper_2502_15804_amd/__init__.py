"""Thin Python binding of libfairkv.so (see include/fairkv.h for the contract).

The functions carry the names of the C entry points and only marshal arguments:
planning runs in the library's host code and attention runs in its HIP kernels.
PyTorch appears solely as the owner of device memory and streams.  There is no
fallback: if the shared library has not been built, importing a symbol raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfairkv.so")

FAIRKV_OK, FAIRKV_EINVAL, FAIRKV_ECAP, FAIRKV_EWORKSPACE, FAIRKV_EUNSUPPORTED, FAIRKV_EHIP = 0, -1, -2, -3, -4, -5
FAIRKV_BF16, FAIRKV_F32, FAIRKV_E4M3, FAIRKV_BF16_VALU = 0, 1, 2, 3
FAIRKV_TRACE_STAMPS = 16
FAIRKV_SHORT_PAIR_TOKENS = 96
FAIRKV_STATIC_WORKSPACE_BYTES = 8 << 20
FAIRKV_POLICY_NAIVE, FAIRKV_POLICY_LPT, FAIRKV_POLICY_LPT_SPLIT, FAIRKV_POLICY_FAIR = 0, 1, 2, 3

FAIRKV_PLACE_AUTO, FAIRKV_PLACE_EXACT, FAIRKV_PLACE_GREEDY = 0, 1, 2

EXPORTS = ("fairkv_default_params", "fairkv_plan", "fairkv_workspace_bytes", "fairkv_workspace_counter_bytes",
           "fairkv_decode_attn",
           "fairkv_decode_attn_multi", "fairkv_decode_attn_kv8", "fairkv_decode_attn_kv8_per_head",
           "fairkv_decode_attn_static", "fairkv_decode_attn_trace",
           "fairkv_place", "fairkv_pack", "fairkv_append", "fairkv_plan_grow", "fairkv_stream_probe", "fairkv_stream_probe_shape", "fairkv_workspace_reset",
           "fairkv_strerror", "fairkv_version")


class fairkv_item(ctypes.Structure):
    _fields_ = [("row", ctypes.c_int64)] + [(n, ctypes.c_int32) for n in
                                            ("tok_count", "b", "h", "chunk", "n_chunks", "part")]


class fairkv_plan_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_slots", "tile", "min_chunk", "max_split", "oversub", "overhead_tokens", "policy", "short_overhead_tokens")]


class fairkv_plan_summary(ctypes.Structure):
    _fields_ = [("total_tokens", ctypes.c_int64), ("max_slot_load", ctypes.c_int64),
                ("min_slot_load", ctypes.c_int64), ("n_items", ctypes.c_int32), ("n_parts", ctypes.c_int32)]


class fairkv_place_params(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("tp", "max_extra", "max_copies", "mode")]


class fairkv_share(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("head", "gpu", "copy", "n_copies", "row_begin", "row_end")]


class fairkv_place_summary(ctypes.Structure):
    _fields_ = [("den", ctypes.c_int64), ("delta_num", ctypes.c_int64), ("max_load_num", ctypes.c_int64),
                ("min_load_num", ctypes.c_int64), ("efficiency", ctypes.c_double), ("n_shares", ctypes.c_int32),
                ("exact", ctypes.c_int32)]


SHARE_DTYPE = np.dtype([(n, np.int32) for n, _ in fairkv_share._fields_])
assert SHARE_DTYPE.itemsize == ctypes.sizeof(fairkv_share) == 24

ITEM_DTYPE = np.dtype([("row", np.int64)] + [(n, np.int32) for n, _ in fairkv_item._fields_[1:]])
assert ITEM_DTYPE.itemsize == ctypes.sizeof(fairkv_item) == 32


class FairKVError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib() -> ctypes.CDLL:
    """The loaded shared library; raises if it was never built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              f"`python -m paper_2502_15804_amd.build` (there is no fallback path)")
        try:
            # PyTorch ships a HIP runtime of its own: load it first, so that this library binds to the same one
            # (two runtimes in one process do not share streams or code objects, and every launch would fail)
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p
        L.fairkv_default_params.restype = ctypes.c_int
        L.fairkv_default_params.argtypes = [ctypes.POINTER(fairkv_plan_params), i32]
        L.fairkv_plan.restype = ctypes.c_int
        L.fairkv_plan.argtypes = [vp, i64p, i32, i32, ctypes.POINTER(fairkv_plan_params), vp, i32, vp, vp,
                                  ctypes.POINTER(fairkv_plan_summary)]
        L.fairkv_workspace_counter_bytes.restype = ctypes.c_size_t
        L.fairkv_workspace_counter_bytes.argtypes = [i32]
        L.fairkv_workspace_bytes.restype = ctypes.c_size_t
        L.fairkv_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.fairkv_decode_attn.restype = ctypes.c_int
        L.fairkv_decode_attn.argtypes = [vp, vp, vp, ctypes.c_int64, vp, vp, i32, vp, i32, i32, vp, ctypes.c_size_t, vp,
                                         vp, i32, i32, i32, i32, i32, i32, ctypes.c_float, vp]
        L.fairkv_place.restype = ctypes.c_int
        L.fairkv_place.argtypes = [vp, i32, i32, ctypes.POINTER(fairkv_place_params), vp, i32, vp,
                                   ctypes.POINTER(fairkv_place_summary)]
        L.fairkv_pack.restype = ctypes.c_int
        L.fairkv_pack.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32, vp, vp, ctypes.c_int64, vp, vp]
        L.fairkv_append.restype = ctypes.c_int
        L.fairkv_append.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, vp, ctypes.c_int64, vp, vp]
        L.fairkv_plan_grow.restype = ctypes.c_int
        L.fairkv_plan_grow.argtypes = [vp, i32, i32, i32, vp, vp]
        L.fairkv_stream_probe.restype = ctypes.c_int
        L.fairkv_stream_probe.argtypes = [vp, vp, ctypes.c_int64, i32, vp, vp]
        L.fairkv_workspace_reset.restype = ctypes.c_int
        L.fairkv_workspace_reset.argtypes = [vp, ctypes.c_size_t, i32, vp]
        L.fairkv_stream_probe_shape.restype = ctypes.c_int
        L.fairkv_stream_probe_shape.argtypes = [vp, vp, ctypes.c_int64, i32, i32, i32, i32, vp, vp]
        L.fairkv_decode_attn_multi.restype = ctypes.c_int
        L.fairkv_decode_attn_multi.argtypes = [vp, vp, vp, ctypes.c_int64, vp, vp, i32, vp, i32, i32, vp,
                                               ctypes.c_size_t, vp, vp, i32, i32, i32, i32, i32, i32, i32,
                                               ctypes.c_float, vp]
        L.fairkv_decode_attn_kv8.restype = ctypes.c_int
        L.fairkv_decode_attn_kv8.argtypes = [vp, vp, vp, ctypes.c_int64, ctypes.c_float, ctypes.c_float, vp, vp, i32, vp,
                                             i32, i32, vp, ctypes.c_size_t, vp, vp, i32, i32, i32, i32, i32, i32,
                                             ctypes.c_float, vp]
        L.fairkv_decode_attn_kv8_per_head.restype = ctypes.c_int
        L.fairkv_decode_attn_kv8_per_head.argtypes = [vp, vp, vp, ctypes.c_int64, vp, vp, vp, vp, i32, vp,
                                                      i32, i32, vp, ctypes.c_size_t, vp, vp, i32, i32, i32, i32, i32, i32,
                                                      ctypes.c_float, vp]
        L.fairkv_decode_attn_static.restype = ctypes.c_int
        L.fairkv_decode_attn_static.argtypes = [vp, vp, vp, ctypes.c_int64, vp, vp, i32, vp, i32, i32, vp, vp,
                                                i32, i32, i32, i32, i32, i32, i32, ctypes.c_float, vp]
        L.fairkv_decode_attn_trace.restype = ctypes.c_int
        L.fairkv_decode_attn_trace.argtypes = [vp, vp, vp, ctypes.c_int64, vp, vp, i32, vp, i32, i32, vp, ctypes.c_size_t,
                                               vp, vp, i32, i32, i32, i32, ctypes.c_float, vp, ctypes.c_size_t, vp]
        L.fairkv_strerror.restype = ctypes.c_char_p
        L.fairkv_strerror.argtypes = [ctypes.c_int]
        L.fairkv_version.restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().fairkv_strerror(int(code)).decode()


def fairkv_version() -> int:
    return int(lib().fairkv_version())


def fairkv_default_params(n_compute_units: int, **overrides) -> fairkv_plan_params:
    p = fairkv_plan_params()
    rc = lib().fairkv_default_params(ctypes.byref(p), int(n_compute_units))
    if rc != FAIRKV_OK:
        raise FairKVError(rc, "fairkv_default_params")
    for k, v in overrides.items():
        if k not in dict(fairkv_plan_params._fields_):
            raise TypeError(f"unknown plan parameter {k!r}")
        setattr(p, k, int(v))
    return p


@dataclass
class Plan:
    """Host-side result of fairkv_plan (numpy arrays, ready to copy to the device)."""
    items: np.ndarray        # structured array of fairkv_item, grouped by slot
    slot_ptr: np.ndarray     # int32 [n_slots+1]
    part_base: np.ndarray    # int32 [B*Hkv+1]
    summary: fairkv_plan_summary
    params: fairkv_plan_params

    @property
    def n_items(self) -> int:
        return int(self.summary.n_items)

    @property
    def n_parts(self) -> int:
        return int(self.summary.n_parts)

    @property
    def n_slots(self) -> int:
        return int(self.params.n_slots)

    def slot_loads(self) -> np.ndarray:
        short = ((self.items["n_chunks"] == 1) & (self.items["tok_count"] <= FAIRKV_SHORT_PAIR_TOKENS)
                 & (int(self.params.short_overhead_tokens) > 0))
        cost = self.items["tok_count"].astype(np.int64) + np.where(short, int(self.params.short_overhead_tokens),
                                                                   int(self.params.overhead_tokens))
        csum = np.concatenate([[0], np.cumsum(cost)])
        return csum[self.slot_ptr[1:]] - csum[self.slot_ptr[:-1]]


def fairkv_plan(lens, off, B: int, Hkv: int, params: fairkv_plan_params) -> Plan:
    """Two calls into the library: one to size the work list, one to fill it."""
    lens = np.ascontiguousarray(np.asarray(lens).reshape(-1), dtype=np.int32)
    off = np.ascontiguousarray(np.asarray(off).reshape(-1), dtype=np.int64)
    if lens.size != int(B) * int(Hkv) or off.size != lens.size:
        raise ValueError("lens and off must have B*Hkv entries")
    L = lib()
    summary = fairkv_plan_summary()
    n_slots = max(int(params.n_slots), 0)
    slot_ptr = np.zeros(n_slots + 1, dtype=np.int32)
    part_base = np.zeros(int(B) * int(Hkv) + 1, dtype=np.int32)
    rc = L.fairkv_plan(lens.ctypes.data, off.ctypes.data, B, Hkv, ctypes.byref(params), None, 0,
                       slot_ptr.ctypes.data, part_base.ctypes.data, ctypes.byref(summary))
    if rc not in (FAIRKV_OK, FAIRKV_ECAP):
        raise FairKVError(rc, "fairkv_plan")
    items = np.zeros(int(summary.n_items), dtype=ITEM_DTYPE)
    if summary.n_items > 0:
        rc = L.fairkv_plan(lens.ctypes.data, off.ctypes.data, B, Hkv, ctypes.byref(params), items.ctypes.data,
                           items.size, slot_ptr.ctypes.data, part_base.ctypes.data, ctypes.byref(summary))
        if rc != FAIRKV_OK:
            raise FairKVError(rc, "fairkv_plan")
    return Plan(items, slot_ptr, part_base, summary, params)


@dataclass
class Placement:
    """Host-side result of fairkv_place."""
    shares: np.ndarray       # structured array of fairkv_share, ordered by (head, copy)
    gpu_load: np.ndarray     # int64 [tp], in units of 1/summary.den tokens
    summary: fairkv_place_summary
    params: fairkv_place_params


def fairkv_place(W, B: int, tp: int, max_extra: int = 0, max_copies: int = 1, mode: int = FAIRKV_PLACE_AUTO) -> Placement:
    W = np.ascontiguousarray(np.asarray(W).reshape(-1), dtype=np.int64)
    p = fairkv_place_params(int(tp), int(max_extra), int(max_copies), int(mode))
    s = fairkv_place_summary()
    shares = np.zeros(W.size + max(int(max_extra), 0), dtype=SHARE_DTYPE)
    load = np.zeros(max(int(tp), 1), dtype=np.int64)
    rc = lib().fairkv_place(W.ctypes.data, W.size, int(B), ctypes.byref(p), shares.ctypes.data, shares.size,
                            load.ctypes.data, ctypes.byref(s))
    if rc != FAIRKV_OK:
        raise FairKVError(rc, "fairkv_place")
    return Placement(shares[:s.n_shares].copy(), load, s, p)


def fairkv_workspace_counter_bytes(n_pairs: int) -> int:
    return int(lib().fairkv_workspace_counter_bytes(int(n_pairs)))


def fairkv_workspace_bytes(n_parts: int, n_pairs: int, G: int, D: int) -> int:
    return int(lib().fairkv_workspace_bytes(int(n_parts), int(n_pairs), int(G), int(D)))


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def fairkv_decode_attn(q, k, v, items, items_host, slot_ptr, n_parts, workspace, out, lse, scale, Hkv, stream=None,
                       bf16_on_valu=False, trace=None):
    """Enqueue decode attention for one layer on `stream` (default: torch's current stream).

    workspace=None calls fairkv_decode_attn_static (the library's own workspace); trace (a zero-filled int64 device
    tensor of n_slots * FAIRKV_TRACE_STAMPS) calls fairkv_decode_attn_trace; bf16_on_valu passes FAIRKV_BF16_VALU.

    Tensor arguments are CUDA/HIP torch tensors owned by the caller: q [B,Hq,D], or [B,q_len,Hq,D] for
    several new tokens per sequence (fairkv_decode_attn_multi; out and lse then carry q_len too); k, v [rows,D];
    items: uint8 view of the plan's item array (n_items * 32 bytes); workspace uint8, zero-filled
    before its first use; out [B,Hq,D] float32 or bfloat16; lse float32 [B,Hq] or None.
    items_host and slot_ptr are the plan's HOST arrays (numpy: fairkv_item records, int32
    [n_slots+1]).  Nothing is allocated or synchronised here.
    """
    import torch

    if q.dim() == 4:
        B, q_len, Hq, D = q.shape
    else:
        (B, Hq, D), q_len = q.shape, 1
    dt = {torch.bfloat16: FAIRKV_BF16, torch.float32: FAIRKV_F32}
    if q.dtype not in dt or k.dtype != q.dtype or v.dtype != q.dtype or out.dtype not in dt:
        raise TypeError("q/k/v must share bf16 or fp32; out must be bf16 or fp32")
    for name, t in (("q", q), ("k", k), ("v", v), ("items", items), ("workspace", workspace), ("out", out),
                    ("lse", lse), ("trace", trace)):
        if t is None:
            continue
        if not t.is_cuda or not t.is_contiguous():
            raise ValueError(f"{name} must be a contiguous device tensor")
    if not isinstance(slot_ptr, np.ndarray) or slot_ptr.dtype != np.int32 or not slot_ptr.flags.c_contiguous:
        raise TypeError("slot_ptr must be a contiguous host int32 array")
    if lse is not None and lse.dtype != torch.float32:
        raise TypeError("lse must be float32")
    if k.shape[1] != D or v.shape != k.shape or tuple(out.shape) != tuple(q.shape) or slot_ptr.size < 2:
        raise ValueError("shape mismatch")
    if lse is not None and tuple(lse.shape) != tuple(q.shape[:-1]):
        raise ValueError("lse must have q's shape without the last dimension")
    item_bytes = items.numel() * items.element_size()
    if item_bytes % 32 != 0:
        raise ValueError("items must be a whole number of 32-byte records")
    if (not isinstance(items_host, np.ndarray) or items_host.dtype != ITEM_DTYPE or not items_host.flags.c_contiguous
            or items_host.size * 32 != item_bytes):
        raise TypeError("items_host must be the plan's contiguous item array, as many records as `items`")
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    in_dt = FAIRKV_BF16_VALU if (bf16_on_valu and q.dtype == torch.bfloat16) else dt[q.dtype]
    head = (_ptr(q), _ptr(k), _ptr(v), k.shape[0], _ptr(items), items_host.ctypes.data, item_bytes // 32,
            slot_ptr.ctypes.data, slot_ptr.size - 1, int(n_parts))
    st = ctypes.c_void_p(stream.cuda_stream)
    if trace is not None:
        if q_len != 1 or workspace is None or trace.dtype != torch.int64:
            raise ValueError("a traced call is a single-token call with a caller's workspace and an int64 trace buffer")
        name = "fairkv_decode_attn_trace"
        rc = lib().fairkv_decode_attn_trace(*head, _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(out),
                                            _ptr(lse), B, Hq, Hkv, D, float(scale), _ptr(trace), trace.numel() * 8, st)
    elif workspace is None:
        name = "fairkv_decode_attn_static"
        rc = lib().fairkv_decode_attn_static(*head, _ptr(out), _ptr(lse), B, q_len, Hq, Hkv, D, in_dt, dt[out.dtype],
                                             float(scale), st)
    else:
        name = "fairkv_decode_attn_multi" if q_len > 1 else "fairkv_decode_attn"
        rc = lib().fairkv_decode_attn_multi(*head, _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(out),
                                            _ptr(lse), B, q_len, Hq, Hkv, D, in_dt, dt[out.dtype], float(scale), st)
    if rc != FAIRKV_OK:
        raise FairKVError(rc, name)


def fairkv_decode_attn_kv8(q, k8, v8, k_scale, v_scale, items, items_host, slot_ptr, n_parts, workspace, out, lse,
                           scale, Hkv, stream=None):
    """fairkv_decode_attn over a cache stored as 8-bit floats (E4M3, finite-only "fn" encoding).

    k8, v8 [rows,D]: torch.float8_e4m3fn or uint8 holding the same bytes; a stored byte stands for
    value * k_scale (v_scale).  k_scale and v_scale are two numbers, or two sequences of Hkv numbers (a scale
    per KV head: fairkv_decode_attn_kv8_per_head).  q [B,Hq,D] or [B,q_len,Hq,D] bfloat16.  Everything else as in
    fairkv_decode_attn.
    """
    import torch

    if q.dim() == 4:
        B, q_len, Hq, D = q.shape
    else:
        (B, Hq, D), q_len = q.shape, 1
    dt = {torch.bfloat16: FAIRKV_BF16, torch.float32: FAIRKV_F32}
    bytes_ok = (torch.uint8, torch.float8_e4m3fn)
    if q.dtype != torch.bfloat16 or k8.dtype not in bytes_ok or v8.dtype not in bytes_ok or out.dtype not in dt:
        raise TypeError("q must be bf16, k8/v8 float8_e4m3fn or uint8, out bf16 or fp32")
    _check_dev(q=q, k8=k8, v8=v8, items=items, workspace=workspace, out=out, lse=lse)
    if not isinstance(slot_ptr, np.ndarray) or slot_ptr.dtype != np.int32 or not slot_ptr.flags.c_contiguous:
        raise TypeError("slot_ptr must be a contiguous host int32 array")
    if lse is not None and lse.dtype != torch.float32:
        raise TypeError("lse must be float32")
    if k8.dim() != 2 or k8.shape[1] != D or v8.shape != k8.shape or tuple(out.shape) != tuple(q.shape) or slot_ptr.size < 2:
        raise ValueError("shape mismatch")
    if lse is not None and tuple(lse.shape) != tuple(q.shape[:-1]):
        raise ValueError("lse must have q's shape without the last dimension")
    item_bytes = items.numel() * items.element_size()
    if item_bytes % 32 != 0:
        raise ValueError("items must be a whole number of 32-byte records")
    if (not isinstance(items_host, np.ndarray) or items_host.dtype != ITEM_DTYPE or not items_host.flags.c_contiguous
            or items_host.size * 32 != item_bytes):
        raise TypeError("items_host must be the plan's contiguous item array, as many records as `items`")
    if stream is None:
        stream = torch.cuda.current_stream(q.device)
    tail = (_ptr(items), items_host.ctypes.data, item_bytes // 32, slot_ptr.ctypes.data, slot_ptr.size - 1, int(n_parts),
            _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(out), _ptr(lse), B, q_len, Hq, Hkv, D,
            dt[out.dtype], float(scale), ctypes.c_void_p(stream.cuda_stream))
    if np.ndim(k_scale) or np.ndim(v_scale):
        ks = np.ascontiguousarray(np.broadcast_to(np.asarray(k_scale, dtype=np.float32), (Hkv,)))
        vs = np.ascontiguousarray(np.broadcast_to(np.asarray(v_scale, dtype=np.float32), (Hkv,)))
        rc = lib().fairkv_decode_attn_kv8_per_head(_ptr(q), _ptr(k8), _ptr(v8), k8.shape[0], ks.ctypes.data, vs.ctypes.data,
                                                   *tail)
        name = "fairkv_decode_attn_kv8_per_head"
    else:
        rc = lib().fairkv_decode_attn_kv8(_ptr(q), _ptr(k8), _ptr(v8), k8.shape[0], float(k_scale), float(v_scale), *tail)
        name = "fairkv_decode_attn_kv8"
    if rc != FAIRKV_OK:
        raise FairKVError(rc, name)


def _dtype_code(t):
    import torch
    return {torch.bfloat16: FAIRKV_BF16, torch.float32: FAIRKV_F32, torch.uint8: FAIRKV_E4M3,
            torch.float8_e4m3fn: FAIRKV_E4M3}[t.dtype]


def _check_dev(**tensors):
    for name, t in tensors.items():
        if t is not None and (not t.is_cuda or not t.is_contiguous()):
            raise ValueError(f"{name} must be a contiguous device tensor")


def fairkv_pack(k_dense, v_dense, keep_ptr, keep_t, off, items, slot_ptr, k_out, v_out, bad=None, stream=None):
    """Enqueue the gather of the kept rows.  All arguments are device tensors: k_dense, v_dense
    [B][Hkv][T][D]; keep_ptr int64 [B*Hkv+1]; keep_t int32; off int64 [B*Hkv]; items uint8 view of a
    plan's item array; slot_ptr int32 [n_slots+1]; k_out, v_out [n_rows][D]; bad int32 [1] or None."""
    import torch

    B, Hkv, T, D = k_dense.shape
    _check_dev(k_dense=k_dense, v_dense=v_dense, keep_ptr=keep_ptr, keep_t=keep_t, off=off, items=items,
               slot_ptr=slot_ptr, k_out=k_out, v_out=v_out, bad=bad)
    if (v_dense.shape != k_dense.shape or k_out.shape != v_out.shape or k_out.shape[1] != D
            or k_out.dtype != k_dense.dtype or v_out.dtype != k_dense.dtype or v_dense.dtype != k_dense.dtype):
        raise ValueError("shape or dtype mismatch")
    if (keep_ptr.dtype != torch.int64 or off.dtype != torch.int64 or keep_t.dtype != torch.int32
            or slot_ptr.dtype != torch.int32 or keep_ptr.numel() != B * Hkv + 1 or off.numel() != B * Hkv
            or (bad is not None and bad.dtype != torch.int32)):
        raise TypeError("keep_ptr/off must be int64, keep_t/slot_ptr/bad int32, sized for B*Hkv pairs")
    if stream is None:
        stream = torch.cuda.current_stream(k_dense.device)
    rc = lib().fairkv_pack(_ptr(k_dense), _ptr(v_dense), B, Hkv, T, D, _dtype_code(k_dense), _ptr(keep_ptr),
                           _ptr(keep_t), _ptr(off), _ptr(items), _ptr(slot_ptr), slot_ptr.numel() - 1, _ptr(k_out),
                           _ptr(v_out), k_out.shape[0], _ptr(bad), ctypes.c_void_p(stream.cuda_stream))
    if rc != FAIRKV_OK:
        raise FairKVError(rc, "fairkv_pack")


def fairkv_append(k_new, v_new, off, lens, cap, k, v, full=None, stream=None):
    """Enqueue the append of one new row per pair.  Device tensors: k_new, v_new [B][Hkv][D]; off int64,
    lens int32 (updated in place), cap int32, all [B*Hkv]; k, v packed [n_rows][D]; full int32 [1] or None."""
    import torch

    B, Hkv, D = k_new.shape
    _check_dev(k_new=k_new, v_new=v_new, off=off, lens=lens, cap=cap, k=k, v=v, full=full)
    if (v_new.shape != k_new.shape or k.shape != v.shape or k.shape[1] != D or k.dtype != k_new.dtype
            or v.dtype != k_new.dtype or v_new.dtype != k_new.dtype):
        raise ValueError("shape or dtype mismatch")
    if (off.dtype != torch.int64 or lens.dtype != torch.int32 or cap.dtype != torch.int32
            or off.numel() != B * Hkv or lens.numel() != B * Hkv or cap.numel() != B * Hkv
            or (full is not None and full.dtype != torch.int32)):
        raise TypeError("off must be int64, lens/cap/full int32, sized for B*Hkv pairs")
    if stream is None:
        stream = torch.cuda.current_stream(k_new.device)
    rc = lib().fairkv_append(_ptr(k_new), _ptr(v_new), B, Hkv, D, _dtype_code(k_new), _ptr(off), _ptr(lens), _ptr(cap),
                             _ptr(k), _ptr(v), k.shape[0], _ptr(full), ctypes.c_void_p(stream.cuda_stream))
    if rc != FAIRKV_OK:
        raise FairKVError(rc, "fairkv_append")


def fairkv_plan_grow(items: np.ndarray, B: int, Hkv: int, lens: np.ndarray, cap: np.ndarray) -> None:
    """Host arrays, updated in place: items (a whole plan, ITEM_DTYPE), lens int32 [B*Hkv]; cap int32 [B*Hkv]."""
    if items.dtype != ITEM_DTYPE or not items.flags.c_contiguous:
        raise TypeError("items must be a contiguous fairkv_item array")
    if lens.dtype != np.int32 or cap.dtype != np.int32 or not lens.flags.c_contiguous or not cap.flags.c_contiguous:
        raise TypeError("lens and cap must be contiguous int32 arrays")
    if lens.size != B * Hkv or cap.size != B * Hkv:
        raise ValueError("lens and cap must have B*Hkv entries")
    rc = lib().fairkv_plan_grow(items.ctypes.data, items.size, int(B), int(Hkv), lens.ctypes.data, cap.ctypes.data)
    if rc != FAIRKV_OK:
        raise FairKVError(rc, "fairkv_plan_grow")


def fairkv_workspace_reset(workspace, n_pairs, stream=None):
    """Enqueue the kernel that zeroes the counter bytes of a device workspace (see the header)."""
    import torch

    _check_dev(workspace=workspace)
    if stream is None:
        stream = torch.cuda.current_stream(workspace.device)
    rc = lib().fairkv_workspace_reset(_ptr(workspace), workspace.numel() * workspace.element_size(), int(n_pairs),
                                      ctypes.c_void_p(stream.cuda_stream))
    if rc != FAIRKV_OK:
        raise FairKVError(rc, "fairkv_workspace_reset")


def fairkv_stream_probe(k, v, n_workgroups, sink, stream=None, shape=None):
    """Enqueue the do-nothing reader over all of the device tensors k and v (see the header).
    shape: (waves, stages, tile_kib) for fairkv_stream_probe_shape; None = the decode kernel's shape."""
    import torch

    _check_dev(k=k, v=v, sink=sink)
    if sink.numel() * sink.element_size() < 4 * n_workgroups:
        raise ValueError("sink too small")
    if stream is None:
        stream = torch.cuda.current_stream(k.device)
    nbytes = min(k.numel() * k.element_size(), v.numel() * v.element_size())
    if shape is not None:
        rc = lib().fairkv_stream_probe_shape(_ptr(k), _ptr(v), nbytes, int(n_workgroups), int(shape[0]), int(shape[1]),
                                             int(shape[2]), _ptr(sink), ctypes.c_void_p(stream.cuda_stream))
    else:
        rc = lib().fairkv_stream_probe(_ptr(k), _ptr(v), nbytes, int(n_workgroups), _ptr(sink),
                                       ctypes.c_void_p(stream.cuda_stream))
    if rc != FAIRKV_OK:
        raise FairKVError(rc, "fairkv_stream_probe")
