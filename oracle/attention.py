"""fp64 attention oracle: ctypes front end of attn_ref.c plus the chunk-merge rule.

TEST INFRASTRUCTURE ONLY (see the package docstring).

`attention` is the definition itself (plain softmax(q K^T scale) V per
(sequence, query head) over that head's retained tokens; the paper's setting is
its Introduction and Section 3.2, the formula is the standard one).
`attention_chunk` and `merge_chunks` state the log-sum-exp combination of token
chunks, which is exact in real arithmetic:

    m* = max_c m_c,   l* = sum_c l_c e^{m_c - m*},
    out = sum_c acc_c e^{m_c - m*} / l*,   lse = m* + log l*.

The paper does not discuss it; it is how one head's tokens can be shared out
the way Fair-Copying shares a heavy head's load (Section 4.2).
"""
from __future__ import annotations

import ctypes
import math

import numpy as np

from . import build as _build

_DT = {np.dtype(np.uint16): 0, np.dtype(np.float32): 1, np.dtype(np.float64): 2}
_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(_build.build())
        lib.fairkv_oracle_attn.restype = ctypes.c_int
        lib.fairkv_oracle_attn.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int]
        lib.fairkv_oracle_attn_chunk.restype = ctypes.c_int
        lib.fairkv_oracle_attn_chunk.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64,
            ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.fairkv_oracle_max_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def max_threads() -> int:
    return int(_load().fairkv_oracle_max_threads())


def _check_inputs(q, k, v):
    q = np.ascontiguousarray(q)
    k = np.ascontiguousarray(k)
    v = np.ascontiguousarray(v)
    if not (q.dtype == k.dtype == v.dtype) or q.dtype not in _DT:
        raise TypeError("q, k, v must share a dtype: uint16 (bf16 bits), float32 or float64")
    return q, k, v, _DT[q.dtype]


def attention(q, k, v, off, lens, scale, sel=None, n_threads=0):
    """out [B,Hq,D] float64, lse [B,Hq] float64.

    q [B,Hq,D]; k, v [rows,D]; off (int64) and lens (int32) [B,Hkv].  bf16 data is
    passed as uint16 bit patterns.  `sel` restricts the work to the listed flat
    indices b*Hq+hq (other entries come back as NaN).
    """
    q, k, v, dt = _check_inputs(q, k, v)
    B, Hq, D = q.shape
    off = np.ascontiguousarray(off, dtype=np.int64)
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    Hkv = lens.shape[1]
    if off.shape != lens.shape or lens.shape[0] != B:
        raise ValueError("off/lens must be [B,Hkv]")
    live = lens > 0
    if live.any() and int((off + lens)[live].max()) > k.shape[0]:
        raise ValueError("a head's rows run past the end of K/V")
    if live.any() and int(off[live].min()) < 0:
        raise ValueError("negative offset")
    out = np.full((B, Hq, D), np.nan, dtype=np.float64)
    lse = np.full((B, Hq), np.nan, dtype=np.float64)
    if sel is not None:
        sel = np.ascontiguousarray(sel, dtype=np.int32)
        sel_p, n_sel = sel.ctypes.data, int(sel.size)
    else:
        sel_p, n_sel = None, 0
    rc = _load().fairkv_oracle_attn(
        q.ctypes.data, k.ctypes.data, v.ctypes.data, off.ctypes.data, lens.ctypes.data,
        B, Hq, Hkv, D, dt, float(scale), sel_p, n_sel, out.ctypes.data, lse.ctypes.data,
        int(n_threads))
    if rc != 0:
        raise ValueError("fairkv_oracle_attn rejected its arguments")
    return out, lse


def attention_multi(q, k, v, off, lens, scale, n_threads=0):
    """q [B,q_len,Hq,D]: q_len new tokens per sequence whose K/V are already the last q_len rows of
    every head; new token i sees rows [0, len - (q_len-1-i)).  out [B,q_len,Hq,D], lse [B,q_len,Hq]."""
    if q.ndim != 4:
        raise ValueError("q must be [B, q_len, Hq, D]")
    B, QL, Hq, D = q.shape
    q3, k, v, dt = _check_inputs(q.reshape(B * QL, Hq, D), k, v)
    off = np.ascontiguousarray(off, dtype=np.int64)
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    Hkv = lens.shape[1]
    if off.shape != lens.shape or lens.shape[0] != B:
        raise ValueError("off/lens must be [B,Hkv]")
    live = lens > 0
    if live.any() and (int((off + lens)[live].max()) > k.shape[0] or int(off[live].min()) < 0):
        raise ValueError("a head's rows lie outside K/V")
    out = np.full((B, QL, Hq, D), np.nan, dtype=np.float64)
    lse = np.full((B, QL, Hq), np.nan, dtype=np.float64)
    fn = _load().fairkv_oracle_attn_multi
    fn.restype = ctypes.c_int
    fn.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int] * 6 + [ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
                                                               ctypes.c_int]
    rc = fn(q3.ctypes.data, k.ctypes.data, v.ctypes.data, off.ctypes.data, lens.ctypes.data, B, QL, Hq, Hkv, D, dt,
            float(scale), out.ctypes.data, lse.ctypes.data, int(n_threads))
    if rc != 0:
        raise ValueError("fairkv_oracle_attn_multi rejected its arguments")
    return out, lse


def decode_e4m3fn(codes):
    """Values of 8-bit floats in the OCP E4M3 format ("FN": finite, no infinities), written out from the
    format's definition: 1 sign bit, 4 exponent bits with bias 7, 3 mantissa bits; exponent field 0 holds
    the subnormals m/8 * 2^-6; the all-ones code S.1111.111 is NaN; everything else is (1 + m/8) * 2^(e-7),
    up to 448.  codes: uint8 array; returns float64 of the same shape."""
    table = np.empty(256, dtype=np.float64)
    for c in range(256):
        sign = -1.0 if c & 0x80 else 1.0
        e, mant = (c >> 3) & 0xF, c & 0x7
        if e == 0xF and mant == 0x7:
            table[c] = np.nan
        elif e == 0:
            table[c] = sign * (mant / 8.0) * 2.0 ** -6
        else:
            table[c] = sign * (1.0 + mant / 8.0) * 2.0 ** (e - 7)
    codes = np.asarray(codes)
    if codes.dtype != np.uint8:
        raise TypeError("codes must be uint8")
    return table[codes]


def attention_kv8(q, k8, v8, off, lens, scale, k_scale, v_scale, n_threads=0):
    """The same attention over a cache stored as 8-bit floats (E4M3) with one scale factor for K and
    one for V (or one per KV head each, as sequences): K = k_scale * decode(k8), V = v_scale * decode(v8),
    everything else in fp64.
    q: bf16 bit patterns (uint16), [B,Hq,D] or [B,q_len,Hq,D]; k8, v8: uint8 [rows,D]."""
    q = np.ascontiguousarray(q)
    if q.dtype != np.uint16:
        raise TypeError("q must be bf16 bit patterns (uint16)")
    q64 = (q.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    k64 = decode_e4m3fn(k8)
    v64 = decode_e4m3fn(v8)
    if np.ndim(k_scale) == 0 and np.ndim(v_scale) == 0:
        k64 *= float(k_scale)
        v64 *= float(v_scale)
    else:                       # a scale per KV head: the rows of pair (b, h) carry the scales of head h
        lens_a, off_a = np.asarray(lens), np.asarray(off)
        ks = np.broadcast_to(np.asarray(k_scale, dtype=np.float64), (lens_a.shape[1],))
        vs = np.broadcast_to(np.asarray(v_scale, dtype=np.float64), (lens_a.shape[1],))
        for b in range(lens_a.shape[0]):
            for h in range(lens_a.shape[1]):
                r0, n = int(off_a[b, h]), int(lens_a[b, h])
                k64[r0:r0 + n] *= ks[h]
                v64[r0:r0 + n] *= vs[h]
    if q.ndim == 4:
        return attention_multi(q64, k64, v64, off, lens, scale, n_threads=n_threads)
    return attention(q64, k64, v64, off, lens, scale, n_threads=n_threads)


def attention_chunk(q, k, v, b, hq, row0, n, scale):
    """(m, l, acc[D]) of rows [row0, row0+n) of K/V for query q[b, hq]."""
    q, k, v, dt = _check_inputs(q, k, v)
    _, Hq, D = q.shape
    if row0 < 0 or row0 + n > k.shape[0]:
        raise ValueError("chunk rows out of range")
    m = ctypes.c_double()
    l = ctypes.c_double()
    acc = np.zeros(D, dtype=np.float64)
    rc = _load().fairkv_oracle_attn_chunk(
        q.ctypes.data, k.ctypes.data, v.ctypes.data, (b * Hq + hq) * D, int(row0), int(n),
        D, dt, float(scale), ctypes.byref(m), ctypes.byref(l), acc.ctypes.data)
    if rc != 0:
        raise ValueError("fairkv_oracle_attn_chunk rejected its arguments")
    return m.value, l.value, acc


def merge_chunks(parts):
    """Combine [(m, l, acc), ...] of disjoint token chunks of one head into (out, lse)."""
    parts = [p for p in parts if p[1] > 0.0]
    D = None
    for p in parts:
        D = len(p[2])
    if not parts:
        return None, -math.inf
    m_star = max(p[0] for p in parts)
    l_star = 0.0
    acc = np.zeros(D, dtype=np.float64)
    for m, l, a in parts:
        w = math.exp(m - m_star)
        l_star += l * w
        acc += np.asarray(a, dtype=np.float64) * w
    return acc / l_star, m_star + math.log(l_star)
