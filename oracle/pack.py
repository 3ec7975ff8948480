"""Oracle for building and growing the packed ragged KV cache.

TEST INFRASTRUCTURE ONLY (see the package docstring).

Per-head compression keeps, for every (sequence, KV head) pair, a subset of the tokens of the
dense cache (Section 2: the compressors "retain" or "select" entries per head; which ones is
their business, not this build's).  Packing is the plain definition: the kept tokens of pair
p = b*Hkv + h, in the order the keep list names them, become the rows off[p], off[p]+1, ... of
the packed K and V.  Appending is what a decode step does before it attends: the new token's
K and V rows go behind the pair's last row and its length grows by one, as long as the pair's
capacity allows.  Both are byte moves, so arrays are handled as raw storage (any dtype).
"""
from __future__ import annotations

import numpy as np


def pack(k_dense, v_dense, keep_ptr, keep_t, off, k_out, v_out):
    """k_dense, v_dense [B][Hkv][T][D]; keep_ptr [B*Hkv+1], keep_t [keep_ptr[-1]] (token index inside
    the pair's T), off [B*Hkv] first packed row of each pair; k_out, v_out [n_rows][D] are updated in
    place (rows that belong to no pair keep their content)."""
    B, Hkv, T, D = k_dense.shape
    for p in range(B * Hkv):
        b, h = divmod(p, Hkv)
        t = np.asarray(keep_t[int(keep_ptr[p]):int(keep_ptr[p + 1])], dtype=np.int64)
        if t.size and (t.min() < 0 or t.max() >= T):
            raise ValueError("token index outside the dense cache")
        r0 = int(off[p])
        k_out[r0:r0 + t.size] = k_dense[b, h, t]
        v_out[r0:r0 + t.size] = v_dense[b, h, t]


def append(k, v, k_new, v_new, off, lens, cap):
    """k, v [n_rows][D] packed; k_new, v_new [B][Hkv][D]; lens [B*Hkv] is updated in place.  A pair
    already at its capacity cap[p] is left alone; returns how many pairs that happened to."""
    B, Hkv, D = k_new.shape
    full = 0
    for p in range(B * Hkv):
        b, h = divmod(p, Hkv)
        if int(lens[p]) >= int(cap[p]):
            full += 1
            continue
        r = int(off[p]) + int(lens[p])
        k[r] = k_new[b, h]
        v[r] = v_new[b, h]
        lens[p] += 1
    return full
