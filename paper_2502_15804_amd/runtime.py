"""Device-side plumbing around the C ABI: keeps one layer's tensors and plan resident.

Nothing here computes: it allocates torch tensors, copies the host plan to the device
once, and forwards to fairkv_decode_attn.  Budgets are static after compression (the
paper's scheme is a static, load-aware one: Section 4.1), so a layer is planned once
and the plan is reused for every decode step.
"""
from __future__ import annotations

import numpy as np

from . import (Plan, fairkv_decode_attn, fairkv_decode_attn_kv8, fairkv_default_params, fairkv_plan,
               fairkv_workspace_bytes)


def device_compute_units(device=None) -> int:
    import torch
    return int(torch.cuda.get_device_properties(device if device is not None else torch.cuda.current_device())
               .multi_processor_count)


class DecodeLayer:
    """One layer's packed ragged KV cache, its plan and its output buffers on the GPU."""

    def __init__(self, q, k, v, off, lens, scale, params=None, out_dtype=None, want_lse=True,
                 workspace=None, k_scale=1.0, v_scale=1.0, static_workspace=False, bf16_on_valu=False):
        import torch

        dev = q.device
        self.q, self.k, self.v = q, k, v
        self.kv8 = k.dtype in (torch.uint8, torch.float8_e4m3fn)   # a cache of 8-bit floats, one scale per tensor
        self.k_scale = k_scale if np.ndim(k_scale) else float(k_scale)     # a number, or one per KV head
        self.v_scale = v_scale if np.ndim(v_scale) else float(v_scale)
        self.q_len = q.shape[1] if q.dim() == 4 else 1     # several new tokens per sequence: q [B,q_len,Hq,D]
        self.B, self.Hq, self.D = q.shape[0], q.shape[-2], q.shape[-1]
        lens_h = np.ascontiguousarray(np.asarray(lens, dtype=np.int32))
        off_h = np.ascontiguousarray(np.asarray(off, dtype=np.int64))
        self.Hkv = lens_h.shape[1]
        self.G = self.Hq // self.Hkv
        self.scale = float(scale)
        if params is None:
            # 8-bit caches: a step covers 32 tokens and a token costs half the bytes, so the per-item
            # overhead is worth twice as many tokens
            extra = {"tile": 32, "min_chunk": 64, "overhead_tokens": 256} if self.kv8 else {}
            params = fairkv_default_params(device_compute_units(dev), **extra)
        self.plan: Plan = fairkv_plan(lens_h, off_h, self.B, self.Hkv, params)
        self.items_d = torch.from_numpy(self.plan.items.view(np.uint8).copy()).to(dev)
        need = fairkv_workspace_bytes(self.plan.n_parts, self.B * self.Hkv, self.G * self.q_len, self.D)
        self.bf16_on_valu = bf16_on_valu
        if static_workspace:
            workspace = None                                               # the library's own (fairkv_decode_attn_static)
        elif workspace is None:
            workspace = torch.zeros(need, dtype=torch.uint8, device=dev)   # arrival counters start at zero
        elif workspace.numel() < need:
            raise ValueError("shared workspace too small for this layer")
        self.workspace = workspace
        self.out = torch.empty(tuple(q.shape), dtype=out_dtype or torch.float32, device=dev)
        self.lse = torch.empty(tuple(q.shape[:-1]), dtype=torch.float32, device=dev) if want_lse else None

    def run(self, stream=None, trace=None):
        if self.kv8:
            fairkv_decode_attn_kv8(self.q, self.k, self.v, self.k_scale, self.v_scale, self.items_d, self.plan.items,
                                   self.plan.slot_ptr, self.plan.n_parts, self.workspace, self.out, self.lse,
                                   self.scale, self.Hkv, stream)
            return self.out, self.lse
        fairkv_decode_attn(self.q, self.k, self.v, self.items_d, self.plan.items, self.plan.slot_ptr, self.plan.n_parts,
                           self.workspace, self.out, self.lse, self.scale, self.Hkv, stream,
                           bf16_on_valu=self.bf16_on_valu, trace=trace)
        return self.out, self.lse


def gpu_share(lens, shares, gpu):
    """One GPU's part of a placement made by fairkv_place: (heads, len_local).

    heads      the KV heads this GPU holds, ascending
    len_local  int32 [B][len(heads)]: len[b][head] for the batch rows this GPU serves of that
               head, 0 for the rows another copy serves (such pairs get empty items, no K/V).
    The GPU then runs fairkv_plan + fairkv_decode_attn on len_local like on any other cache.
    """
    lens = np.asarray(lens)
    mine = [s for s in shares if int(s["gpu"]) == int(gpu)]
    heads = sorted(int(s["head"]) for s in mine)
    out = np.zeros((lens.shape[0], len(heads)), dtype=np.int32)
    for s in mine:
        col = heads.index(int(s["head"]))
        out[int(s["row_begin"]):int(s["row_end"]), col] = lens[int(s["row_begin"]):int(s["row_end"]), int(s["head"])]
    return heads, out
