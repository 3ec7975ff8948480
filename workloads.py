"""Seeded synthetic inputs for ragged per-head decode attention.

This module only *draws inputs*: per-(sequence, KV head) retained-token counts
with the heavy-tailed shapes that per-head KV-cache compressors produce (the
paper's Section 3.1 observation that budgets differ strongly per head), the
packed row offsets that go with them, and random Q/K/V.  It holds none of the
method's arithmetic (no attention, no planning), so both the CPU oracle's tests
and the GPU path's tests may use it to obtain identical bits.

The per-head budget profiles the paper measured (Ada-SnapKV on LongBench v1)
are not available; the distributions below stand in for them.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np

_MASK64 = (1 << 64) - 1


# --------------------------------------------------------------------------
# counter-based generator: splitmix64 finaliser over (key + counter * golden)
# --------------------------------------------------------------------------
def _mix64(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.uint64, copy=True)
    with np.errstate(over="ignore"):
        x ^= x >> np.uint64(30)
        x *= np.uint64(0xBF58476D1CE4E5B9)
        x ^= x >> np.uint64(27)
        x *= np.uint64(0x94D049BB133111EB)
        x ^= x >> np.uint64(31)
    return x


def _key(seed: int, stream: int) -> int:
    k = (seed * 0x9E3779B97F4A7C15 + stream * 0xD1B54A32D192ED03 + 0x2545F4914F6CDD1D) & _MASK64
    return int(_mix64(np.array([k], dtype=np.uint64))[0])


def uniform01(seed: int, stream: int, n: int) -> np.ndarray:
    """n doubles in the open interval (0, 1); element i depends only on (seed, stream, i)."""
    ctr = np.arange(1, n + 1, dtype=np.uint64)
    with np.errstate(over="ignore"):
        x = np.uint64(_key(seed, stream)) + ctr * np.uint64(0x9E3779B97F4A7C15)
    bits = _mix64(x) >> np.uint64(11)
    return (bits.astype(np.float64) + 0.5) / float(1 << 53)


def normal01(seed: int, stream: int, n: int) -> np.ndarray:
    """n standard normals (Box-Muller, cosine branch) from two uniform streams."""
    u1 = uniform01(seed, 2 * stream, n)
    u2 = uniform01(seed, 2 * stream + 1, n)
    return np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)


# --------------------------------------------------------------------------
# workload table
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    B: int
    Hq: int
    Hkv: int
    D: int
    dtype: str          # "bf16" or "f32": storage type of q, K, V
    n_layers: int       # distinct layer buffers the workload defines
    tol: float          # max-abs-error bar against the fp64 oracle
    description: str

    @property
    def G(self) -> int:
        return self.Hq // self.Hkv

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)

    @property
    def elem_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4


WORKLOADS = {
    "tiny": Workload("tiny", 2, 8, 4, 64, "f32", 1, 1e-5,
                     "B=2, 4 KV heads x 2 query heads, D=64, fp32; len uniform in 1..128"),
    "llama70b": Workload("llama70b", 16, 64, 8, 128, "bf16", 32, 1e-2,
                         "Llama-70B-shaped layer: 64 q / 8 KV heads, D=128, bf16, B=16; "
                         "lognormal budgets mean 1024, sigma 0.6, clip 16..8192"),
    "mistral24b": Workload("mistral24b", 32, 32, 8, 128, "bf16", 8, 1e-2,
                           "Mistral-24B-shaped layer: 32 q / 8 KV heads, D=128, bf16, B=32; "
                           "KV heads 2 and 5 heavy (mean 4096), others mean 512, clip 16..16384"),
    "faircopy": Workload("faircopy", 64, 16, 2, 128, "bf16", 8, 1e-2,
                         "one GPU's Fair-Copying share: full head (B=64, mean 2048) + replicated "
                         "heavy head serving rows 32-63 only (mean 6144), clip 16..32768"),
    "stress": Workload("stress", 128, 64, 8, 128, "bf16", 80, 1e-2,
                       "Llama-70B shape, B=128, 80 layers; Pareto(alpha 1.2, min 32) clip 32768"),
}


def _lognormal(seed, stream, n, mean, sigma, lo, hi):
    z = normal01(seed, stream, n)
    mu = math.log(mean) - 0.5 * sigma * sigma
    x = np.rint(np.exp(mu + sigma * z))
    return np.clip(x, lo, hi).astype(np.int32)


def lens(name: str, seed: int = 0, layer: int = 0) -> np.ndarray:
    """Retained-token counts len[b][h] (int32, shape [B, Hkv]) of one layer of a workload."""
    w = WORKLOADS[name]
    n = w.B * w.Hkv
    stream = 1000 * layer
    if name == "tiny":
        u = uniform01(seed, stream, n)
        out = 1 + np.floor(u * 128.0).astype(np.int32)
    elif name == "llama70b":
        out = _lognormal(seed, stream, n, 1024.0, 0.6, 16, 8192)
    elif name == "mistral24b":
        light = _lognormal(seed, stream, n, 512.0, 0.6, 16, 16384).reshape(w.B, w.Hkv)
        heavy = _lognormal(seed, stream + 1, n, 4096.0, 0.6, 16, 16384).reshape(w.B, w.Hkv)
        out = light.copy()
        for h in (2, 5):
            out[:, h] = heavy[:, h]
    elif name == "faircopy":
        full = _lognormal(seed, stream, n, 2048.0, 0.6, 16, 32768).reshape(w.B, w.Hkv)
        copy = _lognormal(seed, stream + 1, n, 6144.0, 0.6, 16, 32768).reshape(w.B, w.Hkv)
        out = full.copy()
        out[:, 1] = copy[:, 1]
        out[: w.B // 2, 1] = 0          # the replica serves only the upper half of the batch
    elif name == "stress":
        u = uniform01(seed, stream, n)
        x = np.floor(32.0 * np.power(u, -1.0 / 1.2))
        out = np.clip(x, 32, 32768).astype(np.int32)
    else:
        raise KeyError(name)
    return np.ascontiguousarray(out.reshape(w.B, w.Hkv), dtype=np.int32)


def packed_offsets(len_bh: np.ndarray, gap_rows: int = 0):
    """Row offsets of a dense (b, h)-ordered packing: off[b][h] (int64) and total rows."""
    flat = len_bh.reshape(-1).astype(np.int64)
    step = flat + gap_rows
    off = np.concatenate([[0], np.cumsum(step)[:-1]]).astype(np.int64)
    total = int(step.sum())
    return off.reshape(len_bh.shape), total


def algorithmic_bytes(w: Workload, len_bh: np.ndarray) -> int:
    """K and V rows read once, q read once, fp32 out written once."""
    n_tok = int(len_bh.astype(np.int64).sum())
    return 2 * n_tok * w.D * w.elem_bytes + w.B * w.Hq * w.D * w.elem_bytes + w.B * w.Hq * w.D * 4


def make_qkv(w: Workload, n_rows: int, seed: int = 0, layer: int = 0, device: str = "cpu"):
    """q [B,Hq,D], K [n_rows,D], V [n_rows,D] ~ N(0,1), rounded once to the storage type.

    Drawn by a seeded torch generator on `device`; a given (seed, layer, device type)
    always yields the same bits.  Callers that need the same bits on host and device
    draw on one side and copy.
    """
    import torch

    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + layer * 7919 + 12345) & 0x7FFFFFFF)
    dt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    rows = max(n_rows, 1)
    q = torch.randn((w.B, w.Hq, w.D), generator=g, device=device, dtype=torch.float32).to(dt)
    k = torch.randn((rows, w.D), generator=g, device=device, dtype=torch.float32).to(dt)
    v = torch.randn((rows, w.D), generator=g, device=device, dtype=torch.float32).to(dt)
    return q, k, v


def make_kv8(w: Workload, n_rows: int, k_scale: float, v_scale: float, seed: int = 0, layer: int = 0,
             device: str = "cpu"):
    """The K and V of make_qkv stored as 8-bit floats (E4M3, finite-only encoding): uint8 [n_rows,D] each.

    A stored byte stands for value / scale, clamped to the format's largest finite magnitude (448) and
    rounded by torch's own conversion; this only manufactures input bytes, what they mean is for the
    oracle and the kernel to decode, each on its own.
    """
    import torch

    _, k, v = make_qkv(w, n_rows, seed=seed, layer=layer, device=device)
    k8 = (k.float() / k_scale).clamp(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
    v8 = (v.float() / v_scale).clamp(-448.0, 448.0).to(torch.float8_e4m3fn).view(torch.uint8)
    return k8, v8


def to_numpy_bits(t):
    """torch tensor -> numpy array the oracle accepts (bf16 as uint16 bit patterns)."""
    import torch

    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def keep_lists(len_bh: np.ndarray, T: int, seed: int = 0, recent: int = 32):
    """Which tokens of a dense cache of T tokens every pair keeps: (keep_ptr int64 [n_pairs+1],
    keep_t int32 [total]), ascending inside a pair.  Shaped like the output of a per-head
    compressor: the most recent `recent` tokens are always kept, the rest of the budget is
    scattered over the earlier positions.  Selection itself is not part of this build."""
    flat = np.asarray(len_bh).reshape(-1).astype(np.int64)
    if flat.size and flat.max() > T:
        raise ValueError("a pair cannot keep more tokens than the dense cache has")
    keep_ptr = np.concatenate([[0], np.cumsum(flat)]).astype(np.int64)
    keep_t = np.empty(int(keep_ptr[-1]), dtype=np.int32)
    rng = np.random.default_rng([seed, 0x6b656570])
    for p, n in enumerate(flat):
        n = int(n)
        tail = min(n, recent)
        old = rng.choice(T - tail, size=n - tail, replace=False) if n > tail else np.empty(0, np.int64)
        keep_t[keep_ptr[p]:keep_ptr[p + 1]] = np.concatenate([np.sort(old), np.arange(T - tail, T)]).astype(np.int32)
    return keep_ptr, keep_t
