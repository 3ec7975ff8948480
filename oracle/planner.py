"""Oracle work planner: integer-only, step by step, for bit-exact comparison.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper balances heads of unequal KV-cache size over GPUs: its objective is to
minimise the largest per-device load (Appendix A, eq. 4), a replicated head
carries weight W/copies on each replica (Algorithm 2, the adjusted weights
W_A), replication is capped (eq. 3), every head must be placed (eq. 2), and a
scheme is judged by max-minus-min group weight (Algorithm 2) and by the
efficiency E = mean load / max load (eq. 5).  Its own search (Algorithms 1 and
2) is exhaustive and meant for a handful of heads and GPUs.  On one GPU the
"devices" are workgroup slots on compute units and the "heads" are hundreds of
(sequence, KV head) pairs, so the same objective is pursued greedily:

  * Fair-Copying becomes an equal split of a heavy pair's tokens into r chunks
    (each carries len/r, the W/copies rule), r capped by max_split (eq. 3);
  * Best-effort Assignment becomes longest-processing-time-first list
    scheduling of the chunks over n_slots.

Several plans can be equally good in the paper's sense; the order and
tie-breaks below are fixed only so that two implementations can be compared
field by field.  All arithmetic is on Python ints.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

POLICY_NAIVE = 0      # one work item per pair, dealt round-robin (static head allocation)
POLICY_LPT = 1        # load-aware assignment, no splitting (Best-effort Assignment only)
POLICY_LPT_SPLIT = 2  # load-aware assignment of equally split pairs (with Fair-Copying)


@dataclass(frozen=True)
class Params:
    n_slots: int = 512
    tile: int = 64
    min_chunk: int = 256
    max_split: int = 128
    oversub: int = 2
    overhead_tokens: int = 64
    policy: int = POLICY_LPT_SPLIT


@dataclass(frozen=True)
class Item:
    b: int
    h: int
    tok_begin: int
    tok_count: int
    chunk: int
    n_chunks: int
    slot: int
    part: int

    def astuple(self) -> Tuple[int, ...]:
        return (self.b, self.h, self.tok_begin, self.tok_count, self.chunk, self.n_chunks,
                self.slot, self.part)


@dataclass(frozen=True)
class Summary:
    total_tokens: int
    max_slot_load: int
    min_slot_load: int
    n_items: int
    n_parts: int


def _ceil_div(a: int, b: int) -> int:
    return (a + b - 1) // b


def validate(B: int, Hkv: int, lens, p: Params) -> None:
    if B <= 0 or Hkv <= 0:
        raise ValueError("B and Hkv must be positive")
    if len(lens) != B * Hkv:
        raise ValueError("lens must have B*Hkv entries")
    if any(int(x) < 0 for x in lens):
        raise ValueError("negative length")
    if p.n_slots < 1 or p.tile < 1 or p.max_split < 1 or p.oversub < 1:
        raise ValueError("n_slots, tile, max_split, oversub must be >= 1")
    if p.min_chunk < p.tile or p.min_chunk % p.tile != 0:
        raise ValueError("min_chunk must be a positive multiple of tile")
    if p.overhead_tokens < 0:
        raise ValueError("overhead_tokens must be >= 0")
    if p.policy not in (POLICY_NAIVE, POLICY_LPT, POLICY_LPT_SPLIT):
        raise ValueError("unknown policy")


def plan(lens, B: int, Hkv: int, p: Params):
    """lens: flat sequence of B*Hkv ints in (b, h) order.

    Returns (items, slot_ptr, slot_items, part_base, summary):
      items      work list in execution order,
      slot_ptr   CSR pointer [n_slots+1] over items grouped by slot,
      slot_items indices into `items`, grouped by slot, list order kept inside a slot,
      part_base  [B*Hkv+1] running count of chunks before each pair (CSR over pairs),
      summary    totals and the largest / smallest slot load (idle slots count as 0).
    """
    lens = [int(x) for x in lens]
    validate(B, Hkv, lens, p)
    n_pairs = B * Hkv
    total = sum(lens)

    def up(x: int) -> int:
        return _ceil_div(x, p.tile) * p.tile

    # -- how many equal chunks each pair is cut into (the W / copies rule) ------------
    if p.policy == POLICY_LPT_SPLIT:
        target = max(p.min_chunk, up(_ceil_div(total, p.n_slots * p.oversub)))
    else:
        target = None  # never split

    chunks: List[Tuple[int, int, int, int, int, int]] = []   # (b,h,t0,n,chunk,n_chunks)
    part_base = [0] * (n_pairs + 1)
    for pair in range(n_pairs):
        n = lens[pair]
        b, h = divmod(pair, Hkv)
        r_final = 0
        if n > 0:
            if target is None:
                r = 1
            else:
                r = min(p.max_split, _ceil_div(n, target))
            cs = up(_ceil_div(n, r))
            r_final = _ceil_div(n, cs)
            for c in range(r_final):
                t0 = c * cs
                chunks.append((b, h, t0, min(cs, n - t0), c, r_final))
        part_base[pair + 1] = part_base[pair] + r_final

    # -- order and assignment --------------------------------------------------------
    load = [0] * p.n_slots
    items: List[Item] = []
    if p.policy == POLICY_NAIVE:
        order = chunks  # already ascending (b, h); one chunk per pair
        for idx, (b, h, t0, n, c, nc) in enumerate(order):
            j = idx % p.n_slots
            load[j] += n + p.overhead_tokens
            items.append(Item(b, h, t0, n, c, nc, j, part_base[b * Hkv + h] + c))
    else:
        order = sorted(chunks, key=lambda x: (-x[3], x[0], x[1], x[4]))
        for (b, h, t0, n, c, nc) in order:
            j = min(range(p.n_slots), key=lambda s: (load[s], s))
            load[j] += n + p.overhead_tokens
            items.append(Item(b, h, t0, n, c, nc, j, part_base[b * Hkv + h] + c))

    # -- CSR by slot (stable) --------------------------------------------------------
    slot_ptr = [0] * (p.n_slots + 1)
    for it in items:
        slot_ptr[it.slot + 1] += 1
    for j in range(p.n_slots):
        slot_ptr[j + 1] += slot_ptr[j]
    slot_items = _stable_by_slot(items, p.n_slots)

    summary = Summary(total, max(load), min(load), len(items), part_base[n_pairs])
    return items, slot_ptr, slot_items, part_base, summary


def _stable_by_slot(items, n_slots):
    buckets = [[] for _ in range(n_slots)]
    for i, it in enumerate(items):
        buckets[it.slot].append(i)
    return [i for bkt in buckets for i in bkt]


# ---- figures of merit, straight from the paper's definitions ------------------------
def slot_loads(items, n_slots: int, overhead_tokens: int):
    load = [0] * n_slots
    for it in items:
        load[it.slot] += it.tok_count + overhead_tokens
    return load


def delta(loads) -> int:
    """Algorithm 2's criterion: largest group weight minus smallest group weight."""
    return max(loads) - min(loads)


def efficiency(loads) -> float:
    """Appendix A, eq. 5: mean over devices of load_j / max_k load_k."""
    mx = max(loads)
    if mx == 0:
        return 1.0
    return sum(x / mx for x in loads) / len(loads)
