"""Oracle work planner: integer-only, step by step, for bit-exact comparison.

TEST INFRASTRUCTURE ONLY (see the package docstring).

The paper balances heads of unequal KV-cache size over GPUs: its objective is to
minimise the largest per-device load (Appendix A, eq. 4), a replicated head
carries weight W/copies on each replica (Algorithm 2, the adjusted weights
W_A), replication is capped (eq. 3), every head must be placed (eq. 2), and a
scheme is judged by max-minus-min group weight (Algorithm 2) and by the
efficiency E = mean load / max load (eq. 5).  Its own search (Algorithms 1 and
2) is exhaustive and meant for a handful of heads and GPUs.  On one GPU the
"devices" are persistent workgroup slots (one per compute unit) and the "heads"
are hundreds of (sequence, KV head) pairs, so the same objective is pursued
without search.  Four policies, mirroring the paper's ablation (Section 5.2.1):

  NAIVE      pairs dealt to slots round-robin, unsplit: static head allocation.
  LPT        load-aware placement of whole pairs, longest first onto the least
             loaded slot: Best-effort Assignment, no replication.
  LPT_SPLIT  Fair-Copying as the paper states it: a heavy pair becomes r equal
             chunks (each carries len/r, the W/copies rule, r capped by
             max_split), then chunks are placed like LPT.
  FAIR       Fair-Copying taken to its limit on one GPU, where a "replica" may
             take any share: pairs are laid end to end and the line is cut into
             n_slots pieces of equal cost, so a pair is shared only by the slots
             whose boundary falls inside it.  Reaches the lower bound of eq. 4
             up to one tile and the per-item overhead.

An item costs tok_count + overhead_tokens (the linear latency model with an
offset of Section 3.2); a short pair (a whole pair of at most SHORT_PAIR_TOKENS
tokens) may be given a fixed cost of its own, short_overhead_tokens.  Pairs with no tokens still get one empty item, so that
some slot writes their zero output.  Several plans can be equally good in the
paper's sense; order and tie-breaks are fixed only so that two implementations
can be compared field by field.  All arithmetic is on Python ints.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

POLICY_NAIVE = 0
POLICY_LPT = 1
POLICY_LPT_SPLIT = 2
POLICY_FAIR = 3


@dataclass(frozen=True)
class Params:
    n_slots: int = 256
    tile: int = 16
    min_chunk: int = 32
    max_split: int = 256
    oversub: int = 2
    overhead_tokens: int = 160
    policy: int = POLICY_FAIR
    short_overhead_tokens: int = 0    # fixed cost of a short pair (a whole pair of at most SHORT_PAIR_TOKENS); 0: overhead_tokens


SHORT_PAIR_TOKENS = 96


@dataclass(frozen=True)
class Item:
    row: int          # first K/V row: off[b][h] + first token of the chunk
    tok_count: int
    b: int
    h: int
    chunk: int        # which piece of the pair, in token order
    n_chunks: int
    part: int         # part_base[pair] + chunk

    def astuple(self) -> Tuple[int, ...]:
        return (self.row, self.tok_count, self.b, self.h, self.chunk, self.n_chunks, self.part)


@dataclass(frozen=True)
class Summary:
    total_tokens: int
    max_slot_load: int
    min_slot_load: int
    n_items: int
    n_parts: int


def _ceil_div(a: int, b: int) -> int:
    return (a + b - 1) // b


def validate(B: int, Hkv: int, lens, offs, p: Params) -> None:
    if B <= 0 or Hkv <= 0:
        raise ValueError("B and Hkv must be positive")
    if len(lens) != B * Hkv or len(offs) != B * Hkv:
        raise ValueError("lens and offs must have B*Hkv entries")
    if any(int(x) < 0 for x in lens):
        raise ValueError("negative length")
    if any(int(o) < 0 for o, n in zip(offs, lens) if int(n) > 0):
        raise ValueError("negative offset")
    if p.n_slots < 1 or p.tile < 1 or p.max_split < 1 or p.oversub < 1:
        raise ValueError("n_slots, tile, max_split, oversub must be >= 1")
    if p.min_chunk < p.tile or p.min_chunk % p.tile != 0:
        raise ValueError("min_chunk must be a positive multiple of tile")
    if p.overhead_tokens < 0 or p.short_overhead_tokens < 0:
        raise ValueError("overhead_tokens and short_overhead_tokens must be >= 0")
    if p.policy not in (POLICY_NAIVE, POLICY_LPT, POLICY_LPT_SPLIT, POLICY_FAIR):
        raise ValueError("unknown policy")


def plan(lens, offs, B: int, Hkv: int, p: Params):
    """lens, offs: flat sequences of B*Hkv ints in (b, h) order (tokens, first row).

    Returns (items, slot_ptr, part_base, summary):
      items      work list grouped by slot; inside a slot, the order the slot runs them,
      slot_ptr   [n_slots+1]: slot j runs items[slot_ptr[j] : slot_ptr[j+1]],
      part_base  [B*Hkv+1]: running count of chunks before each pair,
      summary    totals and the largest / smallest slot load (an idle slot counts 0).
    """
    lens = [int(x) for x in lens]
    offs = [int(x) for x in offs]
    validate(B, Hkv, lens, offs, p)
    n_pairs = B * Hkv
    total = sum(lens)
    S, ov = p.n_slots, p.overhead_tokens

    def item_ov(count: int, whole_pair: bool) -> int:
        """Fixed cost of an item: a short pair taken whole has its own (the kernel runs it on one wave)."""
        if whole_pair and count <= SHORT_PAIR_TOKENS and p.short_overhead_tokens > 0:
            return p.short_overhead_tokens
        return ov

    def up(x: int) -> int:
        return _ceil_div(x, p.tile) * p.tile

    # pieces: (pair, tok_begin, tok_count, chunk index); slots: list of piece lists
    slots: List[List[Tuple[int, int, int, int]]] = [[] for _ in range(S)]
    n_chunks_of = [0] * n_pairs

    if p.policy == POLICY_FAIR:
        # One line of all pairs in (b, h) order, cut into S pieces of equal cost.  When a slot
        # is opened its budget is the cost still to place divided by the slots still unopened
        # (an item is counted as overhead for every pair still unfinished and every slot still
        # to come), so slack or excess of one slot is spread over the later ones.  A pair that
        # does not fit continues in the next slot, cut at a tile boundary.  No piece smaller than
        # min_chunk is made: the slot is overfilled with the whole rest of the pair if that
        # excess is smaller than the room it would otherwise leave unused, else it is closed.
        # The last slot takes whatever is left.
        tokens_left = total
        ov_left = sum(item_ov(n, True) for n in lens)       # fixed costs of the unfinished pairs, each taken whole

        def budget_for(j: int) -> int:
            open_slots = S - j
            return _ceil_div(tokens_left + ov_left + ov * open_slots, open_slots)

        j = 0
        room = budget_for(0)
        for pair in range(n_pairs):
            left, begin, c = lens[pair], 0, 0
            if left == 0:
                if room < item_ov(0, True) and j < S - 1:
                    j += 1
                    room = budget_for(j)
                slots[j].append((pair, 0, 0, 0))
                room -= item_ov(0, True)
                c = 1
            while left > 0:
                last_slot = j == S - 1
                last_copy = c == p.max_split - 1            # eq. 3: no further copy allowed
                ov_take_all = item_ov(left, begin == 0)      # if this item takes all that is left of the pair
                fit_all = max(0, (room - ov_take_all) // p.tile * p.tile)
                fit = max(0, (room - ov) // p.tile * p.tile)  # whole tiles that still fit here (a piece of a cut pair)
                if last_slot or last_copy or left <= fit_all:
                    take = left
                elif fit >= p.min_chunk and left - fit >= p.min_chunk:
                    take = fit                               # cut: neither piece is tiny
                elif left - fit <= fit:
                    take = left                              # a small overfill beats unused room
                else:                                        # too little room: close this slot
                    j += 1
                    room = budget_for(j)
                    continue
                slots[j].append((pair, begin, take, c))
                room -= take + (ov_take_all if take == left else ov)
                begin, left, c = begin + take, left - take, c + 1
                tokens_left -= take
                if left > 0 and j < S - 1:                   # slot is full: go on in the next
                    j += 1
                    room = budget_for(j)
            n_chunks_of[pair] = c
            ov_left -= item_ov(lens[pair], True)
    else:
        if p.policy == POLICY_LPT_SPLIT:
            target = max(p.min_chunk, up(_ceil_div(total, S * p.oversub)))
        else:
            target = None
        pieces: List[Tuple[int, int, int, int]] = []
        for pair in range(n_pairs):
            n = lens[pair]
            if n == 0:
                pieces.append((pair, 0, 0, 0))
                n_chunks_of[pair] = 1
                continue
            r = 1 if target is None else min(p.max_split, _ceil_div(n, target))
            cs = up(_ceil_div(n, r))                       # W / copies, in whole tiles
            r_final = _ceil_div(n, cs)
            for c in range(r_final):
                pieces.append((pair, c * cs, min(cs, n - c * cs), c))
            n_chunks_of[pair] = r_final
        if p.policy == POLICY_NAIVE:
            for idx, pc in enumerate(pieces):
                slots[idx % S].append(pc)
        else:
            load = [0] * S
            for pc in sorted(pieces, key=lambda x: (-x[2], x[0], x[3])):
                j = min(range(S), key=lambda s: (load[s], s))
                load[j] += pc[2] + item_ov(pc[2], n_chunks_of[pc[0]] == 1)
                slots[j].append(pc)

    part_base = [0] * (n_pairs + 1)
    for pair in range(n_pairs):
        part_base[pair + 1] = part_base[pair] + n_chunks_of[pair]

    items: List[Item] = []
    slot_ptr = [0] * (S + 1)
    loads = []
    for j in range(S):
        for (pair, begin, count, c) in slots[j]:
            b, h = divmod(pair, Hkv)
            items.append(Item(offs[pair] + begin, count, b, h, c, n_chunks_of[pair], part_base[pair] + c))
        slot_ptr[j + 1] = len(items)
        loads.append(sum(pc[2] + item_ov(pc[2], n_chunks_of[pc[0]] == 1) for pc in slots[j]))

    summary = Summary(total, max(loads), min(loads), len(items), part_base[n_pairs])
    return items, slot_ptr, part_base, summary


def grow(items, lens, cap, Hkv: int):
    """A decode step appended one row to every pair below its capacity: the pair's last chunk
    covers it.  Returns the new item list; lens is updated in place."""
    out = []
    for it in items:
        pair = it.b * Hkv + it.h
        if it.chunk == it.n_chunks - 1 and lens[pair] < cap[pair]:
            lens[pair] += 1
            it = Item(it.row, it.tok_count + 1, it.b, it.h, it.chunk, it.n_chunks, it.part)
        out.append(it)
    return out


# ---- figures of merit, straight from the paper's definitions ------------------------
def slot_loads(items, slot_ptr, overhead_tokens: int, short_overhead_tokens: int = 0):
    def cost(it):
        short = it.n_chunks == 1 and it.tok_count <= SHORT_PAIR_TOKENS and short_overhead_tokens > 0
        return it.tok_count + (short_overhead_tokens if short else overhead_tokens)
    return [sum(cost(it) for it in items[slot_ptr[j]:slot_ptr[j + 1]]) for j in range(len(slot_ptr) - 1)]


def delta(loads) -> int:
    """Algorithm 2's criterion: largest group weight minus smallest group weight."""
    return max(loads) - min(loads)


def efficiency(loads) -> float:
    """Appendix A, eq. 5: mean over devices of load_j / max_k load_k."""
    mx = max(loads)
    if mx == 0:
        return 1.0
    return sum(x / mx for x in loads) / len(loads)
