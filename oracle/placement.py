"""Oracle for the multi-GPU head placement search (Section 4.3, Algorithms 1 and 2; Appendix A).

TEST INFRASTRUCTURE ONLY (see the package docstring).

What the paper fixes.  A layer has heads with weights W (the KV-cache each head keeps).
Algorithm 1 lists the replication schemes: every head appears once or n >= 2 times.
Algorithm 2 gives every copy of a head the adjusted weight W_A = W / copies, tries the
splits of the copies into tp groups (one group per GPU) and keeps the split whose largest
group weight exceeds its smallest by the least (Delta); the comparison is strict, so the
first split found wins among equals.  Appendix A adds: every head is placed at least once
(eq. 2), a head has at most R_max copies (eq. 3), the objective is the largest GPU load
(eq. 4) and the efficiency is E = mean load / largest load (eq. 5).

Readings where the paper is silent or garbled (each is a decision of this build):
  * Algorithm 1 declares a maximum number of copied heads m but its printed loop bound
    never uses it and grows with the scheme built so far.  Read as: the extra copies of a
    scheme, sum_i (c_i - 1), are at most m, and c_i <= R_max.
  * The copies of one head sit on different GPUs (two copies on one GPU are one copy), so
    also c_i <= tp.
  * GPUs may hold different numbers of heads.
  * Delta in Algorithm 2 is taken over the groups of the split: max over groups of the
    summed W_A minus min over groups (an empty group weighs 0).
  * Orders, which the paper leaves open: schemes in the order of Algorithm 1's recursion
    (head by head, one copy first, then 2, 3, ...); within a scheme the copies are taken
    head by head and the splits in lexicographic order of (group of copy 0, group of
    copy 1, ...).
  * Weights are integers (token counts).  W / copies is kept exact by scaling every
    weight with den = lcm(1..R_max).
  * A head's copies share the batch by contiguous row ranges; with r copies of B rows the
    first B mod r copies take ceil(B / r) rows.

The exhaustive search is meant for a handful of heads and GPUs (the paper's own use).  For
larger layers a greedy variant is defined here: place the copies longest first onto the
least loaded GPU that does not hold the head yet, then, up to m times, give one more copy to
the heaviest copy on the most loaded GPU and keep that if the largest load drops.
"""
from __future__ import annotations

from dataclasses import dataclass
from itertools import product
from math import gcd
from typing import Iterator, List, Optional, Sequence, Tuple

MODE_AUTO = 0
MODE_EXACT = 1
MODE_GREEDY = 2

EXACT_LIMIT = 12     # MODE_AUTO searches exhaustively while n_heads + max_extra <= this


@dataclass(frozen=True)
class PlaceParams:
    tp: int                  # GPUs (groups)
    max_extra: int = 0       # m: extra copies in total
    max_copies: int = 1      # R_max: copies per head
    mode: int = MODE_AUTO


@dataclass(frozen=True)
class Share:
    head: int
    gpu: int
    copy: int
    n_copies: int
    row_begin: int
    row_end: int


@dataclass(frozen=True)
class Summary:
    den: int                 # loads below are in units of 1/den tokens
    delta_num: int           # Algorithm 2's criterion of the chosen scheme
    max_load_num: int
    min_load_num: int
    efficiency: float        # eq. 5
    n_shares: int
    exact: int               # 1: exhaustive search, 0: greedy


def _lcm_upto(n: int) -> int:
    out = 1
    for k in range(2, n + 1):
        out = out * k // gcd(out, k)
    return out


def validate(W: Sequence[int], B: int, p: PlaceParams) -> None:
    if len(W) < 1 or any(int(w) < 0 for w in W):
        raise ValueError("weights must be non-negative and there must be a head")
    if p.tp < 1 or p.max_extra < 0 or p.max_copies < 1 or p.max_copies > 8 or B < 1:
        raise ValueError("bad parameters")
    if p.mode not in (MODE_AUTO, MODE_EXACT, MODE_GREEDY):
        raise ValueError("unknown mode")


def copy_vectors(n: int, m: int, cap: int) -> Iterator[Tuple[int, ...]]:
    """Algorithm 1 under the reading above: all (c_0..c_{n-1}), 1 <= c_i <= cap, with at most m
    extra copies in total, in the order of the recursion (head by head; 1 copy, then 2, 3, ...)."""
    c: List[int] = []

    def backtrack(index: int, extra_left: int) -> Iterator[Tuple[int, ...]]:
        if index == n:
            yield tuple(c)
            return
        c.append(1)                                   # case 1: a single copy
        yield from backtrack(index + 1, extra_left)
        c.pop()
        for k in range(2, min(cap, 1 + extra_left) + 1):   # case 2: k copies
            c.append(k)
            yield from backtrack(index + 1, extra_left - (k - 1))
            c.pop()

    yield from backtrack(0, m)


def splits_all(c: Sequence[int], tp: int) -> Iterator[Tuple[int, ...]]:
    """Every split of the copies into tp groups in lexicographic order, copies of one head on
    different groups: the definition, for tiny cases."""
    owner = [i for i, ci in enumerate(c) for _ in range(ci)]
    for g in product(range(tp), repeat=len(owner)):
        ok = True
        seen = {}
        for k, i in enumerate(owner):
            if g[k] in seen.setdefault(i, set()):
                ok = False
                break
            seen[i].add(g[k])
        if ok:
            yield g


def splits_canonical(c: Sequence[int], tp: int) -> Iterator[Tuple[int, ...]]:
    """The splits that are first, in that order, among all that differ only by renaming GPUs or
    by swapping copies of one head: a new GPU index is used only after all smaller ones, and a
    head's copies go to ascending GPUs.  The first best split of splits_all is one of these."""
    owner = [i for i, ci in enumerate(c) for _ in range(ci)]
    g: List[int] = []

    def rec(k: int, used: int) -> Iterator[Tuple[int, ...]]:
        if k == len(owner):
            yield tuple(g)
            return
        lo = g[k - 1] + 1 if k > 0 and owner[k - 1] == owner[k] else 0
        for x in range(lo, min(tp, used + 1)):
            g.append(x)
            yield from rec(k + 1, max(used, x + 1))
            g.pop()

    yield from rec(0, 0)


def _loads(c, g, w_scaled, tp):
    loads = [0] * tp
    k = 0
    for i, ci in enumerate(c):
        for _ in range(ci):
            loads[g[k]] += w_scaled[i] // ci
            k += 1
    return loads


def search_exact(W: Sequence[int], tp: int, m: int, R: int, literal: bool = False):
    """Algorithms 1 and 2: (copies per head, group of every copy, loads) of the first scheme with
    the smallest Delta.  literal=True walks every split (tiny cases only)."""
    n = len(W)
    den = _lcm_upto(R)
    w_scaled = [int(w) * den for w in W]
    best = None
    best_delta = None
    for c in copy_vectors(n, m, min(R, tp)):
        for g in (splits_all(c, tp) if literal else splits_canonical(c, tp)):
            loads = _loads(c, g, w_scaled, tp)
            d = max(loads) - min(loads)
            if best_delta is None or d < best_delta:
                best_delta, best = d, (c, g, loads)
    return best


def _lpt(c: Sequence[int], w_scaled: Sequence[int], tp: int):
    """Copies longest first (ties: lower head, lower copy) onto the least loaded GPU (ties: lower
    index) that does not hold the head yet."""
    copies = sorted(((w_scaled[i] // ci, i, r) for i, ci in enumerate(c) for r in range(ci)),
                    key=lambda t: (-t[0], t[1], t[2]))
    loads = [0] * tp
    holds = [set() for _ in range(tp)]
    where = {}
    for w, i, r in copies:
        j = min((x for x in range(tp) if i not in holds[x]), key=lambda x: (loads[x], x))
        loads[j] += w
        holds[j].add(i)
        where[(i, r)] = j
    return where, loads


def search_greedy(W: Sequence[int], tp: int, m: int, R: int):
    n = len(W)
    den = _lcm_upto(R)
    w_scaled = [int(w) * den for w in W]
    cap = min(R, tp)
    c = [1] * n
    where, loads = _lpt(c, w_scaled, tp)
    for _ in range(m):
        top = max(range(tp), key=lambda x: (loads[x], -x))
        cand = [(w_scaled[i] // c[i], -i) for (i, r), j in where.items() if j == top and c[i] < cap]
        if not cand:
            break
        i = -max(cand)[1]
        c2 = list(c)
        c2[i] += 1
        where2, loads2 = _lpt(c2, w_scaled, tp)
        if max(loads2) >= max(loads):
            break
        c, where, loads = c2, where2, loads2
    g = []
    for i, ci in enumerate(c):
        g.extend(sorted(where[(i, r)] for r in range(ci)))   # copies numbered by ascending GPU
    return tuple(c), tuple(g), loads


def place(W: Sequence[int], B: int, p: PlaceParams):
    """Returns (shares ordered by (head, copy), loads per GPU in units of 1/den, summary)."""
    validate(W, B, p)
    n = len(W)
    exact = p.mode == MODE_EXACT or (p.mode == MODE_AUTO and n + p.max_extra <= EXACT_LIMIT)
    if exact:
        c, g, loads = search_exact(W, p.tp, p.max_extra, p.max_copies)
    else:
        c, g, loads = search_greedy(W, p.tp, p.max_extra, p.max_copies)
    shares: List[Share] = []
    k = 0
    for i, ci in enumerate(c):
        base, rem = divmod(B, ci)
        for r in range(ci):
            begin = r * base + min(r, rem)
            shares.append(Share(i, g[k], r, ci, begin, begin + base + (1 if r < rem else 0)))
            k += 1
    mx, mn = max(loads), min(loads)
    eff = 1.0 if mx == 0 else sum(loads) / (p.tp * mx)
    return shares, list(loads), Summary(_lcm_upto(p.max_copies), mx - mn, mx, mn, eff, len(shares), 1 if exact else 0)


def static_head_allocation(W: Sequence[int], tp: int) -> List[int]:
    """Plain tensor parallelism (Figure 3 (1)): heads in order, an equal count per GPU; returns the
    loads.  len(W) must be a multiple of tp."""
    n = len(W)
    if n % tp:
        raise ValueError("heads must divide evenly over the GPUs")
    per = n // tp
    return [sum(int(w) for w in W[j * per:(j + 1) * per]) for j in range(tp)]
