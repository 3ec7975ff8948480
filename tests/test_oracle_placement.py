"""Pins of the placement oracle (Section 4.3, Algorithms 1 and 2; Appendix A eq. 2-5) against
things other than itself: closed-form counts, independent brute force, hand-made cases,
the equations' invariants and a classical bound."""
from itertools import product
from math import comb

import numpy as np
import pytest

from oracle import placement as PL


def n_copy_vectors(n, m, cap):
    # vectors of n extras e_i in [0, cap-1] with sum <= m: inclusion-exclusion over capped parts
    total = 0
    for s in range(m + 1):
        for j in range(n + 1):
            rest = s - j * cap
            if rest < 0:
                break
            total += (-1) ** j * comb(n, j) * comb(rest + n - 1, n - 1)
    return total


@pytest.mark.parametrize("n,m,cap", [(1, 0, 1), (3, 0, 4), (3, 2, 2), (4, 3, 3), (4, 6, 3), (5, 4, 8), (2, 9, 4)])
def test_algorithm1_lists_every_scheme_once_in_recursion_order(n, m, cap):
    vs = list(PL.copy_vectors(n, m, cap))
    assert len(vs) == len(set(vs)) == n_copy_vectors(n, m, cap)
    assert all(1 <= c <= cap for v in vs for c in v) and all(sum(v) - n <= m for v in vs)
    assert vs == sorted(vs)                 # one copy first, then 2, 3, ...; head 0 outermost
    assert vs[0] == (1,) * n                # the scheme without replication comes first


def test_canonical_splits_are_a_subset_in_the_same_order():
    for c, tp in [((1, 1, 1), 2), ((2, 1), 3), ((2, 2, 1), 3), ((1, 3), 3)]:
        allv = list(PL.splits_all(c, tp))
        can = list(PL.splits_canonical(c, tp))
        assert set(can) <= set(allv) and can == sorted(can) and allv == sorted(allv)
        # every split is a renaming of GPUs / swap of copies away from a canonical one
        owner = [i for i, ci in enumerate(c) for _ in range(ci)]

        def key(g):
            return sorted(tuple(sorted(owner[k] for k in range(len(g)) if g[k] == j)) for j in range(tp))
        assert {tuple(map(tuple, key(g))) for g in allv} == {tuple(map(tuple, key(g))) for g in can}


def test_canonical_search_finds_the_first_best_of_the_literal_search():
    rng = np.random.default_rng(1)
    for _ in range(120):
        n = int(rng.integers(1, 5))
        tp = int(rng.integers(1, 4))
        m = int(rng.integers(0, 3))
        R = int(rng.integers(1, 4))
        W = [int(x) for x in rng.integers(0, 50, size=n)]
        a = PL.search_exact(W, tp, m, R, literal=True)
        b = PL.search_exact(W, tp, m, R, literal=False)
        assert a == b, (W, tp, m, R)


def brute_partition_delta(W, tp):
    best = None
    for g in product(range(tp), repeat=len(W)):
        loads = [0] * tp
        for w, j in zip(W, g):
            loads[j] += w
        d = max(loads) - min(loads)
        best = d if best is None or d < best else best
    return best


def test_without_replication_it_is_multiway_number_partitioning():
    rng = np.random.default_rng(2)
    for _ in range(60):
        n, tp = int(rng.integers(1, 7)), int(rng.integers(1, 4))
        W = [int(x) for x in rng.integers(1, 100, size=n)]
        c, g, loads = PL.search_exact(W, tp, 0, 1)
        assert c == (1,) * n and sum(loads) == sum(W)
        assert max(loads) - min(loads) == brute_partition_delta(W, tp)


def test_hand_made_cases():
    # one heavy head, two light ones, two GPUs: without copies the best is {6} | {1,1}
    c, g, loads = PL.search_exact([6, 1, 1], 2, 0, 1)
    assert sorted(loads) == [2, 6]
    # one extra copy halves the heavy head: 3+1 | 3+1, Delta 0 (den = 2: loads in half tokens)
    c, g, loads = PL.search_exact([6, 1, 1], 2, 1, 2)
    assert c == (2, 1, 1) and loads == [8, 8] and g == (0, 1, 0, 1)
    # already balanced: the first scheme (no copies) is kept although copying would also give 0
    c, g, loads = PL.search_exact([4, 1, 1, 1, 1], 2, 2, 2)
    assert c == (1, 1, 1, 1, 1) and loads[0] == loads[1]
    # three copies of one head over three GPUs
    c, g, loads = PL.search_exact([9], 3, 2, 3)
    assert c == (3,) and g == (0, 1, 2) and loads == [18, 18, 18]      # den = 6, 9/3 tokens each
    # the cap on copies per head (eq. 3) and the cap on extra copies bind
    assert PL.search_exact([9], 3, 2, 2)[0] == (2,)
    # one extra copy for two equal heads on three GPUs: the scheme met first in Algorithm 1's order is kept
    c, g, loads = PL.search_exact([9, 9], 3, 1, 4)
    assert c == (1, 2) and g == (0, 1, 2) and loads == [108, 54, 54]          # den = 12
    # an idle GPU keeps Delta at the largest load, so a copy that does not fill it changes nothing
    assert PL.search_exact([9, 9], 4, 1, 4)[0] == (1, 1)


def check_invariants(W, B, p, shares, loads, s):
    n = len(W)
    by_head = {}
    for sh in shares:
        by_head.setdefault(sh.head, []).append(sh)
    assert sorted(by_head) == list(range(n))                                   # eq. 2: every head placed
    extra = 0
    for i, lst in by_head.items():
        assert [x.copy for x in lst] == list(range(len(lst))) and all(x.n_copies == len(lst) for x in lst)
        assert len(lst) <= min(p.max_copies, p.tp)                             # eq. 3
        gpus = [x.gpu for x in lst]
        assert gpus == sorted(set(gpus)) and all(0 <= j < p.tp for j in gpus)  # distinct GPUs
        assert lst[0].row_begin == 0 and lst[-1].row_end == B                  # rows: contiguous cover
        assert all(a.row_end == b.row_begin for a, b in zip(lst, lst[1:]))
        sizes = [x.row_end - x.row_begin for x in lst]
        assert max(sizes) - min(sizes) <= 1 and sizes == sorted(sizes, reverse=True)
        extra += len(lst) - 1
    assert extra <= p.max_extra
    ref = [0] * p.tp
    for sh in shares:
        ref[sh.gpu] += int(W[sh.head]) * s.den // sh.n_copies                  # W / copies on every replica
    assert ref == loads and sum(loads) == sum(int(w) for w in W) * s.den
    assert s.max_load_num == max(loads) and s.min_load_num == min(loads) and s.delta_num == max(loads) - min(loads)
    mx = max(loads)
    e = 1.0 if mx == 0 else float(np.mean([x / mx for x in loads]))            # eq. 5 as printed
    assert abs(s.efficiency - e) < 1e-12 and 0 < s.efficiency <= 1.0
    assert s.n_shares == len(shares)


def test_invariants_of_both_modes():
    rng = np.random.default_rng(3)
    for _ in range(80):
        n = int(rng.integers(1, 7))
        p = PL.PlaceParams(tp=int(rng.integers(1, 5)), max_extra=int(rng.integers(0, 4)),
                           max_copies=int(rng.integers(1, 5)), mode=int(rng.integers(1, 3)))
        W = [int(x) for x in rng.integers(0, 3000, size=n)]
        B = int(rng.integers(1, 70))
        shares, loads, s = PL.place(W, B, p)
        check_invariants(W, B, p, shares, loads, s)
        assert s.exact == (1 if p.mode == PL.MODE_EXACT else 0)
    for n in (8, 64):                      # greedy on layers the exhaustive search cannot take
        W = [int(x) for x in np.random.default_rng(n).lognormal(7, 0.8, size=n)]
        p = PL.PlaceParams(tp=8, max_extra=6, max_copies=4, mode=PL.MODE_AUTO if n > 12 else PL.MODE_GREEDY)
        shares, loads, s = PL.place(W, 32, p)
        check_invariants(W, 32, p, shares, loads, s)
        assert s.exact == 0


def test_more_allowed_copies_never_hurt_the_exhaustive_search():
    rng = np.random.default_rng(4)
    for _ in range(25):
        n, tp = int(rng.integers(2, 5)), int(rng.integers(2, 4))
        W = [int(x) for x in rng.integers(1, 500, size=n)]
        prev = None
        for m in range(0, 4):
            c, g, loads = PL.search_exact(W, tp, m, 3)
            d = max(loads) - min(loads)
            assert prev is None or d <= prev
            prev = d


def test_greedy_without_copies_is_longest_first_within_its_classical_bound():
    rng = np.random.default_rng(5)
    for _ in range(40):
        n, tp = int(rng.integers(1, 8)), int(rng.integers(1, 4))
        W = [int(x) for x in rng.integers(1, 100, size=n)]
        c, g, loads = PL.search_greedy(W, tp, 0, 1)
        opt = min(max(sum(w for w, j in zip(W, a) if j == k) for k in range(tp)) for a in product(range(tp), repeat=n))
        assert max(loads) * 3 * tp <= opt * (4 * tp - 1)          # Graham's bound for longest-first
    # and copies only ever lower the largest load
    W = [900, 100, 90, 80, 70, 60, 50, 40]
    base = max(PL.search_greedy(W, 4, 0, 1)[2])
    with_copies = PL.search_greedy(W, 4, 3, 4)
    den = 12
    assert max(with_copies[2]) / den < base and sum(with_copies[0]) - len(W) <= 3


def test_static_head_allocation_baseline():
    assert PL.static_head_allocation([5, 1, 2, 2, 7, 0, 1, 1], 4) == [6, 4, 7, 2]
    with pytest.raises(ValueError):
        PL.static_head_allocation([1, 2, 3], 2)


def test_worked_cases_of_the_fixture_file():
    """tests/golden/placement_worked_cases.txt: cases checked by hand against Algorithms 1 and 2."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "placement_worked_cases.txt")
    n = 0
    for line in open(path):
        if not line.strip() or line.startswith("#"):
            continue
        W, tp, m, cap, copies, gpus, loads, den = [[int(x) for x in f.split()] for f in line.split("|")]
        c, g, ld = PL.search_exact(W, tp[0], m[0], cap[0])
        assert list(c) == copies and list(g) == gpus and list(ld) == loads, line
        shares, ld2, s = PL.place(W, 4, PL.PlaceParams(tp=tp[0], max_extra=m[0], max_copies=cap[0], mode=PL.MODE_EXACT))
        assert ld2 == loads and s.den == den[0] and [sh.gpu for sh in shares] == gpus, line
        assert s.delta_num == max(loads) - min(loads)                                   # eq. 4's quantity
        assert abs(s.efficiency - sum(loads) / (tp[0] * max(loads))) < 1e-12            # eq. 5
        n += 1
    assert n == 6
