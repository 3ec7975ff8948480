"""Pins of the FAIR policy (the line cut) that do not depend on a second implementation of the same loop.

The product planner (C, through the binding; host code only) and the oracle planner are each held to
what the paper's model and the policy's own contract fix: every token of every pair is covered exactly
once (Appendix A, eq. 2), no pair is in more pieces than the cap (eq. 3), cuts fall on tile boundaries,
no piece of a cut pair is smaller than min_chunk, the largest slot load stays within a stated distance of
the lower bound of eq. 4, the efficiency E (eq. 5) stays above a stated floor, and on tiny inputs the
largest load is compared with the true optimum over all contiguous cuts, found by brute force.
"""
import itertools

import numpy as np
import pytest

import workloads as W
from oracle import planner as P


def _c_plan(lens, offs, B, Hkv, **kw):
    import paper_2502_15804_amd as F
    p = F.fairkv_default_params(256, **kw)
    pl = F.fairkv_plan(lens, offs, B, Hkv, p)
    items = [P.Item(int(r["row"]), int(r["tok_count"]), int(r["b"]), int(r["h"]), int(r["chunk"]), int(r["n_chunks"]),
                    int(r["part"])) for r in pl.items]
    return items, [int(x) for x in pl.slot_ptr], int(pl.summary.max_slot_load), int(pl.summary.min_slot_load)


def _o_plan(lens, offs, B, Hkv, **kw):
    p = P.Params(**kw)
    items, slot_ptr, _, s = P.plan(lens, offs, B, Hkv, p)
    return items, slot_ptr, s.max_slot_load, s.min_slot_load


IMPLS = [pytest.param(_o_plan, id="oracle"), pytest.param(_c_plan, id="library")]


def _random_case(rng):
    B, Hkv = int(rng.integers(1, 9)), int(rng.integers(1, 9))
    kind = int(rng.integers(0, 3))
    if kind == 0:
        lens = rng.integers(0, 5000, size=B * Hkv)
    elif kind == 1:          # heavy tailed, like per-head budgets
        lens = np.clip(np.rint(np.exp(rng.normal(6.0, 1.0, size=B * Hkv))), 0, 30000)
    else:
        lens = rng.integers(0, 200, size=B * Hkv)
    lens = lens.astype(np.int32)
    tile = int(rng.choice([1, 16, 32, 64]))
    kw = dict(n_slots=int(rng.choice([1, 2, 3, 7, 16, 64, 256, 320])), tile=tile, min_chunk=tile * int(rng.integers(1, 5)),
              overhead_tokens=int(rng.choice([0, 16, 128, 256])), max_split=int(rng.choice([2, 8, 1 << 20, 1 << 20, 1 << 20])),
              policy=P.POLICY_FAIR)
    kw["short_overhead_tokens"] = int(rng.choice([0, kw["overhead_tokens"] // 3]))     # short pairs may cost less
    offs = W.packed_offsets(lens.reshape(B, Hkv), gap_rows=int(rng.integers(0, 3)))[0].reshape(-1)
    return lens, offs, B, Hkv, kw


def _check_contract(lens, offs, B, Hkv, kw, items, slot_ptr, max_load, min_load):
    tile, mc, ov, S, cap = kw["tile"], kw["min_chunk"], kw["overhead_tokens"], kw["n_slots"], kw["max_split"]
    pieces = {}
    for it in items:
        pieces.setdefault(it.b * Hkv + it.h, []).append(it)
    # eq. 2: every pair placed, every token exactly once, in order
    assert sorted(pieces) == list(range(B * Hkv))
    for pair, its in pieces.items():
        its.sort(key=lambda x: x.chunk)
        n = int(lens[pair])
        assert [x.chunk for x in its] == list(range(len(its))) and all(x.n_chunks == len(its) for x in its)
        assert len({x.part - x.chunk for x in its}) == 1                     # consecutive partial slots
        assert len(its) <= max(1, cap)                                       # eq. 3
        if n == 0:
            assert len(its) == 1 and its[0].tok_count == 0
            continue
        pos = 0
        for x in its:
            assert x.row == offs[pair] + pos and x.tok_count > 0
            assert pos % tile == 0                                           # cuts on tile boundaries
            pos += x.tok_count
        assert pos == n
        if len(its) > 1:
            assert all(x.tok_count >= mc for x in its), "a piece of a cut pair below min_chunk"
    assert sorted(x.part for x in items) == list(range(len(items)))
    # a line cut: the pairs' pieces appear in (pair, chunk) order along the slots
    assert [(x.b * Hkv + x.h, x.chunk) for x in items] == sorted((x.b * Hkv + x.h, x.chunk) for x in items)
    loads = P.slot_loads(items, slot_ptr, ov, kw.get("short_overhead_tokens", 0))
    assert max(loads) == max_load and min(loads) == min_load and len(loads) == S
    return loads


@pytest.mark.parametrize("impl", IMPLS)
def test_fair_contract_on_random_cases(impl):
    rng = np.random.default_rng(2024)
    checked_bound = 0
    for _ in range(600):
        lens, offs, B, Hkv, kw = _random_case(rng)
        items, slot_ptr, mx, mn = impl(lens, offs, B, Hkv, **kw)
        loads = _check_contract(lens, offs, B, Hkv, kw, items, slot_ptr, mx, mn)
        tile, mc, ov, S = kw["tile"], kw["min_chunk"], kw["overhead_tokens"], kw["n_slots"]
        total = int(lens.sum())
        # eq. 4's lower bound: no plan can have a largest load below the mean cost per slot
        assert mx >= -(-(total + min(ov, kw["short_overhead_tokens"] or ov) * len(items)) // S)
        if kw["max_split"] < (1 << 20):
            continue                     # a capped pair ends in one long piece: the balance bound is not claimed
        # The budget of a slot never exceeds ceil((tokens + overhead * (pairs + slots)) / slots) by more than the
        # slack earlier slots left (below min_chunk + tile each, spread over the slots to come), and a slot
        # overshoots its budget by less than min_chunk + tile.  Claimed where a slot's share is not tiny:
        share = -(-(total + ov * (B * Hkv + S)) // S)
        if share >= 2 * mc + tile + ov:
            assert mx <= share + 2 * (mc + tile) + ov, (lens.tolist(), kw, mx, share)
            checked_bound += 1
            if share >= 8 * (mc + tile + ov):
                assert P.efficiency(loads) >= 0.8, (lens.tolist(), kw, P.efficiency(loads))
    assert checked_bound >= 150


def _best_contiguous_cut(lens, S, tile, ov):
    """Smallest possible largest slot load over ALL ways of cutting the line of pairs (in order) into S
    contiguous runs, cuts at tile boundaries inside a pair or between pairs; a run costs its tokens plus
    `ov` per pair it touches.  Plain enumeration of cut positions."""
    marks = [0]                                   # candidate cut positions along the line, in tokens
    starts = []
    pos = 0
    for n in lens:
        starts.append(pos)
        marks.extend(pos + t for t in range(tile, n, tile))
        pos += n
        marks.append(pos)
    marks = sorted(set(marks))
    ends = [s + n for s, n in zip(starts, lens)]

    def cost(a, b):
        if a == b:
            return 0
        touched = sum(1 for s, e, n in zip(starts, ends, lens) if n > 0 and s < b and e > a)
        return (b - a) + ov * touched

    best = None
    inner = marks[1:-1]
    for cuts in itertools.combinations_with_replacement(inner, S - 1):
        edges = [0, *cuts, marks[-1]]
        mx = max(cost(a, b) for a, b in zip(edges[:-1], edges[1:]))
        best = mx if best is None else min(best, mx)
    return best if best is not None else cost(0, marks[-1])


@pytest.mark.parametrize("impl", IMPLS)
def test_fair_against_the_brute_force_optimum_on_tiny_inputs(impl):
    rng = np.random.default_rng(7)
    tile, mc = 16, 16
    gaps = []
    for _ in range(120):
        n_pairs = int(rng.integers(1, 5))
        S = int(rng.integers(1, 4))
        lens = rng.integers(1, 9, size=n_pairs).astype(np.int32) * 16 + rng.integers(0, 16, size=n_pairs).astype(np.int32)
        ov = int(rng.choice([0, 8, 32]))
        offs = W.packed_offsets(lens.reshape(n_pairs, 1))[0].reshape(-1)
        kw = dict(n_slots=S, tile=tile, min_chunk=mc, overhead_tokens=ov, max_split=1 << 20, policy=P.POLICY_FAIR,
                  short_overhead_tokens=0)
        items, slot_ptr, mx, _ = impl(lens, offs, n_pairs, 1, **kw)
        opt = _best_contiguous_cut([int(x) for x in lens], S, tile, ov)
        assert opt <= mx, "a line cut cannot beat the best line cut"
        assert mx <= opt + mc + tile + ov, (lens.tolist(), S, ov, mx, opt)
        gaps.append(mx - opt)
    assert np.mean(gaps) <= 24          # and on average it is close


@pytest.mark.parametrize("impl", IMPLS)
def test_fair_on_the_workloads(impl):
    # the four benchmark workloads: contract, balance within the stated distance, efficiency (eq. 5)
    for name, floor in (("llama70b", 0.93), ("mistral24b", 0.95), ("faircopy", 0.95), ("stress", 0.88)):
        w = W.WORKLOADS[name]
        for layer in (0, 1):
            lens = W.lens(name, layer=layer).reshape(-1)
            offs = W.packed_offsets(lens.reshape(w.B, w.Hkv))[0].reshape(-1)
            kw = dict(n_slots=256, tile=16, min_chunk=32, overhead_tokens=128, max_split=256, policy=P.POLICY_FAIR,
                      short_overhead_tokens=48)
            items, slot_ptr, mx, mn = impl(lens, offs, w.B, w.Hkv, **kw)
            loads = _check_contract(lens, offs, w.B, w.Hkv, kw, items, slot_ptr, mx, mn)
            share = -(-(int(lens.sum()) + 128 * (lens.size + 256)) // 256)
            assert mx <= share + 2 * (32 + 16) + 128
            assert P.efficiency(loads) >= floor, (name, P.efficiency(loads))
            assert len(items) <= lens.size + 256 - 1        # a line cut adds at most one item per slot boundary
