"""Pins of the oracle planner: the paper's constraints and figures of merit
(Appendix A eq. 2-5, Algorithm 2's adjusted weights and max-minus-min
criterion), closed forms, and textbook facts about longest-processing-time
scheduling checked by brute force on tiny inputs."""
import itertools

import numpy as np
import pytest

import workloads as W
from oracle import planner as P

ALL_POLICIES = [P.POLICY_NAIVE, P.POLICY_LPT, P.POLICY_LPT_SPLIT, P.POLICY_FAIR]


def run(lens, B, Hkv, offs=None, **kw):
    p = P.Params(**kw)
    lens = np.asarray(lens).reshape(-1)
    if offs is None:
        offs = W.packed_offsets(lens.reshape(B, Hkv), gap_rows=1)[0]
    return (p, np.asarray(offs).reshape(-1)) + P.plan(lens, np.asarray(offs).reshape(-1), B, Hkv, p)


def check_invariants(lens, B, Hkv, p, offs, items, slot_ptr, part_base, s):
    lens = np.asarray(lens).reshape(-1)
    # eq. 2: every pair is covered exactly once, by ascending disjoint chunks
    by_pair = {}
    for it in items:
        by_pair.setdefault((it.b, it.h), []).append(it)
    for pair, n in enumerate(lens):
        b, h = divmod(pair, Hkv)
        its = sorted(by_pair.get((b, h), []), key=lambda x: x.part)
        assert [x.part for x in its] == [part_base[pair] + c for c in range(len(its))]
        assert part_base[pair + 1] - part_base[pair] == len(its)
        assert all(x.n_chunks == len(its) for x in its)
        if n == 0:      # an empty pair has one empty item: somebody must write its zero output
            assert len(its) == 1 and its[0].tok_count == 0
            continue
        # eq. 3: replication (here: split) factor is capped
        cap = {P.POLICY_NAIVE: 1, P.POLICY_LPT: 1}.get(p.policy, p.max_split)
        assert 1 <= len(its) <= cap
        pos = 0
        for c, x in enumerate(its):
            assert x.chunk == c and x.tok_count > 0 and x.row == offs[pair] + pos
            assert pos % p.tile == 0                    # cuts fall on tile boundaries of the pair
            pos += x.tok_count
        assert pos == n
        if p.policy == P.POLICY_LPT_SPLIT and len(its) > 1:
            # Algorithm 2's W / copies: equal shares, rounded up to whole tiles; only the last is short
            cs = its[0].tok_count
            assert cs % p.tile == 0
            assert all(x.tok_count == cs for x in its[:-1]) and 0 < its[-1].tok_count <= cs
            assert cs - n / len(its) < p.tile        # within one tile of the equal share
        if p.policy == P.POLICY_FAIR and len(its) > 1 and len(its) < p.max_split:
            assert all(x.tok_count >= p.min_chunk for x in its)     # no tiny pieces
    assert sum(it.tok_count for it in items) == int(lens.sum()) == s.total_tokens
    assert s.n_items == len(items) and s.n_parts == part_base[-1] == len(items)
    assert slot_ptr[0] == 0 and slot_ptr[-1] == len(items) and len(slot_ptr) == p.n_slots + 1
    assert all(a <= b for a, b in zip(slot_ptr[:-1], slot_ptr[1:]))
    loads = P.slot_loads(items, slot_ptr, p.overhead_tokens)
    assert s.max_slot_load == max(loads) and s.min_slot_load == min(loads)
    # lower bounds any schedule obeys
    costs = [it.tok_count + p.overhead_tokens for it in items]
    assert s.max_slot_load >= -(-sum(costs) // p.n_slots)
    if p.policy != P.POLICY_FAIR:
        assert s.max_slot_load >= max(costs)


@pytest.mark.parametrize("name", list(W.WORKLOADS))
@pytest.mark.parametrize("policy", ALL_POLICIES)
def test_invariants_on_workloads(name, policy):
    w = W.WORKLOADS[name]
    lens = W.lens(name)
    out = run(lens, w.B, w.Hkv, policy=policy)
    check_invariants(lens, w.B, w.Hkv, *out)


def test_invariants_on_random_cases():
    rng = np.random.default_rng(0)
    for _ in range(400):
        B, Hkv = int(rng.integers(1, 7)), int(rng.integers(1, 7))
        lens = rng.integers(0, 3000, size=B * Hkv)
        lens[rng.random(B * Hkv) < 0.15] = 0
        tile = int(rng.choice([1, 16, 64]))
        kw = dict(n_slots=int(rng.integers(1, 40)), tile=tile, min_chunk=tile * int(rng.integers(1, 6)),
                  max_split=int(rng.integers(1, 20)), oversub=int(rng.integers(1, 4)),
                  overhead_tokens=int(rng.integers(0, 100)), policy=int(rng.integers(0, 4)))
        out = run(lens, B, Hkv, **kw)
        check_invariants(lens, B, Hkv, *out)


def test_equal_lengths_closed_form_delta_zero_efficiency_one():
    B, Hkv, L = 4, 8, 200
    lens = np.full(B * Hkv, L)
    for policy in ALL_POLICIES:
        p, offs, items, slot_ptr, _, s = run(lens, B, Hkv, n_slots=16, min_chunk=256, tile=16, policy=policy,
                                             overhead_tokens=10)
        assert s.max_slot_load == s.min_slot_load == 2 * (L + 10), policy
        loads = P.slot_loads(items, slot_ptr, 10)
        assert P.delta(loads) == 0 and P.efficiency(loads) == 1.0


def test_efficiency_and_delta_definitions_on_a_hand_example():
    # three devices with loads 4, 2, 2: E = (4/4 + 2/4 + 2/4) / 3 = 2/3 (eq. 5); delta = 2
    assert P.efficiency([4, 2, 2]) == pytest.approx(2.0 / 3.0)
    assert P.delta([4, 2, 2]) == 2
    assert P.efficiency([0, 0]) == 1.0


def test_single_heavy_head_is_shared_like_a_replicated_head():
    # one pair of 4096 tokens, 8 slots: Fair-Copying's W/copies => 8 chunks of 512, one per slot
    for policy in (P.POLICY_LPT_SPLIT, P.POLICY_FAIR):
        p, offs, items, slot_ptr, _, s = run([4096], 1, 1, n_slots=8, oversub=1, min_chunk=64, tile=64,
                                             overhead_tokens=0, policy=policy)
        assert sorted(it.tok_count for it in items) == [512] * 8
        assert slot_ptr == list(range(9))
        assert s.max_slot_load == s.min_slot_load == 512
        # the cap on copies (eq. 3) binds
        p, offs, items, *_ = run([4096], 1, 1, n_slots=8, oversub=1, min_chunk=64, tile=64, overhead_tokens=0,
                                 max_split=2, policy=policy)
        assert len(items) == 2 and sum(it.tok_count for it in items) == 4096
    # without splitting the whole head lands on one slot
    p, offs, items, slot_ptr, _, s = run([4096], 1, 1, n_slots=8, policy=P.POLICY_LPT, overhead_tokens=0)
    assert len(items) == 1 and s.max_slot_load == 4096 and s.min_slot_load == 0


def test_split_ragged_tail_and_tile_rounding():
    kw = dict(policy=P.POLICY_LPT_SPLIT, oversub=1, tile=64, overhead_tokens=0)
    # 1000 tokens, target 256 -> r = 4, cs = up(250) = 256, chunks 256,256,256,232
    p, offs, items, *_ = run([1000], 1, 1, n_slots=4, min_chunk=256, **kw)
    by_chunk = sorted(items, key=lambda x: x.part)
    assert [(x.row - offs[0], x.tok_count) for x in by_chunk] == [(0, 256), (256, 256), (512, 256), (768, 232)]
    # 130 tokens, target 64 -> r = 3, cs = up(44) = 64 -> 64, 64, 2
    p, offs, items, *_ = run([130], 1, 1, n_slots=100, min_chunk=64, **kw)
    assert sorted(x.tok_count for x in items) == [2, 64, 64]
    # 129 tokens, min_chunk 128 -> r = 2, cs = up(65) = 128 -> 128 + 1
    p, offs, items, *_ = run([129], 1, 1, n_slots=100, min_chunk=128, **kw)
    assert sorted(x.tok_count for x in items) == [1, 128]


def test_fair_cut_by_hand():
    # two slots, no overhead: 100 + 300 tokens -> budget 200: slot 0 = pair 0 whole + 96 of pair 1
    # (the 100 that fit, cut down to whole tiles of 16), slot 1 = the other 204
    p, offs, items, slot_ptr, part_base, s = run([100, 300], 2, 1, offs=[0, 1000], n_slots=2, tile=16, min_chunk=32,
                                                 overhead_tokens=0, policy=P.POLICY_FAIR)
    assert [it.astuple() for it in items] == [(0, 100, 0, 0, 0, 1, 0), (1000, 96, 1, 0, 0, 2, 1),
                                              (1096, 204, 1, 0, 1, 2, 2)]
    assert slot_ptr == [0, 2, 3] and part_base == [0, 1, 3]
    assert (s.max_slot_load, s.min_slot_load) == (204, 196)
    # room for 48 of the next 70 tokens: the rest (22) would be below min_chunk, and the excess is
    # smaller than the room, so the slot is overfilled with the whole pair
    p, offs, items, slot_ptr, *_ = run([150, 70, 180], 3, 1, n_slots=2, tile=16, min_chunk=32, overhead_tokens=0,
                                       policy=P.POLICY_FAIR)
    assert [(it.b, it.tok_count) for it in items] == [(0, 150), (1, 70), (2, 180)] and slot_ptr == [0, 2, 3]
    # room for nothing of the next 40 tokens: the slot is closed instead
    p, offs, items, slot_ptr, *_ = run([190, 40, 170], 3, 1, n_slots=2, tile=16, min_chunk=32, overhead_tokens=0,
                                       policy=P.POLICY_FAIR)
    assert [(it.b, it.tok_count) for it in items] == [(0, 190), (1, 40), (2, 170)] and slot_ptr == [0, 1, 3]
    # room for 48 of the next 100: both pieces are at least min_chunk, so the pair is cut
    p, offs, items, slot_ptr, *_ = run([150, 100, 150], 3, 1, n_slots=2, tile=16, min_chunk=32, overhead_tokens=0,
                                       policy=P.POLICY_FAIR)
    assert [(it.b, it.tok_count) for it in items] == [(0, 150), (1, 48), (1, 52), (2, 150)] and slot_ptr == [0, 2, 4]


def test_fair_balance_bound():
    # every slot but the last stays within min_chunk + tile + overhead of its budget, so the spread is small
    for name in ("llama70b", "mistral24b", "faircopy", "stress"):
        w = W.WORKLOADS[name]
        lens = W.lens(name)
        p, offs, items, slot_ptr, _, s = run(lens, w.B, w.Hkv, policy=P.POLICY_FAIR)
        ideal = -(-(s.total_tokens + p.overhead_tokens * len(items)) // p.n_slots)
        assert s.max_slot_load <= ideal + 2 * (p.min_chunk + p.tile + p.overhead_tokens)
        assert P.efficiency(P.slot_loads(items, slot_ptr, p.overhead_tokens)) > 0.85


def test_naive_policy_is_round_robin_in_pair_order():
    lens = [5, 0, 7, 9, 11]
    p, offs, items, slot_ptr, part_base, s = run(lens, 5, 1, n_slots=2, policy=P.POLICY_NAIVE, overhead_tokens=1)
    assert [(it.b, it.tok_count) for it in items] == [(0, 5), (2, 7), (4, 11), (1, 0), (3, 9)]
    assert slot_ptr == [0, 3, 5]
    assert s.max_slot_load == 5 + 7 + 11 + 3 and s.min_slot_load == 0 + 9 + 2
    assert part_base == [0, 1, 2, 3, 4, 5]


def test_lpt_order_and_tie_breaks():
    lens = [300, 500, 500, 100]
    p, offs, items, slot_ptr, *_ = run(lens, 2, 2, n_slots=2, policy=P.POLICY_LPT, overhead_tokens=0)
    # longest first; equal lengths by (b, h); each goes to the least loaded slot, lowest index on ties
    assert [(it.b, it.h) for it in items] == [(0, 1), (0, 0), (1, 0), (1, 1)] and slot_ptr == [0, 2, 4]


def _opt_makespan(costs, m):
    best = None
    for assign in itertools.product(range(m), repeat=len(costs)):
        load = [0] * m
        for c, j in zip(costs, assign):
            load[j] += c
        mk = max(load)
        best = mk if best is None else min(best, mk)
    return best


def test_lpt_within_graham_bound_of_brute_force_optimum():
    rng = np.random.default_rng(5)
    for _ in range(60):
        m = int(rng.integers(2, 4))
        n = int(rng.integers(1, 9))
        lens = rng.integers(1, 50, size=n)
        p, offs, items, slot_ptr, _, s = run(lens, n, 1, n_slots=m, policy=P.POLICY_LPT, overhead_tokens=0, tile=1,
                                             min_chunk=1)
        opt = _opt_makespan([int(x) for x in lens], m)
        assert opt <= s.max_slot_load
        assert 3 * m * s.max_slot_load <= (4 * m - 1) * opt      # makespan <= (4/3 - 1/(3m)) OPT


def test_balanced_gain_is_bounded_by_naive_idle_share():
    # the gain of balancing cannot exceed 1 / (efficiency of the unbalanced plan): the same
    # consistency that links the paper's busy rates (Table 2) to its 1.66x throughput gain
    for name in ("llama70b", "mistral24b", "stress"):
        w = W.WORKLOADS[name]
        lens = W.lens(name)
        _, _, it_n, sp_n, _, s_n = run(lens, w.B, w.Hkv, policy=P.POLICY_NAIVE, overhead_tokens=0)
        e_naive = P.efficiency(P.slot_loads(it_n, sp_n, 0))
        for policy in (P.POLICY_LPT_SPLIT, P.POLICY_FAIR):
            _, _, it_b, sp_b, _, s_b = run(lens, w.B, w.Hkv, policy=policy, overhead_tokens=0)
            assert s_n.max_slot_load / s_b.max_slot_load <= 1.0 / e_naive + 1e-9
            assert s_n.max_slot_load / s_b.max_slot_load >= 1.5


def test_determinism():
    lens = W.lens("stress")
    a = run(lens, 128, 8)
    b = run(lens, 128, 8)
    assert [x.astuple() for x in a[2]] == [x.astuple() for x in b[2]] and a[3:] == b[3:]


def test_rejects_bad_arguments():
    with pytest.raises(ValueError):
        run([1, -1], 2, 1)
    with pytest.raises(ValueError):
        run([1, 2], 2, 1, min_chunk=100, tile=64)
    with pytest.raises(ValueError):
        run([1, 2], 2, 1, n_slots=0)
    with pytest.raises(ValueError):
        run([1, 2, 3], 2, 1, offs=[0, 1, 2])
    with pytest.raises(ValueError):
        run([1, 2], 2, 1, policy=7)
    with pytest.raises(ValueError):
        run([1, 2], 2, 1, offs=[0, -5])
