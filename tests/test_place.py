"""fairkv_place (host code of the library, through the C ABI) against the placement oracle,
field by field, and its argument checks."""
import ctypes

import numpy as np
import pytest

import paper_2502_15804_amd as F
from oracle import placement as PL


def same_as_oracle(W, B, tp, m, R, mode):
    got = F.fairkv_place(W, B, tp, m, R, mode)
    shares, loads, s = PL.place([int(x) for x in W], B, PL.PlaceParams(tp, m, R, mode))
    ref = [(x.head, x.gpu, x.copy, x.n_copies, x.row_begin, x.row_end) for x in shares]
    assert [tuple(int(v) for v in r) for r in got.shares] == ref, (W, B, tp, m, R, mode)
    assert got.gpu_load.tolist() == loads
    g = got.summary
    assert (g.den, g.delta_num, g.max_load_num, g.min_load_num, g.n_shares, g.exact) == \
        (s.den, s.delta_num, s.max_load_num, s.min_load_num, s.n_shares, s.exact)
    assert g.efficiency == s.efficiency
    return got


def test_exhaustive_walk_matches_the_oracle_field_by_field():
    rng = np.random.default_rng(11)
    for _ in range(400):
        n = int(rng.integers(1, 7))
        W = rng.integers(0, int(rng.choice([4, 60, 5000])), size=n)
        same_as_oracle(W, int(rng.integers(1, 100)), int(rng.integers(1, 5)), int(rng.integers(0, 4)),
                       int(rng.integers(1, 5)), F.FAIRKV_PLACE_EXACT)


def test_greedy_and_auto_match_the_oracle_field_by_field():
    rng = np.random.default_rng(12)
    for _ in range(300):
        n = int(rng.integers(1, 40))
        W = np.asarray(rng.lognormal(6, 1.0, size=n), dtype=np.int64)
        mode = int(rng.choice([F.FAIRKV_PLACE_GREEDY, F.FAIRKV_PLACE_AUTO]))
        m = int(rng.integers(0, 9))
        if mode == F.FAIRKV_PLACE_AUTO and n + m <= 12:
            n, W = 13, np.asarray(rng.lognormal(6, 1.0, size=13), dtype=np.int64)   # keep the oracle's walk short
        same_as_oracle(W, int(rng.integers(1, 65)), int(rng.integers(1, 9)), m, int(rng.integers(1, 9)), mode)


def test_a_layer_of_eight_heads_on_four_and_eight_gpus():
    # the paper's own scale: 8 KV heads, a few copies; exact through AUTO
    W = [5200, 900, 760, 640, 520, 410, 300, 180]
    for tp, m, R in ((2, 0, 1), (4, 0, 1), (4, 2, 2), (8, 2, 4)):
        got = same_as_oracle(W, 32, tp, m, R, F.FAIRKV_PLACE_AUTO)
        assert got.summary.exact == 1
    base = F.fairkv_place(W, 32, 4, 0, 1)
    fair = F.fairkv_place(W, 32, 4, 3, 4)
    assert fair.summary.max_load_num / fair.summary.den < base.summary.max_load_num / base.summary.den
    assert fair.summary.efficiency > base.summary.efficiency


def test_argument_checks():
    L = F.lib()
    W = (ctypes.c_int64 * 3)(5, 1, 1)
    s = F.fairkv_place_summary()
    sh = (F.fairkv_share * 4)()

    def call(n=3, B=4, tp=2, m=1, R=2, mode=0, cap=4, w=W, shares=sh, summ=s):
        p = F.fairkv_place_params(tp, m, R, mode)
        return L.fairkv_place(w, n, B, ctypes.byref(p), shares, cap, None, ctypes.byref(summ) if summ is not None else None)

    assert call() == F.FAIRKV_OK
    assert call(cap=0, shares=None) == F.FAIRKV_ECAP and s.n_shares == 4
    for kw in (dict(n=0), dict(B=0), dict(tp=0), dict(m=-1), dict(R=0), dict(R=9), dict(mode=3), dict(w=None),
               dict(summ=None), dict(cap=2, shares=None)):
        assert call(**kw) == F.FAIRKV_EINVAL, kw
    bad = (ctypes.c_int64 * 3)(5, -1, 1)
    assert call(w=bad) == F.FAIRKV_EINVAL
    with pytest.raises(F.FairKVError):
        F.fairkv_place([1, 2], 0, 2)


def test_every_token_is_served_by_exactly_one_gpu_share():
    import workloads as W
    from paper_2502_15804_amd.runtime import gpu_share
    lens = W.lens("mistral24b")
    Wh = lens.astype(np.int64).sum(axis=0)
    for tp, m in ((2, 0), (4, 2), (8, 4)):
        pl = F.fairkv_place(Wh, lens.shape[0], tp, m, 4 if m else 1)
        seen = np.zeros_like(lens)
        for gpu in range(tp):
            heads, ll = gpu_share(lens, pl.shares, gpu)
            assert heads == sorted(set(heads)) and ll.shape == (lens.shape[0], len(heads))
            for col, h in enumerate(heads):
                assert ((ll[:, col] == lens[:, h]) | (ll[:, col] == 0)).all()
                seen[:, h] += ll[:, col]
        assert (seen == lens).all()
