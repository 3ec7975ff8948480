"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU code involved).

fairkv_plan.cpp, fairkv_place.cpp and the C oracle attn_ref.c are compiled with
-fsanitize=address,undefined into a small driver (sanitize_driver.cpp) whose buffers are sized exactly, so
that any read or write past an array, any signed overflow or misaligned access aborts the run.  The
planner and placement differential cases go through that build and are compared with the Python oracles
field by field; the attention oracle's sanitized build is compared with the ordinary build.
"""
import os
import subprocess

import numpy as np
import pytest

import workloads as W
from oracle import attention as OA
from oracle import placement as PL
from oracle import planner as P

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2502_15804_amd", "csrc")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    out = tmp_path_factory.mktemp("san")
    exe = str(out / "sanitize_driver")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]
    obj = str(out / "attn_ref.o")
    subprocess.run(["gcc", "-std=c11", "-fopenmp", *san, "-c", os.path.join(ROOT, "oracle", "attn_ref.c"), "-o", obj],
                   check=True, capture_output=True, text=True)
    res = subprocess.run(["g++", "-std=c++17", "-fopenmp", *san, "-static-libasan", "-I", os.path.join(ROOT, "include"),
                          os.path.join(ROOT, "tests", "sanitize_driver.cpp"), os.path.join(CSRC, "fairkv_plan.cpp"),
                          os.path.join(CSRC, "fairkv_place.cpp"), obj, "-o", exe, "-lm"],
                         capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return exe


def _run(exe, lines):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:verify_asan_link_order=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
    res = subprocess.run([exe], input="\n".join(lines) + "\n", capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0 and "ERROR: AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, \
        res.stderr[-4000:]
    out = res.stdout.strip().split("\n")
    assert len(out) == len(lines)
    return out


def _plan_line(cmd, B, Hkv, kw, cap_mode, lens, offs, tail=""):
    return (f"{cmd} {B} {Hkv} {kw['n_slots']} {kw['tile']} {kw['min_chunk']} {kw['max_split']} {kw['oversub']} "
            f"{kw['overhead_tokens']} {kw['policy']} {kw['short_overhead_tokens']} {int(cap_mode)} " + " ".join(str(int(x)) for x in lens) + " " +
            " ".join(str(int(x)) for x in offs) + tail)


def _plan_cases(rng, n):
    for _ in range(n):
        B, Hkv = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        lens = rng.integers(0, int(rng.choice([4, 300, 5000])), size=B * Hkv).astype(np.int32)
        tile = int(rng.choice([1, 16, 64]))
        kw = dict(n_slots=int(rng.choice([1, 2, 5, 64, 320])), tile=tile, min_chunk=tile * int(rng.integers(1, 5)),
                  max_split=int(rng.choice([1, 2, 8, 256])), oversub=int(rng.integers(1, 4)),
                  overhead_tokens=int(rng.choice([0, 16, 128])), policy=int(rng.integers(0, 4)),
                  short_overhead_tokens=int(rng.choice([0, 8, 48])))
        offs = W.packed_offsets(lens.reshape(B, Hkv), gap_rows=int(rng.integers(0, 3)))[0].reshape(-1)
        yield B, Hkv, kw, lens, offs


def test_planner_differential_cases_under_sanitizers(driver):
    rng = np.random.default_rng(31)
    cases = list(_plan_cases(rng, 300))
    lines = [_plan_line("plan", B, Hkv, kw, i % 5 == 4, lens, offs) for i, (B, Hkv, kw, lens, offs) in enumerate(cases)]
    # arguments the planner must refuse without touching anything
    lines.append("plan 1 1 0 16 32 8 2 128 3 0 0 5 0")
    lines.append("plan 1 2 4 16 24 8 2 128 3 0 0 5 7 0 5")
    lines.append("plan 1 1 4 16 32 8 2 128 3 0 0 -5 0")
    out = _run(driver, lines)
    assert out[-3:] == ["plan -1", "plan -1", "plan -1"]
    for i, ((B, Hkv, kw, lens, offs), got) in enumerate(zip(cases, out)):
        items, slot_ptr, part_base, s = P.plan(lens, offs, B, Hkv, P.Params(**kw))
        head, recs, sp, pb = [x.split() for x in got.split("|")]
        short = i % 5 == 4 and s.n_items > 0
        assert head[0] == "plan" and [int(x) for x in head[1:]] == [-2 if short else 0, s.n_items, s.n_parts,
                                                                     s.max_slot_load, s.min_slot_load]
        recs = [int(x) for x in recs]
        if short:      # the capacity error: no record was written
            assert recs[6::7] == [-99] * (s.n_items - 1)
        else:
            assert recs == [v for it in items for v in it.astuple()]
        assert [int(x) for x in sp] == slot_ptr and [int(x) for x in pb] == part_base


def test_plan_grow_under_sanitizers(driver):
    rng = np.random.default_rng(32)
    cases = list(_plan_cases(rng, 60))
    lines = [_plan_line("grow", B, Hkv, kw, 0, lens, offs, f" {3 + i % 4} {i % 3}") for i, (B, Hkv, kw, lens, offs) in
             enumerate(cases)]
    out = _run(driver, lines)
    for i, ((B, Hkv, kw, lens, offs), got) in enumerate(zip(cases, out)):
        items, *_ = P.plan(lens, offs, B, Hkv, P.Params(**kw))
        cur = [int(x) for x in lens]
        cap = [int(x) + i % 3 + j % 3 for j, x in enumerate(lens)]
        for _ in range(3 + i % 4):
            items = P.grow(items, cur, cap, Hkv)
        assert got.split() == ["grow", "0"] + [str(it.tok_count) for it in items]


def test_placement_differential_cases_under_sanitizers(driver):
    rng = np.random.default_rng(33)
    cases = []
    for i in range(160):
        if i % 2 == 0:       # the paper's scale: exhaustive
            n, m, mode = int(rng.integers(1, 7)), int(rng.integers(0, 4)), PL.MODE_EXACT
            Wt = rng.integers(0, int(rng.choice([4, 60, 5000])), size=n)
        else:
            n, m, mode = int(rng.integers(13, 40)), int(rng.integers(0, 9)), PL.MODE_GREEDY
            Wt = np.asarray(rng.lognormal(6, 1.0, size=n), dtype=np.int64)
        cases.append(([int(x) for x in Wt], int(rng.integers(1, 65)), int(rng.integers(1, 9 if i % 2 else 5)), m,
                      int(rng.integers(1, 9 if i % 2 else 5)), mode))
    lines = [f"place {len(Wt)} {B} {tp} {m} {R} {mode} " + " ".join(map(str, Wt)) for Wt, B, tp, m, R, mode in cases]
    lines.append("place 2 4 0 0 1 0 5 5")          # no GPUs: refused
    out = _run(driver, lines)
    assert out[-1] == "place -1"
    for (Wt, B, tp, m, R, mode), got in zip(cases, out):
        shares, loads, s = PL.place(Wt, B, PL.PlaceParams(tp, m, R, mode))
        head, recs, ld = [x.split() for x in got.split("|")]
        assert [int(x) for x in head[1:]] == [0, s.den, s.delta_num, s.max_load_num, s.min_load_num, s.n_shares, s.exact]
        assert [int(x) for x in recs] == [v for x in shares for v in (x.head, x.gpu, x.copy, x.n_copies, x.row_begin, x.row_end)]
        assert [int(x) for x in ld] == loads


def _lcg_stream(seed, n):
    x = np.uint64(seed)
    out = np.empty(n, np.float64)
    a, c = np.uint64(6364136223846793005), np.uint64(1442695040888963407)
    with np.errstate(over="ignore"):
        for i in range(n):
            x = x * a + c
            out[i] = (float(x >> np.uint64(11)) / 9007199254740992.0 - 0.5) * 4.0
    return out


def test_attention_oracle_under_sanitizers(driver):
    rng = np.random.default_rng(34)
    cases = []
    for i in range(12):
        B, Hkv, G, D = int(rng.integers(1, 4)), int(rng.integers(1, 4)), int(rng.choice([1, 2, 4])), int(rng.choice([4, 16, 64]))
        lens = rng.integers(0, 60, size=B * Hkv).astype(np.int32)
        lens[-1] = max(int(lens[-1]), 1)        # the last head ends exactly at the end of the K/V buffers
        cases.append((B, Hkv * G, Hkv, D, 1000 + i, lens))
    lines = [f"attn {B} {Hq} {Hkv} {D} {seed} " + " ".join(map(str, lens.tolist())) for B, Hq, Hkv, D, seed, lens in cases]
    out = _run(driver, lines)
    for (B, Hq, Hkv, D, seed, lens), got in zip(cases, out):
        rows = int(lens.sum())
        data = _lcg_stream(seed, B * Hq * D + 2 * rows * D)
        q = data[:B * Hq * D].reshape(B, Hq, D)
        k = data[B * Hq * D:B * Hq * D + rows * D].reshape(rows, D)
        v = data[B * Hq * D + rows * D:].reshape(rows, D)
        off = np.concatenate([[0], np.cumsum(lens)[:-1]]).astype(np.int64).reshape(B, Hkv)
        ro, rl = OA.attention(q, k, v, off, lens.reshape(B, Hkv), 1.0 / np.sqrt(D))
        name, rc, so, sl = got.split()
        assert name == "attn" and rc == "0"
        assert abs(float(so) - ro.sum()) <= 1e-9 * max(1.0, np.abs(ro).sum())
        assert abs(float(sl) - rl[np.isfinite(rl)].sum()) <= 1e-9 * max(1.0, np.abs(rl[np.isfinite(rl)]).sum())
