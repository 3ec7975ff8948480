#!/usr/bin/env python3
"""Benchmark: ragged per-head decode attention on one MI355X.

A step is one call of fairkv_decode_attn (one persistent kernel: split-KV decode with the
chunk merge folded in) on one layer's packed ragged KV cache.  Steps rotate over distinct layer buffers whose
total size is several times the GPU's 256 MB memory-side cache, so that the K/V rows of a
step are streamed from HBM and not from a cache.  Plans are built once per layer before
the timed region (budgets are static once the cache is compressed; the paper's scheme is a
static one, Section 4.1) and the planner's host time is reported separately.

Prints ONE JSON line.  value = algorithmic bytes per second over the whole timed region:
K and V rows of every retained token read once, q read once, out written once.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1280)
    ap.add_argument("--warmup", type=int, default=128)
    ap.add_argument("--workload", default="llama70b")
    ap.add_argument("--layers", type=int, default=0, help="distinct layer buffers to rotate over (0 = workload default)")
    ap.add_argument("--policy", type=int, default=3, help="0 naive, 1 LPT, 2 LPT with equal split, 3 fair line cut")
    ap.add_argument("--no-graph", action="store_true", help="enqueue from Python instead of replaying a HIP graph")
    ap.add_argument("--no-extras", action="store_true", help="skip the policy comparison and the CPU baseline")
    ap.add_argument("--cpu-seconds", type=float, default=12.0)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--q-len", type=int, default=1,
                    help="new tokens per sequence in one call (fairkv_decode_attn_multi): 8 heads x 2 tokens fill the "
                         "16 columns of a matrix-core tile; K and V are still streamed once")
    ap.add_argument("--kv-dtype", choices=("bf16", "fp8"), default="bf16",
                    help="fp8: the same workload with K and V stored as E4M3 bytes (fairkv_decode_attn_kv8); a side "
                         "measurement, never the headline")
    ap.add_argument("--latency-model", action="store_true",
                    help="instead of the benchmark: decode latency of one Llama-70B-shaped layer against batch size "
                         "and against a uniform per-head budget (the paper's Section 3.2 / Figure 2 experiment), "
                         "with least-squares lines L = alpha*B + beta and L = gamma*C + delta")
    ap.add_argument("--placement-table", action="store_true",
                    help="instead of the benchmark: place the KV heads of one mistral24b-shaped layer on 2, 4 and 8 "
                         "GPUs (static, Best-effort Assignment, Fair-Copying) with fairkv_place and time every GPU's "
                         "share on this GPU (the paper's Section 4.3; busy rate and step time per scheme)")
    ap.add_argument("--pack", action="store_true",
                    help="instead of the benchmark: time fairkv_pack (dense cache -> packed ragged cache) on the "
                         "llama70b budgets")
    ap.add_argument("--bf16-kernel", choices=("mfma", "valu"), default="mfma",
                    help="valu: the bf16 workload through the vector-ALU kernel (FAIRKV_BF16_VALU) instead of the "
                         "matrix-core kernel: the A/B measurement behind the choice of the matrix cores")
    ap.add_argument("--phases", action="store_true",
                    help="instead of the benchmark: one traced launch per layer (fairkv_decode_attn_trace) after a "
                         "warm rotation; prints where the time of a launch goes, per phase, from the GPU's wall clock")
    ap.add_argument("--plan-sweep", action="store_true",
                    help="instead of the benchmark: microseconds per layer of the four full-size workloads with the "
                         "planner's cost parameters (overhead_tokens, short_overhead_tokens, min_chunk) varied one at a "
                         "time around the defaults: the measurements the defaults of fairkv_default_params rest on")
    ap.add_argument("--probe-shapes", action="store_true",
                    help="instead of the benchmark: the do-nothing reader in other launch shapes (waves per workgroup, "
                         "ring stages, tile size, workgroups per compute unit) over the buffers of llama70b and mistral24b")
    ap.add_argument("--phases-raw", default=None, metavar="FILE.npz",
                    help="with --phases: also save the stamps of every workgroup and what its slot held")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MiB",
                    help="only run three plain device-to-device copies of this size and exit: a kernel of "
                         "known traffic for scaling the rocprofv3 FETCH_SIZE / WRITE_SIZE counters")
    for name in ("n_slots", "tile", "min_chunk", "max_split", "oversub", "overhead_tokens", "short_overhead_tokens"):
        ap.add_argument("--" + name.replace("_", "-"), type=int, default=None)
    return ap.parse_args()


KV8_PLAN_DEFAULTS = {"tile": 32, "min_chunk": 64, "overhead_tokens": 256}


class Rotation:
    """Distinct layer buffers of one workload, resident on the GPU, with their plans."""

    K_SCALE, V_SCALE = 0.02, 0.03      # per-tensor scales of the 8-bit variant (N(0,1) data: well inside +-448)

    def __init__(self, name, n_layers, seed, policy, overrides, q_len=1, kv8=False, bf16_on_valu=False):
        import numpy as np
        import torch
        import workloads as W
        import paper_2502_15804_amd as F
        from paper_2502_15804_amd.runtime import DecodeLayer, device_compute_units

        self.w = W.WORKLOADS[name]
        self.n_cu = device_compute_units()
        self.params = F.fairkv_default_params(self.n_cu, policy=policy, **overrides)
        self.lens, self.offs, self.layers, self.bytes = [], [], [], []
        plan_times = []
        need = 0
        for li in range(n_layers):
            lens = W.lens(name, seed=seed, layer=li)
            off, _ = W.packed_offsets(lens)
            t0 = time.perf_counter()
            plan = F.fairkv_plan(lens, off, self.w.B, self.w.Hkv, self.params)
            plan_times.append(time.perf_counter() - t0)
            need = max(need, F.fairkv_workspace_bytes(plan.n_parts, self.w.B * self.w.Hkv, self.w.G * q_len, self.w.D))
        self.workspace = torch.zeros(need, dtype=torch.uint8, device="cuda")   # shared by all layers, one stream
        for li in range(n_layers):
            lens = W.lens(name, seed=seed, layer=li)
            off, total = W.packed_offsets(lens)
            q, k, v = W.make_qkv(self.w, total, seed=seed, layer=li, device="cuda")
            if q_len > 1:       # q_len new tokens per sequence; their K/V are the last rows of every pair already
                gq = torch.Generator(device="cuda").manual_seed(1000 * seed + li)
                q = torch.randn((self.w.B, q_len, self.w.Hq, self.w.D), generator=gq, device="cuda").to(q.dtype)
            if kv8:
                k, v = W.make_kv8(self.w, total, self.K_SCALE, self.V_SCALE, seed=seed, layer=li, device="cuda")
            self.layers.append(DecodeLayer(q, k, v, off, lens, self.w.scale, params=self.params,
                                           workspace=self.workspace, k_scale=self.K_SCALE, v_scale=self.V_SCALE,
                                           bf16_on_valu=bf16_on_valu))
            self.lens.append(lens)
            self.offs.append(off)
            self.bytes.append(W.algorithmic_bytes(self.w, lens) + (q_len - 1) * self.w.B * self.w.Hq * self.w.D *
                              (self.w.elem_bytes + 4)
                              - (int(lens.astype(np.int64).sum()) * self.w.D * 2 * (self.w.elem_bytes - 1) if kv8 else 0))
        self.plan_us = 1e6 * sorted(plan_times)[len(plan_times) // 2]
        torch.cuda.synchronize()

    def run_eager(self, first, count):
        n = len(self.layers)
        for i in range(first, first + count):
            self.layers[i % n].run()

    def capture(self, count):
        """A HIP graph of `count` launches: layers 0 .. count-1 of the rotation."""
        import torch
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            self.run_eager(0, count)                   # load code objects before capturing
        torch.cuda.current_stream().wait_stream(s)
        torch.cuda.synchronize()
        with torch.cuda.graph(g):
            self.run_eager(0, count)
        return g


MAX_GRAPH_LAUNCHES = 4096      # longest graph the timed region is captured as (replays of a rotation beyond that)


def timed(rot, steps, warmup, use_graph):
    """Returns (seconds by host clock, seconds by HIP events, bytes moved) for exactly `steps` steps.

    With use_graph the timed region consists of graph replays only, whatever `steps` is: up to MAX_GRAPH_LAUNCHES
    steps are one replay of one graph of exactly that many launches (the launches rotate over the layers); longer
    runs replay a graph of one rotation and a graph of the remainder.  Without it every step is enqueued from Python."""
    import torch
    n = len(rot.layers)
    full, rest = divmod(steps, n)
    if use_graph and steps <= MAX_GRAPH_LAUNCHES:
        full, rest = 0, steps                  # one graph of exactly `steps` launches, rotating over the layers
    g_full = rot.capture(n) if (use_graph and full) else None
    g_rest = rot.capture(rest) if (use_graph and rest) else None

    def go(count_full, count_rest):
        if use_graph:
            for _ in range(count_full):
                g_full.replay()
            if count_rest:
                g_rest.replay()
        else:
            rot.run_eager(0, count_full * n + count_rest)

    rot.run_eager(0, warmup)                   # the W untimed steps, then one untimed pass of what is timed
    go(min(full, 1), rest)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    go(full, rest)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    moved = full * sum(rot.bytes) + sum(rot.bytes[i % n] for i in range(rest))
    return t1 - t0, e0.elapsed_time(e1) * 1e-3, moved


def measured_traffic(workload):
    """(HBM bytes per launch, file) from the committed rocprofv3 counter summary of this workload, or (None, None).
    Counters cannot be read from inside the timed run: the figure is the one of the summary under profiles/,
    which names the commands that made it, and the JSON line says so."""
    rel = os.path.join("profiles", f"fairkv_decode_mfma_kernel_{workload}.txt")
    try:
        for line in open(os.path.join(ROOT, rel)):
            if line.strip().startswith("traffic_bytes_per_launch:"):
                return int(line.split(":")[1]), rel
    except OSError:
        pass
    return None, None


def spot_check(rot, n_layers=2, n_samples=48, ran=None):
    """After the timed region: sampled outputs of a few layers, as the timed launches left them,
    against the oracle (the same launch configuration that was timed).  `ran`: how many layers of the
    rotation the timed region launched, when it was shorter than one rotation."""
    import numpy as np
    import workloads as W
    from oracle import attention as OA

    worst = 0.0
    rng = np.random.default_rng(0)
    ran = min(ran or len(rot.layers), len(rot.layers))
    for li in sorted({0, ran - 1, ran // 2})[:max(1, n_layers + 1)]:
        layer = rot.layers[li]
        sel = rng.choice(rot.w.B * rot.w.Hq, size=min(n_samples, rot.w.B * rot.w.Hq), replace=False).astype(np.int32)
        got = layer.out.float().cpu().numpy().astype(np.float64).reshape(-1, rot.w.D)
        if layer.kv8:            # every output of one layer: the oracle decodes the whole cache anyway
            ro, _ = OA.attention_kv8(W.to_numpy_bits(layer.q), layer.k.cpu().numpy(), layer.v.cpu().numpy(), rot.offs[li],
                                     rot.lens[li], rot.w.scale, layer.k_scale, layer.v_scale)
            return float(np.abs(got - ro.reshape(-1, rot.w.D)).max())
        bits = [W.to_numpy_bits(t) for t in (layer.q, layer.k, layer.v)]
        if layer.q_len > 1:      # every output: the oracle for several new tokens has no selection list
            ro, _ = OA.attention_multi(*bits, rot.offs[li], rot.lens[li], rot.w.scale)
            worst = max(worst, float(np.abs(got - ro.reshape(-1, rot.w.D)).max()))
            continue
        ro, _ = OA.attention(*bits, rot.offs[li], rot.lens[li], rot.w.scale, sel=sel)
        worst = max(worst, float(np.abs(got[sel] - ro.reshape(-1, rot.w.D)[sel]).max()))
    return worst


def graph_time_us(layers, bytes_layer):
    """Microseconds per launch of a rotation of DecodeLayer objects, replayed as one HIP graph."""
    import torch
    n_buf = len(layers)
    g = torch.cuda.CUDAGraph()
    for l in layers:
        l.run()
    torch.cuda.synchronize()
    with torch.cuda.graph(g):
        for l in layers:
            l.run()
    reps = max(3, int(2e-3 / (n_buf * max(bytes_layer, 1) / 4e12)))
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return 1e3 * e0.elapsed_time(e1) / (reps * n_buf)


def placement_table(seed=0, name="mistral24b"):
    """Section 4.3 / Section 5 of the paper at kernel level on this GPU: the KV heads of one layer are placed
    on tp GPUs by static head allocation, by Best-effort Assignment (no copies) and by Fair-Copying with up to
    CH extra copies (fairkv_place); every GPU's share then runs through fairkv_plan + fairkv_decode_attn here,
    one share at a time, and the step time of the group is the slowest share's.  Busy rate = mean / max."""
    import numpy as np
    import workloads as W
    import paper_2502_15804_amd as F
    from paper_2502_15804_amd.runtime import DecodeLayer, gpu_share

    w0 = W.WORKLOADS[name]
    # four layers' budgets stacked as batch rows: B = 128, so that a GPU's share of one layer is tens of MB
    lens = np.concatenate([W.lens(name, seed=seed, layer=i) for i in range(4)], axis=0)
    w = W.Workload(name, lens.shape[0], w0.Hq, w0.Hkv, w0.D, w0.dtype, 1, w0.tol, "")
    Wh = lens.astype(np.int64).sum(axis=0)
    rows = []

    def run_scheme(tp, label, shares, eff_model):
        times = []
        for gpu in range(tp):
            heads, ll = gpu_share(lens, shares, gpu)
            if not heads:
                times.append(0.0)
                continue
            wl = W.Workload("share", w.B, len(heads) * w.G, len(heads), w.D, w.dtype, 1, w.tol, "")
            off, total = W.packed_offsets(ll)
            bytes_layer = W.algorithmic_bytes(wl, ll)
            n_buf = max(2, min(48, int(1.0e9 // max(bytes_layer, 1)) + 1))
            layers = []
            for i in range(n_buf):
                q, k, v = W.make_qkv(wl, max(total, 1), seed=seed, layer=i, device="cuda")
                layers.append(DecodeLayer(q, k, v, off, ll, wl.scale, want_lse=False))
            times.append(graph_time_us(layers, bytes_layer))
            del layers
        mx = max(times)
        rows.append({"tp": tp, "scheme": label, "copies": int(len(shares) - len(Wh)),
                     "efficiency_model": round(eff_model, 4), "busy_rate_measured": round(float(np.mean(times)) / mx, 4),
                     "step_us": round(mx, 2), "per_gpu_us": [round(t, 2) for t in times]})

    for tp in (2, 4, 8):
        per = len(Wh) // tp
        sha = np.zeros(len(Wh), dtype=F.SHARE_DTYPE)
        for h in range(len(Wh)):
            sha[h] = (h, h // per, 0, 1, 0, w.B)
        loads = [int(Wh[j * per:(j + 1) * per].sum()) for j in range(tp)]
        run_scheme(tp, "static", sha, sum(loads) / (tp * max(loads)))
        for ch in (0, 1, 2, 4):
            pl = F.fairkv_place(Wh, w.B, tp, ch, 4 if ch else 1)
            run_scheme(tp, "best-effort" if ch == 0 else f"fair-copying CH<={ch}", pl.shares, pl.summary.efficiency)
    for tp in (2, 4, 8):
        base = [r for r in rows if r["tp"] == tp and r["scheme"] == "static"][0]["step_us"]
        for r in rows:
            if r["tp"] == tp:
                r["speedup_vs_static"] = round(base / r["step_us"], 3)
    return {"experiment": "head placement over a tensor-parallel group, each GPU's share timed on this GPU "
                          "(paper Section 4.3 and Figure 4 / Table 2 analogue)",
            "profile": f"{name} recipe, B={w.B}: summed budgets per KV head = {Wh.tolist()}", "rows": rows}


def pack_bench(seed=0, name="llama70b", T=8192, n_slots=None):
    """The step before the path: fairkv_pack gathers the kept rows of a dense [B][Hkv][T][D] cache into the
    packed layout.  Bytes per token moved: K and V rows read and written once plus the 4-byte index."""
    import numpy as np
    import torch
    import workloads as W
    import paper_2502_15804_amd as F
    from paper_2502_15804_amd.runtime import device_compute_units

    w = W.WORKLOADS[name]
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    sets, moved = [], 0
    n_slots = n_slots or 8 * device_compute_units()
    for li in range(3):                                   # 3 x 0.5 GB of dense cache: past the memory-side cache
        lens = W.lens(name, seed=seed, layer=li)
        keep_ptr, keep_t = W.keep_lists(lens, T, seed=seed + li)
        off, total = W.packed_offsets(lens)
        plan = F.fairkv_plan(lens, off, w.B, w.Hkv, F.fairkv_default_params(n_slots, overhead_tokens=16, min_chunk=64))
        kd = torch.randn((w.B, w.Hkv, T, w.D), device="cuda", dtype=torch.float32).to(tdt)
        vd = torch.randn((w.B, w.Hkv, T, w.D), device="cuda", dtype=torch.float32).to(tdt)
        dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
        sets.append((kd, vd, dev(keep_ptr), dev(keep_t), dev(off.reshape(-1)), dev(plan.items.view(np.uint8).copy()),
                     dev(plan.slot_ptr), torch.empty((total, w.D), dtype=tdt, device="cuda"),
                     torch.empty((total, w.D), dtype=tdt, device="cuda")))
        moved += int(lens.sum()) * (4 * w.D * w.elem_bytes + 4)
    bad = torch.zeros(1, dtype=torch.int32, device="cuda")

    def run_all():
        for s in sets:
            F.fairkv_pack(*s, bad)

    run_all()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 20
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) * 1e-3 / reps
    assert int(bad.item()) == 0
    gbs = moved / sec / 1e9
    return {"experiment": "fairkv_pack: gather of the kept rows of a dense cache into the packed ragged layout",
            "config": {"workload": f"{name} budgets out of a dense cache of T={T} tokens per pair", "n_slots": n_slots,
                       "layers": len(sets)},
            "us_per_layer": round(1e6 * sec / len(sets), 2), "value": round(gbs, 1), "unit": "GB/s",
            "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                         "frac": round(gbs / HBM_PEAK_GBS, 4), "traffic": None,
                         "kernel": f"fairkv_pack_kernel<{w.D * w.elem_bytes}>", "bytes_per_launch": moved // len(sets)}}


def latency_model(seed=0):
    """Section 3.2 of the paper on this GPU: one layer (64 query / 8 KV heads, D=128, bf16), every head with the
    same budget C, batch B; time per decode step through the whole path (plan resident, one launch)."""
    import numpy as np
    import torch
    import workloads as W
    from paper_2502_15804_amd.runtime import DecodeLayer

    budgets, batches = (128, 256, 512, 1024), (32, 64, 128, 256, 512)
    table = {}
    for B in batches:
        for C in budgets:
            w = W.Workload("uniform", B, 64, 8, 128, "bf16", 1, 1e-2, "")
            lens = np.full((B, 8), C, np.int32)
            off, total = W.packed_offsets(lens)
            bytes_layer = W.algorithmic_bytes(w, lens)
            n_buf = max(2, min(16, int(1.5e9 // bytes_layer) + 1))      # rotate past the memory-side cache
            layers = []
            for i in range(n_buf):
                q, k, v = W.make_qkv(w, total, seed=seed, layer=i, device="cuda")
                layers.append(DecodeLayer(q, k, v, off, lens, w.scale, want_lse=False))
            us = graph_time_us(layers, bytes_layer)
            table[(B, C)] = (us, bytes_layer / us / 1e3)
            del layers
            torch.cuda.empty_cache()

    def fit(xs, ys):
        A = np.vstack([xs, np.ones(len(xs))]).T
        (a, b), res, *_ = np.linalg.lstsq(A, ys, rcond=None)
        ss = float(((ys - ys.mean()) ** 2).sum())
        r2 = 1.0 - float(((A @ [a, b] - ys) ** 2).sum()) / ss if ss > 0 else 1.0
        return float(a), float(b), r2

    rec = {"experiment": "decode latency of one layer vs batch size and vs per-head budget (paper Section 3.2)",
           "shape": "64 query / 8 KV heads, D=128, bf16, uniform budget per head", "unit": "us per layer",
           "latency_us": {f"B={B}": {f"C={C}": round(table[(B, C)][0], 2) for C in budgets} for B in batches},
           "GBs": {f"B={B}": {f"C={C}": round(table[(B, C)][1]) for C in budgets} for B in batches},
           "vs_batch": {}, "vs_budget": {}}
    for C in budgets:
        a_, b_, r2 = fit(np.array(batches, float), np.array([table[(B, C)][0] for B in batches]))
        rec["vs_batch"][f"C={C}"] = {"alpha_us_per_seq": round(a_, 4), "beta_us": round(b_, 2), "r2": round(r2, 5)}
    for B in batches:
        a_, b_, r2 = fit(np.array(budgets, float), np.array([table[(B, C)][0] for C in budgets]))
        rec["vs_budget"][f"B={B}"] = {"gamma_us_per_token": round(a_, 5), "delta_us": round(b_, 2), "r2": round(r2, 5)}
    return rec


def stream_probe(rot, gbs, shape=None, wg_per_cu=1):
    """The same K/V bytes of the same rotation through fairkv_stream_probe: a reader with the decode kernel's
    data path and launch shape and nothing to do.  Its rate is the ceiling this path can reach for this size.
    shape = (waves, stages, tile_kib) and wg_per_cu select another launch shape (fairkv_stream_probe_shape)."""
    import torch
    import paper_2502_15804_amd as F

    sink = torch.zeros(rot.n_cu * wg_per_cu, dtype=torch.int32, device="cuda")
    n = len(rot.layers)

    def run_all():
        for l in rot.layers:
            F.fairkv_stream_probe(l.k, l.v, rot.n_cu * wg_per_cu, sink, shape=shape)

    run_all()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_all()
    g.replay()
    torch.cuda.synchronize()
    reps = max(3, 640 // n)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    sec = e0.elapsed_time(e1) * 1e-3 / (reps * n)
    kv_bytes = sum(2 * l.k.numel() * l.k.element_size() for l in rot.layers) / n
    return {"us_per_layer": round(1e6 * sec, 2), "GBs": round(kv_bytes / sec / 1e9, 1),
            "decode_rate_over_probe_rate": round(gbs / (kv_bytes / sec / 1e9), 3),
            "what": "K and V of the same layers streamed HBM -> LDS by 256 workgroups, nothing computed or written"}


def cpu_baseline(rot, seconds):
    """The fp64 oracle, as it stands, on the host cores: whole layers of the same workload."""
    import workloads as W
    from oracle import attention as OA

    done_bytes, spent, n_done = 0, 0.0, 0
    threads = OA.max_threads()
    host = [tuple(W.to_numpy_bits(t) for t in (l.q, l.k, l.v)) for l in rot.layers[:8]]
    while spent < seconds:
        li = n_done % len(host)
        q, k, v = host[li]
        t0 = time.perf_counter()
        OA.attention(q, k, v, rot.offs[li], rot.lens[li], rot.w.scale)
        spent += time.perf_counter() - t0
        done_bytes += rot.bytes[li]
        n_done += 1
    q, k, v = host[0]                                     # the same oracle on one core, one layer
    t0 = time.perf_counter()
    OA.attention(q, k, v, rot.offs[0], rot.lens[0], rot.w.scale, n_threads=1)
    one = time.perf_counter() - t0
    return {"value": round(done_bytes / spent / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
            "sample": f"{n_done} whole-layer passes over {len(host)} layer(s) of {rot.w.name}, every output, {spent:.1f} s",
            "ms_per_layer": round(1e3 * spent / n_done, 2), "ms_per_layer_one_core": round(1e3 * one, 1)}


def cold_launch_us(rot):
    """A launch whose K/V are in no cache: every launch is preceded by a 1 GB fill, both replayed as one HIP
    graph; the time of the fills alone (a second graph) is subtracted."""
    import torch
    junk = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
    layers = rot.layers[:8]

    def graph_of(with_launches):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for l in layers:
                junk.fill_(1)
                if with_launches:
                    l.run()
        return g

    def time_of(g):
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return 1e3 * e0.elapsed_time(e1) / (5 * len(layers))

    for l in layers:
        l.run()
    torch.cuda.synchronize()
    return round(time_of(graph_of(True)) - time_of(graph_of(False)), 2)


def max_split_sweep(a, n_layers, overrides, gbs_fair):
    """Fair-Copying as the paper states it (equal shares, Algorithm 2's W / copies) with the cap on copies per
    pair swept: the one-GPU analogue of the paper's sweep over the count of copied heads (Section 5.2.1)."""
    import torch
    out = {}
    for ms in (1, 2, 4, 8, 16, 64):
        ov = dict(overrides)
        ov["max_split"] = ms
        r2 = Rotation(a.workload, n_layers, a.seed, 2, ov)
        _, ev2, moved2 = timed(r2, max(n_layers * 4, 64), n_layers, not a.no_graph)
        out[f"max_split={ms}"] = round(moved2 / ev2 / 1e9, 1)
        del r2
        torch.cuda.empty_cache()
    out["fair_line_cut"] = round(gbs_fair, 1)
    return out


def uniform_same_bytes(rot, seed):
    """A layer of about the same bytes as the workload's, perfectly balanced and with nothing to merge: one whole
    pair per slot, all of one length.  What the same kernel needs when raggedness costs nothing."""
    import numpy as np
    import torch
    import workloads as W
    from paper_2502_15804_amd.runtime import DecodeLayer

    w = rot.w
    n_slots = int(rot.params.n_slots)
    B = max(1, n_slots // w.Hkv)
    C = int(round(float(np.mean([l.sum() for l in rot.lens])) / (B * w.Hkv) / 16.0)) * 16
    wu = W.Workload("uniform", B, w.Hq, w.Hkv, w.D, w.dtype, 1, w.tol, "")
    lens = np.full((B, w.Hkv), C, np.int32)
    off, total = W.packed_offsets(lens)
    nbytes = W.algorithmic_bytes(wu, lens)
    layers = []
    for i in range(max(2, min(32, int(2.0e9 // nbytes)))):
        q, k, v = W.make_qkv(wu, total, seed=seed, layer=i, device="cuda")
        layers.append(DecodeLayer(q, k, v, off, lens, wu.scale, params=rot.params, want_lse=True))
    us = graph_time_us(layers, nbytes)
    items = layers[0].plan.n_items
    del layers
    torch.cuda.empty_cache()
    return {"us_per_layer": round(us, 2), "GBs": round(nbytes / us / 1e3, 1), "B": B, "tokens_per_pair": C,
            "bytes_per_launch": nbytes, "items": items,
            "what": "same kernel, same plan parameters, one whole pair of equal length per slot: balanced, nothing to merge"}


def other_workloads(a, overrides):
    """The other full-size workloads through the same path and the same timing (graph replays over their own
    rotation of distinct layers): microseconds per layer, GB/s and fraction of the HBM peak."""
    import torch
    import workloads as W
    out = {}
    for name in ("mistral24b", "faircopy", "stress"):
        if name == a.workload:
            continue
        n = W.WORKLOADS[name].n_layers
        r = Rotation(name, n, a.seed, a.policy, overrides)
        steps = max(4 * n, 128) // n * n
        _, ev, moved = timed(r, steps, n, not a.no_graph)
        gbs = moved / ev / 1e9
        err = spot_check(r, n_layers=1, n_samples=32)
        out[name] = {"us_per_layer": round(1e6 * ev / steps, 2), "GBs": round(gbs, 1), "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
                     "bytes_per_launch": round(moved / steps), "layers_rotated": n, "rotation_GB": round(sum(r.bytes) / 1e9, 3),
                     "steps": steps, "items_layer0": r.layers[0].plan.n_items, "spot_check_max_abs_err": round(err, 6)}
        if not err <= W.WORKLOADS[name].tol:
            print(f"bench: {name}: outputs of the timed launches are off by {err}", file=sys.stderr)
            sys.exit(1)
        del r
        torch.cuda.empty_cache()
        if a.policy == 3:      # the same kernel with one whole pair per workgroup: the balanced-against-naive gain here too
            r0 = Rotation(name, n, a.seed, 0, overrides)
            _, ev0, moved0 = timed(r0, steps, n, not a.no_graph)
            out[name]["naive_GBs"] = round(moved0 / ev0 / 1e9, 1)
            out[name]["gain_vs_naive"] = round(gbs / (moved0 / ev0 / 1e9), 3)
            del r0
            torch.cuda.empty_cache()
    return out


def phases(a, overrides):
    """Where the time of one launch goes: every layer of a warm rotation is launched once through
    fairkv_decode_attn_trace (the same kernel with wall-clock stamps), preceded by the untraced launch of the
    layer before it so that the GPU is in the state of a running rotation."""
    import numpy as np
    import torch
    import paper_2502_15804_amd as F

    w_name = a.workload
    rot = Rotation(w_name, a.layers or min(16, __import__("workloads").WORKLOADS[w_name].n_layers), a.seed, a.policy, overrides)
    n_slots = int(rot.params.n_slots)
    S = F.FAIRKV_TRACE_STAMPS
    for _ in range(3):
        rot.run_eager(0, len(rot.layers))
    torch.cuda.synchronize()
    names = ["start", "item list ready", "first tile landed", "first item streamed (wave 0)", "first item finished",
             "last item streamed (wave 0)", "hand-over begins", "partials' stores issued", "counted in", "merged",
             "hand-over ends", "end"]
    per_layer = []
    rows = {k: [] for k in ("has_handover", "merges", "n_items", "tokens", "n_cut", "n_solo", "n_whole")}
    for li, layer in enumerate(rot.layers):
        trace = torch.zeros(n_slots * S, dtype=torch.int64, device="cuda")
        rot.layers[li - 1].run()                      # keeps the pipeline as in a running rotation
        layer.run(trace=trace)
        torch.cuda.synchronize()
        t = trace.cpu().numpy().reshape(n_slots, S).astype(np.float64)
        used = t[:, 0] > 0
        t0 = t[used, 0].min()
        us = np.where(t > 0, (t - t0) / 100.0, np.nan)          # 100 MHz wall clock
        per_layer.append(us)
        pl = layer.plan
        cnt = np.diff(pl.slot_ptr)
        rows["n_items"].append(cnt)
        rows["tokens"].append(np.array([pl.items["tok_count"][pl.slot_ptr[j]:pl.slot_ptr[j + 1]].sum() for j in range(n_slots)]))
        it = pl.items
        solo_max = 96                                            # whole pairs up to this many tokens run on one wave
        for key, mask in (("n_cut", it["n_chunks"] > 1), ("n_solo", (it["n_chunks"] == 1) & (it["tok_count"] <= solo_max)),
                          ("n_whole", (it["n_chunks"] == 1) & (it["tok_count"] > solo_max))):
            csum = np.concatenate([[0], np.cumsum(mask.astype(np.int64))])
            rows[key].append(csum[pl.slot_ptr[1:]] - csum[pl.slot_ptr[:-1]])
        rows["has_handover"].append(~np.isnan(us[:, 6]))
        rows["merges"].append((us[:, 9] - us[:, 8]) > 0.15)
    us = np.stack(per_layer)                                      # [layers, slots, stamps]
    q = lambda x, p: float(np.nanpercentile(x, p))
    table = {}
    for k, nm in enumerate(names):
        col = us[:, :, k]
        table[nm] = {"median": round(q(col, 50), 2), "p90": round(q(col, 90), 2), "max_mean_over_layers": round(float(np.nanmean(np.nanmax(col, axis=1))), 2)}
    ho = np.concatenate([u[:, 10] - u[:, 6] for u in per_layer])
    merged = np.concatenate(rows["merges"])
    has = np.concatenate(rows["has_handover"])
    span = float(np.mean([np.nanmax(u[:, 11]) for u in per_layer]))
    stream_end = np.stack([u[:, 5] for u in per_layer])
    rec = {"experiment": "phases of one launch by the GPU's 100 MHz wall clock (fairkv_decode_attn_trace), microseconds "
                         "since the launch's first stamp; per workgroup, pooled over the layers",
           "workload": w_name, "layers": len(rot.layers), "n_slots": n_slots, "stamps": table,
           "launch_span_us_mean": round(span, 2),
           "last_item_streamed_spread_us": {"p10": round(q(stream_end, 10), 2), "median": round(q(stream_end, 50), 2),
                                            "p90": round(q(stream_end, 90), 2), "max_mean": round(float(np.nanmean(np.nanmax(stream_end, axis=1))), 2)},
           "hand_over_us": {"workgroups_with_one": int(has.sum()), "that_merged": int((merged & has).sum()),
                            "median_no_merge": round(q(ho[has & ~merged], 50), 2) if (has & ~merged).any() else None,
                            "median_merge": round(q(ho[has & merged], 50), 2) if (has & merged).any() else None,
                            "p90_merge": round(q(ho[has & merged], 90), 2) if (has & merged).any() else None},
           "steps_of_the_hand_over_us_median": {
               "publish (issue stores)": round(q(np.concatenate([u[:, 7] - u[:, 6] for u in per_layer]), 50), 2),
               "count in (one atomic round trip)": round(q(np.concatenate([u[:, 8] - u[:, 7] for u in per_layer]), 50), 2),
               "merge, for those that merge": round(q(np.concatenate([u[:, 9] - u[:, 8] for u in per_layer])[merged & has], 50), 2) if (merged & has).any() else None},
           }
    n_items = np.concatenate(rows["n_items"])
    dur = np.concatenate([u[:, 11] - u[:, 0] for u in per_layer])
    # least squares: what a token and an item of each kind cost a slot (the planner's cost model, Section 3.2's
    # L = gamma C + delta at the level of one workgroup); the streaming part alone, and up to the end
    feats = np.stack([np.ones_like(dur), np.concatenate(rows["tokens"]).astype(float), np.concatenate(rows["n_cut"]).astype(float),
                      np.concatenate(rows["n_whole"]).astype(float), np.concatenate(rows["n_solo"]).astype(float)], axis=1)
    ok_rows = ~np.isnan(dur)
    fit = {}
    for label, y in (("until_end", dur), ("until_last_item_streamed", np.concatenate([u[:, 5] - u[:, 0] for u in per_layer]))):
        m = ok_rows & ~np.isnan(y)
        use = [j for j in range(feats.shape[1]) if feats[m, j].std() > 0 or j == 0]
        coef, *_ = np.linalg.lstsq(feats[m][:, use], y[m], rcond=None)
        full = dict(zip([["fixed_us", "us_per_token", "us_per_cut_piece", "us_per_whole_pair", "us_per_short_pair"][j] for j in use],
                        [round(float(c), 4) for c in coef]))
        if full.get("us_per_token", 0) > 0:
            for k_ in list(full):
                if k_.startswith("us_per_") and k_ != "us_per_token":
                    full[k_.replace("us_per_", "tokens_per_")] = round(full[k_] / full["us_per_token"], 1)
        resid = y[m] - feats[m][:, use] @ coef
        full["residual_rms_us"] = round(float(np.sqrt((resid ** 2).mean())), 3)
        fit[label] = full
    rec["slot_time_model"] = fit
    if a.phases_raw:
        np.savez_compressed(a.phases_raw, us=us, tokens=np.stack(rows["tokens"]), n_cut=np.stack(rows["n_cut"]),
                            n_whole=np.stack(rows["n_whole"]), n_solo=np.stack(rows["n_solo"]), merges=np.stack(rows["merges"]),
                            max_chunks=np.stack([np.array([l.plan.items["n_chunks"][l.plan.slot_ptr[j]:l.plan.slot_ptr[j + 1]].max(initial=0)
                                                           for j in range(n_slots)]) for l in rot.layers]))
    rec["by_items_in_slot"] = {str(int(k)): {"slots": int((n_items == k).sum()), "median_us": round(q(dur[n_items == k], 50), 2),
                                             "median_tokens": int(np.median(np.concatenate(rows["tokens"])[n_items == k]))}
                               for k in np.unique(n_items) if (n_items == k).sum() >= 8}
    return rec


def probe_shapes(a):
    """What the data path reaches as a function of the launch shape: waves per workgroup, ring stages, tile size
    and workgroups per compute unit, hence bytes in flight per compute unit, on the K/V buffers of two workloads."""
    import torch

    out = {"experiment": "fairkv_stream_probe_shape over the layer buffers of a rotation, HIP-graph replay; "
                         "us per layer and GB/s of K+V bytes", "shapes": {}}
    shapes = [(4, 2, 2, 1), (4, 4, 2, 1), (4, 2, 4, 1), (4, 3, 4, 1), (4, 4, 4, 1), (4, 2, 8, 1),
              (8, 2, 2, 1), (8, 4, 2, 1), (8, 2, 4, 1), (16, 2, 2, 1),
              (4, 2, 2, 2), (4, 4, 2, 2), (4, 2, 4, 2), (4, 2, 2, 4)]
    shapes = [x for x in shapes if x[0] * x[1] * 2 * x[2] * x[3] <= 160]      # rings side by side in 160 KB of LDS
    for name, nl in (("llama70b", 32), ("mistral24b", 8)):
        rot = Rotation(name, nl, a.seed, 3, {})
        res = {}
        for waves, stages, kib, per_cu in shapes:
            r = min((stream_probe(rot, 1.0, (waves, stages, kib), per_cu) for _ in range(3)), key=lambda x: x["us_per_layer"])
            key = f"{waves} waves x {stages} stages x 2x{kib} KiB, {per_cu} wg/CU"
            res[key] = {"KiB_in_flight_per_CU": waves * stages * 2 * kib * per_cu, "us_per_layer": r["us_per_layer"],
                        "GBs": r["GBs"]}
            print(f"probe-shapes {name} {key}: {r['us_per_layer']} us {r['GBs']} GB/s", file=sys.stderr, flush=True)
        out["shapes"][name] = res
        del rot
        torch.cuda.empty_cache()
    return out


def plan_sweep(a):
    """The planner's cost parameters varied one at a time around the defaults, on every full-size workload: an item
    costs tok_count + overhead (Section 3.2's offset of the linear latency model, in token units), and what that
    offset should be is a property of the kernel that only a measurement gives."""
    import torch
    import workloads as W
    import paper_2502_15804_amd as F

    d = F.fairkv_default_params(256)
    base = {"overhead_tokens": int(d.overhead_tokens), "short_overhead_tokens": int(d.short_overhead_tokens),
            "min_chunk": int(d.min_chunk)}
    grid = {"overhead_tokens": (32, 64, 96, 128, 160, 192, 256), "short_overhead_tokens": (16, 32, 48, 64, 96, 128),
            "min_chunk": (16, 32, 64, 128, 256)}
    layers = {"llama70b": 32, "mistral24b": 8, "faircopy": 8, "stress": 40}
    out = {"experiment": "planner cost parameters, one varied at a time around the defaults; microseconds per layer "
                         "(best of 3 graph-replayed passes over the rotation)", "defaults": base, "us_per_layer": {}}
    for name, nl in layers.items():
        res = {}
        for key, values in grid.items():
            row = {}
            for v in values:
                ov = dict(base)
                ov[key] = v
                r = Rotation(name, nl, a.seed, 3, ov)
                best = min(1e6 * timed(r, nl * 8, nl, True)[1] / (nl * 8) for _ in range(3))
                loads = r.layers[0].plan.slot_loads()
                row[str(v)] = {"us": round(best, 2), "items_layer0": r.layers[0].plan.n_items,
                               "E_layer0": round(float(loads.mean() / loads.max()), 3)}
                del r
                torch.cuda.empty_cache()
            print(f"plan-sweep {name} {key}: " + " ".join(f"{v}:{x['us']}" for v, x in row.items()), file=sys.stderr,
                  flush=True)
            res[key] = row
        out["us_per_layer"][name] = res
    return out


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)
    import torch
    import workloads as W
    import paper_2502_15804_amd as F

    if not torch.cuda.is_available():
        print("bench.py needs the GPU", file=sys.stderr)
        sys.exit(2)
    if a.copy_calibration:
        n = a.copy_calibration << 20
        src = torch.ones(n, dtype=torch.uint8, device="cuda")
        dst = torch.zeros(n, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": n, "copies": 3}))
        return
    F.lib()
    if a.latency_model:
        print(json.dumps(latency_model(a.seed)))
        return
    if a.placement_table:
        print(json.dumps(placement_table(a.seed)))
        return
    if a.pack:
        print(json.dumps(pack_bench(a.seed, n_slots=a.n_slots)))
        return
    if a.plan_sweep:
        print(json.dumps(plan_sweep(a)))
        return
    if a.probe_shapes:
        print(json.dumps(probe_shapes(a)))
        return
    w = W.WORKLOADS[a.workload]
    n_layers = a.layers or w.n_layers
    overrides = {k: getattr(a, k) for k in ("n_slots", "tile", "min_chunk", "max_split", "oversub", "overhead_tokens",
                                            "short_overhead_tokens") if getattr(a, k) is not None}
    if a.phases:
        print(json.dumps(phases(a, overrides)))
        return
    kv8 = a.kv_dtype == "fp8"
    valu = a.bf16_kernel == "valu"
    if valu:
        a.no_extras = True
    if kv8:
        a.no_extras = True      # the comparisons and the CPU baseline belong to the headline configuration
        # half the bytes per token: the planner's per-item overhead is worth twice the tokens, and a step is 32 tokens
        overrides = {**KV8_PLAN_DEFAULTS, **overrides}
    rot = Rotation(a.workload, n_layers, a.seed, a.policy, overrides, a.q_len, kv8, valu)
    host_s, ev_s, moved = timed(rot, a.steps, a.warmup, not a.no_graph)
    gbs = moved / ev_s / 1e9
    ms_step = 1e3 * ev_s / a.steps

    plan0 = rot.layers[0].plan
    loads_max, loads_min = int(plan0.summary.max_slot_load), int(plan0.summary.min_slot_load)
    loads0 = plan0.slot_loads()
    eff0 = float(loads0.mean() / max(1, loads0.max()))      # the paper's efficiency E (eq. 5) of the plan
    rec = {
        "metric": "achieved HBM GB/s, ragged per-head GQA decode attention (algorithmic bytes / time)",
        "value": round(gbs, 1), "unit": "GB/s", "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": round(ms_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 (fp32 accumulate)" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": w.name, "shape": w.description,
                   "storage": "e4m3 K/V, bf16 q" if kv8 else w.dtype, "B": w.B, "q_len": a.q_len, "Hq": w.Hq, "Hkv": w.Hkv,
                   "D": w.D, "layers_rotated": n_layers, "rotation_GB": round(sum(rot.bytes) / 1e9, 3),
                   "policy": a.policy, "n_slots": int(rot.params.n_slots), "min_chunk": int(rot.params.min_chunk),
                   "oversub": int(rot.params.oversub), "graph_replay": not a.no_graph,
                   "timed_region": (f"{a.steps} launches enqueued from Python" if a.no_graph else
                                    f"one replay of one HIP graph of {a.steps} launches rotating over the layers"
                                    if a.steps <= MAX_GRAPH_LAUNCHES else
                                    f"HIP graph replays only: {a.steps // n_layers} x a graph of {n_layers} launches"
                                    + (f" + 1 x a graph of {a.steps % n_layers} launches" if a.steps % n_layers else "")),
                   "kernel": "vector ALU (A/B run)" if valu else "matrix cores",
                   "items_layer0": plan0.n_items},
        "us_per_layer": round(1e3 * ms_step, 3), "pct_of_hbm_peak": round(100.0 * gbs / HBM_PEAK_GBS, 2),
        "host_clock_GBs": round(moved / host_s / 1e9, 1),
        "plan_host_us_per_layer": round(rot.plan_us, 1),
        "plan_layer0": {"max_slot_load": loads_max, "min_slot_load": loads_min, "efficiency_E": round(eff0, 4)},
        "roofline": {"bound": "hbm", "achieved": round(gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(gbs / HBM_PEAK_GBS, 4),
                     "traffic": None if (kv8 or valu or a.q_len > 1) else measured_traffic(a.workload)[0],
                     "traffic_source": None if (kv8 or valu or a.q_len > 1) else
                     f"not measured in this run: read from {measured_traffic(a.workload)[1]} (rocprofv3 FETCH_SIZE and WRITE_SIZE)",
                     "kernel": f"fairkv_decode_valu_kernel<bf16, {w.D}, {w.G}>" if valu else
                     f"fairkv_decode_mfma_kernel<{w.D}, {w.G * a.q_len}, DEEP, {'true' if kv8 else 'false'}, SOLO> (DEEP and SOLO "
                     "are chosen per plan: pairs cut in 32 or more pieces, short whole pairs)",
                     "bytes_per_launch": round(moved / a.steps), "us_per_launch": round(1e3 * ms_step, 3)},
        "paper_context": "FairKV reports up to 1.66x throughput over plain tensor parallelism on 8x A100-80G "
                         "(Llama-3.3-70B, Section 5.2.2); other hardware, not this metric",
    }
    rec["spot_check_max_abs_err"] = round(spot_check(rot, ran=a.steps), 6)
    if not rec["spot_check_max_abs_err"] <= w.tol:
        print(f"bench: outputs of the timed launches are off by {rec['spot_check_max_abs_err']}", file=sys.stderr)
        sys.exit(1)
    if not a.no_extras:
        short = max(n_layers * 4, 64)
        for pol, key in ((0, "naive"), (1, "lpt_nosplit"), (2, "lpt_equal_split")):
            if pol == a.policy:
                continue
            r2 = Rotation(a.workload, n_layers, a.seed, pol, overrides)
            _, ev2, moved2 = timed(r2, short, n_layers, not a.no_graph)
            rec[f"{key}_GBs"] = round(moved2 / ev2 / 1e9, 1)
            rec[f"gain_vs_{key}"] = round(gbs / (moved2 / ev2 / 1e9), 3)
            del r2
            torch.cuda.empty_cache()
        rec["stream_probe"] = stream_probe(rot, gbs)
        rec["uniform_same_bytes"] = uniform_same_bytes(rot, a.seed)
        rec["probe_uniform_ragged_us"] = [rec["stream_probe"]["us_per_layer"], rec["uniform_same_bytes"]["us_per_layer"],
                                          rec["us_per_layer"]]
        rec["workloads"] = other_workloads(a, overrides)
        rec["cold_single_launch_us"] = cold_launch_us(rot)
        rec["lpt_equal_split_GBs_by_max_split"] = max_split_sweep(a, n_layers, overrides, gbs)
        rec["cpu_baseline"] = cpu_baseline(rot, a.cpu_seconds)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
