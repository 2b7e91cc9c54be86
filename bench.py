#!/usr/bin/env python3
"""Benchmark of the fused segment-KV decode attention on one MI355X.

A "step" is one pass of the whole hot path for one decoder layer over one batch:
a single segkv_sdpa_decode call with fused append (row copy, ancestor
resolution, prompt + response attention, split-KV merge).  Inputs are synthetic
fp16 N(0,1) tensors of the benchmark shapes, resident in HBM before timing.  To
keep every launch HBM-cold the timed loop cycles through several independent
buffer sets ("layers") whose total footprint exceeds 4x the 256 MB Infinity
Cache, as a real model cycles through its layers' caches.

One clock: a pair of HIP events on the launch stream around the whole timed
region (at least --steps launches, and as many as it takes to fill 50 ms, so
that 50 us kernels are not timed over a millisecond); `value`, `ms_per_step`
and `roofline.achieved` all come from it.  The host's wall clock over the same
region and a per-launch event-pair spread are reported beside it.

Prints ONE JSON line; besides the headline
workload it carries the other benchmark configurations, the paper's Figure 6
batch-size sweep in both prompt layouts, and the prefill attention shapes.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E peak
MALL_BYTES = 256 << 20

# HBM bytes per launch of the decode kernel as rocprofv3 counted them (FETCH_SIZE +
# WRITE_SIZE, each scaled by a copy kernel of known size).  Not measured by this
# script: every figure names the summary under profiles/ that holds it and the
# commit whose kernel was profiled; a kernel changed since then needs a new profile.
PROFILED_TRAFFIC = {
    "llama2_7b_greedy": {"bytes": 2420529004, "profile": "profiles/sdpa_decode_mfma_llama2_7b_greedy.md", "kernel_commit": "cde399a"},
    "llama2_70b_gqa": {"bytes": 309474961, "profile": "profiles/sdpa_decode_mfma_llama2_70b_gqa.md", "kernel_commit": "cde399a"},
    "gptj6b": {"bytes": 307609518, "profile": "profiles/sdpa_decode_mfma_gptj6b.md", "kernel_commit": "cde399a"},
    "bloom176b_alibi": {"bytes": 537425832, "profile": "profiles/sdpa_decode_mfma_bloom176b_alibi.md", "kernel_commit": "cde399a"},
    "gptj6b_1024_1024": {"bytes": 1088715927, "profile": "profiles/sdpa_decode_mfma_gptj6b_1024_1024.md", "kernel_commit": "cde399a"},
    "llama2_13b_1024_1024": {"bytes": 1358428767, "profile": "profiles/sdpa_decode_mfma_llama2_13b_1024_1024.md", "kernel_commit": "cde399a"},
    "llama2_13b_bs8": {"bytes": 192381079, "profile": "profiles/sdpa_decode_mfma_llama2_13b_bs8.md", "kernel_commit": "cde399a"},
}
MIN_TIMED_REGION_S = 0.05      # short kernels are launched often enough to fill this
MAX_TIMED_LAUNCHES = 4000


def algorithmic_bytes(wl, unique_rows: int) -> dict:
    """Bytes one layer-step must move: prompt K/V once per request, the distinct
    response rows referenced, Q read + O write, append read + write, parent table."""
    row = wl.Hkv * wl.D * 2
    qo = 2 * wl.N * wl.Hq * wl.D * 2
    fixed = 2 * wl.B * wl.Lp * row + qo + 4 * wl.N * row + wl.T * wl.N * 4
    return {"unique": fixed + 2 * unique_rows * row,
            "nominal": fixed + 2 * wl.T * wl.N * row}


class DeviceSet:
    """One independent set of operands on the GPU (one "layer")."""

    def __init__(self, wl, seed, parent_np, slopes_np, segkv, torch, prompt_seq_first=False,
                 lineage=None, lineage_capacity=0):
        dev = torch.device("cuda:0")
        g = torch.Generator(device=dev)
        g.manual_seed(seed)

        def rnd(*shape):
            return torch.randn(*shape, generator=g, device=dev, dtype=torch.float32).half()

        self.dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
        # K buffers sit on an 8 KB boundary, V buffers at the library's recommended byte
        # offset from one: see segkv_value_stagger_bytes
        stagger = segkv.value_stagger_bytes(self.dims)

        def placed(t, offset):
            big = torch.empty(t.numel() + 8192, dtype=torch.float16, device=dev)
            start = (-big.data_ptr()) % 8192 + offset
            v = big[start // 2: start // 2 + t.numel()].view_as(t)
            assert (v.data_ptr() - offset) % 8192 == 0
            v.copy_(t)
            return v

        def staggered(t):
            return placed(t, stagger)

        self.q = rnd(wl.N, wl.Hq, wl.D)
        # Section 4.1's layout comparison: [Lp, B, Hkv, D] when prompt_seq_first
        pshape = (wl.Lp, wl.B, wl.Hkv, wl.D) if prompt_seq_first else (wl.B, wl.Lp, wl.Hkv, wl.D)
        self.prompt_seq_first = prompt_seq_first
        self.pk = placed(rnd(*pshape), 0)
        self.pv = staggered(rnd(*pshape))
        self.rk = placed(torch.full((wl.Tcap, wl.N, wl.Hkv, wl.D), float("nan"), dtype=torch.float16, device=dev), 0)
        self.rv = staggered(torch.full((wl.Tcap, wl.N, wl.Hkv, wl.D), float("nan"), dtype=torch.float16,
                                       device=dev))
        if wl.T > 1:
            self.rk[: wl.T - 1] = rnd(wl.T - 1, wl.N, wl.Hkv, wl.D)
            self.rv[: wl.T - 1] = rnd(wl.T - 1, wl.N, wl.Hkv, wl.D)
        self.kn = rnd(wl.N, wl.Hkv, wl.D)
        self.vn = rnd(wl.N, wl.Hkv, wl.D)
        self.parent = torch.from_numpy(parent_np).to(dev)
        self.slopes = None if slopes_np is None else torch.from_numpy(slopes_np).to(dev)
        self.out = torch.empty(wl.N, wl.Hq, wl.D, dtype=torch.float16, device=dev)
        nb = segkv.workspace_bytes(self.dims)
        self.ws = torch.empty(max(nb, 16) // 4, dtype=torch.float32, device=dev) if nb else None
        self.call = segkv.prepare_sdpa_decode(self.out, self.q, self.pk, self.pv, self.rk, self.rv,
                                              self.parent, self.dims, wl.scale, k_new=self.kn,
                                              v_new=self.vn, alibi_slopes=self.slopes,
                                              workspace=self.ws, prompt_seq_first=prompt_seq_first,
                                              lineage=lineage, lineage_capacity=lineage_capacity)

    def to_numpy(self):
        c = lambda t: None if t is None else t.cpu().numpy()
        return {"q": c(self.q), "prompt_k": c(self.pk), "prompt_v": c(self.pv), "resp_k": c(self.rk),
                "resp_v": c(self.rv), "k_new": c(self.kn), "v_new": c(self.vn),
                "parent": c(self.parent), "slopes": c(self.slopes)}


def distinct_response_rows(parent, B, W):
    """Bookkeeping for the byte count: how many distinct (step, slot) response rows the
    beams of all requests descend from.  Walks the parent table backwards from the last
    step (slot of beam j at step T-1 is j; one step earlier it is parent[s][slot])."""
    import numpy as np
    T = parent.shape[0]
    base = (np.arange(B * W) // W) * W
    slot = np.arange(B * W) % W
    total = 0
    for s in range(T - 1, -1, -1):
        total += np.unique(base + slot).size
        if s > 0:
            slot = parent[s][base + slot]
    return int(total)


def timed_region(call_list, n_launches, torch):
    """n_launches calls (cycling through call_list) between ONE pair of HIP events on the
    launch stream, bracketed by synchronisations.  Returns (event seconds, wall seconds)."""
    e0 = torch.cuda.Event(enable_timing=True)
    e1 = torch.cuda.Event(enable_timing=True)
    k = len(call_list)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    e0.record()
    for i in range(n_launches):
        call_list[i % k]()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return e0.elapsed_time(e1) * 1e-3, wall


def launches_for(call_list, steps, torch):
    """At least `steps` launches, and enough of them that the timed region lasts
    MIN_TIMED_REGION_S (estimated from a short burst)."""
    ev_s, _ = timed_region(call_list, 10, torch)
    per = max(ev_s / 10, 1e-7)
    return int(min(MAX_TIMED_LAUNCHES, max(steps, math.ceil(MIN_TIMED_REGION_S / per))))


def build_lineage(wl, parent_np, segkv, torch):
    """The lineage list after wl.T steps: one segkv_lineage_update per step, as a
    generation loop would have issued them (once per token, shared by all layers)."""
    cap = ((wl.Tcap * wl.W + 3) // 4) * 4
    dims = segkv.make_dims(wl.B, wl.W, wl.Hq, wl.Hkv, wl.D, wl.Lp, wl.T, wl.Tcap)
    buf = torch.zeros(segkv.lineage_bytes(dims, cap) // 4, dtype=torch.int32, device="cuda:0")
    rows = torch.from_numpy(parent_np).to("cuda:0")
    for t in range(wl.T):
        segkv.lineage_update(buf, cap, rows[t] if t > 0 else None, t, dims)
    torch.cuda.synchronize()
    return buf, cap


def time_workload(wl, steps, warmup, segkv, torch, want_cpu_baseline, cpu_seconds,
                  prompt_seq_first=False, use_lineage=False, probe=True):
    import numpy as np
    from paper_2401_05391_amd.workloads import alibi_slopes, make_parent

    rng = np.random.default_rng(wl.seed)
    parent_np = make_parent(wl, rng)
    slopes_np = alibi_slopes(wl.Hq) if wl.alibi else None

    row = wl.Hkv * wl.D * 2
    set_bytes = 2 * wl.B * wl.Lp * row + 2 * wl.T * wl.N * row
    n_sets = max(2, math.ceil(4 * MALL_BYTES / set_bytes))
    lin, lin_cap = build_lineage(wl, parent_np, segkv, torch) if use_lineage else (None, 0)
    sets = [DeviceSet(wl, 1000 * wl.seed + i, parent_np, slopes_np, segkv, torch, prompt_seq_first,
                      lin, lin_cap)
            for i in range(n_sets)]
    torch.cuda.synchronize()

    s0 = sets[0]
    cpu_inputs = s0.to_numpy() if want_cpu_baseline else None
    U = distinct_response_rows(parent_np, wl.B, wl.W)
    nbytes = algorithmic_bytes(wl, U)
    calls = [st.call for st in sets]

    for i in range(warmup):
        calls[i % n_sets]()
    torch.cuda.synchronize()

    # (1) THE clock: HIP events on the launch stream around the whole timed region.
    # `steps` launches at least; short kernels get more, so that the region lasts
    # MIN_TIMED_REGION_S and the events' own cost (a few us) disappears in it.
    n_launches = launches_for(calls, steps, torch)
    ev_s, wall_s = timed_region(calls, n_launches, torch)
    ms_per_step = ev_s * 1e3 / n_launches

    # (2) beside it: one event pair per launch (adds 1-3 us to every launch: the pair's
    # own records sit between the kernels), for the spread only
    n_pairs = min(n_launches, 400)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
           for _ in range(n_pairs)]
    for i in range(n_pairs):
        evs[i][0].record()
        calls[i % n_sets]()
        evs[i][1].record()
    torch.cuda.synchronize()
    dev_ms = np.array([a.elapsed_time(b) for a, b in evs])

    # (3) practical streaming-read ceiling: same bytes, pure 128-bit loads
    probe_gbs = None
    if probe and wl.Lp > 0:
        sink = torch.empty(4096, dtype=torch.int32, device="cuda:0")
        probe_src = [torch.cat([s.pk.view(-1), s.pv.view(-1)]) for s in sets[:2]]
        probe_calls = [lambda i=i: segkv.stream_read_probe(probe_src[i], sink) for i in range(2)]
        for i in range(3):
            probe_calls[i % 2]()
        n_probe = launches_for(probe_calls, 10, torch) // 4 + 10
        probe_s, _ = timed_region(probe_calls, n_probe, torch)
        probe_gbs = probe_src[0].numel() * 2 / (probe_s / n_probe) / 1e9
        del probe_src, probe_calls

    gbs = nbytes["unique"] / (ms_per_step * 1e-3) / 1e9
    prof = PROFILED_TRAFFIC.get(wl.name)
    res = {
        "workload": wl.name,
        "shape": {"B": wl.B, "beam": wl.W, "Hq": wl.Hq, "Hkv": wl.Hkv, "D": wl.D, "Lp": wl.Lp,
                  "T": wl.T, "alibi": wl.alibi},
        "buffer_sets": n_sets,
        "unique_response_rows": U,
        "bytes_unique": nbytes["unique"], "bytes_nominal": nbytes["nominal"],
        "timed_launches": n_launches,
        "clock": "HIP events on the launch stream around the timed region of timed_launches launches",
        "ms_per_step": ms_per_step,
        "us_per_layer_step": ms_per_step * 1e3,
        "wall_clock_us_per_layer_step": wall_s * 1e6 / n_launches,
        "gbs_unique": gbs,
        "gbs_nominal": nbytes["nominal"] / (ms_per_step * 1e-3) / 1e9,
        "per_launch_event_pairs_us": {
            "n": n_pairs, "mean": float(dev_ms.mean() * 1e3), "median": float(np.median(dev_ms) * 1e3),
            "min": float(dev_ms.min() * 1e3), "p90": float(np.percentile(dev_ms, 90) * 1e3)},
        "stream_read_probe_gbs": probe_gbs,
        "workspace_bytes": segkv.workspace_bytes(s0.dims),
    }
    res["roofline"] = {
        "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": gbs / HBM_PEAK_GBS,
        "traffic": prof["bytes"] if prof else None,
        "traffic_source": ({"profile": prof["profile"], "kernel_commit": prof["kernel_commit"],
                            "note": "rocprofv3 FETCH_SIZE + WRITE_SIZE per launch, not measured in this run"}
                           if prof else None),
    }

    if want_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(wl, cpu_inputs, nbytes["unique"], cpu_seconds, U)
    # The buffers go back to torch's pool, not to the driver: device memory that was
    # released and mapped again measured 1-3 % slower for the workloads that follow (70B
    # 53.0 against 51.9 us, Bloom 88.7 against 86.0 us), and a serving process keeps its
    # cache memory anyway.
    del sets
    return res


def cpu_baseline(wl, x, bytes_unique, budget_s, U):
    """The fp64 oracle as it stands, timed on this machine's host cores on a bounded
    sample of the same batch: the first requests (all of them if they fit the
    budget), repeated until about `budget_s` CPU-core-seconds have been spent."""
    import numpy as np
    from oracle import segkv_oracle as oracle

    rk, rv = x["resp_k"], x["resp_v"]
    oracle.append_kv(rk, rv, x["k_new"], x["v_new"], wl.T - 1)
    per_req = wl.W * wl.Hq
    cores = oracle.num_threads()
    # the byte count's distinct-row figure against the oracle's own ancestor table
    anc = oracle.ancestors(x["parent"], wl.B, wl.W)
    offs = (np.arange(wl.N) // wl.W) * wl.W
    U_oracle = int(sum(np.unique(offs + anc[s]).size for s in range(wl.T)))
    assert U_oracle == U, f"distinct response rows: {U} counted here, {U_oracle} by the oracle"

    def run(nreq):
        pairs = np.array([(n, h) for n in range(nreq * wl.W) for h in range(wl.Hq)], dtype=np.int32)
        t0 = time.perf_counter()
        oracle.sdpa_decode(x["q"], x["prompt_k"], x["prompt_v"], rk, rv, x["parent"], wl.W, wl.T,
                           wl.scale, slopes=x["slopes"], pairs=pairs)
        return time.perf_counter() - t0

    t1 = run(1)                                   # calibrate on one request
    wall_budget = budget_s / max(cores, 1)
    nreq = int(max(1, min(wl.B, wall_budget / max(t1, 1e-5))))
    times = [run(nreq)]
    while sum(times) < wall_budget and len(times) < 50:
        times.append(run(nreq))
    t = float(np.median(times))
    frac = nreq / wl.B
    tiny_us = tiny_single_thread_us(oracle)
    return {"value": bytes_unique * frac / t / 1e9, "unit": "GB/s", "cores": cores,
            "tiny_config_single_thread_us": tiny_us,
            "kind": "oracle",
            "unique_response_rows_by_oracle": U_oracle,
            "sample": f"first {nreq} of {wl.B} requests ({nreq * per_req} of {wl.B * per_req} "
                      f"query rows), {len(times)} repeats, median {t:.3f} s wall each, "
                      f"{sum(times) * cores:.0f} core-seconds in total",
            "ms_per_step_extrapolated": t / frac * 1e3}


def tiny_single_thread_us(oracle):
    """The smallest benchmark configuration (B=1, beam 4, 4 heads of 64, 32 + 8 keys)
    through the same oracle on ONE host thread: the OpenMP runtime is told to use
    one thread for the call and its previous setting is restored."""
    import ctypes
    import numpy as np
    from paper_2401_05391_amd.workloads import CONFIGS, make_inputs
    try:
        gomp = ctypes.CDLL("libgomp.so.1")
    except OSError:
        return None
    wl = CONFIGS["tiny"]
    x = make_inputs(wl)
    rk, rv = x["resp_k"].copy(), x["resp_v"].copy()
    oracle.append_kv(rk, rv, x["k_new"], x["v_new"], wl.T - 1)
    before = oracle.num_threads()
    gomp.omp_set_num_threads(1)
    try:
        times = []
        for _ in range(20):
            t0 = time.perf_counter()
            oracle.sdpa_decode(x["q"], x["prompt_k"], x["prompt_v"], rk, rv, x["parent"], wl.W, wl.T,
                               wl.scale, slopes=x["slopes"])
            times.append(time.perf_counter() - t0)
    finally:
        gomp.omp_set_num_threads(before)
    return float(np.median(times)) * 1e6


MFMA_F16_PEAK_TFLOPS = 2500.0     # MI355X published dense fp16 matrix-core peak

# (name, B, N0, Hq, Hkv, D): prompt batches of the benchmark models' attention shapes
PREFILL_SHAPES = [
    ("llama2_7b_prefill", 16, 1024, 32, 32, 128),
    ("llama2_70b_gqa_prefill", 4, 2048, 64, 8, 128),
    ("gptj6b_prefill", 16, 1024, 16, 16, 256),
    ("llama2_7b_prefill_4k", 4, 4096, 32, 32, 128),
]


def prefill_rows(steps, warmup, segkv, torch):
    """Causal prefill attention on the prompt shapes of the benchmark models:
    4 * B * Hq * D * N0 (N0 + 1) / 2 flops per call, timed like the decode step
    (one HIP-event pair around the timed region)."""
    dev = torch.device("cuda:0")
    rows = []
    for name, B, N0, Hq, Hkv, D in PREFILL_SHAPES:
        g = torch.Generator(device=dev)
        g.manual_seed(7)
        rnd = lambda *s: torch.randn(*s, generator=g, device=dev, dtype=torch.float32).half()
        q, k, v = rnd(B, N0, Hq, D), rnd(B, N0, Hkv, D), rnd(B, N0, Hkv, D)
        out = torch.empty_like(q)
        dims = segkv.make_dims(B, 1, Hq, Hkv, D, N0, 1, 1)
        call = [lambda: segkv.sdpa_prefill(out, q, k, v, dims, D ** -0.5)]
        for _ in range(warmup):
            call[0]()
        n = launches_for(call, steps, torch)
        ev_s, wall_s = timed_region(call, n, torch)
        flops = 4.0 * B * Hq * D * N0 * (N0 + 1) / 2
        tflops = flops / (ev_s / n) / 1e12
        rows.append({"workload": name, "shape": {"B": B, "N0": N0, "Hq": Hq, "Hkv": Hkv, "D": D},
                     "timed_launches": n, "ms_per_step": ev_s * 1e3 / n,
                     "wall_clock_ms_per_step": wall_s * 1e3 / n, "flops": flops, "tflops": tflops,
                     "tokens_per_s": B * N0 / (ev_s / n),
                     "roofline": {"bound": "mfma", "achieved": tflops, "peak": MFMA_F16_PEAK_TFLOPS,
                                  "unit": "TFLOP/s", "frac": tflops / MFMA_F16_PEAK_TFLOPS,
                                  "traffic": None}})
        del q, k, v, out
    return rows


def mfma_sustained_rates(segkv, torch):
    """What the matrix cores sustain on register-resident operands (segkv_probe_mfma_rate): a
    chain of the fp16 32x32x16 instruction on constant operands and on random ones.  The
    random-operand rate is the ceiling the power limit leaves for prefill on real Q/K/V;
    `roofline.peak` stays the published 2.5 PFLOP/s."""
    import numpy as np
    dev = torch.device("cuda:0")
    n_groups, iters = 2048, 12000
    out = torch.empty(n_groups * 256, dtype=torch.float32, device=dev)
    clocks = torch.zeros(n_groups * 2, dtype=torch.int64, device=dev)
    g = torch.Generator(device=dev)
    g.manual_seed(3)
    res = {}
    for kind in ("constant", "random"):
        if kind == "constant":
            ops = torch.full((16 * 256 * 8,), 0.5, dtype=torch.float16, device=dev)
        else:
            ops = torch.randn(16 * 256 * 8, generator=g, device=dev, dtype=torch.float32).half()
        call = [lambda: segkv.probe_mfma_rate(ops, out, clocks, n_groups, iters)]
        call[0]()
        ev_s, _ = timed_region(call, 3, torch)
        c = clocks.cpu().numpy().reshape(n_groups, 2).astype(np.float64)
        flop = n_groups * 4.0 * iters * 16 * 32768.0
        res[kind + "_operands"] = {"tflops": flop / (ev_s / 3) / 1e12,
                                   "clock_mhz": float(np.median(c[:, 0] / c[:, 1]) * 100.0)}
        del ops
    return res


def relate_to_sustained_rate(rows, rates):
    """Each prefill shape's TFLOP/s as a fraction of what the matrix cores sustained on random
    register operands in the same process (the power limit differs from one box to the next)."""
    ref = rates["random_operands"]["tflops"]
    for r in rows:
        r["frac_of_mfma_sustained_random_operands"] = r["tflops"] / ref


def prefill_bench(steps, warmup, segkv, torch):
    rows = prefill_rows(steps, warmup, segkv, torch)
    rates = mfma_sustained_rates(segkv, torch)
    relate_to_sustained_rate(rows, rates)
    head = rows[0]
    return {"metric": "prefill causal SDPA (segkv_sdpa_prefill): achieved fp16 TFLOP/s",
            "value": head["tflops"], "unit": "TFLOP/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak",
            "vs_baseline": None, "dtype": "f16", "data": "synthetic",
            "config": {"workload": head["workload"], **head["shape"]},
            "roofline": head["roofline"], "cpu_baseline": None, "shapes": rows,
            "mfma_sustained": rates}


def fig6_rows(steps, warmup, segkv, torch):
    """Section 4.1, Figure 6: Llama2-13B attention shape, beam 4, 1024 prompt / 128
    response tokens, batch size 1..64, with the prompt segment stored batch first
    (the paper's choice) and sequence first (the other arm of its comparison)."""
    from paper_2401_05391_amd.workloads import FIG6_BATCH_SIZES, fig6_workload
    rows = []
    for bs in FIG6_BATCH_SIZES:
        r = time_workload(fig6_workload(bs), steps, warmup, segkv, torch, False, 0, probe=False)
        r2 = time_workload(fig6_workload(bs), steps, warmup, segkv, torch, False, 0,
                           prompt_seq_first=True, probe=False)
        rows.append({"batch_size": bs, "timed_launches": r["timed_launches"],
                     "us_per_layer_step": r["us_per_layer_step"],
                     "seq_first_prompt_us_per_layer_step": r2["us_per_layer_step"],
                     "bytes_unique": r["bytes_unique"], "bytes_nominal": r["bytes_nominal"],
                     "gbs_unique": r["gbs_unique"], "gbs_nominal": r["gbs_nominal"],
                     "seq_first_prompt_gbs_unique": r2["gbs_unique"],
                     "roofline": {k: r["roofline"][k] for k in ("bound", "achieved", "peak", "unit", "frac")},
                     "seq_first_prompt_roofline_frac": r2["roofline"]["frac"]})
    return rows


def run_counter_calibration(segkv, torch):
    """Kernels of known HBM traffic for scaling hardware counters: a copy
    (append of one very wide row: 2 x 128 MiB read, 2 x 128 MiB written) and a
    pure read of 1 GiB.  Each runs three times on cold buffers."""
    dev = torch.device("cuda:0")
    n_rows, hkv, d = 1 << 15, 16, 128                      # 32768*16*128*2 B = 128 MiB per tensor
    dims = segkv.make_dims(n_rows, 1, hkv, hkv, d, 0, 1, 1)
    row = n_rows * hkv * d
    for _ in range(3):
        src_k = torch.ones(row, dtype=torch.float16, device=dev)
        src_v = torch.ones(row, dtype=torch.float16, device=dev)
        dst_k = torch.empty(row, dtype=torch.float16, device=dev)
        dst_v = torch.empty(row, dtype=torch.float16, device=dev)
        flush = torch.zeros(1 << 28, dtype=torch.float16, device=dev)   # 512 MiB: evicts the caches
        flush.add_(1)
        torch.cuda.synchronize()
        segkv.append_kv(dst_k, dst_v, src_k, src_v, 0, dims)
        torch.cuda.synchronize()
        del src_k, src_v, dst_k, dst_v, flush
    sink = torch.empty(4096, dtype=torch.int32, device=dev)
    for _ in range(3):
        buf = torch.ones(1 << 29, dtype=torch.float16, device=dev)      # 1 GiB
        flush = torch.zeros(1 << 28, dtype=torch.float16, device=dev)
        flush.add_(1)
        torch.cuda.synchronize()
        segkv.stream_read_probe(buf, sink)
        torch.cuda.synchronize()
        del buf, flush
    return {"append_kv_kernel": {"bytes_read": 2 * row * 2, "bytes_written": 2 * row * 2},
            "stream_read_probe_kernel": {"bytes_read": 1 << 30, "bytes_written": 4096 * 4}}


def graph_bench(layers, steps, warmup, segkv, torch):
    """Small batches are launch-bound: `layers` decode layer-steps (each on its own
    K/V buffers, as the layers of a model) launched one by one from Python against
    the same launches replayed from one HIP graph."""
    import numpy as np
    from paper_2401_05391_amd.workloads import alibi_slopes, fig6_workload, make_parent
    rows = []
    for bs in (1, 2, 4, 16):
        wl = fig6_workload(bs)
        parent_np = make_parent(wl, np.random.default_rng(wl.seed))
        sets = [DeviceSet(wl, 1000 * wl.seed + i, parent_np, None, segkv, torch) for i in range(layers)]
        torch.cuda.synchronize()

        def token_step():
            for s in sets:
                s.call()

        # the prepared calls above are bound to the stream that was current when
        # they were made; the recorded ones must go to the capturing stream
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for s in sets:
                segkv.prepare_sdpa_decode(s.out, s.q, s.pk, s.pv, s.rk, s.rv, s.parent, s.dims, wl.scale,
                                          k_new=s.kn, v_new=s.vn, workspace=s.ws)()
        torch.cuda.synchronize()
        res = {}
        for name, fn in (("eager", token_step), ("graph", graph.replay)):
            for _ in range(warmup):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                fn()
            torch.cuda.synchronize()
            res[name] = (time.perf_counter() - t0) / (steps * layers) * 1e6
        rows.append({"batch_size": bs, "eager_us_per_layer_step": res["eager"],
                     "graph_us_per_layer_step": res["graph"]})
    last = rows[0]
    return {"metric": "fused segment-KV decode SDPA: us per layer-step, launches replayed from one HIP graph",
            "value": last["graph_us_per_layer_step"], "unit": "us", "n_gpus": 1, "steps": steps,
            "warmup": warmup, "ms_per_step": last["graph_us_per_layer_step"] * layers * 1e-3,
            "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
            "data": "synthetic",
            "config": {"workload": "fig6_llama2_13b_graph", "beam": 4, "Hq": 40, "Hkv": 40, "D": 128,
                       "Lp": 1024, "T": 128, "layers_per_graph": layers,
                       "value_is_batch_size": last["batch_size"]},
            "sweep": rows}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="llama2_7b_greedy")
    ap.add_argument("--others", default="llama2_70b_gqa,gptj6b,bloom176b_alibi",
                    help="comma list of further workloads reported under other_workloads ('' = none)")
    ap.add_argument("--cpu-seconds", type=float, default=20.0,
                    help="CPU-core-seconds to spend on the oracle baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="leave out the fig6 (Figure 6 batch-size sweep, both prompt layouts) and prefill "
                         "sub-records of the default line")
    ap.add_argument("--fig6-sweep", action="store_true",
                    help="instead of the headline workload, time the paper's Figure 6 experiment "
                         "(Llama2-13B attention shape, beam 4, 1024/128 tokens, batch size 1..64) and "
                         "print its table as one JSON line")
    ap.add_argument("--prefill", action="store_true",
                    help="instead of the decode step, time segkv_sdpa_prefill (causal prompt attention, "
                         "the step that writes the prompt segment) on the shapes of the benchmark "
                         "models and print one JSON line with an MFMA roofline")
    ap.add_argument("--graph", type=int, default=0, metavar="LAYERS",
                    help="instead of the headline workload, time LAYERS decode layer-steps per token "
                         "(Figure 6 shape, small batches) launched one by one and replayed from one "
                         "HIP graph, and print one JSON line")
    ap.add_argument("--lineage", action="store_true",
                    help="time segkv_sdpa_decode_lineage (the list of response rows kept across steps by "
                         "segkv_lineage_update) instead of segkv_sdpa_decode (raw parent table)")
    ap.add_argument("--calibrate-counters", action="store_true",
                    help="also launch a plain copy of known size (segkv_append_kv, 2 x 128 MiB read and "
                         "written) and a plain read of known size (segkv_stream_read_probe, 1 GiB), "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled")
    a = ap.parse_args()
    if a.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2401_05391_amd as segkv
    from paper_2401_05391_amd.workloads import RESPONSE_HEAVY, find_workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    segkv.load_library()

    if a.prefill:
        print(json.dumps(prefill_bench(a.steps, a.warmup, segkv, torch)), flush=True)
        return

    if a.graph:
        print(json.dumps(graph_bench(a.graph, a.steps, a.warmup, segkv, torch)), flush=True)
        return

    if a.fig6_sweep:
        rows = fig6_rows(a.steps, a.warmup, segkv, torch)
        last = rows[-1]
        print(json.dumps({
            "metric": "fused segment-KV decode SDPA: achieved HBM GB/s, Figure 6 batch-size sweep",
            "value": last["gbs_unique"], "unit": "GB/s", "n_gpus": 1, "steps": a.steps,
            "warmup": a.warmup, "ms_per_step": last["us_per_layer_step"] * 1e-3,
            "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16",
            "data": "synthetic",
            "config": {"workload": "fig6_llama2_13b_sweep", "beam": 4, "Hq": 40, "Hkv": 40, "D": 128,
                       "Lp": 1024, "T": 128, "value_is_batch_size": last["batch_size"]},
            "roofline": last["roofline"], "sweep": rows}), flush=True)
        return

    wl = find_workload(a.workload)
    main_res = time_workload(wl, a.steps, a.warmup, segkv, torch, not a.no_cpu_baseline, a.cpu_seconds,
                             use_lineage=a.lineage)
    others = []
    for name in [n for n in a.others.split(",") if n and n != a.workload]:
        others.append(time_workload(find_workload(name), a.steps, a.warmup, segkv, torch, False, 0,
                                    use_lineage=a.lineage))

    # the rows next to the path: the paper's Figure 6 sweep (both prompt layouts) and the
    # prefill attention, each timed the same way, each with its own roofline
    resp_heavy = None
    if not a.no_extras:
        resp_heavy = []
        for w in RESPONSE_HEAVY.values():
            r = time_workload(w, max(a.steps // 2, 10), a.warmup, segkv, torch, False, 0, probe=False)
            resp_heavy.append({k: r[k] for k in ("workload", "shape", "timed_launches", "us_per_layer_step",
                                                 "gbs_unique", "gbs_nominal", "bytes_unique",
                                                 "unique_response_rows", "roofline", "buffer_sets")})
    fig6 = None if a.no_extras else fig6_rows(a.steps, a.warmup, segkv, torch)
    prefill = None if a.no_extras else prefill_rows(max(a.steps // 4, 10), a.warmup, segkv, torch)
    mfma_rates = None if a.no_extras else mfma_sustained_rates(segkv, torch)
    if prefill is not None:
        relate_to_sustained_rate(prefill, mfma_rates)

    calibration = None
    if a.calibrate_counters:
        calibration = run_counter_calibration(segkv, torch)

    line = {
        "metric": "fused segment-KV decode SDPA: achieved HBM GB/s (us/layer-step in us_per_layer_step)",
        "value": main_res["gbs_unique"], "unit": "GB/s",
        "n_gpus": 1, "steps": a.steps, "warmup": a.warmup,
        "ms_per_step": main_res["ms_per_step"], "us_per_layer_step": main_res["us_per_layer_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "timed_launches": main_res["timed_launches"], "clock": main_res["clock"],
        "wall_clock_us_per_layer_step": main_res["wall_clock_us_per_layer_step"],
        "config": {"workload": wl.name, **main_res["shape"], "append": "fused",
                   "beam_lineage": "list kept across steps" if a.lineage else "parent table",
                   "buffer_sets": main_res["buffer_sets"]},
        "pct_of_hbm_peak": 100.0 * main_res["gbs_unique"] / HBM_PEAK_GBS,
        "roofline": main_res["roofline"],
        "cpu_baseline": main_res.get("cpu_baseline"),
        "detail": {k: main_res[k] for k in ("bytes_unique", "bytes_nominal", "unique_response_rows",
                                            "gbs_nominal", "per_launch_event_pairs_us",
                                            "stream_read_probe_gbs", "workspace_bytes")},
        "counter_calibration": calibration,
        "other_workloads": [{k: r[k] for k in ("workload", "shape", "timed_launches", "us_per_layer_step",
                                               "wall_clock_us_per_layer_step", "gbs_unique",
                                               "gbs_nominal", "bytes_unique", "unique_response_rows",
                                               "per_launch_event_pairs_us", "roofline",
                                               "stream_read_probe_gbs", "buffer_sets")}
                            for r in others],
        "response_heavy": None if resp_heavy is None else {
            "what": "Section 3.2's sizes (N_prompt = N_response = 1024, beam 4, batch 32) on the GPT-J-6B and "
                    "Llama2-13B attention shapes: the response segment as long as the prompt",
            "workloads": resp_heavy},
        "fig6": None if fig6 is None else {
            "what": "Section 4.1, Figure 6: Llama2-13B attention shape (40 heads of 128), beam 4, 1024 "
                    "prompt / 128 response tokens; prompt segment batch first and sequence first",
            "sweep": fig6},
        "prefill": None if prefill is None else {
            "what": "segkv_sdpa_prefill (causal prompt attention, Section 3.3's special case) on the "
                    "prompt shapes of the benchmark models; roofline: fp16 dense MFMA.  mfma_sustained: "
                    "what a register-resident chain of the same matrix instruction reaches on this part "
                    "with constant and with random operands (the power limit's ceiling for real Q/K/V)",
            "shapes": prefill, "mfma_sustained": mfma_rates},
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
