#!/usr/bin/env python3
"""Benchmark of the FlowCache denoising-step hot path on one MI355X.

One *step* is one pass of the whole hot path over one batch of synthetic input.  The headline
workload is the largest single-GPU configuration, the MAGI-1-like single layer (24 heads x 128,
4 active chunks of 9360 tokens, 74880 clean tokens compressed to 37440); the SkyReels-V2-1.3B-
like layer (12 heads x 128, 2 chunks of 10200, 40800 -> 20400) is measured in the same run and
reported as a second object of the same JSON line (``secondary``).

    flowcache_chunk_decide   change metric + decision + gather of x
    flowcache_scatter_kv     new K/V of the recompute chunks into their cache slots
    flowcache_attend         chunk-causal bf16 attention (all chunks recompute: eps = 0)
    flowcache_attention_mass importance of the first L_k cache positions (50 observation rows)
    flowcache_kv_compress    scoring, top-B selection, in-place compaction (fresh cache per step)

The calls run back to back on one stream, timed with HIP events on that stream.  The importance
mass and the selection only read K, so with ``--overlap`` the step runs them on a second HIP
stream beside the attention kernel and the compaction waits for both (not the default: every
stage time is then no longer that call alone).  After the timed region a few more steps time
every call, and the halves of the decide and compress calls, alone (``calls``); the operands of
the bandwidth-bound calls rotate over several buffer sets so that none is served from the caches.

Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C3|C2|mid]
                    [--secondary C2|C3|mid|none] [--no-cpu] [--overlap]
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E peak
# What the chip sustains (peak_probe, profiles/peaks_measured.md): a loop of nothing but bf16
# MFMAs on random operands; a plain read and a plain copy (read + written bytes) from cold.
MEASURED_MFMA_TFLOPS = 1370.0
MEASURED_READ_GBPS = 6100.0
MEASURED_COPY_GBPS = 5200.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attend_hbm_traffic.md")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C3", choices=["C2", "C3", "mid"])
    ap.add_argument("--secondary", default="C2", choices=["C2", "C3", "mid", "none"],
                    help="a second workload measured in the same run and reported under 'secondary'")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle (cpu_baseline) leg")
    ap.add_argument("--cpu-rows", type=int, default=480, help="oracle attention rows per chunk")
    ap.add_argument("--overlap", action="store_true",
                    help="two streams: mass and selection beside the attention instead of after it")
    ap.add_argument("--qkv", default="normal", choices=["normal", "const"],
                    help="const: constant Q/K/V (same instruction stream, full clocks) -- shows how "
                         "much of the attention time is the power limit; not a valid bench result")
    return ap.parse_args()


def attend_traffic_bytes(workload_name):
    """HBM bytes per launch of the attention kernel, as measured with rocprofv3 counters and
    recorded in profiles/ (lines 'traffic_bytes_per_launch <kernel> <workload> <bytes>');
    None when no measurement of this workload is on file."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                m = re.match(r"\s*traffic_bytes_per_launch\s+(\S+)\s+(\S+)\s+(\d+)", line)
                if m and m.group(2) == workload_name:
                    return int(m.group(3))
    except OSError:
        pass
    return None


def compress_min_bytes(wl, L_k, budget):
    """Algorithmic HBM bytes of one kv_compress call: K read once for scoring, kept K and V
    rows read and written once, 12 B/token/head of mass + score, 4 B per kept index."""
    esz = 2 if wl.dtype == "bf16" else 4
    row = wl.d * esz
    return wl.H_k * (L_k * row + 4 * budget * row + 12 * L_k + 4 * budget)


def cpu_baseline(wl, d, a, rows_per_chunk):
    """Time the fp64 oracle, as it stands, single-threaded, on a bounded sample of the same
    workload: attention on sampled query rows of two heads; the change metric on the full
    tensors; scoring + selection + compaction of every head (about 10-20 s in all at the
    MAGI-1-like shape)."""
    from oracle import flowcache_oracle as O
    from threadpoolctl import threadpool_limits
    rec = list(range(wl.A))
    rng = np.random.default_rng(0)
    rows = []
    for r in rec:
        pick = {0, wl.L_c - 1, 255, 256}
        pick |= set(rng.integers(0, wl.L_c, size=rows_per_chunk).tolist())
        rows += [r * wl.L_c + int(x) for x in sorted(pick) if x < wl.L_c][:rows_per_chunk]
    heads = sorted({0, wl.H_q - 1})
    G = wl.H_q // wl.H_k
    kheads = sorted({h // G for h in heads})
    n_cmp = wl.H_k
    with threadpool_limits(limits=1):
        # the sample: the chosen heads only (the oracle widens whatever it is given to float64)
        kc = O.scatter_kv(a["k_cache"][kheads], a["k_new"][:, kheads], rec, a["active_off"], wl.L_c)
        vc = O.scatter_kv(a["v_cache"][kheads], a["v_new"][:, kheads], rec, a["active_off"], wl.L_c)
        q = np.ascontiguousarray(a["q"][:, heads])
        t0 = time.perf_counter()
        O.attend(q, kc, vc, wl.L_clean, a["active_off"], wl.L_c, rec, rows=rows)
        t_att = time.perf_counter() - t0
        pairs = sum(wl.L_clean + (rows_i // wl.L_c + 1) * wl.L_c for rows_i in rows)
        flops = 4.0 * wl.d * pairs * len(heads)
        t0 = time.perf_counter()
        O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, 0.0, d["acc"])
        t_dec = time.perf_counter() - t0
        mass = np.full((n_cmp, wl.L_k), 1.0 / wl.L_k, dtype=np.float32)
        kh = np.ascontiguousarray(a["k_cache"][:n_cmp, :wl.L_k])
        vh = np.ascontiguousarray(a["v_cache"][:n_cmp, :wl.L_k])
        t0 = time.perf_counter()
        O.kv_compress(kh, vh, wl.L_k, wl.budget, mass, wl.pool_k, wl.lam)
        t_cmp = time.perf_counter() - t0
    esz = 2 if wl.dtype == "bf16" else 4
    cmp_bytes = compress_min_bytes(wl, wl.L_k, wl.budget) * n_cmp / wl.H_k
    return {
        "value": flops / t_att / 1e12, "unit": "TFLOP/s", "cores": 1, "nproc": os.cpu_count(),
        "kind": "oracle",
        "sample": (f"fp64 numpy oracle on one thread: attention on {len(rows)} query rows x {len(heads)} "
                   f"heads ({flops / 1e9:.1f} GFLOP in {t_att:.2f} s; the whole tensor would take "
                   f"{wl.attention_flops() / (flops / t_att):.0f} s); change metric on the full tensors "
                   f"in {t_dec:.2f} s ({2 * wl.A * wl.chunk_elems * esz / t_dec / 1e9:.2f} GB/s); "
                   f"compression of {n_cmp} of {wl.H_k} heads in {t_cmp:.2f} s "
                   f"({cmp_bytes / t_cmp / 1e9:.3f} GB/s)"),
        "attention_s": t_att, "decide_s": t_dec, "compress_s": t_cmp,
        "decide_GBps": 2 * wl.A * wl.chunk_elems * esz / t_dec / 1e9, "compress_GBps": cmp_bytes / t_cmp / 1e9,
    }


def run_workload(wl, args, K, W, with_cpu, torch, B, synth):
    """All measurements of one workload -> the fields of the JSON line."""
    dev = "cuda"
    K_ALONE = 5     # steps after the timed region in which every call is timed alone
    nset = K + W + 2 * K_ALONE + 2
    code = B.FC_BF16 if wl.dtype == "bf16" else B.FC_F32
    esz = 2 if wl.dtype == "bf16" else 4

    # ---- synthetic inputs, resident in HBM before the timed region -------------------
    d = synth.decide_inputs(wl, seed=0)
    a = synth.attend_inputs(wl, seed=0)
    NDEC = 4   # rotate the streaming operands so they never sit in the 256 MB Infinity Cache
    x_cur = [B.to_device(d["x_cur"], wl.dtype, dev) for _ in range(NDEC)]
    x_prev = [B.to_device(d["x_prev"], wl.dtype, dev) for _ in range(NDEC)]
    x_compact = [torch.empty_like(x_cur[0]) for _ in range(2)]
    step_idx = torch.from_numpy(d["step_idx"]).to(dev)
    acc = torch.zeros(wl.A, dtype=torch.float64, device=dev)
    q = B.to_device(a["q"], wl.dtype, dev)
    k_new = [B.to_device(a["k_new"], wl.dtype, dev) for _ in range(2)]
    v_new = [B.to_device(a["v_new"], wl.dtype, dev) for _ in range(2)]
    out = torch.empty_like(q)
    k0 = B.to_device(a["k_cache"], wl.dtype, dev)
    v0 = B.to_device(a["v_cache"], wl.dtype, dev)
    if args.qkv == "const":
        q.fill_(0.125); k0.fill_(0.5); v0.fill_(1.0)
        for t in k_new: t.fill_(0.5)
        for t in v_new: t.fill_(1.0)
    k_sets = [k0] + [k0.clone() for _ in range(nset - 1)]   # a fresh cache for every step:
    v_sets = [v0] + [v0.clone() for _ in range(nset - 1)]   # compression is destructive
    active_off = a["active_off"]
    L_k, budget = wl.L_k, wl.budget
    Wobs = wl.obs_window
    kept = torch.empty((wl.H_k, budget), dtype=torch.int32, device=dev)
    L = B.lib()

    def ws(nbytes):
        return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=dev)

    ws_dec = ws(L.flowcache_chunk_decide_workspace(wl.A, wl.chunk_elems))
    ws_att = ws(L.flowcache_attend_workspace(wl.A, wl.L_c, wl.H_q, wl.H_k, wl.d, 0, Wobs))
    ws_mass = ws(L.flowcache_attention_mass_workspace(Wobs, wl.H_q, wl.H_k, wl.d, L_k))
    ws_cmp = ws(L.flowcache_kv_compress_workspace(wl.H_k, L_k, wl.d, budget, code))
    q_obs = q[wl.A * wl.L_c - Wobs:]          # last W rows of the last active chunk

    names = ["decide", "scatter", "attend", "mass", "compress"]
    main_stream = torch.cuda.current_stream()
    side_stream = torch.cuda.Stream()          # default priority

    def new_events(n):
        return [torch.cuda.Event(enable_timing=True) for _ in range(n)]

    def step_sequential(i, events=None):
        s = i % NDEC
        if events: events[0].record()
        dec = B.flowcache_chunk_decide(x_cur[s], x_prev[s], step_idx, wl.warmup_m, 0.0, acc,
                                       x_compact=x_compact[i % 2], workspace=ws_dec)
        if events: events[1].record()
        B.flowcache_scatter_kv(k_new[i % 2], v_new[i % 2], k_sets[i], v_sets[i], wl.L_c, wl.L_clean,
                               active_off, dec["recompute_idx"], dec["n_recompute"])
        if events: events[2].record()
        B.flowcache_attend(q, None, None, k_sets[i], v_sets[i], wl.L_c, wl.L_clean, active_off,
                           dec["recompute_idx"], dec["n_recompute"], out=out, want_lse=False,
                           workspace=ws_att)
        if events: events[3].record()
        mass = B.flowcache_attention_mass(q_obs, k_sets[i], L_k, workspace=ws_mass)
        if events: events[4].record()
        B.flowcache_kv_compress(k_sets[i], v_sets[i], L_k, budget, mass, wl.pool_k, wl.lam,
                                kept_idx=kept, workspace=ws_cmp)
        if events: events[5].record()
        return dec

    def step_overlapped(i, events=None):
        """events: 0-3 decide / scatter / attend on the main stream, 4-5 around the compaction,
        6-8 mass / selection on the side stream."""
        s = i % NDEC
        if events: events[0].record()
        dec = B.flowcache_chunk_decide(x_cur[s], x_prev[s], step_idx, wl.warmup_m, 0.0, acc,
                                       x_compact=x_compact[i % 2], workspace=ws_dec)
        if events: events[1].record()
        B.flowcache_scatter_kv(k_new[i % 2], v_new[i % 2], k_sets[i], v_sets[i], wl.L_c, wl.L_clean,
                               active_off, dec["recompute_idx"], dec["n_recompute"])
        if events: events[2].record()
        fork = torch.cuda.Event()
        fork.record(main_stream)
        with torch.cuda.stream(side_stream):       # K is final after the scatter: read-only work
            side_stream.wait_event(fork)
            if events: events[6].record(side_stream)
            mass = B.flowcache_attention_mass(q_obs, k_sets[i], L_k, workspace=ws_mass)
            if events: events[7].record(side_stream)
            B.flowcache_kv_select(k_sets[i], L_k, budget, mass, wl.pool_k, wl.lam, kept_idx=kept,
                                  workspace=ws_cmp)
            if events: events[8].record(side_stream)
            join = torch.cuda.Event()
            join.record(side_stream)
        B.flowcache_attend(q, None, None, k_sets[i], v_sets[i], wl.L_c, wl.L_clean, active_off,
                           dec["recompute_idx"], dec["n_recompute"], out=out, want_lse=False,
                           workspace=ws_att)
        if events: events[3].record()
        main_stream.wait_event(join)               # the compaction overwrites what both read
        if events: events[4].record()
        B.flowcache_kv_compact(k_sets[i], v_sets[i], L_k, budget, kept, workspace=ws_cmp)
        if events: events[5].record()
        return dec

    step = step_overlapped if args.overlap else step_sequential
    ev = [new_events(9) for _ in range(K)]
    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        dec = step(W + i, ev[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert int(dec["n_recompute"].item()) == wl.A, "eps = 0 must recompute every chunk"

    def mean_ms(evs, j0, j1):
        return float(np.mean([e[j0].elapsed_time(e[j1]) for e in evs]))

    if not args.overlap:
        stage_ms = {n: mean_ms(ev, j, j + 1) for j, n in enumerate(names)}
    else:
        stage_ms = {"decide": mean_ms(ev, 0, 1), "scatter": mean_ms(ev, 1, 2), "attend": mean_ms(ev, 2, 3),
                    "mass (side stream, beside attend)": mean_ms(ev, 6, 7),
                    "select (side stream, beside attend)": mean_ms(ev, 7, 8),
                    "compact": mean_ms(ev, 4, 5)}

    # ---- every call alone: sequential steps outside the timed region --------------------
    base = W + K
    ev_alone = [new_events(6) for _ in range(K_ALONE)]
    step_sequential(base)
    for i in range(K_ALONE):
        step_sequential(base + 1 + i, ev_alone[i])
    torch.cuda.synchronize()
    alone = {n: mean_ms(ev_alone, j, j + 1) for j, n in enumerate(names)}

    # ---- the halves of the decide and compress calls, and the calls beside the step -----
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def timed(fn, reps=K_ALONE):
        """Mean duration of fn's kernels on the GPU.  A spin kernel that touches no memory is
        queued first, so that both events and the call's launches are already waiting when
        it ends: the figure is GPU time, without the host's launch latency."""
        ts = []
        for i in range(reps + 1):
            torch.cuda._sleep(400_000)
            e0.record(); fn(i); e1.record(); e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.mean(ts[1:]))

    alone["decide_metric"] = timed(lambda i: B.flowcache_chunk_decide(
        x_cur[i % NDEC], x_prev[i % NDEC], step_idx, wl.warmup_m, 0.0, acc, gather=False, workspace=ws_dec))
    base2 = base + 1 + K_ALONE
    mass_d = B.flowcache_attention_mass(q_obs, k_sets[0], L_k, workspace=ws_mass)
    alone["select"] = timed(lambda i: B.flowcache_kv_select(
        k_sets[base2 + i], L_k, budget, mass_d, wl.pool_k, wl.lam, kept_idx=kept, workspace=ws_cmp))
    alone["compact"] = timed(lambda i: B.flowcache_kv_compact(
        k_sets[base2 + i], v_sets[base2 + i], L_k, budget, kept, workspace=ws_cmp))
    one = wl.A * wl.chunk_elems * esz
    res = torch.zeros_like(x_cur[0])
    outx = torch.empty_like(x_cur[0])
    none = torch.full((wl.A,), -1, dtype=torch.int32, device=dev)
    zero = torch.zeros(1, dtype=torch.int32, device=dev)
    accg = torch.zeros(1, dtype=torch.float64, device=dev)
    alone["residual_store"] = timed(lambda i: B.flowcache_residual_apply(
        x_cur[i % NDEC], x_compact[i % 2], res, dec["recompute_idx"], dec["n_recompute"], out=outx))
    alone["residual_apply"] = timed(lambda i: B.flowcache_residual_apply(
        x_cur[i % NDEC], None, res, none, zero, out=outx))
    alone["uniform_decide"] = timed(lambda i: B.flowcache_uniform_decide(
        x_cur[i % NDEC], x_prev[i % NDEC], step_idx, wl.warmup_m, 0.0, accg, x_compact=x_compact[i % 2],
        workspace=ws_dec))
    Wf = wl.L_c // 5                         # frame-level observation queries: one fifth of a chunk
    q_frame = q[wl.A * wl.L_c - Wf:]
    alone["mass_frame_queries"] = timed(lambda i: B.flowcache_attention_mass(q_frame, k_sets[0], L_k), reps=3)

    ms_per_step = wall * 1e3 / K
    flops = float(wl.attention_flops())
    att_tflops = flops / (stage_ms["attend"] * 1e-3) / 1e12      # in the timed region
    k_bytes = wl.H_k * L_k * wl.d * esz
    cmp_bytes = compress_min_bytes(wl, L_k, budget)
    kept_rw = 4 * wl.H_k * budget * wl.d * esz

    def hbm(name, key, nbytes, note=None, read_only=0):
        """frac: against the datasheet rate.  frac_measured: against the time the same bytes take
        at the rates a plain read and a plain copy sustain on this chip from cold (peak_probe):
        `read_only` of the bytes are only read, the rest is read-and-written."""
        g = nbytes / (alone[key] * 1e-3) / 1e9
        floor_ms = (read_only / MEASURED_READ_GBPS + (nbytes - read_only) / MEASURED_COPY_GBPS) / 1e6
        r = {"call": name, "bound": "hbm", "algorithmic_bytes": int(nbytes), "ms": alone[key],
             "achieved": g, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": g / PEAK_HBM_GBPS,
             "frac_measured": floor_ms / alone[key]}
        if note:
            r["note"] = note
        return r

    gather_ms = max(alone["decide"] - alone["decide_metric"], 1e-6)
    alone["gather"] = gather_ms
    calls = [
        hbm("decide (metric + decision + gather)", "decide", 4 * one, read_only=2 * one),
        hbm("decide_metric (metric + decision, no gather)", "decide_metric", 2 * one, read_only=2 * one),
        hbm("gather (decide minus decide_metric)", "gather", 2 * one),
        hbm("scatter", "scatter", 2 * 2 * wl.A * wl.L_c * wl.H_k * wl.d * esz),
        hbm("mass", "mass", k_bytes, "algorithmic bytes = K once; the kernels read K twice", read_only=k_bytes),
        hbm("compress", "compress", cmp_bytes, read_only=cmp_bytes - kept_rw),
        hbm("select (scoring + top-B, first half of compress)", "select", cmp_bytes - kept_rw,
            read_only=cmp_bytes - kept_rw),
        hbm("compact (second half of compress)", "compact", kept_rw + 4 * wl.H_k * budget),
        hbm("residual_apply (all chunks recomputed: store)", "residual_store", 4 * one),
        hbm("residual_apply (all chunks reused: apply)", "residual_apply", 3 * one, read_only=one),
        hbm("uniform_decide (+ gather)", "uniform_decide", 4 * one, read_only=2 * one),
    ]
    fl = 2.0 * 2 * wl.d * Wf * wl.H_q * L_k                # two passes of Q K^T
    calls.append({"call": f"attention_mass, frame-level queries (W = {Wf})", "bound": "mfma",
                  "ms": alone["mass_frame_queries"], "algorithmic_flops": fl,
                  "achieved": fl / alone["mass_frame_queries"] / 1e9, "peak": PEAK_BF16_TFLOPS,
                  "unit": "TFLOP/s", "frac": fl / alone["mass_frame_queries"] / 1e9 / PEAK_BF16_TFLOPS,
                  "frac_measured": fl / alone["mass_frame_queries"] / 1e9 / MEASURED_MFMA_TFLOPS})

    result = {
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s (attention FLOPs / whole-step time)",
        "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "dtype": wl.dtype,
        "data": "synthetic" if args.qkv == "normal" else "synthetic-constant-qkv (NOT a bench result)",
        "config": {"workload": wl.name, "H_q": wl.H_q, "H_k": wl.H_k, "d": wl.d, "A": wl.A,
                   "L_c": wl.L_c, "L_clean": wl.L_clean, "budget": wl.budget, "eps": 0.0,
                   "recompute": "all chunks", "obs_window": Wobs, "pool_k": wl.pool_k,
                   "lambda": wl.lam},
        "roofline": {"kernel": "attend_bf16_kernel", "bound": "mfma", "achieved": att_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": att_tflops / PEAK_BF16_TFLOPS,
                     "traffic": attend_traffic_bytes(wl.name), "algorithmic_flops": flops,
                     "algorithmic_bytes": int(2 * wl.A * wl.L_c * wl.H_q * wl.d * esz
                                              + 2 * wl.H_k * wl.capacity * wl.d * esz),
                     "ms": stage_ms["attend"],
                     "peak_measured": MEASURED_MFMA_TFLOPS, "frac_measured": att_tflops / MEASURED_MFMA_TFLOPS,
                     "note": "a loop of nothing but bf16 MFMAs on random operands sustains 1330-1410 "
                             "TFLOP/s on this chip (power-limited; profiles/peaks_measured.md)"},
        "kv_compress_GBps": cmp_bytes / (alone["compress"] * 1e-3) / 1e9,
        "calls": calls,
        "stage_ms": stage_ms,
        "stage_ms_alone": {n: alone[n] for n in names},
        "streams": "one" if not args.overlap else
                   "two: mass and selection run beside the attention kernel, the compaction after both",
    }
    result["cpu_baseline"] = cpu_baseline(wl, d, a, args.cpu_rows) if with_cpu else None
    return result


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (every box has one MI355X); "
              "run it with --gpus 1.  The path would shard by attention heads across GPUs.",
              file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2602_10825_amd import binding as B
    from paper_2602_10825_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if not os.path.exists(B.LIB_PATH):      # load what is built; build only if nothing is
        from paper_2602_10825_amd.build import build
        build(verbose=False)
    B.lib()   # fail loudly if the HIP library is missing
    table = {"C2": synth.C2, "C3": synth.C3, "mid": synth.MID_BF16}
    main_res = run_workload(table[args.workload], args, args.steps, args.warmup, not args.no_cpu,
                            torch, B, synth)
    result = {"metric": "denoise-step attention TFLOP/s (% MFMA peak) + KV-compress HBM GB/s",
              "value": main_res.pop("value"), "unit": main_res.pop("unit"), "n_gpus": 1,
              "steps": main_res.pop("steps"), "warmup": main_res.pop("warmup"),
              "ms_per_step": main_res.pop("ms_per_step"), "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None}
    result.update(main_res)
    if args.secondary != "none" and args.secondary != args.workload:
        gc.collect()
        torch.cuda.empty_cache()
        sec = run_workload(table[args.secondary], args, min(args.steps, 10), min(args.warmup, 5), False,
                           torch, B, synth)
        sec.pop("cpu_baseline", None)
        result["secondary"] = sec
    print(json.dumps(result))


if __name__ == "__main__":
    main()
