#!/usr/bin/env python3
"""Benchmark of the FlowCache denoising-step hot path on one MI355X.

One *step* is one pass of the whole hot path over one batch of synthetic input, at the
SkyReels-V2-1.3B-like single-layer shape (12 heads x 128, 2 active chunks of 10200 tokens,
40800 clean tokens compressed to 20400):

    flowcache_chunk_decide   change metric + decision + gather of x
    flowcache_scatter_kv     new K/V of the recompute chunks into their cache slots
    flowcache_attend         chunk-causal bf16 attention (all chunks recompute: eps = 0)
    flowcache_attention_mass importance of the first L_k cache positions (50 observation rows)
    flowcache_kv_select      scoring and top-B selection  } together = flowcache_kv_compress
    flowcache_kv_compact     in-place compaction          } (fresh cache copy per step)

The calls run back to back on one stream.  The importance mass and the selection only read K,
so with ``--overlap`` the step runs them on a second HIP stream beside the attention kernel
(they fit into the partly empty last round of its launch) and the compaction, which overwrites
K and V, waits for both: about 1 % more steps per second on C2, at the price of an attention
kernel that is itself about 1 % slower, so it is not the default.  After the timed region a
few sequential steps give every call's duration alone (``stage_ms_alone``).

Inputs are resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2|C3|mid] [--no-cpu]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 matrix peak
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E peak
# HBM bytes per launch of the attention kernel on C2, from two rocprofv3 --pmc runs of this
# script (FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 KiB, factors calibrated on the 188 MB copy kernel
# of the same runs; profiles/bench_C2_hbm_traffic.md)
ATTEND_TRAFFIC_BYTES = {"C2-skyreels-v2-1.3B-like-bf16": int((916401.8 * 2.0 + 88487.9 * 1.0) * 1024)}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="C2", choices=["C2", "C3", "mid"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle (cpu_baseline) leg")
    ap.add_argument("--cpu-rows", type=int, default=768, help="oracle attention rows per chunk")
    ap.add_argument("--overlap", action="store_true",
                    help="two streams: mass and selection beside the attention instead of after it")
    ap.add_argument("--qkv", default="normal", choices=["normal", "const"],
                    help="const: constant Q/K/V (same instruction stream, full clocks) -- shows how "
                         "much of the attention time is the power limit; not a valid bench result")
    return ap.parse_args()


def compress_min_bytes(wl, L_k, budget):
    """Algorithmic HBM bytes of one kv_compress call: K read once for scoring, kept K and V
    rows read and written once, 12 B/token/head of mass + score, 4 B per kept index."""
    esz = 2 if wl.dtype == "bf16" else 4
    row = wl.d * esz
    return wl.H_k * (L_k * row + 4 * budget * row + 12 * L_k + 4 * budget)


def cpu_baseline(wl, d, a, rows_per_chunk):
    """Time the fp64 oracle, as it stands, on a bounded sample of the same workload."""
    from oracle import flowcache_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    rec = list(range(wl.A))
    rng = np.random.default_rng(0)
    rows = []
    for r in rec:
        pick = {0, wl.L_c - 1, 255, 256}
        pick |= set(rng.integers(0, wl.L_c, size=rows_per_chunk).tolist())
        rows += [r * wl.L_c + int(x) for x in sorted(pick) if x < wl.L_c][:rows_per_chunk]
    heads = [0, wl.H_q - 1]
    kc = O.scatter_kv(a["k_cache"], a["k_new"], rec, a["active_off"], wl.L_c)
    vc = O.scatter_kv(a["v_cache"], a["v_new"], rec, a["active_off"], wl.L_c)
    t0 = time.perf_counter()
    out, _ = O.attend(a["q"], kc, vc, wl.L_clean, a["active_off"], wl.L_c, rec, rows=rows, heads=heads)
    t_att = time.perf_counter() - t0
    pairs = sum(wl.L_clean + (rows_i // wl.L_c + 1) * wl.L_c for rows_i in rows)
    flops = 4.0 * wl.d * pairs * len(heads)
    t0 = time.perf_counter()
    O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, 0.0, d["acc"])
    t_dec = time.perf_counter() - t0
    mass = np.full((wl.H_k, wl.L_k), 1.0 / wl.L_k, dtype=np.float32)
    t0 = time.perf_counter()
    O.kv_compress(kc[:, :wl.L_k], vc[:, :wl.L_k], wl.L_k, wl.budget, mass, wl.pool_k, wl.lam)
    t_cmp = time.perf_counter() - t0
    esz = 2 if wl.dtype == "bf16" else 4
    return {
        "value": flops / t_att / 1e12, "unit": "TFLOP/s", "cores": int(cores), "kind": "oracle",
        "sample": (f"fp64 numpy oracle: attention on {len(rows)} query rows x {len(heads)} heads "
                   f"({flops / 1e9:.1f} GFLOP in {t_att:.2f} s; whole tensor would take "
                   f"{wl.attention_flops() / (flops / t_att):.0f} s); change metric on the full "
                   f"tensors in {t_dec:.2f} s ({2 * wl.A * wl.chunk_elems * esz / t_dec / 1e9:.2f} GB/s); "
                   f"compression of all {wl.H_k} heads in {t_cmp:.2f} s "
                   f"({compress_min_bytes(wl, wl.L_k, wl.budget) / t_cmp / 1e9:.3f} GB/s)"),
        "attention_s": t_att, "decide_s": t_dec, "compress_s": t_cmp,
    }


def widened_rows(wl, B, x_cur, x_prev, x_compact, step_idx, dec, q, k_cache, ws_dec, L_k, reps=5):
    """Calls outside the timed step (rows widened into after the hot path): timed alone, HIP
    events, operands rotated like the step's."""
    import torch
    esz = 2 if wl.dtype == "bf16" else 4
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def best(fn):
        ts = []
        for i in range(reps + 1):
            e0.record(); fn(i); e1.record(); e1.synchronize()
            ts.append(e0.elapsed_time(e1))
        return float(np.mean(ts[1:]))

    one = wl.A * wl.chunk_elems * esz
    res = torch.zeros_like(x_cur[0])
    out = torch.empty_like(x_cur[0])
    none = torch.full((wl.A,), -1, dtype=torch.int32, device=q.device)
    zero = torch.zeros(1, dtype=torch.int32, device=q.device)
    accg = torch.zeros(1, dtype=torch.float64, device=q.device)
    rows = []
    ms = best(lambda i: B.flowcache_residual_apply(x_cur[i % len(x_cur)], x_compact, res,
                                                   dec["recompute_idx"], dec["n_recompute"], out=out))
    rows.append({"call": "residual_apply (all chunks recomputed: store)", "ms": ms,
                 "algorithmic_bytes": 4 * one, "GBps": 4 * one / ms / 1e6})
    ms = best(lambda i: B.flowcache_residual_apply(x_cur[i % len(x_cur)], None, res, none, zero, out=out))
    rows.append({"call": "residual_apply (all chunks reused: apply)", "ms": ms,
                 "algorithmic_bytes": 3 * one, "GBps": 3 * one / ms / 1e6})
    ms = best(lambda i: B.flowcache_uniform_decide(x_cur[i % len(x_cur)], x_prev[i % len(x_prev)], step_idx,
                                                   wl.warmup_m, 0.0, accg, x_compact=x_compact,
                                                   workspace=ws_dec))
    rows.append({"call": "uniform_decide (+ gather)", "ms": ms, "algorithmic_bytes": 4 * one,
                 "GBps": 4 * one / ms / 1e6})
    Wf = wl.L_c // 5                         # frame-level observation queries: one fifth of a chunk
    q_frame = q[wl.A * wl.L_c - Wf:]
    ms = best(lambda i: B.flowcache_attention_mass(q_frame, k_cache, L_k))
    fl = 2.0 * 2 * wl.d * Wf * wl.H_q * L_k                # two passes of Q K^T
    rows.append({"call": f"attention_mass, frame-level queries (W = {Wf})", "ms": ms,
                 "algorithmic_flops": fl, "TFLOPps": fl / ms / 1e9})
    for r in rows:
        if "GBps" in r:
            r["frac_of_hbm_peak"] = r["GBps"] / PEAK_HBM_GBPS
    return rows


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
    wl = {"C2": synth.C2, "C3": synth.C3, "mid": synth.MID_BF16}[args.workload]
    dev = "cuda"
    K, W = args.steps, args.warmup
    K_ALONE = 5     # sequential steps after the timed region: every call's duration alone
    nset = K + W + K_ALONE + 1

    # ---- synthetic inputs, resident in HBM before the timed region -------------------
    d = synth.decide_inputs(wl, seed=0)
    a = synth.attend_inputs(wl, seed=0)
    NDEC = 4   # rotate the change-metric operands so they never sit in the 256 MB MALL
    x_cur = [B.to_device(d["x_cur"], wl.dtype, dev) for _ in range(NDEC)]
    x_prev = [B.to_device(d["x_prev"], wl.dtype, dev) for _ in range(NDEC)]
    x_compact = torch.empty_like(x_cur[0])
    step_idx = torch.from_numpy(d["step_idx"]).to(dev)
    acc = torch.zeros(wl.A, dtype=torch.float64, device=dev)
    q = B.to_device(a["q"], wl.dtype, dev)
    k_new = B.to_device(a["k_new"], wl.dtype, dev)
    v_new = B.to_device(a["v_new"], wl.dtype, dev)
    out = torch.empty_like(q)
    k0 = B.to_device(a["k_cache"], wl.dtype, dev)
    v0 = B.to_device(a["v_cache"], wl.dtype, dev)
    if args.qkv == "const":
        q.fill_(0.125); k_new.fill_(0.5); v_new.fill_(1.0); k0.fill_(0.5); v0.fill_(1.0)
    k_sets = [k0] + [k0.clone() for _ in range(nset - 1)]   # a fresh cache for every step:
    v_sets = [v0] + [v0.clone() for _ in range(nset - 1)]   # compression is destructive
    active_off = a["active_off"]
    L_k, budget = wl.L_k, wl.budget
    Wobs = wl.obs_window
    kept = torch.empty((wl.H_k, budget), dtype=torch.int32, device=dev)
    L = B.lib()
    ws_dec = torch.empty(L.flowcache_chunk_decide_workspace(wl.A, wl.chunk_elems), dtype=torch.uint8, device=dev)
    ws_att = torch.empty(L.flowcache_attend_workspace(wl.A, wl.L_c, wl.H_q, wl.H_k, wl.d, 0, Wobs),
                         dtype=torch.uint8, device=dev)
    ws_mass = torch.empty(L.flowcache_attention_mass_workspace(Wobs, wl.H_q, wl.H_k, wl.d, L_k),
                          dtype=torch.uint8, device=dev)
    ws_cmp = torch.empty(L.flowcache_kv_compress_workspace(wl.H_k, L_k, wl.d, budget, B.FC_BF16 if wl.dtype == "bf16" else B.FC_F32),
                         dtype=torch.uint8, device=dev)
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
                                       x_compact=x_compact, workspace=ws_dec)
        if events: events[1].record()
        B.flowcache_scatter_kv(k_new, v_new, k_sets[i], v_sets[i], wl.L_c, wl.L_clean, active_off,
                               dec["recompute_idx"], dec["n_recompute"])
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
                                       x_compact=x_compact, workspace=ws_dec)
        if events: events[1].record()
        B.flowcache_scatter_kv(k_new, v_new, k_sets[i], v_sets[i], wl.L_c, wl.L_clean, active_off,
                               dec["recompute_idx"], dec["n_recompute"])
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
    # every call alone: a few sequential steps outside the timed region
    ev_alone = [new_events(6) for _ in range(K_ALONE)]
    step_sequential(W + K)
    for i in range(K_ALONE):
        step_sequential(W + K + 1 + i, ev_alone[i])
    torch.cuda.synchronize()
    stage_alone = {n: mean_ms(ev_alone, j, j + 1) for j, n in enumerate(names)}
    ms_per_step = wall * 1e3 / K
    flops = float(wl.attention_flops())
    esz = 2 if wl.dtype == "bf16" else 4
    att_tflops = flops / (stage_ms["attend"] * 1e-3) / 1e12      # in the timed region
    dec_bytes = 2 * wl.A * wl.chunk_elems * esz + 2 * wl.A * wl.chunk_elems * esz   # metric + gather r/w
    cmp_bytes = compress_min_bytes(wl, L_k, budget)
    sc_bytes = 2 * 2 * wl.A * wl.L_c * wl.H_k * wl.d * esz
    mass_bytes = 2 * wl.H_k * L_k * wl.d * esz

    def hbm(name, nbytes):
        g = nbytes / (stage_alone[name] * 1e-3) / 1e9
        return {"call": name, "bound": "hbm", "algorithmic_bytes": int(nbytes), "ms": stage_alone[name],
                "achieved": g, "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": g / PEAK_HBM_GBPS}

    result = {
        "metric": "denoise-step attention TFLOP/s (% MFMA peak) + KV-compress HBM GB/s",
        "value": flops / (ms_per_step * 1e-3) / 1e12,
        "unit": "TFLOP/s (attention FLOPs / whole-step time)",
        "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic" if args.qkv == "normal" else "synthetic-constant-qkv (NOT a bench result)",
        "config": {"workload": wl.name, "H_q": wl.H_q, "H_k": wl.H_k, "d": wl.d, "A": wl.A,
                   "L_c": wl.L_c, "L_clean": wl.L_clean, "budget": wl.budget, "eps": 0.0,
                   "recompute": "all chunks", "obs_window": Wobs, "pool_k": wl.pool_k,
                   "lambda": wl.lam},
        "roofline": {"kernel": "attend_bf16_kernel", "bound": "mfma", "achieved": att_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": att_tflops / PEAK_BF16_TFLOPS,
                     "traffic": ATTEND_TRAFFIC_BYTES.get(wl.name), "algorithmic_flops": flops,
                     "ms": stage_ms["attend"],
                     "note": "a loop of nothing but bf16 MFMAs on random operands sustains 1330-1410 "
                             "TFLOP/s on this chip (power-limited; profiles/peaks_measured.md)"},
        "kv_compress_GBps": cmp_bytes / (stage_alone["compress"] * 1e-3) / 1e9,
        "calls": [hbm("decide", dec_bytes), hbm("scatter", sc_bytes), hbm("mass", mass_bytes),
                  hbm("compress", cmp_bytes)],
        "stage_ms": stage_ms,
        "stage_ms_alone": stage_alone,
        "streams": "one" if not args.overlap else
                   "two: mass and selection run beside the attention kernel, the compaction after both",
    }
    result["widened_rows"] = widened_rows(wl, B, x_cur, x_prev, x_compact, step_idx, dec, q, k_sets[0],
                                          ws_dec, L_k)
    if not args.no_cpu:
        result["cpu_baseline"] = cpu_baseline(wl, d, a, args.cpu_rows)
    else:
        result["cpu_baseline"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
