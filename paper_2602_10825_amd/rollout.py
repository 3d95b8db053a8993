"""Synthetic long rollout driven through the library: scheduler -> per tick { chunk decide +
gather, per layer { stand-in projections, K/V scatter, chunk-causal attention }, cached-
activation store/apply } -> per commit { move the finished chunk next to the clean region,
importance mass, compression }.

The "model" is a stand-in: random-init bf16 projection matrices applied with torch.matmul
(harness work, not part of the path) and a prescribed per-step change of each chunk's input.
What is real is every FlowCache step, which runs in the library's kernels on device-resident
decisions.  ``run_rollout`` returns per-tick decisions, per-commit kept indices (optionally)
and timing / work totals, so that a thresholded run can be set beside the eps = 0 run.

    python -m paper_2602_10825_amd.rollout --layers 4 --units 6 --steps 12
"""
from __future__ import annotations

import argparse
import json
import sys
import time
from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional

import numpy as np
import torch

from . import binding as B


@dataclass
class RolloutConfig:
    H: int = 12                 # heads (MHA)
    d: int = 128                # head dim
    L_c: int = 10200            # tokens per chunk
    n_layers: int = 30
    n_units: int = 16           # chunks to generate
    steps: int = 30             # denoising steps per chunk
    stagger: int = 15           # ticks between chunk starts (window = steps / stagger)
    budget_chunks: int = 4      # clean-cache budget, in chunks
    warmup_m: int = 4
    eps: float = 0.1
    obs_window: int = 50
    pool_k: int = 7
    lam: float = 0.07
    delta0: float = 0.03        # relative change per step for the first 5 steps of a chunk ...
    decay: float = 0.85         # ... then multiplied by this every step
    seed: int = 0

    @property
    def D(self) -> int:
        return self.H * self.d


def step_delta(cfg: RolloutConfig, s: int) -> float:
    """Prescribed relative change of a chunk's input at its local step s."""
    return cfg.delta0 if s < 5 else cfg.delta0 * cfg.decay ** (s - 5)


@dataclass
class RolloutResult:
    masks: List[List[int]] = field(default_factory=list)         # per tick, per active chunk
    units: List[List[int]] = field(default_factory=list)
    kept: List[np.ndarray] = field(default_factory=list)         # per compressing commit, layer 0
    stats: Dict[str, float] = field(default_factory=dict)


def run_rollout(cfg: RolloutConfig, device: str = "cuda", keep_indices: bool = False,
                observer: Optional[Callable[[str, Dict], None]] = None) -> RolloutResult:
    """Runs the whole schedule.  ``observer(event, info)`` is called with device tensors after
    "decide", after layer 0's "attend" and after layer 0's "commit" (the tests use it to
    mirror the run on the host)."""
    L_c, H, d, D = cfg.L_c, cfg.H, cfg.d, cfg.D
    budget = cfg.budget_chunks * L_c
    sch = B.Scheduler(cfg.n_units, cfg.steps, cfg.stagger, L_c, budget)
    cap = sch.capacity
    window = -(-cfg.steps // cfg.stagger)
    g = torch.Generator(device=device)
    g.manual_seed(cfg.seed)
    bf = torch.bfloat16
    w_qkv = [(torch.randn((D, 3 * D), device=device, generator=g) * D ** -0.5).to(bf)
             for _ in range(cfg.n_layers)]
    k_cache = [torch.zeros((H, cap, d), dtype=bf, device=device) for _ in range(cfg.n_layers)]
    v_cache = [torch.zeros((H, cap, d), dtype=bf, device=device) for _ in range(cfg.n_layers)]
    # per ring slot: current / previous input of the chunk living there, residual cache
    x_slot = torch.zeros((window, L_c, D), dtype=bf, device=device)
    res_slot = torch.zeros((window, L_c * D), dtype=bf, device=device)
    acc_slot = torch.zeros(window, dtype=torch.float64, device=device)
    q_obs_cache = [torch.zeros((cfg.obs_window, H, d), dtype=bf, device=device)
                   for _ in range(cfg.n_layers)]
    L = B.lib()
    res = RolloutResult()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    att_ms = cmp_ms = dec_ms = 0.0
    att_flops = 0.0
    n_dec = n_rec_total = n_commit = 0
    cmp_bytes = 0.0
    t_wall = time.perf_counter()

    def timed(fn):
        ev0.record()
        out = fn()
        ev1.record()
        ev1.synchronize()
        return out, ev0.elapsed_time(ev1)

    for tk in sch:
        A = tk["A"]
        slots = [u % window for u in tk["unit"]]
        # ---- stand-in denoiser input: a new chunk starts from noise, others drift -------------
        x_prev = x_slot[slots].reshape(A, L_c * D).contiguous()
        for a, (s, sl) in enumerate(zip(tk["step_idx"], slots)):
            if s == 0:
                x_slot[sl] = torch.randn((L_c, D), device=device, generator=g).to(bf)
                x_prev[a] = x_slot[sl].reshape(-1)
                acc_slot[sl] = 0.0
                res_slot[sl].zero_()
            else:
                noise = torch.randn((L_c, D), device=device, generator=g)
                x_slot[sl] = (x_slot[sl].float() + step_delta(cfg, s) * noise).to(bf)
        x_cur = x_slot[slots].reshape(A, L_c * D).contiguous()
        step_idx = torch.tensor(tk["step_idx"], dtype=torch.int32, device=device)
        acc = acc_slot[slots].contiguous()
        acc_before = acc.clone() if observer else None
        # ---- a1 + a2: change metric, decision, gather ------------------------------------------
        dec, ms = timed(lambda: B.flowcache_chunk_decide(x_cur, x_prev, step_idx, cfg.warmup_m,
                                                         cfg.eps, acc))
        dec_ms += ms
        acc_slot[slots] = acc
        mask = dec["recompute_mask"].cpu().tolist()      # host copy: the harness sizes its GEMMs
        R = sum(mask)
        n_dec += A
        n_rec_total += R
        res.masks.append(mask)
        res.units.append(list(tk["unit"]))
        if observer:
            observer("decide", {"tick": tk, "x_cur": x_cur, "x_prev": x_prev, "acc_before": acc_before,
                                "dec": dec})
        y = dec["x_compact"].view(A, L_c, D).clone()        # running activation of the layer stack
        rec = [i for i in range(A) if mask[i]]
        for l in range(cfg.n_layers if R else 0):
            qkv = torch.matmul(y[:R].reshape(R * L_c, D), w_qkv[l])            # harness work
            q = torch.zeros((A * L_c, H, d), dtype=bf, device=device)
            kn, vn = torch.zeros_like(q), torch.zeros_like(q)
            q[:R * L_c] = qkv[:, :D].reshape(R * L_c, H, d)
            kn[:R * L_c] = qkv[:, D:2 * D].reshape(R * L_c, H, d)
            vn[:R * L_c] = qkv[:, 2 * D:].reshape(R * L_c, H, d)
            # ---- a2 (scatter) + a3: new K/V into the slots, chunk-causal attention -------------
            out, ms = timed(lambda: B.flowcache_attend(
                q, kn, vn, k_cache[l], v_cache[l], L_c, tk["L_clean"], tk["active_off"],
                dec["recompute_idx"], dec["n_recompute"], want_lse=False))
            att_ms += ms
            att_flops += sum(4.0 * d * H * L_c * (tk["L_clean"] + (c + 1) * L_c) for c in rec)
            o = out["out"].view(A, L_c, D)
            y[:R] = (y[:R].float() + o[:R].float()).to(bf)                    # stand-in block
            if mask[-1]:    # the newest chunk was recomputed: remember its observation queries
                q_obs_cache[l] = q[R * L_c - cfg.obs_window:R * L_c].clone()
            if observer and l == 0:
                observer("attend", {"tick": tk, "q": q, "k_new": kn, "v_new": vn, "out": out["out"],
                                    "dec": dec, "rec": rec, "k_cache": k_cache[0], "v_cache": v_cache[0]})
        # ---- cached-activation store / apply: full-layout output of the stack -----------------
        rs = res_slot[slots].contiguous()
        full = B.flowcache_residual_apply(x_cur, y.reshape(A, L_c * D) if R else None, rs,
                                          dec["recompute_idx"], dec["n_recompute"])
        res_slot[slots] = rs
        del full
        # ---- commit: the oldest chunk has taken its last step ---------------------------------
        if tk["commit_unit"] >= 0:
            n_commit += 1
            src, dst, merged = tk["commit_src_off"], tk["commit_dst_off"], tk["merged_len"]
            for l in range(cfg.n_layers):
                k_cache[l][:, dst:dst + L_c] = k_cache[l][:, src:src + L_c].clone()
                v_cache[l][:, dst:dst + L_c] = v_cache[l][:, src:src + L_c].clone()
                if not tk["compress"]:              # cache-filling phase: the append is all
                    if observer and l == 0:
                        observer("commit", {"tick": tk, "q_obs": None, "mass": None, "kept": None,
                                            "k_cache": k_cache[0], "v_cache": v_cache[0]})
                    continue
                # observation queries: last W rows of the newest chunk, from its last recompute
                q_obs = q_obs_cache[l]
                (mass, kept), ms = timed(lambda: _mass_and_compress(cfg, q_obs, k_cache[l], v_cache[l],
                                                                    merged, budget))
                cmp_ms += ms
                cmp_bytes += H * (merged * d * 2 + 4 * budget * d * 2 + 12 * merged + 4 * budget)
                if l == 0:
                    if keep_indices:
                        res.kept.append(kept.cpu().numpy())
                    if observer:
                        observer("commit", {"tick": tk, "q_obs": q_obs, "mass": mass, "kept": kept,
                                            "k_cache": k_cache[0], "v_cache": v_cache[0]})
    torch.cuda.synchronize()
    res.stats = {
        "ticks": sch.total_ticks, "decisions": n_dec, "recomputed": n_rec_total,
        "reuse_ratio": 1.0 - n_rec_total / max(n_dec, 1), "commits": n_commit,
        "decide_ms": dec_ms, "attention_ms": att_ms, "compress_ms": cmp_ms,
        "attention_TFLOPs": att_flops / 1e12,
        "attention_TFLOP_per_s": att_flops / max(att_ms, 1e-9) / 1e9,
        "compress_GB_per_s": cmp_bytes / max(cmp_ms, 1e-9) / 1e6,
        "path_ms": dec_ms + att_ms + cmp_ms, "wall_s": time.perf_counter() - t_wall,
    }
    return res


def _mass_and_compress(cfg, q_obs, k, v, merged, budget):
    mass = B.flowcache_attention_mass(q_obs, k, merged)
    # the caller synchronises right after this anyway (timing): check the compaction's status word
    kept = B.flowcache_kv_compress(k, v, merged, budget, mass, cfg.pool_k, cfg.lam, check_status=True)
    return mass, kept


def main() -> None:
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawTextHelpFormatter)
    ap.add_argument("--layers", type=int, default=4)
    ap.add_argument("--units", type=int, default=8)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--stagger", type=int, default=15)
    ap.add_argument("--budget-chunks", type=int, default=4)
    ap.add_argument("--L_c", type=int, default=10200)
    ap.add_argument("--eps", type=float, default=0.1)
    args = ap.parse_args()
    base = RolloutConfig(n_layers=args.layers, n_units=args.units, steps=args.steps,
                         stagger=args.stagger, budget_chunks=args.budget_chunks, L_c=args.L_c)
    out = {}
    for name, eps in (("eps0", 0.0), (f"eps{args.eps}", args.eps)):
        cfg = RolloutConfig(**{**base.__dict__, "eps": eps})

        def progress(event, info, name=name):
            if event == "decide" and info["tick"]["tick"] % 32 == 0:
                print(f"[{name}] tick {info['tick']['tick']}", file=sys.stderr, flush=True)

        out[name] = run_rollout(cfg, observer=progress).stats
    a, b = out["eps0"], out[f"eps{args.eps}"]
    out["path_speedup_vs_eps0"] = a["path_ms"] / max(b["path_ms"], 1e-9)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
