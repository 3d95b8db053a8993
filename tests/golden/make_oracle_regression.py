"""Writes ``oracle_regression.json``: the oracle's own outputs on the tiny fp32 step.

Calls only ``oracle/`` (plus the seeded input generators).  Run from the repo root:
    python -m tests.golden.make_oracle_regression
"""
import json
import os

import numpy as np

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import synth


def compute():
    wl = synth.C1
    d = synth.decide_inputs(wl, seed=0)
    a = synth.attend_inputs(wl, seed=0)
    dec = O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, wl.eps, d["acc"])
    rec = [0, 1]
    kc = O.scatter_kv(a["k_cache"], a["k_new"], rec, a["active_off"], wl.L_c)
    vc = O.scatter_kv(a["v_cache"], a["v_new"], rec, a["active_off"], wl.L_c)
    out, lse = O.attend(a["q"], kc, vc, wl.L_clean, a["active_off"], wl.L_c, rec)
    q_obs = O.observation_rows(a["q"], 2, wl.L_c, wl.obs_window)
    mass = O.attention_mass(q_obs, kc, wl.L_k)
    kept, _, _, sc = O.kv_compress(kc, vc, wl.L_k, wl.budget, mass.astype(np.float32),
                                   wl.pool_k, wl.lam)
    return {
        "workload": wl.name, "seed": 0,
        "mask": dec["mask"].tolist(), "l1rel": dec["l1rel"].tolist(),
        "out_sample": out[[0, 127, 128, 255], :, :4].ravel().tolist(),
        "mass_sample": mass[0, :16].tolist(),
        "score_sample": sc[0, :16].tolist(),
        "kept_head0": kept[0].tolist(),
    }


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "oracle_regression.json")
    with open(path, "w") as f:
        json.dump(compute(), f)
    print("wrote", path)
