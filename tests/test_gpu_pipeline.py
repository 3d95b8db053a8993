"""The whole pipeline on a small synthetic rollout: scheduler -> decide/gather -> per layer
scatter + chunk-causal attention -> cached-activation store/apply -> commit (append, then
mass + compression once the budget is reached).  A host mirror built from the oracle follows
layer 0 through every tick: decisions and accumulators, cache contents after every scatter,
attention outputs, importance mass, kept indices and the compacted caches."""
import numpy as np
import pytest
import torch

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import binding as B
from paper_2602_10825_amd.rollout import RolloutConfig, run_rollout
from tests._checks import assert_mass_close

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


def small_config(eps):
    return RolloutConfig(H=2, d=64, L_c=96, n_layers=2, n_units=6, steps=8, stagger=4,
                         budget_chunks=2, warmup_m=2, eps=eps, obs_window=20, delta0=0.03,
                         decay=0.8, seed=3)


def make_observer(cfg, mirror, rows_per_chunk=None, heads=None):
    """Host mirror of layer 0.  ``rows_per_chunk`` / ``heads``: compare the attention output on
    a seeded sample of query rows of each recompute chunk (first and last row included) and on
    these heads only -- for shapes where the float64 oracle cannot do every row."""
    budget = cfg.budget_chunks * cfg.L_c
    rng = np.random.default_rng(cfg.seed)

    def observer(event, info):
        tk = info["tick"]
        mirror["events"].append(event)
        if event == "decide":
            ref = O.chunk_decide(B.to_host(info["x_cur"]), B.to_host(info["x_prev"]),
                                 np.array(tk["step_idx"], np.int32), cfg.warmup_m, cfg.eps,
                                 info["acc_before"].cpu().numpy())
            assert ref["margin"].min() > 1e-9
            assert info["dec"]["recompute_mask"].cpu().numpy().tolist() == ref["mask"].tolist(), tk["tick"]
            assert np.allclose(info["dec"]["acc"].cpu().numpy(), ref["acc"], rtol=1e-12, atol=0)
            mirror["rec"] = ref["recompute_idx"].tolist()
        elif event == "attend":
            if mirror["k"] is None:
                mirror["k"] = np.zeros(tuple(info["k_cache"].shape), np.uint16)
                mirror["v"] = np.zeros_like(mirror["k"])
            rec = mirror["rec"]
            assert rec == info["rec"]
            R = len(rec)
            q, kn, vn = (B.to_host(info[n])[:R * cfg.L_c] for n in ("q", "k_new", "v_new"))
            off = np.array(tk["active_off"], np.int32)
            mirror["k"] = O.scatter_kv(mirror["k"], kn, rec, off, cfg.L_c)
            mirror["v"] = O.scatter_kv(mirror["v"], vn, rec, off, cfg.L_c)
            assert np.array_equal(B.to_host(info["k_cache"]), mirror["k"]), tk["tick"]
            assert np.array_equal(B.to_host(info["v_cache"]), mirror["v"]), tk["tick"]
            got = O.widen(B.to_host(info["out"]))[:R * cfg.L_c]
            if rows_per_chunk is None:
                ref, _ = O.attend(q, mirror["k"], mirror["v"], tk["L_clean"], off, cfg.L_c, rec)
            else:
                rows = []
                for r in range(R):
                    pick = {0, cfg.L_c - 1} | set(rng.integers(0, cfg.L_c, rows_per_chunk).tolist())
                    rows += [r * cfg.L_c + x for x in sorted(pick)]
                hs = list(heads)
                ref, _ = O.attend(np.ascontiguousarray(q[:, hs]), mirror["k"][hs], mirror["v"][hs],
                                  tk["L_clean"], off, cfg.L_c, rec, rows=rows)
                got = got[rows][:, hs]
                mirror["attend_rows"] = mirror.get("attend_rows", 0) + len(rows)
            err = np.abs(got - ref)
            assert err.max() <= 2e-2 and np.sqrt((err ** 2).sum() / (ref ** 2).sum()) <= 1e-2, tk["tick"]
        elif event == "commit":
            src, dst, L_c = tk["commit_src_off"], tk["commit_dst_off"], cfg.L_c
            mirror["k"][:, dst:dst + L_c] = mirror["k"][:, src:src + L_c]
            mirror["v"][:, dst:dst + L_c] = mirror["v"][:, src:src + L_c]
            if tk["compress"]:
                merged = tk["merged_len"]
                m = info["mass"].cpu().numpy()
                ref_mass = O.attention_mass(B.to_host(info["q_obs"]), mirror["k"][:, :merged], merged)
                assert_mass_close(m, ref_mass, "bf16", f"tick {tk['tick']}")
                rk, mirror["k"], mirror["v"], _ = O.kv_compress(mirror["k"], mirror["v"], merged, budget,
                                                                m, cfg.pool_k, cfg.lam)
                assert np.array_equal(info["kept"].cpu().numpy(), rk), tk["tick"]
                mirror["compressions"] = mirror.get("compressions", 0) + 1
            L_after = tk["L_clean_after"]
            assert np.array_equal(B.to_host(info["k_cache"][:, :L_after]), mirror["k"][:, :L_after])
            assert np.array_equal(B.to_host(info["v_cache"][:, :L_after]), mirror["v"][:, :L_after])

    return observer


def test_rollout_matches_host_mirror():
    cfg = small_config(eps=0.08)
    mirror = {"k": None, "v": None, "acc": {}, "events": []}
    observer = make_observer(cfg, mirror)
    res = run_rollout(cfg, observer=observer, keep_indices=True)
    st = res.stats
    assert st["ticks"] == (cfg.n_units - 1) * cfg.stagger + cfg.steps == len(res.masks)
    assert st["commits"] == cfg.n_units and len(res.kept) == cfg.n_units - cfg.budget_chunks
    assert 0.0 < st["reuse_ratio"] < 1.0                       # chunks were skipped, and not all
    assert mirror["events"].count("commit") == cfg.n_units
    # a chunk in its first warmup_m steps is never skipped
    for mask, tk_units in zip(res.masks, res.units):
        assert len(mask) == len(tk_units)


def test_rollout_with_eps_zero_recomputes_everything_and_costs_more_attention():
    full = run_rollout(small_config(eps=0.0)).stats
    fast = run_rollout(small_config(eps=0.08)).stats
    assert full["reuse_ratio"] == 0.0 and full["recomputed"] == full["decisions"]
    assert fast["attention_TFLOPs"] < full["attention_TFLOPs"]
    assert fast["commits"] == full["commits"]


def test_rollout_at_the_skyreels_layer_shape_matches_host_mirror():
    """The multi-step sweep's layer shape (12 heads x 128, chunks of 10200 tokens), a few ticks
    of it: 3 chunks x 4 steps, window of 2, clean-cache budget of one chunk, so the second and
    third commits compress.  Decisions, every scatter, the importance mass, kept indices and the
    compacted caches are compared in full; the attention output on sampled rows and heads."""
    cfg = RolloutConfig(H=12, d=128, L_c=10200, n_layers=2, n_units=3, steps=4, stagger=2,
                        budget_chunks=1, warmup_m=1, eps=0.05, obs_window=50, delta0=0.03, decay=0.85,
                        seed=5)
    mirror = {"k": None, "v": None, "acc": {}, "events": []}
    res = run_rollout(cfg, observer=make_observer(cfg, mirror, rows_per_chunk=12, heads=(0, 5, 11)),
                      keep_indices=True)
    st = res.stats
    assert st["ticks"] == (cfg.n_units - 1) * cfg.stagger + cfg.steps == 8
    assert st["commits"] == 3 and mirror["compressions"] == 2 and len(res.kept) == 2
    assert 0.0 < st["reuse_ratio"] < 1.0 and mirror["attend_rows"] >= 60
    print(f"C2-shape rollout: {st['ticks']} ticks, reuse ratio {st['reuse_ratio']:.2f}, "
          f"{mirror['attend_rows']} attention rows checked", flush=True)
