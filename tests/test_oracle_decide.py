"""Pins for the oracle's change metric and reuse policy (Eq. (5), (8)): hand-worked
numbers, closed forms and invariants.  CPU only."""
import json
import math
import os

import numpy as np
import pytest
import torch

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")))


def test_widen_bf16_matches_library_conversion():
    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    ref = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    got = O.widen(bits)
    ok = np.isfinite(ref)
    assert np.array_equal(got[ok], ref[ok])
    assert np.all(np.isnan(got[np.isnan(ref)]))


def test_bf16_rounding_of_generator_is_nearest_even():
    x = np.random.default_rng(0).standard_normal(100000).astype(np.float32)
    x[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-39]   # ties (both parities), subnormal
    bits = synth.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(bits, ref)


def test_relative_l1_hand_worked():
    g = GOLD["relative_l1"]
    xp, xc = np.array(g["x_prev"]), np.array(g["x_cur"])
    for i in range(2):
        assert O.relative_l1(xc[i], xp[i]) == g["l1rel"][i]
    # a swapped denominator (current instead of previous tick) must not give the same
    assert 3.0 / np.abs(xc[1]).sum() != g["l1rel"][1]


def test_policy_hand_worked_cases():
    g = GOLD["reuse_policy"]
    for c in g["cases"]:
        f, rec = O.reuse_policy(c["l1rel"], c["acc_old"], c["step_idx"], g["warmup_m"], g["eps"])
        assert f == c["f_new"], c["why"]
        assert rec == c["recompute"], c["why"]


def test_chunk_decide_combines_metric_and_policy():
    g = GOLD["relative_l1"]
    xp, xc = np.array(g["x_prev"]), np.array(g["x_cur"])
    out = O.chunk_decide(xc, xp, step_idx=[5, 5], warmup_m=2, eps=0.125, acc=[0.03125, 0.0])
    assert out["l1rel"].tolist() == g["l1rel"]
    assert out["mask"].tolist() == [0, 1]
    assert out["acc"].tolist() == [0.125, 0.0]
    assert out["recompute_idx"].tolist() == [1] and int(out["n_recompute"]) == 1
    assert out["margin"][0] == 0.0 and out["margin"][1] == pytest.approx(0.0625)


def test_zero_denominator_forces_recompute():
    z = np.zeros((1, 8))
    out = O.chunk_decide(z + 1.0, z, [9], 2, 0.5, [0.0])
    assert math.isinf(out["l1rel"][0]) and out["mask"][0] == 1 and out["acc"][0] == 0.0
    out = O.chunk_decide(z, z, [9], 2, 0.5, [0.0])          # 0/0
    assert out["mask"][0] == 1


@pytest.mark.parametrize("same", [False, True])
def test_eps_zero_recomputes_every_chunk(same):
    wl = synth.C1
    d = synth.decide_inputs(wl, seed=3)
    xc = d["x_prev"] if same else d["x_cur"]
    out = O.chunk_decide(xc, d["x_prev"], d["step_idx"], wl.warmup_m, 0.0, d["acc"])
    assert out["mask"].tolist() == [1] * wl.A
    assert out["acc"].tolist() == [0.0] * wl.A


def test_expected_relative_l1_equals_sigma():
    # x_cur = x_prev + sigma*n, iid normals: E|sigma n| / E|x_prev| = sigma (half-normal means)
    rng = np.random.default_rng(1)
    n = 1_000_000
    for sigma in (0.001, 0.05, 0.3):
        xp = rng.standard_normal(n)
        xc = xp + sigma * rng.standard_normal(n)
        assert O.relative_l1(xc, xp) == pytest.approx(sigma, rel=5e-3)


def test_c1_generator_gives_one_reuse_one_recompute():
    wl = synth.C1
    d = synth.decide_inputs(wl, seed=0)
    out = O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, wl.eps, d["acc"])
    assert out["mask"].tolist() == [0, 1]
    assert out["l1rel"][0] == pytest.approx(0.001, rel=0.05)
    assert out["l1rel"][1] == pytest.approx(0.1, rel=0.05)
    d = synth.decide_inputs(wl, seed=0, sigmas=[0.1, 0.001])
    out = O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, wl.eps, d["acc"])
    assert out["mask"].tolist() == [1, 0]


def test_constant_change_reuse_run_length_is_floor_eps_over_c():
    for eps, c in ((0.1, 0.03), (0.15, 0.04), (0.01, 0.003), (0.1, 0.2)):
        acc, runs, run = 0.0, [], 0
        for tick in range(200):
            acc, rec = O.reuse_policy(c, acc, step_idx=10, warmup_m=4, eps=eps)
            assert 0.0 <= acc <= eps
            if rec:
                runs.append(run)
                run = 0
            else:
                run += 1
        assert set(runs[1:]) == {math.floor(eps / c)}


def test_accumulator_invariants_on_random_trajectory():
    rng = np.random.default_rng(5)
    acc = 0.0
    for step in range(500):
        l1 = float(rng.exponential(0.02))
        new, rec = O.reuse_policy(l1, acc, step, warmup_m=5, eps=0.05)
        assert 0.0 <= new <= 0.05
        assert rec == (new == 0.0)
        if step < 5:
            assert rec and new == 0.0
        elif acc + l1 > 0.05:
            assert rec
        else:
            assert new == acc + l1
        acc = new


def test_uniform_policy_shares_one_decision_but_new_chunk_computes():
    xp = np.ones((3, 16))
    xc = xp.copy()
    xc[0] += 0.01
    xc[1] += 0.30
    out = O.uniform_decide(xc, xp, step_idx=[9, 9, 0], warmup_m=4, eps=0.2, acc_global=0.0)
    # pooled metric over the two old chunks = (0.16 + 4.8) / 32 = 0.155 <= 0.2: both reuse
    assert out["mask"].tolist() == [0, 0, 1]
    assert out["l1rel"] == pytest.approx(0.155)
    per = O.chunk_decide(xc, xp, [9, 9, 0], 4, 0.2, [0.0, 0.0, 0.0])
    assert per["mask"].tolist() == [0, 1, 1]                # chunkwise policy differs


def test_gather_is_a_bit_copy():
    x = synth.decide_inputs(synth.C1, seed=2)["x_cur"]
    g = O.gather_chunks(x, [1])
    assert g.shape == (1, x.shape[1]) and np.array_equal(g[0], x[1])
    assert O.gather_chunks(x, []).shape[0] == 0
