"""Seeded sweep of small random shapes through every entry point, against the oracle, to the
same bars as the fixed parity cases.  Shapes are drawn inside the documented limits (head
dimension 64 or 128, 1-16 active chunks, any chunk length, any clean length, grouped heads,
slots with gaps and in any physical order, ragged chunk sizes for the change metric); every
draw is reproducible from its case number."""
import numpy as np
import pytest
import torch

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import binding as B
from paper_2602_10825_amd import synth
from tests._checks import assert_mass_close
from tests.test_gpu_parity import DEV, check_attend, dev, run_attend, run_compress

pytestmark = pytest.mark.gpu


def draw_workload(case: int) -> synth.Workload:
    r = np.random.default_rng(1000 + case)
    dtype = "bf16" if r.random() < 0.7 else "f32"
    d = int(r.choice([64, 128]))
    H_k = int(r.integers(1, 4))
    G = int(r.choice([1, 1, 2, 4]))
    A = int(r.integers(1, 6))
    L_c = int(r.choice([1, 7, 31, 32, 33, 63, 64, 65, 100, 129, 200, 255, 256, 257, 300]))
    L_clean = int(r.choice([0, 1, 63, 64, 65, 130, 400]))
    return synth.Workload(f"sweep{case}", dtype, H_k * G, H_k, d, A, L_c, L_clean, 1)


@pytest.mark.parametrize("case", range(24))
def test_attend_and_mass_random_shapes(case):
    wl = draw_workload(case)
    r = np.random.default_rng(5000 + case)
    a = synth.attend_inputs(wl, seed=case)
    # slots: random physical order, random gaps (multiples of 8 tokens keep nothing special)
    gaps = r.integers(0, 3, wl.A) * 8
    order = r.permutation(wl.A)
    off = np.zeros(wl.A, np.int64)
    pos = wl.L_clean
    for c in order:
        pos += int(gaps[c])
        off[c] = pos
        pos += wl.L_c
    cap = pos + int(r.integers(0, 9))
    sd = a["k_cache"].dtype
    kc = np.zeros((wl.H_k, cap, wl.d), sd)
    vc = np.zeros_like(kc)
    kc[:, :wl.L_clean] = a["k_cache"][:, :wl.L_clean]
    vc[:, :wl.L_clean] = a["v_cache"][:, :wl.L_clean]
    old = wl.active_off()
    for c in range(wl.A):                      # the stale K/V of each chunk moves with its slot
        kc[:, off[c]:off[c] + wl.L_c] = a["k_cache"][:, old[c]:old[c] + wl.L_c]
        vc[:, off[c]:off[c] + wl.L_c] = a["v_cache"][:, old[c]:old[c] + wl.L_c]
    a["k_cache"], a["v_cache"], a["active_off"] = kc, vc, off.astype(np.int32)
    rec = [c for c in range(wl.A) if r.random() < 0.6]
    # the mass needs the last chunk in the last compact block and a non-empty prefix to score
    want_mass = bool(rec) and rec[-1] == wl.A - 1
    mass_len = 0
    W = int(r.choice([0, 1, 50, 64, 70]))
    if want_mass and wl.L_clean > 0:
        mass_len = int(r.integers(1, wl.L_clean + 1))
    got, ref, res, ref_lse, q_c, kc_ref = run_attend(wl, a, rec, mass_len=mass_len, obs_window=W)
    if rec:
        check_attend(wl, got, ref, res, ref_lse, len(rec))
    if mass_len:
        q_obs = O.observation_rows(q_c, len(rec), wl.L_c, W)
        ref_mass = O.attention_mass(q_obs, kc_ref, mass_len)
        assert_mass_close(res["mass"].cpu().numpy(), ref_mass, wl.dtype, wl.name)


@pytest.mark.parametrize("case", range(16))
def test_compress_random_shapes(case):
    r = np.random.default_rng(7000 + case)
    dtype = "bf16" if r.random() < 0.7 else "f32"
    d = int(r.choice([64, 128]))
    H_k = int(r.integers(1, 5))
    L_k = int(r.choice([2, 17, 64, 65, 255, 256, 257, 1000, 2048, 2049, 4100, 6000]))
    budget = int(r.integers(1, L_k + 1)) if r.random() < 0.9 else L_k + 5
    pool_k = int(r.choice([1, 3, 7, 15]))
    lam = float(r.choice([0.0, 0.07, 0.5, 1.0]))
    kind = str(r.choice(["normal", "clustered", "heavy_dup"]))
    wl = synth.Workload(f"csweep{case}", dtype, H_k, H_k, d, 1, 8, L_k, min(budget, L_k))
    c = synth.compress_inputs(wl, seed=case, kind=kind)
    run_compress(wl, c, L_k, budget, pool_k, lam)


@pytest.mark.parametrize("case", range(12))
def test_decide_and_residual_random_shapes(case):
    r = np.random.default_rng(9000 + case)
    dtype = "bf16" if r.random() < 0.6 else "f32"
    A = int(r.integers(1, 17))
    elems = int(r.choice([1, 5, 8, 1000, 1003, 4096, 4099, 20000, 65537]))
    m = int(r.integers(0, 5))
    eps = float(r.choice([0.0, 0.05, 0.2]))
    xp = r.standard_normal((A, elems)).astype(np.float32)
    sig = np.exp(r.uniform(np.log(1e-3), np.log(0.3), A)).astype(np.float32)
    xc = xp + sig[:, None] * r.standard_normal((A, elems)).astype(np.float32)
    if A > 2:
        xc[1] = xp[1]                                   # a chunk that did not change at all
    xp_s, xc_s = synth.to_storage(xp, dtype), synth.to_storage(xc, dtype)
    step = r.integers(0, 9, A).astype(np.int32)
    acc0 = (r.random(A) * eps).astype(np.float64)
    ref = O.chunk_decide(xc_s, xp_s, step, m, eps, acc0)
    if np.any((ref["margin"] <= 1e-9) & (ref["l1rel"] != 0)):
        pytest.skip("drawn decision sits on the threshold")
    acc = torch.from_numpy(acc0.copy()).to(DEV)
    xcd = dev(xc_s, dtype)
    out = B.flowcache_chunk_decide(xcd, dev(xp_s, dtype), torch.from_numpy(step).to(DEV), m, eps, acc)
    torch.cuda.synchronize()
    assert out["recompute_mask"].cpu().numpy().tolist() == ref["mask"].tolist()
    n = int(out["n_recompute"].item())
    idx = out["recompute_idx"].cpu().numpy()
    assert n == int(ref["n_recompute"]) and idx[:n].tolist() == ref["recompute_idx"].tolist()
    assert np.allclose(out["acc"].cpu().numpy(), ref["acc"], rtol=1e-12, atol=0)
    xcomp = B.to_host(out["x_compact"])
    assert np.array_equal(xcomp[:n], O.gather_chunks(xc_s, ref["recompute_idx"]))
    # the stack's output for the gathered chunks, then store / apply of the difference
    y = np.zeros_like(xcomp)                            # blocks past n are never read
    y[:n] = synth.to_storage(O.widen(xcomp[:n]) * 0.5 + 0.25, dtype)
    res0 = synth.to_storage(r.standard_normal((A, elems)).astype(np.float32), dtype)
    res_d = dev(res0, dtype)
    full = B.flowcache_residual_apply(xcd, dev(y, dtype), res_d, out["recompute_idx"], out["n_recompute"])
    ref_res, ref_full = O.residual_apply(xc_s, y, res0, ref["recompute_idx"])
    assert np.array_equal(B.to_host(full), ref_full) and np.array_equal(B.to_host(res_d), ref_res)
