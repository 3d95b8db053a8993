"""Parity of the HIP path (through the C ABI) with the fp64 oracle, element by element on
the same seeded inputs.  Bars: decisions and kept indices bit-exact; attention within
1e-5 relative (fp32) / 2e-2 max-abs (bf16, plus 1e-2 relative Frobenius)."""
import numpy as np
import pytest
import torch

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import binding as B
from paper_2602_10825_amd import synth
from tests._checks import assert_mass_close

pytestmark = pytest.mark.gpu
DEV = "cuda"


def dev(arr, dtype):
    return B.to_device(arr, dtype, DEV)


# ------------------------------------------------------------------ decide + gather
def run_decide(wl, d, eps=None, warmup_m=None, gather=True):
    xc, xp = dev(d["x_cur"], wl.dtype), dev(d["x_prev"], wl.dtype)
    acc = torch.from_numpy(d["acc"].copy()).to(DEV)
    step = torch.from_numpy(d["step_idx"]).to(DEV)
    eps = wl.eps if eps is None else eps
    m = wl.warmup_m if warmup_m is None else warmup_m
    out = B.flowcache_chunk_decide(xc, xp, step, m, eps, acc, gather=gather)
    torch.cuda.synchronize()
    ref = O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], m, eps, d["acc"])
    return out, ref


def check_decide(wl, d, out, ref):
    assert ref["margin"].min() > 1e-9, "generator produced a knife-edge decision"
    assert out["recompute_mask"].cpu().numpy().tolist() == ref["mask"].tolist()
    n = int(out["n_recompute"].item())
    assert n == int(ref["n_recompute"])
    idx = out["recompute_idx"].cpu().numpy()
    assert idx[:n].tolist() == ref["recompute_idx"].tolist() and np.all(idx[n:] == -1)
    got_l1 = out["l1rel"].cpu().numpy()
    assert np.allclose(got_l1, ref["l1rel"], rtol=1e-12, atol=0)
    assert np.allclose(out["acc"].cpu().numpy(), ref["acc"], rtol=1e-12, atol=0)
    if out["x_compact"] is not None and n:
        xc = B.to_host(out["x_compact"])
        assert np.array_equal(xc[:n], O.gather_chunks(d["x_cur"], ref["recompute_idx"]))


@pytest.mark.parametrize("wl,sig", [(synth.C1, None), (synth.C1, [0.1, 0.001]),
                                    (synth.MID_BF16, [0.003, 0.5, 0.02]),
                                    (synth.MID_F32, [0.2, 0.001, 0.04])])
def test_decide_matches_oracle(wl, sig):
    d = synth.decide_inputs(wl, seed=0, sigmas=sig)
    out, ref = run_decide(wl, d)
    check_decide(wl, d, out, ref)
    assert 0 < int(ref["n_recompute"]) < wl.A          # mixed reuse / recompute


def test_decide_eps_zero_warmup_and_zero_denominator():
    wl = synth.C1
    d = synth.decide_inputs(wl, seed=1)
    out, ref = run_decide(wl, d, eps=0.0)
    assert out["recompute_mask"].cpu().tolist() == [1, 1] == ref["mask"].tolist()
    d2 = synth.decide_inputs(wl, seed=1, sigmas=[1e-4, 1e-4], step_idx=[1, 9])
    out, ref = run_decide(wl, d2)
    check_decide(wl, d2, out, ref)
    assert ref["mask"].tolist() == [1, 0]                 # warm-up chunk computes
    d3 = synth.decide_inputs(wl, seed=1)
    d3["x_prev"][0] = 0
    out, ref = run_decide(wl, d3)
    assert np.isinf(out["l1rel"].cpu().numpy()[0]) and out["recompute_mask"].cpu().tolist()[0] == 1
    d3["x_cur"][0] = 0                                     # 0/0
    out, ref = run_decide(wl, d3)
    assert out["recompute_mask"].cpu().tolist()[0] == 1 == ref["mask"][0]


@pytest.mark.parametrize("dtype,elems", [("bf16", 1003), ("f32", 4099), ("bf16", 8 * 3000 + 8),
                                         ("f32", 7), ("bf16", 1)])
def test_decide_ragged_and_unaligned_chunks(dtype, elems):
    wl = synth.Workload("t", dtype, 1, 1, elems, 3, 1, 0, 1, warmup_m=2, eps=0.05)
    d = synth.decide_inputs(wl, seed=2, sigmas=[0.001, 0.2, 0.01])
    out, ref = run_decide(wl, d)
    check_decide(wl, d, out, ref)


def test_decide_accumulates_over_ticks_like_the_oracle():
    wl = synth.Workload("t", "bf16", 2, 2, 64, 4, 96, 0, 1, warmup_m=2, eps=0.1)
    rng = np.random.default_rng(0)
    acc_ref = np.zeros(wl.A)
    acc_gpu = torch.zeros(wl.A, dtype=torch.float64, device=DEV)
    x_prev = synth.to_storage(rng.standard_normal((wl.A, wl.chunk_elems)).astype(np.float32), "bf16")
    masks = []
    for tick in range(12):
        sig = np.array([0.03, 0.012, 0.06, 0.2])
        x_cur = synth.to_storage((O.widen(x_prev) + sig[:, None] * rng.standard_normal(x_prev.shape)
                                  ).astype(np.float32), "bf16")
        step = np.array([tick, tick + 1, tick, max(0, tick - 3)], dtype=np.int32)
        ref = O.chunk_decide(x_cur, x_prev, step, wl.warmup_m, wl.eps, acc_ref)
        out = B.flowcache_chunk_decide(dev(x_cur, "bf16"), dev(x_prev, "bf16"),
                                       torch.from_numpy(step).to(DEV), wl.warmup_m, wl.eps, acc_gpu)
        assert out["recompute_mask"].cpu().numpy().tolist() == ref["mask"].tolist(), tick
        assert np.allclose(acc_gpu.cpu().numpy(), ref["acc"], rtol=1e-12)
        acc_ref = ref["acc"]
        masks.append(ref["mask"].tolist())
        x_prev = x_cur
    assert any(0 in m for m in masks) and any(m.count(1) > 1 for m in masks)


# ------------------------------------------------------------------ attention
def run_attend(wl, a, rec, mass_len=0, obs_window=50, scale=0.0):
    A = wl.A
    q_all = a["q"].reshape(A, wl.L_c, wl.H_q, wl.d)
    kn_all = a["k_new"].reshape(A, wl.L_c, wl.H_k, wl.d)
    vn_all = a["v_new"].reshape(A, wl.L_c, wl.H_k, wl.d)
    R = len(rec)
    pad = [0] * (A - R)
    order = list(rec) + pad
    q_c = np.concatenate([q_all[c] for c in order]).reshape(A * wl.L_c, wl.H_q, wl.d)
    kn_c = np.concatenate([kn_all[c] for c in order]).reshape(A * wl.L_c, wl.H_k, wl.d)
    vn_c = np.concatenate([vn_all[c] for c in order]).reshape(A * wl.L_c, wl.H_k, wl.d)
    idx = torch.tensor(list(rec) + [-1] * (A - R), dtype=torch.int32, device=DEV)
    n = torch.tensor([R], dtype=torch.int32, device=DEV)
    kc, vc = dev(a["k_cache"], wl.dtype), dev(a["v_cache"], wl.dtype)
    qd = dev(q_c, wl.dtype)
    out0 = torch.full_like(qd, 7.0)
    res = B.flowcache_attend(qd, dev(kn_c, wl.dtype), dev(vn_c, wl.dtype), kc, vc, wl.L_c,
                             wl.L_clean, a["active_off"], idx, n, softmax_scale=scale, out=out0,
                             mass_len=mass_len, obs_window=obs_window)
    torch.cuda.synchronize()
    # oracle on the same bits
    kc_ref = O.scatter_kv(a["k_cache"], kn_c[:R * wl.L_c], rec, a["active_off"], wl.L_c)
    vc_ref = O.scatter_kv(a["v_cache"], vn_c[:R * wl.L_c], rec, a["active_off"], wl.L_c)
    assert np.array_equal(B.to_host(kc), kc_ref) and np.array_equal(B.to_host(vc), vc_ref)
    ref_out, ref_lse = O.attend(q_c[:R * wl.L_c], kc_ref, vc_ref, wl.L_clean, a["active_off"], wl.L_c,
                                rec, scale=(scale if scale > 0 else None))
    got = O.widen(B.to_host(res["out"]))
    assert np.all(got[R * wl.L_c:] == 7.0)               # rows of non-recomputed blocks untouched
    return got[:R * wl.L_c], ref_out, res, ref_lse, q_c, kc_ref


def check_attend(wl, got, ref, res, ref_lse, R):
    err = np.abs(got - ref)
    if wl.dtype == "f32":
        assert err.max() / np.abs(ref).max() <= 1e-5
        row = np.sqrt((err ** 2).sum(-1)) / np.sqrt((ref ** 2).sum(-1))
        assert row.max() <= 1e-5
        lse_tol = 1e-5
    else:
        assert err.max() <= 2e-2
        assert np.sqrt((err ** 2).sum()) / np.sqrt((ref ** 2).sum()) <= 1e-2
        lse_tol = 2e-2
    lse = res["lse"].cpu().numpy()[:, :R * wl.L_c]
    assert np.abs(lse - ref_lse).max() <= lse_tol


@pytest.mark.parametrize("wl,rec", [
    (synth.C1, [0, 1]), (synth.C1, [1]), (synth.C1_MHA, [0, 1]), (synth.C1_MHA, [0]),
    (synth.MID_F32, [0, 1, 2]), (synth.MID_F32, [0, 2]), (synth.MID_F32_D128, [1, 2]),
    (synth.MID_BF16, [0, 1, 2]), (synth.MID_BF16, [2]), (synth.MID_BF16, [0, 2]),
    (synth.MID_BF16_GQA, [0, 1, 2]), (synth.MID_BF16_GQA, [1]),
])
def test_attend_matches_oracle(wl, rec):
    a = synth.attend_inputs(wl, seed=0)
    got, ref, res, ref_lse, _, _ = run_attend(wl, a, rec)
    check_attend(wl, got, ref, res, ref_lse, len(rec))


def test_attend_bf16_d64_and_noncontiguous_slots_and_scale():
    wl = synth.Workload("t", "bf16", 4, 2, 64, 3, 150, 333, 100)
    a = synth.attend_inputs(wl, seed=3)
    got, ref, res, ref_lse, _, _ = run_attend(wl, a, [0, 1, 2], scale=0.2)
    check_attend(wl, got, ref, res, ref_lse, 3)
    # slots in a different physical order with gaps: capacity grows, offsets permuted
    wl2 = synth.Workload("t2", "bf16", 2, 2, 128, 3, 70, 100, 50)
    a2 = synth.attend_inputs(wl2, seed=4)
    cap = wl2.capacity + 200
    kc = np.zeros((wl2.H_k, cap, wl2.d), np.uint16); vc = np.zeros_like(kc)
    kc[:, :wl2.capacity] = a2["k_cache"]; vc[:, :wl2.capacity] = a2["v_cache"]
    a2["k_cache"], a2["v_cache"] = kc, vc
    a2["active_off"] = np.array([wl2.L_clean + 160, wl2.L_clean + 8, wl2.L_clean + 240], np.int32)
    got, ref, res, ref_lse, _, _ = run_attend(wl2, a2, [0, 1, 2])
    check_attend(wl2, got, ref, res, ref_lse, 3)


def test_attend_no_clean_context_and_nothing_to_recompute():
    wl = synth.Workload("t", "f32", 2, 2, 64, 2, 90, 0, 1)
    a = synth.attend_inputs(wl, seed=5)
    got, ref, res, ref_lse, _, _ = run_attend(wl, a, [0, 1])
    check_attend(wl, got, ref, res, ref_lse, 2)
    wlb = synth.Workload("t", "bf16", 2, 2, 128, 2, 90, 0, 1)
    ab = synth.attend_inputs(wlb, seed=5)
    got, ref, res, ref_lse, _, _ = run_attend(wlb, ab, [0, 1])
    check_attend(wlb, got, ref, res, ref_lse, 2)
    got, ref, res, _, _, _ = run_attend(wlb, ab, [])      # R = 0: no row written, cache untouched
    assert got.shape[0] == 0


@pytest.mark.parametrize("wl", [synth.MID_BF16, synth.MID_F32])
def test_malformed_recompute_list_is_skipped_not_followed(wl):
    """A count above A is cut to A and entries outside [0, A) are skipped by the kernels' own
    checks: the valid entry gives the bits of the well-formed call, nothing else is touched."""
    a = synth.attend_inputs(wl, seed=11)
    n_rows = wl.A * wl.L_c
    tdt = torch.bfloat16 if wl.dtype == "bf16" else torch.float32
    gen = torch.Generator(device=DEV)
    gen.manual_seed(0)

    def randn(*shape):
        return torch.randn(shape, device=DEV, generator=gen).to(tdt)

    q, kn, vn = randn(n_rows, wl.H_q, wl.d), randn(n_rows, wl.H_k, wl.d), randn(n_rows, wl.H_k, wl.d)
    outs = []
    for lst, cnt in (([1, -1, -1], 1), ([1, 99, -3], 9)):
        kc, vc = dev(a["k_cache"], wl.dtype), dev(a["v_cache"], wl.dtype)
        out0 = torch.full_like(q, 7.0)
        idx = torch.tensor(lst, dtype=torch.int32, device=DEV)
        n = torch.tensor([cnt], dtype=torch.int32, device=DEV)
        B.flowcache_attend(q, kn, vn, kc, vc, wl.L_c, wl.L_clean, a["active_off"], idx, n, out=out0,
                           want_lse=False)
        x = randn(wl.A, 1000) if not outs else outs[0][3]
        y = randn(wl.A, 1000) if not outs else outs[0][4]
        res = torch.ones_like(x)
        full = B.flowcache_residual_apply(x, y, res, idx, n)
        torch.cuda.synchronize()
        outs.append((B.to_host(out0), B.to_host(kc), B.to_host(vc), x, y, B.to_host(res), B.to_host(full)))
    good, bad = outs
    for i in (0, 1, 2, 5, 6):
        assert np.array_equal(good[i], bad[i])
    assert np.all(O.widen(bad[0])[wl.L_c:] == 7.0)
    # no y_compact: the list is not consulted, every chunk is reused
    x, res = good[3], torch.ones_like(good[3])
    idx = torch.tensor([1, 0, 2], dtype=torch.int32, device=DEV)
    n = torch.tensor([2], dtype=torch.int32, device=DEV)
    full = B.flowcache_residual_apply(x, None, res, idx, n)
    ref_res, ref_full = O.residual_apply(B.to_host(x), None, B.to_host(res), [])
    assert np.array_equal(B.to_host(full), ref_full) and np.array_equal(B.to_host(res), ref_res)


@pytest.mark.parametrize("dtype,d,A,L_c,L_clean", [
    ("bf16", 128, 1, 1, 0), ("bf16", 128, 2, 1, 1), ("bf16", 64, 3, 33, 63), ("bf16", 128, 2, 257, 64),
    ("bf16", 128, 1, 64, 65), ("bf16", 128, 4, 31, 0), ("f32", 64, 2, 1, 1), ("f32", 128, 1, 65, 0),
    ("bf16", 128, 16, 20, 30), ("f32", 64, 16, 9, 0),      # the largest window the ABI allows
])
def test_attend_edge_sizes(dtype, d, A, L_c, L_clean):
    """One-row chunks, chunks and clean regions one short of / equal to / one past a 64-key tile
    and a 256-row block, no clean context."""
    wl = synth.Workload("edge", dtype, 2, 2, d, A, L_c, L_clean, max(1, L_clean // 2))
    a = synth.attend_inputs(wl, seed=8)
    rec = list(range(A))
    got, ref, res, ref_lse, _, _ = run_attend(wl, a, rec)
    check_attend(wl, got, ref, res, ref_lse, A)


def test_attend_bf16_when_later_keys_dwarf_earlier_ones():
    """Key magnitudes grow along the cache, so the scores of later tiles exceed the exponent
    reference of the earlier ones by far more than 2^40: the kernel has to raise its reference
    (rescale its running output and row sums) several times, in the clean region and again in
    the active chunks."""
    wl = synth.MID_BF16
    a = synth.attend_inputs(wl, seed=6)
    ramp = np.linspace(0.05, 30.0, wl.capacity)[None, :, None]
    a["k_cache"] = synth.to_storage((O.widen(a["k_cache"]) * ramp).astype(np.float32), "bf16")
    kn = O.widen(a["k_new"]).reshape(wl.A, wl.L_c, wl.H_k, wl.d)
    grow = np.linspace(20.0, 60.0, wl.A * wl.L_c).reshape(wl.A, wl.L_c, 1, 1)
    a["k_new"] = synth.to_storage((kn * grow).astype(np.float32).reshape(-1, wl.H_k, wl.d), "bf16")
    got, ref, res, ref_lse, _, _ = run_attend(wl, a, [0, 1, 2])
    err = np.abs(got - ref)
    # outputs are O(1) here (a few keys dominate each row): relative bars
    assert np.sqrt((err ** 2).sum()) / np.sqrt((ref ** 2).sum()) <= 1e-2
    assert err.max() <= 2e-2 * max(1.0, np.abs(ref).max())
    lse = res["lse"].cpu().numpy()[:, :3 * wl.L_c]
    assert np.abs(lse - ref_lse).max() <= 2e-2 * np.abs(ref_lse).max()


# ------------------------------------------------------------------ importance mass
@pytest.mark.parametrize("wl,W", [(synth.C1, 50), (synth.C1_MHA, 50), (synth.MID_BF16, 50),
                                  (synth.MID_BF16_GQA, 0), (synth.MID_F32, 100)])
def test_mass_matches_oracle(wl, W):
    a = synth.attend_inputs(wl, seed=0)
    rec = list(range(wl.A))
    mass_len = wl.L_clean + wl.L_c                        # clean region + the finished chunk
    got, ref, res, _, q_c, kc_ref = run_attend(wl, a, rec, mass_len=mass_len, obs_window=W)
    q_obs = O.observation_rows(q_c, len(rec), wl.L_c, W)
    ref_mass = O.attention_mass(q_obs, kc_ref, mass_len)
    assert_mass_close(res["mass"].cpu().numpy(), ref_mass, wl.dtype, wl.name)
    # the standalone entry point gives the same bits for the same rows
    m2 = B.flowcache_attention_mass(dev(np.ascontiguousarray(q_obs), wl.dtype),
                                    dev(kc_ref, wl.dtype), mass_len)
    assert torch.equal(m2, res["mass"])


@pytest.mark.parametrize("dtype,d,H_q,H_k,W,mass_len", [
    ("bf16", 128, 2, 2, 1, 1), ("bf16", 128, 2, 1, 3, 31), ("bf16", 64, 4, 2, 64, 129),
    ("bf16", 128, 2, 2, 65, 1025), ("bf16", 128, 1, 1, 130, 2049), ("f32", 64, 2, 2, 5, 257),
])
def test_standalone_mass_edge_sizes(dtype, d, H_q, H_k, W, mass_len):
    """One key, fewer keys than a tile, one key past a tile / a block span; one row, 65 and 130
    rows (two and three row groups); grouped heads."""
    rng = np.random.default_rng(mass_len)
    q = synth.to_storage(rng.standard_normal((W, H_q, d)).astype(np.float32), dtype)
    k = synth.to_storage(rng.standard_normal((H_k, mass_len + 7, d)).astype(np.float32), dtype)
    got = B.flowcache_attention_mass(dev(q, dtype), dev(k, dtype), mass_len).cpu().numpy().astype(np.float64)
    ref = O.attention_mass(q, k, mass_len)
    assert_mass_close(got, ref, dtype, f"W={W} L={mass_len}")


def test_mass_is_nan_when_last_chunk_is_not_recomputed():
    wl = synth.C1
    a = synth.attend_inputs(wl, seed=0)
    _, _, res, _, _, _ = run_attend(wl, a, [0], mass_len=wl.L_clean)
    assert torch.isnan(res["mass"]).all()


# ------------------------------------------------------------------ compression
def run_compress(wl, c, L_k, budget, pool_k=7, lam=0.07):
    k, v = dev(c["k"], wl.dtype), dev(c["v"], wl.dtype)
    mass = torch.from_numpy(c["mass"][:, :L_k].copy()).to(DEV)
    kept = B.flowcache_kv_compress(k, v, L_k, budget, mass, pool_k, lam)
    torch.cuda.synchronize()
    rk, rk_k, rk_v, sc = O.kv_compress(c["k"], c["v"], L_k, budget, c["mass"][:, :L_k], pool_k, lam)
    gaps = [O.boundary_gap(sc[h], budget) for h in range(wl.H_k)]
    assert all(g == 0.0 or g > 1e-12 for g in gaps), f"ambiguous boundary {gaps}"
    assert np.array_equal(kept.cpu().numpy(), rk)
    assert np.array_equal(B.to_host(k), rk_k) and np.array_equal(B.to_host(v), rk_v)
    return kept, rk


@pytest.mark.parametrize("wl,kind", [(synth.C1, "normal"), (synth.C1_MHA, "clustered"),
                                     (synth.MID_BF16, "normal"), (synth.MID_BF16, "clustered"),
                                     (synth.MID_BF16, "heavy_dup"), (synth.MID_F32, "heavy_dup"),
                                     (synth.MID_F32_D128, "clustered"), (synth.MID_BF16_GQA, "normal")])
def test_compress_matches_oracle(wl, kind):
    c = synth.compress_inputs(wl, seed=0, kind=kind)
    run_compress(wl, c, wl.L_k, wl.budget)


@pytest.mark.parametrize("pool_k,lam,budget", [(1, 1.0, 100), (7, 0.0, 100), (15, 0.5, 1),
                                               (3, 0.07, 999), (7, 0.07, 1000), (7, 0.07, 5000)])
def test_compress_parameter_corners(pool_k, lam, budget):
    wl = synth.MID_BF16
    c = synth.compress_inputs(wl, seed=1, kind="clustered")
    kept, rk = run_compress(wl, c, wl.L_k, budget, pool_k, lam)
    if budget >= wl.L_k:
        assert kept.shape[1] == wl.L_k and np.array_equal(rk[0], np.arange(wl.L_k))


def test_compress_exact_ties_and_bf16_d64():
    # duplicated keys + mass plateaus give exactly equal scores: lower position must win
    wl = synth.Workload("t", "bf16", 2, 2, 64, 1, 8, 600, 300)
    c = synth.compress_inputs(wl, seed=2)
    c["k"][:, 300:600] = c["k"][:, 0:300]
    c["mass"][:] = np.float32(1.0 / 600)
    kept, rk = run_compress(wl, c, 600, 300)
    sc = O.selection_scores(c["k"][0], c["mass"][0], 7, 0.07)
    assert np.array_equal(sc[:300], sc[300:])             # the ties are real
    wl2 = synth.Workload("t", "f32", 1, 1, 64, 1, 8, 64, 32)
    c2 = synth.compress_inputs(wl2, seed=3)
    c2["k"][:] = c2["k"][:, :1]
    c2["mass"][:] = np.float32(0.5)
    kept, rk = run_compress(wl2, c2, 64, 32)
    assert kept.cpu().numpy()[0].tolist() == list(range(32))


@pytest.mark.parametrize("wl", [synth.MID_BF16,
                                synth.Workload("long", "bf16", 2, 2, 128, 1, 8, 9000, 4000)])   # > 4096 keys in a bin
def test_compress_with_infinite_importance_entries(wl):
    """Importance values that are not finite switch the first selection digit from the score
    bounds to the full key range (the bounds would not hold).  The oracle takes finite scores
    only, so it gets 1e30 where the kernel gets +inf: either way these tokens (and their pool
    windows, Eq. (10)) outrank everything else, and the rest of the selection is the same."""
    c = synth.compress_inputs(wl, seed=21, kind="clustered")
    where = [(0, 3), (0, 500), (0, 999), (1, 64), (1, 65)]
    huge = c["mass"].copy()
    for h, j in where:
        c["mass"][h, j] = np.inf
        huge[h, j] = np.float32(1e30)
    k, v = dev(c["k"], wl.dtype), dev(c["v"], wl.dtype)
    mass = torch.from_numpy(c["mass"][:, :wl.L_k].copy()).to(DEV)
    kept = B.flowcache_kv_compress(k, v, wl.L_k, wl.budget, mass, 7, 0.07, check_status=True)
    torch.cuda.synchronize()
    rk, rk_k, rk_v, sc = O.kv_compress(c["k"], c["v"], wl.L_k, wl.budget, huge[:, :wl.L_k], 7, 0.07)
    assert all(O.boundary_gap(sc[h], wl.budget) > 1e-12 for h in range(wl.H_k))
    got = kept.cpu().numpy()
    assert np.array_equal(got, rk)
    assert np.array_equal(B.to_host(k), rk_k) and np.array_equal(B.to_host(v), rk_v)
    for h, j in where:
        for jj in range(max(0, j - 3), min(wl.L_k, j + 4)):
            assert jj in got[h]


def test_compress_status_word_is_clear_after_normal_calls():
    wl = synth.MID_BF16
    c = synth.compress_inputs(wl, seed=9)
    k, v = dev(c["k"], wl.dtype), dev(c["v"], wl.dtype)
    mass = torch.from_numpy(c["mass"][:, :wl.L_k].copy()).to(DEV)
    L = B.lib()
    ws = torch.full((L.flowcache_kv_compress_workspace(wl.H_k, wl.L_k, wl.d, wl.budget, B.FC_BF16),), 0xFF,
                    dtype=torch.uint8, device=DEV)           # the call must reset the word itself
    B.flowcache_kv_compress(k, v, wl.L_k, wl.budget, mass, workspace=ws)
    assert B.kv_compress_status(ws, wl.H_k, wl.L_k, wl.d, wl.budget, B.FC_BF16) == 0
    k, v = dev(c["k"], wl.dtype), dev(c["v"], wl.dtype)
    ws = torch.full((L.flowcache_kv_compress_grouped_workspace(wl.H_k, wl.L_k, wl.d, 500, 50, B.FC_BF16),),
                    0xFF, dtype=torch.uint8, device=DEV)
    B.flowcache_kv_compress_grouped(k, v, wl.L_k, 500, 50, mass, workspace=ws)
    assert B.kv_compress_status(ws, wl.H_k, wl.L_k, wl.d, 500, B.FC_BF16, group=50) == 0
    with pytest.raises(B.FlowCacheError):
        B.kv_compress_status(ws, wl.H_k, wl.L_k, wl.d, 510, B.FC_BF16, group=50)


@pytest.mark.parametrize("wl,kind,budget", [(synth.MID_BF16, "heavy_dup", 500), (synth.MID_F32, "clustered", 333),
                                            (synth.MID_BF16, "normal", 5000)])
def test_select_then_compact_equals_compress(wl, kind, budget):
    """The two halves as calls of their own: K untouched by the selection, then the same kept
    list and the same cache bits as the one-call form and as the oracle."""
    c = synth.compress_inputs(wl, seed=12, kind=kind)
    L_k = wl.L_k
    mass = torch.from_numpy(c["mass"][:, :L_k].copy()).to(DEV)
    k, v = dev(c["k"], wl.dtype), dev(c["v"], wl.dtype)
    kept = B.flowcache_kv_select(k, L_k, budget, mass, 7, 0.07)
    torch.cuda.synchronize()
    assert np.array_equal(B.to_host(k), c["k"])                       # selection only reads K
    ws = torch.full((B.lib().flowcache_kv_compress_workspace(wl.H_k, L_k, wl.d, budget,
                                                              B.FC_BF16 if wl.dtype == "bf16" else B.FC_F32),),
                    0xFF, dtype=torch.uint8, device=DEV)              # a workspace the selection never saw
    B.flowcache_kv_compact(k, v, L_k, budget, kept, workspace=ws)
    torch.cuda.synchronize()
    rk, rk_k, rk_v, _ = O.kv_compress(c["k"], c["v"], L_k, budget, c["mass"][:, :L_k], 7, 0.07)
    assert np.array_equal(kept.cpu().numpy(), rk)
    assert np.array_equal(B.to_host(k), rk_k) and np.array_equal(B.to_host(v), rk_v)
    if budget < L_k:
        assert B.kv_compress_status(ws, wl.H_k, L_k, wl.d, budget,
                                    B.FC_BF16 if wl.dtype == "bf16" else B.FC_F32) == 0
    k2, v2 = dev(c["k"], wl.dtype), dev(c["v"], wl.dtype)
    kept2 = B.flowcache_kv_compress(k2, v2, L_k, budget, mass, 7, 0.07)
    assert torch.equal(kept2, kept) and torch.equal(k2, k) and torch.equal(v2, v)


def test_compress_on_strided_cache_prefix_leaves_the_rest_untouched():
    wl = synth.MID_BF16
    c = synth.compress_inputs(wl, seed=4)
    cap = wl.L_k + 77
    kfull = np.random.default_rng(0).integers(0, 2 ** 15, (wl.H_k, cap, wl.d)).astype(np.uint16)
    vfull = kfull[::-1].copy()
    kfull[:, :wl.L_k] = c["k"]; vfull[:, :wl.L_k] = c["v"]
    run_compress(wl, {"k": kfull, "v": vfull, "mass": c["mass"]}, wl.L_k, wl.budget)


@pytest.mark.parametrize("wl,group,budget_groups,kind", [
    (synth.MID_BF16, 50, 8, "normal"),            # 1000 tokens = 20 "frames" of 50
    (synth.MID_BF16, 250, 2, "clustered"),        # 4 "chunks" of 250
    (synth.MID_BF16, 8, 60, "heavy_dup"),
    (synth.MID_F32, 70, 4, "normal"),             # 700 tokens, d = 64
    (synth.MID_BF16, 1, 500, "normal"),           # group 1 = token granularity
    (synth.MID_BF16, 50, 20, "normal"),           # budget covers everything: identity
])
def test_grouped_compress_matches_oracle(wl, group, budget_groups, kind):
    c = synth.compress_inputs(wl, seed=7, kind=kind)
    L_k, budget = wl.L_k, group * budget_groups
    k, v = dev(c["k"], wl.dtype), dev(c["v"], wl.dtype)
    mass = torch.from_numpy(c["mass"][:, :L_k].copy()).to(DEV)
    kept = B.flowcache_kv_compress_grouped(k, v, L_k, budget, group, mass, 3, 0.3)
    torch.cuda.synchronize()
    rk, rk_k, rk_v, sc = O.kv_compress_grouped(c["k"], c["v"], L_k, budget, group, c["mass"][:, :L_k], 3, 0.3)
    if sc is not None:
        gaps = [O.boundary_gap(sc[h], budget_groups) for h in range(wl.H_k)]
        assert all(g == 0.0 or g > 1e-12 for g in gaps), f"ambiguous boundary {gaps}"
    assert np.array_equal(kept.cpu().numpy(), rk)
    assert np.array_equal(B.to_host(k), rk_k) and np.array_equal(B.to_host(v), rk_v)


# ------------------------------------------------------------------ the whole step, chained
@pytest.mark.parametrize("wl,eps", [(synth.C1, None), (synth.C1, 0.0), (synth.MID_BF16, 0.0)])
def test_full_step_chain(wl, eps):
    d = synth.decide_inputs(wl, seed=0)
    a = synth.attend_inputs(wl, seed=0)
    eps = wl.eps if eps is None else eps
    # force the last chunk into warm-up so it is recomputed and can serve as observation rows
    d["step_idx"][-1] = 0
    xc, xp = dev(d["x_cur"], wl.dtype), dev(d["x_prev"], wl.dtype)
    acc = torch.zeros(wl.A, dtype=torch.float64, device=DEV)
    dec = B.flowcache_chunk_decide(xc, xp, torch.from_numpy(d["step_idx"]).to(DEV), wl.warmup_m, eps,
                                   acc, gather=False)
    ref = O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, eps, d["acc"])
    rec = ref["recompute_idx"].tolist()
    assert dec["recompute_mask"].cpu().tolist() == ref["mask"].tolist()
    if eps == 0.0:
        assert rec == list(range(wl.A))
    A, R = wl.A, len(rec)
    order = rec + [0] * (A - R)
    pick = lambda arr, H: np.concatenate([arr.reshape(A, wl.L_c, H, wl.d)[c] for c in order])
    q_c, kn_c, vn_c = pick(a["q"], wl.H_q), pick(a["k_new"], wl.H_k), pick(a["v_new"], wl.H_k)
    kc, vc = dev(a["k_cache"], wl.dtype), dev(a["v_cache"], wl.dtype)
    mass_len = wl.L_clean + wl.L_c
    res = B.flowcache_attend(dev(q_c, wl.dtype), dev(kn_c, wl.dtype), dev(vn_c, wl.dtype), kc, vc,
                             wl.L_c, wl.L_clean, a["active_off"], dec["recompute_idx"],
                             dec["n_recompute"], mass_len=mass_len, obs_window=wl.obs_window)
    kc_ref = O.scatter_kv(a["k_cache"], kn_c[:R * wl.L_c], rec, a["active_off"], wl.L_c)
    vc_ref = O.scatter_kv(a["v_cache"], vn_c[:R * wl.L_c], rec, a["active_off"], wl.L_c)
    ref_out, _ = O.attend(q_c[:R * wl.L_c], kc_ref, vc_ref, wl.L_clean, a["active_off"], wl.L_c, rec)
    got = O.widen(B.to_host(res["out"]))[:R * wl.L_c]
    tol = 1e-5 * np.abs(ref_out).max() if wl.dtype == "f32" else 2e-2
    assert np.abs(got - ref_out).max() <= tol
    if eps == 0.0:   # equals uncached full chunk-causal attention built directly from k_new
        kfull = np.concatenate([a["k_cache"][:, :wl.L_clean], np.transpose(a["k_new"], (1, 0, 2))], 1)
        vfull = np.concatenate([a["v_cache"][:, :wl.L_clean], np.transpose(a["v_new"], (1, 0, 2))], 1)
        unc, _ = O.attend(a["q"], kfull, vfull, wl.L_clean, a["active_off"], wl.L_c, list(range(A)))
        assert np.abs(got - unc).max() <= tol
    # commit: compress [clean | chunk 0] with the mass the GPU emitted (shared-mass protocol)
    mass_gpu = res["mass"]
    ref_mass = O.attention_mass(O.observation_rows(q_c, R, wl.L_c, wl.obs_window), kc_ref, mass_len)
    assert_mass_close(mass_gpu.cpu().numpy(), ref_mass, wl.dtype, wl.name)
    budget = wl.budget
    kept = B.flowcache_kv_compress(kc, vc, mass_len, budget, mass_gpu, wl.pool_k, wl.lam)
    torch.cuda.synchronize()
    rk, rk_k, rk_v, _ = O.kv_compress(kc_ref, vc_ref, mass_len, budget, mass_gpu.cpu().numpy(),
                                      wl.pool_k, wl.lam)
    assert np.array_equal(kept.cpu().numpy(), rk)
    assert np.array_equal(B.to_host(kc), rk_k) and np.array_equal(B.to_host(vc), rk_v)
