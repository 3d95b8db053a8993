"""Pins for the oracle's chunk-causal attention and importance mass (Sec. 3.3, Eq. (9)):
brute force with an explicit mask, the library's dense attention as a special case,
closed forms and invariants.  CPU only."""
import json
import os

import numpy as np
import pytest
import torch
from scipy.special import logsumexp

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import synth

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_worked.json")))


def tiny(seed=0, A=3, L_c=5, L_clean=7, H_q=4, H_k=2, d=8, gap=2):
    """Random tiny problem with non-contiguous active slots (gap between slots)."""
    rng = np.random.default_rng(seed)
    off = np.array([L_clean + 1 + a * (L_c + gap) for a in range(A)], dtype=np.int32)
    cap = int(off[-1] + L_c + 3)
    return dict(q=rng.standard_normal((A * L_c, H_q, d)),
                k=rng.standard_normal((H_k, cap, d)), v=rng.standard_normal((H_k, cap, d)),
                off=off, L_c=L_c, L_clean=L_clean, A=A, H_q=H_q, H_k=H_k, d=d, cap=cap)


def masked_dense_attention(p, recompute_idx):
    """Independent formulation: full [row, capacity] boolean mask + library softmax."""
    q = torch.from_numpy(p["q"])
    k = torch.from_numpy(p["k"])
    v = torch.from_numpy(p["v"])
    G = p["H_q"] // p["H_k"]
    n = len(recompute_idx) * p["L_c"]
    mask = torch.zeros(n, p["cap"], dtype=torch.bool)
    for r, c in enumerate(recompute_idx):
        rows = slice(r * p["L_c"], (r + 1) * p["L_c"])
        mask[rows, :p["L_clean"]] = True
        for a in range(c + 1):
            mask[rows, p["off"][a]:p["off"][a] + p["L_c"]] = True
    out = torch.zeros(n, p["H_q"], p["d"], dtype=torch.float64)
    for h in range(p["H_q"]):
        s = q[:n, h] @ k[h // G].T / np.sqrt(p["d"])
        s = s.masked_fill(~mask, float("-inf"))
        out[:, h] = torch.softmax(s, dim=-1) @ v[h // G]
    return out.numpy(), mask.numpy()


@pytest.mark.parametrize("rec", [[0, 1, 2], [1], [0, 2], [2]])
def test_matches_masked_dense_formulation(rec):
    p = tiny(seed=1)
    q = np.concatenate([p["q"][c * p["L_c"]:(c + 1) * p["L_c"]] for c in rec])
    pp = dict(p, q=q)
    ref, _ = masked_dense_attention(pp, rec)
    out, lse = O.attend(q, p["k"], p["v"], p["L_clean"], p["off"], p["L_c"], rec)
    assert np.allclose(out, ref, rtol=1e-12, atol=1e-13)


def test_mask_is_block_lower_triangular_with_full_diagonal_blocks():
    p = tiny(seed=2, gap=0)
    _, mask = masked_dense_attention(p, [0, 1, 2])
    for c in range(p["A"]):
        vis = set(O.visible_positions(c, p["L_clean"], p["off"], p["L_c"]).tolist())
        assert vis == set(np.flatnonzero(mask[c * p["L_c"]]).tolist())
        own = range(p["off"][c], p["off"][c] + p["L_c"])
        assert all(j in vis for j in own)                        # bidirectional inside
        if c + 1 < p["A"]:
            assert p["off"][c + 1] not in vis                    # causal across chunks


def test_single_chunk_no_clean_context_is_textbook_attention():
    rng = np.random.default_rng(3)
    L, H, d = 33, 3, 16
    q = rng.standard_normal((L, H, d))
    k = rng.standard_normal((H, L, d))
    v = rng.standard_normal((H, L, d))
    out, lse = O.attend(q, k, v, 0, [0], L, [0])
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).permute(1, 0, 2), torch.from_numpy(k), torch.from_numpy(v))
    assert np.allclose(out, ref.permute(1, 0, 2).numpy(), rtol=1e-12, atol=1e-13)
    s = np.einsum("lhd,hjd->hlj", q, k) / np.sqrt(d)
    assert np.allclose(lse, logsumexp(s, axis=-1), rtol=1e-13)


def test_hand_worked_three_key_row():
    e = GOLD["attention_2keys"]["e"]
    q = np.zeros((1, 1, 4)); q[0, 0, 0] = 2.0
    k = np.zeros((1, 3, 4)); k[0, 0, 0] = 1.0; k[0, 1, 1] = 1.0
    v = np.zeros((1, 3, 4)); v[0, 0] = 1.0; v[0, 1] = 2.0; v[0, 2] = 4.0
    out, lse = O.attend(q, k, v, 2, [2], 1, [0])
    assert np.allclose(out[0, 0], (e * 1 + 2 + 4) / (e + 2), rtol=1e-15)
    assert lse[0, 0] == pytest.approx(np.log(e + 2), rel=1e-15)


def test_rows_sum_to_one_and_output_in_convex_hull():
    p = tiny(seed=4)
    out, lse, probs = O.attend(p["q"], p["k"], p["v"], p["L_clean"], p["off"], p["L_c"],
                               [0, 1, 2], return_probs=True)
    G = p["H_q"] // p["H_k"]
    for r, h, sel, vis, pr in probs:
        assert np.allclose(pr.sum(axis=1), 1.0, rtol=0, atol=1e-14)
        assert np.all(pr >= 0)
        vv = p["v"][h // G][vis]
        assert np.all(out[sel, h] <= vv.max(axis=0) + 1e-12)
        assert np.all(out[sel, h] >= vv.min(axis=0) - 1e-12)


def test_equal_keys_give_plain_mean_of_visible_values():
    p = tiny(seed=5)
    p["k"][:] = p["k"][:, :1, :]
    out, _ = O.attend(p["q"], p["k"], p["v"], p["L_clean"], p["off"], p["L_c"], [0, 1, 2])
    G = p["H_q"] // p["H_k"]
    for c in range(p["A"]):
        vis = O.visible_positions(c, p["L_clean"], p["off"], p["L_c"])
        for h in range(p["H_q"]):
            ref = p["v"][h // G][vis].mean(axis=0)
            assert np.allclose(out[c * p["L_c"]:(c + 1) * p["L_c"], h], ref, atol=1e-13)


def test_permuting_clean_tokens_changes_nothing():
    p = tiny(seed=6)
    perm = np.random.default_rng(0).permutation(p["L_clean"])
    k2, v2 = p["k"].copy(), p["v"].copy()
    k2[:, :p["L_clean"]] = p["k"][:, perm]
    v2[:, :p["L_clean"]] = p["v"][:, perm]
    a, _ = O.attend(p["q"], p["k"], p["v"], p["L_clean"], p["off"], p["L_c"], [0, 1, 2])
    b, _ = O.attend(p["q"], k2, v2, p["L_clean"], p["off"], p["L_c"], [0, 1, 2])
    assert np.allclose(a, b, rtol=1e-12, atol=1e-13)


def test_gqa_equals_mha_with_repeated_key_heads():
    p = tiny(seed=7, H_q=6, H_k=2)
    a, la = O.attend(p["q"], p["k"], p["v"], p["L_clean"], p["off"], p["L_c"], [0, 1, 2])
    k3, v3 = np.repeat(p["k"], 3, axis=0), np.repeat(p["v"], 3, axis=0)
    b, lb = O.attend(p["q"], k3, v3, p["L_clean"], p["off"], p["L_c"], [0, 1, 2])
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_row_and_head_sampling_matches_full_result():
    p = tiny(seed=8)
    full, lse = O.attend(p["q"], p["k"], p["v"], p["L_clean"], p["off"], p["L_c"], [0, 1, 2])
    rows, heads = [0, 4, 5, 9, 14], [1, 3]
    part, lp = O.attend(p["q"], p["k"], p["v"], p["L_clean"], p["off"], p["L_c"], [0, 1, 2],
                        rows=rows, heads=heads)
    assert np.allclose(part, full[np.ix_(rows, heads)], rtol=1e-13, atol=1e-14)
    assert np.allclose(lp, lse[np.ix_(heads, rows)], rtol=1e-13)


def test_eps_zero_chain_equals_uncached_attention_and_reuse_sees_stale_kv():
    wl = synth.C1
    d = synth.decide_inputs(wl, seed=0)
    a = synth.attend_inputs(wl, seed=0)
    # eps = 0: all chunks recompute; gather is the identity; every slot gets its new K/V.
    dec = O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, 0.0, d["acc"])
    rec = dec["recompute_idx"]
    assert rec.tolist() == [0, 1]
    kc = O.scatter_kv(a["k_cache"], a["k_new"], rec, a["active_off"], wl.L_c)
    vc = O.scatter_kv(a["v_cache"], a["v_new"], rec, a["active_off"], wl.L_c)
    out, _ = O.attend(a["q"], kc, vc, wl.L_clean, a["active_off"], wl.L_c, rec)
    # uncached reference: one sequence [clean | chunk0 | chunk1] built directly from k_new
    kfull = np.concatenate([a["k_cache"][:, :wl.L_clean], np.transpose(a["k_new"], (1, 0, 2))], axis=1)
    vfull = np.concatenate([a["v_cache"][:, :wl.L_clean], np.transpose(a["v_new"], (1, 0, 2))], axis=1)
    ref, _ = O.attend(a["q"], kfull, vfull, wl.L_clean, a["active_off"], wl.L_c, [0, 1])
    assert np.array_equal(out, ref)
    # threshold 0.05: chunk 0 reuses, chunk 1 recomputes and attends chunk 0's STALE slot.
    dec = O.chunk_decide(d["x_cur"], d["x_prev"], d["step_idx"], wl.warmup_m, wl.eps, d["acc"])
    rec = dec["recompute_idx"]
    assert rec.tolist() == [1]
    qc = O.gather_chunks(a["q"].reshape(wl.A, wl.L_c, wl.H_q, wl.d), rec).reshape(-1, wl.H_q, wl.d)
    kn = O.gather_chunks(a["k_new"].reshape(wl.A, wl.L_c, wl.H_k, wl.d), rec).reshape(-1, wl.H_k, wl.d)
    kc1 = O.scatter_kv(a["k_cache"], kn, rec, a["active_off"], wl.L_c)
    s0 = slice(a["active_off"][0], a["active_off"][0] + wl.L_c)
    assert np.array_equal(kc1[:, s0], a["k_cache"][:, s0])            # slot 0 untouched
    out1, _ = O.attend(qc, kc1, vc, wl.L_clean, a["active_off"], wl.L_c, rec)
    assert not np.allclose(out1, ref[wl.L_c:])                        # differs from uncached


# ------------------------------------------------------------------ importance, Eq. (9)
def brute_mass(q_obs, k, L_k):
    W, H_q, d = q_obs.shape
    H_k = k.shape[0]
    G = H_q // H_k
    mass = np.zeros((H_k, L_k))
    for hk in range(H_k):
        for w in range(W):
            for g in range(G):
                s = [float(np.dot(q_obs[w, hk * G + g], k[hk, j])) / np.sqrt(d) for j in range(L_k)]
                z = sum(np.exp(x) for x in s)
                for j in range(L_k):
                    mass[hk, j] += np.exp(s[j]) / z / (W * G)
    return mass


def test_mass_matches_brute_force_and_is_a_distribution():
    rng = np.random.default_rng(9)
    q = rng.standard_normal((5, 4, 8))
    k = rng.standard_normal((2, 19, 8))
    m = O.attention_mass(q, k, 13)
    assert np.allclose(m, brute_mass(q, k, 13), rtol=1e-12)
    assert np.allclose(m.sum(axis=1), 1.0, atol=1e-14) and np.all(m > 0)
    # keys beyond L_k do not enter the softmax
    k2 = k.copy(); k2[:, 13:] += 100.0
    assert np.array_equal(O.attention_mass(q, k2, 13), m)


def test_mass_of_identical_keys_is_uniform():
    rng = np.random.default_rng(10)
    q = rng.standard_normal((7, 2, 8))
    k = np.tile(rng.standard_normal((2, 1, 8)), (1, 11, 1))
    assert np.allclose(O.attention_mass(q, k, 11), 1.0 / 11, rtol=1e-13)


def test_mass_is_mean_of_attention_probability_columns():
    # with one active chunk and L_k = every visible key, Eq. (9) is the column mean of the
    # probabilities the attention itself uses
    p = tiny(seed=11, A=1, L_c=6, L_clean=9, H_q=2, H_k=2, gap=0)
    p["off"] = np.array([p["L_clean"]], dtype=np.int32)
    L_k = p["L_clean"] + p["L_c"]
    _, _, probs = O.attend(p["q"], p["k"], p["v"], p["L_clean"], p["off"], p["L_c"], [0],
                           return_probs=True)
    m = O.attention_mass(p["q"], p["k"], L_k)
    for r, h, sel, vis, pr in probs:
        assert np.array_equal(vis, np.arange(L_k))
        assert np.allclose(m[h], pr.mean(axis=0), rtol=1e-12)


def test_observation_rows_are_the_tail_of_the_last_block():
    q = np.arange(3 * 10 * 2).reshape(30, 1, 2)
    assert np.array_equal(O.observation_rows(q, 2, 10, 4), q[16:20])
    assert np.array_equal(O.observation_rows(q, 3, 10, 0), q[20:30])
    assert np.array_equal(O.observation_rows(q, 1, 10, 50), q[0:10])
