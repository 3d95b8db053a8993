"""CPU oracle for the FlowCache denoising-step hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct float64 numpy implementation of what the paper defines,
written from the paper and sharing no code with the HIP library.  Only the test suite,
the smoke check and the benchmark's ``cpu_baseline`` leg may import it; the product path
never does.

Every function names the passage it follows.  Where the paper is silent the reading is
stated in the function's docstring.  Pins (closed forms, invariants, brute force, library
special cases) live in ``tests/test_oracle_*.py``.  Pin status:

  relative_l1, reuse_policy, chunk_decide .. pinned (hand-worked case, closed forms)
  gather_chunks, scatter_kv ................ pinned (exact copies)
  narrow, residual_apply ................... pinned (brute-force nearest neighbour, ties,
                                             exact round trips, hand-worked case)
  uniform_decide ........................... pinned (hand-worked case, reduction to the
                                             chunkwise policy for one chunk)
  attend, attention_mass ................... pinned (brute force loops, library special
                                             case, invariants)
  maxpool1d ................................ pinned (library max-pool, brute force)
  redundancy (linear / quadratic) .......... pinned (identity of App. C.2, closed forms)
  select_top_b ............................. pinned (brute-force rank count)
  compact_kv, kv_compress .................. pinned (identity case, exact copies)
  kv_compress_grouped ...................... pinned (group = 1 is kv_compress; identical tokens
                                             inside each group reduce it to kv_compress on one
                                             token per group; hand-worked case; means stay float64)
  Parity unpinned (the paper gives no value): the max-pool kernel size, the exact
  attention mask and the order of the surviving tokens rest on the readings below.

Inputs arrive either as float arrays or as uint16 arrays of bfloat16 bit patterns;
``widen`` turns both into float64 exactly.
"""
from __future__ import annotations

from typing import Dict, Iterable, List, Optional, Sequence, Tuple

import numpy as np

NORM_FLOOR = 1e-12


def widen(a: np.ndarray) -> np.ndarray:
    """Exact widening to float64 (bfloat16 bit patterns come as uint16)."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# ======================================================================================
# Change metric and reuse decision -- Sec. 3.2, Eq. (4), (5), (8)
# ======================================================================================
def relative_l1(x_cur: np.ndarray, x_prev: np.ndarray) -> float:
    """Eq. (5): ||X_{t-1} - X_t||_1 / ||X_t||_1 for one chunk.

    Time counts down, so X_t is the earlier (previous-tick) tensor: it is the one in the
    denominator.  A zero denominator gives +inf (0/0 included), which forces recompute.
    """
    x_cur = widen(x_cur).ravel()
    x_prev = widen(x_prev).ravel()
    num = float(np.sum(np.abs(x_cur - x_prev)))
    den = float(np.sum(np.abs(x_prev)))
    if den == 0.0:
        return float("inf")
    return num / den


def reuse_policy(l1rel: float, acc_old: float, step_idx: int, warmup_m: int,
                 eps: float) -> Tuple[float, bool]:
    """Eq. (8) for one chunk at one tick -> (f_new, recompute).

    Case 1: the chunk's first ``m`` local steps never reuse, f = 0.
    Case 2: accumulated change above eps -> f = 0.
    Case 3: otherwise f = accumulated change.
    Forward computation happens exactly when f = 0 (Sec. 3.2, text after Eq. (8)); this
    literal reading also recomputes when the accumulated change is exactly zero.
    The warm-up window of Eq. (8) is read per chunk in local steps (``step_idx`` counts
    the steps the chunk has already taken).
    """
    if step_idx < warmup_m:
        f_new = 0.0
    else:
        a = acc_old + l1rel
        f_new = 0.0 if a > eps else a
    return f_new, (f_new == 0.0)


def chunk_decide(x_cur: np.ndarray, x_prev: np.ndarray, step_idx: Sequence[int],
                 warmup_m: int, eps: float, acc: Sequence[float]) -> Dict[str, np.ndarray]:
    """Eq. (5) + Eq. (8) over the ``A`` active chunks; x_* are ``[A, chunk_elems]``.

    Returns mask (1 = recompute), acc_new, l1rel, the ascending list of chunks to
    recompute and ``margin`` = |acc_old + l1rel - eps| (how far the comparison is from
    flipping; inf during warm-up).
    """
    A = x_cur.shape[0]
    mask = np.zeros(A, dtype=np.uint8)
    acc_new = np.zeros(A, dtype=np.float64)
    l1 = np.zeros(A, dtype=np.float64)
    margin = np.full(A, np.inf)
    for i in range(A):
        l1[i] = relative_l1(x_cur[i], x_prev[i])
        acc_new[i], rec = reuse_policy(l1[i], float(acc[i]), int(step_idx[i]), warmup_m, eps)
        mask[i] = 1 if rec else 0
        if int(step_idx[i]) >= warmup_m:
            margin[i] = abs(float(acc[i]) + l1[i] - eps)
    idx = np.flatnonzero(mask).astype(np.int32)
    return {"mask": mask, "acc": acc_new, "l1rel": l1, "recompute_idx": idx,
            "n_recompute": np.int32(idx.size), "margin": margin}


def uniform_decide(x_cur, x_prev, step_idx, warmup_m, eps, acc_global):
    """The uniform ("traditional reuse") policy of Fig. 2, top: one accumulator driven by
    the relative L1 over all chunks past warm-up; every such chunk shares the decision,
    while a newly initialised chunk (still in warm-up) always computes."""
    A = x_cur.shape[0]
    old = [i for i in range(A) if int(step_idx[i]) >= warmup_m]
    mask = np.ones(A, dtype=np.uint8)
    if not old:
        return {"mask": mask, "acc": 0.0, "l1rel": float("nan")}
    num = sum(float(np.sum(np.abs(widen(x_cur[i]) - widen(x_prev[i])))) for i in old)
    den = sum(float(np.sum(np.abs(widen(x_prev[i])))) for i in old)
    l1 = float("inf") if den == 0.0 else num / den
    a = acc_global + l1
    f_new = 0.0 if a > eps else a
    for i in old:
        mask[i] = 1 if f_new == 0.0 else 0
    return {"mask": mask, "acc": f_new, "l1rel": l1}


def narrow(x: np.ndarray, like: np.ndarray) -> np.ndarray:
    """Round float64 values ONCE, to nearest with ties to even, to the storage type of
    ``like``: float32, or bfloat16 returned as uint16 bit patterns (8 significant bits, the
    exponent range of float32, gradual underflow below 2^-126)."""
    x = np.asarray(x, dtype=np.float64)
    if np.asarray(like).dtype != np.uint16:
        return x.astype(np.float32)
    _, e = np.frexp(x)                                # x = m * 2^e, 0.5 <= |m| < 1
    ulp_exp = np.maximum(e - 8, -133)                 # spacing of bfloat16 numbers around x
    q = np.rint(np.ldexp(x, -ulp_exp))                # np.rint rounds halves to even
    y = np.ldexp(q, ulp_exp).astype(np.float32)       # exact: at most 8 significant bits
    return (y.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


# ======================================================================================
# Cached-activation reuse around a skipped forward pass -- Sec. 3.2 (text after Eq. (8))
# ======================================================================================
def residual_apply(x_cur: np.ndarray, y_compact: Optional[np.ndarray], residual: np.ndarray,
                   recompute_idx: Sequence[int]) -> Tuple[np.ndarray, np.ndarray]:
    """Returns (new residual cache, full-layout output).

    The paper only says that a chunk with f != 0 reuses its cached activations.  Reading:
    the cached quantity is output minus input of the layer stack at the chunk's last
    recompute (inputs and outputs stay close along the trajectory, Sec. 3.2, third
    observation), so a reused chunk returns input + cached difference.  Each value is
    computed in float64 and rounded once to the storage type.
    """
    res = np.array(residual, copy=True)
    out = np.empty_like(np.asarray(x_cur))
    rec = [int(c) for c in recompute_idx]
    for c in range(x_cur.shape[0]):
        if c in rec:
            r = rec.index(c)
            res[c] = narrow(widen(y_compact[r]) - widen(x_cur[c]), x_cur)
            out[c] = y_compact[r]
        else:
            out[c] = narrow(widen(x_cur[c]) + widen(residual[c]), x_cur)
    return res, out


# ======================================================================================
# Gather of the chunks to recompute; scatter of their new K/V -- Sec. 3.2 (Fig. 2)
# ======================================================================================
def gather_chunks(x: np.ndarray, recompute_idx: Sequence[int]) -> np.ndarray:
    """x_compact[r] = x[recompute_idx[r]] (bit copy)."""
    return np.stack([x[i] for i in recompute_idx]) if len(recompute_idx) else x[:0].copy()


def scatter_kv(cache: np.ndarray, new: np.ndarray, recompute_idx: Sequence[int],
               active_off: Sequence[int], L_c: int) -> np.ndarray:
    """Write the recomputed chunks' rows of ``new`` (compact ``[R*L_c, H_k, d]``, block r
    <-> chunk recompute_idx[r]) into their slots of the head-major cache
    ``[H_k, capacity, d]``.  Slots of reused chunks keep their stale contents."""
    out = cache.copy()
    for r, c in enumerate(recompute_idx):
        blk = new[r * L_c:(r + 1) * L_c]                 # [L_c, H_k, d]
        out[:, active_off[c]:active_off[c] + L_c, :] = np.transpose(blk, (1, 0, 2))
    return out


# ======================================================================================
# Chunk-causal attention -- Sec. 3.3 first paragraph; scale d^-1/2 as in Eq. (9)
# ======================================================================================
def visible_positions(c: int, L_clean: int, active_off: Sequence[int], L_c: int) -> np.ndarray:
    """Cache positions a query of active chunk ``c`` attends to: every clean token, then
    the tokens of active chunks 0..c (all of its own chunk: attention is bidirectional
    inside a chunk and causal across chunks)."""
    parts = [np.arange(L_clean)]
    for a in range(c + 1):
        parts.append(np.arange(active_off[a], active_off[a] + L_c))
    return np.concatenate(parts)


def attend(q: np.ndarray, k_cache: np.ndarray, v_cache: np.ndarray, L_clean: int,
           active_off: Sequence[int], L_c: int, recompute_idx: Sequence[int],
           scale: Optional[float] = None, rows: Optional[Iterable[int]] = None,
           heads: Optional[Iterable[int]] = None, return_probs: bool = False):
    """softmax(q K^T * scale) V for the recompute chunks.

    q is compact ``[R*L_c, H_q, d]``; caches are ``[H_k, capacity, d]`` and already hold
    the new K/V of the recompute chunks.  Query head h reads key head h // (H_q/H_k).
    ``rows`` (indices into the compact row axis) and ``heads`` restrict the work to a
    sample.  Returns (out ``[n_rows, n_heads, d]``, lse ``[n_heads, n_rows]``) and, on
    request, the list of probability rows.
    """
    qf = widen(q)
    kf = widen(k_cache)
    vf = widen(v_cache)
    n_rows_all, H_q, d = qf.shape
    H_k = kf.shape[0]
    G = H_q // H_k
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    rows = list(range(n_rows_all)) if rows is None else [int(r) for r in rows]
    heads = list(range(H_q)) if heads is None else [int(h) for h in heads]
    out = np.zeros((len(rows), len(heads), d))
    lse = np.zeros((len(heads), len(rows)))
    probs: List = []
    by_chunk: Dict[int, List[int]] = {}
    for n, row in enumerate(rows):
        by_chunk.setdefault(row // L_c, []).append(n)
    for r, members in by_chunk.items():
        c = int(recompute_idx[r])
        vis = visible_positions(c, L_clean, active_off, L_c)
        sel = np.array([rows[n] for n in members])
        for hn, h in enumerate(heads):
            kk = kf[h // G][vis]                          # [n_vis, d]
            vv = vf[h // G][vis]
            s = (qf[sel, h, :] @ kk.T) * scale            # [n_sel, n_vis]
            mx = s.max(axis=1, keepdims=True)
            e = np.exp(s - mx)
            z = e.sum(axis=1, keepdims=True)
            p = e / z
            out[members, hn, :] = p @ vv
            lse[hn, members] = (mx + np.log(z))[:, 0]
            if return_probs:
                probs.append((r, h, sel, vis, p))
    if return_probs:
        return out, lse, probs
    return out, lse


# ======================================================================================
# Importance -- Sec. 3.3, Eq. (9); observation window: App. C.2 and App. D.2.1
# ======================================================================================
def attention_mass(q_obs: np.ndarray, k_cache: np.ndarray, L_k: int,
                   scale: Optional[float] = None) -> np.ndarray:
    """Eq. (9): mass[h_k, j] = mean over observation rows of softmax_j(q K^T / sqrt d).

    ``q_obs`` is ``[W, H_q, d]`` (the paper's implementation uses the last 50 tokens of the
    last denoising chunk).  The softmax runs over the first ``L_k`` cache positions only --
    the keys about to be compressed.  The rows of key head h_k are the W tokens times its
    G query heads; their mean keeps sum_j mass = 1.
    """
    qf = widen(q_obs)
    kf = widen(k_cache)[:, :L_k, :]
    W, H_q, d = qf.shape
    H_k = kf.shape[0]
    G = H_q // H_k
    if scale is None:
        scale = 1.0 / np.sqrt(d)
    mass = np.zeros((H_k, L_k))
    for hk in range(H_k):
        for g in range(G):
            s = (qf[:, hk * G + g, :] @ kf[hk].T) * scale
            e = np.exp(s - s.max(axis=1, keepdims=True))
            mass[hk] += (e / e.sum(axis=1, keepdims=True)).sum(axis=0)
        mass[hk] /= (W * G)
    return mass


def observation_rows(q_compact: np.ndarray, n_recompute: int, L_c: int, W: int) -> np.ndarray:
    """Last W tokens of the last compact row block (W = 0 or W > L_c: the whole block)."""
    if W <= 0 or W > L_c:
        W = L_c
    end = n_recompute * L_c
    return q_compact[end - W:end]


def maxpool1d(x: np.ndarray, k: int) -> np.ndarray:
    """Eq. (10): stride-1 max-pool of odd width k with k//2 padding on both sides (padded
    with -inf), along the last axis: same length out as in."""
    if k < 1 or k % 2 == 0:
        raise ValueError("pool width must be odd and >= 1")
    x = np.asarray(x, dtype=np.float64)
    L = x.shape[-1]
    half = k // 2
    pad = np.full(x.shape[:-1] + (half,), -np.inf)
    xp = np.concatenate([pad, x, pad], axis=-1)          # xp[..., j + half] = x[..., j]
    out = xp[..., 0:L].copy()
    for u in range(1, k):                                # window offsets -half .. +half
        out = np.maximum(out, xp[..., u:u + L])
    return out


# ======================================================================================
# Redundancy -- Sec. 3.3, Eq. (11); linear form: App. C.2
# ======================================================================================
def normalize_keys(k: np.ndarray) -> np.ndarray:
    """l2-normalise each key; a key with norm below 1e-12 is divided by 1e-12 instead
    (a zero key stays zero)."""
    k = widen(k)
    nrm = np.sqrt(np.sum(k * k, axis=-1, keepdims=True))
    return k / np.maximum(nrm, NORM_FLOOR)


def mean_similarity_quadratic(k: np.ndarray) -> np.ndarray:
    """Eq. (11) as printed, for one head: S = K^ K^T, S_ii = 0, column mean.  O(L^2)."""
    kh = normalize_keys(k)
    S = kh @ kh.T
    np.fill_diagonal(S, 0.0)
    return S.sum(axis=0) / kh.shape[0]


def mean_similarity_linear(k: np.ndarray) -> np.ndarray:
    """App. C.2: sum the normalised keys first, then one matrix-vector product.  The
    diagonal term that Eq. (11) zeroes is subtracted explicitly so that both forms agree
    for every input (zero keys included)."""
    kh = normalize_keys(k)
    s = kh.sum(axis=0)
    return (kh @ s - np.sum(kh * kh, axis=1)) / kh.shape[0]


def softmax_1d(r: np.ndarray) -> np.ndarray:
    e = np.exp(r - r.max())
    return e / e.sum()


def redundancy(k: np.ndarray, quadratic: bool = False) -> np.ndarray:
    """Eq. (11): softmax over the token index of the mean cosine similarity."""
    r = mean_similarity_quadratic(k) if quadratic else mean_similarity_linear(k)
    return softmax_1d(r)


def selection_scores(k: np.ndarray, mass: np.ndarray, pool_k: int, lam: float,
                     quadratic: bool = False) -> np.ndarray:
    """Eq. (12) for one head: lambda * pooled importance - (1 - lambda) * redundancy."""
    imp = maxpool1d(np.asarray(mass, dtype=np.float64), pool_k)
    return lam * imp - (1.0 - lam) * redundancy(k, quadratic)


# ======================================================================================
# Selection and compaction -- Sec. 3.3 (top-B per head), App. C.1 (fill phase)
# ======================================================================================
def select_top_b(score: np.ndarray, B: int) -> np.ndarray:
    """Indices of the B highest scores, ties to the lower index, returned ascending.
    B >= L keeps everything (cache-filling phase: no compression)."""
    score = np.asarray(score, dtype=np.float64)
    L = score.shape[0]
    if not np.all(np.isfinite(score)):
        raise ValueError("scores must be finite")
    if B >= L:
        return np.arange(L, dtype=np.int32)
    order = np.lexsort((np.arange(L), -score))           # by score desc, then index asc
    return np.sort(order[:B]).astype(np.int32)


def select_top_b_bruteforce(score: np.ndarray, B: int) -> np.ndarray:
    """Definition by rank count, O(L^2), no sort: j is kept iff fewer than B tokens beat
    it, where u beats j if score_u > score_j, or they tie and u < j."""
    score = np.asarray(score, dtype=np.float64)
    L = score.shape[0]
    keep = []
    for j in range(L):
        beat = 0
        for u in range(L):
            if score[u] > score[j] or (score[u] == score[j] and u < j):
                beat += 1
        if beat < B:
            keep.append(j)
    return np.array(keep, dtype=np.int32)


def boundary_gap(score: np.ndarray, B: int) -> float:
    """Relative gap between the B-th and (B+1)-th highest score (0 for an exact tie)."""
    score = np.asarray(score, dtype=np.float64)
    if B >= score.shape[0] or B <= 0:
        return float("inf")
    s = np.sort(score)[::-1]
    return float(abs(s[B - 1] - s[B]) / max(abs(s[B - 1]), abs(s[B]), 1e-300))


def compact_kv(cache: np.ndarray, kept: np.ndarray) -> np.ndarray:
    """Move kept rows (per head, ascending original position) to positions 0..B-1.
    ``cache`` is ``[H_k, n, d]`` storage; rows beyond B keep whatever they held."""
    out = cache.copy()
    for h in range(cache.shape[0]):
        out[h, :kept.shape[1]] = cache[h, kept[h]]
    return out


def kv_compress(k_cache: np.ndarray, v_cache: np.ndarray, L_k: int, budget: int,
                mass: np.ndarray, pool_k: int, lam: float):
    """One commit: score (Eq. (10)-(12)), keep top-``budget`` per key head, compact K and
    V in place.  Returns (kept ``[H_k, min(budget, L_k)]``, new K, new V, scores)."""
    H_k = k_cache.shape[0]
    B = min(budget, L_k)
    kept = np.empty((H_k, B), dtype=np.int32)
    scores = np.empty((H_k, L_k))
    for h in range(H_k):
        scores[h] = selection_scores(k_cache[h, :L_k], mass[h, :L_k], pool_k, lam)
        kept[h] = select_top_b(scores[h], budget)
    if budget >= L_k:
        return kept, k_cache.copy(), v_cache.copy(), scores
    return kept, compact_kv(k_cache, kept), compact_kv(v_cache, kept), scores


# ======================================================================================
# Key granularity above the token -- App. D.2.1 (frame- / chunk-level keys)
# ======================================================================================
def kv_compress_grouped(k_cache: np.ndarray, v_cache: np.ndarray, L_k: int, budget: int, group: int,
                        mass: np.ndarray, pool_k: int = 7, lam: float = 0.07):
    """Compression with keys scored and kept in groups of ``group`` consecutive tokens.

    The paper names the granularities (token, frame, chunk) without saying how a group of keys
    is represented.  Reading: the group's key is the mean of its keys, its importance the mean
    of its tokens' mass, both plain float64 means (no intermediate rounding); Eq. (10)-(12) and
    the top-B selection then run over groups exactly as they do over tokens, and all tokens of
    a kept group are kept.  Returns (kept token indices [H, budget], new K, new V, group scores).
    """
    assert L_k % group == 0 and budget % group == 0
    H = k_cache.shape[0]
    G, Bg = L_k // group, budget // group
    k_new, v_new = np.array(k_cache, copy=True), np.array(v_cache, copy=True)
    if budget >= L_k:
        kept = np.tile(np.arange(L_k, dtype=np.int32), (H, 1))
        return kept, k_new, v_new, None
    kept = np.empty((H, budget), dtype=np.int32)
    scores = []
    for h in range(H):
        kw = widen(k_cache[h, :L_k]).reshape(G, group, -1)
        kg = kw.sum(axis=1) / group
        mg = np.asarray(mass[h, :L_k], dtype=np.float64).reshape(G, group).sum(axis=1) / group
        sc = selection_scores(kg, mg, pool_k, lam)
        groups = select_top_b(sc, Bg)
        kept[h] = (np.asarray(groups, dtype=np.int64)[:, None] * group
                   + np.arange(group)[None, :]).reshape(-1).astype(np.int32)
        k_new[h, :budget] = k_cache[h, kept[h]]
        v_new[h, :budget] = v_cache[h, kept[h]]
        scores.append(sc)
    return kept, k_new, v_new, scores
