"""Seeded synthetic inputs for the FlowCache hot path.

This module only draws random numbers and lays them out in memory.  It holds none of
the method's arithmetic (no change metric, no attention, no scoring, no selection), so
both the CPU oracle's tests and the HIP path's tests may feed from it: both sides then
consume exactly the same bits.

Storage convention
------------------
* dtype ``"f32"``: numpy ``float32`` arrays.
* dtype ``"bf16"``: numpy ``uint16`` arrays holding bfloat16 bit patterns (numpy has no
  bfloat16).  Values are drawn in float32 and rounded once, round-to-nearest-even.

Shapes mirror the token grids of the two autoregressive video DiTs the paper evaluates
(Sec. 4.1): a SkyReels-V2-1.3B-like layer (12 heads x 128, chunk of 5 latent frames x
34 x 60 patches) and a MAGI-1-like layer (24 heads x 128, chunk of 6 latent frames x
30 x 52 patches).  No item of any public benchmark is reproduced: only shapes.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict, Optional, Tuple

import numpy as np


# --------------------------------------------------------------------------------------
# storage helpers (bit manipulation only)
# --------------------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest even) and return the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    if dtype == "f32":
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(f"unknown dtype {dtype!r}")


def storage_dtype(dtype: str):
    return {"f32": np.float32, "bf16": np.uint16}[dtype]


def elem_bytes(dtype: str) -> int:
    return {"f32": 4, "bf16": 2}[dtype]


# --------------------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    """One configuration of the denoising-step hot path.

    ``A`` active chunks of ``L_c`` tokens each are denoised against a clean-context KV
    cache of ``L_clean`` tokens; on commit the first ``L_k`` cache positions are
    compressed to ``budget`` tokens per key head.
    """

    name: str
    dtype: str          # "f32" | "bf16"
    H_q: int
    H_k: int
    d: int
    A: int
    L_c: int
    L_clean: int
    budget: int
    warmup_m: int = 4
    eps: float = 0.1
    pool_k: int = 7
    lam: float = 0.07
    obs_window: int = 50
    keys: str = "normal"      # "normal" | "clustered" | "heavy_dup"

    @property
    def D(self) -> int:
        return self.H_q * self.d

    @property
    def chunk_elems(self) -> int:
        return self.L_c * self.D

    @property
    def capacity(self) -> int:
        return self.L_clean + self.A * self.L_c

    @property
    def L_k(self) -> int:
        return self.L_clean

    def active_off(self) -> np.ndarray:
        return (self.L_clean + self.L_c * np.arange(self.A)).astype(np.int32)

    def attention_pairs_per_head(self, recompute=None) -> int:
        chunks = range(self.A) if recompute is None else recompute
        return sum(self.L_c * (self.L_clean + (c + 1) * self.L_c) for c in chunks)

    def attention_flops(self, recompute=None) -> int:
        return 4 * self.d * self.H_q * self.attention_pairs_per_head(recompute)


# C1: tiny fp32 step (1 key head shared by 4 query heads; 2 chunks of 2 x 8 x 8 tokens).
C1 = Workload("C1-tiny-f32", "f32", H_q=4, H_k=1, d=64, A=2, L_c=128, L_clean=512,
              budget=256, warmup_m=4, eps=0.05)
C1_MHA = replace(C1, name="C1-tiny-f32-mha", H_k=4)
# C2: SkyReels-V2-1.3B-like layer: 12 x 128, chunk 5 x 34 x 60 = 10200 tokens.
C2 = Workload("C2-skyreels-v2-1.3B-like-bf16", "bf16", H_q=12, H_k=12, d=128, A=2,
              L_c=10200, L_clean=40800, budget=20400, warmup_m=4, eps=0.1)
# C3: MAGI-1-like layer: 24 x 128, chunk 6 x 30 x 52 = 9360 tokens, clustered keys.
C3 = Workload("C3-magi-1-like-bf16", "bf16", H_q=24, H_k=24, d=128, A=4, L_c=9360,
              L_clean=74880, budget=37440, warmup_m=5, eps=0.015, keys="clustered")
# Reduced shapes: same structure, sized so the fp64 oracle finishes in seconds while
# still spanning several key/query tiles and ragged tails (none is a multiple of 64).
MID_BF16 = Workload("mid-bf16", "bf16", H_q=4, H_k=4, d=128, A=3, L_c=328, L_clean=1000,
                    budget=500, warmup_m=4, eps=0.1)
MID_BF16_GQA = replace(MID_BF16, name="mid-bf16-gqa", H_q=8, H_k=2, L_c=200, L_clean=520,
                       budget=300)
MID_F32 = Workload("mid-f32", "f32", H_q=4, H_k=2, d=64, A=3, L_c=168, L_clean=700,
                   budget=333, warmup_m=4, eps=0.05)
MID_F32_D128 = replace(MID_F32, name="mid-f32-d128", d=128, H_q=2, H_k=2, L_c=100,
                       L_clean=300, budget=150)

WORKLOADS: Dict[str, Workload] = {w.name: w for w in
                                  (C1, C1_MHA, C2, C3, MID_BF16, MID_BF16_GQA, MID_F32,
                                   MID_F32_D128)}


def _rng(seed: int, stream: int) -> np.random.Generator:
    """Independent stream ``stream`` of base seed ``seed``."""
    return np.random.default_rng(np.random.SeedSequence(entropy=seed, spawn_key=(stream,)))


def _normal(rng: np.random.Generator, shape, scale: float = 1.0) -> np.ndarray:
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        out *= np.float32(scale)
    return out


# --------------------------------------------------------------------------------------
# change-metric inputs (streams 0-9)
# --------------------------------------------------------------------------------------
def chunk_sigmas(wl: Workload, seed: int, sigmas=None) -> np.ndarray:
    """Per-chunk step-to-step change magnitude.

    Default: log-uniform in [1e-3, 1e-1] (staggered noise levels give each chunk its own
    change rate).  C1 uses the fixed pair (0.001, 0.1) so that one chunk reuses and one
    recomputes at its threshold.
    """
    if sigmas is not None:
        return np.asarray(sigmas, dtype=np.float64)
    if wl.name.startswith("C1"):
        return np.array([0.001, 0.1], dtype=np.float64)
    r = _rng(seed, 0)
    return np.exp(r.uniform(np.log(1e-3), np.log(1e-1), size=wl.A))


def decide_inputs(wl: Workload, seed: int = 0, sigmas=None, step_idx=None,
                  acc=None) -> Dict[str, np.ndarray]:
    """``x_prev ~ N(0,1)``; ``x_cur = x_prev + sigma_i * N(0,1)`` per chunk ``i``."""
    sig = chunk_sigmas(wl, seed, sigmas)
    x_prev = np.empty((wl.A, wl.chunk_elems), dtype=storage_dtype(wl.dtype))
    x_cur = np.empty_like(x_prev)
    for i in range(wl.A):
        r = _rng(seed, 1 + i)
        p = _normal(r, wl.chunk_elems)
        n = _normal(r, wl.chunk_elems, float(sig[i]))
        x_prev[i] = to_storage(p, wl.dtype)
        n += p
        x_cur[i] = to_storage(n, wl.dtype)
    if step_idx is None:
        step_idx = np.full(wl.A, wl.warmup_m + 3, dtype=np.int32)
    if acc is None:
        acc = np.zeros(wl.A, dtype=np.float64)
    return {"x_prev": x_prev, "x_cur": x_cur, "sigma": sig,
            "step_idx": np.asarray(step_idx, dtype=np.int32).copy(),
            "acc": np.asarray(acc, dtype=np.float64).copy()}


# --------------------------------------------------------------------------------------
# keys / values / queries (streams 10-99)
# --------------------------------------------------------------------------------------
def _keys(rng: np.random.Generator, kind: str, L: int, d: int,
          earlier: Optional[np.ndarray] = None) -> np.ndarray:
    """``L`` key vectors (float32) of one head.

    ``normal``     N(0, I).
    ``clustered``  32 Gaussian centroids c ~ N(0, I); key = c_a + 0.1 * N(0, I), cluster
                   ``a`` uniform per token (spatio-temporal redundancy of video tokens).
    ``heavy_dup``  Student-t (nu = 3) entries; 20 % of the tokens are then replaced by a
                   near-copy (cosine > 0.99) of a random earlier token.
    """
    if kind == "normal":
        return _normal(rng, (L, d))
    if kind == "clustered":
        cent = _normal(rng, (32, d))
        a = rng.integers(0, 32, size=L)
        return cent[a] + _normal(rng, (L, d), 0.1)
    if kind == "heavy_dup":
        g = _normal(rng, (L, d))
        chi = rng.chisquare(3.0, size=(L, d)).astype(np.float32)
        k = g / np.sqrt(chi / np.float32(3.0))
        pool = k if earlier is None else np.concatenate([earlier, k], axis=0)
        base = 0 if earlier is None else earlier.shape[0]
        dup = np.flatnonzero(rng.random(L) < 0.2)
        for j in dup:
            hi = base + j
            if hi == 0:
                continue
            src = pool[rng.integers(0, hi)]
            nrm = float(np.sqrt(np.sum(src.astype(np.float64) ** 2)))
            k[j] = src + _normal(rng, d, 0.01 * nrm / np.sqrt(d))
            pool[base + j] = k[j]
        return k
    raise ValueError(kind)


def attend_inputs(wl: Workload, seed: int = 0) -> Dict[str, np.ndarray]:
    """Q, new K/V of every active chunk (compact token-major) and the KV cache.

    The cache is head-major ``[H_k, capacity, d]``: clean tokens at ``[0, L_clean)``,
    active chunk ``a`` at ``[L_clean + a*L_c, L_clean + (a+1)*L_c)``.  Active slots are
    pre-filled with *stale* K/V (what the slot holds from the chunk's last recompute);
    a recompute overwrites its slot with the chunk's rows of ``k_new``/``v_new``.
    """
    n_act = wl.A * wl.L_c
    cap = wl.capacity
    sd = storage_dtype(wl.dtype)
    q = to_storage(_normal(_rng(seed, 10), (n_act, wl.H_q, wl.d)), wl.dtype)
    k_new = to_storage(_normal(_rng(seed, 11), (n_act, wl.H_k, wl.d)), wl.dtype)
    v_new = to_storage(_normal(_rng(seed, 12), (n_act, wl.H_k, wl.d)), wl.dtype)
    k_cache = np.empty((wl.H_k, cap, wl.d), dtype=sd)
    v_cache = np.empty((wl.H_k, cap, wl.d), dtype=sd)
    for h in range(wl.H_k):
        r = _rng(seed, 20 + h)
        k_cache[h, :wl.L_clean] = to_storage(_keys(r, wl.keys, wl.L_clean, wl.d), wl.dtype)
        k_cache[h, wl.L_clean:] = to_storage(_normal(r, (cap - wl.L_clean, wl.d)), wl.dtype)
        v_cache[h] = to_storage(_normal(r, (cap, wl.d)), wl.dtype)
    return {"q": q, "k_new": k_new, "v_new": v_new, "k_cache": k_cache,
            "v_cache": v_cache, "active_off": wl.active_off()}


def synthetic_mass(H_k: int, L: int, seed: int = 0, plateau: bool = True) -> np.ndarray:
    """A float32 stand-in for an attention-mass vector per key head: positive, heavy
    tailed (exponential draws raised to a power), with a few exactly repeated values so
    that score ties occur.  Used where a test wants importance bits that do not depend on
    an attention kernel."""
    r = _rng(seed, 100)
    m = r.exponential(size=(H_k, L)) ** 2.0
    m /= m.sum(axis=1, keepdims=True)
    m = m.astype(np.float32)
    if plateau and L >= 16:
        for h in range(H_k):
            j = r.integers(0, L - 8, size=max(1, L // 64))
            for s in j:
                m[h, s:s + 4] = m[h, s]
    return m


def compress_inputs(wl: Workload, seed: int = 0, L_k: Optional[int] = None,
                    kind: Optional[str] = None) -> Dict[str, np.ndarray]:
    """K, V of the set to compress (``[H_k, L_k, d]``) and a synthetic mass."""
    L = wl.L_k if L_k is None else L_k
    kind = wl.keys if kind is None else kind
    sd = storage_dtype(wl.dtype)
    k = np.empty((wl.H_k, L, wl.d), dtype=sd)
    v = np.empty((wl.H_k, L, wl.d), dtype=sd)
    for h in range(wl.H_k):
        r = _rng(seed, 200 + h)
        k[h] = to_storage(_keys(r, kind, L, wl.d), wl.dtype)
        v[h] = to_storage(_normal(r, (L, wl.d)), wl.dtype)
    return {"k": k, "v": v, "mass": synthetic_mass(wl.H_k, L, seed)}


def rollout_chunk_keys(wl: Workload, seed: int, commit: int,
                       earlier: Optional[np.ndarray], kind: str = "heavy_dup"
                       ) -> Tuple[np.ndarray, np.ndarray]:
    """K, V (``[H_k, L_c, d]`` storage) of the chunk committed at step ``commit`` of a long
    rollout.  ``earlier`` (``[H_k, n, d]`` float32 or None) are keys already in the cache,
    from which near-duplicates are drawn."""
    sd = storage_dtype(wl.dtype)
    k = np.empty((wl.H_k, wl.L_c, wl.d), dtype=sd)
    v = np.empty((wl.H_k, wl.L_c, wl.d), dtype=sd)
    for h in range(wl.H_k):
        r = _rng(seed, 1000 + 64 * commit + h)
        e = None if earlier is None else earlier[h]
        k[h] = to_storage(_keys(r, kind, wl.L_c, wl.d, e), wl.dtype)
        v[h] = to_storage(_normal(r, (wl.L_c, wl.d)), wl.dtype)
    return k, v


def observation_queries(wl: Workload, seed: int, commit: int, W: int) -> np.ndarray:
    """``[W, H_q, d]`` storage: the observation-window queries used at one commit."""
    return to_storage(_normal(_rng(seed, 5000 + commit), (W, wl.H_q, wl.d)), wl.dtype)
