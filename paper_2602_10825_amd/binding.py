"""Thin ctypes binding of libflowcache (argument marshalling only).

Every step of the hot path runs in the HIP kernels behind the C ABI declared in
``include/flowcache.h``; this module turns torch tensors into device pointers, allocates
outputs and workspaces with torch, passes the current torch stream, and raises on a
non-zero status.  There is no CPU fallback: if the shared library is missing the import
of :func:`lib` fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libflowcache.so")

FC_F32, FC_BF16 = 0, 1
FC_OK = 0
FC_INVALID_ARGUMENT = 1
FC_HIP_ERROR = 4
FC_MAX_ACTIVE = 16

EXPORTS = (
    "flowcache_status_string", "flowcache_version",
    "flowcache_chunk_decide", "flowcache_chunk_decide_workspace", "flowcache_chunk_decide_noalloc",
    "flowcache_uniform_decide", "flowcache_residual_apply",
    "flowcache_attend", "flowcache_attend_workspace", "flowcache_scatter_kv",
    "flowcache_attention_mass", "flowcache_attention_mass_workspace",
    "flowcache_kv_compress", "flowcache_kv_compress_workspace",
    "flowcache_kv_select", "flowcache_kv_compact",
    "flowcache_kv_compress_grouped", "flowcache_kv_compress_grouped_workspace",
    "flowcache_kv_compress_status_offset",
    "flowcache_sched_state_bytes", "flowcache_sched_init", "flowcache_sched_capacity",
    "flowcache_sched_total_ticks", "flowcache_sched_next",
)

_lib = None


class FlowCacheError(RuntimeError):
    def __init__(self, call: str, status: int):
        self.status = status
        super().__init__(f"{call} failed: {status_string(status)} (status {status})")


def lib() -> ctypes.CDLL:
    """Load libflowcache.so (built in-tree by ``python -m paper_2602_10825_amd.build``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} not found: build it with `python -m paper_2602_10825_amd.build` "
            "(the FlowCache hot path has no CPU fallback)")
    L = ctypes.CDLL(LIB_PATH)
    c_int, c_i64, c_sz, c_vp = ctypes.c_int, ctypes.c_int64, ctypes.c_size_t, ctypes.c_void_p
    c_f, c_d = ctypes.c_float, ctypes.c_double
    L.flowcache_status_string.restype = ctypes.c_char_p
    L.flowcache_status_string.argtypes = [c_int]
    L.flowcache_version.restype = c_int
    L.flowcache_version.argtypes = []
    L.flowcache_chunk_decide_workspace.restype = c_sz
    L.flowcache_chunk_decide_workspace.argtypes = [c_int, c_i64]
    L.flowcache_chunk_decide.restype = c_int
    L.flowcache_chunk_decide.argtypes = [c_vp, c_vp, c_int, c_int, c_i64, c_vp, c_int, c_d, c_vp,
                                         c_vp, c_vp, c_vp, c_vp, c_vp, c_vp, c_sz, c_vp]
    L.flowcache_chunk_decide_noalloc.restype = c_int
    L.flowcache_chunk_decide_noalloc.argtypes = [c_vp, c_vp, c_int, c_int, c_i64, c_vp, c_int, c_d, c_vp,
                                                 c_vp, c_vp, c_vp, c_vp, c_vp, c_vp]
    L.flowcache_uniform_decide.restype = c_int
    L.flowcache_uniform_decide.argtypes = L.flowcache_chunk_decide.argtypes
    L.flowcache_residual_apply.restype = c_int
    L.flowcache_residual_apply.argtypes = [c_vp, c_vp, c_vp, c_vp, c_int, c_int, c_i64, c_vp, c_vp, c_vp]
    L.flowcache_attend_workspace.restype = c_sz
    L.flowcache_attend_workspace.argtypes = [c_int] * 7
    L.flowcache_attend.restype = c_int
    L.flowcache_attend.argtypes = [c_vp, c_vp, c_vp, c_vp, c_vp, c_i64, c_i64, c_int, c_int, c_int,
                                   c_int, c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_f, c_vp,
                                   c_vp, c_vp, c_int, c_int, c_vp, c_sz, c_vp]
    L.flowcache_scatter_kv.restype = c_int
    L.flowcache_scatter_kv.argtypes = [c_vp, c_vp, c_vp, c_vp, c_i64, c_i64, c_int, c_int, c_int,
                                       c_int, c_int, c_int, c_int, c_vp, c_vp, c_vp, c_vp]
    L.flowcache_attention_mass_workspace.restype = c_sz
    L.flowcache_attention_mass_workspace.argtypes = [c_int] * 5
    L.flowcache_attention_mass.restype = c_int
    L.flowcache_attention_mass.argtypes = [c_vp, c_int, c_vp, c_i64, c_i64, c_int, c_int, c_int,
                                           c_int, c_int, c_f, c_vp, c_vp, c_sz, c_vp]
    L.flowcache_kv_compress_workspace.restype = c_sz
    L.flowcache_kv_compress_workspace.argtypes = [c_int, c_int, c_int, c_int, c_int]
    L.flowcache_kv_compress.restype = c_int
    L.flowcache_kv_compress.argtypes = [c_vp, c_vp, c_i64, c_i64, c_int, c_int, c_int, c_int, c_int,
                                        c_vp, c_int, c_d, c_vp, c_vp, c_sz, c_vp]
    L.flowcache_kv_select.restype = c_int
    L.flowcache_kv_select.argtypes = [c_vp, c_i64, c_i64, c_int, c_int, c_int, c_int, c_int, c_vp, c_int,
                                      c_d, c_vp, c_vp, c_sz, c_vp]
    L.flowcache_kv_compact.restype = c_int
    L.flowcache_kv_compact.argtypes = [c_vp, c_vp, c_i64, c_i64, c_int, c_int, c_int, c_int, c_int, c_vp,
                                       c_vp, c_sz, c_vp]
    L.flowcache_kv_compress_grouped_workspace.restype = c_sz
    L.flowcache_kv_compress_grouped_workspace.argtypes = [c_int] * 6
    L.flowcache_kv_compress_grouped.restype = c_int
    L.flowcache_kv_compress_grouped.argtypes = [c_vp, c_vp, c_i64, c_i64, c_int, c_int, c_int, c_int, c_int,
                                                c_int, c_vp, c_int, c_d, c_vp, c_vp, c_sz, c_vp]
    L.flowcache_kv_compress_status_offset.restype = c_sz
    L.flowcache_kv_compress_status_offset.argtypes = [c_int] * 6
    L.flowcache_sched_state_bytes.restype = c_sz
    L.flowcache_sched_state_bytes.argtypes = []
    L.flowcache_sched_init.restype = c_int
    L.flowcache_sched_init.argtypes = [c_vp, c_sz, c_vp]
    L.flowcache_sched_capacity.restype = c_i64
    L.flowcache_sched_capacity.argtypes = [c_vp]
    L.flowcache_sched_total_ticks.restype = c_i64
    L.flowcache_sched_total_ticks.argtypes = [c_vp]
    L.flowcache_sched_next.restype = c_int
    L.flowcache_sched_next.argtypes = [c_vp, c_vp]
    _lib = L
    return L


def status_string(status: int) -> str:
    return lib().flowcache_status_string(int(status)).decode()


def _check(call: str, status: int) -> None:
    if status != FC_OK:
        raise FlowCacheError(call, status)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return FC_F32
    if t.dtype == torch.bfloat16:
        return FC_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream) -> ctypes.c_void_p:
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


# --------------------------------------------------------------------------------------
def flowcache_chunk_decide(x_cur: torch.Tensor, x_prev: torch.Tensor, step_idx: torch.Tensor,
                           warmup_m: int, eps: float, acc: torch.Tensor,
                           x_compact: Optional[torch.Tensor] = None, gather: bool = True,
                           workspace: Optional[torch.Tensor] = None, stream=None
                           ) -> Dict[str, torch.Tensor]:
    """x_cur/x_prev: ``[A, chunk_elems]`` contiguous; acc (float64 ``[A]``) is updated in place."""
    A = x_cur.shape[0]
    chunk_elems = x_cur[0].numel()
    dev = x_cur.device
    assert x_cur.is_contiguous() and x_prev.is_contiguous() and x_prev.shape == x_cur.shape
    assert acc.dtype == torch.float64 and step_idx.dtype == torch.int32
    l1rel = torch.empty(A, dtype=torch.float64, device=dev)
    mask = torch.empty(A, dtype=torch.uint8, device=dev)
    idx = torch.empty(A, dtype=torch.int32, device=dev)
    n_rec = torch.empty(1, dtype=torch.int32, device=dev)
    if x_compact is None and gather:
        x_compact = torch.empty_like(x_cur)
    L = lib()
    if workspace is None:
        workspace = _workspace(L.flowcache_chunk_decide_workspace(A, chunk_elems), dev)
    st = L.flowcache_chunk_decide(_ptr(x_cur), _ptr(x_prev), _dtype_code(x_cur), A, chunk_elems,
                                  _ptr(step_idx), int(warmup_m), float(eps), _ptr(acc), _ptr(l1rel),
                                  _ptr(mask), _ptr(idx), _ptr(n_rec), _ptr(x_compact),
                                  _ptr(workspace), workspace.numel(), _stream(stream))
    _check("flowcache_chunk_decide", st)
    return {"recompute_mask": mask, "recompute_idx": idx, "n_recompute": n_rec, "l1rel": l1rel,
            "acc": acc, "x_compact": x_compact}


def flowcache_chunk_decide_noalloc(x_cur: torch.Tensor, x_prev: torch.Tensor, step_idx: torch.Tensor,
                                   warmup_m: int, eps: float, acc: torch.Tensor, l1rel: torch.Tensor,
                                   recompute_mask: torch.Tensor, recompute_idx: torch.Tensor,
                                   n_recompute: torch.Tensor, x_compact: Optional[torch.Tensor] = None,
                                   stream=None) -> None:
    """flowcache_chunk_decide without a workspace: the caller passes every input and output, the
    library uses its own fixed scratch buffer, and nothing is allocated on either side."""
    A = x_cur.shape[0]
    st = lib().flowcache_chunk_decide_noalloc(
        _ptr(x_cur), _ptr(x_prev), _dtype_code(x_cur), A, x_cur[0].numel(), _ptr(step_idx),
        int(warmup_m), float(eps), _ptr(acc), _ptr(l1rel), _ptr(recompute_mask), _ptr(recompute_idx),
        _ptr(n_recompute), _ptr(x_compact), _stream(stream))
    _check("flowcache_chunk_decide_noalloc", st)


def flowcache_uniform_decide(x_cur: torch.Tensor, x_prev: torch.Tensor, step_idx: torch.Tensor,
                             warmup_m: int, eps: float, acc_global: torch.Tensor,
                             x_compact: Optional[torch.Tensor] = None, gather: bool = True,
                             workspace: Optional[torch.Tensor] = None, stream=None
                             ) -> Dict[str, torch.Tensor]:
    """Uniform policy: acc_global (float64 ``[1]``) is the one shared accumulator, updated in place."""
    A = x_cur.shape[0]
    chunk_elems = x_cur[0].numel()
    dev = x_cur.device
    assert x_cur.is_contiguous() and x_prev.is_contiguous() and x_prev.shape == x_cur.shape
    assert acc_global.dtype == torch.float64 and acc_global.numel() == 1 and step_idx.dtype == torch.int32
    l1rel = torch.empty(1, dtype=torch.float64, device=dev)
    mask = torch.empty(A, dtype=torch.uint8, device=dev)
    idx = torch.empty(A, dtype=torch.int32, device=dev)
    n_rec = torch.empty(1, dtype=torch.int32, device=dev)
    if x_compact is None and gather:
        x_compact = torch.empty_like(x_cur)
    L = lib()
    if workspace is None:
        workspace = _workspace(L.flowcache_chunk_decide_workspace(A, chunk_elems), dev)
    st = L.flowcache_uniform_decide(_ptr(x_cur), _ptr(x_prev), _dtype_code(x_cur), A, chunk_elems,
                                    _ptr(step_idx), int(warmup_m), float(eps), _ptr(acc_global),
                                    _ptr(l1rel), _ptr(mask), _ptr(idx), _ptr(n_rec), _ptr(x_compact),
                                    _ptr(workspace), workspace.numel(), _stream(stream))
    _check("flowcache_uniform_decide", st)
    return {"recompute_mask": mask, "recompute_idx": idx, "n_recompute": n_rec, "l1rel": l1rel,
            "acc": acc_global, "x_compact": x_compact}


def flowcache_residual_apply(x_cur: torch.Tensor, y_compact: Optional[torch.Tensor],
                             residual: torch.Tensor, recompute_idx: torch.Tensor,
                             n_recompute: torch.Tensor, out: Optional[torch.Tensor] = None,
                             stream=None) -> torch.Tensor:
    """x_cur/residual/out ``[A, chunk_elems]``; y_compact the stack's output for the recompute
    chunks, compact.  Updates ``residual`` in place and returns ``out`` (full layout)."""
    A = x_cur.shape[0]
    chunk_elems = x_cur[0].numel()
    assert x_cur.is_contiguous() and residual.is_contiguous() and residual.shape == x_cur.shape
    assert residual.dtype == x_cur.dtype and (y_compact is None or y_compact.is_contiguous())
    if out is None:
        out = torch.empty_like(x_cur)
    st = lib().flowcache_residual_apply(_ptr(x_cur), _ptr(y_compact), _ptr(residual), _ptr(out),
                                        _dtype_code(x_cur), A, chunk_elems, _ptr(recompute_idx),
                                        _ptr(n_recompute), _stream(stream))
    _check("flowcache_residual_apply", st)
    return out


def flowcache_attend(q: torch.Tensor, k_new: Optional[torch.Tensor], v_new: Optional[torch.Tensor],
                     k_cache: torch.Tensor, v_cache: torch.Tensor, L_c: int, L_clean: int,
                     active_off: Sequence[int], recompute_idx: torch.Tensor,
                     n_recompute: torch.Tensor, softmax_scale: float = 0.0,
                     out: Optional[torch.Tensor] = None, want_lse: bool = True,
                     mass_len: int = 0, obs_window: int = 50,
                     workspace: Optional[torch.Tensor] = None, stream=None
                     ) -> Dict[str, Optional[torch.Tensor]]:
    """q ``[A*L_c, H_q, d]`` compact; caches ``[H_k, capacity, d]`` (last dim contiguous)."""
    rows, H_q, d = q.shape
    H_k, capacity, _ = k_cache.shape
    A = len(active_off)
    dev = q.device
    assert q.is_contiguous() and k_cache.stride(2) == 1 and v_cache.stride() == k_cache.stride()
    assert rows == A * L_c
    if out is None:
        out = torch.empty_like(q)
    lse = torch.empty((H_q, rows), dtype=torch.float32, device=dev) if want_lse else None
    mass = torch.empty((H_k, mass_len), dtype=torch.float32, device=dev) if mass_len > 0 else None
    off = (ctypes.c_int32 * A)(*[int(x) for x in active_off])
    L = lib()
    if workspace is None:
        workspace = _workspace(L.flowcache_attend_workspace(A, L_c, H_q, H_k, d, mass_len, obs_window), dev)
    st = L.flowcache_attend(_ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                            k_cache.stride(0), k_cache.stride(1), capacity, _dtype_code(q), H_q, H_k,
                            d, int(L_c), int(L_clean), A, ctypes.cast(off, ctypes.c_void_p),
                            _ptr(recompute_idx), _ptr(n_recompute), float(softmax_scale), _ptr(out),
                            _ptr(lse), _ptr(mass), int(mass_len), int(obs_window), _ptr(workspace),
                            workspace.numel(), _stream(stream))
    _check("flowcache_attend", st)
    return {"out": out, "lse": lse, "mass": mass}


def flowcache_scatter_kv(k_new: torch.Tensor, v_new: torch.Tensor, k_cache: torch.Tensor,
                         v_cache: torch.Tensor, L_c: int, L_clean: int, active_off: Sequence[int],
                         recompute_idx: torch.Tensor, n_recompute: torch.Tensor, stream=None) -> None:
    """Copy the recompute chunks' rows of k_new/v_new ``[A*L_c, H_k, d]`` into their slots."""
    H_k, capacity, d = k_cache.shape
    A = len(active_off)
    assert k_new.is_contiguous() and v_new.is_contiguous() and k_cache.stride(2) == 1
    assert v_cache.stride() == k_cache.stride()
    off = (ctypes.c_int32 * A)(*[int(x) for x in active_off])
    st = lib().flowcache_scatter_kv(_ptr(k_new), _ptr(v_new), _ptr(k_cache), _ptr(v_cache),
                                    k_cache.stride(0), k_cache.stride(1), capacity,
                                    _dtype_code(k_cache), H_k, d, int(L_c), int(L_clean), A,
                                    ctypes.cast(off, ctypes.c_void_p), _ptr(recompute_idx),
                                    _ptr(n_recompute), _stream(stream))
    _check("flowcache_scatter_kv", st)


def flowcache_attention_mass(q_obs: torch.Tensor, k_cache: torch.Tensor, mass_len: int,
                             softmax_scale: float = 0.0, workspace: Optional[torch.Tensor] = None,
                             stream=None) -> torch.Tensor:
    """q_obs ``[W, H_q, d]``; returns mass ``[H_k, mass_len]`` float32."""
    W, H_q, d = q_obs.shape
    H_k = k_cache.shape[0]
    dev = q_obs.device
    assert q_obs.is_contiguous() and k_cache.stride(2) == 1
    mass = torch.empty((H_k, mass_len), dtype=torch.float32, device=dev)
    L = lib()
    if workspace is None:
        workspace = _workspace(L.flowcache_attention_mass_workspace(W, H_q, H_k, d, mass_len), dev)
    st = L.flowcache_attention_mass(_ptr(q_obs), W, _ptr(k_cache), k_cache.stride(0),
                                    k_cache.stride(1), _dtype_code(q_obs), H_q, H_k, d, int(mass_len),
                                    float(softmax_scale), _ptr(mass), _ptr(workspace),
                                    workspace.numel(), _stream(stream))
    _check("flowcache_attention_mass", st)
    return mass


def flowcache_kv_compress(k_cache: torch.Tensor, v_cache: torch.Tensor, L_k: int, budget: int,
                          mass: torch.Tensor, pool_k: int = 7, lam: float = 0.07,
                          kept_idx: Optional[torch.Tensor] = None,
                          workspace: Optional[torch.Tensor] = None, stream=None,
                          check_status: bool = False) -> torch.Tensor:
    """Compress positions [0, L_k) of the caches to ``budget`` per head, in place.  Returns
    kept_idx ``[H_k, min(budget, L_k)]`` int32 (ascending original positions).  With
    ``check_status`` the call synchronises and raises if a bounded wait of the in-place
    compaction ran out (the caches are then unspecified)."""
    H_k, capacity, d = k_cache.shape
    dev = k_cache.device
    assert k_cache.stride(2) == 1 and v_cache.stride() == k_cache.stride()
    assert mass.dtype == torch.float32 and mass.is_contiguous() and mass.shape == (H_k, L_k)
    assert L_k <= capacity
    if kept_idx is None:
        kept_idx = torch.empty((H_k, min(budget, L_k)), dtype=torch.int32, device=dev)
    L = lib()
    code = _dtype_code(k_cache)
    if workspace is None:
        workspace = _workspace(L.flowcache_kv_compress_workspace(H_k, L_k, d, budget, code), dev)
    st = L.flowcache_kv_compress(_ptr(k_cache), _ptr(v_cache), k_cache.stride(0), k_cache.stride(1),
                                 code, H_k, d, int(L_k), int(budget), _ptr(mass), int(pool_k),
                                 float(lam), _ptr(kept_idx), _ptr(workspace), workspace.numel(),
                                 _stream(stream))
    _check("flowcache_kv_compress", st)
    if check_status:
        _raise_on_compaction_status("flowcache_kv_compress", workspace, H_k, L_k, d, budget, code, 1)
    return kept_idx


def flowcache_kv_select(k_cache: torch.Tensor, L_k: int, budget: int, mass: torch.Tensor,
                        pool_k: int = 7, lam: float = 0.07, kept_idx: Optional[torch.Tensor] = None,
                        workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """Scoring and selection only: returns kept_idx ``[H_k, min(budget, L_k)]``; K is not modified."""
    H_k, capacity, d = k_cache.shape
    dev = k_cache.device
    assert k_cache.stride(2) == 1 and L_k <= capacity
    assert mass.dtype == torch.float32 and mass.is_contiguous() and mass.shape == (H_k, L_k)
    nkeep = min(budget, L_k)
    if kept_idx is None:
        kept_idx = torch.empty((H_k, nkeep), dtype=torch.int32, device=dev)
    L = lib()
    code = _dtype_code(k_cache)
    if workspace is None:
        workspace = _workspace(L.flowcache_kv_compress_workspace(H_k, L_k, d, budget, code), dev)
    st = L.flowcache_kv_select(_ptr(k_cache), k_cache.stride(0), k_cache.stride(1), code, H_k, d,
                               int(L_k), int(budget), _ptr(mass), int(pool_k), float(lam),
                               _ptr(kept_idx), _ptr(workspace), workspace.numel(), _stream(stream))
    _check("flowcache_kv_select", st)
    return kept_idx


def flowcache_kv_compact(k_cache: torch.Tensor, v_cache: torch.Tensor, L_k: int, budget: int,
                         kept_idx: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                         stream=None, check_status: bool = False) -> None:
    """Moves row ``kept_idx[h][i]`` of K and V to position i, in place."""
    H_k, capacity, d = k_cache.shape
    dev = k_cache.device
    assert k_cache.stride(2) == 1 and v_cache.stride() == k_cache.stride() and L_k <= capacity
    assert kept_idx.dtype == torch.int32 and kept_idx.is_contiguous()
    assert kept_idx.shape == (H_k, min(budget, L_k))
    L = lib()
    code = _dtype_code(k_cache)
    if workspace is None:
        workspace = _workspace(L.flowcache_kv_compress_workspace(H_k, L_k, d, budget, code), dev)
    st = L.flowcache_kv_compact(_ptr(k_cache), _ptr(v_cache), k_cache.stride(0), k_cache.stride(1),
                                code, H_k, d, int(L_k), int(budget), _ptr(kept_idx), _ptr(workspace),
                                workspace.numel(), _stream(stream))
    _check("flowcache_kv_compact", st)
    if check_status:
        _raise_on_compaction_status("flowcache_kv_compact", workspace, H_k, L_k, d, budget, code, 1)


def flowcache_kv_compress_grouped(k_cache: torch.Tensor, v_cache: torch.Tensor, L_k: int, budget: int,
                                  group: int, mass: torch.Tensor, pool_k: int = 7, lam: float = 0.07,
                                  kept_idx: Optional[torch.Tensor] = None,
                                  workspace: Optional[torch.Tensor] = None, stream=None,
                                  check_status: bool = False) -> torch.Tensor:
    """As flowcache_kv_compress, with keys scored and kept in groups of ``group`` consecutive
    tokens (``L_k`` and ``budget`` are token counts, multiples of ``group``)."""
    H_k, capacity, d = k_cache.shape
    dev = k_cache.device
    assert k_cache.stride(2) == 1 and v_cache.stride() == k_cache.stride()
    assert mass.dtype == torch.float32 and mass.is_contiguous() and mass.shape == (H_k, L_k)
    assert L_k <= capacity
    if kept_idx is None:
        kept_idx = torch.empty((H_k, min(budget, L_k)), dtype=torch.int32, device=dev)
    L = lib()
    code = _dtype_code(k_cache)
    if workspace is None:
        workspace = _workspace(L.flowcache_kv_compress_grouped_workspace(H_k, L_k, d, budget, group, code), dev)
    st = L.flowcache_kv_compress_grouped(_ptr(k_cache), _ptr(v_cache), k_cache.stride(0), k_cache.stride(1),
                                         code, H_k, d, int(L_k), int(budget), int(group), _ptr(mass),
                                         int(pool_k), float(lam), _ptr(kept_idx), _ptr(workspace),
                                         workspace.numel(), _stream(stream))
    _check("flowcache_kv_compress_grouped", st)
    if check_status:
        _raise_on_compaction_status("flowcache_kv_compress_grouped", workspace, H_k, L_k, d, budget, code, group)
    return kept_idx


# --------------------------------------------------------------------------------------
def kv_compress_status(workspace: torch.Tensor, H_k: int, L_k: int, d: int, budget: int,
                       dtype_code: int, group: int = 1) -> int:
    """Status word of the last compress call that used ``workspace`` (synchronises): 0 = ok."""
    off = lib().flowcache_kv_compress_status_offset(H_k, L_k, d, budget, group, dtype_code)
    if off == ctypes.c_size_t(-1).value:
        raise FlowCacheError("flowcache_kv_compress_status_offset", FC_INVALID_ARGUMENT)
    return int(workspace[off:off + 4].view(torch.int32).item())


def _raise_on_compaction_status(call: str, workspace: torch.Tensor, H_k: int, L_k: int, d: int,
                                budget: int, dtype_code: int, group: int) -> None:
    if budget < L_k and kv_compress_status(workspace, H_k, L_k, d, budget, dtype_code, group) != 0:
        raise FlowCacheError(call + ": a wait of the in-place compaction ran out, caches unspecified",
                             FC_HIP_ERROR)


# ---- host-side tick scheduler (flowcache_sched.h) ------------------------------------------
FC_SCHED_DONE = 5


class SchedConfig(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("n_units", "steps", "stagger", "window", "L_c", "budget", "prefix_tokens")]


class Tick(ctypes.Structure):
    _fields_ = [("tick", ctypes.c_int32), ("A", ctypes.c_int32),
                ("unit", ctypes.c_int32 * FC_MAX_ACTIVE), ("step_idx", ctypes.c_int32 * FC_MAX_ACTIVE),
                ("active_off", ctypes.c_int32 * FC_MAX_ACTIVE), ("L_clean", ctypes.c_int32),
                ("commit_unit", ctypes.c_int32), ("commit_src_off", ctypes.c_int32),
                ("commit_dst_off", ctypes.c_int32), ("merged_len", ctypes.c_int32),
                ("compress", ctypes.c_int32), ("L_clean_after", ctypes.c_int32)]

    def as_dict(self) -> Dict[str, object]:
        A = self.A
        return {"tick": self.tick, "A": A, "unit": list(self.unit[:A]), "step_idx": list(self.step_idx[:A]),
                "active_off": list(self.active_off[:A]), "L_clean": self.L_clean,
                "commit_unit": self.commit_unit, "commit_src_off": self.commit_src_off,
                "commit_dst_off": self.commit_dst_off, "merged_len": self.merged_len,
                "compress": self.compress, "L_clean_after": self.L_clean_after}


class Scheduler:
    """Iterator over the ticks of a chunk-autoregressive denoising schedule (argument
    marshalling only: the state machine lives in the library)."""

    def __init__(self, n_units: int, steps: int, stagger: int, L_c: int, budget: int,
                 window: int = 0, prefix_tokens: int = 0):
        L = lib()
        self._cfg = SchedConfig(n_units, steps, stagger, window, L_c, budget, prefix_tokens)
        self._state = ctypes.create_string_buffer(L.flowcache_sched_state_bytes())
        _check("flowcache_sched_init",
               L.flowcache_sched_init(self._state, len(self._state), ctypes.byref(self._cfg)))
        self.capacity = int(L.flowcache_sched_capacity(self._state))
        self.total_ticks = int(L.flowcache_sched_total_ticks(self._state))

    def __iter__(self):
        return self

    def __next__(self) -> Dict[str, object]:
        t = Tick()
        st = lib().flowcache_sched_next(self._state, ctypes.byref(t))
        if st == FC_SCHED_DONE:
            raise StopIteration
        _check("flowcache_sched_next", st)
        return t.as_dict()


def to_device(arr, dtype: str, device="cuda") -> torch.Tensor:
    """numpy storage array (float32, or uint16 bfloat16 bit patterns) -> device tensor."""
    import numpy as np
    if dtype == "bf16":
        assert arr.dtype == np.uint16
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def to_host(t: torch.Tensor):
    """device tensor -> numpy storage array (bfloat16 comes back as uint16 bit patterns)."""
    import numpy as np
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()
