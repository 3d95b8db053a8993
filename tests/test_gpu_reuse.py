"""GPU parity of the reuse-side steps: the uniform comparison policy (Fig. 2, top) and
the cached-activation store/apply around a skipped forward pass (Sec. 3.2).  Decisions and
stored values are bit-exact: both sides work in float64 and round once."""
import numpy as np
import pytest
import torch

from oracle import flowcache_oracle as O
from paper_2602_10825_amd import binding as B
from paper_2602_10825_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


@pytest.mark.parametrize("dtype,elems", [("bf16", 4096), ("f32", 1003)])
def test_uniform_policy_matches_oracle_over_a_schedule(dtype, elems):
    A, m, eps = 3, 3, 0.08
    rng = np.random.default_rng(0)
    x_prev = synth.to_storage(rng.standard_normal((A, elems)).astype(np.float32), dtype)
    acc_ref = 0.0
    acc_gpu = torch.zeros(1, dtype=torch.float64, device=DEV)
    seen = set()
    for tick in range(14):
        sig = np.array([0.03, 0.01, 0.02])
        x_cur = synth.to_storage((O.widen(x_prev) + sig[:, None] * rng.standard_normal(x_prev.shape)
                                  ).astype(np.float32), dtype)
        # chunk 2 is re-initialised at tick 8 (a new chunk entering the window)
        step = np.array([tick, tick, tick if tick < 8 else tick - 8], dtype=np.int32)
        ref = O.uniform_decide(x_cur, x_prev, step, m, eps, acc_ref)
        out = B.flowcache_uniform_decide(B.to_device(x_cur, dtype, DEV), B.to_device(x_prev, dtype, DEV),
                                         torch.from_numpy(step).to(DEV), m, eps, acc_gpu)
        mask = out["recompute_mask"].cpu().numpy().tolist()
        assert mask == ref["mask"].tolist(), tick
        n = int(out["n_recompute"].item())
        assert out["recompute_idx"].cpu().numpy()[:n].tolist() == [i for i in range(A) if mask[i]]
        got_l1 = float(out["l1rel"].item())
        assert (np.isnan(got_l1) and np.isnan(ref["l1rel"])) or np.isclose(got_l1, ref["l1rel"], rtol=1e-12)
        assert np.isclose(float(acc_gpu.item()), ref["acc"], rtol=1e-12, atol=0)
        xc = B.to_host(out["x_compact"])
        for r, c in enumerate([i for i in range(A) if mask[i]]):
            assert np.array_equal(xc[r], x_cur[c])
        acc_ref = ref["acc"]
        seen.add(tuple(mask))
        x_prev = x_cur
    # all-compute, all-reuse, and "only the new chunk computes" all occur
    assert (1, 1, 1) in seen and (0, 0, 0) in seen and (0, 0, 1) in seen


@pytest.mark.parametrize("dtype,elems,rec", [
    ("bf16", 8 * 1000, [0, 2]), ("bf16", 8 * 1000, []), ("bf16", 8 * 1000, [0, 1, 2, 3]),
    ("bf16", 1003, [1]), ("f32", 4 * 777, [3]), ("f32", 7, [0, 3]), ("bf16", 1, [0]),
])
def test_residual_apply_matches_oracle(dtype, elems, rec):
    A = 4
    rng = np.random.default_rng(1)
    mk = lambda scale: synth.to_storage((scale * rng.standard_normal((A, elems))).astype(np.float32), dtype)
    x, y, res = mk(1.0), mk(3.0), mk(0.05)
    # values whose float64 sum is NOT representable in float32: single rounding is visible
    if elems >= 4:
        x[0, :2] = synth.to_storage(np.array([1.0, 256.0], np.float32), dtype)
        res[0, :2] = synth.to_storage(np.array([2.0 ** -20, 2.0 ** -9], np.float32), dtype)
    R = len(rec)
    y_c = np.ascontiguousarray(y[:max(R, 1)])
    idx = torch.tensor(rec + [-1] * (A - R), dtype=torch.int32, device=DEV)
    n = torch.tensor([R], dtype=torch.int32, device=DEV)
    ref_res, ref_out = O.residual_apply(x, y_c, res, rec)
    res_gpu = B.to_device(res, dtype, DEV)
    out = B.flowcache_residual_apply(B.to_device(x, dtype, DEV), B.to_device(y_c, dtype, DEV),
                                     res_gpu, idx, n)
    torch.cuda.synchronize()
    assert np.array_equal(B.to_host(res_gpu), ref_res)
    assert np.array_equal(B.to_host(out), ref_out)
    # in place: the output may overwrite the input
    x_gpu = B.to_device(x, dtype, DEV)
    res_gpu = B.to_device(res, dtype, DEV)
    B.flowcache_residual_apply(x_gpu, B.to_device(y_c, dtype, DEV), res_gpu, idx, n, out=x_gpu)
    torch.cuda.synchronize()
    assert np.array_equal(B.to_host(x_gpu), ref_out) and np.array_equal(B.to_host(res_gpu), ref_res)


def test_decide_then_residual_round_trip_over_ticks():
    """Chunks alternate between recompute and reuse; a stand-in 'forward pass' y = 2x + 1 runs on
    the gathered chunks only.  The GPU chain and the oracle chain stay bit-identical."""
    wl = synth.Workload("t", "bf16", 2, 2, 64, 3, 40, 0, 1, warmup_m=2, eps=0.1)
    rng = np.random.default_rng(2)
    x_prev = synth.to_storage(rng.standard_normal((wl.A, wl.chunk_elems)).astype(np.float32), "bf16")
    acc_ref = np.zeros(wl.A)
    acc_gpu = torch.zeros(wl.A, dtype=torch.float64, device=DEV)
    res_ref = np.zeros_like(x_prev)
    res_gpu = B.to_device(res_ref, "bf16", DEV)
    reused = 0
    for tick in range(10):
        sig = np.array([0.04, 0.015, 0.3])
        x_cur = synth.to_storage((O.widen(x_prev) + sig[:, None] * rng.standard_normal(x_prev.shape)
                                  ).astype(np.float32), "bf16")
        step = np.full(wl.A, tick, dtype=np.int32)
        ref = O.chunk_decide(x_cur, x_prev, step, wl.warmup_m, wl.eps, acc_ref)
        xg = B.to_device(x_cur, "bf16", DEV)
        dec = B.flowcache_chunk_decide(xg, B.to_device(x_prev, "bf16", DEV),
                                       torch.from_numpy(step).to(DEV), wl.warmup_m, wl.eps, acc_gpu)
        rec = ref["recompute_idx"].tolist()
        assert dec["recompute_mask"].cpu().numpy().tolist() == ref["mask"].tolist()
        y_gpu = (dec["x_compact"].float() * 2 + 1).to(torch.bfloat16)      # harness-side stand-in
        y_ref = B.to_host(y_gpu)
        out = B.flowcache_residual_apply(xg, y_gpu, res_gpu, dec["recompute_idx"], dec["n_recompute"])
        res_ref, out_ref = O.residual_apply(x_cur, y_ref, res_ref, rec)
        assert np.array_equal(B.to_host(out), out_ref), tick
        assert np.array_equal(B.to_host(res_gpu), res_ref), tick
        reused += wl.A - len(rec)
        acc_ref, x_prev = ref["acc"], x_cur
    assert reused > 0
