"""The whole step recorded once into a HIP graph and replayed: every call of the library only
enqueues kernels on the caller's stream (no allocation, no synchronisation, no host read), so
a capture must replay to the same bits as the eager run -- on every replay, with other work
and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2602_10825_amd import binding as B
from paper_2602_10825_amd import synth

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_captured_step_replays_to_the_eager_bits():
    wl = synth.MID_BF16
    d = synth.decide_inputs(wl, seed=0, sigmas=[0.003, 0.5, 0.02])
    d["step_idx"][-1] = 0                                   # the newest chunk is in warm-up: recomputed
    a = synth.attend_inputs(wl, seed=0)
    L = B.lib()
    xc, xp = B.to_device(d["x_cur"], "bf16", DEV), B.to_device(d["x_prev"], "bf16", DEV)
    step = torch.from_numpy(d["step_idx"]).to(DEV)
    acc0 = torch.zeros(wl.A, dtype=torch.float64, device=DEV)
    q = B.to_device(a["q"], "bf16", DEV)
    kn, vn = B.to_device(a["k_new"], "bf16", DEV), B.to_device(a["v_new"], "bf16", DEV)
    k0, v0 = B.to_device(a["k_cache"], "bf16", DEV), B.to_device(a["v_cache"], "bf16", DEV)
    mass_len = wl.L_clean + wl.L_c
    code = B.FC_BF16
    ws = {
        "dec": torch.empty(L.flowcache_chunk_decide_workspace(wl.A, wl.chunk_elems), dtype=torch.uint8, device=DEV),
        "att": torch.empty(L.flowcache_attend_workspace(wl.A, wl.L_c, wl.H_q, wl.H_k, wl.d, mass_len, wl.obs_window),
                           dtype=torch.uint8, device=DEV),
        "cmp": torch.empty(L.flowcache_kv_compress_workspace(wl.H_k, mass_len, wl.d, wl.budget, code),
                           dtype=torch.uint8, device=DEV),
    }
    # static buffers of the captured step
    acc = acc0.clone()
    k, v = k0.clone(), v0.clone()
    xcomp = torch.empty_like(xc)
    out = torch.empty_like(q)
    kept = torch.empty((wl.H_k, wl.budget), dtype=torch.int32, device=DEV)
    res_cache = torch.zeros_like(xc)
    full = torch.empty_like(xc)
    holder = {}

    def step_fn():
        acc.copy_(acc0); k.copy_(k0); v.copy_(v0)           # compression and the accumulator are destructive
        dec = B.flowcache_chunk_decide(xc, xp, step, wl.warmup_m, wl.eps, acc, x_compact=xcomp,
                                       workspace=ws["dec"])
        att = B.flowcache_attend(q, kn, vn, k, v, wl.L_c, wl.L_clean, a["active_off"], dec["recompute_idx"],
                                 dec["n_recompute"], out=out, mass_len=mass_len, obs_window=wl.obs_window,
                                 workspace=ws["att"])
        B.flowcache_residual_apply(xc, out.view(wl.A, -1), res_cache, dec["recompute_idx"],
                                   dec["n_recompute"], out=full)
        B.flowcache_kv_compress(k, v, mass_len, wl.budget, att["mass"], wl.pool_k, wl.lam, kept_idx=kept,
                                workspace=ws["cmp"])
        holder.update(dec=dec, att=att)

    def snapshot():
        torch.cuda.synchronize()
        return [t.clone() for t in (holder["dec"]["recompute_mask"], holder["dec"]["recompute_idx"], acc, xcomp,
                                    out, holder["att"]["lse"], holder["att"]["mass"], res_cache, full, kept, k, v)]

    step_fn()                                               # eager reference (also warms everything up)
    ref = snapshot()
    assert 0 < int(holder["dec"]["n_recompute"].item()) < wl.A
    res_cache.zero_()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step_fn()
    for replay in range(3):
        # unrelated eager work and a synchronisation between replays
        junk = torch.randn(1 << 20, device=DEV).sum().item()
        assert np.isfinite(junk)
        for t in (out, xcomp, full, kept):
            t.zero_()
        res_cache.zero_()
        g.replay()
        got = snapshot()
        n_rows = int(holder["dec"]["n_recompute"].item()) * wl.L_c
        for i, (x, y) in enumerate(zip(got, ref)):
            if i == 5:      # the row log-sum-exp is only written for the recomputed blocks
                x, y = x[:, :n_rows], y[:, :n_rows]
            if x.is_floating_point():
                assert torch.equal(torch.nan_to_num(x.float()), torch.nan_to_num(y.float())), (replay, i)
            else:
                assert torch.equal(x, y), (replay, i)
