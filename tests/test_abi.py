"""The C-ABI library loads, exports every function the header declares, and rejects bad
arguments before touching the GPU.  CPU only: no compute call is made here."""
import ctypes
import os
import re

import pytest

from paper_2602_10825_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = sorted(os.path.join(ROOT, "include", f) for f in os.listdir(os.path.join(ROOT, "include"))
                 if f.endswith(".h"))

INVALID, UNSUPPORTED, WS_SMALL = 1, 2, 3
P = ctypes.c_void_p(0x10000)       # never dereferenced: validation fails first
NULL = None


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_10825_amd.build import build
        build(verbose=False)
    return binding.lib()


def declared_functions():
    text = "\n".join(open(h).read() for h in HEADERS)
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(flowcache_\w+)\s*\(", text)))


def test_every_declared_function_is_exported(L):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_status_strings_and_version(L):
    assert binding.status_string(0) == "ok"
    assert "invalid" in binding.status_string(INVALID)
    assert "workspace" in binding.status_string(WS_SMALL)
    assert binding.status_string(99) == "unknown status"
    assert L.flowcache_version() >= 100


def decide(L, **kw):
    a = dict(x_cur=P, x_prev=P, dtype=1, A=2, chunk_elems=1024, step_idx=P, m=4, eps=0.1, acc=P,
             l1rel=P, mask=P, idx=P, n=P, xc=P, ws=P, wsb=1 << 20, stream=NULL)
    a.update(kw)
    return L.flowcache_chunk_decide(a["x_cur"], a["x_prev"], a["dtype"], a["A"], a["chunk_elems"],
                                    a["step_idx"], a["m"], a["eps"], a["acc"], a["l1rel"], a["mask"],
                                    a["idx"], a["n"], a["xc"], a["ws"], a["wsb"], a["stream"])


def test_chunk_decide_rejects_bad_arguments(L):
    assert decide(L, x_cur=NULL) == INVALID
    assert decide(L, acc=NULL) == INVALID
    assert decide(L, A=0) == INVALID
    assert decide(L, A=17) == INVALID
    assert decide(L, chunk_elems=0) == INVALID
    assert decide(L, m=-1) == INVALID
    assert decide(L, eps=-0.5) == INVALID
    assert decide(L, eps=float("nan")) == INVALID
    assert decide(L, eps=float("inf")) == INVALID
    assert decide(L, dtype=7) == INVALID
    assert decide(L, wsb=8) == WS_SMALL
    assert L.flowcache_chunk_decide_workspace(2, 1024) >= 2 * 2 * 8
    assert L.flowcache_chunk_decide_workspace(0, 1024) == 0


def attend(L, **kw):
    off = (ctypes.c_int32 * 2)(512, 640)
    a = dict(q=P, k_new=P, v_new=P, kc=P, vc=P, hs=768 * 64, ts=64, cap=768, dtype=0, H_q=4, H_k=1,
             d=64, L_c=128, L_clean=512, A=2, off=off, idx=P, n=P, scale=0.0, out=P, lse=P, mass=NULL,
             mass_len=0, W=50, ws=P, wsb=1 << 24, stream=NULL)
    a.update(kw)
    return L.flowcache_attend(a["q"], a["k_new"], a["v_new"], a["kc"], a["vc"], a["hs"], a["ts"],
                              a["cap"], a["dtype"], a["H_q"], a["H_k"], a["d"], a["L_c"], a["L_clean"],
                              a["A"], ctypes.cast(a["off"], ctypes.c_void_p), a["idx"], a["n"],
                              a["scale"], a["out"], a["lse"], a["mass"], a["mass_len"], a["W"],
                              a["ws"], a["wsb"], a["stream"])


def test_attend_rejects_bad_arguments(L):
    assert attend(L, q=NULL) == INVALID
    assert attend(L, k_new=NULL) == INVALID                    # k_new without v_new
    assert attend(L, H_q=3, H_k=2) == INVALID                  # H_q % H_k
    assert attend(L, d=96) == UNSUPPORTED
    assert attend(L, ts=32) == INVALID                         # token stride < d
    assert attend(L, hs=100) == INVALID                        # head stride < capacity rows
    assert attend(L, ts=66, hs=768 * 66) == UNSUPPORTED        # rows not 16-byte aligned
    big = (1 << 24) + 8
    assert attend(L, ts=big, hs=768 * big) == UNSUPPORTED      # stride beyond the 32-bit tile offsets
    assert attend(L, off=(ctypes.c_int32 * 2)(512, 700)) == INVALID   # slot past capacity
    assert attend(L, off=(ctypes.c_int32 * 2)(512, 600)) == INVALID   # overlapping slots
    assert attend(L, off=(ctypes.c_int32 * 2)(400, 640)) == INVALID   # slot inside clean region
    assert attend(L, scale=-1.0) == INVALID
    assert attend(L, A=0) == INVALID
    assert attend(L, mass=P, mass_len=0) == INVALID
    assert attend(L, mass=P, mass_len=9999) == INVALID
    assert attend(L, mass=P, mass_len=512, wsb=16) == WS_SMALL
    assert attend(L, q=ctypes.c_void_p(0x10004)) == UNSUPPORTED
    assert L.flowcache_attend_workspace(2, 128, 4, 1, 64, 512, 50) > \
        L.flowcache_attend_workspace(2, 128, 4, 1, 64, 0, 50)


def compress(L, **kw):
    a = dict(kc=P, vc=P, hs=512 * 64, ts=64, dtype=0, H_k=1, d=64, L_k=512, B=256, mass=P, k=7,
             lam=0.07, kept=P, ws=P, wsb=1 << 26, stream=NULL)
    a.update(kw)
    return L.flowcache_kv_compress(a["kc"], a["vc"], a["hs"], a["ts"], a["dtype"], a["H_k"], a["d"],
                                   a["L_k"], a["B"], a["mass"], a["k"], a["lam"], a["kept"], a["ws"],
                                   a["wsb"], a["stream"])


def test_kv_compress_rejects_bad_arguments(L):
    assert compress(L, kc=NULL) == INVALID
    assert compress(L, mass=NULL) == INVALID
    assert compress(L, k=4) == INVALID                         # even pool width
    assert compress(L, k=0) == INVALID
    assert compress(L, lam=1.5) == INVALID
    assert compress(L, lam=float("nan")) == INVALID
    assert compress(L, B=0) == INVALID
    assert compress(L, L_k=0) == INVALID
    assert compress(L, d=80) == UNSUPPORTED
    assert compress(L, wsb=64) == WS_SMALL
    need = L.flowcache_kv_compress_workspace(1, 512, 64, 256, 0)
    assert need >= 512 * (16 + 8 + 8)
    assert L.flowcache_kv_compress_workspace(1, 512, 96, 256, 0) == 0


def test_attention_mass_rejects_bad_arguments(L):
    def mass(**kw):
        a = dict(q=P, W=50, kc=P, hs=512 * 64, ts=64, dtype=1, H_q=4, H_k=2, d=64, n=512, scale=0.0,
                 mass=P, ws=P, wsb=1 << 24, stream=NULL)
        a.update(kw)
        return L.flowcache_attention_mass(a["q"], a["W"], a["kc"], a["hs"], a["ts"], a["dtype"],
                                          a["H_q"], a["H_k"], a["d"], a["n"], a["scale"], a["mass"],
                                          a["ws"], a["wsb"], a["stream"])
    assert mass(W=0) == INVALID
    assert mass(mass=NULL) == INVALID
    assert mass(H_q=3) == INVALID
    assert mass(d=32) == UNSUPPORTED
    assert mass(wsb=8) == WS_SMALL
    assert mass(n=0) == INVALID


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "missing.so"))
    with pytest.raises(ImportError):
        binding.lib()


def test_uniform_decide_and_residual_apply_reject_bad_arguments(L):
    def uni(**kw):
        a = dict(x_cur=P, x_prev=P, dtype=1, A=2, chunk_elems=1024, step_idx=P, m=4, eps=0.1, acc=P,
                 l1rel=P, mask=P, idx=P, n=P, xc=P, ws=P, wsb=1 << 20, stream=NULL)
        a.update(kw)
        return L.flowcache_uniform_decide(a["x_cur"], a["x_prev"], a["dtype"], a["A"], a["chunk_elems"],
                                          a["step_idx"], a["m"], a["eps"], a["acc"], a["l1rel"], a["mask"],
                                          a["idx"], a["n"], a["xc"], a["ws"], a["wsb"], a["stream"])

    assert uni(acc=NULL) == INVALID and uni(A=0) == INVALID and uni(eps=-1.0) == INVALID
    assert uni(eps=float("nan")) == INVALID and uni(dtype=5) == INVALID and uni(wsb=8) == WS_SMALL

    def res(**kw):
        a = dict(x=P, y=P, r=P, o=P, dtype=1, A=2, ce=1024, idx=P, n=P, stream=NULL)
        a.update(kw)
        return L.flowcache_residual_apply(a["x"], a["y"], a["r"], a["o"], a["dtype"], a["A"], a["ce"],
                                          a["idx"], a["n"], a["stream"])

    assert res(x=NULL) == INVALID and res(r=NULL) == INVALID and res(o=NULL) == INVALID
    assert res(idx=NULL) == INVALID and res(n=NULL) == INVALID
    assert res(A=0) == INVALID and res(A=17) == INVALID and res(ce=0) == INVALID and res(dtype=2) == INVALID


def test_grouped_compress_rejects_bad_arguments(L):
    def grp(**kw):
        a = dict(kc=P, vc=P, hs=1024 * 128, ts=128, dtype=1, H=2, d=128, L_k=1000, budget=500, group=50,
                 mass=P, pool=7, lam=0.07, kept=P, ws=P, wsb=1 << 26, stream=NULL)
        a.update(kw)
        return L.flowcache_kv_compress_grouped(a["kc"], a["vc"], a["hs"], a["ts"], a["dtype"], a["H"], a["d"],
                                               a["L_k"], a["budget"], a["group"], a["mass"], a["pool"],
                                               a["lam"], a["kept"], a["ws"], a["wsb"], a["stream"])

    assert grp(group=0) == INVALID and grp(group=30) == INVALID        # 1000 % 30 != 0
    assert grp(budget=510) == INVALID and grp(pool=4) == INVALID and grp(lam=1.5) == INVALID
    assert grp(mass=NULL) == INVALID and grp(d=96) == UNSUPPORTED and grp(wsb=64) == WS_SMALL
    assert L.flowcache_kv_compress_grouped_workspace(2, 1000, 128, 500, 30, 1) == 0
    assert L.flowcache_kv_compress_grouped_workspace(2, 1000, 128, 500, 1, 1) == \
        L.flowcache_kv_compress_workspace(2, 1000, 128, 500, 1)


def test_kv_select_and_compact_reject_bad_arguments(L):
    def sel(**kw):
        a = dict(kc=P, hs=1024 * 128, ts=128, dtype=1, H=2, d=128, L_k=1000, budget=500, mass=P, pool=7,
                 lam=0.07, kept=P, ws=P, wsb=1 << 26, stream=NULL)
        a.update(kw)
        return L.flowcache_kv_select(a["kc"], a["hs"], a["ts"], a["dtype"], a["H"], a["d"], a["L_k"],
                                     a["budget"], a["mass"], a["pool"], a["lam"], a["kept"], a["ws"],
                                     a["wsb"], a["stream"])

    def cpt(**kw):
        a = dict(kc=P, vc=P, hs=1024 * 128, ts=128, dtype=1, H=2, d=128, L_k=1000, budget=500, kept=P,
                 ws=P, wsb=1 << 26, stream=NULL)
        a.update(kw)
        return L.flowcache_kv_compact(a["kc"], a["vc"], a["hs"], a["ts"], a["dtype"], a["H"], a["d"],
                                      a["L_k"], a["budget"], a["kept"], a["ws"], a["wsb"], a["stream"])

    assert sel(kc=NULL) == INVALID and sel(mass=NULL) == INVALID and sel(kept=NULL) == INVALID
    assert sel(pool=2) == INVALID and sel(lam=-0.1) == INVALID and sel(budget=0) == INVALID
    assert sel(d=96) == UNSUPPORTED and sel(wsb=64) == WS_SMALL and sel(ts=64) == INVALID
    assert cpt(kc=NULL) == INVALID and cpt(vc=NULL) == INVALID and cpt(kept=NULL) == INVALID
    assert cpt(L_k=0) == INVALID and cpt(budget=0) == INVALID
    assert cpt(d=96) == UNSUPPORTED and cpt(wsb=64) == WS_SMALL and cpt(hs=100) == INVALID
