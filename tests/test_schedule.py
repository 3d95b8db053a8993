"""The host-side tick scheduler of the library against the schedule oracle (tick by tick,
every field) and against closed forms of the schedule of Sec. 3.1, Eq. (3) and the cache
phases of App. C.1.  No GPU involved: the scheduler is host code behind the C ABI."""
import ctypes

import pytest

from oracle import schedule_oracle as S
from paper_2602_10825_amd import binding as B

CASES = [
    # MAGI-1-like: 10 chunks, 64 steps, window 4 (stagger T/l = 16), budget 5 chunks
    dict(n_units=10, steps=64, stagger=16, L_c=9360, budget=5 * 9360),
    # SkyReels-V2-like: blocks inside a chunk, 50 steps per block, a block starts every 5 steps,
    # the overlap frames of the previous chunk are the clean prefix
    dict(n_units=16, steps=50, stagger=5, L_c=1560, budget=40000, prefix_tokens=17 * 1560 // 4),
    # the 255-tick rollout: 16 chunks, 30 steps, 2 active, budget 4 chunks
    dict(n_units=16, steps=30, stagger=15, L_c=10200, budget=4 * 10200),
    dict(n_units=1, steps=7, stagger=7, L_c=5, budget=0),
    dict(n_units=5, steps=4, stagger=4, L_c=3, budget=7, window=3, prefix_tokens=7),
    dict(n_units=6, steps=9, stagger=2, L_c=8, budget=20, window=16),
]


@pytest.mark.parametrize("cfg", CASES)
def test_scheduler_matches_oracle_tick_by_tick(cfg):
    sch = B.Scheduler(**cfg)
    ticks = list(sch)
    ref = list(S.schedule(**cfg))
    assert len(ticks) == len(ref) == sch.total_ticks
    for got, want in zip(ticks, ref):
        if want["commit_unit"] < 0:                       # commit fields are unspecified without one
            for k in ("commit_src_off", "commit_dst_off", "merged_len", "compress"):
                got[k] = want[k]
        assert got == want, got["tick"]
    with pytest.raises(StopIteration):
        next(sch)


@pytest.mark.parametrize("cfg", CASES)
def test_schedule_closed_forms(cfg):
    n, T, sg, L_c, bud = cfg["n_units"], cfg["steps"], cfg["stagger"], cfg["L_c"], cfg["budget"]
    P0 = cfg.get("prefix_tokens", 0)
    window = cfg.get("window", 0) or -(-T // sg)
    for ticks in (list(B.Scheduler(**cfg)), list(S.schedule(**cfg))):
        assert len(ticks) == (n - 1) * sg + T
        seen = {}
        for t in ticks:
            assert 1 <= t["A"] <= window
            assert t["unit"] == sorted(t["unit"])                  # causal order
            assert len(set(t["active_off"])) == t["A"]             # slots never shared
            assert all(bud + L_c <= o <= bud + L_c + (window - 1) * L_c for o in t["active_off"])
            for u, s in zip(t["unit"], t["step_idx"]):
                assert seen.get(u, -1) == s - 1                    # steps 0, 1, 2, ... in order
                seen[u] = s
                assert u * sg <= t["tick"] < u * sg + T            # Eq. (3), 0-based units
            assert t["L_clean"] <= bud
        assert seen == {u: T - 1 for u in range(n)}                # every unit takes exactly T steps
        commits = [t for t in ticks if t["commit_unit"] >= 0]
        assert [t["commit_unit"] for t in commits] == list(range(n))
        assert [t["tick"] for t in commits] == [u * sg + T - 1 for u in range(n)]
        for j, t in enumerate(commits):
            # filling: length grows by one unit per commit until one more would not fit
            L = P0
            for _ in range(j):
                L = L + L_c if L + L_c <= bud else bud
            assert t["L_clean"] == L == t["commit_dst_off"]
            assert t["merged_len"] == L + L_c
            assert t["compress"] == (1 if L + L_c > bud else 0)
            assert t["L_clean_after"] == (bud if L + L_c > bud else L + L_c)
        # once the compression phase has started it never ends
        flags = [t["compress"] for t in commits]
        assert flags == sorted(flags)


def test_magi_window_matches_eq3_ranges():
    T, l, k = 64, 4, 10
    ticks = list(B.Scheduler(n_units=k, steps=T, stagger=T // l, L_c=8, budget=64))
    for i in range(1, k + 1):                                       # units counted from 1, as in Eq. (3)
        mine = [t["tick"] for t in ticks if (i - 1) in t["unit"]]
        assert mine[0] == (i - 1) * T // l and mine[-1] == (i + l - 1) * T // l - 1
    # in the steady state exactly l chunks are denoised together, at l different noise levels
    mid = ticks[len(ticks) // 2]
    assert mid["A"] == l and len(set(mid["step_idx"])) == l


def test_scheduler_rejects_bad_configurations():
    L = B.lib()
    buf = ctypes.create_string_buffer(L.flowcache_sched_state_bytes())
    ok = dict(n_units=4, steps=8, stagger=4, window=0, L_c=16, budget=64, prefix_tokens=0)

    def init(**kw):
        c = B.SchedConfig(**{**ok, **kw})
        return L.flowcache_sched_init(buf, len(buf), ctypes.byref(c))

    assert init() == 0
    for bad in (dict(n_units=0), dict(steps=0), dict(stagger=0), dict(stagger=9), dict(L_c=0),
                dict(budget=-1), dict(prefix_tokens=65), dict(window=1), dict(window=17)):
        assert init(**bad) == 1, bad
    assert L.flowcache_sched_init(None, len(buf), ctypes.byref(B.SchedConfig(**ok))) == 1
    assert L.flowcache_sched_init(buf, 4, ctypes.byref(B.SchedConfig(**ok))) == 1
    blank = ctypes.create_string_buffer(len(buf))
    assert L.flowcache_sched_next(blank, ctypes.byref(B.Tick())) == 1      # never initialised
    assert L.flowcache_sched_capacity(blank) == 0
    assert B.Scheduler(**{k: v for k, v in ok.items() if k != "window"}).capacity == 64 + 16 + 2 * 16
