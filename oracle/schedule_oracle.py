"""CPU oracle for the tick schedule and cache phases.  TEST INFRASTRUCTURE ONLY.

Written from the definition, tick by tick, with no state carried except the clean length:
unit ``i`` (0-based) is being denoised at tick ``t`` iff ``i*stagger <= t < i*stagger + steps``
(Sec. 3.1, Eq. (3): with a window of ``l`` units and ``stagger = T/l`` this is the range
``[(i-1)T/l, (i+l-1)T/l]`` for units counted from 1), and a unit that takes its last step is
committed to the clean cache: appended while ``L_clean + L_c <= budget`` (cache-filling phase),
otherwise merged and compressed to ``budget`` rows (compression phase) -- App. C.1.
Pins: closed forms in ``tests/test_schedule.py``.  Shares no code with the library.
"""
from __future__ import annotations

from typing import Dict, Iterator, List


def schedule(n_units: int, steps: int, stagger: int, L_c: int, budget: int, window: int = 0,
             prefix_tokens: int = 0) -> Iterator[Dict[str, object]]:
    need = -(-steps // stagger)
    window = window or need
    ring_base = budget + L_c
    L_clean = prefix_tokens
    total = (n_units - 1) * stagger + steps
    for t in range(total):
        active = [i for i in range(n_units) if i * stagger <= t < i * stagger + steps]
        tick = {"tick": t, "A": len(active), "unit": active,
                "step_idx": [t - i * stagger for i in active],
                "active_off": [ring_base + (i % window) * L_c for i in active],
                "L_clean": L_clean, "commit_unit": -1, "commit_src_off": 0, "commit_dst_off": 0,
                "merged_len": 0, "compress": 0, "L_clean_after": L_clean}
        done = [i for i in active if t - i * stagger == steps - 1]
        if done:
            (i,) = done                              # stagger >= 1: at most one unit finishes per tick
            merged = L_clean + L_c
            tick.update(commit_unit=i, commit_src_off=ring_base + (i % window) * L_c,
                        commit_dst_off=L_clean, merged_len=merged,
                        compress=1 if merged > budget else 0)
            L_clean = budget if merged > budget else merged
            tick["L_clean_after"] = L_clean
        yield tick
