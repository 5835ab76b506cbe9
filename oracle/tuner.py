"""Oracle of the run-time parameter search and of the analytical model (section 6 of the
paper: "Performance-Resource Analytical Modeling" and "Heuristic-based Cross Iteration
Optimization").  TEST INFRASTRUCTURE ONLY; shares no code with the library.

The search is a heuristic, so this is not a closed form but the paper's steps, in its order
and notation (ps = neighbour-partition size, dist = interleaving distance, wpb = warps per
block), written out plainly:

  1. all three knobs start at 1;
  2. ps is increased while the latency keeps falling; the first increase that raises the
     latency ends this step and ps goes back to the last good value;
  3. the same for dist;
  4. the same for wpb;
  5. "retreat": ps is lowered to its next smaller value and the increase of wpb is started
     again; this repeats until a trial of this step is slower than the third-lowest latency
     seen so far (or ps cannot be lowered further);
  6. every trial is recorded in a lookup table; the configuration with the lowest latency wins.

Readings where the text is silent: "increase" doubles the knob (the search spaces are
1..32, 1..16, 1..16 and the paper reports about ten trials); an increase that would leave the
range ends its step; "restart the increase of wpb" restarts it from 1; a configuration that
is already in the table is not measured twice.  The model's constraints (section 6, constraint on
SMEM) bound the search space: a configuration that violates them is never measured and never
enters the table; where the search would try one, it counts as slower than anything measured
(an upward step onto it does not pay; a retreat trial on it ends the search).
"""
from __future__ import annotations

from typing import Callable, Dict, List, Tuple

Knobs = Tuple[int, int, int]          # (ps, dist, wpb)


def model(n_local: int, n_remote: int, ps: int, dist: int, wpb: int, dim: int,
          num_units: int, smem_limit: int) -> Dict[str, float]:
    """Equations (1)-(3): workload per warp, shared-memory bytes per block, warps, blocks,
    blocks per processing unit, and the feasibility of the shared-memory constraint."""
    int_s = float_s = 4
    wpw = 2 * ps * dim * dist
    smem = ps * wpb * int_s + 2 * wpb * dim * float_s
    num_warps = -(-max(n_local, n_remote) // dist)
    num_blocks = -(-num_warps // wpb)
    return {"wpw": wpw, "smem": smem, "num_warps": num_warps, "num_blocks": num_blocks,
            "blocks_per_unit": num_blocks / num_units, "feasible": smem <= smem_limit}


def search(latency: Callable[[Knobs], float], ps_max: int = 32, dist_max: int = 16, wpb_max: int = 16,
           feasible: Callable[[Knobs], bool] = None):
    """Runs the search against a latency function.  Returns (best knobs, table) where table is
    the list of (knobs, latency) in the order the trials were made; best is None when not even the
    starting point is feasible."""
    table: List[Tuple[Knobs, float]] = []
    seen: Dict[Knobs, float] = {}

    def measure(k: Knobs) -> float:
        if feasible is not None and not feasible(k):
            return float("inf")
        if k not in seen:
            seen[k] = latency(k)
            table.append((k, seen[k]))
        return seen[k]

    limits = (ps_max, dist_max, wpb_max)
    cur = [1, 1, 1]
    best_lat = measure(tuple(cur))
    for axis in (0, 1, 2):                      # steps 2, 3, 4
        while cur[axis] * 2 <= limits[axis]:
            trial = list(cur)
            trial[axis] *= 2
            lat = measure(tuple(trial))
            if lat >= best_lat:
                break
            cur, best_lat = trial, lat
    def third_lowest() -> float:
        lats = sorted(v for _, v in table)
        return lats[min(2, len(lats) - 1)] if lats else float("inf")

    ps, dist = cur[0], cur[1]
    stop = False
    while ps > 1 and not stop:                  # step 5
        ps //= 2
        wpb = 1
        lat = measure((ps, dist, wpb))
        if lat > third_lowest():
            break
        while wpb * 2 <= wpb_max:
            lat2 = measure((ps, dist, wpb * 2))
            if lat2 > third_lowest():
                stop = True
                break
            if lat2 >= lat:
                break
            wpb, lat = wpb * 2, lat2
    best = min(table, key=lambda kv: kv[1])[0] if table else None  # step 6
    return best, table
