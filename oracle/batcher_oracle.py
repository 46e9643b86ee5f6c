"""Plain reference of the offline quality-tiered batcher (Sec. 3.3.2, temporal separation).

TEST INFRASTRUCTURE ONLY: tests compare the library's planner (host C++) with this, request
by request.  Written from the description, one step at a time:

  1. the waiting queue is sorted by (k, arrival): lower budgets first, FIFO inside a tier;
  2. tiers are scanned in ascending k and batches are filled under the token budget M;
  3. when a tier ends with an under-filled (residual) batch, it is either dispatched at its
     budget k or promoted to the next tier's budget k_next and merged with it, whichever has
     the higher token throughput by the profiled table T(n, k)  (Eq. 5):
         (n_cur + n_next) / T(n_cur + n_next, k_next)  >=  n_cur / T(n_cur, k)
     where n_next is what the next tier contributes under the remaining budget.

Readings where the text is silent: a batch is filled strictly in queue order (no skipping
ahead to a smaller request that would still fit); n_next is the longest FIFO prefix of the
next tier that fits in M - n_cur (if nothing fits the residual is dispatched); a request
longer than M forms a batch of its own; T(n, k) between grid points is bilinear in (n, k) and
constant outside the grid; the comparison is evaluated in binary64 as
(n_cur + n_next) * T(n_cur, k) >= n_cur * T(n_cur + n_next, k_next).
"""
from __future__ import annotations

import bisect
from typing import List, Sequence, Tuple


def time_table(n_grid: Sequence[int], k_grid: Sequence[int], ms, n: float, k: float) -> float:
    """T(n, k): bilinear interpolation on the profiled grid, clamped at its border."""
    def locate(grid, v):
        if v <= grid[0]:
            return 0, 0, 0.0
        if v >= grid[-1]:
            return len(grid) - 1, len(grid) - 1, 0.0
        hi = bisect.bisect_right(grid, v)
        lo = hi - 1
        return lo, hi, (float(v) - float(grid[lo])) / (float(grid[hi]) - float(grid[lo]))
    i0, i1, fn = locate(list(n_grid), n)
    j0, j1, fk = locate(list(k_grid), k)
    a = float(ms[i0][j0]) + (float(ms[i0][j1]) - float(ms[i0][j0])) * fk
    b = float(ms[i1][j0]) + (float(ms[i1][j1]) - float(ms[i1][j0])) * fk
    return a + (b - a) * fn


def plan(arrival: Sequence[float], n_tokens: Sequence[int], k_qos: Sequence[int], M: int,
         n_grid, k_grid, ms) -> Tuple[List[List[int]], List[int]]:
    """Returns (batches, batch_k): request indices per batch in dispatch order and the budget
    each batch runs at (the largest budget among its requests)."""
    order = sorted(range(len(k_qos)), key=lambda i: (k_qos[i], arrival[i], i))
    tiers: List[Tuple[int, List[int]]] = []
    for i in order:
        if tiers and tiers[-1][0] == k_qos[i]:
            tiers[-1][1].append(i)
        else:
            tiers.append((k_qos[i], [i]))
    batches: List[List[int]] = []
    batch_k: List[int] = []
    cur: List[int] = []
    cur_n, cur_k = 0, 0

    def dispatch():
        nonlocal cur, cur_n
        if cur:
            batches.append(cur)
            batch_k.append(cur_k)
        cur, cur_n = [], 0

    for k, reqs in tiers:
        if cur:                                     # residual batch of a lower tier
            n_next = 0
            for i in reqs:
                if cur_n + n_next + n_tokens[i] > M:
                    break
                n_next += n_tokens[i]
            merge = False
            if n_next > 0:
                t_cur = time_table(n_grid, k_grid, ms, cur_n, cur_k)
                t_new = time_table(n_grid, k_grid, ms, cur_n + n_next, k)
                merge = float(cur_n + n_next) * t_cur >= float(cur_n) * t_new
            if merge:
                cur_k = k                           # promoted; the tier's requests join below
            else:
                dispatch()
        for i in reqs:
            if cur and cur_n + n_tokens[i] > M:
                dispatch()
            cur.append(i)
            cur_n += n_tokens[i]
            cur_k = k
    dispatch()
    return batches, batch_k
