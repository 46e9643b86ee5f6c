"""Offline quality-tiered batcher (Sec. 3.3.2, Eq. 5): the reference in oracle/ pinned to
closed forms and a hand-worked example, and the library's host planner compared with it
request by request.  No GPU involved."""
import numpy as np
import pytest

from oracle import batcher_oracle as BO
from paper_2510_19366_amd import binding as B

# T(n, k) of the fine layout measured on MI355X (ms per layer): the tracked summary of
# `compare_modes --table` under profiles/
from paper_2510_19366_amd.compare_modes import read_time_table

N_GRID, K_GRID, MEASURED = read_time_table()


def test_measured_table_is_a_time_table():
    assert N_GRID == sorted(N_GRID) and K_GRID == sorted(K_GRID) and len(MEASURED) == len(N_GRID)
    ms = np.asarray(MEASURED)
    assert ms.shape == (len(N_GRID), len(K_GRID)) and (ms > 0).all()
    assert (np.diff(ms, axis=0) > 0).all()              # more tokens never cost less


def table(fn):
    return [[fn(n, k) for k in K_GRID] for n in N_GRID]


def requests(seed, R=200, k_lo=8, k_hi=32, n_lo=16, n_hi=600):
    rng = np.random.default_rng(seed)
    return (np.sort(rng.random(R) * 100.0), rng.integers(n_lo, n_hi + 1, R).astype(np.int32),
            rng.integers(k_lo, k_hi + 1, R).astype(np.int32))


def check_invariants(batches, batch_k, arrival, n, k, M):
    flat = [i for b in batches for i in b]
    assert sorted(flat) == list(range(len(k)))                       # every request exactly once
    keys = [(k[i], arrival[i], i) for i in flat]
    assert keys == sorted(keys)                                      # queue order is never broken
    for b, bk in zip(batches, batch_k):
        assert bk == max(k[i] for i in b)                            # runs at its largest budget
        assert sum(n[i] for i in b) <= M or len(b) == 1              # token budget


def test_time_table_interpolation():
    ms = table(lambda n, k: 3.0 + 0.5 * n + 2.0 * k)                 # bilinear: reproduced exactly
    for n, k in [(256, 8), (700, 11), (16384, 32), (5000, 20.5)]:
        assert BO.time_table(N_GRID, K_GRID, ms, n, k) == pytest.approx(3.0 + 0.5 * n + 2.0 * k, rel=1e-12)
    assert BO.time_table(N_GRID, K_GRID, ms, 10, 2) == ms[0][0]       # constant outside the grid
    assert BO.time_table(N_GRID, K_GRID, ms, 10 ** 6, 99) == ms[-1][-1]


def test_hand_worked_merge_decision():
    # T = 1 + n*k/1000 ms.  Tier k=8: one request of 1000 tokens (M = 4096 -> residual).
    # Next tier k=16 contributes 2000 tokens.  Alone: 1000 / (1 + 8) = 111.1 tokens/ms;
    # merged: 3000 / (1 + 48) = 61.2 tokens/ms  -> dispatch the residual alone.
    ms = [[1 + n * k / 1000 for k in (8, 16)] for n in (1000, 3000)]
    arr, n, k = [0.0, 1.0], [1000, 2000], [8, 16]
    assert BO.plan(arr, n, k, 4096, [1000, 3000], [8, 16], ms) == ([[0], [1]], [8, 16])
    # with a large fixed cost the same queue merges: T = 100 + n*k/1000:
    # alone 1000 / 108 = 9.26 tokens/ms, merged 3000 / 148 = 20.3 tokens/ms
    ms = [[100 + n * k / 1000 for k in (8, 16)] for n in (1000, 3000)]
    assert BO.plan(arr, n, k, 4096, [1000, 3000], [8, 16], ms) == ([[0, 1]], [16])


def test_closed_forms():
    arr, n, k = requests(1)
    M = 4096
    # time independent of n and k (pure fixed cost): a fuller batch is always better -> always
    # merge: the plan is the greedy fill of the sorted queue, tiers ignored
    b, bk = BO.plan(arr, n, k, M, N_GRID, K_GRID, table(lambda nn, kk: 1.0))
    order = sorted(range(len(k)), key=lambda i: (k[i], arr[i], i))
    greedy, cur, tot = [], [], 0
    for i in order:
        if cur and tot + n[i] > M:
            greedy.append(cur)
            cur, tot = [], 0
        cur.append(i)
        tot += n[i]
    greedy.append(cur)
    assert b == greedy
    # time proportional to pairs n*k, no fixed cost: a promoted batch is always slower per token
    # -> never merge: no batch mixes budgets
    b, bk = BO.plan(arr, n, k, M, N_GRID, K_GRID, table(lambda nn, kk: 1e-5 * nn * kk))
    assert all(len({k[i] for i in batch}) == 1 for batch in b)
    check_invariants(b, bk, arr, n, k, M)


@pytest.mark.parametrize("seed", range(6))
def test_library_planner_equals_reference(seed):
    arr, n, k = requests(seed, R=300 if seed else 1)
    if seed == 3:
        n[::17] = 9000                                               # requests longer than M
    if seed == 4:
        arr[:] = 0.0                                                 # ties in arrival -> index order
    M = 4096
    for ms in (MEASURED, table(lambda nn, kk: 0.3 + 1e-5 * nn * kk), table(lambda nn, kk: 0.001 * nn)):
        ms = np.asarray(ms, np.float32)                              # the table's type at the boundary
        ref = BO.plan(arr, n, k, M, N_GRID, K_GRID, ms)
        got = B.moe_prism_plan_batches(arr, n, k, M, N_GRID, K_GRID, ms)
        assert got == ref
        check_invariants(got[0], got[1], arr, n, k, M)


def test_library_planner_arguments():
    assert B.moe_prism_plan_batches([], [], [], 100, N_GRID, K_GRID, MEASURED) == ([], [])
    with pytest.raises(B.MoePrismError):
        B.moe_prism_plan_batches([0.0], [0], [8], 100, N_GRID, K_GRID, MEASURED)      # empty request
    with pytest.raises(B.MoePrismError):
        B.moe_prism_plan_batches([0.0], [5], [8], 100, [4, 4], [8, 16], [[1, 1], [1, 1]])  # grid not ascending
