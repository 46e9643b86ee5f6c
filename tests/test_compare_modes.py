"""Execution modes of paper_2510_19366_amd.compare_modes: host bookkeeping on the CPU,
and on the GPU the property the comparison rests on: a token's output depends only on
its own budget, so running a batch at the batch-wide maximum changes exactly the tokens
whose budget was below it (Sec. 2.4, Sec. 3.3.1)."""
import os

import numpy as np
import pytest

from paper_2510_19366_amd import compare_modes as M
from paper_2510_19366_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_mode_budgets_golden_example():
    # Sec. 2.4 worked example: budgets {2,4,5,6}; at the batch maximum every token runs 6
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLD, "mixed_k_example.txt"))
            if l.strip() and not l.startswith("#")]
    k = np.array([r[0] for r in rows], np.int32)
    own = M.mode_budgets(k, 1, ("fine", "per-token"))
    bmax = M.mode_budgets(k, 1, ("fine", "batch-max"))
    assert own.tolist() == [r[1] for r in rows]
    assert bmax.tolist() == [r[2] for r in rows]
    assert M.executed_units(bmax, 1, "fine") / M.executed_units(own, 1, "fine") == 24 / 17


def test_mode_budgets_coarse_rounds_up_to_whole_experts():
    k = np.array([1, 4, 5, 8, 9, 32], np.int32)
    S = 4
    coarse = M.mode_budgets(k, S, ("coarse", "per-token"))
    assert coarse.tolist() == [1, 1, 2, 2, 3, 8]
    assert M.executed_units(coarse, S, "coarse") == 4 * (1 + 1 + 2 + 2 + 3 + 8)
    both = M.mode_budgets(k, S, ("coarse", "batch-max"))
    assert both.tolist() == [8] * 6
    # over-serving is never below 1 and is exactly 1 for the per-token fine mode
    req = int(k.sum())
    for mode in M.MODES:
        units = M.executed_units(M.mode_budgets(k, S, mode), S, mode[0])
        assert units >= req
    assert M.executed_units(M.mode_budgets(k, S, ("fine", "per-token")), S, "fine") == req


def test_request_budgets_shape_and_range():
    req_k, k_tok = M.request_budgets(1000, 7, 8, 32, seed=1)
    assert req_k.shape == (7,) and k_tok.shape == (1000,) and k_tok.dtype == np.int32
    assert req_k.min() >= 8 and req_k.max() <= 32
    assert np.array_equal(k_tok[:142], np.full(142, req_k[0]))
    assert set(np.unique(k_tok)) <= set(req_k.tolist())


def test_fifo_batches_helper():
    assert M.fifo_batches([5, 5, 5, 20, 3], 10) == [[0, 1], [2], [3], [4]]


@pytest.mark.gpu
def test_batch_max_changes_only_under_budget_tokens():
    import torch
    from paper_2510_19366_amd import binding as B
    from gpu_util import run_layer, to_np

    a = W.make_workload("modes", dtype="bf16", d=256, n_experts=16, n_sub=1, inter_sub=128,
                        req_tokens=(6, 50), k_lo=1, k_hi=2, k_max=2, seed=21, routed_scale=1.0)
    f = W.split_workload(a, 4)                       # 64 sub-experts, k in [4, 8], k_max 8
    _, k_sub = M.request_budgets(f.T, 6, 3, 8, seed=5)
    f.k_tok[:] = k_sub
    dev = B.to_device(f)
    ws = B.alloc_workspace(dev["shape"])
    own, _, _ = run_layer(f, dev, ws)
    own = to_np(own).copy()
    _, pairs_own = B.moe_prism_status(ws)
    k_bmax = M.mode_budgets(k_sub, 4, ("fine", "batch-max"))
    dev["k_tok"] = torch.from_numpy(k_bmax).cuda()
    bmax, _, _ = run_layer(f, dev, ws)
    bmax = to_np(bmax)
    _, pairs_bmax = B.moe_prism_status(ws)
    assert pairs_own == int(k_sub.sum()) and pairs_bmax == f.T * int(k_sub.max())
    at_max = k_sub == k_sub.max()
    assert at_max.any() and (~at_max).any()
    assert np.array_equal(own[at_max].view(np.uint32), bmax[at_max].view(np.uint32))
    assert np.all(np.any(own[~at_max] != bmax[~at_max], axis=1))
    # each mode against the oracle run with that mode's budgets
    from oracle import oracle as O
    from gpu_util import max_rel
    for k_mode, got in ((k_sub, own), (k_bmax, bmax)):
        ref = O.layer(f.x, f.w_router, f.router_bias, k_mode.astype(np.int32), f.w_gate_up, f.w_down,
                      f.k_max, f.renormalize, f.routed_scale)
        assert max_rel(got, ref) <= 2e-2
