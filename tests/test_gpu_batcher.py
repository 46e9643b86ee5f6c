"""The offline quality-tiered batcher (Sec. 3.3.2, Eq. 5) driving the layer on the GPU: the plan
of moe_prism_plan_batches is executed batch by batch through moe_prism_layer, once with every
token at its request's budget and once with the whole batch at its largest budget (how the
paper's runtime executes a batch, Sec. 3.3.1); every token's output is checked against the
oracle run with the same budgets, and the executed work and measured time of the two modes are
compared with what the plan's accounting says."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2510_19366_amd import binding as B
from paper_2510_19366_amd import compare_modes as M
from paper_2510_19366_amd import workloads as W
from gpu_util import max_rel, row_rel, to_np

pytestmark = pytest.mark.gpu


def test_planned_batches_through_the_layer():
    rng = np.random.default_rng(5)
    R, Mtok = 40, 1024
    n_tok = rng.integers(16, 201, R).astype(np.int32)
    req_k = rng.integers(4, 17, R).astype(np.int32)
    arrival = np.sort(rng.random(R) * 50.0)
    req_off = np.zeros(R + 1, np.int64)
    req_off[1:] = np.cumsum(n_tok)
    T_all = int(req_off[-1])
    # a narrow-sub-expert layer (fused FFN kernel), 64 sub-experts, budgets up to 16
    wl = W.make_workload("plan", dtype="bf16", d=256, n_experts=16, n_sub=4, inter_sub=64,
                         req_tokens=[T_all], req_k=[16], k_max=16, seed=9, bias_std=0.7, w_std=0.05)
    # a time table with a fixed cost and a per-pair cost: mixes of merge and dispatch decisions
    n_grid, k_grid = [64, 256, 1024], [4, 8, 16]
    ms = [[0.05 + 2e-5 * n * k for k in k_grid] for n in n_grid]
    batches, batch_k = B.moe_prism_plan_batches(arrival, n_tok, req_k, Mtok, n_grid, k_grid, ms)
    assert sorted(i for b in batches for i in b) == list(range(R))
    assert any(len({req_k[i] for i in b}) > 1 for b in batches)      # some batch mixes budgets

    dev = B.to_device(wl)
    ws = B.alloc_workspace(B.make_shape(Mtok + 256, wl.d, wl.n_experts, wl.n_sub, wl.inter_sub, wl.k_max, "bf16"))
    total = {"per-token": [0.0, 0], "batch-max": [0.0, 0]}
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for b, bk in zip(batches, batch_k):
        rows = np.concatenate([np.arange(req_off[i], req_off[i + 1]) for i in b])
        k_own = np.concatenate([np.full(n_tok[i], req_k[i], np.int32) for i in b])
        assert bk == k_own.max() and (len(rows) <= Mtok or len(b) == 1)
        shape = B.make_shape(len(rows), wl.d, wl.n_experts, wl.n_sub, wl.inter_sub, wl.k_max, "bf16")
        x_dev = dev["x"][torch.from_numpy(rows).cuda()].contiguous()
        for mode, k in (("per-token", k_own), ("batch-max", np.full_like(k_own, bk))):
            k_dev = torch.from_numpy(k).cuda()
            B.moe_prism_layer(shape, x_dev, dev["w_router"], dev["router_bias"], k_dev,
                              dev["w_gate_up"], dev["w_down"], ws)               # warm-up
            e0.record()
            out = B.moe_prism_layer(shape, x_dev, dev["w_router"], dev["router_bias"], k_dev,
                                    dev["w_gate_up"], dev["w_down"], ws)
            e1.record()
            e1.synchronize()
            flags, pairs = B.moe_prism_status(ws)
            assert flags == 0 and pairs == int(k.sum())
            total[mode][0] += e0.elapsed_time(e1)
            total[mode][1] += pairs
            ref = O.layer(wl.x[rows], wl.w_router, wl.router_bias, k, wl.w_gate_up, wl.w_down, wl.k_max,
                          wl.renormalize, wl.routed_scale)
            got = to_np(out)
            assert max_rel(got, ref) <= 2e-2 and row_rel(got, ref) <= 4e-2, (mode, b)
    requested = int((n_tok.astype(np.int64) * req_k).sum())
    assert total["per-token"][1] == requested                         # no over-serving
    assert total["batch-max"][1] == sum(int(bk) * int(sum(n_tok[i] for i in b))
                                        for b, bk in zip(batches, batch_k)) > requested
    print(f"planned batches: {len(batches)}, requested units {requested}; per-token "
          f"{total['per-token'][0]:.3f} ms, batch-max {total['batch-max'][0]:.3f} ms "
          f"({total['batch-max'][1] / requested:.3f}x units)")
