#!/usr/bin/env python3
"""What per-token budgets buy: the same layer, the same tokens and the same per-request
budgets executed four ways, plus the latency table T(n, k) of the scheduler's cost model.

Modes (all through moe_prism_layer; only k_tok and the expert layout differ):
  fine / per-token   S sub-experts per expert, every token runs exactly its request's k
                     (this library's normal mode)
  fine / batch-max   the whole batch runs at the largest budget present: how the paper's
                     runtime executes a mixed batch (Sec. 3.3.1, Sec. 3.4.2)
  coarse / per-token undivided experts (S = 1), each token runs ceil(k / S) experts: the
                     finest budget the original model offers (Sec. 2.3)
  coarse / batch-max both restrictions together (a stock top-k MoE runtime)
"Executed" counts sub-expert-sized units of FFN work (an undivided expert is S of them);
over-serving = executed / requested (Sec. 2.4).  The layer is the fine-grained 128-expert
shape with a repeated-row gate (Sec. 3.2.2), so all four modes route consistently.

T(n, k): layer time for n tokens that all carry budget k, the quantity the offline
scheduler's merge test looks up (Sec. 3.3.2, Eq. 5).

Usage: python -m paper_2510_19366_amd.compare_modes [--tokens 16384] [--steps 20] [--table]
Prints markdown.  Needs the GPU library; there is no CPU path.
"""
import argparse
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


from paper_2510_19366_amd.workloads import request_budgets  # noqa: E402  (re-exported for callers)


def mode_budgets(k_sub, S, mode):
    """k_tok handed to the layer in `mode`, in units of that layout's experts."""
    layout, policy = mode
    k = k_sub if layout == "fine" else (k_sub + S - 1) // S
    if policy == "batch-max":
        k = np.full_like(k, k.max())
    return k.astype(np.int32)


def executed_units(k_mode, S, layout):
    return int(k_mode.sum()) * (1 if layout == "fine" else S)


MODES = [("fine", "per-token"), ("fine", "batch-max"), ("coarse", "per-token"), ("coarse", "batch-max")]


def time_layer(B, torch, dev, ws, out, k_tok_dev, steps, warmup=3):
    shape = dev["shape"]

    def step():
        B.moe_prism_layer(shape, dev["x"], dev["w_router"], dev["router_bias"], k_tok_dev,
                          dev["w_gate_up"], dev["w_down"], ws, out=out)
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    flags, pairs = B.moe_prism_status(ws)
    assert flags == 0
    return ms, pairs


def read_time_table(path=None):
    """(n_grid, k_grid, ms) from the T(n, k) summary under profiles/ (rows: n, then one time per k)."""
    path = path or os.path.join(ROOT, "profiles", "time_table_fine_128x4.txt")
    n_grid, k_grid, ms = [], None, []
    for line in open(path):
        line = line.split("#", 1)[0].split()
        if not line:
            continue
        if line[0] == "k":
            k_grid = [int(v) for v in line[1:]]
        else:
            n_grid.append(int(line[0]))
            ms.append([float(v) for v in line[1:]])
    return n_grid, k_grid, ms


def fifo_batches(n_tokens, M):
    """Arrival-order batching under the token budget M (a request longer than M runs alone)."""
    batches, cur, tot = [], [], 0
    for i, n in enumerate(n_tokens):
        if cur and tot + n > M:
            batches.append(cur)
            cur, tot = [], 0
        cur.append(i)
        tot += int(n)
    if cur:
        batches.append(cur)
    return batches


def run_batches(B, torch, dev, x_all, req_off, req_k, batches, policy, T_cap):
    """Execute every batch through moe_prism_layer; returns (total ms from HIP events around
    the whole sequence, pairs executed).  policy: "per-token" (every token its request's
    budget) or "batch-max" (the batch's largest budget for all)."""
    fine = dev["wl"]
    shape_of = {}
    ws = B.alloc_workspace(B.make_shape(T_cap, fine.d, fine.n_experts, fine.n_sub, fine.inter_sub,
                                        fine.k_max, fine.dtype, fine.renormalize, fine.routed_scale))
    out = torch.empty((T_cap, fine.d), dtype=torch.bfloat16, device="cuda")
    staged = []
    for b in batches:                      # inputs are staged in HBM before the clock starts
        rows = np.concatenate([np.arange(req_off[i], req_off[i + 1]) for i in b])
        k = np.concatenate([np.full(req_off[i + 1] - req_off[i], req_k[i], np.int32) for i in b])
        if policy == "batch-max":
            k[:] = k.max()
        n = len(rows)
        if n not in shape_of:
            shape_of[n] = B.make_shape(n, fine.d, fine.n_experts, fine.n_sub, fine.inter_sub, fine.k_max,
                                       fine.dtype, fine.renormalize, fine.routed_scale)
        staged.append((shape_of[n], x_all[torch.from_numpy(rows).cuda()].contiguous(),
                       torch.from_numpy(k).cuda(), int(k.sum())))
    def once():
        for shape, x, k, _ in staged:
            B.moe_prism_layer(shape, x, dev["w_router"], dev["router_bias"], k, dev["w_gate_up"],
                              dev["w_down"], ws, out=out[:shape.T])
    once()                                 # warm-up
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    once()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1), sum(s[3] for s in staged)


def batching_experiment(B, torch, W, R, M, seed=7):
    """Sec. 3.3.2 on the GPU: R requests (prompt lengths uniform in [64, 512], budgets uniform in
    [8, 32]) batched in arrival order or by the quality-tiered planner (moe_prism_plan_batches,
    fed with the measured T(n, k) of profiles/), and every batch executed at its maximum budget
    (the paper's runtime) or with per-token budgets."""
    rng = np.random.default_rng(seed)
    n_tok = rng.integers(64, 513, R).astype(np.int32)
    req_k = rng.integers(8, 33, R).astype(np.int32)
    arrival = np.sort(rng.random(R) * 1000.0)
    req_off = np.zeros(R + 1, np.int64)
    req_off[1:] = np.cumsum(n_tok)
    coarse = W.config("c5a_s1_k8", T=16384)
    fine = W.split_workload(coarse, 4)
    dev = B.to_device(fine)
    dev["wl"] = fine
    # token rows: the workload's 16384 rows reused cyclically (the values do not matter for time)
    idx = torch.arange(int(req_off[-1]), device="cuda") % fine.T
    x_all = dev["x"][idx].contiguous()
    n_grid, k_grid, ms = read_time_table()
    tiered, batch_k = B.moe_prism_plan_batches(arrival, n_tok, req_k, M, n_grid, k_grid, ms)
    fifo = fifo_batches(n_tok, M)
    requested = int((n_tok.astype(np.int64) * req_k).sum())
    print(f"### Offline batching executed: {R} requests, {int(req_off[-1])} tokens, token budget M = {M}, "
          f"requested units {requested}\n")
    print("| batching | execution | batches | units executed | over-serving | measured total ms | tokens/s |")
    print("|---|---|---|---|---|---|---|")
    for bname, batches in (("arrival order (FIFO)", fifo), ("quality-tiered + Eq. 5 merge test", tiered)):
        for policy in ("batch-max", "per-token"):
            t_ms, units = run_batches(B, torch, dev, x_all, req_off, req_k, batches, policy, M + 512)
            print(f"| {bname} | {policy} | {len(batches)} | {units} | {units / requested:.3f} | {t_ms:.1f} | "
                  f"{int(req_off[-1]) / t_ms * 1e3:.3g} |", flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--requests", type=int, default=64)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--table", action="store_true", help="also print T(n, k)")
    ap.add_argument("--batching", type=int, default=0, metavar="R",
                    help="instead: plan R requests with the offline batcher and execute the batches "
                         "(Sec. 3.3.2), four combinations of batching policy and execution mode")
    ap.add_argument("--token-budget", type=int, default=16384, help="M of the batching experiment")
    args = ap.parse_args()

    import torch
    from paper_2510_19366_amd import binding as B
    from paper_2510_19366_amd import workloads as W

    assert torch.cuda.is_available(), "compare_modes needs a GPU"
    if args.batching:
        batching_experiment(B, torch, W, args.batching, args.token_budget)
        return
    S = 4
    coarse = W.config("c5a_s1_k8", T=args.tokens)     # 128 undivided experts, Is = 768, k_max 8
    fine = W.split_workload(coarse, S)                 # 512 sub-experts, Is = 192, k_max 32
    _, k_sub = request_budgets(args.tokens, args.requests, 8, 32, seed=3)
    devs = {"coarse": B.to_device(coarse), "fine": B.to_device(fine)}
    wss = {k: B.alloc_workspace(v["shape"]) for k, v in devs.items()}
    out = torch.empty((args.tokens, coarse.d), dtype=torch.bfloat16, device="cuda")
    requested = int(k_sub.sum())

    print(f"### Execution modes, T = {args.tokens}, {args.requests} requests, k per request uniform in "
          f"[8, 32] sub-experts (requested units: {requested})\n")
    print("| layout / policy | units executed | over-serving | ms per layer | tokens/s |")
    print("|---|---|---|---|---|")
    for mode in MODES:
        layout = mode[0]
        k_mode = mode_budgets(k_sub, S, mode)
        k_dev = torch.from_numpy(k_mode).cuda()
        ms, pairs = time_layer(B, torch, devs[layout], wss[layout], out, k_dev, args.steps)
        units = executed_units(k_mode, S, layout)
        assert pairs == int(k_mode.sum())
        print(f"| {layout} / {mode[1]} | {units} | {units / requested:.3f} | {ms:.3f} | "
              f"{args.tokens / ms * 1e3:.3g} |", flush=True)

    if args.table:
        ks = [8, 16, 24, 32]
        ns = [n for n in (256, 1024, 4096, 16384) if n <= args.tokens]
        print(f"\n### T(n, k): ms per layer, fine layout, all n tokens at budget k\n")
        print("| n \\ k | " + " | ".join(str(k) for k in ks) + " |")
        print("|---|" + "---|" * len(ks))
        dev_f = devs["fine"]
        for n in ns:
            sub = dict(dev_f)
            sub["x"] = dev_f["x"][:n].contiguous()
            sub["shape"] = B.make_shape(n, fine.d, fine.n_experts, fine.n_sub, fine.inter_sub,
                                        fine.k_max, fine.dtype, fine.renormalize, fine.routed_scale)
            ws_n = B.alloc_workspace(sub["shape"])
            out_n = torch.empty((n, fine.d), dtype=torch.bfloat16, device="cuda")
            row = []
            for k in ks:
                k_dev = torch.full((n,), k, dtype=torch.int32, device="cuda")
                ms, _ = time_layer(B, torch, sub, ws_n, out_n, k_dev, args.steps)
                row.append(f"{ms:.3f}")
            print(f"| {n} | " + " | ".join(row) + " |", flush=True)


if __name__ == "__main__":
    main()
