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


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--requests", type=int, default=64)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--table", action="store_true", help="also print T(n, k)")
    args = ap.parse_args()

    import torch
    from paper_2510_19366_amd import binding as B
    from paper_2510_19366_amd import workloads as W

    assert torch.cuda.is_available(), "compare_modes needs a GPU"
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
