#!/usr/bin/env python3
"""Benchmark of the routed-expert forward (route -> dispatch -> grouped FFN -> combine).

One "step" is one call of moe_prism_layer over one batch of synthetic tokens that is
already resident in HBM.  Prints ONE JSON line: whole-layer routed tokens/s, the
roofline of the dominant kernel (gate-up GEMM) from HIP events recorded around it inside the
timed region, the other kernels' times from up to 10 further steps with events around every
kernel (outside the timed region, so that the throughput figure carries two event records per
step instead of eighteen), and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0          # MI355X HBM3E

# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# (see profiles/); None until measured for that workload.
TRAFFIC_BYTES = {"c3_fine_128x4": 2.27e9,   # gate-up kernel: 2.143 GB fetched + 0.122 GB written
                 "c2_mixtral_8x4": 4.51e9,  # 4.361 + 0.152 (weights of a group reach several XCDs' L2)
                 "c4_decode_64x2": 1.70e9}  # 1.608 + 0.093


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3_fine_128x4",
                    help="c2_mixtral_8x4 | c3_fine_128x4 | c4_decode_64x2 | c5a_s1_k8 | c5b_s4_k32")
    ap.add_argument("--tokens", type=int, default=None, help="token count for the c5 sweep")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=15.0)
    ap.add_argument("--route", default="linear", choices=["linear", "proxy"],
                    help="linear: the expanded linear gate (default, the headline); proxy: the "
                         "training-free proxy gate on the 128-expert layer split in 4 (m = 8 "
                         "original experts, r = 4 gate neurons), per-request budgets in [8, 32]")
    ap.add_argument("--graph", action="store_true",
                    help="additionally time the same steps replayed from one captured HIP graph "
                         "(reported as graph_ms_per_step; the headline numbers stay the eager ones)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 1 GiB device copy 5 times (known traffic, for scaling "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--microbench", action="store_true",
                    help="run the machine-peak microbenchmarks instead (matrix cores from registers "
                         "and from LDS, LDS reads, operand streams, HBM copy) and print them as one "
                         "JSON line")
    args = ap.parse_args()

    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (no collectives, no sharding); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_19366_amd import binding as B
    from paper_2510_19366_amd import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.microbench:
        rows = B.moe_prism_microbench()
        print(json.dumps({"microbench": [{"name": n, "value": v, "unit": u, "shader_mhz": m}
                                         for n, v, u, m in rows]}))
        return
    if args.route == "proxy":
        from paper_2510_19366_amd.compare_modes import request_budgets
        whole = W.config("c5a_s1_k8", T=args.tokens)
        wl = W.split_workload(whole, 4)
        wl.name, wl.routed_scale = "c5b_s4_proxy_gate", 1.0
        wl.req_k, wl.k_tok = request_budgets(wl.T, 64, 8, 32, seed=3)
        pg = W.make_proxy_gate(whole, wl, m=8, r=4, seed=6)
        del whole
    else:
        wl = W.config(args.workload, T=args.tokens) if args.workload.startswith("c5") else W.config(args.workload)
    dev = B.to_device(wl)
    shape = dev["shape"]
    ws = B.alloc_workspace(shape)
    out = torch.empty((wl.T, wl.d), dtype=B.act_dtype(shape), device="cuda")

    if args.route == "proxy":
        pdev = B.proxy_to_device(pg, wl.dtype)

        def step():
            B.moe_prism_layer_proxy(shape, dev["x"], pdev, dev["k_tok"], dev["w_gate_up"],
                                    dev["w_down"], ws, out=out)
    else:
        def step():
            B.moe_prism_layer(shape, dev["x"], dev["w_router"], dev["router_bias"], dev["k_tok"],
                              dev["w_gate_up"], dev["w_down"], ws, out=out)

    if args.copy_calibration:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # timed region: HIP events around the dominant kernel only (the roofline figure); the other
    # kernels' durations come from a short pass of their own afterwards, outside the timing
    dom = "ffn_fused" if B.ffn_path(shape) == "fused" else "ffn_gate_up"
    B.moe_prism_timing_select([dom])
    B.moe_prism_timing_enable(True)
    B.moe_prism_timing_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kt = B.moe_prism_timing_read()
    B.moe_prism_timing_select(None)
    for _ in range(min(args.steps, 10)):
        step()
    torch.cuda.synchronize()
    kt_all = B.moe_prism_timing_read()
    B.moe_prism_timing_enable(False)
    kt = {k: (kt[k] if k == dom else v) for k, v in kt_all.items()}
    flags, pairs = B.moe_prism_status(ws)
    assert flags == 0 and pairs == wl.pairs, (flags, pairs, wl.pairs)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = wl.T / (ms_per_step * 1e-3)
    # average launch duration; with the proxy gate the route stage launches the logits, top-k,
    # dispatch, tile and gate-up kernels a second time on small shapes, so there the figures
    # are per-step sums
    if args.route == "proxy":
        kern_ms = {k: v[0] / (args.steps if k == dom else min(args.steps, 10))
                   for k, v in kt.items()}
    else:
        kern_ms = {k: (v[0] / max(v[1], 1)) for k, v in kt.items()}
    P, d, Is, E = wl.pairs, wl.d, wl.inter_sub, wl.E

    # dominant kernel: the gate-up GEMM (2/3 of the FFN FLOPs); algorithmic FLOPs = 4*d*Is per pair
    ffn_flops = 6.0 * d * Is * P
    gu_flops = ffn_flops if dom == "ffn_fused" else 4.0 * d * Is * P
    gu_tflops = gu_flops / (kern_ms[dom] * 1e-3) / 1e12
    ffn_ms = kern_ms["ffn_gate_up"] + kern_ms["ffn_down"] + kern_ms["ffn_tiles"] + kern_ms["ffn_fused"]
    ffn_tflops = ffn_flops / (ffn_ms * 1e-3) / 1e12
    el = 2 if wl.dtype == "bf16" else 4
    stage_bytes = {
        "logits": wl.T * d * el + E * d * el + wl.T * E * 4,
        "topk": wl.T * E * 4 + 2 * wl.T * wl.k_max * 4,
        "combine": P * d * el + wl.T * d * el + 2 * P * 4,
        "ffn_down": P * Is * el + E * d * Is * el + P * d * el,
    }
    res = {
        "metric": "routed tokens/sec (whole layer, mixed per-request k, 1 GPU); grouped-FFN MFMA util in ffn_mfma_util_pct",
        "value": tokens_per_s,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": wl.dtype,
        "data": "synthetic",
        "config": {"workload": wl.name, "T": wl.T, "d": d, "n_experts": wl.n_experts,
                   "n_sub": wl.n_sub, "inter_sub": Is, "k_max": wl.k_max, "pairs": P,
                   "requests": int(len(wl.req_k)), "k_mix": "per-request", "route": args.route},
        "ffn_mfma_util_pct": 100.0 * ffn_tflops / PEAK_BF16_TFLOPS,
        "ffn_tflops": ffn_tflops,
        "ffn_ms": ffn_ms,
        "roofline": {"kernel": dom, "bound": "mfma", "achieved": gu_tflops,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": gu_tflops / PEAK_BF16_TFLOPS,
                     "traffic": TRAFFIC_BYTES.get(wl.name)},
        "kernels_ms": kern_ms,
        "stage_gbs": {k: v / (kern_ms[k] * 1e-3) / 1e9 for k, v in stage_bytes.items()
                      if kern_ms.get(k, 0) > 0},
    }

    if args.graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            step()
        torch.cuda.synchronize()
        for _ in range(args.warmup):
            g.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            g.replay()
        torch.cuda.synchronize()
        res["graph_ms_per_step"] = (time.perf_counter() - t0) * 1e3 / args.steps

    if not args.no_cpu_baseline and args.route == "linear":
        from oracle import oracle as O
        x32, wr32 = wl.x, wl.w_router
        rng = np.random.default_rng(0)
        n, spent, done = 4, 0.0, 0
        perm = rng.permutation(wl.T)
        # grow the sample until ~cpu-seconds of oracle work has been spent
        while done < wl.T and spent < args.cpu_seconds:
            n = min(n, wl.T - done)
            tok = np.sort(perm[done:done + n]).astype(np.int32)
            c0 = time.perf_counter()
            O.layer_tokens(tok, x32, wr32, wl.router_bias, wl.k_tok, wl.w_gate_up, wl.w_down,
                           wl.k_max, wl.renormalize, wl.routed_scale)
            dt = time.perf_counter() - c0
            spent += dt
            done += n
            rate = n / max(dt, 1e-9)
            n = int(max(4, min(rate * (args.cpu_seconds - spent) * 0.9, 4 * n)))
        res["cpu_baseline"] = {"value": done / spent, "unit": "tokens/s", "cores": O.n_threads(),
                               "kind": "oracle",
                               "sample": f"{done} of {wl.T} tokens of {wl.name} drawn at random, "
                                         f"whole layer per token (fp64 plain C, OpenMP), {spent:.1f} s"}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
