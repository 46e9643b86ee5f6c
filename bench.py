#!/usr/bin/env python3
"""Benchmark of the routed-expert forward (route -> dispatch -> grouped FFN -> combine).

One "step" is one call of moe_prism_layer over one batch of synthetic tokens that is
already resident in HBM.  Prints ONE JSON line:

  * value / ms_per_step: whole-layer routed tokens/s over exactly --steps back-to-back steps
    (wall clock between two device synchronisations); in that region only the dominant
    kernel (the grouped FFN) is bracketed by HIP events, recorded on the launch stream, which
    give the `roofline` object;
  * a second, untimed pass of max(--steps, 50) steps with events around every kernel and
    around the whole step gives per-stage medians with p10/p90 (`layer_ms`, `kernels_ms`,
    `kernels_ms_p10`, `kernels_ms_p90`), achieved GB/s and % of HBM peak per stage;
  * ragged-group figures of the batch (`groups`): largest group, m-tiles, rows-per-tile
    histogram, padding of the 256-row tiles and of the 32-row blocks the matrix cores run;
  * `roofline` names the roof that bounds the dominant kernel at the datasheet peaks (the larger
    of flops / 2.5 PFLOP/s and algorithmic bytes / 8 TB/s); `roofline_other_roof` is the same
    launch against the other roof; `ffn_traffic_probe_ms` is the fused kernel run without its
    matrix products (its memory traffic alone);
  * the FFN's utilisation against the datasheet peak and against the ceilings measured on this
    chip (profiles/microbench_mi355x.txt: matrix cores with random data, from registers / LDS);
  * the CPU oracle timed on a bounded sample of the same workload.

`roofline.traffic` (HBM bytes per launch of the dominant kernel from rocprofv3 FETCH_SIZE /
WRITE_SIZE runs) is read from profiles/hbm_traffic.txt, the summary of those runs.
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


def read_table(name):
    """Whitespace-separated rows of a summary under profiles/ ('#' starts a comment)."""
    rows = []
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return rows
    for line in open(path):
        line = line.split("#", 1)[0].strip()
        if line:
            rows.append(line.split())
    return rows


def traffic_bytes(workload, kernel):
    """HBM bytes per launch (fetch + write) of `kernel` on `workload`, or None if not measured."""
    for r in read_table("hbm_traffic.txt"):
        if len(r) >= 4 and r[0] == workload and r[1] == kernel:
            return float(r[2]) + float(r[3])
    return None


def measured_peaks():
    """Matrix-core ceilings measured by `bench.py --microbench` (TFLOP/s), or {}."""
    peaks = {}
    for r in read_table("microbench_mi355x.txt"):
        if len(r) >= 3 and r[2] == "TFLOP/s":
            peaks[r[0]] = float(r[1])
    out = {}
    lds = [v for k, v in peaks.items() if k.startswith("mfma_lds_fed") and k.endswith("_random")]
    reg = [v for k, v in peaks.items() if "registers_random" in k]
    if lds:
        out["lds_fed_random_data"] = max(lds)
    if reg:
        out["registers_random_data"] = max(reg)
    return out


def pct(v, q):
    import numpy as np
    return float(np.percentile(np.asarray(v, dtype=np.float64), q)) if len(v) else 0.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="c3_fine_128x4",
                    help="c2_mixtral_8x4 | c3_fine_128x4 | c4_decode_64x2 | c5a_s1_k8 | c5b_s4_k32 | "
                         "c3_paper_k (the c3 layer with the paper's budget generator, Sec. 4.2 Eq. 7) | "
                         "t1_olmoe_p | t1_deepseek_p (the paper's other two layer shapes, Table I)")
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
        whole = W.config("c5a_s1_k8", T=args.tokens)
        wl = W.split_workload(whole, 4)
        wl.name, wl.routed_scale = "c5b_s4_proxy_gate", 1.0
        wl.req_k, wl.k_tok = W.request_budgets(wl.T, 64, 8, 32, seed=3)
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
    # ---- timed region: HIP events around the dominant kernel only (the roofline figure)
    fused = B.ffn_path(shape) == "fused"
    dom = "ffn_fused" if fused else "ffn_gate_up"
    B.moe_prism_timing_select([dom])
    B.moe_prism_timing_enable(True)
    B.moe_prism_timing_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    kt_dom = B.moe_prism_timing_read()[dom]
    flags, pairs = B.moe_prism_status(ws)
    assert flags == 0 and pairs == wl.pairs, (flags, pairs, wl.pairs)

    # ---- distribution pass (untimed): events around every kernel and around the step
    B.moe_prism_timing_select(None)
    n_dist = max(args.steps, 50)
    per_kernel = {k: [] for k in B.KERNEL_NAMES}
    layer_samples = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(n_dist):
        e0.record()
        step()
        e1.record()
        e1.synchronize()
        layer_samples.append(e0.elapsed_time(e1))
        for k, (ms, calls) in B.moe_prism_timing_read().items():
            per_kernel[k].append(ms)          # per-step sum (the proxy gate launches some kernels twice)
    # ---- traffic probe (untimed): the fused kernel's copies, waits, barriers and stores over
    # the same tile table without the matrix products = the time its memory traffic takes alone
    probe_ms = None
    if fused and args.route == "linear":
        im = B.layer_intermediates(shape, ws)
        y_probe = torch.empty((wl.T * wl.k_max, wl.d), dtype=B.act_dtype(shape), device="cuda")
        B.moe_prism_timing_select(["ffn_traffic"])
        samples = []
        for i in range(22):
            B.moe_prism_ffn_traffic_probe(shape, dev["x"], dev["w_gate_up"], dev["w_down"],
                                          im["group_offset"], im["sorted_pair"], ws, y_probe)
            torch.cuda.synchronize()
            ms = B.moe_prism_timing_read()["ffn_traffic"][0]
            if i >= 2:
                samples.append(ms)
        probe_ms = pct(samples, 50)
        del y_probe
        B.moe_prism_timing_select(None)
    B.moe_prism_timing_enable(False)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    tokens_per_s = wl.T / (ms_per_step * 1e-3)
    # launches of the dominant kernel per step: 1, or 2 with the proxy gate on the two-kernel path
    dom_ms = kt_dom[0] / max(kt_dom[1], 1)    # average launch duration inside the timed region
    kern_med = {k: pct(v, 50) for k, v in per_kernel.items()}
    P, d, Is, E = wl.pairs, wl.d, wl.inter_sub, wl.E

    # dominant kernel: the fused FFN (6*d*Is FLOP per pair) or, on the two-kernel path, the
    # gate-up GEMM (4*d*Is per pair, 2/3 of the FFN)
    ffn_flops = 6.0 * d * Is * P
    dom_flops = ffn_flops if fused else 4.0 * d * Is * P
    dom_tflops = dom_flops / (dom_ms * 1e-3) / 1e12
    ffn_ms = sum(kern_med[k] for k in ("ffn_tiles", "ffn_gate_up", "ffn_down", "ffn_fused"))
    ffn_tflops = ffn_flops / (ffn_ms * 1e-3) / 1e12
    el = 2 if wl.dtype == "bf16" else 4
    # algorithmic bytes per stage
    stage_bytes = {
        "logits": wl.T * d * el + E * d * el + wl.T * E * 4,
        "topk": wl.T * E * 4 + 2 * wl.T * wl.k_max * 4,
        "dispatch_count": wl.T * wl.k_max * 4,
        "dispatch_place": 3 * wl.T * wl.k_max * 4,
        "combine": P * d * el + wl.T * d * el + 2 * P * 4,
        "ffn_gate_up": P * d * el + 2 * E * d * Is * el + P * Is * el,
        "ffn_down": P * Is * el + E * d * Is * el + P * d * el,
        "ffn_fused": P * d * el + 3 * E * d * Is * el + P * d * el,
    }
    stage_gbs = {k: v / (kern_med[k] * 1e-3) / 1e9 for k, v in stage_bytes.items() if kern_med.get(k, 0) > 0}

    # ragged groups of this batch, from the dispatch tables the layer left in the workspace
    cnt = B.layer_intermediates(shape, ws)["group_count"].cpu().numpy().astype(np.int64)
    tiles = []
    for n in cnt[cnt > 0]:
        tiles += [256] * int(n // 256) + ([int(n % 256)] if n % 256 else [])
    tiles = np.asarray(tiles, dtype=np.int64)
    hist_edges = [(1, 32), (33, 64), (65, 128), (129, 255), (256, 256)]
    groups = {
        "non_empty": int((cnt > 0).sum()), "of": int(E), "max_group": int(cnt.max()) if cnt.size else 0,
        "median_group": float(np.median(cnt)) if cnt.size else 0.0,
        "m_tiles": int(tiles.size),
        "rows_per_tile_hist": {f"{a}-{b}" if a != b else str(a): int(((tiles >= a) & (tiles <= b)).sum())
                               for a, b in hist_edges},
        "pad_waste_pct_256_row_tiles": 100.0 * (1.0 - P / max(256.0 * tiles.size, 1.0)),
        "pad_waste_pct_32_row_blocks": 100.0 * (1.0 - P / max(float((-(-tiles // 32) * 32).sum()), 1.0)),
    }

    # Which roof bounds the dominant kernel: the larger of its matrix-core time and its HBM time
    # at the datasheet peaks (a kernel whose arithmetic intensity is below the ridge is HBM-bound).
    dom_bytes = stage_bytes[dom]
    dom_gbs = dom_bytes / (dom_ms * 1e-3) / 1e9
    roof_mfma = {"bound": "mfma", "achieved": dom_tflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                 "frac": dom_tflops / PEAK_BF16_TFLOPS}
    roof_hbm = {"bound": "hbm", "achieved": dom_gbs, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": dom_gbs / PEAK_HBM_GBS}
    hbm_bound = dom_bytes / PEAK_HBM_GBS > dom_flops / (PEAK_BF16_TFLOPS * 1e3)   # both in 1e-9 s
    roof, other = (roof_hbm, roof_mfma) if hbm_bound else (roof_mfma, roof_hbm)

    peaks = measured_peaks()
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
                   "requests": int(len(wl.req_k)), "k_mix": "per-request", "route": args.route,
                   "ffn_path": "fused" if fused else "split"},
        "ffn_mfma_util_pct": 100.0 * ffn_tflops / PEAK_BF16_TFLOPS,
        "ffn_mfma_util_pct_measured": {k: 100.0 * ffn_tflops / v for k, v in peaks.items()},
        "ffn_tflops": ffn_tflops,
        "ffn_ms": ffn_ms,
        "roofline": {"kernel": dom, **roof, "traffic": traffic_bytes(wl.name, dom),
                     "avg_launch_ms": dom_ms, "algorithmic_bytes": dom_bytes,
                     "algorithmic_flops": dom_flops,
                     "flop_per_byte": dom_flops / dom_bytes,
                     "ridge_flop_per_byte": PEAK_BF16_TFLOPS * 1e3 / PEAK_HBM_GBS},
        "roofline_other_roof": other,
        "ffn_traffic_probe_ms": probe_ms,
        "layer_ms": {"median": pct(layer_samples, 50), "p10": pct(layer_samples, 10),
                     "p90": pct(layer_samples, 90), "samples": n_dist},
        "kernels_ms": kern_med,
        "kernels_ms_p10": {k: pct(v, 10) for k, v in per_kernel.items()},
        "kernels_ms_p90": {k: pct(v, 90) for k, v in per_kernel.items()},
        "stage_gbs": stage_gbs,
        "stage_pct_hbm": {k: 100.0 * v / PEAK_HBM_GBS for k, v in stage_gbs.items()},
        "groups": groups,
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
