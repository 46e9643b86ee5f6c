"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by
element on the same seeded inputs.  Routing ids, logits and dispatch tables are
compared bit for bit; routing weights to 1e-5; FFN rows and layer outputs to
2e-2 (bf16) / 1e-4 (fp32) of the largest reference magnitude."""
import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2510_19366_amd import binding as B
from paper_2510_19366_amd import workloads as W
from gpu_util import max_rel, row_rel, run_layer, run_stages, to_np

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-4, "bf16": 2e-2}


def check_against_oracle(wl, r, ref):
    assert np.array_equal(r["logits"].view(np.uint32), ref["logits"].view(np.uint32)), "logits bits"
    assert np.array_equal(r["ids"], ref["ids"]), "top-k ids"
    np.testing.assert_allclose(r["w"], ref["w"], rtol=1e-5, atol=1e-7)
    for k in ("cnt", "off", "sorted_pair", "slot_of_pair"):
        assert np.array_equal(r[k], ref[k]), k
    assert r["pairs"] == int(np.clip(wl.k_tok, 0, wl.k_max).sum()) == int(ref["off"][-1])
    tol = TOL[wl.dtype]
    assert max_rel(r["y"], ref["y"]) <= tol
    assert max_rel(r["out"], ref["out"]) <= tol


def test_config1_tiny_f32_stage_by_stage():
    wl = W.config("c1_tiny_f32")
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)
    assert r["flags"] == 0
    out, _, _ = run_layer(wl, r["dev"], r["ws"])
    assert max_rel(to_np(out), ref["out"]) <= 1e-4
    assert np.array_equal(to_np(out), r["out"])          # fused entry point == staged calls


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", [
    # T, d, N, S, Is, k_max: several m-tiles per group, ragged tails, n-tile and K tails
    dict(T=700, d=256, N=6, S=4, Is=96, k_max=9),
    dict(T=333, d=128, N=3, S=2, Is=32, k_max=6),
    dict(T=1, d=64, N=2, S=2, Is=64, k_max=4),
    dict(T=1500, d=192, N=40, S=4, Is=160, k_max=20),
    # long enough K for the global->LDS ring in both GEMMs; 96-neuron and 128-neuron tiles,
    # a 192-column down tile (d = 320 pads less with 192), partial last n-tiles
    dict(T=900, d=320, N=4, S=2, Is=224, k_max=5),
    dict(T=2100, d=512, N=3, S=4, Is=352, k_max=7),
    dict(T=600, d=256, N=2, S=1, Is=1024, k_max=2),
    dict(T=500, d=128, N=4, S=2, Is=128, k_max=4),
    # K of 12 or more stages: the two-group schedule, with 192-wide tiles (the cases above reach
    # it with 256-wide tiles, and the in-step ring schedule with both widths)
    dict(T=800, d=384, N=4, S=2, Is=192, k_max=4),
    dict(T=600, d=192, N=2, S=2, Is=416, k_max=3),
])
def test_small_cases_full_oracle(dtype, case):
    rng = np.random.default_rng(case["T"])
    k = rng.integers(0, case["k_max"] + 1, size=case["T"]).astype(np.int32)
    wl = W.make_workload("small", dtype=dtype, d=case["d"], n_experts=case["N"], n_sub=case["S"],
                         inter_sub=case["Is"], req_tokens=[1] * case["T"], req_k=k,
                         k_max=case["k_max"], seed=case["T"], bias_std=1.0, w_std=0.05)
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)
    out, _, _ = run_layer(wl, r["dev"], r["ws"])
    assert np.array_equal(to_np(out), r["out"])


@pytest.mark.parametrize("path", ["fused", "split"])
@pytest.mark.parametrize("case", [
    # narrow sub-experts (Is in {64, 128, 192}, d >= 256): the fused gate-up/SwiGLU/down kernel.
    # Several m-tiles per group with ragged tails, groups smaller than one wave's 32 rows, empty
    # groups, one workgroup walking many tiles (more tiles than compute units in the last case),
    # the shortest supported K (d = 256) and K lengths that are not powers of two
    dict(T=900, d=256, N=5, S=4, Is=64, k_max=6),
    dict(T=1200, d=512, N=3, S=4, Is=128, k_max=5),
    dict(T=2000, d=320, N=6, S=4, Is=192, k_max=8),
    dict(T=3, d=256, N=2, S=2, Is=192, k_max=4),
    dict(T=700, d=704, N=40, S=4, Is=192, k_max=20),
    dict(T=9000, d=256, N=64, S=4, Is=64, k_max=16),
])
def test_narrow_sub_experts_both_ffn_paths(case, path, monkeypatch):
    # MOE_PRISM_FFN=split sends the same shapes through the gate-up and down kernels
    monkeypatch.setenv("MOE_PRISM_FFN", "split" if path == "split" else "auto")
    rng = np.random.default_rng(case["T"])
    k = rng.integers(0, case["k_max"] + 1, size=case["T"]).astype(np.int32)
    wl = W.make_workload("narrow", dtype="bf16", d=case["d"], n_experts=case["N"], n_sub=case["S"],
                         inter_sub=case["Is"], req_tokens=[1] * case["T"], req_k=k,
                         k_max=case["k_max"], seed=case["T"], bias_std=1.0, w_std=0.05)
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)
    assert row_rel(r["y"], ref["y"]) <= 4e-2 and row_rel(r["out"], ref["out"]) <= 4e-2
    B.moe_prism_timing_enable(True)
    B.moe_prism_timing_read()
    out, _, _ = run_layer(wl, r["dev"], r["ws"])
    calls = {k: v[1] for k, v in B.moe_prism_timing_read().items()}
    B.moe_prism_timing_enable(False)
    assert np.array_equal(to_np(out), r["out"])
    # the intended kernels ran
    assert (calls["ffn_fused"], calls["ffn_gate_up"], calls["ffn_down"]) == \
        ((1, 0, 0) if path == "fused" else (0, 1, 1))


@pytest.mark.parametrize("stage_k", ["64", "32"])
@pytest.mark.parametrize("case", [
    dict(T=900, d=512, N=3, S=2, Is=256, k_max=4),      # both GEMMs in 64-element stages, 256-wide tiles
    dict(T=1500, d=256, N=5, S=2, Is=320, k_max=6),     # shortest K the 64-element driver takes (4 stages)
    dict(T=700, d=1024, N=4, S=2, Is=704, k_max=5),     # 192-wide gate-up tiles (1408 rows), 11 down stages
    dict(T=1100, d=448, N=3, S=4, Is=352, k_max=7),     # Is % 64 != 0: the down GEMM keeps 32-element stages
    dict(T=5, d=320, N=2, S=1, Is=512, k_max=2),        # a handful of rows: most waves multiply nothing
    dict(T=2600, d=384, N=2, S=1, Is=1024, k_max=2),    # groups of many m-tiles, several items per workgroup
])
def test_wide_sub_experts_both_stage_widths(case, stage_k, monkeypatch):
    # MOE_PRISM_FFN_K=32 sends the same shapes through the drivers with 32-element K stages
    monkeypatch.setenv("MOE_PRISM_FFN_K", stage_k)
    rng = np.random.default_rng(case["T"] + 1)
    k = rng.integers(0, case["k_max"] + 1, size=case["T"]).astype(np.int32)
    wl = W.make_workload("wide", dtype="bf16", d=case["d"], n_experts=case["N"], n_sub=case["S"],
                         inter_sub=case["Is"], req_tokens=[1] * case["T"], req_k=k,
                         k_max=case["k_max"], seed=case["T"], bias_std=1.0, w_std=0.05)
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)
    assert row_rel(r["y"], ref["y"]) <= 4e-2 and row_rel(r["out"], ref["out"]) <= 4e-2
    out, _, _ = run_layer(wl, r["dev"], r["ws"])
    assert np.array_equal(to_np(out), r["out"])


def test_traffic_probe_runs_beside_the_ffn_and_leaves_it_alone():
    # the measurement entry point walks the same tile table with the products left out: it
    # must stay inside y's rows [0, P) (guard rows and the rows >= P keep their fill), refuse
    # shapes the fused kernel does not serve, and leave the tables so that the next FFN call
    # still gives the result it gave before
    wl = W.make_workload("probe", dtype="bf16", d=512, n_experts=12, n_sub=4, inter_sub=192,
                         req_tokens=[1] * 1500, req_k=np.random.default_rng(5).integers(0, 9, 1500).astype(np.int32),
                         k_max=8, seed=5, bias_std=1.0, w_std=0.05)
    r = run_stages(wl)
    dev, ws, shape = r["dev"], r["ws"], r["shape"]
    P = int(r["off"][-1])
    off = torch.from_numpy(r["off"]).cuda()
    sp = torch.from_numpy(r["sorted_pair"]).cuda()
    y = torch.full((wl.T * wl.k_max, wl.d), 7.0, dtype=torch.bfloat16, device="cuda")
    B.moe_prism_timing_enable(True)
    B.moe_prism_timing_read()
    B.moe_prism_ffn_traffic_probe(shape, dev["x"], dev["w_gate_up"], dev["w_down"], off, sp, ws, y)
    torch.cuda.synchronize()
    t = B.moe_prism_timing_read()
    B.moe_prism_timing_enable(False)
    assert t["ffn_traffic"][1] == 1 and t["ffn_fused"][1] == 0
    assert P < wl.T * wl.k_max and bool((y[P:] == 7.0).all())
    y2 = B.moe_prism_grouped_ffn(shape, dev["x"], dev["w_gate_up"], dev["w_down"], off, sp, ws)
    torch.cuda.synchronize()
    assert np.array_equal(to_np(y2[:P]), r["y"])
    wide = W.make_workload("wide", dtype="bf16", d=256, n_experts=4, n_sub=1, inter_sub=256,
                           req_tokens=[40], req_k=[2], k_max=2, seed=1)
    rw = run_stages(wide)
    with pytest.raises(B.MoePrismError):
        B.moe_prism_ffn_traffic_probe(rw["shape"], rw["dev"]["x"], rw["dev"]["w_gate_up"],
                                      rw["dev"]["w_down"], torch.from_numpy(rw["off"]).cuda(),
                                      torch.from_numpy(rw["sorted_pair"]).cuda(), rw["ws"],
                                      torch.empty((80, 256), dtype=torch.bfloat16, device="cuda"))


def test_no_renormalize_and_repeated_rows():
    # repeated-row router: exact S-way ties decided by id; full-softmax weights
    base = W.make_workload("a", dtype="bf16", d=128, n_experts=16, n_sub=1, inter_sub=128,
                           req_tokens=[300], req_k=[3], k_max=3, seed=7, routed_scale=1.0,
                           w_std=0.05, renormalize=0)
    wl = W.split_workload(base, 4)
    wl.k_tok = np.random.default_rng(7).integers(0, wl.k_max + 1, size=wl.T).astype(np.int32)
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)


def test_edge_cases():
    wl = W.make_workload("e", dtype="bf16", d=64, n_experts=4, n_sub=2, inter_sub=32,
                         req_tokens=[5, 7], req_k=[0, 0], k_max=3, seed=1)
    r = run_stages(wl)                                  # nobody routed anywhere
    assert r["pairs"] == 0 and np.all(r["out"] == 0) and np.all(r["ids"] == -1)
    assert np.all(r["cnt"] == 0) and np.all(r["off"] == 0) and np.all(r["sorted_pair"] == -1)
    # budgets outside [0, k_max] are clamped and flagged
    wl.k_tok = np.array([-2, 9, 1, 3, 0, 2, 2, 2, 3, 1, 1, 0], np.int32)
    r = run_stages(wl)
    assert r["flags"] & 1
    ref = O.layer_of(wl, return_all=True)               # the oracle clamps the same way
    check_against_oracle(wl, r, ref)
    # T = 0
    wl0 = W.make_workload("z", dtype="bf16", d=64, n_experts=4, n_sub=2, inter_sub=32,
                          req_tokens=[], req_k=[], k_max=3, seed=1)
    r0 = run_stages(wl0)
    assert r0["pairs"] == 0 and r0["out"].shape == (0, 64) and np.all(r0["off"] == 0)
    out, _, _ = run_layer(wl0)
    assert out.shape == (0, 64)


def test_wide_router_and_large_k():
    # E = 2048 sub-experts (32 logits per lane), k up to 200
    T = 96
    k = np.random.default_rng(3).integers(0, 201, size=T).astype(np.int32)
    wl = W.make_workload("wide", dtype="bf16", d=64, n_experts=512, n_sub=4, inter_sub=32,
                         req_tokens=[1] * T, req_k=k, k_max=200, seed=3, w_std=0.1)
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_full_oracle(seed):
    # seeded random layer shapes: K lengths on both sides of every kernel-selection threshold
    # (register-staged, in-step ring, two-group ring; 192- and 256-wide tiles; all three logits
    # kernels' neighbours), ragged groups, empty groups, budgets from 0 to k_max
    rng = np.random.default_rng(1000 + seed)
    d = 64 * int(rng.integers(1, 11))
    Is = 32 * int(rng.integers(1, 14))
    N, S = int(rng.integers(1, 7)), int(rng.choice([1, 2, 4]))
    T = int(rng.choice([1, 37, 256, 700, 1300, 2500]))
    k_max = int(rng.integers(1, min(N * S, 12) + 1))
    k = rng.integers(0, k_max + 1, size=T).astype(np.int32)
    dtype = "bf16" if seed % 4 else "f32"
    wl = W.make_workload("rnd", dtype=dtype, d=d, n_experts=N, n_sub=S, inter_sub=Is,
                         req_tokens=[1] * T, req_k=k, k_max=k_max, seed=seed, bias_std=1.0,
                         w_std=0.05, renormalize=int(rng.integers(0, 2)))
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)
    out, _, _ = run_layer(wl, r["dev"], r["ws"])
    assert np.array_equal(to_np(out), r["out"])


def test_largest_supported_router_and_budget():
    # the documented limits: E = 4096 sub-experts (64 logits per lane), k_max = 1024
    T = 40
    k = np.random.default_rng(5).integers(0, 1025, size=T).astype(np.int32)
    k[:3] = [1024, 0, 1]
    wl = W.make_workload("max", dtype="bf16", d=64, n_experts=1024, n_sub=4, inter_sub=32,
                         req_tokens=[1] * T, req_k=k, k_max=1024, seed=5, w_std=0.1)
    r = run_stages(wl)
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)
    # one past either limit is refused on the host
    for bad in (B.make_shape(T, 64, 1025, 4, 32, 8, "bf16"), B.make_shape(T, 64, 1024, 4, 32, 1025, "bf16")):
        with pytest.raises(B.MoePrismError) as e:
            B.alloc_workspace(bad)
        assert e.value.code == -2


@pytest.mark.parametrize("T,E,k_max", [(33000, 4096, 3),   # two 64-token words per chunk: the largest LDS footprint
                                       (70000, 1000, 5),   # four words per chunk, E not a multiple of 4
                                       (1, 7, 7), (257, 33, 2)])
def test_dispatch_alone_on_synthetic_picks(T, E, k_max):
    # the dispatch stage by itself on picks that no router produced: distinct ids per token,
    # -1 padded to a random budget; tables bit for bit
    rng = np.random.default_rng(T + E)
    ids = np.full((T, k_max), -1, np.int32)
    for t in range(T):
        kt = int(rng.integers(0, k_max + 1))
        ids[t, :kt] = rng.choice(E, size=kt, replace=False)
    shape = B.make_shape(T, 64, E, 1, 32, k_max, "bf16")
    ws = B.alloc_workspace(shape)
    cnt, off, sp, sl = B.moe_prism_dispatch(shape, torch.from_numpy(ids).cuda(), ws)
    torch.cuda.synchronize()
    rc, ro, rsp, rsl = O.dispatch(ids, E)
    assert np.array_equal(to_np(cnt), rc) and np.array_equal(to_np(off), ro)
    assert np.array_equal(to_np(sp), rsp) and np.array_equal(to_np(sl), rsl)
    assert B.moe_prism_status(ws)[1] == int(ro[-1])   # the status word belongs to the route stage


def test_everything_routed_to_one_sub_expert():
    # the degenerate load: one group holds all T rows (many m-tiles), every other group is empty
    T = 3000
    wl = W.make_workload("one", dtype="bf16", d=128, n_experts=8, n_sub=4, inter_sub=64,
                         req_tokens=[T], req_k=[1], k_max=2, seed=9, w_std=0.05)
    wl.router_bias = np.zeros(wl.E, np.float32)
    wl.router_bias[13] = 1000.0
    r = run_stages(wl)
    assert r["cnt"][13] == T and r["cnt"].sum() == T
    ref = O.layer_of(wl, return_all=True)
    check_against_oracle(wl, r, ref)


@pytest.mark.parametrize("scale", [1.0, 1e-19])
@pytest.mark.parametrize("T,E", [(6200, 1000), (2100, 500), (300, 100)])
def test_matrix_core_logits_are_the_same_chain(T, E, scale):
    # the three logits kernels (128 x 128 tiles of 32x32x1 MFMAs; 64 x 64 and 32 x 32 tiles of
    # 4x4x1 MFMAs, picked by problem size) each issue one fused multiply-add per k and
    # instruction; each must reproduce the oracle's binary32 chain bit for bit, ragged edges
    # and subnormal partial sums (scale 1e-19: products ~1e-40) included
    d = 192
    rng = np.random.default_rng(11)
    wl = W.make_workload("wide", dtype="f32", d=d, n_experts=E, n_sub=1, inter_sub=32,
                         req_tokens=[T], req_k=[5], k_max=5, seed=11, w_std=0.05,
                         with_weights=False)
    wl.x = (wl.x * np.float32(scale)).astype(np.float32)
    wl.w_router = (wl.w_router * np.float32(scale)).astype(np.float32)
    bias = (rng.standard_normal(E) * scale * scale).astype(np.float32)
    shape = B.make_shape(T, d, E, 1, 32, 5, "f32")
    ws = B.alloc_workspace(shape)
    x, wr = torch.from_numpy(wl.x).cuda(), torch.from_numpy(wl.w_router).cuda()
    ids, w, lg = B.moe_prism_route(shape, x, wr, torch.from_numpy(bias).cuda(),
                                   torch.from_numpy(wl.k_tok).cuda(), ws, want_logits=True)
    torch.cuda.synchronize()
    ref = O.logits(wl.x, wl.w_router, bias)
    assert np.array_equal(to_np(lg).view(np.uint32), ref.view(np.uint32))
    assert np.array_equal(to_np(ids), O.select(ref, wl.k_tok, 5))
    if scale != 1.0:
        assert np.any((np.abs(ref) < 1.2e-38) & (ref != 0))     # subnormal logits do occur


def test_expand_k_and_errors():
    req_k = torch.tensor([3, 0, 5], dtype=torch.int32, device="cuda")
    req_off = torch.tensor([0, 4, 4, 9], dtype=torch.int32, device="cuda")
    k_tok = B.moe_prism_expand_k(req_k, req_off, 9)
    torch.cuda.synchronize()
    assert k_tok.cpu().tolist() == [3] * 4 + [5] * 5
    assert k_tok.cpu().tolist() == W.expand_requests(np.array([3, 0, 5]), np.array([0, 4, 4, 9])).tolist()
    shape = B.make_shape(8, 64, 2, 2, 32, 2, "bf16")
    small = torch.empty(256, dtype=torch.uint8, device="cuda")
    ids = torch.zeros((8, 2), dtype=torch.int32, device="cuda")
    with pytest.raises(B.MoePrismError) as e:
        B.moe_prism_dispatch(shape, ids, small[(-small.data_ptr()) % 256:][:0])
    assert e.value.code in (-1, -3)


def test_bitwise_reproducible():
    wl = W.config("c3_fine_128x4", scale_down=16)       # 1024 tokens of the 128x4 layer
    out1, dev, ws = run_layer(wl)
    a = to_np(out1).copy()
    t1 = {k: to_np(v).copy() for k, v in B.layer_intermediates(dev["shape"], ws).items()}
    out2, _, _ = run_layer(wl, dev, ws)
    assert np.array_equal(a, to_np(out2))
    for k, v in B.layer_intermediates(dev["shape"], ws).items():
        assert np.array_equal(t1[k], to_np(v)), k


def test_other_tokens_budgets_do_not_matter():
    # Sec. 3.3.1: no over-serving - a token's output depends only on its own budget
    wl = W.config("c4_decode_64x2", scale_down=16)
    out1, dev, ws = run_layer(wl)
    a = to_np(out1).copy()
    k2 = wl.k_tok.copy()
    k2[::2] = 12
    dev["k_tok"] = torch.from_numpy(k2).cuda()
    out2, _, _ = run_layer(wl, dev, ws)
    b = to_np(out2)
    same = wl.k_tok == k2
    assert np.array_equal(a[same], b[same]) and not np.array_equal(a[~same], b[~same])


def test_combine_never_reads_the_row_of_a_pick_without_a_slot():
    # standalone combine: a pick whose slot is -1 contributes nothing, whatever y holds (here
    # NaN in every row, so that reading any row for it, even times zero, would show)
    T, d, k_max = 5, 128, 3
    shape = B.make_shape(T, d, 4, 2, 32, k_max, "bf16")
    rng = np.random.default_rng(2)
    y = torch.from_numpy(rng.standard_normal((T * k_max, d)).astype(np.float32)).cuda().bfloat16()
    slot = rng.permutation(T * k_max).astype(np.int32).reshape(T, k_max)
    slot[1, 0] = -1
    slot[3, 2] = -1
    y[0] = float("nan")                      # row 0 is where a redirected pick would have read
    used0 = np.argwhere(slot == 0)
    slot[used0[:, 0], used0[:, 1]] = -1     # nobody legitimately reads row 0
    w = rng.random((T, k_max)).astype(np.float32)
    k_tok = np.full(T, k_max, np.int32)
    out = B.moe_prism_combine(shape, y, torch.from_numpy(slot.reshape(-1)).cuda(),
                              torch.from_numpy(w).cuda(), torch.from_numpy(k_tok).cuda())
    torch.cuda.synchronize()
    got = to_np(out)
    assert np.isfinite(got).all()
    yf = to_np(y).astype(np.float64)
    ref = np.zeros((T, d))
    for t in range(T):
        for j in range(k_max):
            if slot[t, j] >= 0:
                ref[t] += float(w[t, j]) * yf[slot[t, j]]
    assert max_rel(got, ref) <= 2e-2


@pytest.mark.parametrize("case", [
    dict(dtype="bf16", T=777, d=320, N=6, S=4, Is=192, k_max=8),     # fused FFN kernel
    dict(dtype="bf16", T=500, d=192, N=5, S=2, Is=96, k_max=5),      # two-kernel FFN
    dict(dtype="f32", T=130, d=128, N=4, S=2, Is=64, k_max=4),
])
def test_guard_bands_around_workspace_y_and_out_stay_intact(case):
    # the workspace, y (staged call: exactly P valid rows wide, the rest of its T*k_max rows must
    # stay untouched) and out sit between 4 KiB bands of a known byte; no kernel may write outside
    dtype = case["dtype"]
    rng = np.random.default_rng(case["T"])
    k = rng.integers(0, case["k_max"] + 1, size=case["T"]).astype(np.int32)
    wl = W.make_workload("guard", dtype=dtype, d=case["d"], n_experts=case["N"], n_sub=case["S"],
                         inter_sub=case["Is"], req_tokens=[1] * case["T"], req_k=k,
                         k_max=case["k_max"], seed=case["T"], bias_std=1.0, w_std=0.05)
    dev = B.to_device(wl)
    shape = dev["shape"]
    G, FILL = 4096, 0xA5
    el = 2 if dtype == "bf16" else 4
    tdt = B.act_dtype(shape)

    def banded(nbytes):
        buf = torch.full((nbytes + 2 * G + 256,), FILL, dtype=torch.uint8, device="cuda")
        o = (-(buf.data_ptr() + G)) % 256 + G
        return buf, buf[o:o + nbytes], o

    def intact(buf, o, nbytes):
        b = buf.cpu().numpy()
        return bool((b[:o] == FILL).all() and (b[o + nbytes:] == FILL).all())

    n_ws = B.moe_prism_workspace_bytes(shape)
    ws_buf, ws, ws_o = banded(n_ws)
    n_y = wl.T * wl.k_max * wl.d * el
    y_buf, y_raw, y_o = banded(n_y)
    n_out = wl.T * wl.d * el
    out_buf, out_raw, out_o = banded(n_out)
    y = y_raw.view(tdt).view(wl.T * wl.k_max, wl.d)
    out = out_raw.view(tdt).view(wl.T, wl.d)

    ids, w = B.moe_prism_route(shape, dev["x"], dev["w_router"], dev["router_bias"], dev["k_tok"], ws)
    cnt, off, sp, sl = B.moe_prism_dispatch(shape, ids, ws)
    B.moe_prism_grouped_ffn(shape, dev["x"], dev["w_gate_up"], dev["w_down"], off, sp, ws, y=y)
    B.moe_prism_combine(shape, y, sl, w, dev["k_tok"], out=out)
    torch.cuda.synchronize()
    P = int(off[-1].item())
    assert intact(ws_buf, ws_o, n_ws) and intact(y_buf, y_o, n_y) and intact(out_buf, out_o, n_out)
    # rows of y beyond the P pairs are never written either
    tail = y_raw[P * wl.d * el:].cpu().numpy()
    assert (tail == FILL).all()
    staged = to_np(out).copy()
    B.moe_prism_layer(shape, dev["x"], dev["w_router"], dev["router_bias"], dev["k_tok"],
                      dev["w_gate_up"], dev["w_down"], ws, out=out)
    torch.cuda.synchronize()
    assert intact(ws_buf, ws_o, n_ws) and intact(out_buf, out_o, n_out)
    assert np.array_equal(staged, to_np(out))
    ref = O.layer_of(wl)
    assert max_rel(staged, ref) <= TOL[dtype]
