"""GPU parity at the benchmark's full sizes, through moe_prism_layer (the launch
configuration bench.py times).  Routing ids and dispatch tables are compared with the
oracle for ALL tokens, bit for bit; layer outputs on a random sample of tokens the
oracle evaluates one by one."""
import functools

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2510_19366_amd import binding as B
from paper_2510_19366_amd import workloads as W
from gpu_util import max_rel, run_layer, to_np

pytestmark = pytest.mark.gpu


@functools.lru_cache(maxsize=2)
def workload(name, T=None):
    return W.config(name, T=T) if T else W.config(name)


def check_full(wl, n_sample, seed=0):
    out, dev, ws = run_layer(wl)
    flags, pairs = B.moe_prism_status(ws)
    assert flags == 0 and pairs == wl.pairs
    inter = {k: to_np(v) for k, v in B.layer_intermediates(dev["shape"], ws).items()}
    # route + dispatch: everything, bit-exact
    lg = O.logits(wl.x, wl.w_router, wl.router_bias)
    assert np.array_equal(inter["logits"].view(np.uint32), lg.view(np.uint32))
    ids = O.select(lg, wl.k_tok, wl.k_max)
    assert np.array_equal(inter["topk_ids"], ids)
    w = O.weights(lg, ids, wl.k_tok, wl.renormalize, wl.routed_scale)
    np.testing.assert_allclose(inter["topk_w"], w, rtol=1e-5, atol=1e-7)
    cnt, off, sp, sl = O.dispatch(ids, wl.E)
    assert np.array_equal(inter["group_count"], cnt) and np.array_equal(inter["group_offset"], off)
    assert np.array_equal(inter["sorted_pair"], sp) and np.array_equal(inter["slot_of_pair"], sl)
    # outputs: sampled tokens, one by one
    tok = np.sort(np.random.default_rng(seed).choice(wl.T, size=n_sample, replace=False)).astype(np.int32)
    ref, _, _ = O.layer_tokens(tok, wl.x, wl.w_router, wl.router_bias, wl.k_tok, wl.w_gate_up,
                               wl.w_down, wl.k_max, wl.renormalize, wl.routed_scale)
    got = to_np(out)
    err = max_rel(got[tok], ref)
    assert err <= 2e-2, err
    assert np.isfinite(got).all()
    assert np.all(got[wl.k_tok == 0] == 0)
    return got, cnt


def test_c3_fine_128x4_full():
    wl = workload("c3_fine_128x4")
    assert (wl.T, wl.E, wl.inter_sub, wl.k_max) == (16384, 512, 192, 32)
    _, cnt = check_full(wl, n_sample=96)
    assert cnt.max() > 8 * max(1, int(np.median(cnt)))       # the bias makes the load skewed


def test_c4_decode_64x2_full():
    wl = workload("c4_decode_64x2")
    assert (wl.T, wl.E, wl.inter_sub) == (8192, 128, 704) and set(np.unique(wl.k_tok)) == {4, 12}
    check_full(wl, n_sample=96)


def test_c2_mixtral_8x4_full():
    wl = workload("c2_mixtral_8x4")
    assert (wl.T, wl.d, wl.E, wl.inter_sub) == (4096, 4096, 32, 3584)
    check_full(wl, n_sample=24)


@pytest.mark.parametrize("T", [512, 2048, 16384, 65536])
def test_c5_matched_budget_split_vs_whole(T):
    # Sec. 3.2.2: repeated-row gate at k = S*k_orig with scale S reproduces the undivided layer
    a = W.config("c5a_s1_k8", T=T)
    b = W.split_workload(a, 4)
    assert (b.E, b.k_max, b.inter_sub, b.routed_scale) == (512, 32, 192, 4.0)
    got_a, _ = check_full(a, n_sample=32, seed=1)
    got_b, _ = check_full(b, n_sample=32, seed=1)
    assert max_rel(got_b, got_a) <= 2e-2
