"""Pins of the CPU oracle to things other than itself.

Each oracle function is checked against what the mathematics or the paper
fixes: closed forms, brute force on tiny inputs, library routines in special
cases, invariants, and the neuron-split identity (Sec. 3.2.1, Eq. 3).
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import softmax as sp_softmax

from oracle import oracle as O
from paper_2510_19366_amd import workloads as W

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# ----------------------------------------------------------------- helpers
def f32_round(fr: Fraction) -> float:
    """Exact round-to-nearest-even of a rational to binary32 (normal range)."""
    if fr == 0:
        return 0.0
    s = -1 if fr < 0 else 1
    fr = abs(fr)
    e = math.floor(math.log2(fr))
    while Fraction(2) ** e > fr:
        e -= 1
    while Fraction(2) ** (e + 1) <= fr:
        e += 1
    assert e >= -126
    q = fr / (Fraction(2) ** (e - 23))          # in [2^23, 2^24)
    n = q.numerator // q.denominator
    rem = q - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    return s * float(n) * 2.0 ** (e - 23)


def dense_swiglu64(x, wg, wu, wd):
    """Undivided SwiGLU FFN (Eq. 1) with dense float64 matmuls.  wg, wu: [I, d]; wd: [d, I]."""
    x = x.astype(np.float64)
    a = x @ wg.astype(np.float64).T
    u = x @ wu.astype(np.float64).T
    h = a / (1.0 + np.exp(-a)) * u
    return h @ wd.astype(np.float64).T


def standard_topk_moe64(x, w_r, wg, wu, wd, k, renorm, scale):
    """Ordinary uniform top-k softmax MoE over undivided experts, written with numpy
    library calls only (float64 logits; used where logits are well separated)."""
    lg = x.astype(np.float64) @ w_r.astype(np.float64).T
    order = np.argsort(-lg, axis=1, kind="stable")[:, :k]
    p = sp_softmax(lg, axis=1)
    out = np.zeros((x.shape[0], x.shape[1]))
    for t in range(x.shape[0]):
        w = p[t, order[t]]
        if renorm:
            w = w / w.sum()
        for e, we in zip(order[t], w):
            out[t] += scale * we * dense_swiglu64(x[t:t + 1], wg[e], wu[e], wd[e])[0]
    return out


def small_layer(seed=0, T=12, d=24, N=5, S=3, Is=8, k_max=None, dtype="f32"):
    rng = np.random.default_rng(seed)
    E = N * S
    k_max = k_max or E
    k = rng.integers(0, k_max + 1, size=T).astype(np.int32)
    return W.make_workload("small", dtype=dtype, d=d, n_experts=N, n_sub=S, inter_sub=Is,
                           req_tokens=[1] * T, req_k=k, k_max=k_max, seed=seed, w_std=0.3)


# ----------------------------------------------------------------- logits
def test_logits_exact_on_small_integers():
    # every summation order gives the same exact result -> checks indexing / layout only
    rng = np.random.default_rng(1)
    x = rng.integers(-8, 9, size=(7, 33)).astype(np.float32)
    w = rng.integers(-8, 9, size=(5, 33)).astype(np.float32)
    b = rng.integers(-4, 5, size=5).astype(np.float32)
    ref = x.astype(np.int64) @ w.astype(np.int64).T + b.astype(np.int64)
    got = O.logits(x, w, b)
    assert got.dtype == np.float32 and got.shape == (7, 5)
    assert np.array_equal(got.astype(np.int64), ref)
    assert np.array_equal(O.logits(x, w, None).astype(np.int64), ref - b.astype(np.int64))


def test_logits_are_one_fma_chain_in_ascending_order():
    # exact rational emulation of: acc = RN32(x_j * w_j + acc), j ascending, then RN32(acc + b)
    rng = np.random.default_rng(2)
    x = rng.standard_normal((3, 19)).astype(np.float32)
    w = rng.standard_normal((4, 19)).astype(np.float32)
    b = rng.standard_normal(4).astype(np.float32)
    got = O.logits(x, w, b)
    differs_from_unfused = 0
    for t in range(3):
        for g in range(4):
            acc = Fraction(0)
            acc_unfused = np.float32(0)
            for j in range(19):
                acc = Fraction(f32_round(Fraction(float(x[t, j])) * Fraction(float(w[g, j])) + acc))
                acc_unfused = np.float32(acc_unfused + np.float32(x[t, j] * w[g, j]))
            want = f32_round(acc + Fraction(float(b[g])))
            assert float(got[t, g]) == want, (t, g)
            differs_from_unfused += float(np.float32(acc_unfused + b[g])) != want
    assert differs_from_unfused > 0      # the test can tell a fused chain from mul-then-add


def test_logits_within_fp64_bound():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((16, 512)).astype(np.float32)
    w = (rng.standard_normal((24, 512)) * 0.02).astype(np.float32)
    got = O.logits(x, w).astype(np.float64)
    ref = x.astype(np.float64) @ w.astype(np.float64).T
    bound = 512 * 2.0 ** -24 * (np.abs(x).astype(np.float64) @ np.abs(w).astype(np.float64).T)
    assert np.all(np.abs(got - ref) <= bound)
    assert np.abs(got - ref).max() > 0          # not accidentally a float64 path


# ----------------------------------------------------------------- selection
def test_select_brute_force_tiny():
    rng = np.random.default_rng(4)
    E = 9
    lg = rng.standard_normal((20, E)).astype(np.float32)
    k_tok = rng.integers(0, E + 1, size=20).astype(np.int32)
    ids = O.select(lg, k_tok, E)
    for t in range(20):
        k = int(k_tok[t])
        chosen = ids[t, :k]
        assert np.all(ids[t, k:] == -1)
        assert len(set(chosen.tolist())) == k
        best = max(itertools.combinations(range(E), k), key=lambda c: sum(float(lg[t, i]) for i in c))
        assert set(chosen.tolist()) == set(best)
        assert np.all(np.diff(lg[t, chosen]) <= 0)      # descending logit order


def test_select_matches_stable_sort_and_is_nested():
    rng = np.random.default_rng(5)
    T, E, k_max = 50, 40, 17
    # coarse values -> many exact ties
    lg = (rng.integers(-3, 4, size=(T, E)) * 0.5).astype(np.float32)
    order = np.argsort(-lg, axis=1, kind="stable")
    full = O.select(lg, np.full(T, k_max, np.int32), k_max)
    assert np.array_equal(full, order[:, :k_max])
    k_tok = rng.integers(0, k_max + 1, size=T).astype(np.int32)
    ids = O.select(lg, k_tok, k_max)
    for t in range(T):
        assert np.array_equal(ids[t, :k_tok[t]], full[t, :k_tok[t]])
        assert np.all(ids[t, k_tok[t]:] == -1)


def test_select_repeated_rows_and_signed_zero():
    # a repeated-row router gives exact S-way ties: sub-experts of one expert in id order
    N, S = 4, 3
    base = np.array([[0.3, 2.0, -1.0, 0.7]], np.float32)
    lg = np.repeat(base, S, axis=1)
    ids = O.select(lg, np.array([7], np.int32), 8)
    assert ids[0, :7].tolist() == [3, 4, 5, 9, 10, 11, 0] and ids[0, 7] == -1
    z = np.array([[-0.0, 0.0, -0.0, -1.0]], np.float32)          # -0.0 == +0.0: lower id first
    assert O.select(z, np.array([3], np.int32), 3)[0].tolist() == [0, 1, 2]
    with pytest.raises(ValueError):
        O.select(z, np.array([1], np.int32), 5)
    # out-of-range budgets are clamped to [0, k_max]
    assert O.select(z, np.array([9], np.int32), 2)[0].tolist() == [0, 1]
    assert O.select(z, np.array([-3], np.int32), 2)[0].tolist() == [-1, -1]


# ----------------------------------------------------------------- weights
def test_weights_closed_forms():
    rng = np.random.default_rng(6)
    T, E, k_max = 9, 12, 12
    lg = rng.standard_normal((T, E)).astype(np.float32)
    k_tok = rng.integers(1, k_max + 1, size=T).astype(np.int32)
    ids = O.select(lg, k_tok, k_max)
    p = sp_softmax(lg.astype(np.float64), axis=1)
    w0 = O.weights(lg, ids, k_tok, 0, 2.5)
    w1 = O.weights(lg, ids, k_tok, 1, 2.5)
    for t in range(T):
        k = k_tok[t]
        sel = ids[t, :k]
        np.testing.assert_allclose(w0[t, :k], 2.5 * p[t, sel], rtol=1e-13)
        np.testing.assert_allclose(w1[t, :k], 2.5 * p[t, sel] / p[t, sel].sum(), rtol=1e-13)
        assert abs(w1[t, :k].sum() - 2.5) < 1e-13
        assert np.all(w0[t, k:] == 0) and np.all(w1[t, k:] == 0)
    # all E selected without renormalisation is the full softmax
    full = O.weights(lg, O.select(lg, np.full(T, E, np.int32), E), np.full(T, E, np.int32), 0, 1.0)
    order = np.argsort(-lg, axis=1, kind="stable")
    np.testing.assert_allclose(full, np.take_along_axis(p, order, 1), rtol=1e-13)


def test_weights_repeated_row_router_closed_form():
    # with every original row repeated S times a sub-expert's full-softmax mass is p_e / S
    N, S = 5, 4
    rng = np.random.default_rng(7)
    le = rng.standard_normal((3, N)).astype(np.float32)
    lg = np.repeat(le, S, axis=1)
    k = np.full(3, N * S, np.int32)
    ids = O.select(lg, k, N * S)
    w = O.weights(lg, ids, k, 0, float(S))
    pe = sp_softmax(le.astype(np.float64), axis=1)
    for t in range(3):
        np.testing.assert_allclose(w[t], pe[t, ids[t] // S], rtol=1e-13)


# ----------------------------------------------------------------- dispatch
def test_dispatch_invariants_and_counting_sort():
    rng = np.random.default_rng(8)
    T, E, k_max = 300, 23, 9
    lg = rng.standard_normal((T, E)).astype(np.float32)
    k_tok = rng.integers(0, k_max + 1, size=T).astype(np.int32)
    ids = O.select(lg, k_tok, k_max)
    cnt, off, sp, sl = O.dispatch(ids, E)
    P = int(k_tok.sum())
    assert cnt.sum() == P == off[E] and off[0] == 0
    assert np.array_equal(np.diff(off), cnt)
    assert np.array_equal(cnt, np.bincount(ids[ids >= 0], minlength=E))
    flat = ids.reshape(-1)
    valid = np.flatnonzero(flat >= 0)
    want = valid[np.argsort(flat[valid], kind="stable")]          # textbook counting sort
    assert np.array_equal(sp[:P], want) and np.all(sp[P:] == -1)
    assert np.array_equal(sl[sp[:P]], np.arange(P))
    assert np.all(sl[flat < 0] == -1)
    for g in range(E):
        toks = sp[off[g]:off[g + 1]] // k_max
        assert np.all(np.diff(toks) > 0)                          # tokens strictly ascending
        assert np.all(flat[sp[off[g]:off[g + 1]]] == g)
    with pytest.raises(ValueError):
        O.dispatch(np.array([[E]], np.int32), E)


def test_pairs_equal_sum_of_budgets_golden():
    # Sec. 2.4 worked example: budgets {2,4,5,6}; batch-max execution gives 6 picks per token
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(GOLD, "mixed_k_example.txt"))
            if l.strip() and not l.startswith("#")]
    req_k = np.array([r[0] for r in rows], np.int32)
    n_tok = 5
    req_off = np.arange(len(rows) + 1, dtype=np.int32) * n_tok
    k_tok = W.expand_requests(req_k, req_off)
    lg = np.random.default_rng(9).standard_normal((len(k_tok), 16)).astype(np.float32)
    k_max = int(req_k.max())
    own = O.dispatch(O.select(lg, k_tok, k_max), 16)[1][-1]
    bmax = O.dispatch(O.select(lg, np.full_like(k_tok, k_max), k_max), 16)[1][-1]
    assert own == n_tok * sum(r[1] for r in rows) == 85
    assert bmax == n_tok * sum(r[2] for r in rows) == 120


# ----------------------------------------------------------------- sub-expert FFN
def test_ffn_one_hand_computed():
    # d = 2, one neuron: a = 1*0.5 + 2*0.25 = 1, u = 1*2 + 2*(-1) = 0... use u = 1*2 + 2*1 = 4
    x = np.array([1.0, 2.0], np.float32)
    w_gu = np.array([[0.5, 0.25], [2.0, 1.0]], np.float32)      # gate row, up row
    w_dn = np.array([[3.0], [-0.5]], np.float32)                # [d, Is]
    h = 1.0 / (1.0 + math.exp(-1.0)) * 4.0
    np.testing.assert_allclose(O.ffn_one(x, w_gu, w_dn), [3.0 * h, -0.5 * h], rtol=1e-15)


@pytest.mark.parametrize("permute", [False, True])
def test_split_sum_identity(permute):
    # Eq. 3: the S neuron subsets of an expert sum to the undivided expert
    rng = np.random.default_rng(10)
    d, I, S = 40, 48, 4
    Is = I // S
    x = rng.standard_normal((6, d)).astype(np.float32)
    wg = (rng.standard_normal((I, d)) * 0.3).astype(np.float32)
    wu = (rng.standard_normal((I, d)) * 0.3).astype(np.float32)
    wd = (rng.standard_normal((d, I)) * 0.3).astype(np.float32)
    ref = dense_swiglu64(x, wg, wu, wd)
    perm = rng.permutation(I) if permute else np.arange(I)
    for t in range(6):
        acc = np.zeros(d)
        parts = []
        for s in range(S):
            idx = perm[s * Is:(s + 1) * Is]
            w_gu = np.concatenate([wg[idx], wu[idx]], axis=0)
            parts.append(O.ffn_one(x[t], w_gu, wd[:, idx]))
            acc += parts[-1]
        np.testing.assert_allclose(acc, ref[t], rtol=1e-12, atol=1e-13)
        assert np.abs(parts[0] - ref[t]).max() > 1e-3       # a single part is not the whole


def test_grouped_ffn_rows_follow_the_tables():
    wl = small_layer(seed=11)
    r = O.layer_of(wl, return_all=True)
    P = r["off"][-1]
    assert r["y"].shape == (P, wl.d)
    for p in range(0, P, 7):
        g = int(np.searchsorted(r["off"], p, side="right") - 1)
        t = r["sorted_pair"][p] // wl.k_max
        Is = wl.inter_sub
        ref = dense_swiglu64(wl.x[t:t + 1], wl.w_gate_up[g, :Is], wl.w_gate_up[g, Is:], wl.w_down[g])[0]
        np.testing.assert_allclose(r["y"][p], ref, rtol=1e-11, atol=1e-13)


# ----------------------------------------------------------------- layer
def test_layer_matched_budget_equals_standard_moe():
    # Sec. 3.2.2: repeated-row router, k = S*k_orig, scale S  ==  top-k_orig MoE on whole experts
    rng = np.random.default_rng(12)
    T, d, N, I, S, k_orig = 10, 32, 6, 24, 4, 2
    base = W.make_workload("a", dtype="f32", d=d, n_experts=N, n_sub=1, inter_sub=I,
                           req_tokens=[T], req_k=[k_orig], k_max=k_orig, seed=12,
                           routed_scale=1.0, w_std=0.3)
    for renorm in (0, 1):
        base.renormalize = renorm
        sp = W.split_workload(base, S)
        assert sp.k_max == S * k_orig and sp.routed_scale == S and sp.E == N * S
        got = O.layer_of(sp)
        ref = standard_topk_moe64(base.x, base.w_router, base.w_gate_up[:, :I],
                                  base.w_gate_up[:, I:], base.w_down, k_orig, renorm, 1.0)
        # the reference takes float64 logits, the oracle binary32 ones: weights agree to ~1e-6
        np.testing.assert_allclose(got, ref, rtol=5e-5, atol=1e-8)
        # and the undivided layer through the oracle is the same standard MoE
        np.testing.assert_allclose(O.layer_of(base), ref, rtol=5e-5, atol=1e-8)
        # split vs undivided share the logits, so they differ by summation order only
        np.testing.assert_allclose(got, O.layer_of(base), rtol=1e-11, atol=1e-14)


def test_layer_all_selected_is_dense_mixture():
    wl = small_layer(seed=13)
    E = wl.E
    k = np.full(wl.T, E, np.int32)
    out = O.layer(wl.x, wl.w_router, None, k, wl.w_gate_up, wl.w_down, E, 0, 1.0)
    p = sp_softmax(wl.x.astype(np.float64) @ wl.w_router.astype(np.float64).T, axis=1)
    Is = wl.inter_sub
    ref = np.zeros_like(out)
    for g in range(E):
        ref += p[:, g:g + 1] * dense_swiglu64(wl.x, wl.w_gate_up[g, :Is], wl.w_gate_up[g, Is:], wl.w_down[g])
    # p from float64 logits vs binary32 logits: ~1e-6 relative on the weights
    np.testing.assert_allclose(out, ref, rtol=1e-5, atol=2e-6 * np.abs(ref).max())


def test_layer_properties():
    wl = small_layer(seed=14, T=16)
    args = (wl.w_router, None)
    base = O.layer(wl.x, *args, wl.k_tok, wl.w_gate_up, wl.w_down, wl.k_max, 1, 2.0)
    # token-permutation equivariance (bitwise)
    perm = np.random.default_rng(0).permutation(wl.T)
    outp = O.layer(wl.x[perm], *args, wl.k_tok[perm], wl.w_gate_up, wl.w_down, wl.k_max, 1, 2.0)
    assert np.array_equal(outp, base[perm])
    # linear in routed_scale
    np.testing.assert_allclose(O.layer(wl.x, *args, wl.k_tok, wl.w_gate_up, wl.w_down, wl.k_max, 1, 6.0),
                               3.0 * base, rtol=1e-13)
    # k_t = 0 rows are exactly zero; other tokens' budgets do not matter (bitwise)
    k2 = wl.k_tok.copy()
    k2[::2] = 0
    out2 = O.layer(wl.x, *args, k2, wl.w_gate_up, wl.w_down, wl.k_max, 1, 2.0)
    assert np.all(out2[::2] == 0) and np.array_equal(out2[1::2], base[1::2])
    # per-token evaluation reproduces the staged path
    sel = np.array([3, 0, 15, 7], np.int32)
    o, ids, w = O.layer_tokens(sel, wl.x, wl.w_router, None, wl.k_tok, wl.w_gate_up, wl.w_down,
                               wl.k_max, 1, 2.0)
    full = O.layer(wl.x, *args, wl.k_tok, wl.w_gate_up, wl.w_down, wl.k_max, 1, 2.0, return_all=True)
    assert np.array_equal(o, full["out"][sel]) and np.array_equal(ids, full["ids"][sel])
    assert np.array_equal(w, full["w"][sel])


def test_layer_uniform_k_is_ordinary_topk_moe_with_bias():
    wl = small_layer(seed=15, T=8, N=4, S=2, k_max=3)
    rng = np.random.default_rng(15)
    bias = rng.standard_normal(wl.E).astype(np.float32)
    k = np.full(wl.T, 3, np.int32)
    got = O.layer(wl.x, wl.w_router, bias, k, wl.w_gate_up, wl.w_down, 3, 1, 1.0)
    Is = wl.inter_sub
    lg = wl.x.astype(np.float64) @ wl.w_router.astype(np.float64).T + bias
    order = np.argsort(-lg, axis=1, kind="stable")[:, :3]
    ref = np.zeros_like(got)
    for t in range(wl.T):
        w = sp_softmax(lg[t, order[t]])
        for g, wg_ in zip(order[t], w):
            ref[t] += wg_ * dense_swiglu64(wl.x[t:t + 1], wl.w_gate_up[g, :Is], wl.w_gate_up[g, Is:],
                                           wl.w_down[g])[0]
    np.testing.assert_allclose(got, ref, rtol=1e-5, atol=2e-6 * np.abs(ref).max())


def test_table1_split_shapes():
    # Table I: a x4 split multiplies experts and active count by 4, divides the intermediate by 4
    for line in open(os.path.join(GOLD, "table1_shapes.txt")):
        if not line.strip() or line.startswith("#"):
            continue
        _, e0, e1, a0, a1, i0, i1 = line.split()
        e0, e1, a0, a1, i0, i1 = map(int, (e0, e1, a0, a1, i0, i1))
        assert e1 == 4 * e0 and a1 == 4 * a0 and i0 == 4 * i1
    a = W.make_workload("t", dtype="f32", d=8, n_experts=64, n_sub=1, inter_sub=1024,
                        req_tokens=[2], req_k=[8], k_max=8, seed=0, with_weights=False)
    b = W.split_workload(a, 4)
    assert (b.E, b.k_max, b.inter_sub) == (256, 32, 256)


def test_config1_recipe():
    wl = W.config("c1_tiny_f32")
    assert (wl.T, wl.d, wl.E, wl.inter_sub, wl.k_max, wl.pairs) == (64, 256, 32, 128, 8, 320)
    assert wl.k_tok.tolist() == [2] * 16 + [4] * 16 + [6] * 16 + [8] * 16
    assert abs(float(wl.w_router.std()) - 0.02) < 2e-3 and abs(float(wl.x.std()) - 1.0) < 2e-2
    b = W.round_to_bf16(np.array([1.00390625, 1.01171875, -3.0e38, 1e-40], np.float32))
    assert b.tolist()[:2] == [1.0, 1.015625]          # ties to even both ways


# ----------------------------------------------------------------- proxy gate (Sec. 3.2.2)
def proxy_fixture(seed=31, T=14, d=32, N=6, I=32, S=4, m=3, r=2, renorm=1):
    base = W.make_workload("whole", dtype="f32", d=d, n_experts=N, n_sub=1, inter_sub=I,
                           req_tokens=[T], req_k=[m], k_max=m, seed=seed, routed_scale=1.0,
                           w_std=0.3, renormalize=renorm)
    sp = W.split_workload(base, S)
    pg = W.make_proxy_gate(base, sp, m=m, r=r, seed=seed + 1)
    return base, sp, pg


def proxy_layer(sp, pg, k_tok, routed_scale=1.0):
    S = sp.n_sub
    k_max = pg.m * S
    ids, w = O.route_proxy(sp.x, pg.w_router0, pg.bias0, pg.w_proxy, k_tok, pg.kappa, S, pg.r,
                           pg.m, k_max, sp.renormalize, routed_scale)
    cnt, off, spair, slot = O.dispatch(ids, sp.E)
    y = O.grouped_ffn(sp.x, sp.w_gate_up, sp.w_down, off, spair, k_max)
    k_eff = (ids >= 0).sum(1).astype(np.int32)
    return O.combine(y, slot, w, k_eff, sp.T), ids, w


def test_proxy_scores_hand_computed():
    # d = 2, one expert, two sub-experts with one gate neuron each
    x = np.array([[1.0, 2.0]], np.float32)
    w_proxy = np.array([[[0.5, 0.25], [-1.0, 0.0],        # gate rows of sub-experts 0, 1
                         [2.0, 1.0], [1.0, 1.0]]], np.float32)   # their up rows
    ids0 = np.array([[0]], np.int32)
    s = O.proxy_scores(x, w_proxy, ids0, S=2, r=1)
    s0 = abs(1.0 / (1.0 + math.exp(-1.0)) * 4.0)          # a = 1, u = 4
    s1 = abs(-1.0 / (1.0 + math.exp(1.0)) * 3.0)          # a = -1, u = 3
    np.testing.assert_allclose(s[0, 0], [s0, s1], rtol=1e-15)
    kappa = np.array([[0], [1], [2]], np.int32)
    ids, w = O.proxy_select(s, ids0, np.array([[0.7]]), np.array([1], np.int32), kappa, 2)
    assert ids.tolist() == [[0, -1]] and w.tolist() == [[0.7, 0.0]]
    ids, w = O.proxy_select(s, ids0, np.array([[0.7]]), np.array([2], np.int32), kappa, 2)
    assert ids.tolist() == [[0, 1]] and w.tolist() == [[0.7, 0.7]]


def test_proxy_scores_with_every_neuron_equal_mean_abs_activation():
    # r = Is: the score is the mean |h_c| over the sub-expert, h from dense numpy code
    base, sp, _ = proxy_fixture(seed=33, S=4, I=32)
    S, Is, N, d = sp.n_sub, sp.inter_sub, sp.n_experts, sp.d
    w_proxy = np.empty((N, 2 * S * Is, d), np.float32)
    for e in range(N):
        w_proxy[e, :S * Is] = base.w_gate_up[e, :S * Is]            # gate rows, neuron order
        w_proxy[e, S * Is:] = base.w_gate_up[e, S * Is:]            # up rows
    ids0 = np.tile(np.arange(N, dtype=np.int32), (sp.T, 1))
    s = O.proxy_scores(sp.x, w_proxy, ids0, S=S, r=Is)
    x64 = sp.x.astype(np.float64)
    for e in range(N):
        a = x64 @ base.w_gate_up[e, :S * Is].astype(np.float64).T
        u = x64 @ base.w_gate_up[e, S * Is:].astype(np.float64).T
        h = np.abs(a / (1.0 + np.exp(-a)) * u).reshape(sp.T, S, Is).mean(2)
        np.testing.assert_allclose(s[:, e], h, rtol=1e-12)


def test_proxy_select_brute_force_and_ties():
    rng = np.random.default_rng(34)
    T, m, S = 40, 3, 5
    scores = rng.integers(0, 4, size=(T, m, S)).astype(np.float64)      # many exact ties
    ids0 = np.stack([rng.permutation(7)[:m] for _ in range(T)]).astype(np.int32)
    w0 = rng.random((T, m))
    kappa = np.array([[a, b, k - a - b] for k in range(m * S + 1)
                      for a, b in [(min(S, k), min(S, max(0, k - S)))]], np.int32)
    k_tok = rng.integers(0, m * S + 1, size=T).astype(np.int32)
    ids, w = O.proxy_select(scores, ids0, w0, k_tok, kappa, m * S)
    for t in range(T):
        pos = 0
        for j in range(m):
            kap = kappa[k_tok[t], j]
            got = ids[t, pos:pos + kap]
            assert np.all(got // S == ids0[t, j]) and np.all(w[t, pos:pos + kap] == w0[t, j])
            sub = (got % S).tolist()
            best = max(sum(scores[t, j, list(c)]) for c in itertools.combinations(range(S), kap))
            assert sum(scores[t, j, sub]) == best                         # an optimal subset
            # the unique order: score descending, equal scores by ascending index
            assert sub == sorted(range(S), key=lambda n: (-scores[t, j, n], n))[:kap]
            pos += kap
        assert pos == k_tok[t] and np.all(ids[t, pos:] == -1) and np.all(w[t, pos:] == 0)


@pytest.mark.parametrize("renorm", [0, 1])
def test_proxy_full_allocation_reconstructs_the_original_layer(renorm):
    # selecting all S sub-experts of every selected expert gives the undivided top-m MoE
    base, sp, pg = proxy_fixture(seed=35, renorm=renorm)
    k_tok = np.full(sp.T, pg.m * sp.n_sub, np.int32)
    out, ids, w = proxy_layer(sp, pg, k_tok)
    I = base.inter_sub
    ref = standard_topk_moe64(base.x, base.w_router, base.w_gate_up[:, :I], base.w_gate_up[:, I:],
                              base.w_down, pg.m, renorm, 1.0)
    np.testing.assert_allclose(out, ref, rtol=5e-5, atol=1e-8)
    for t in range(sp.T):
        experts = ids[t] // sp.n_sub
        assert sorted(ids[t].tolist()) == sorted(e * sp.n_sub + n for e in set(experts) for n in range(sp.n_sub))


def test_proxy_partial_budgets_follow_the_allocation_table():
    base, sp, pg = proxy_fixture(seed=36)
    S, m = sp.n_sub, pg.m
    rng = np.random.default_rng(36)
    k_tok = rng.integers(0, m * S + 1, size=sp.T).astype(np.int32)
    r = O.route_proxy(sp.x, pg.w_router0, pg.bias0, pg.w_proxy, k_tok, pg.kappa, S, pg.r, m, m * S,
                      1, 1.0, return_all=True)
    ids, w = r["ids"], r["w"]
    np.testing.assert_allclose(r["w0"].sum(1), 1.0, rtol=1e-12)          # renormalised over the m experts
    for t in range(sp.T):
        valid = ids[t][ids[t] >= 0]
        assert len(valid) == k_tok[t] == len(set(valid.tolist()))
        for j in range(m):
            mine = valid[valid // S == r["ids0"][t, j]]
            assert len(mine) == pg.kappa[k_tok[t], j]
            assert np.all(w[t][ids[t] // S == r["ids0"][t, j]][:len(mine)] == r["w0"][t, j])
        # each token's output is the weighted sum of exactly those sub-experts
    out, _, _ = proxy_layer(sp, pg, k_tok)
    for t in (0, 5, 9):
        ref = sum(w[t, i] * O.ffn_one(sp.x[t], sp.w_gate_up[ids[t, i]], sp.w_down[ids[t, i]])
                  for i in range(k_tok[t])) if k_tok[t] else np.zeros(sp.d)
        np.testing.assert_allclose(out[t], ref, rtol=1e-12, atol=1e-15)


def test_default_kappa_table():
    tab = W.default_kappa_table(8, 4)
    assert tab.shape == (33, 8) and np.array_equal(tab.sum(1), np.arange(33)) and tab.max() == 4
    assert tab[20].tolist() == [3, 3, 3, 3, 2, 2, 2, 2]
    assert np.all(np.diff(tab, axis=1) <= 0)          # never more for a lower-ranked expert
