"""Seeded synthetic inputs for the variable-k sub-expert MoE layer.

This module only draws random numbers and shapes them; it holds none of the
layer's arithmetic (no logits, no top-k, no FFN), so that both the CPU oracle
and the HIP path can be fed from it without sharing any method code.

The inputs stand in for the paper's serving workloads (Sec. 4.2: trace-shaped
requests, each carrying a routing budget k in sub-expert units; Table I model
shapes after a x4 split).  A workload is a set of requests; every token of a
request inherits the request's budget (Sec. 3.3.1), which yields the per-token
vector ``k_tok``.

Draw order is fixed: x, w_router, router_bias, w_gate_up, w_down, request k.
bf16 workloads are rounded once (round-to-nearest-even) to bf16; the fp32
arrays handed out are the exactly-widened bf16 values, so both sides see the
same real numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np

__all__ = [
    "Workload", "make_workload", "config", "CONFIG_NAMES", "round_to_bf16",
    "bf16_bits", "bf16_bits_to_f32", "expand_requests", "paper_k_targets",
    "repeat_router_rows",
]


def bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + r) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array whose values are all exactly representable in bf16."""
    return bf16_bits_to_f32(bf16_bits(a))


def expand_requests(req_k: np.ndarray, req_off: np.ndarray) -> np.ndarray:
    """Per-token budget from per-request budgets (token inherits its request's k)."""
    T = int(req_off[-1])
    k_tok = np.empty(T, dtype=np.int32)
    for r in range(len(req_k)):
        k_tok[req_off[r]:req_off[r + 1]] = req_k[r]
    return k_tok


def request_budgets(T, n_req, k_lo, k_hi, seed):
    """Per-request budgets in sub-expert units, uniform in [k_lo, k_hi], and their per-token
    expansion (equal-length requests)."""
    rng = np.random.default_rng(seed)
    req_k = rng.integers(k_lo, k_hi + 1, size=n_req).astype(np.int32)
    per = T // n_req
    k_tok = np.repeat(req_k, per)
    k_tok = np.concatenate([k_tok, np.full(T - k_tok.size, req_k[-1], np.int32)]).astype(np.int32)
    return req_k, k_tok


def paper_k_targets(rng: np.random.Generator, n: int, mu: float, sigma: float,
                    k_max: int) -> np.ndarray:
    """Budget generator of Sec. 4.2, Eq. 7: clip(round(N(mu, sigma^2)), 1, k_max)."""
    x = rng.normal(mu, sigma, size=n)
    return np.clip(np.rint(x), 1, k_max).astype(np.int32)


def repeat_router_rows(w_router: np.ndarray, S: int) -> np.ndarray:
    """Expanded linear gate initialisation (Sec. 3.2.2): every original row S times."""
    return np.repeat(w_router, S, axis=0)


@dataclass
class Workload:
    name: str
    dtype: str                 # "f32" or "bf16"
    T: int
    d: int
    n_experts: int             # N
    n_sub: int                 # S
    inter_sub: int             # Is
    k_max: int
    renormalize: int
    routed_scale: float
    x: np.ndarray              # [T, d] f32 (bf16-representable when dtype == "bf16")
    w_router: np.ndarray       # [E, d]
    router_bias: Optional[np.ndarray]   # [E] f32 or None
    w_gate_up: np.ndarray      # [E, 2*Is, d]  rows 0..Is-1 gate, Is..2Is-1 up
    w_down: np.ndarray         # [E, d, Is]
    req_k: np.ndarray          # [R] i32
    req_off: np.ndarray        # [R+1] i32
    k_tok: np.ndarray          # [T] i32
    meta: dict = field(default_factory=dict)

    @property
    def E(self) -> int:
        return self.n_experts * self.n_sub

    @property
    def pairs(self) -> int:
        return int(self.k_tok.sum())


def _normal(rng, shape, std, dtype):
    # chunked standard_normal keeps the peak footprint at one fp32 copy
    out = np.empty(shape, dtype=np.float32)
    flat = out.reshape(-1)
    step = 1 << 24
    for i in range(0, flat.size, step):
        n = min(step, flat.size - i)
        flat[i:i + n] = rng.standard_normal(n, dtype=np.float32) * np.float32(std)
    if dtype == "bf16":
        for i in range(0, flat.size, step):
            flat[i:i + step] = round_to_bf16(flat[i:i + step])
    return out


def make_workload(name: str, *, dtype: str, d: int, n_experts: int, n_sub: int,
                  inter_sub: int, req_tokens, req_k=None, k_lo: int = 1, k_hi: int = 1,
                  k_choices=None, k_max: Optional[int] = None, seed: int = 0,
                  bias_std: float = 0.0, bias_per_original_expert: bool = True,
                  renormalize: int = 1, routed_scale: Optional[float] = None,
                  w_std: float = 0.02, with_weights: bool = True) -> Workload:
    """Draw one workload.  ``req_tokens``: tokens per request (list or (R, n))."""
    rng = np.random.default_rng(seed)
    if isinstance(req_tokens, tuple):
        R, n = req_tokens
        req_tokens = [n] * R
    req_tokens = np.asarray(req_tokens, dtype=np.int64)
    R = len(req_tokens)
    req_off = np.zeros(R + 1, dtype=np.int32)
    req_off[1:] = np.cumsum(req_tokens)
    T = int(req_off[-1])
    E = n_experts * n_sub

    x = _normal(rng, (T, d), 1.0, dtype)
    w_router = _normal(rng, (E, d), w_std, dtype)
    bias = None
    if bias_std > 0.0:
        if bias_per_original_expert:
            b = rng.standard_normal(n_experts).astype(np.float32) * np.float32(bias_std)
            bias = np.repeat(b, n_sub).astype(np.float32)
        else:
            bias = rng.standard_normal(E).astype(np.float32) * np.float32(bias_std)
    if with_weights:
        w_gate_up = _normal(rng, (E, 2 * inter_sub, d), w_std, dtype)
        w_down = _normal(rng, (E, d, inter_sub), w_std, dtype)
    else:
        w_gate_up = np.zeros((0,), np.float32)
        w_down = np.zeros((0,), np.float32)
    if req_k is None:
        if k_choices is not None:
            req_k = rng.choice(np.asarray(k_choices, dtype=np.int32), size=R)
        else:
            req_k = rng.integers(k_lo, k_hi + 1, size=R)
    req_k = np.asarray(req_k, dtype=np.int32)
    assert len(req_k) == R
    if k_max is None:
        k_max = int(req_k.max()) if R else 1
    if routed_scale is None:
        routed_scale = float(n_sub)
    return Workload(name=name, dtype=dtype, T=T, d=d, n_experts=n_experts, n_sub=n_sub,
                    inter_sub=inter_sub, k_max=int(k_max), renormalize=int(renormalize),
                    routed_scale=float(routed_scale), x=x, w_router=w_router,
                    router_bias=bias, w_gate_up=w_gate_up, w_down=w_down, req_k=req_k,
                    req_off=req_off, k_tok=expand_requests(req_k, req_off),
                    meta={"seed": seed})


CONFIG_NAMES = ("c1_tiny_f32", "c2_mixtral_8x4", "c3_fine_128x4", "c4_decode_64x2",
                "c5a_s1_k8", "c5b_s4_k32", "c3_paper_k", "t1_olmoe_p", "t1_deepseek_p")


def config(name: str, *, T: Optional[int] = None, with_weights: bool = True,
           scale_down: int = 1) -> Workload:
    """The benchmark workloads.  ``scale_down`` divides the token count (and only
    that) to give the oracle a case of the same layer it finishes in seconds."""
    if name == "c1_tiny_f32":
        return make_workload(name, dtype="f32", d=256, n_experts=8, n_sub=4, inter_sub=128,
                             req_tokens=(4, 16), req_k=[2, 4, 6, 8], k_max=8, seed=0,
                             with_weights=with_weights)
    if name == "c2_mixtral_8x4":
        return make_workload(name, dtype="bf16", d=4096, n_experts=8, n_sub=4, inter_sub=3584,
                             req_tokens=(32, 128 // scale_down), k_lo=2, k_hi=8, k_max=8,
                             seed=2, with_weights=with_weights)
    if name == "c3_fine_128x4":
        return make_workload(name, dtype="bf16", d=2048, n_experts=128, n_sub=4, inter_sub=192,
                             req_tokens=(64, 256 // scale_down), k_lo=8, k_hi=32, k_max=32,
                             seed=3, bias_std=1.0, with_weights=with_weights)
    if name == "c3_paper_k":
        # the c3 layer with the paper's own budget generator (Sec. 4.2, Eq. 7): one budget per
        # request, clip(round(N(16, 5^2)), 1, 32); an extra workload, not one of the five configs
        req_k = paper_k_targets(np.random.default_rng(33), 64, 16.0, 5.0, 32)
        return make_workload(name, dtype="bf16", d=2048, n_experts=128, n_sub=4, inter_sub=192,
                             req_tokens=(64, 256 // scale_down), req_k=req_k, k_max=32,
                             seed=3, bias_std=1.0, with_weights=with_weights)
    if name in ("t1_olmoe_p", "t1_deepseek_p"):
        # the layer shapes of the paper's two other refactored models (Table I: 64 -> 256 routed
        # experts, 8 -> 32 resp. 6 -> 24 activated, intermediate 1024 -> 256 resp. 1408 -> 352;
        # hidden size 2048), random weights, per-request budgets uniform up to the activated count
        olmoe = name == "t1_olmoe_p"
        return make_workload(name, dtype="bf16", d=2048, n_experts=64, n_sub=4,
                             inter_sub=256 if olmoe else 352, req_tokens=(64, 256 // scale_down),
                             k_lo=8 if olmoe else 6, k_hi=32 if olmoe else 24,
                             k_max=32 if olmoe else 24, seed=11 if olmoe else 12,
                             with_weights=with_weights)
    if name == "c4_decode_64x2":
        return make_workload(name, dtype="bf16", d=2048, n_experts=64, n_sub=2, inter_sub=704,
                             req_tokens=(8192 // scale_down, 1), k_choices=[4, 12], k_max=12,
                             seed=4, with_weights=with_weights)
    if name in ("c5a_s1_k8", "c5b_s4_k32"):
        T = 16384 if T is None else T
        a = make_workload("c5a_s1_k8", dtype="bf16", d=2048, n_experts=128, n_sub=1,
                          inter_sub=768, req_tokens=(1, T), req_k=[8], k_max=8, seed=5,
                          routed_scale=1.0, with_weights=with_weights)
        if name == "c5a_s1_k8":
            return a
        return split_workload(a, 4)
    raise KeyError(name)


def split_workload(a: Workload, S: int) -> Workload:
    """The same layer with every expert cut into S contiguous neuron slices
    (Sec. 3.2.1, Eq. 3), the router rows repeated S times (Sec. 3.2.2), budgets
    multiplied by S and the routed scale multiplied by S (matched budget)."""
    assert a.n_sub == 1 and a.inter_sub % S == 0
    N, I, d = a.n_experts, a.inter_sub, a.d
    Is = I // S
    if a.w_gate_up.size:
        gu = a.w_gate_up.reshape(N, 2, S, Is, d).transpose(0, 2, 1, 3, 4)
        gu = np.ascontiguousarray(gu).reshape(N * S, 2 * Is, d)
        dn = a.w_down.reshape(N, d, S, Is).transpose(0, 2, 1, 3)
        dn = np.ascontiguousarray(dn).reshape(N * S, d, Is)
    else:
        gu, dn = a.w_gate_up, a.w_down
    bias = None if a.router_bias is None else np.repeat(a.router_bias, S)
    return Workload(name=f"{a.name}_split{S}", dtype=a.dtype, T=a.T, d=d, n_experts=N,
                    n_sub=S, inter_sub=Is, k_max=a.k_max * S, renormalize=a.renormalize,
                    routed_scale=a.routed_scale * S, x=a.x,
                    w_router=repeat_router_rows(a.w_router, S), router_bias=bias,
                    w_gate_up=gu, w_down=dn, req_k=a.req_k * S, req_off=a.req_off,
                    k_tok=a.k_tok * S, meta=dict(a.meta))


# ---------------------------------------------------------------- proxy gate inputs
def default_kappa_table(m: int, S: int) -> np.ndarray:
    """Allocation table of the proxy gate (Sec. 3.2.2): row k is (kappa_1..kappa_m) with
    sum k and 0 <= kappa_j <= S, for every budget k in 0..m*S.  The paper leaves the split
    to configuration; this one spreads the budget evenly and gives the remainder to the
    experts the router ranked first."""
    tab = np.zeros((m * S + 1, m), np.int32)
    for k in range(m * S + 1):
        base, rem = divmod(k, m)
        tab[k] = base + (np.arange(m) < rem)
    assert tab.max() <= S and np.array_equal(tab.sum(1), np.arange(m * S + 1))
    return tab


@dataclass
class ProxyGate:
    m: int                      # experts the original router selects
    r: int                      # gate neurons per sub-expert
    r_pad: int                  # S*r_pad is the padded row count per half of w_proxy (multiple of 32)
    w_router0: np.ndarray       # [N, d] original router
    bias0: Optional[np.ndarray]
    gate_neurons: np.ndarray    # [N*S, r] neuron indices inside each sub-expert
    w_proxy: np.ndarray         # [N, 2*S*r, d]   gate rows (sub-expert-major), then up rows
    kappa: np.ndarray           # [(m*S)+1, m]


def make_proxy_gate(whole: Workload, split: Workload, m: int, r: int, seed: int = 0) -> ProxyGate:
    """Synthetic proxy-gate metadata for `split` = split_workload(whole, S): r gate neurons
    drawn at random inside every sub-expert (the paper picks them by co-activation on
    calibration data, which does not exist here), their gate/up rows gathered per original
    expert, and the default allocation table."""
    assert whole.n_sub == 1 and split.n_experts == whole.n_experts
    N, S, Is, d = split.n_experts, split.n_sub, split.inter_sub, split.d
    rng = np.random.default_rng(seed)
    G = np.stack([np.sort(rng.choice(Is, size=r, replace=False)) for _ in range(N * S)]).astype(np.int32)
    w_proxy = np.empty((N, 2 * S * r, d), np.float32)
    for e in range(N):
        for n in range(S):
            g = e * S + n
            w_proxy[e, n * r:(n + 1) * r] = split.w_gate_up[g, G[g]]
            w_proxy[e, S * r + n * r:S * r + (n + 1) * r] = split.w_gate_up[g, Is + G[g]]
    return ProxyGate(m=m, r=r, r_pad=r, w_router0=whole.w_router, bias0=whole.router_bias,
                     gate_neurons=G, w_proxy=w_proxy, kappa=default_kappa_table(m, S))
