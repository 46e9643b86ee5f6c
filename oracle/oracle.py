"""ctypes front end of the CPU oracle (``moe_prism_oracle.c``).

TEST INFRASTRUCTURE ONLY.  Importable from tests/, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``; the product path never touches it
and it never touches the product path.

All arrays are host numpy arrays.  Inputs (x, weights) are float32; for bf16
workloads they hold the exactly-widened bf16 values.  Logits are float32 (the
precision the routing decision is taken in); routing weights, FFN rows and
layer outputs are float64.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = C.CDLL(path)
    return _lib


def n_threads() -> int:
    """Threads the oracle's OpenMP loops use."""
    v = os.environ.get("OMP_NUM_THREADS")
    if v:
        return int(v.split(",")[0])
    return len(os.sched_getaffinity(0))


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def _f32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.float32)


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def logits(x, w_router, bias=None):
    """Router logits [T, E], float32 (Sec. 3.2.2, linear gate)."""
    x, w_router, bias = _f32(x), _f32(w_router), _f32(bias)
    T, d = x.shape
    E = w_router.shape[0]
    assert w_router.shape[1] == d
    out = np.empty((T, E), np.float32)
    rc = lib().oracle_logits(T, d, E, _p(x, C.c_float), _p(w_router, C.c_float),
                             _p(bias, C.c_float), _p(out, C.c_float))
    assert rc == 0
    return out


def select(lg, k_tok, k_max):
    """Per-token top-k_t ids [T, k_max] int32, -1 padded."""
    lg, k_tok = _f32(lg), _i32(k_tok)
    T, E = lg.shape
    ids = np.empty((T, k_max), np.int32)
    rc = lib().oracle_select(T, E, k_max, _p(lg, C.c_float), _p(k_tok, C.c_int32),
                             _p(ids, C.c_int32))
    if rc:
        raise ValueError("k_max > E")
    return ids


def weights(lg, ids, k_tok, renormalize, routed_scale):
    lg, ids, k_tok = _f32(lg), _i32(ids), _i32(k_tok)
    T, E = lg.shape
    k_max = ids.shape[1]
    w = np.empty((T, k_max), np.float64)
    rc = lib().oracle_weights(T, E, k_max, _p(lg, C.c_float), _p(ids, C.c_int32),
                              _p(k_tok, C.c_int32), int(renormalize),
                              C.c_double(routed_scale), _p(w, C.c_double))
    assert rc == 0
    return w


def dispatch(ids, E):
    """(cnt[E], off[E+1], sorted_pair[T*k_max], slot_of_pair[T*k_max])."""
    ids = _i32(ids)
    T, k_max = ids.shape
    cnt = np.empty(E, np.int32)
    off = np.empty(E + 1, np.int32)
    sp = np.empty(T * k_max, np.int32)
    sl = np.empty(T * k_max, np.int32)
    rc = lib().oracle_dispatch(T, E, k_max, _p(ids, C.c_int32), _p(cnt, C.c_int32),
                               _p(off, C.c_int32), _p(sp, C.c_int32), _p(sl, C.c_int32))
    if rc:
        raise ValueError("sub-expert id out of range")
    return cnt, off, sp, sl


def ffn_one(x_row, w_gu, w_dn):
    """One sub-expert ([2*Is, d], [d, Is]) applied to one token; float64 [d]."""
    x_row, w_gu, w_dn = _f32(x_row), _f32(w_gu), _f32(w_dn)
    d = x_row.shape[0]
    Is = w_dn.shape[1]
    assert w_gu.shape == (2 * Is, d) and w_dn.shape == (d, Is)
    y = np.empty(d, np.float64)
    lib().oracle_ffn_one(d, Is, _p(x_row, C.c_float), _p(w_gu, C.c_float),
                         _p(w_dn, C.c_float), _p(y, C.c_double))
    return y


def grouped_ffn(x, w_gate_up, w_down, off, sorted_pair, k_max):
    """y [P, d] float64, one row per slot."""
    x, w_gate_up, w_down = _f32(x), _f32(w_gate_up), _f32(w_down)
    off, sorted_pair = _i32(off), _i32(sorted_pair)
    T, d = x.shape
    E, twoIs, _ = w_gate_up.shape
    Is = twoIs // 2
    assert w_down.shape == (E, d, Is)
    P = int(off[E])
    y = np.empty((P, d), np.float64)
    lib().oracle_grouped_ffn(T, d, E, Is, k_max, _p(x, C.c_float), _p(w_gate_up, C.c_float),
                             _p(w_down, C.c_float), _p(off, C.c_int32),
                             _p(sorted_pair, C.c_int32), _p(y, C.c_double))
    return y


def combine(y, slot_of_pair, w, k_tok, T):
    y = np.ascontiguousarray(y, np.float64)
    w = np.ascontiguousarray(w, np.float64)
    slot_of_pair, k_tok = _i32(slot_of_pair), _i32(k_tok)
    d = y.shape[1]
    k_max = w.shape[1]
    out = np.empty((T, d), np.float64)
    lib().oracle_combine(T, d, k_max, _p(y, C.c_double), _p(slot_of_pair, C.c_int32),
                         _p(w, C.c_double), _p(k_tok, C.c_int32), _p(out, C.c_double))
    return out


def layer(x, w_router, bias, k_tok, w_gate_up, w_down, k_max, renormalize, routed_scale,
          return_all=False):
    """The whole path, stage by stage: route -> dispatch -> grouped FFN -> combine."""
    E = w_router.shape[0]
    lg = logits(x, w_router, bias)
    ids = select(lg, k_tok, k_max)
    w = weights(lg, ids, k_tok, renormalize, routed_scale)
    cnt, off, sp, sl = dispatch(ids, E)
    y = grouped_ffn(x, w_gate_up, w_down, off, sp, k_max)
    out = combine(y, sl, w, k_tok, x.shape[0])
    if return_all:
        return dict(logits=lg, ids=ids, w=w, cnt=cnt, off=off, sorted_pair=sp,
                    slot_of_pair=sl, y=y, out=out)
    return out


def layer_tokens(tokens, x, w_router, bias, k_tok, w_gate_up, w_down, k_max, renormalize,
                 routed_scale):
    """Layer output rows for the listed tokens only: (out[n,d] f64, ids[n,k_max], w[n,k_max])."""
    tokens = _i32(tokens)
    x, w_router, bias = _f32(x), _f32(w_router), _f32(bias)
    w_gate_up, w_down, k_tok = _f32(w_gate_up), _f32(w_down), _i32(k_tok)
    T, d = x.shape
    E, twoIs, _ = w_gate_up.shape
    Is = twoIs // 2
    n = len(tokens)
    out = np.empty((n, d), np.float64)
    ids = np.empty((n, k_max), np.int32)
    w = np.empty((n, k_max), np.float64)
    rc = lib().oracle_layer_tokens(n, _p(tokens, C.c_int32), d, E, Is, k_max, int(renormalize),
                                   C.c_double(routed_scale), _p(x, C.c_float),
                                   _p(w_router, C.c_float), _p(bias, C.c_float),
                                   _p(k_tok, C.c_int32), _p(w_gate_up, C.c_float),
                                   _p(w_down, C.c_float), _p(out, C.c_double),
                                   _p(ids, C.c_int32), _p(w, C.c_double))
    if rc:
        raise ValueError("k_max > E")
    return out, ids, w


def layer_of(wl, **kw):
    """Convenience: run ``layer`` on a workloads.Workload-shaped object."""
    return layer(wl.x, wl.w_router, wl.router_bias, wl.k_tok, wl.w_gate_up, wl.w_down,
                 wl.k_max, wl.renormalize, wl.routed_scale, **kw)


# ---------------------------------------------------------------- proxy gating (Sec. 3.2.2)
def proxy_scores(x, w_proxy, ids0, S, r):
    """scores [T, m, S] float64: mean |activation| of the r gate neurons of every
    sub-expert of the experts in ids0 [T, m].  w_proxy is [N, 2*S*r, d]."""
    x, w_proxy, ids0 = _f32(x), _f32(w_proxy), _i32(ids0)
    T, d = x.shape
    m = ids0.shape[1]
    assert w_proxy.shape[1] == 2 * S * r and w_proxy.shape[2] == d
    s = np.empty((T, m, S), np.float64)
    rc = lib().oracle_proxy_scores(T, d, S, r, m, _p(x, C.c_float), _p(w_proxy, C.c_float),
                                   _p(ids0, C.c_int32), _p(s, C.c_double))
    assert rc == 0
    return s


def proxy_select(scores, ids0, w0, k_tok, kappa, k_max):
    """ids [T, k_max] (flat sub-expert ids, -1 padded) and weights [T, k_max] float64."""
    scores = np.ascontiguousarray(scores, np.float64)
    w0 = np.ascontiguousarray(w0, np.float64)
    ids0, k_tok, kappa = _i32(ids0), _i32(k_tok), _i32(kappa)
    T, m, S = scores.shape
    assert S <= 64 and kappa.shape[1] == m
    ids = np.empty((T, k_max), np.int32)
    w = np.empty((T, k_max), np.float64)
    rc = lib().oracle_proxy_select(T, S, m, k_max, kappa.shape[0] - 1, _p(scores, C.c_double),
                                   _p(ids0, C.c_int32), _p(w0, C.c_double), _p(k_tok, C.c_int32),
                                   _p(kappa, C.c_int32), _p(ids, C.c_int32), _p(w, C.c_double))
    if rc:
        raise ValueError("allocation table entry outside [0, S]")
    return ids, w


def route_proxy(x, w_router0, bias0, w_proxy, k_tok, kappa, S, r, m, k_max, renormalize,
                routed_scale, return_all=False):
    """The whole proxy-gate route stage: (ids, w) over the N*S sub-experts."""
    T = x.shape[0]
    lg0 = logits(x, w_router0, bias0)
    k_m = np.full(T, m, np.int32)
    ids0 = select(lg0, k_m, m)
    w0 = weights(lg0, ids0, k_m, renormalize, routed_scale)
    sc = proxy_scores(x, w_proxy, ids0, S, r)
    ids, w = proxy_select(sc, ids0, w0, k_tok, kappa, k_max)
    if return_all:
        return dict(logits0=lg0, ids0=ids0, w0=w0, scores=sc, ids=ids, w=w)
    return ids, w
