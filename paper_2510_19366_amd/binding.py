"""Thin Python binding of the C ABI in ``include/moe_prism.h``.

Argument marshalling only: every function takes torch device tensors, passes
their raw pointers and the current torch stream to the entry point of the same
name, and returns the outputs.  No step of the path runs in Python or torch.
The library must be present: there is no fallback.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmoe_prism.so")

KERNEL_NAMES = ("logits", "topk", "dispatch_count", "dispatch_scan", "dispatch_place",
                "ffn_tiles", "ffn_gate_up", "ffn_down", "combine", "proxy_select", "ffn_fused",
                "ffn_traffic")

EXPORTS = ("moe_prism_workspace_bytes", "moe_prism_expand_k", "moe_prism_route",
           "moe_prism_dispatch", "moe_prism_grouped_ffn", "moe_prism_combine", "moe_prism_layer",
           "moe_prism_layer_static",
           "moe_prism_route_proxy", "moe_prism_layer_proxy", "moe_prism_plan_batches",
           "moe_prism_partition_greedy", "moe_prism_partition_objective", "moe_prism_partition_anneal",
           "moe_prism_layer_offsets", "moe_prism_status", "moe_prism_timing_enable",
           "moe_prism_timing_select", "moe_prism_timing_read", "moe_prism_microbench",
           "moe_prism_ffn_traffic_probe",
           "moe_prism_strerror")


class Shape(C.Structure):
    _fields_ = [("T", C.c_int32), ("d", C.c_int32), ("n_experts", C.c_int32),
                ("n_sub", C.c_int32), ("inter_sub", C.c_int32), ("k_max", C.c_int32),
                ("dtype", C.c_int32), ("renormalize", C.c_int32), ("routed_scale", C.c_float)]

    @property
    def E(self):
        return self.n_experts * self.n_sub


class MoePrismError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"moe_prism error {code}: {msg}")
        self.code = code


_lib = None


def lib():
    """Load the HIP library; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; "
                              "g.build()'` (the HIP library is required; there is no fallback)")
        _lib = C.CDLL(LIB_PATH)
        _lib.moe_prism_strerror.restype = C.c_char_p
        for name in EXPORTS:
            getattr(_lib, name)
    return _lib


def _check(rc):
    if rc != 0:
        raise MoePrismError(rc, lib().moe_prism_strerror(rc).decode())


def _ptr(t):
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def make_shape(T, d, n_experts, n_sub, inter_sub, k_max, dtype, renormalize=1, routed_scale=None):
    dt = {"f32": 0, "bf16": 1, torch.float32: 0, torch.bfloat16: 1, 0: 0, 1: 1}[dtype]
    if routed_scale is None:
        routed_scale = float(n_sub)
    return Shape(int(T), int(d), int(n_experts), int(n_sub), int(inter_sub), int(k_max), dt,
                 int(renormalize), float(routed_scale))


def act_dtype(shape):
    return torch.float32 if shape.dtype == 0 else torch.bfloat16


def moe_prism_workspace_bytes(shape) -> int:
    n = C.c_size_t(0)
    _check(lib().moe_prism_workspace_bytes(C.byref(shape), C.byref(n)))
    return n.value


def alloc_workspace(shape, device="cuda"):
    n = moe_prism_workspace_bytes(shape)
    ws = torch.empty(n + 256, dtype=torch.uint8, device=device)
    off = (-ws.data_ptr()) % 256
    return ws[off:off + n]


def moe_prism_expand_k(req_k, req_off, T):
    R = req_k.numel()
    k_tok = torch.empty(T, dtype=torch.int32, device=req_k.device)
    _check(lib().moe_prism_expand_k(R, int(T), _ptr(req_k), _ptr(req_off), _ptr(k_tok), _stream()))
    return k_tok


def moe_prism_route(shape, x, w_router, router_bias, k_tok, ws, want_logits=False):
    T, km = shape.T, shape.k_max
    ids = torch.empty((T, km), dtype=torch.int32, device=x.device)
    w = torch.empty((T, km), dtype=torch.float32, device=x.device)
    lg = torch.empty((T, shape.E), dtype=torch.float32, device=x.device) if want_logits else None
    _check(lib().moe_prism_route(C.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias),
                                 _ptr(k_tok), _ptr(ids), _ptr(w), _ptr(lg), _ptr(ws),
                                 C.c_size_t(ws.numel()), _stream()))
    return (ids, w, lg) if want_logits else (ids, w)


def moe_prism_dispatch(shape, topk_ids, ws):
    E, n = shape.E, shape.T * shape.k_max
    dev = topk_ids.device
    cnt = torch.empty(E, dtype=torch.int32, device=dev)
    off = torch.empty(E + 1, dtype=torch.int32, device=dev)
    sp = torch.empty(n, dtype=torch.int32, device=dev)
    sl = torch.empty(n, dtype=torch.int32, device=dev)
    _check(lib().moe_prism_dispatch(C.byref(shape), _ptr(topk_ids), _ptr(cnt), _ptr(off), _ptr(sp),
                                    _ptr(sl), _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return cnt, off, sp, sl


def moe_prism_grouped_ffn(shape, x, w_gate_up, w_down, group_offset, sorted_pair, ws, y=None):
    if y is None:
        y = torch.empty((shape.T * shape.k_max, shape.d), dtype=act_dtype(shape), device=x.device)
    _check(lib().moe_prism_grouped_ffn(C.byref(shape), _ptr(x), _ptr(w_gate_up), _ptr(w_down),
                                       _ptr(group_offset), _ptr(sorted_pair), _ptr(y), _ptr(ws),
                                       C.c_size_t(ws.numel()), _stream()))
    return y


def moe_prism_ffn_traffic_probe(shape, x, w_gate_up, w_down, group_offset, sorted_pair, ws, y):
    """The fused FFN kernel's memory operations alone (timed as kernel "ffn_traffic"); y is
    overwritten with values that mean nothing."""
    _check(lib().moe_prism_ffn_traffic_probe(C.byref(shape), _ptr(x), _ptr(w_gate_up), _ptr(w_down),
                                             _ptr(group_offset), _ptr(sorted_pair), _ptr(y),
                                             _ptr(ws), C.c_size_t(ws.numel()), _stream()))


def moe_prism_combine(shape, y, slot_of_pair, topk_w, k_tok, out=None):
    if out is None:
        out = torch.empty((shape.T, shape.d), dtype=act_dtype(shape), device=y.device)
    _check(lib().moe_prism_combine(C.byref(shape), _ptr(y), _ptr(slot_of_pair), _ptr(topk_w),
                                   _ptr(k_tok), _ptr(out), _stream()))
    return out


def moe_prism_layer(shape, x, w_router, router_bias, k_tok, w_gate_up, w_down, ws, out=None):
    if out is None:
        out = torch.empty((shape.T, shape.d), dtype=act_dtype(shape), device=x.device)
    _check(lib().moe_prism_layer(C.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias),
                                 _ptr(k_tok), _ptr(w_gate_up), _ptr(w_down), _ptr(out), _ptr(ws),
                                 C.c_size_t(ws.numel()), _stream()))
    return out


def ffn_path(shape):
    """Which grouped-FFN kernels moe_prism_grouped_ffn / _layer launch for this shape: "fused"
    (bf16, inter_sub in {64, 128, 192}, d >= 256, unless MOE_PRISM_FFN=split) or "split"."""
    ok = (shape.dtype == 1 and shape.inter_sub in (64, 128, 192) and shape.d % 64 == 0
          and shape.d >= 256 and shape.T * shape.d * 2 < 2 ** 32)
    return "fused" if ok and os.environ.get("MOE_PRISM_FFN") != "split" else "split"


STATIC_WS_BYTES = 64 << 20  # MOE_PRISM_STATIC_WS_BYTES


def moe_prism_layer_static(shape, x, w_router, router_bias, k_tok, w_gate_up, w_down, out):
    """moe_prism_layer on the library's own static device workspace: allocates nothing, so
    `out` is the caller's."""
    _check(lib().moe_prism_layer_static(C.byref(shape), _ptr(x), _ptr(w_router), _ptr(router_bias),
                                        _ptr(k_tok), _ptr(w_gate_up), _ptr(w_down), _ptr(out),
                                        _stream()))
    return out


def moe_prism_layer_offsets(shape):
    arr = (C.c_size_t * 8)()
    _check(lib().moe_prism_layer_offsets(C.byref(shape), arr))
    names = ("topk_ids", "topk_w", "group_count", "group_offset", "sorted_pair", "slot_of_pair",
             "y", "logits")
    return dict(zip(names, list(arr)))


def layer_intermediates(shape, ws):
    """Views of the tables moe_prism_layer left in ws (for tests)."""
    o = moe_prism_layer_offsets(shape)
    T, km, E = shape.T, shape.k_max, shape.E

    def view(name, n, dtype):
        nbytes = n * torch.empty((), dtype=dtype).element_size()
        return ws[o[name]:o[name] + nbytes].view(dtype)

    return dict(topk_ids=view("topk_ids", T * km, torch.int32).view(T, km),
                topk_w=view("topk_w", T * km, torch.float32).view(T, km),
                group_count=view("group_count", E, torch.int32),
                group_offset=view("group_offset", E + 1, torch.int32),
                sorted_pair=view("sorted_pair", T * km, torch.int32),
                slot_of_pair=view("slot_of_pair", T * km, torch.int32),
                logits=view("logits", T * E, torch.float32).view(T, E))


def moe_prism_status(ws):
    flags, pairs = C.c_int32(0), C.c_int32(0)
    _check(lib().moe_prism_status(_ptr(ws), C.byref(flags), C.byref(pairs), _stream()))
    return flags.value, pairs.value


def proxy_to_device(pg, dtype, device="cuda"):
    """Upload a workloads.ProxyGate: the original router, the gate-neuron rows padded to a
    multiple of 32 rows per half, and the allocation table."""
    import numpy as np
    from . import workloads as W

    def act(a):
        if dtype == "bf16":
            bits = W.bf16_bits(a).view(np.int16)
            return torch.from_numpy(bits).to(device).view(torch.bfloat16).reshape(a.shape)
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device)

    N, two_sr, d = pg.w_proxy.shape
    sr = two_sr // 2
    rows_half = (sr + 31) // 32 * 32
    padded = np.zeros((N, 2 * rows_half, d), np.float32)
    padded[:, :sr] = pg.w_proxy[:, :sr]
    padded[:, rows_half:rows_half + sr] = pg.w_proxy[:, sr:]
    return dict(w_router0=act(pg.w_router0),
                bias0=None if pg.bias0 is None else torch.from_numpy(pg.bias0).to(device),
                w_proxy=act(padded), rows_half=rows_half, m=pg.m, r=pg.r,
                kappa=torch.from_numpy(np.ascontiguousarray(pg.kappa, np.int32)).to(device))


def moe_prism_route_proxy(shape, x, pdev, k_tok, ws):
    """Proxy-gate route stage; pdev from proxy_to_device().  Returns (topk_ids, topk_w)."""
    T, km = shape.T, shape.k_max
    ids = torch.empty((T, km), dtype=torch.int32, device=x.device)
    w = torch.empty((T, km), dtype=torch.float32, device=x.device)
    _check(lib().moe_prism_route_proxy(C.byref(shape), _ptr(x), _ptr(pdev["w_router0"]),
                                       _ptr(pdev["bias0"]), _ptr(pdev["w_proxy"]),
                                       C.c_int32(pdev["m"]), C.c_int32(pdev["r"]),
                                       C.c_int32(pdev["rows_half"]), _ptr(pdev["kappa"]),
                                       _ptr(k_tok), _ptr(ids), _ptr(w), _ptr(ws),
                                       C.c_size_t(ws.numel()), _stream()))
    return ids, w


def moe_prism_layer_proxy(shape, x, pdev, k_tok, w_gate_up, w_down, ws, out=None):
    if out is None:
        out = torch.empty((shape.T, shape.d), dtype=act_dtype(shape), device=x.device)
    _check(lib().moe_prism_layer_proxy(C.byref(shape), _ptr(x), _ptr(pdev["w_router0"]),
                                       _ptr(pdev["bias0"]), _ptr(pdev["w_proxy"]),
                                       C.c_int32(pdev["m"]), C.c_int32(pdev["r"]),
                                       C.c_int32(pdev["rows_half"]), _ptr(pdev["kappa"]),
                                       _ptr(k_tok), _ptr(w_gate_up), _ptr(w_down), _ptr(out),
                                       _ptr(ws), C.c_size_t(ws.numel()), _stream()))
    return out


class TimeTable(C.Structure):
    _fields_ = [("n_n", C.c_int32), ("n_k", C.c_int32), ("n_grid", C.POINTER(C.c_int32)),
                ("k_grid", C.POINTER(C.c_int32)), ("ms", C.POINTER(C.c_float))]


def moe_prism_plan_batches(arrival, n_tokens, k_qos, M, n_grid, k_grid, ms):
    """Offline quality-tiered batching (host only, numpy in and out).
    Returns (batches, batch_k): lists of request indices per batch in dispatch order."""
    import numpy as np
    arrival = np.ascontiguousarray(arrival, np.float64)
    n_tokens = np.ascontiguousarray(n_tokens, np.int32)
    k_qos = np.ascontiguousarray(k_qos, np.int32)
    n_grid = np.ascontiguousarray(n_grid, np.int32)
    k_grid = np.ascontiguousarray(k_grid, np.int32)
    ms = np.ascontiguousarray(ms, np.float32)
    assert ms.shape == (n_grid.size, k_grid.size)
    R = int(k_qos.size)
    tab = TimeTable(n_grid.size, k_grid.size, n_grid.ctypes.data_as(C.POINTER(C.c_int32)),
                    k_grid.ctypes.data_as(C.POINTER(C.c_int32)),
                    ms.ctypes.data_as(C.POINTER(C.c_float)))
    order = np.empty(max(R, 1), np.int32)
    start = np.empty(R + 1, np.int32)
    bk = np.empty(max(R, 1), np.int32)
    nb = C.c_int32(0)
    _check(lib().moe_prism_plan_batches(
        C.c_int32(R), arrival.ctypes.data_as(C.POINTER(C.c_double)),
        n_tokens.ctypes.data_as(C.POINTER(C.c_int32)), k_qos.ctypes.data_as(C.POINTER(C.c_int32)),
        C.c_int32(int(M)), C.byref(tab), order.ctypes.data_as(C.POINTER(C.c_int32)),
        start.ctypes.data_as(C.POINTER(C.c_int32)), bk.ctypes.data_as(C.POINTER(C.c_int32)),
        C.byref(nb)))
    n = nb.value
    return [order[start[b]:start[b + 1]].tolist() for b in range(n)], bk[:n].tolist()


def _part_args(A):
    import numpy as np
    A = np.ascontiguousarray(A, np.float32)
    return A, A.ctypes.data_as(C.POINTER(C.c_float))


def moe_prism_partition_greedy(A, S):
    """Greedy initial partition (host only): group_of [C] int32."""
    import numpy as np
    A, pA = _part_args(A)
    g = np.empty(A.shape[1], np.int32)
    _check(lib().moe_prism_partition_greedy(C.c_int32(A.shape[0]), C.c_int32(A.shape[1]),
                                            C.c_int32(S), pA, g.ctypes.data_as(C.POINTER(C.c_int32))))
    return g


def moe_prism_partition_objective(A, group_of, S, k_in):
    import numpy as np
    A, pA = _part_args(A)
    g = np.ascontiguousarray(group_of, np.int32)
    loss = C.c_double(0.0)
    _check(lib().moe_prism_partition_objective(C.c_int32(A.shape[0]), C.c_int32(A.shape[1]),
                                               C.c_int32(S), C.c_int32(k_in), pA,
                                               g.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(loss)))
    return loss.value


def moe_prism_partition_anneal(A, group_of, S, k_in, steps, t0, t1, seed):
    """Simulated annealing from group_of (host only): (new group_of, loss)."""
    import numpy as np
    A, pA = _part_args(A)
    g = np.array(group_of, np.int32)
    loss = C.c_double(0.0)
    _check(lib().moe_prism_partition_anneal(C.c_int32(A.shape[0]), C.c_int32(A.shape[1]),
                                            C.c_int32(S), C.c_int32(k_in), pA,
                                            g.ctypes.data_as(C.POINTER(C.c_int32)),
                                            C.c_int64(int(steps)), C.c_double(t0), C.c_double(t1),
                                            C.c_uint64(int(seed)), C.byref(loss)))
    return g, loss.value


def moe_prism_timing_enable(on: bool):
    _check(lib().moe_prism_timing_enable(1 if on else 0))


def moe_prism_timing_select(names=None):
    """Time only the named kernels (KERNEL_NAMES); None = all."""
    mask = 0xFFFFFFFF if names is None else sum(1 << KERNEL_NAMES.index(n) for n in names)
    _check(lib().moe_prism_timing_select(C.c_uint32(mask)))


def moe_prism_timing_read():
    n = len(KERNEL_NAMES)
    ms = (C.c_float * n)()
    calls = (C.c_int32 * n)()
    _check(lib().moe_prism_timing_read(ms, calls))
    return {k: (ms[i], calls[i]) for i, k in enumerate(KERNEL_NAMES)}


class MicrobenchResult(C.Structure):
    _fields_ = [("name", C.c_char * 64), ("unit", C.c_char * 16), ("value", C.c_double),
                ("shader_mhz", C.c_double)]


def moe_prism_microbench(max_results=64):
    """Machine-peak microbenchmarks: list of (name, value, unit, shader MHz)."""
    res = (MicrobenchResult * max_results)()
    n = C.c_int32(0)
    _check(lib().moe_prism_microbench(C.c_int32(max_results), res, C.byref(n)))
    return [(res[i].name.decode(), res[i].value, res[i].unit.decode(), res[i].shader_mhz)
            for i in range(n.value)]


def to_device(wl, device="cuda"):
    """Upload a workloads.Workload (host numpy) as device tensors in its dtype."""
    import numpy as np
    from . import workloads as W

    def act(a):
        if wl.dtype == "bf16":
            bits = W.bf16_bits(a).view(np.int16)
            return torch.from_numpy(bits).to(device).view(torch.bfloat16).reshape(a.shape)
        return torch.from_numpy(np.ascontiguousarray(a, np.float32)).to(device)

    shape = make_shape(wl.T, wl.d, wl.n_experts, wl.n_sub, wl.inter_sub, wl.k_max, wl.dtype,
                       wl.renormalize, wl.routed_scale)
    t = dict(shape=shape, x=act(wl.x), w_router=act(wl.w_router),
             router_bias=None if wl.router_bias is None else torch.from_numpy(wl.router_bias).to(device),
             k_tok=torch.from_numpy(wl.k_tok).to(device),
             w_gate_up=act(wl.w_gate_up), w_down=act(wl.w_down))
    return t
