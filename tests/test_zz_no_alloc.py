"""The entry point that allocates nothing (moe_prism_layer_static, for callers that cannot
call hipMalloc) against moe_prism_layer on a caller-owned workspace: same kernels, so the
outputs must be identical bit for bit; two calls in a row, the second on a smaller input, so
that whatever the first call left in the library's static workspace is still there."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import oracle as O
from paper_2510_19366_amd import binding as B
from paper_2510_19366_amd import workloads as W
from gpu_util import max_rel, to_np

pytestmark = pytest.mark.gpu


def _case(T, d, N, S, Is, k_max, dtype, seed):
    return W.make_workload(f"static_{T}", dtype=dtype, d=d, n_experts=N, n_sub=S, inter_sub=Is,
                           k_max=k_max, req_tokens=[T // 4] * 3 + [T - 3 * (T // 4)],
                           k_lo=1, k_hi=k_max, seed=seed, bias_std=0.5)


def _run_both(wl):
    dev = B.to_device(wl)
    shape = dev["shape"]
    n = C.c_size_t(0)
    assert B.lib().moe_prism_workspace_bytes(C.byref(shape), C.byref(n)) == 0
    assert n.value <= B.STATIC_WS_BYTES
    args = (shape, dev["x"], dev["w_router"], dev["router_bias"], dev["k_tok"], dev["w_gate_up"],
            dev["w_down"])
    out_static = torch.full((wl.T, wl.d), float("nan"), dtype=B.act_dtype(shape), device="cuda")
    B.moe_prism_layer_static(*args, out_static)
    ws = B.alloc_workspace(shape)
    out_ws = B.moe_prism_layer(*args, ws)
    torch.cuda.synchronize()
    return to_np(out_static), to_np(out_ws)


@pytest.mark.parametrize("dtype,tol", [("bf16", 2e-2), ("f32", 1e-4)])
def test_static_workspace_twice_second_smaller(dtype, tol):
    big = _case(700, 256, 6, 4, 96, 9, dtype, seed=11)
    small = _case(130, 256, 6, 4, 96, 9, dtype, seed=12)
    for wl in (big, small):
        got, want = _run_both(wl)
        assert np.array_equal(got, want), wl.name
        ref = O.layer_of(wl)
        assert max_rel(got, ref) <= tol


def test_static_workspace_refuses_large_shapes():
    lib = B.lib()
    s = B.make_shape(16384, 2048, 128, 4, 192, 32, "bf16")
    n = C.c_size_t(0)
    assert lib.moe_prism_workspace_bytes(C.byref(s), C.byref(n)) == 0 and n.value > B.STATIC_WS_BYTES
    dummy = torch.zeros(16, device="cuda")
    p = C.c_void_p(dummy.data_ptr())
    assert lib.moe_prism_layer_static(C.byref(s), p, p, None, p, p, p, p, None) == -3
