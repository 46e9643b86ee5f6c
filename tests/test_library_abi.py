"""Host-only checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2510_19366_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_exports_match_header():
    hdr = open(os.path.join(ROOT, "include", "moe_prism.h")).read()
    declared = set(re.findall(r"MOE_PRISM_API\s+[\w\s\*]+?\b(moe_prism_\w+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    lib = B.lib()
    for name in declared:
        assert hasattr(lib, name), name


def test_host_side_validation():
    lib = B.lib()
    n = C.c_size_t(0)
    ok = B.make_shape(64, 256, 8, 4, 128, 8, "f32")
    assert lib.moe_prism_workspace_bytes(C.byref(ok), C.byref(n)) == 0 and n.value > 0
    assert lib.moe_prism_workspace_bytes(C.byref(ok), None) == -1
    bad = [B.make_shape(64, 250, 8, 4, 128, 8, "f32"),        # d % 64
           B.make_shape(64, 256, 8, 4, 100, 8, "f32"),        # Is % 32
           B.make_shape(64, 256, 8, 4, 128, 33, "f32"),       # k_max > E
           B.make_shape(64, 256, 2048, 4, 128, 8, "f32")]     # E > 4096
    for s in bad:
        assert lib.moe_prism_workspace_bytes(C.byref(s), C.byref(n)) == -2
    neg = B.make_shape(-1, 256, 8, 4, 128, 8, "f32")
    assert lib.moe_prism_workspace_bytes(C.byref(neg), C.byref(n)) == -1
    # null pointers / missing workspace are refused on the host, nothing is launched
    assert lib.moe_prism_layer(C.byref(ok), None, None, None, None, None, None, None, None,
                               C.c_size_t(0), None) == -1
    assert lib.moe_prism_route(C.byref(ok), None, None, None, None, None, None, None, None,
                               C.c_size_t(0), None) == -1
    assert b"workspace" in lib.moe_prism_strerror(-3)
    # workspace grows with the pair capacity
    big = B.make_shape(128, 256, 8, 4, 128, 8, "f32")
    m = C.c_size_t(0)
    lib.moe_prism_workspace_bytes(C.byref(big), C.byref(m))
    assert m.value > n.value
    offs = B.moe_prism_layer_offsets(ok)
    assert all(v % 256 == 0 for v in offs.values()) and max(offs.values()) < n.value


def test_proxy_stage_that_would_overflow_the_tile_table_is_refused():
    # the proxy-gate stage cuts T*m pairs over N groups into the layer's tile table of
    # T*k_max/256 + E entries; a shape where they do not fit is refused on the host
    # (k_max = 2, m = 8: 2048 tiles needed, 1024 + 64 available)
    lib = B.lib()
    s = B.make_shape(65536, 256, 16, 4, 128, 2, "bf16")
    n = C.c_size_t(0)
    assert lib.moe_prism_workspace_bytes(C.byref(s), C.byref(n)) == 0
    dummy = (C.c_char * 256)()
    p = C.cast(dummy, C.c_void_p)
    rc = lib.moe_prism_route_proxy(C.byref(s), p, p, None, p, C.c_int32(8), C.c_int32(1),
                                   C.c_int32(32), p, p, p, p, p, C.c_size_t(n.value), None)
    assert rc == -2
    ok = B.make_shape(65536, 256, 16, 4, 128, 8, "bf16")          # m <= k_max always fits
    assert lib.moe_prism_workspace_bytes(C.byref(ok), C.byref(n)) == 0
    rc = lib.moe_prism_route_proxy(C.byref(ok), None, None, None, None, C.c_int32(8), C.c_int32(1),
                                   C.c_int32(32), None, None, None, None, None, C.c_size_t(0), None)
    assert rc == -1                                                 # passes the shape check, then null pointers
