"""Helpers shared by the GPU parity tests: run the HIP path stage by stage through
the C ABI binding and bring the results back as numpy arrays."""
import numpy as np
import torch

from paper_2510_19366_amd import binding as B


def to_np(t):
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


def run_stages(wl, want_y=True):
    dev = B.to_device(wl)
    shape = dev["shape"]
    ws = B.alloc_workspace(shape)
    ids, w, lg = B.moe_prism_route(shape, dev["x"], dev["w_router"], dev["router_bias"],
                                   dev["k_tok"], ws, want_logits=True)
    flags, _ = B.moe_prism_status(ws)
    cnt, off, sp, sl = B.moe_prism_dispatch(shape, ids, ws)
    _, pairs = B.moe_prism_status(ws)
    y = B.moe_prism_grouped_ffn(shape, dev["x"], dev["w_gate_up"], dev["w_down"], off, sp, ws)
    out = B.moe_prism_combine(shape, y, sl, w, dev["k_tok"])
    torch.cuda.synchronize()
    r = dict(logits=to_np(lg), ids=to_np(ids), w=to_np(w), cnt=to_np(cnt), off=to_np(off),
             sorted_pair=to_np(sp), slot_of_pair=to_np(sl), out=to_np(out), flags=flags,
             pairs=pairs, dev=dev, ws=ws, shape=shape)
    if want_y:
        P = int(r["off"][-1])
        r["y"] = to_np(y[:P])
    return r


def run_layer(wl, dev=None, ws=None):
    dev = dev or B.to_device(wl)
    shape = dev["shape"]
    ws = ws if ws is not None else B.alloc_workspace(shape)
    out = B.moe_prism_layer(shape, dev["x"], dev["w_router"], dev["router_bias"], dev["k_tok"],
                            dev["w_gate_up"], dev["w_down"], ws)
    torch.cuda.synchronize()
    return out, dev, ws


def max_rel(got, ref):
    """max |got - ref| / max |ref| over the whole array (the layer tolerance's definition)."""
    ref = np.asarray(ref, np.float64)
    den = np.abs(ref).max() if ref.size else 1.0
    if den == 0:
        den = 1.0
    return float(np.abs(np.asarray(got, np.float64) - ref).max() / den) if ref.size else 0.0


def row_rel(got, ref):
    """Largest per-row error: max over rows of max|got_row - ref_row| / max|ref_row| (rows whose
    reference is all zero must be exactly zero).  Catches a wrong low-magnitude row that the
    whole-array figure of max_rel would hide."""
    got = np.asarray(got, np.float64).reshape(len(ref), -1)
    ref = np.asarray(ref, np.float64).reshape(len(ref), -1)
    if ref.size == 0:
        return 0.0
    num = np.abs(got - ref).max(axis=1)
    den = np.abs(ref).max(axis=1)
    zero = den == 0
    if np.any(num[zero] != 0):
        return float("inf")
    return float((num[~zero] / den[~zero]).max()) if np.any(~zero) else 0.0
