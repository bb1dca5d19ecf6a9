"""Helpers for the GPU parity tests (device memory via torch, nothing else)."""
import numpy as np
import torch

import paper_1706_00095_amd as cg


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def max_abs_rel(got, ref):
    """max_i |got_i - ref_i| / max(max_i |ref_i|, 1e-30): the parity metric for fp32 tensors."""
    got, ref = np.asarray(got, np.float64), np.asarray(ref, np.float64)
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def ws_tensor(nbytes):
    return torch.empty(max(nbytes, 16), dtype=torch.uint8, device="cuda") if nbytes else None


def conv_fwd(d, x, w, b, math=None):
    """math = None: cg_conv_fwd; otherwise cg_conv_fwd_math with that CG_MATH_* mode."""
    OH, OW = cg.cg_conv_out_shape(d)
    y = torch.full((d.N, d.M, OH, OW), float("nan"), device="cuda")
    ws = ws_tensor(cg.cg_conv_workspace_bytes(d, cg.CG_PASS_FWD))
    if math is None:
        cg.cg_conv_fwd(d, x, w, b, y, ws)
    else:
        cg.cg_conv_fwd_math(d, x, w, b, y, ws, math)
    return y


def conv_bwd_data(d, dy, w, math=None):
    dx = torch.full((d.N, d.C, d.H, d.W), float("nan"), device="cuda")
    ws = ws_tensor(cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_DATA))
    if math is None:
        cg.cg_conv_bwd_data(d, dy, w, dx, ws)
    else:
        cg.cg_conv_bwd_data_math(d, dy, w, dx, ws, math)
    return dx


def conv_bwd_weight(d, x, dy, math=None):
    dw = torch.full((d.M, d.C // d.groups, d.KH, d.KW), float("nan"), device="cuda")
    db = torch.full((d.M,), float("nan"), device="cuda")
    ws = ws_tensor(cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_WEIGHT))
    if math is None:
        cg.cg_conv_bwd_weight(d, x, dy, dw, db, ws)
    else:
        cg.cg_conv_bwd_weight_math(d, x, dy, dw, db, ws, math)
    return dw, db
