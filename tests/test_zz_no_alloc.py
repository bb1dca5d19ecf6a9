"""The backward-weight entry point that takes no workspace (its partial sums live in a device array
of the library's own) against the entry point that takes the caller's: same kernels, same slices,
so the results must be identical bit for bit -- on two calls in a row, the second on a smaller
problem, which reuses the array with the first call's contents still in it."""
import numpy as np
import pytest
import torch

import cg_synth
import paper_1706_00095_amd as cg
from gpu_util import conv_bwd_weight, dev

pytestmark = pytest.mark.gpu

CASES = [
    # (B, cfg): first a reduction cut into many K slices with a bias gradient in two passes, then a smaller one
    (48, dict(C=32, H=13, M=384, k=3, stride=1, pad=1, groups=1)),
    (5, dict(C=16, H=9, W=11, M=40, k=3, stride=1, pad=1, groups=2)),
]


def _run(B, cfg, seed):
    c, x, w, b, dy = cg_synth.conv_layer_tensors("noalloc", B, seed=seed, cfg=cfg)
    Wd = c.get("W", c["H"])
    d = cg.conv_desc(B, c["C"], c["H"], Wd, c["M"], c["k"], stride=c["stride"], pad=c["pad"], groups=c["groups"])
    assert 0 < cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_WEIGHT) <= cg.CG_NOALLOC_SCRATCH_BYTES
    dx_, dy_ = dev(x), dev(dy)
    dw = torch.full((c["M"], c["C"] // c["groups"], c["k"], c["k"]), float("nan"), device="cuda")
    db = torch.full((c["M"],), float("nan"), device="cuda")
    cg.cg_conv_bwd_weight_noalloc(d, dx_, dy_, dw, db)
    torch.cuda.synchronize()
    return d, dx_, dy_, dw, db


def test_two_calls_in_a_row_match_the_workspace_entry_point():
    results = [_run(B, cfg, seed=70 + i) for i, (B, cfg) in enumerate(CASES)]     # both calls first ...
    for d, dx_, dy_, dw, db in results:                                            # ... then the references
        rw, rb = conv_bwd_weight(d, dx_, dy_)
        torch.cuda.synchronize()
        assert torch.isfinite(dw).all() and torch.isfinite(db).all()
        assert np.array_equal(dw.cpu().numpy().view(np.uint32), rw.cpu().numpy().view(np.uint32))
        assert np.array_equal(db.cpu().numpy().view(np.uint32), rb.cpu().numpy().view(np.uint32))


def test_a_problem_beyond_the_array_is_refused():
    """256 x 8192 gradients in 64 tiles, cut into 8 K slices: 64 MiB of partial sums plus the bias
    partials.  The call must return CG_ENOSPC and launch nothing (dw stays as it was)."""
    d = cg.conv_desc(64, 512, 16, 16, 256, 4, stride=1, pad=1, groups=1)
    assert cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_WEIGHT) > cg.CG_NOALLOC_SCRATCH_BYTES
    x = torch.zeros((64, 512, 16, 16), device="cuda")
    dy = torch.zeros((64, 256, 15, 15), device="cuda")
    dw = torch.full((256, 512, 4, 4), 7.0, device="cuda")
    with pytest.raises(cg.CgError) as e:
        cg.cg_conv_bwd_weight_noalloc(d, x, dy, dw, None)
    assert e.value.code == cg.CG_ENOSPC
    torch.cuda.synchronize()
    assert bool((dw == 7.0).all())
