"""CPU-only checks of the library boundary: it loads, exports what include/cg.h declares,
rejects bad arguments before touching a GPU, and the implicit-GEMM index maps address
exactly the tensor elements the convolution definition names (and nothing out of bounds)."""
import ctypes as C
import itertools
import os
import re

import numpy as np
import pytest

import paper_1706_00095_amd as cg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in sorted(os.listdir(os.path.join(ROOT, "include"))))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cg_[a-z_0-9]+)\s*\(", text)))


def test_library_loads_and_exports_every_declared_symbol():
    lib = cg.lib()
    names = _declared_functions()
    assert len(names) >= 16
    for n in names:
        assert hasattr(lib, n), n
    assert set(cg.EXPORTS) == set(names)
    assert "gfx950" in cg.version()
    assert cg.strerror(cg.CG_ENOSPC) == "workspace too small"


def test_conv_out_shape_and_bad_descriptors():
    assert cg.cg_conv_out_shape(cg.conv_desc(256, 3, 227, 227, 96, 11, stride=4)) == (55, 55)
    assert cg.cg_conv_out_shape(cg.conv_desc(1, 96, 27, 27, 256, 5, pad=2, groups=2)) == (27, 27)
    for bad in (cg.conv_desc(1, 3, 4, 4, 4, 5), cg.conv_desc(1, 3, 8, 8, 4, 3, groups=2),
                cg.conv_desc(0, 3, 8, 8, 4, 3), cg.conv_desc(1, 3, 8, 8, 4, 3, stride=0)):
        with pytest.raises(cg.CgError) as e:
            cg.cg_conv_out_shape(bad)
        assert e.value.code == cg.CG_EINVAL
    # a tensor of 2^31 bytes or more is outside what the 32-bit offsets cover
    with pytest.raises(cg.CgError) as e:
        cg.cg_conv_out_shape(cg.conv_desc(4096, 256, 64, 64, 256, 3, pad=1))
    assert e.value.code == cg.CG_EUNSUPPORTED


def test_entry_points_reject_null_and_misaligned_arguments_without_launching():
    lib = cg.lib()
    d = cg.conv_desc(1, 3, 8, 8, 4, 3)
    assert lib.cg_conv_fwd(C.byref(d), None, None, None, None, None, 0, None) == cg.CG_EINVAL
    assert lib.cg_conv_fwd(C.byref(d), 4, 16, None, 32, None, 0, None) == cg.CG_EINVAL      # x misaligned
    assert lib.cg_conv_bwd_data(C.byref(d), None, 16, 32, None, 0, None) == cg.CG_EINVAL
    assert lib.cg_conv_bwd_weight(None, 16, 32, 48, None, None, 0, None) == cg.CG_EINVAL
    s = cg.cg_sgd(0.1, 0.9, 0.0, 1.0)
    assert lib.cg_grad_reduce_sgd(16, 32, 48, None, -1, 8, C.byref(s), None) == cg.CG_EINVAL
    assert lib.cg_grad_reduce_sgd(16, 32, 48, None, 65, 8, C.byref(s), None) == cg.CG_EINVAL
    assert lib.cg_grad_reduce_sgd(16, 32, 48, None, 2, 8, C.byref(s), None) == cg.CG_EINVAL   # K>0, no peers
    assert lib.cg_grad_reduce_sgd(16, 16, 48, None, 0, 8, C.byref(s), None) == cg.CG_EINVAL   # w aliases v
    assert lib.cg_grad_reduce_sgd(16, 4096, 32, None, 0, 8, C.byref(s), None) == cg.CG_EINVAL  # g_local inside w's range
    assert lib.cg_grad_reduce_sgd(4096, 16, 32, None, 0, 8, C.byref(s), None) == cg.CG_EINVAL  # g_local inside v's range
    peers = (C.c_void_p * 2)(8192, 4096 + 16)
    assert lib.cg_grad_reduce_sgd(4096, 16384, 32768, peers, 2, 8, C.byref(s), None) == cg.CG_EINVAL  # a peer overlaps w
    assert lib.cg_grad_reduce_sgd(16, 36, 48, None, 0, 8, C.byref(s), None) == cg.CG_EINVAL   # misaligned
    assert lib.cg_grad_reduce_sgd(None, None, None, None, 0, 0, C.byref(s), None) == cg.CG_OK  # n == 0: no-op
    assert lib.cg_grad_reduce_sgd(16, 32, 48, None, 0, 8, None, None) == cg.CG_EINVAL
    assert lib.cg_grad_reduce_sgd_tree(16, 32, 48, None, 65, 8, C.byref(s), None) == cg.CG_EINVAL
    assert lib.cg_grad_reduce_sgd_tree(16, 32, 48, None, 3, 8, C.byref(s), None) == cg.CG_EINVAL   # K>0, no peers
    assert lib.cg_grad_reduce_sgd_tree(16, 36, 48, None, 0, 8, C.byref(s), None) == cg.CG_EINVAL   # misaligned
    assert lib.cg_grad_reduce_sgd_tree(None, None, None, None, 0, 0, C.byref(s), None) == cg.CG_OK
    assert lib.cg_grad_reduce_sgd_tree_multi(1, None, None, None, None, 0, None, C.byref(s), None) == cg.CG_EINVAL


def test_workspace_sizes():
    d = cg.conv_desc(256, 256, 13, 13, 384, 3, pad=1)
    assert cg.cg_conv_workspace_bytes(d, cg.CG_PASS_FWD) == 384 * 256 * 9 * 4           # tap-major filter copy
    assert cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_DATA) >= 384 * 256 * 9 * 4      # transposed filters (+ K slices)
    ws = cg.cg_conv_workspace_bytes(d, cg.CG_PASS_BWD_WEIGHT)
    assert ws > 2 * 384 * 256 * 9 * 4                   # at least two K slices of dw + bias partials
    small = cg.conv_desc(2, 64, 13, 13, 64, 3, pad=1)
    assert cg.cg_conv_workspace_bytes(small, cg.CG_PASS_FWD) > 0                    # few tiles: K is sliced
    d1 = cg.conv_desc(256, 3, 227, 227, 96, 11, stride=4)
    # strided backward-data: the filters rearranged by stride phase, 48 rows x (96 channels x 3 x 3 taps)
    assert cg.cg_conv_workspace_bytes(d1, cg.CG_PASS_BWD_DATA) == 48 * 96 * 9 * 4
    # a single input channel at stride 2: four (channel, phase) rows, the kernel by stride phase, no workspace
    assert cg.cg_conv_workspace_bytes(cg.conv_desc(4, 1, 17, 17, 12, 3, stride=2, pad=1), cg.CG_PASS_BWD_DATA) == 0


CASES = [
    # N, C, H, W, M, KH, KW, stride, pad, groups
    (2, 4, 7, 6, 6, 3, 3, 1, 1, 2),
    (1, 3, 11, 13, 4, 5, 3, 2, 1, 1),
    (2, 2, 9, 9, 2, 3, 3, 3, 0, 1),
    (1, 6, 5, 4, 4, 1, 1, 1, 0, 2),
    (1, 3, 23, 23, 4, 11, 11, 4, 0, 1),
]


@pytest.mark.parametrize("case", CASES)
def test_forward_and_backward_weight_maps_address_the_definition(case):
    N, Cin, H, W, M, KH, KW, s, p, G = case
    d = cg.cg_conv_desc(N, Cin, H, W, M, KH, KW, s, s, p, p, G)
    OH, OW = cg.cg_conv_out_shape(d)
    Cg, Mg = Cin // G, M // G
    K = Cg * KH * KW
    Pp = (OH * OW + 3) // 4 * 4
    for g in range(G):
        # forward: A = filters, B = x gathered through the window
        for m, k in itertools.product(range(Mg), range(K)):
            off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_FWD, 0, m, k, g)
            assert ok and off == (g * Mg + m) * K + k
        for n, oh, ow in itertools.product(range(N), range(OH), range(OW)):
            row = (n * OH + oh) * OW + ow
            for c, kh, kw in itertools.product(range(Cg), range(KH), range(KW)):
                k = (c * KH + kh) * KW + kw
                ih, iw = oh * s - p + kh, ow * s - p + kw
                inside = 0 <= ih < H and 0 <= iw < W
                off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_FWD, 1, row, k, g)
                assert ok == inside
                if inside:
                    assert off == ((n * Cin + g * Cg + c) * H + ih) * W + iw
                # backward-weight swaps the roles: rows are filter taps, the reduction runs over pixels,
                # every image's pixels padded to a multiple of four in the index space
                off2, ok2 = cg.cg_debug_conv_operand(d, cg.CG_PASS_BWD_WEIGHT, 1, k, n * Pp + oh * OW + ow, g)
                assert ok2 == inside and (not inside or off2 == off)
        for k in (0, K - 1):
            for n, q in itertools.product(range(N), range(OH * OW, Pp)):
                assert not cg.cg_debug_conv_operand(d, cg.CG_PASS_BWD_WEIGHT, 1, k, n * Pp + q, g)[1]   # padding index
        for m in range(Mg):
            for n, q in itertools.product(range(N), range(OH * OW)):
                off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_BWD_WEIGHT, 0, m, n * Pp + q, g)
                assert ok and off == (n * M + g * Mg + m) * OH * OW + q


@pytest.mark.parametrize("case", [c for c in CASES if c[7] == 1])
def test_backward_data_maps_address_the_adjoint(case):
    N, Cin, H, W, M, KH, KW, s, p, G = case
    d = cg.cg_conv_desc(N, Cin, H, W, M, KH, KW, s, s, p, p, G)
    OH, OW = cg.cg_conv_out_shape(d)
    Cg, Mg = Cin // G, M // G
    Kp = Mg * KH * KW
    for g in range(G):
        for c, k in itertools.product(range(Cg), range(Kp)):
            off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_BWD_DATA, 0, c, k, g)
            if KH == 1 and KW == 1 and p == 0:
                assert ok and off == (g * Mg + k) * Cg + c          # w itself: no transposed copy for one tap
            else:
                assert ok and off == (g * Cg + c) * Kp + k
        for n, ih, iw in itertools.product(range(N), range(H), range(W)):
            row = (n * H + ih) * W + iw
            for ml, kh, kw in itertools.product(range(Mg), range(KH), range(KW)):
                k = (ml * KH + kh) * KW + kw
                oh, ow = ih + p - kh, iw + p - kw
                inside = 0 <= oh < OH and 0 <= ow < OW
                off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_BWD_DATA, 1, row, k, g)
                assert ok == inside
                if inside:
                    assert off == ((n * M + g * Mg + ml) * OH + oh) * OW + ow


def test_maps_at_alexnet_sizes_stay_in_bounds():
    """Corners and random samples of every AlexNet-shaped layer at B=256: valid elements lie
    inside their tensor (the kernels read offset 0 for invalid ones)."""
    import cg_synth
    rng = np.random.default_rng(0)
    for name, c in cg_synth.ALEXNET_CONVS.items():
        d = cg.conv_desc(256, c["C"], c["H"], c["H"], c["M"], c["k"], stride=c["stride"], pad=c["pad"],
                         groups=c["groups"])
        OH, OW = cg.cg_conv_out_shape(d)
        G = c["groups"]
        Cg, Mg = c["C"] // G, c["M"] // G
        K, NP = Cg * c["k"] ** 2, 256 * OH * OW
        Pp = (OH * OW + 3) // 4 * 4
        x_elems, y_elems = 256 * c["C"] * c["H"] ** 2, 256 * c["M"] * OH * OW
        rows = [0, NP - 1] + list(rng.integers(0, NP, 200))
        ks = [0, K - 1] + list(rng.integers(0, K, 20))
        for g in (0, G - 1):
            for row in rows:
                for k in ks:
                    off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_FWD, 1, int(row), int(k), g)
                    assert not ok or 0 <= off < x_elems
                    rowp = int(row) // (OH * OW) * Pp + int(row) % (OH * OW)       # the padded reduction index
                    off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_BWD_WEIGHT, 1, int(k), rowp, g)
                    assert not ok or 0 <= off < x_elems
                off, ok = cg.cg_debug_conv_operand(d, cg.CG_PASS_BWD_WEIGHT, 0, Mg - 1, rowp, g)
                assert ok and 0 <= off < y_elems
