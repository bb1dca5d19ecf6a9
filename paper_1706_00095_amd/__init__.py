"""Python binding of libcg (argument marshalling only).

Every function has the name and the argument order of its C entry point in
include/cg.h.  Tensors are torch CUDA (ROCm) tensors used purely as device
memory; streams are torch.cuda.Stream objects (or None for the current
stream).  Nothing here computes: a missing or unloadable libcg.so raises.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("CG_LIB_PATH", os.path.join(_HERE, "libcg.so"))

CG_OK, CG_EINVAL, CG_ENOSPC, CG_EUNSUPPORTED, CG_EHIP = 0, -1, -2, -3, -4
CG_PASS_FWD, CG_PASS_BWD_DATA, CG_PASS_BWD_WEIGHT = 0, 1, 2
CG_STEP_OVERLAP, CG_STEP_SERIAL, CG_STEP_JOIN, CG_STEP_TREE_SUM, CG_STEP_BF16, CG_STEP_BF16X3 = 0, 1, 2, 4, 8, 16
CG_MATH_FP32, CG_MATH_BF16, CG_MATH_BF16X3 = 0, 1, 2
CG_MAX_PEERS = 64
CG_NOALLOC_SCRATCH_BYTES = 64 << 20
LAYER_KINDS = {"conv": 0, "relu": 1, "lrn": 2, "maxpool": 3, "avgpool": 4, "fc": 5, "dropout": 6,
               "concat": 7, "softmax_ce": 8}

EXPORTS = [
    "cg_conv_out_shape", "cg_conv_workspace_bytes", "cg_conv_fwd", "cg_conv_bwd_data", "cg_conv_bwd_weight", "cg_conv_bwd_weight_noalloc",
    "cg_conv_fwd_math", "cg_conv_bwd_data_math", "cg_conv_bwd_weight_math",
    "cg_grad_reduce_sgd", "cg_grad_reduce_sgd_multi", "cg_grad_reduce_sgd_tree", "cg_grad_reduce_sgd_tree_multi", "cg_net_create", "cg_net_destroy", "cg_net_param_count", "cg_net_layer_fused", "cg_net_bind",
    "cg_net_workspace_bytes", "cg_train_step", "cg_net_tensor", "cg_net_tensor_image_stride", "cg_strerror", "cg_version", "cg_last_hip_error", "cg_debug_conv_operand", "cg_debug_copy", "cg_debug_stream", "cg_debug_mfma_loop", "cg_debug_launch_count", "cg_debug_fuse_lrn_pool", "cg_debug_patch_min_tiles", "cg_debug_resident_blocks", "cg_debug_band_kernel",
    "cg_profile_enable", "cg_profile_count", "cg_profile_get",
]


class CgError(RuntimeError):
    def __init__(self, code, where):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} (code {code})")


class cg_conv_desc(C.Structure):
    _fields_ = [(n, C.c_int) for n in
                ("N", "C", "H", "W", "M", "KH", "KW", "stride_h", "stride_w", "pad_h", "pad_w", "groups")]


class cg_sgd(C.Structure):
    _fields_ = [("lr", C.c_float), ("mu", C.c_float), ("wd", C.c_float), ("grad_scale", C.c_float)]


class cg_layer_desc(C.Structure):
    _fields_ = [("kind", C.c_int), ("n_inputs", C.c_int), ("inputs", C.c_int * 4), ("conv", cg_conv_desc),
                ("k", C.c_int), ("stride", C.c_int), ("pad", C.c_int), ("lrn_size", C.c_int),
                ("lrn_alpha", C.c_float), ("lrn_beta", C.c_float), ("lrn_kappa", C.c_float),
                ("fc_out", C.c_int), ("drop_p", C.c_float)]


class cg_profile_record(C.Structure):
    _fields_ = [("kernel", C.c_char * 64), ("pass_", C.c_char * 32), ("layer", C.c_int), ("ms", C.c_float),
                ("flops", C.c_double), ("bytes", C.c_double)]


_lib = None


def lib():
    """The loaded shared library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = C.CDLL(LIB_PATH)
        vp, sz, ip = C.c_void_p, C.c_size_t, C.POINTER(C.c_int)
        dp = C.POINTER(cg_conv_desc)
        L.cg_conv_out_shape.argtypes = [dp, ip, ip]
        L.cg_conv_workspace_bytes.argtypes = [dp, C.c_int]
        L.cg_conv_workspace_bytes.restype = sz
        L.cg_conv_fwd.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.cg_conv_bwd_data.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        L.cg_conv_bwd_weight.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        L.cg_conv_bwd_weight_noalloc.argtypes = [dp, vp, vp, vp, vp, vp]
        L.cg_conv_fwd_math.argtypes = [dp, vp, vp, vp, vp, vp, sz, C.c_int, vp]
        L.cg_conv_bwd_data_math.argtypes = [dp, vp, vp, vp, vp, sz, C.c_int, vp]
        L.cg_conv_bwd_weight_math.argtypes = [dp, vp, vp, vp, vp, vp, sz, C.c_int, vp]
        L.cg_grad_reduce_sgd.argtypes = [vp, vp, vp, C.POINTER(vp), C.c_int, sz, C.POINTER(cg_sgd), vp]
        L.cg_grad_reduce_sgd_multi.argtypes = [C.c_int, C.POINTER(vp), C.POINTER(vp), C.POINTER(vp),
                                               C.POINTER(C.POINTER(vp)), C.c_int, C.POINTER(sz), C.POINTER(cg_sgd), vp]
        L.cg_grad_reduce_sgd_tree.argtypes = L.cg_grad_reduce_sgd.argtypes
        L.cg_grad_reduce_sgd_tree_multi.argtypes = L.cg_grad_reduce_sgd_multi.argtypes
        L.cg_net_create.argtypes = [C.POINTER(cg_layer_desc), C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                    C.POINTER(vp)]
        L.cg_net_destroy.argtypes = [vp]
        L.cg_debug_copy.argtypes = [vp, vp, sz, vp]
        L.cg_debug_stream.argtypes = [vp, vp, vp, sz, C.c_int, vp]
        L.cg_debug_mfma_loop.argtypes = [vp, C.c_int, C.c_int, vp]
        L.cg_debug_launch_count.restype = C.c_ulonglong
        L.cg_net_param_count.argtypes = [vp, C.c_int]
        L.cg_net_param_count.restype = C.c_longlong
        L.cg_net_layer_fused.argtypes = [vp, C.c_int]
        L.cg_net_layer_fused.restype = C.c_int
        L.cg_net_tensor_image_stride.argtypes = [vp, C.c_int]
        L.cg_net_tensor_image_stride.restype = C.c_longlong
        L.cg_net_bind.argtypes = [vp, C.c_int, vp, vp, vp, C.POINTER(vp), C.c_int]
        L.cg_net_workspace_bytes.argtypes = [vp]
        L.cg_net_workspace_bytes.restype = sz
        L.cg_train_step.argtypes = [vp, vp, vp, C.POINTER(vp), C.POINTER(cg_sgd), vp, sz, vp, vp, vp, C.c_int]
        L.cg_net_tensor.argtypes = [vp, C.c_int, C.c_int, vp, C.POINTER(vp), C.POINTER(sz)]
        L.cg_debug_conv_operand.argtypes = [dp, C.c_int, C.c_int, C.c_uint, C.c_uint, C.c_uint,
                                            C.POINTER(C.c_longlong), ip]
        L.cg_profile_enable.argtypes = [C.c_int]
        L.cg_profile_get.argtypes = [C.c_int, C.POINTER(cg_profile_record)]
        L.cg_strerror.argtypes = [C.c_int]
        L.cg_strerror.restype = C.c_char_p
        L.cg_version.restype = C.c_char_p
        L.cg_last_hip_error.restype = C.c_int
        _lib = L
    return _lib


def strerror(code):
    return lib().cg_strerror(code).decode()


def version():
    return lib().cg_version().decode()


def _check(rc, where):
    if rc != CG_OK:
        raise CgError(rc, where)


def _ptr(t):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError("expected a contiguous device tensor")
    return t.data_ptr()


def _stream(s):
    if s is None:
        s = torch.cuda.current_stream()
    return s.cuda_stream


def _ptr_array(tensors):
    arr = (C.c_void_p * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        arr[i] = _ptr(t)
    return arr


def conv_desc(N, Cin, H, W, M, KH, KW=None, stride=1, pad=0, groups=1):
    return cg_conv_desc(N, Cin, H, W, M, KH, KH if KW is None else KW, stride, stride, pad, pad, groups)


def cg_conv_out_shape(d):
    oh, ow = C.c_int(), C.c_int()
    _check(lib().cg_conv_out_shape(C.byref(d), C.byref(oh), C.byref(ow)), "cg_conv_out_shape")
    return oh.value, ow.value


def cg_conv_workspace_bytes(d, which):
    return int(lib().cg_conv_workspace_bytes(C.byref(d), which))


def _ws_args(ws):
    return (_ptr(ws), ws.numel() * ws.element_size()) if ws is not None else (None, 0)


def cg_conv_fwd(d, x, w, bias, y, ws=None, stream=None):
    _check(lib().cg_conv_fwd(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), *_ws_args(ws), _stream(stream)),
           "cg_conv_fwd")


def cg_conv_bwd_data(d, dy, w, dx, ws=None, stream=None):
    _check(lib().cg_conv_bwd_data(C.byref(d), _ptr(dy), _ptr(w), _ptr(dx), *_ws_args(ws), _stream(stream)),
           "cg_conv_bwd_data")


def cg_conv_bwd_weight(d, x, dy, dw, dbias, ws=None, stream=None):
    _check(lib().cg_conv_bwd_weight(C.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(dbias), *_ws_args(ws),
                                    _stream(stream)), "cg_conv_bwd_weight")


def cg_conv_fwd_math(d, x, w, bias, y, ws, math, stream=None):
    _check(lib().cg_conv_fwd_math(C.byref(d), _ptr(x), _ptr(w), _ptr(bias), _ptr(y), *_ws_args(ws), math, _stream(stream)),
           "cg_conv_fwd_math")


def cg_conv_bwd_data_math(d, dy, w, dx, ws, math, stream=None):
    _check(lib().cg_conv_bwd_data_math(C.byref(d), _ptr(dy), _ptr(w), _ptr(dx), *_ws_args(ws), math, _stream(stream)),
           "cg_conv_bwd_data_math")


def cg_conv_bwd_weight_math(d, x, dy, dw, dbias, ws, math, stream=None):
    _check(lib().cg_conv_bwd_weight_math(C.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(dbias), *_ws_args(ws), math,
                                         _stream(stream)), "cg_conv_bwd_weight_math")


def cg_conv_bwd_weight_noalloc(d, x, dy, dw, dbias, stream=None):
    _check(lib().cg_conv_bwd_weight_noalloc(C.byref(d), _ptr(x), _ptr(dy), _ptr(dw), _ptr(dbias), _stream(stream)),
           "cg_conv_bwd_weight_noalloc")


def _reduce_sgd(name, w, v, g_local, g_peers, n, sgd, stream):
    K = len(g_peers)
    _check(getattr(lib(), name)(_ptr(w), _ptr(v), _ptr(g_local), _ptr_array(g_peers), K, n, C.byref(sgd),
                                _stream(stream)), name)


def cg_grad_reduce_sgd(w, v, g_local, g_peers, n, sgd, stream=None):
    """g_peers: sequence of K device tensors; sgd: cg_sgd."""
    _reduce_sgd("cg_grad_reduce_sgd", w, v, g_local, g_peers, n, sgd, stream)


def cg_grad_reduce_sgd_tree(w, v, g_local, g_peers, n, sgd, stream=None):
    """The same arguments; the sum is taken in binomial-tree association."""
    _reduce_sgd("cg_grad_reduce_sgd_tree", w, v, g_local, g_peers, n, sgd, stream)


def cg_grad_reduce_sgd_tree_multi(ws, vs, gs, peers, ns, sgd, stream=None):
    """cg_grad_reduce_sgd_multi's arguments; the sums are taken in binomial-tree association."""
    cg_grad_reduce_sgd_multi(ws, vs, gs, peers, ns, sgd, stream, _name="cg_grad_reduce_sgd_tree_multi")


def cg_grad_reduce_sgd_multi(ws, vs, gs, peers, ns, sgd, stream=None, _name="cg_grad_reduce_sgd_multi"):
    """One launch for several buckets: ws, vs, gs sequences of device tensors, peers a sequence of
    sequences of K device tensors each, ns the element counts."""
    nb = len(ws)
    K = len(peers[0]) if nb else 0
    assert all(len(p) == K for p in peers)
    rows = [_ptr_array(p) for p in peers]
    table = (C.POINTER(C.c_void_p) * max(nb, 1))()
    for i, r in enumerate(rows):
        table[i] = C.cast(r, C.POINTER(C.c_void_p))
    counts = (C.c_size_t * max(nb, 1))(*ns)
    _check(getattr(lib(), _name)(nb, _ptr_array(ws), _ptr_array(vs), _ptr_array(gs), table, K, counts,
                                 C.byref(sgd), _stream(stream)), _name)


def cg_debug_patch_min_tiles(tiles):
    _check(lib().cg_debug_patch_min_tiles(int(tiles)), "cg_debug_patch_min_tiles")


def cg_debug_resident_blocks(blocks):
    _check(lib().cg_debug_resident_blocks(int(blocks)), "cg_debug_resident_blocks")


def cg_debug_band_kernel(on):
    _check(lib().cg_debug_band_kernel(int(bool(on))), "cg_debug_band_kernel")


def cg_debug_copy(dst, src, nbytes, stream=None):
    _check(lib().cg_debug_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)), "cg_debug_copy")


def cg_debug_fuse_lrn_pool(mode):
    _check(lib().cg_debug_fuse_lrn_pool(int(mode)), "cg_debug_fuse_lrn_pool")


def cg_debug_launch_count():
    return int(lib().cg_debug_launch_count())


def cg_debug_stream(dst, src, src2, nbytes, mode, stream=None):
    _check(lib().cg_debug_stream(_ptr(dst), _ptr(src), _ptr(src2), nbytes, mode, _stream(stream)), "cg_debug_stream")


def cg_debug_mfma_loop(out, blocks, iters, stream=None):
    _check(lib().cg_debug_mfma_loop(_ptr(out), blocks, iters, _stream(stream)), "cg_debug_mfma_loop")


def cg_debug_conv_operand(d, which_pass, operand, row, k, group):
    """(element offset in floats, valid) -- host-side evaluation, launches nothing."""
    off, ok = C.c_longlong(), C.c_int()
    _check(lib().cg_debug_conv_operand(C.byref(d), which_pass, operand, row, k, group, C.byref(off), C.byref(ok)),
           "cg_debug_conv_operand")
    return off.value, bool(ok.value)


def cg_profile_enable(on):
    _check(lib().cg_profile_enable(1 if on else 0), "cg_profile_enable")


def cg_profile_count():
    return int(lib().cg_profile_count())


def cg_profile_get(i):
    r = cg_profile_record()
    _check(lib().cg_profile_get(i, C.byref(r)), "cg_profile_get")
    return dict(kernel=r.kernel.decode(), pass_=r.pass_.decode(), layer=r.layer, ms=float(r.ms),
                flops=float(r.flops), bytes=float(r.bytes))


def layer_descs(layers):
    """cg_layer_desc array from the plain-dict layer list used throughout the tests."""
    arr = (cg_layer_desc * len(layers))()
    for i, ly in enumerate(layers):
        d = arr[i]
        d.kind = LAYER_KINDS[ly["kind"]]
        d.n_inputs = len(ly["inputs"])
        for k, s in enumerate(ly["inputs"]):
            d.inputs[k] = s
        if ly["kind"] == "conv":
            d.conv = cg_conv_desc(0, 0, 0, 0, ly["M"], ly["k"], ly["k"], ly["stride"], ly["stride"], ly["pad"],
                                  ly["pad"], ly["groups"])
        elif ly["kind"] == "maxpool":
            d.k, d.stride, d.pad = ly["k"], ly["stride"], ly["pad"]
        elif ly["kind"] == "lrn":
            d.lrn_size, d.lrn_alpha, d.lrn_beta, d.lrn_kappa = ly["size"], ly["alpha"], ly["beta"], ly["kappa"]
        elif ly["kind"] == "fc":
            d.fc_out = ly["out"]
        elif ly["kind"] == "dropout":
            d.drop_p = ly["p"]
    return arr


class Net:
    """Owner of a cg_net handle (cg_net_create / cg_net_destroy)."""

    def __init__(self, layers, B, in_shape):
        self.layers = layers
        self.B = B
        self.handle = C.c_void_p()
        descs = layer_descs(layers)
        _check(lib().cg_net_create(descs, len(layers), B, *in_shape, C.byref(self.handle)), "cg_net_create")
        self._keep = []

    def close(self):
        if self.handle:
            lib().cg_net_destroy(self.handle)
            self.handle = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def cg_net_param_count(net, layer):
    n = lib().cg_net_param_count(net.handle, layer)
    if n < 0:
        raise CgError(int(n), "cg_net_param_count")
    return int(n)


def cg_net_layer_fused(net, layer):
    r = lib().cg_net_layer_fused(net.handle, layer)
    if r < 0:
        raise CgError(int(r), "cg_net_layer_fused")
    return int(r)


def cg_net_bind(net, layer, w, v, g_local, g_peers):
    net._keep.append((w, v, g_local, list(g_peers)))
    _check(lib().cg_net_bind(net.handle, layer, _ptr(w), _ptr(v), _ptr(g_local), _ptr_array(g_peers), len(g_peers)),
           "cg_net_bind")


def cg_net_workspace_bytes(net):
    return int(lib().cg_net_workspace_bytes(net.handle))


def cg_train_step(net, x, labels, dropout_masks, sgd, ws, compute_stream, update_stream, loss_dev, flags=0):
    """dropout_masks: {layer index: uint8 device tensor} or None."""
    L = len(net.layers)
    marr = None
    if dropout_masks:
        marr = (C.c_void_p * L)()
        for i, t in dropout_masks.items():
            marr[i] = _ptr(t)
    _check(lib().cg_train_step(net.handle, _ptr(x), _ptr(labels), marr, C.byref(sgd), *_ws_args(ws),
                               _stream(compute_stream), update_stream.cuda_stream if update_stream is not None else None,
                               _ptr(loss_dev), flags), "cg_train_step")


def cg_net_tensor(net, layer, which, ws):
    """A float32 view (torch tensor sharing the workspace memory) of a layer's output or gradient."""
    p, n = C.c_void_p(), C.c_size_t()
    _check(lib().cg_net_tensor(net.handle, layer, which, _ptr(ws), C.byref(p), C.byref(n)), "cg_net_tensor")
    off = (p.value - ws.data_ptr()) // 4
    flat = ws.view(torch.float32)[off:off + n.value]
    if which == 0:
        stride = int(lib().cg_net_tensor_image_stride(net.handle, layer))
        per_image = n.value - (net.B - 1) * stride
        if per_image != stride:       # a channel slice of a wider tensor: gathered into a dense copy
            return torch.as_strided(flat, (net.B, per_image), (stride, 1)).reshape(-1)
    return flat
