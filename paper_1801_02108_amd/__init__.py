"""Thin Python binding of libsbnet_hip.so (see include/sbnet.h for the contract of every call).

Argument marshalling only: torch tensors supply device memory and the current stream; every
step of the path runs in the library's HIP kernels.  There is no CPU or PyTorch fallback: if
the shared library is missing, importing a symbol from it raises.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsbnet_hip.so")

F32, BF16, F16, U8 = 0, 1, 2, 3
POOL_MAX, POOL_AVG = 0, 1
OK, EINVAL, ECAP, EUNSUPPORTED, EHIP = 0, 1, 2, 3, 4

_DTYPES = {torch.float32: F32, torch.bfloat16: BF16, torch.float16: F16, torch.uint8: U8}


class SbnetError(RuntimeError):
    def __init__(self, code, text):
        super().__init__("sbnet status %d: %s" % (code, text))
        self.code = code


class Tuning(ctypes.Structure):
    """sbnet_tuning: the compute-tile choices the kernels make from the device-side count of active blocks."""
    _fields_ = [(n, ctypes.c_int) for n in (
        "unit_small_item_cost_eighths", "conv3_small_item_cost_eighths", "wgrad_split_factor_3x3", "wgrad_split_factor_1x1")]

    def asdict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class Geom(ctypes.Structure):
    """sbnet_geom: block extent, stride, origin and count along h and w."""
    _fields_ = [(n, ctypes.c_int) for n in (
        "bsize_h", "bsize_w", "bstride_h", "bstride_w", "boffset_h", "boffset_w", "bcount_h", "bcount_w")]

    def astuple(self):
        return tuple(getattr(self, n) for n, _ in self._fields_)


_lib = None
_vp, _ci, _sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
_gp = ctypes.POINTER(Geom)

_SIGNATURES = {
    "sbnet_last_error": (ctypes.c_char_p, []),
    "sbnet_set_tuning": (_ci, [ctypes.POINTER(Tuning)]),
    "sbnet_get_tuning": (_ci, [ctypes.POINTER(Tuning)]),
    "sbnet_geometry": (_ci, [_ci] * 8 + [_gp, _gp, ctypes.POINTER(_ci), ctypes.POINTER(_ci)]),
    "sbnet_coarse_geometry": (_ci, [_gp, _ci, _gp]),
    "sbnet_workspace_bytes": (_sz, [_ci, _gp]),
    "sbnet_reduce_mask": (_ci, [_vp, _ci, _ci, _ci, _ci, _gp, _ci, ctypes.c_float, _vp, _vp, _ci, _vp, _sz, _vp]),
    "sbnet_reduce_mask_static": (_ci, [_vp, _ci, _ci, _ci, _ci, _gp, _ci, ctypes.c_float, _vp, _vp, _ci, _vp]),
    "sbnet_read_count": (_ci, [_vp, _ci, ctypes.POINTER(_ci), _vp]),
    "sbnet_sparse_gather": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _vp, _vp]),
    "sbnet_sparse_scatter": (_ci, [_vp, _ci, _vp, _vp, _ci, _gp, _vp, _ci, _ci, _ci, _ci, _ci, _vp]),
    "sbnet_sparse_gather_chw": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _vp, _vp]),
    "sbnet_sparse_scatter_chw": (_ci, [_vp, _ci, _vp, _vp, _ci, _gp, _vp, _ci, _ci, _ci, _ci, _ci, _vp]),
    "sbnet_gather_backward_workspace_bytes": (_sz, [_ci, _gp]),
    "sbnet_sparse_gather_backward": (_ci, [_vp, _ci, _vp, _vp, _ci, _gp, _vp, _ci, _ci, _ci, _ci, _vp, _sz, _vp]),
    "sbnet_bn_stats_workspace_bytes": (_sz, [_ci, _ci]),
    "sbnet_sparse_bn_stats": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _vp, _vp, _vp, _sz, _vp]),
    "sbnet_sparse_bn_apply": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _vp, _vp, _vp, _vp, ctypes.c_float,
                                    _ci, _vp, _vp]),
    "sbnet_bn_backward_workspace_bytes": (_sz, [_ci, _ci]),
    "sbnet_sparse_bn_backward": (_ci, [_vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _vp, _vp, _vp, _vp,
                                       ctypes.c_float, _ci, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sbnet_relu_backward_on_tiles": (_ci, [_vp, _vp, _ci, _vp, _ci, _sz, _vp, _vp]),
    "sbnet_bias_backward_workspace_bytes": (_sz, [_ci, _ci]),
    "sbnet_bias_backward_on_tiles": (_ci, [_vp, _ci, _vp, _ci, _ci, _ci, _vp, _vp, _sz, _vp]),
    "sbnet_relu_bias_backward_on_tiles": (_ci, [_vp, _vp, _ci, _vp, _ci, _ci, _ci, _vp, _vp, _vp, _sz, _vp]),
    "sbnet_quantize_f8": (_ci, [_vp, _ci, _sz, ctypes.c_float, _vp, _vp]),
    "sbnet_pack_weights_f8": (_ci, [_vp, _ci, _ci, _ci, _ci, _vp, ctypes.POINTER(_sz), _vp]),
    "sbnet_conv_on_tiles_f8": (_ci, [_vp, _vp, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _ci,
                                     ctypes.c_float, _vp, _vp]),
    "sbnet_bottleneck_forward_keep_on_tiles": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _vp, _vp, _vp, _vp,
                                                     _vp, _vp, _vp, _vp, _vp, _vp]),
    "sbnet_bottleneck_backward_workspace_bytes": (_sz, [_ci, _ci, _ci, _ci, _ci, _ci]),
    "sbnet_bottleneck_backward_on_tiles": (_ci, [_vp, _vp, _vp, _vp, _ci, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _vp,
                                                 _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _sz, _vp]),
    "sbnet_pack_weights": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, ctypes.POINTER(_sz), _vp]),
    "sbnet_pack_weights_transposed": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, ctypes.POINTER(_sz), _vp]),
    "sbnet_conv_backward_data_workspace_bytes": (_sz, [_ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci]),
    "sbnet_conv_on_tiles_backward_data": (_ci, [_vp, _ci, _vp, _ci, _ci, _ci, _ci, _vp, _ci, _ci, _ci, _ci, _ci, _vp,
                                                _vp, _sz, _vp]),
    "sbnet_conv_backward_weights_workspace_bytes": (_sz, [_ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci]),
    "sbnet_conv_on_tiles_backward_weights": (_ci, [_vp, _vp, _ci, _vp, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _vp,
                                                   _vp, _sz, _vp]),
    "sbnet_conv_on_tiles": (_ci, [_vp, _ci, _vp, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _ci, _vp, _vp]),
    "sbnet_sparse_conv": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _gp, _vp, _vp,
                                _ci, _ci, _ci, _ci, _ci, _ci, _vp, _ci, _ci, _ci, _vp]),
    "sbnet_block_flags_bytes": (_sz, [_ci, _gp]),
    "sbnet_block_flags": (_ci, [_vp, _ci, _ci, _ci, _ci, _gp, _ci, ctypes.c_float, _vp, _sz, _vp]),
    "sbnet_sparse_conv_from_flags": (_ci, [_vp, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _gp, _vp, _vp,
                                           _ci, _ci, _ci, _ci, _ci, _ci, _vp, _ci, _ci, _ci, _vp]),
    "sbnet_sparse_conv_from_mask": (_ci, [_vp, _ci, _ci, _ci, _gp, _ci, ctypes.c_float, _vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci,
                                          _gp, _gp, _vp, _vp, _ci, _ci, _ci, _ci, _ci, _ci, _vp, _ci, _ci, _ci, _vp, _sz, _vp]),
    "sbnet_sparse_unit_workspace_bytes": (_sz, [_ci, _ci, _gp, _gp, _ci, _ci, _ci]),
    "sbnet_sparse_unit": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _gp, _vp, _vp, _vp, _vp, _vp,
                                _vp, _vp, _vp, _vp, _ci, _ci, _vp, _sz, _vp]),
    "sbnet_zero_outside": (_ci, [_vp, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _vp]),
    "sbnet_bottleneck_on_tiles": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _gp,
                                        _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "sbnet_sparse_bottleneck": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _gp,
                                      _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "sbnet_bottleneck_on_tiles_preact": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _gp,
                                               _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
    "sbnet_sparse_bottleneck_preact": (_ci, [_vp, _ci, _ci, _ci, _ci, _ci, _ci, _vp, _vp, _ci, _gp, _gp,
                                             _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp, _vp]),
}


def exported_symbols():
    """Names include/sbnet.h declares; the loader resolves each of them."""
    return sorted(_SIGNATURES)


def lib():
    """Load libsbnet_hip.so (built by build.py / __graft_entry__.build()); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("%s not found: run `python -m paper_1801_02108_amd.build` first" % LIB_PATH)
        l = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in _SIGNATURES.items():
            fn = getattr(l, name)
            fn.restype, fn.argtypes = res, args
        _lib = l
    return _lib


def get_tuning():
    """The compute-tile choices in force, as a dict."""
    t = Tuning()
    _check(lib().sbnet_get_tuning(ctypes.byref(t)))
    return t.asdict()


def set_tuning(**kw):
    """Change some of the compute-tile choices (keyword = field of sbnet_tuning); no keyword restores the defaults.
    Returns what is in force afterwards."""
    if not kw:
        _check(lib().sbnet_set_tuning(None))
        return get_tuning()
    t = Tuning()
    _check(lib().sbnet_get_tuning(ctypes.byref(t)))
    for k, v in kw.items():
        if k not in dict(Tuning._fields_):
            raise KeyError(k)
        setattr(t, k, int(v))
    _check(lib().sbnet_set_tuning(ctypes.byref(t)))
    return get_tuning()


def _check(code):
    if code != OK:
        raise SbnetError(code, lib().sbnet_last_error().decode())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _dev(t, name, dtype=None):
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise TypeError("%s must be a contiguous device tensor" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must be %s" % (name, dtype))
    return t


def _dt(t):
    try:
        return _DTYPES[t.dtype]
    except KeyError:
        raise TypeError("unsupported dtype %s" % t.dtype)


# ---------------------------------------------------------------------------------------------
def geometry(H, W, k, s, bo):
    """(g_in, g_out, H_out, W_out) for a k x k, stride-s SAME convolution with bo x bo output blocks."""
    g_in, g_out, ho, wo = Geom(), Geom(), _ci(), _ci()
    _check(lib().sbnet_geometry(H, W, k, k, s, s, bo, bo, g_in, g_out, ho, wo))
    return g_in, g_out, ho.value, wo.value


def coarse_geometry(g, factor):
    """Geometry of the same block windows on a map `factor` times coarser (sbnet_coarse_geometry)."""
    c = Geom()
    _check(lib().sbnet_coarse_geometry(g, factor, c))
    return c


def workspace_bytes(N, g):
    return int(lib().sbnet_workspace_bytes(N, g))


def reduce_mask(mask, g, pool=POOL_AVG, threshold=0.0, indices=None, count=None, workspace=None):
    """mask [N,H,W] u8/f32 -> (indices int32 [cap,3], count int32 [1]) on the device."""
    _dev(mask, "mask")
    N, H, W = mask.shape
    cap = N * g.bcount_h * g.bcount_w if indices is None else indices.shape[0]
    if indices is None:
        indices = torch.empty((cap, 3), dtype=torch.int32, device=mask.device)
    if count is None:
        count = torch.empty((1,), dtype=torch.int32, device=mask.device)
    need = workspace_bytes(N, g)
    if workspace is None:
        workspace = torch.empty((need,), dtype=torch.uint8, device=mask.device)
    _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32), _dev(workspace, "workspace")
    _check(lib().sbnet_reduce_mask(_ptr(mask), _dt(mask), N, H, W, g, pool, float(threshold), _ptr(indices),
                                   _ptr(count), cap, _ptr(workspace), workspace.numel() * workspace.element_size(),
                                   _stream()))
    return indices, count


def reduce_mask_static(mask, g, indices, count, pool=POOL_AVG, threshold=0.0):
    """reduce_mask without a workspace argument (the library's built-in scratch): the caller passes every
    buffer, nothing is allocated on the way.  Returns (indices, count) as passed."""
    _dev(mask, "mask"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W = mask.shape
    _check(lib().sbnet_reduce_mask_static(_ptr(mask), _dt(mask), N, H, W, g, pool, float(threshold), _ptr(indices),
                                          _ptr(count), indices.shape[0], _stream()))
    return indices, count


def read_count(count, cap):
    out = _ci()
    _check(lib().sbnet_read_count(_ptr(count), cap, out, _stream()))
    return out.value


def sparse_gather(x, indices, count, g, tiles=None):
    """x [N,H,W,C] -> tiles [cap, bsize_h, bsize_w, C]; rows beyond the active count are untouched."""
    _dev(x, "x"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = x.shape
    cap = indices.shape[0]
    if tiles is None:
        tiles = torch.empty((cap, g.bsize_h, g.bsize_w, C), dtype=x.dtype, device=x.device)
    _dev(tiles, "tiles", x.dtype)
    assert tiles.shape == (cap, g.bsize_h, g.bsize_w, C)
    _check(lib().sbnet_sparse_gather(_ptr(x), _dt(x), N, H, W, C, _ptr(indices), _ptr(count), cap, g, _ptr(tiles),
                                     _stream()))
    return tiles


def sparse_scatter(tiles, indices, count, g, y, add=False):
    """tiles [cap, bsize_h, bsize_w, C] -> written or added into y [N,H,W,C] in place; returns y."""
    _dev(tiles, "tiles"), _dev(y, "y", tiles.dtype)
    _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = y.shape
    cap = indices.shape[0]
    assert tiles.shape == (cap, g.bsize_h, g.bsize_w, C), (tuple(tiles.shape), (cap, g.bsize_h, g.bsize_w, C))
    _check(lib().sbnet_sparse_scatter(_ptr(tiles), _dt(tiles), _ptr(indices), _ptr(count), cap, g, _ptr(y), N, H, W,
                                      C, int(bool(add)), _stream()))
    return y


def sparse_gather_chw(x, indices, count, g, tiles=None):
    """Gather with the transpose fused in: x [N,H,W,C] -> channel-major tiles [cap,C,h,w]."""
    _dev(x, "x"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = x.shape
    cap = indices.shape[0]
    if tiles is None:
        tiles = torch.empty((cap, C, g.bsize_h, g.bsize_w), dtype=x.dtype, device=x.device)
    _dev(tiles, "tiles", x.dtype)
    assert tiles.shape == (cap, C, g.bsize_h, g.bsize_w)
    _check(lib().sbnet_sparse_gather_chw(_ptr(x), _dt(x), N, H, W, C, _ptr(indices), _ptr(count), cap, g, _ptr(tiles),
                                         _stream()))
    return tiles


def sparse_scatter_chw(tiles, indices, count, g, y, add=False):
    """Scatter (or scatter-add) of channel-major tiles [cap,C,h,w] into y [N,H,W,C] in place; returns y."""
    _dev(tiles, "tiles"), _dev(y, "y", tiles.dtype)
    _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = y.shape
    cap = indices.shape[0]
    assert tiles.shape == (cap, C, g.bsize_h, g.bsize_w)
    _check(lib().sbnet_sparse_scatter_chw(_ptr(tiles), _dt(tiles), _ptr(indices), _ptr(count), cap, g, _ptr(y), N, H, W,
                                          C, int(bool(add)), _stream()))
    return y


def sparse_gather_backward(dtiles, indices, count, g, dx, workspace=None):
    """Gradient of sparse_gather: adds the tile gradients [cap,h,w,C] (overlapping halos included) into dx [N,H,W,C]."""
    _dev(dtiles, "dtiles"), _dev(dx, "dx", dtiles.dtype)
    _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = dx.shape
    cap = indices.shape[0]
    assert dtiles.shape == (cap, g.bsize_h, g.bsize_w, C)
    need = lib().sbnet_gather_backward_workspace_bytes(N, g)
    if workspace is None:
        workspace = torch.empty((max(need, 4),), dtype=torch.uint8, device=dx.device)
    _dev(workspace, "workspace", torch.uint8)
    _check(lib().sbnet_sparse_gather_backward(_ptr(dtiles), _dt(dtiles), _ptr(indices), _ptr(count), cap, g, _ptr(dx),
                                              N, H, W, C, _ptr(workspace), workspace.numel(), _stream()))
    return dx


def sparse_bn_stats(x, indices, count, g, workspace=None):
    """Per-channel mean and biased variance of x [N,H,W,C] over the pixels of the active blocks; returns (mean, var)."""
    _dev(x, "x"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = x.shape
    cap = indices.shape[0]
    need = lib().sbnet_bn_stats_workspace_bytes(cap, C)
    if workspace is None:
        workspace = torch.empty((max(need, 4),), dtype=torch.uint8, device=x.device)
    _dev(workspace, "workspace", torch.uint8)
    mean = torch.empty((C,), dtype=torch.float32, device=x.device)
    var = torch.empty((C,), dtype=torch.float32, device=x.device)
    _check(lib().sbnet_sparse_bn_stats(_ptr(x), _dt(x), N, H, W, C, _ptr(indices), _ptr(count), cap, g, _ptr(mean),
                                       _ptr(var), _ptr(workspace), workspace.numel(), _stream()))
    return mean, var


def _vec(t, name, C):
    if t is not None:
        _dev(t, name, torch.float32)
        assert t.shape == (C,)
    return _ptr(t)


def sparse_bn_apply(x, indices, count, g, mean, var, gamma=None, beta=None, eps=1e-5, relu=False, y=None):
    """y = act(gamma (x - mean) / sqrt(var + eps) + beta) on the pixels of the active blocks, y untouched elsewhere
    (y defaults to x: in place); returns y."""
    _dev(x, "x"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = x.shape
    if y is None:
        y = x
    _dev(y, "y", x.dtype)
    assert y.shape == x.shape
    _check(lib().sbnet_sparse_bn_apply(_ptr(x), _dt(x), N, H, W, C, _ptr(indices), _ptr(count), indices.shape[0], g,
                                       _vec(mean, "mean", C), _vec(var, "var", C), _vec(gamma, "gamma", C),
                                       _vec(beta, "beta", C), float(eps), int(bool(relu)), _ptr(y), _stream()))
    return y


def sparse_bn_backward(x, dy, indices, count, g, mean, var, gamma=None, beta=None, eps=1e-5, relu=False, dx=None,
                       workspace=None):
    """Gradients through sparse_bn_apply in training mode (mean, var = sparse_bn_stats of x over the same blocks);
    returns (dx, dgamma, dbeta); dx defaults to a new zero tensor and is written on the active blocks only."""
    _dev(x, "x"), _dev(dy, "dy", x.dtype), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    N, H, W, C = x.shape
    cap = indices.shape[0]
    if dx is None:
        dx = torch.zeros_like(x)
    _dev(dx, "dx", x.dtype)
    assert dy.shape == x.shape and dx.shape == x.shape
    need = lib().sbnet_bn_backward_workspace_bytes(cap, C)
    if workspace is None:
        workspace = torch.empty((max(need, 4),), dtype=torch.uint8, device=x.device)
    _dev(workspace, "workspace", torch.uint8)
    dgamma = torch.empty((C,), dtype=torch.float32, device=x.device)
    dbeta = torch.empty((C,), dtype=torch.float32, device=x.device)
    _check(lib().sbnet_sparse_bn_backward(_ptr(x), _ptr(dy), _dt(x), N, H, W, C, _ptr(indices), _ptr(count), cap, g,
                                          _vec(mean, "mean", C), _vec(var, "var", C), _vec(gamma, "gamma", C),
                                          _vec(beta, "beta", C), float(eps), int(bool(relu)), _ptr(dx), _ptr(dgamma),
                                          _ptr(dbeta), _ptr(workspace), workspace.numel(), _stream()))
    return dx, dgamma, dbeta


def relu_backward_on_tiles(y_tiles, dy_tiles, count, out=None):
    """dy where the forward activation y is positive, else 0, on the active tiles of two stacks of one shape."""
    _dev(y_tiles, "y_tiles"), _dev(dy_tiles, "dy_tiles", y_tiles.dtype), _dev(count, "count", torch.int32)
    assert y_tiles.shape == dy_tiles.shape
    if out is None:
        out = torch.empty_like(dy_tiles)
    _dev(out, "out", y_tiles.dtype)
    cap = y_tiles.shape[0]
    _check(lib().sbnet_relu_backward_on_tiles(_ptr(y_tiles), _ptr(dy_tiles), _dt(y_tiles), _ptr(count), cap,
                                              y_tiles[0].numel() if cap else 1, _ptr(out), _stream()))
    return out


def bias_backward_on_tiles(dy_tiles, count, workspace=None):
    """Sum of dy [cap,h,w,C] over the active tiles and their pixels: float32 [C]."""
    _dev(dy_tiles, "dy_tiles"), _dev(count, "count", torch.int32)
    cap, h, w, C = dy_tiles.shape
    need = lib().sbnet_bias_backward_workspace_bytes(cap, C)
    if workspace is None:
        workspace = torch.empty((max(need, 4),), dtype=torch.uint8, device=dy_tiles.device)
    _dev(workspace, "workspace", torch.uint8)
    db = torch.empty((C,), dtype=torch.float32, device=dy_tiles.device)
    _check(lib().sbnet_bias_backward_on_tiles(_ptr(dy_tiles), _dt(dy_tiles), _ptr(count), cap, h * w, C, _ptr(db),
                                              _ptr(workspace), workspace.numel(), _stream()))
    return db


def relu_bias_backward_on_tiles(y_tiles, dy_tiles, count, out=None, workspace=None):
    """(dout, db): dy [cap,h,w,C] masked by y > 0 on the active tiles, and its per-channel sum (float32 [C]), in one pass."""
    _dev(y_tiles, "y_tiles"), _dev(dy_tiles, "dy_tiles", y_tiles.dtype), _dev(count, "count", torch.int32)
    assert y_tiles.shape == dy_tiles.shape
    cap, h, w, C = dy_tiles.shape
    if out is None:
        out = torch.empty_like(dy_tiles)
    _dev(out, "out", dy_tiles.dtype)
    assert out.shape == dy_tiles.shape
    need = lib().sbnet_bias_backward_workspace_bytes(cap, C)
    if workspace is None:
        workspace = torch.empty((max(need, 4),), dtype=torch.uint8, device=dy_tiles.device)
    _dev(workspace, "workspace", torch.uint8)
    db = torch.empty((C,), dtype=torch.float32, device=dy_tiles.device)
    _check(lib().sbnet_relu_bias_backward_on_tiles(_ptr(y_tiles), _ptr(dy_tiles), _dt(dy_tiles), _ptr(count), cap, h * w, C,
                                                   _ptr(out), _ptr(db), _ptr(workspace), workspace.numel(), _stream()))
    return out, db


def quantize_f8(x, scale=1.0, out=None):
    """x (f32 / bf16 / f16 device tensor) -> uint8 tensor of FP8 E4M3 (e4m3fn) codes of clamp(x * scale, +-448)."""
    _dev(x, "x")
    if out is None:
        out = torch.empty(x.shape, dtype=torch.uint8, device=x.device)
    _dev(out, "out", torch.uint8)
    assert out.shape == x.shape
    _check(lib().sbnet_quantize_f8(_ptr(x), _dt(x), x.numel(), float(scale), _ptr(out), _stream()))
    return out


def pack_weights_f8(w_f8):
    """FP8 codes [kh,kw,Cin,Cout] (uint8 device tensor) -> packed buffer for conv_on_tiles_f8."""
    _dev(w_f8, "w_f8", torch.uint8)
    kh, kw, Cin, Cout = w_f8.shape
    nbytes = _sz()
    _check(lib().sbnet_pack_weights_f8(None, kh, kw, Cin, Cout, None, nbytes, None))
    buf = torch.empty((nbytes.value,), dtype=torch.uint8, device=w_f8.device)
    _check(lib().sbnet_pack_weights_f8(_ptr(w_f8), kh, kw, Cin, Cout, _ptr(buf), nbytes, _stream()))
    return PackedWeights(buf, (kh, kw, Cin, Cout), torch.uint8)


def conv_on_tiles_f8(tiles_f8, count, w_packed, bias=None, stride=1, relu=False, out_scale=1.0, out=None):
    """Valid convolution of FP8 tiles [cap,th,tw,Cin] (uint8 codes) with FP8 weights -> bf16 [cap,th',tw',Cout]."""
    _dev(tiles_f8, "tiles_f8", torch.uint8), _dev(count, "count", torch.int32)
    kh, kw, Cin, Cout = w_packed.shape
    cap, th, tw, C = tiles_f8.shape
    assert C == Cin and w_packed.dtype == torch.uint8
    oh, ow = (th - kh) // stride + 1, (tw - kw) // stride + 1
    if out is None:
        out = torch.empty((cap, oh, ow, Cout), dtype=torch.bfloat16, device=tiles_f8.device)
    _dev(out, "out", torch.bfloat16)
    if bias is not None:
        _dev(bias, "bias", torch.float32)
    _check(lib().sbnet_conv_on_tiles_f8(_ptr(tiles_f8), _ptr(count), cap, th, tw, Cin, _ptr(w_packed.buf), _ptr(bias), kh,
                                        kw, stride, stride, Cout, int(bool(relu)), float(out_scale), _ptr(out), _stream()))
    return out


def bottleneck_forward_keep_on_tiles(tiles, indices, count, g_in, H, W, weights):
    """Residual branch on tiles with its activations kept for the backward pass: returns (t1, t2, t3).
    weights = (w1, b1, w2, b2, w3, b3) as sparse_bottleneck takes them."""
    _dev(tiles, "tiles"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    w1, b1, w2, b2, w3, b3 = weights
    cap, th, tw, C = tiles.shape
    Cm = w1.shape[3]
    assert (th, tw) == (g_in.bsize_h, g_in.bsize_w) and cap == indices.shape[0]
    new = lambda h, w, c: torch.empty((cap, h, w, c), dtype=tiles.dtype, device=tiles.device)
    t1, t2, t3 = new(th, tw, Cm), new(th - 2, tw - 2, Cm), new(th - 2, tw - 2, C)
    _check(lib().sbnet_bottleneck_forward_keep_on_tiles(_ptr(tiles), _dt(tiles), H, W, C, Cm, _ptr(indices), _ptr(count), cap,
                                                        g_in, _ptr(w1.buf), _ptr(b1), _ptr(w2.buf), _ptr(b2), _ptr(w3.buf),
                                                        _ptr(b3), _ptr(t1), _ptr(t2), _ptr(t3), _stream()))
    return t1, t2, t3


def bottleneck_backward_on_tiles(tiles, t1, t2, dt3, count, weights_t, workspace=None):
    """Backward of the residual branch on tiles from kept activations: returns (dtiles, dw1, db1, dw2, db2, dw3, db3).
    weights_t = (w1_t, w2_t, w3_t) from pack_weights_transposed of the three forward weight arrays."""
    for name, t in (("tiles", tiles), ("t1", t1), ("t2", t2), ("dt3", dt3)):
        _dev(t, name, tiles.dtype)
    _dev(count, "count", torch.int32)
    cap, th, tw, C = tiles.shape
    Cm = t1.shape[3]
    assert t1.shape == (cap, th, tw, Cm) and t2.shape == (cap, th - 2, tw - 2, Cm) and dt3.shape == (cap, th - 2, tw - 2, C)
    w1_t, w2_t, w3_t = weights_t
    assert w1_t.shape == (1, 1, C, Cm) and w2_t.shape == (3, 3, Cm, Cm) and w3_t.shape == (1, 1, Cm, C)
    need = lib().sbnet_bottleneck_backward_workspace_bytes(_dt(tiles), cap, th, tw, C, Cm)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=tiles.device)
    _dev(workspace, "workspace", torch.uint8)
    dev = tiles.device
    dtiles = torch.empty_like(tiles)
    f32 = lambda *shape: torch.empty(shape, dtype=torch.float32, device=dev)
    dw1, db1, dw2, db2, dw3, db3 = f32(1, 1, C, Cm), f32(Cm), f32(3, 3, Cm, Cm), f32(Cm), f32(1, 1, Cm, C), f32(C)
    _check(lib().sbnet_bottleneck_backward_on_tiles(_ptr(tiles), _ptr(t1), _ptr(t2), _ptr(dt3), _dt(tiles), _ptr(count), cap,
                                                    th, tw, C, Cm, _ptr(w1_t.buf), _ptr(w2_t.buf), _ptr(w3_t.buf),
                                                    _ptr(dtiles), _ptr(dw1), _ptr(db1), _ptr(dw2), _ptr(db2), _ptr(dw3),
                                                    _ptr(db3), _ptr(workspace), workspace.numel(), _stream()))
    return dtiles, dw1, db1, dw2, db2, dw3, db3


class PackedWeights:
    """Device buffer in the library's private weight layout plus the shape it was packed for."""

    def __init__(self, buf, shape, dtype):
        self.buf, self.shape, self.dtype = buf, tuple(shape), dtype


def pack_weights(w_hwio):
    """w [kh,kw,Cin,Cout] device tensor -> opaque packed device buffer for the conv calls."""
    _dev(w_hwio, "w_hwio")
    kh, kw, Cin, Cout = w_hwio.shape
    nbytes = _sz()
    _check(lib().sbnet_pack_weights(None, _dt(w_hwio), kh, kw, Cin, Cout, None, nbytes, None))
    buf = torch.empty((nbytes.value,), dtype=torch.uint8, device=w_hwio.device)
    _check(lib().sbnet_pack_weights(_ptr(w_hwio), _dt(w_hwio), kh, kw, Cin, Cout, _ptr(buf), nbytes, _stream()))
    return PackedWeights(buf, (kh, kw, Cin, Cout), w_hwio.dtype)


def conv_on_tiles(tiles, count, w_packed, bias=None, stride=1, relu=False, out=None):
    """Valid convolution on a tile stack [cap,th,tw,Cin] -> [cap,th',tw',Cout]."""
    _dev(tiles, "tiles"), _dev(count, "count", torch.int32)
    kh, kw, Cin, Cout = w_packed.shape
    cap, th, tw, C = tiles.shape
    assert C == Cin and w_packed.dtype == tiles.dtype
    oh, ow = (th - kh) // stride + 1, (tw - kw) // stride + 1
    if out is None:
        out = torch.empty((cap, oh, ow, Cout), dtype=tiles.dtype, device=tiles.device)
    _dev(out, "out", tiles.dtype)
    if bias is not None:
        _dev(bias, "bias", torch.float32)
    _check(lib().sbnet_conv_on_tiles(_ptr(tiles), _dt(tiles), _ptr(count), cap, th, tw, Cin, _ptr(w_packed.buf),
                                     _ptr(bias), kh, kw, stride, stride, Cout, int(bool(relu)), _ptr(out), _stream()))
    return out


def pack_weights_transposed(w_hwio):
    """Forward weights [kh,kw,Cin,Cout] -> packed buffer for conv_on_tiles_backward_data (taps mirrored, channel
    roles exchanged); .shape keeps the forward convolution's (kh, kw, Cin, Cout)."""
    _dev(w_hwio, "w_hwio")
    kh, kw, Cin, Cout = w_hwio.shape
    nbytes = _sz()
    _check(lib().sbnet_pack_weights_transposed(None, _dt(w_hwio), kh, kw, Cin, Cout, None, nbytes, None))
    buf = torch.empty((nbytes.value,), dtype=torch.uint8, device=w_hwio.device)
    _check(lib().sbnet_pack_weights_transposed(_ptr(w_hwio), _dt(w_hwio), kh, kw, Cin, Cout, _ptr(buf), nbytes,
                                               _stream()))
    return PackedWeights(buf, (kh, kw, Cin, Cout), w_hwio.dtype)


def conv_backward_data_workspace_bytes(dtype, cap, th, tw, kh, kw, stride, Cout):
    return int(lib().sbnet_conv_backward_data_workspace_bytes(_DTYPES[dtype], cap, th, tw, kh, kw, stride, stride, Cout))


def conv_on_tiles_backward_data(dout_tiles, count, w_packed_t, th, tw, stride=1, out=None, workspace=None):
    """dL/d(tiles_in) [cap,th,tw,Cin] of conv_on_tiles (no bias, no activation) from dL/d(tiles_out)
    [cap,oh,ow,Cout]; w_packed_t from pack_weights_transposed of the forward weights."""
    _dev(dout_tiles, "dout_tiles"), _dev(count, "count", torch.int32)
    kh, kw, Cin, Cout = w_packed_t.shape
    cap, oh, ow, C = dout_tiles.shape
    assert C == Cout and w_packed_t.dtype == dout_tiles.dtype
    assert oh == (th - kh) // stride + 1 and ow == (tw - kw) // stride + 1
    if out is None:
        out = torch.empty((cap, th, tw, Cin), dtype=dout_tiles.dtype, device=dout_tiles.device)
    _dev(out, "out", dout_tiles.dtype)
    need = conv_backward_data_workspace_bytes(dout_tiles.dtype, cap, th, tw, kh, kw, stride, Cout)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=dout_tiles.device)
    _dev(workspace, "workspace", torch.uint8)
    _check(lib().sbnet_conv_on_tiles_backward_data(_ptr(dout_tiles), _dt(dout_tiles), _ptr(count), cap, th, tw, Cin,
                                                   _ptr(w_packed_t.buf), kh, kw, stride, stride, Cout, _ptr(out),
                                                   _ptr(workspace), workspace.numel(), _stream()))
    return out


def conv_backward_weights_workspace_bytes(dtype, cap, th, tw, Cin, k, stride, Cout):
    return int(lib().sbnet_conv_backward_weights_workspace_bytes(_DTYPES[dtype], cap, th, tw, Cin, k, k, stride, stride, Cout))


def conv_on_tiles_backward_weights(tiles, dout_tiles, count, k, stride=1, out=None, workspace=None):
    """dL/dw [k,k,Cin,Cout] (float32) of conv_on_tiles from its input tiles [cap,th,tw,Cin] and dL/d(tiles_out)
    [cap,oh,ow,Cout], summed over the active tiles."""
    _dev(tiles, "tiles"), _dev(dout_tiles, "dout_tiles", tiles.dtype), _dev(count, "count", torch.int32)
    cap, th, tw, Cin = tiles.shape
    cap2, oh, ow, Cout = dout_tiles.shape
    assert cap2 == cap and oh == (th - k) // stride + 1 and ow == (tw - k) // stride + 1
    if out is None:
        out = torch.empty((k, k, Cin, Cout), dtype=torch.float32, device=tiles.device)
    _dev(out, "out", torch.float32)
    assert out.shape == (k, k, Cin, Cout)
    need = conv_backward_weights_workspace_bytes(tiles.dtype, cap, th, tw, Cin, k, stride, Cout)
    if workspace is None:
        workspace = torch.empty((max(need, 16),), dtype=torch.uint8, device=tiles.device)
    _dev(workspace, "workspace", torch.uint8)
    _check(lib().sbnet_conv_on_tiles_backward_weights(_ptr(tiles), _ptr(dout_tiles), _dt(tiles), _ptr(count), cap, th, tw,
                                                      Cin, k, k, stride, stride, Cout, _ptr(out), _ptr(workspace),
                                                      workspace.numel(), _stream()))
    return out


def sparse_conv(x, indices, count, g_in, g_out, w_packed, bias, y, stride=1, relu=False, add=False):
    """Fused gather -> valid conv -> scatter(-add) into y [N,H_out,W_out,Cout] in place; returns y."""
    _dev(x, "x"), _dev(y, "y", x.dtype)
    _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    kh, kw, Cin, Cout = w_packed.shape
    N, H, W, C = x.shape
    assert C == Cin and w_packed.dtype == x.dtype
    Ny, Ho, Wo, Cy = y.shape
    assert Ny == N and Cy == Cout
    if bias is not None:
        _dev(bias, "bias", torch.float32)
    _check(lib().sbnet_sparse_conv(_ptr(x), _dt(x), N, H, W, Cin, _ptr(indices), _ptr(count), indices.shape[0],
                                   g_in, g_out, _ptr(w_packed.buf), _ptr(bias), kh, kw, stride, stride, Cout,
                                   int(bool(relu)), _ptr(y), Ho, Wo, int(bool(add)), _stream()))
    return y


def block_flags(mask, g, pool=POOL_AVG, threshold=0.0, flags=None):
    """mask [N,H,W] u8/f32 -> one flag byte per block (lexicographic), padded to a multiple of 16 bytes."""
    _dev(mask, "mask")
    N, H, W = mask.shape
    need = lib().sbnet_block_flags_bytes(N, g)
    if flags is None:
        flags = torch.empty((need,), dtype=torch.uint8, device=mask.device)
    _dev(flags, "flags", torch.uint8)
    _check(lib().sbnet_block_flags(_ptr(mask), _dt(mask), N, H, W, g, pool, float(threshold), _ptr(flags), flags.numel(),
                                   _stream()))
    return flags


def sparse_conv_from_flags(flags, x, g_in, g_out, w_packed, bias, y, indices, count, stride=1, relu=False, add=False):
    """Fused sparse conv fed by block flags; fills y in place and writes the index list and count.  Returns y."""
    _dev(flags, "flags", torch.uint8), _dev(x, "x"), _dev(y, "y", x.dtype)
    _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    kh, kw, Cin, Cout = w_packed.shape
    N, H, W, C = x.shape
    assert C == Cin and w_packed.dtype == x.dtype
    Ny, Ho, Wo, Cy = y.shape
    assert Ny == N and Cy == Cout and flags.numel() >= lib().sbnet_block_flags_bytes(N, g_in)
    if bias is not None:
        _dev(bias, "bias", torch.float32)
    _check(lib().sbnet_sparse_conv_from_flags(_ptr(flags), _ptr(x), _dt(x), N, H, W, Cin, _ptr(indices), _ptr(count),
                                              indices.shape[0], g_in, g_out, _ptr(w_packed.buf), _ptr(bias), kh, kw, stride,
                                              stride, Cout, int(bool(relu)), _ptr(y), Ho, Wo, int(bool(add)), _stream()))
    return y


def sparse_conv_from_mask(mask, g_mask, x, g_in, g_out, w_packed, bias, y, indices, count, workspace, pool=POOL_AVG,
                          threshold=0.0, stride=1, relu=False, add=False):
    """reduce_mask + fused sparse conv in one call (two launches where the convolution kernel takes block flags);
    fills y in place and leaves the index list and the count in indices / count.  Returns y."""
    _dev(mask, "mask"), _dev(x, "x"), _dev(y, "y", x.dtype), _dev(workspace, "workspace")
    _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    kh, kw, Cin, Cout = w_packed.shape
    N, H, W, C = x.shape
    Nm, mH, mW = mask.shape
    assert C == Cin and w_packed.dtype == x.dtype and Nm == N
    Ny, Ho, Wo, Cy = y.shape
    assert Ny == N and Cy == Cout
    if bias is not None:
        _dev(bias, "bias", torch.float32)
    _check(lib().sbnet_sparse_conv_from_mask(_ptr(mask), _dt(mask), mH, mW, g_mask, pool, float(threshold), _ptr(x), _dt(x),
                                             N, H, W, Cin, _ptr(indices), _ptr(count), indices.shape[0], g_in, g_out,
                                             _ptr(w_packed.buf), _ptr(bias), kh, kw, stride, stride, Cout, int(bool(relu)),
                                             _ptr(y), Ho, Wo, int(bool(add)), _ptr(workspace),
                                             workspace.numel() * workspace.element_size(), _stream()))
    return y


def _unit_args(weights):
    """(w1p, b1, w2p, b2, w3p, b3) -> checked pointers plus (C, Cm)."""
    w1, b1, w2, b2, w3, b3 = weights
    _, _, C, Cm = w1.shape
    assert w2.shape == (3, 3, Cm, Cm) and w3.shape == (1, 1, Cm, C), (w1.shape, w2.shape, w3.shape)
    for b, n in ((b1, Cm), (b2, Cm), (b3, C)):
        _dev(b, "bias", torch.float32)
        assert b.numel() == n
    return (_ptr(w1.buf), _ptr(b1), _ptr(w2.buf), _ptr(b2), _ptr(w3.buf), _ptr(b3)), C, Cm


def _pre_args(pre, C):
    scale, shift = pre
    _dev(scale, "pre_scale", torch.float32), _dev(shift, "pre_shift", torch.float32)
    assert scale.numel() == C and shift.numel() == C
    return _ptr(scale), _ptr(shift)


def bottleneck_on_tiles(tiles, indices, count, g_in, g_out, H, W, weights, out=None, pre=None):
    """Residual branch (1x1+ReLU, 3x3+ReLU, 1x1) on gathered tiles [cap,h,w,C] -> t3 [cap,bo,bo,C];
    pre = (scale, shift): pre-activation ReLU(scale * x + shift) in front of the first convolution."""
    _dev(tiles, "tiles"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    ptrs, C, Cm = _unit_args(weights)
    cap = indices.shape[0]
    assert tiles.shape == (cap, g_in.bsize_h, g_in.bsize_w, C)
    if out is None:
        out = torch.empty((cap, g_out.bsize_h, g_out.bsize_w, C), dtype=tiles.dtype, device=tiles.device)
    _dev(out, "out", tiles.dtype)
    if pre is not None:
        _check(lib().sbnet_bottleneck_on_tiles_preact(_ptr(tiles), _dt(tiles), H, W, C, Cm, _ptr(indices), _ptr(count),
                                                      cap, g_in, g_out, *_pre_args(pre, C), *ptrs, _ptr(out), _stream()))
        return out
    _check(lib().sbnet_bottleneck_on_tiles(_ptr(tiles), _dt(tiles), H, W, C, Cm, _ptr(indices), _ptr(count), cap,
                                           g_in, g_out, *ptrs, _ptr(out), _stream()))
    return out


def sparse_bottleneck(x, indices, count, g_in, g_out, weights, y, pre=None):
    """Fused sparse residual unit: y[active] = x[active] + branch(x); y is a second buffer. Returns y.
    pre = (scale, shift): pre-activation form."""
    _dev(x, "x"), _dev(y, "y", x.dtype), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    ptrs, C, Cm = _unit_args(weights)
    N, H, W, Cx = x.shape
    assert Cx == C and y.shape == x.shape
    if pre is not None:
        _check(lib().sbnet_sparse_bottleneck_preact(_ptr(x), _dt(x), N, H, W, C, Cm, _ptr(indices), _ptr(count),
                                                    indices.shape[0], g_in, g_out, *_pre_args(pre, C), *ptrs, _ptr(y),
                                                    _stream()))
        return y
    _check(lib().sbnet_sparse_bottleneck(_ptr(x), _dt(x), N, H, W, C, Cm, _ptr(indices), _ptr(count),
                                         indices.shape[0], g_in, g_out, *ptrs, _ptr(y), _stream()))
    return y


def zero_outside(tiles, indices, count, g, H, W):
    """Zero, in place, the positions of tiles [cap,h,w,C] that lie outside the H x W image."""
    _dev(tiles, "tiles"), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    cap, h, w, C = tiles.shape
    assert (h, w) == (g.bsize_h, g.bsize_w) and cap == indices.shape[0]
    _check(lib().sbnet_zero_outside(_ptr(tiles), _dt(tiles), H, W, C, _ptr(indices), _ptr(count), cap, g, _stream()))
    return tiles


def sparse_unit(x, indices, count, g_in, g_out, weights, y, stride=1, shortcut=None, workspace=None):
    """Residual unit of any width: weights = (w1p, b1, w2p, b2, w3p, b3) packed, shortcut = (wsp, bs) packed 1x1 with the
    unit's stride or None for the identity.  Writes the active blocks of y [N,H_out,W_out,Cout] in place; returns y."""
    _dev(x, "x"), _dev(y, "y", x.dtype), _dev(indices, "indices", torch.int32), _dev(count, "count", torch.int32)
    w1, b1, w2, b2, w3, b3 = weights
    _, _, Cin, Cm = w1.shape
    Cout = w3.shape[3]
    assert w2.shape == (3, 3, Cm, Cm) and w3.shape[:3] == (1, 1, Cm)
    for b, n in ((b1, Cm), (b2, Cm), (b3, Cout)):
        _dev(b, "bias", torch.float32)
        assert b.numel() == n
    N, H, W, C = x.shape
    Ny, Ho, Wo, Cy = y.shape
    assert C == Cin and Cy == Cout and Ny == N
    wsp, bs = (None, None) if shortcut is None else shortcut
    if wsp is not None:
        assert wsp.shape == (1, 1, Cin, Cout) and bs.numel() == Cout
        _dev(bs, "shortcut bias", torch.float32)
    cap = indices.shape[0]
    need = lib().sbnet_sparse_unit_workspace_bytes(_dt(x), cap, g_in, g_out, Cin, Cm, Cout)
    if workspace is None:
        workspace = torch.empty((max(need, 256),), dtype=torch.uint8, device=x.device)
    _dev(workspace, "workspace")
    _check(lib().sbnet_sparse_unit(_ptr(x), _dt(x), N, H, W, Cin, Cm, Cout, stride, _ptr(indices), _ptr(count), cap, g_in, g_out,
                                   _ptr(w1.buf), _ptr(b1), _ptr(w2.buf), _ptr(b2), _ptr(w3.buf), _ptr(b3),
                                   _ptr(wsp.buf) if wsp is not None else None, _ptr(bs), _ptr(y), Ho, Wo, _ptr(workspace),
                                   workspace.numel() * workspace.element_size(), _stream()))
    return y
