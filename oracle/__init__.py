"""CPU oracle for SBNet's tiled sparse convolution (arXiv 1801.02108).

TEST INFRASTRUCTURE ONLY: a plain, slow, fp64 statement of what the method computes.
Only the tests, the smoke check and the benchmark's CPU-baseline leg may import it; the
GPU library never does, and the two share no code.

The arithmetic lives in ``sbnet_oracle.c`` (direct loops in double precision).  This
module marshals numpy arrays into it and composes the steps in the order the paper gives
them (Fig. 1: reduce mask -> gather -> convolution -> scatter; Fig. 4 / Sec. 3.3: a whole
residual unit between one gather and one scatter-add).  Every function is pinned by
``tests/test_oracle_pins.py`` to facts that do not come from this code.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sbnet_oracle.c")
_LIB = os.path.join(_HERE, "libsbnet_oracle.so")

POOL_MAX = 0
POOL_AVG = 1


def build(force=False):
    """Compile the C oracle with gcc (no tuning flags beyond -O2)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-shared", "-fPIC", "-o", _LIB, _SRC])
    return _LIB


class Geom(ctypes.Structure):
    """Block geometry: extent, stride, origin and count of blocks along h and w."""
    _fields_ = [(n, ctypes.c_int) for n in (
        "size_h", "size_w", "stride_h", "stride_w", "off_h", "off_w", "count_h", "count_w")]

    def astuple(self):
        return tuple(getattr(self, n) for n, _ in self._fields_)


_lib = None


def _c():
    """The loaded C library.  It is never compiled from here: build() runs once per process, before the process
    touches a GPU (tests: a session hook; benchmark and smoke check: their first statement)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise ImportError("%s not found: call oracle.build() first" % _LIB)
        _lib = ctypes.CDLL(_LIB)
        _lib.orc_reduce_mask.restype = ctypes.c_int
    return _lib


def _d(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _i(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


# ---------------------------------------------------------------------------------------
# geometry (Sec. 3.1, Fig. 3)
# ---------------------------------------------------------------------------------------
def conv_out_size(h, k, s, pad=0):
    """Output extent of a convolution: floor((h + 2 pad - k) / s) + 1."""
    return (h + 2 * pad - k) // s + 1


def geometry(H, W, k, s, bo):
    """Input-tile and output-block geometry for a k x k, stride-s, SAME convolution whose
    output is cut into bo x bo blocks.  Returns (g_in, g_out, H_out, W_out)."""
    p = (k - 1) // 2
    H_out, W_out = conv_out_size(H, k, s, p), conv_out_size(W, k, s, p)
    bh, bw = -(-H_out // bo), -(-W_out // bo)
    bsize = (bo - 1) * s + k
    g_in = Geom(bsize, bsize, bo * s, bo * s, -p, -p, bh, bw)
    g_out = Geom(bo, bo, bo, bo, 0, 0, bh, bw)
    return g_in, g_out, H_out, W_out


# ---------------------------------------------------------------------------------------
# the four steps
# ---------------------------------------------------------------------------------------
def reduce_mask(mask, g, pool=POOL_AVG, threshold=0.0):
    """mask [N,H,W] -> int32 [B,3] active block coordinates (n, by, bx), lexicographic."""
    mask, pm = _d(mask)
    N, H, W = mask.shape
    cap = N * g.count_h * g.count_w
    idx = np.zeros((max(cap, 1), 3), dtype=np.int32)
    cnt = _c().orc_reduce_mask(pm, N, H, W, ctypes.byref(g), int(pool),
                               ctypes.c_double(float(threshold)),
                               idx.ctypes.data_as(ctypes.c_void_p), cap)
    return idx[:cnt].copy()


def gather(x, idx, g):
    """x [N,H,W,C], idx [B,3] -> tiles [B, size_h, size_w, C]; zero outside the image."""
    x, px = _d(x)
    idx, pi = _i(idx)
    N, H, W, C = x.shape
    B = idx.shape[0]
    tiles = np.zeros((B, g.size_h, g.size_w, C), dtype=np.float64)
    _c().orc_gather(px, N, H, W, C, pi, B, ctypes.byref(g), tiles.ctypes.data_as(ctypes.c_void_p))
    return tiles


def scatter(tiles, idx, g, y, add=False):
    """Write (or add) tiles [B, size_h, size_w, C] into a copy of y [N,H,W,C]; returns it."""
    tiles, pt = _d(tiles)
    idx, pi = _i(idx)
    y = np.array(y, dtype=np.float64, order="C", copy=True)
    N, H, W, C = y.shape
    B = idx.shape[0]
    assert tiles.shape == (B, g.size_h, g.size_w, C), (tiles.shape, (B, g.size_h, g.size_w, C))
    _c().orc_scatter(pt, pi, B, ctypes.byref(g), y.ctypes.data_as(ctypes.c_void_p), N, H, W, C,
                     int(bool(add)))
    return y


def gather_backward(dtiles, idx, g, dx):
    """Gradient of gather (end of Sec. 3.3): every tile gradient is added onto its window of a copy of dx, also
    where windows of neighbouring tiles overlap; positions outside the image are dropped."""
    return scatter(dtiles, idx, g, dx, add=True)


def gather_chw(x, idx, g):
    """Gather with the transpose of Sec. 3.4 ("Fused transpose+gather"): channel-major tiles [B, C, size_h, size_w]."""
    return np.ascontiguousarray(np.transpose(gather(x, idx, g), (0, 3, 1, 2)))


def scatter_chw(tiles_chw, idx, g, y, add=False):
    """Scatter(-add) of channel-major tiles [B, C, size_h, size_w] (Sec. 3.4, "transpose+scatter")."""
    return scatter(np.transpose(np.asarray(tiles_chw), (0, 2, 3, 1)), idx, g, y, add=add)


def conv_valid(tiles, w, bias=None, stride=1, relu=False):
    """Unpadded cross-correlation on a tile stack; w is HWIO [kh,kw,Cin,Cout]."""
    tiles, pt = _d(tiles)
    w, pw = _d(w)
    B, h, wi, Cin = tiles.shape
    kh, kw, Cin2, Cout = w.shape
    assert Cin == Cin2
    pb = None
    if bias is not None:
        bias, pb = _d(bias)
        assert bias.shape == (Cout,)
    ho, wo = conv_out_size(h, kh, stride), conv_out_size(wi, kw, stride)
    out = np.zeros((B, ho, wo, Cout), dtype=np.float64)
    _c().orc_conv_valid(pt, B, h, wi, Cin, pw, pb, kh, kw, stride, stride, Cout, int(bool(relu)),
                        out.ctypes.data_as(ctypes.c_void_p))
    return out


def conv_valid_backward_data(dout, w, th, tw, stride=1):
    """Gradient of conv_valid (no bias, no activation) with respect to its input tiles [B, th, tw, Cin]: the
    forward sum out[b,i,j,o] = sum_{r,t,c} x[b, r + s i, t + s j, c] w[r,t,c,o] (Sec. 2, Sec. 3.2) hands
    dout[b,i,j,o] w[r,t,c,o] back to each input element it read.  Training support, not part of the paper's
    evaluated path."""
    dout = np.asarray(dout, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    B, ho, wo, Cout = dout.shape
    kh, kw, Cin, Cout2 = w.shape
    assert Cout == Cout2
    assert ho == conv_out_size(th, kh, stride) and wo == conv_out_size(tw, kw, stride)
    din = np.zeros((B, th, tw, Cin), dtype=np.float64)
    for r in range(kh):
        for t in range(kw):
            din[:, r:r + stride * (ho - 1) + 1:stride, t:t + stride * (wo - 1) + 1:stride, :] += dout @ w[r, t].T
    return din


def conv_valid_backward_weights(tiles, dout, kh, kw, stride=1):
    """Gradient of conv_valid with respect to its weights, summed over the whole tile stack:
    dw[r,t,c,o] = sum_{b,i,j} tiles[b, r + s i, t + s j, c] dout[b,i,j,o]."""
    tiles = np.asarray(tiles, dtype=np.float64)
    dout = np.asarray(dout, dtype=np.float64)
    B, th, tw, Cin = tiles.shape
    _, ho, wo, Cout = dout.shape
    assert ho == conv_out_size(th, kh, stride) and wo == conv_out_size(tw, kw, stride)
    dw = np.zeros((kh, kw, Cin, Cout), dtype=np.float64)
    g2 = dout.reshape(-1, Cout)
    for r in range(kh):
        for t in range(kw):
            xs = tiles[:, r:r + stride * (ho - 1) + 1:stride, t:t + stride * (wo - 1) + 1:stride, :]
            dw[r, t] = xs.reshape(-1, Cin).T @ g2
    return dw


def conv_dense(x, w, bias=None, stride=1, relu=False):
    """Zero-padded (SAME, pad = (k-1)/2) cross-correlation of the whole feature map."""
    x, px = _d(x)
    w, pw = _d(w)
    N, H, W, Cin = x.shape
    kh, kw, Cin2, Cout = w.shape
    assert Cin == Cin2
    ph, pwd = (kh - 1) // 2, (kw - 1) // 2
    pb = None
    if bias is not None:
        bias, pb = _d(bias)
    Ho, Wo = conv_out_size(H, kh, stride, ph), conv_out_size(W, kw, stride, pwd)
    out = np.zeros((N, Ho, Wo, Cout), dtype=np.float64)
    _c().orc_conv_dense(px, N, H, W, Cin, pw, pb, kh, kw, stride, stride, ph, pwd, Cout,
                        int(bool(relu)), out.ctypes.data_as(ctypes.c_void_p))
    return out


def zero_outside(tiles, idx, g, H, W):
    """Copy of tiles with every position outside the H x W image set to zero."""
    tiles = np.array(tiles, dtype=np.float64, order="C", copy=True)
    idx, pi = _i(idx)
    B, h, w, C = tiles.shape
    assert (h, w) == (g.size_h, g.size_w)
    _c().orc_zero_outside(tiles.ctypes.data_as(ctypes.c_void_p), pi, B, ctypes.byref(g), H, W, C)
    return tiles


def block_mask(idx, g_out, N, H_out, W_out):
    """Boolean [N,H_out,W_out]: pixel lies in one of the listed output blocks."""
    m = np.zeros((N, H_out, W_out), dtype=bool)
    for n, by, bx in np.asarray(idx).reshape(-1, 3):
        y0, x0 = g_out.off_h + by * g_out.stride_h, g_out.off_w + bx * g_out.stride_w
        m[n, max(y0, 0):y0 + g_out.size_h, max(x0, 0):x0 + g_out.size_w] = True
    return m


def bn_stats(x, idx, g_out):
    """Batch-norm statistics over the active blocks only (Sec. 3.3): per channel, mean and biased variance of x
    [N,H,W,C] over the pixels that lie in a listed block; zeros when there is none."""
    x = np.asarray(x, dtype=np.float64)
    N, H, W, C = x.shape
    vals = x[block_mask(idx, g_out, N, H, W)]                  # [pixels, C]
    if vals.shape[0] == 0:
        return np.zeros(C), np.zeros(C)
    mean = vals.sum(axis=0) / vals.shape[0]
    return mean, ((vals - mean) ** 2).sum(axis=0) / vals.shape[0]


def bn_apply(x, idx, g_out, mean, var, gamma, beta, eps, y, relu=False):
    """Normalisation over the active blocks (Sec. 3.3): act(gamma (x - mean) / sqrt(var + eps) + beta) on the pixels
    of the listed blocks, a copy of y elsewhere."""
    x = np.asarray(x, dtype=np.float64)
    out = np.array(y, dtype=np.float64)
    m = block_mask(idx, g_out, *x.shape[:3])
    z = np.asarray(gamma, dtype=np.float64) * (x[m] - mean) / np.sqrt(np.asarray(var, dtype=np.float64) + eps) + beta
    out[m] = np.maximum(z, 0.0) if relu else z
    return out


def bn_backward(x, dy, idx, g_out, gamma, beta, eps, dx, relu=False):
    """Gradients of L through out = bn_apply(x, ...) when mean and var are bn_stats of the same active pixels
    (training mode): returns (dx, dgamma, dbeta); dx is a copy of the argument outside the active blocks.  Written
    as the chain rule through the three steps mean -> variance -> normalised value, not as the collapsed formula."""
    x = np.asarray(x, dtype=np.float64)
    dy = np.asarray(dy, dtype=np.float64)
    gamma = np.asarray(gamma, dtype=np.float64)
    out = np.array(dx, dtype=np.float64)
    m = block_mask(idx, g_out, *x.shape[:3])
    xa, ga = x[m], dy[m]                                       # [n, C]
    n = xa.shape[0]
    C = x.shape[-1]
    if n == 0:
        return out, np.zeros(C), np.zeros(C)
    mean = xa.sum(axis=0) / n
    xc = xa - mean
    var = (xc ** 2).sum(axis=0) / n
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = xc * rstd
    if relu:
        ga = np.where(gamma * xhat + beta > 0.0, ga, 0.0)
    dbeta = ga.sum(axis=0)
    dgamma = (ga * xhat).sum(axis=0)
    dxhat = ga * gamma
    dvar = (dxhat * xc).sum(axis=0) * (-0.5) * rstd ** 3
    dmean = -(dxhat * rstd).sum(axis=0) + dvar * (-2.0 * xc.sum(axis=0) / n)
    out[m] = dxhat * rstd + dvar * 2.0 * xc / n + dmean / n
    return out, dgamma, dbeta


# ---------------------------------------------------------------------------------------
# FP8 E4M3 (OCP "e4m3fn": bias 7, no infinities, NaN = S.1111.111, largest finite 448)
# ---------------------------------------------------------------------------------------
def e4m3_decode(codes):
    """Values of FP8 E4M3 codes (uint8 array): (-1)^s 2^(e-7) (1 + m/8) for e > 0, (-1)^s 2^-6 (m/8) for e = 0."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    s, e, m = c >> 7, (c >> 3) & 15, c & 7
    mag = np.where(e > 0, np.ldexp(1.0 + m / 8.0, e - 7), np.ldexp(m / 8.0, -6))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(s == 1, -mag, mag)


def e4m3_encode(x):
    """Nearest FP8 E4M3 code of each element (ties to the even mantissa), magnitudes above 448 clamped to 448: a
    search over the 127 non-negative finite values, which are what e4m3_decode says they are."""
    x = np.asarray(x, dtype=np.float64)
    grid = e4m3_decode(np.arange(127, dtype=np.uint8))           # codes 0x00..0x7e: ascending magnitudes
    a = np.minimum(np.abs(x), 448.0)
    hi = np.clip(np.searchsorted(grid, a, side="left"), 0, 126)
    lo = np.clip(hi - 1, 0, 126)
    dlo, dhi = a - grid[lo], grid[hi] - a
    pick_hi = (dhi < dlo) | ((dhi == dlo) & (hi % 2 == 0))
    code = np.where(pick_hi, hi, lo).astype(np.uint8)
    code = np.where(np.isnan(x), np.uint8(0x7f), code)
    return (code | np.where(np.signbit(x) & ~np.isnan(x), 0x80, 0).astype(np.uint8)).astype(np.uint8)


def quantize_f8(x, scale):
    """Codes of x * scale, the product rounded to fp32 first (the precision the product is formed in)."""
    prod = (np.asarray(x, dtype=np.float32) * np.float32(scale)).astype(np.float32)
    return e4m3_encode(prod.astype(np.float64))


def conv_valid_f8(tile_codes, w_codes, bias=None, stride=1, relu=False, out_scale=1.0):
    """The FP8 variant of the tile convolution: act(out_scale * conv_valid(decoded tiles, decoded weights) + bias)."""
    acc = conv_valid(e4m3_decode(tile_codes), e4m3_decode(w_codes), None, stride=stride, relu=False)
    z = acc * float(np.float32(out_scale)) + (0.0 if bias is None else np.asarray(bias, dtype=np.float64))
    return np.maximum(z, 0.0) if relu else z


# ---------------------------------------------------------------------------------------
# compositions
# ---------------------------------------------------------------------------------------
def sparse_conv_tiled(x, idx, g_in, g_out, w, bias, y, stride=1, relu=False, add=False):
    """The method, step by step (Fig. 1): gather -> valid conv -> scatter (or scatter-add)."""
    tiles = gather(x, idx, g_in)
    out = conv_valid(tiles, w, bias, stride=stride, relu=relu)
    return scatter(out, idx, g_out, y, add=add)


def sparse_conv_dense(x, idx, g_out, w, bias, y, stride=1, relu=False, add=False):
    """What the method must equal (Sec. 3.2): the dense zero-padded convolution on the
    pixels of active blocks, y unchanged elsewhere."""
    d = conv_dense(x, w, bias, stride=stride, relu=relu)
    y = np.asarray(y, dtype=np.float64)
    m = block_mask(idx, g_out, *d.shape[:3])[..., None]
    return np.where(m, y + d if add else d, y)


def _pre_activate(v, pre):
    """ReLU(scale * v + shift) per channel (a batch norm and ReLU in front of the first convolution), or v."""
    if pre is None:
        return np.asarray(v, dtype=np.float64)
    scale, shift = (np.asarray(a, dtype=np.float64) for a in pre)
    return np.maximum(np.asarray(v, dtype=np.float64) * scale + shift, 0.0)


def bottleneck_on_tiles(tiles, idx, g_in, H, W, w1, b1, w2, b2, w3, b3, pre=None):
    """Residual branch of a bottleneck unit on gathered tiles (Sec. 3.3, Fig. 4, BN folded
    into w, b): 1x1 + ReLU on the whole tile, zero outside the image, valid 3x3 + ReLU,
    1x1.  Returns [B, bo, bo, Cout].  pre = (scale, shift): the pre-activation form, whose
    first convolution reads ReLU(scale * x + shift) while the residual stays x."""
    t1 = conv_valid(_pre_activate(tiles, pre), w1, b1, relu=True)
    t1 = zero_outside(t1, idx, g_in, H, W)
    t2 = conv_valid(t1, w2, b2, relu=True)
    return conv_valid(t2, w3, b3, relu=False)


def relu_backward(y, dy):
    """Gradient through y = ReLU(z): dy where y > 0."""
    return np.where(np.asarray(y, dtype=np.float64) > 0.0, np.asarray(dy, dtype=np.float64), 0.0)


def bias_backward(dy):
    """Gradient of a bias added to every pixel of every tile: the sum of dy over tiles and pixels."""
    return np.asarray(dy, dtype=np.float64).sum(axis=(0, 1, 2))


def bottleneck_backward_on_tiles(tiles, idx, g_in, H, W, w1, b1, w2, b2, w3, b3, dt3, saved=None):
    """Gradients of L through t3 = bottleneck_on_tiles(tiles, ...) (Sec. 3.3, the unit's residual branch), given
    dt3 = dL/dt3: the chain rule through the three convolutions in reverse, each ReLU passing the gradient where
    its output is positive.  The zeroing of t1 outside the image needs no step of its own: t1 is zero there, so
    its ReLU mask already blocks the gradient.  saved = (t1, t2): activations kept from a forward pass, used in
    place of recomputed ones (a forward pass that rounds them to a storage type decides the ReLU masks on the
    rounded values).  Returns (dtiles, dw1, db1, dw2, db2, dw3, db3)."""
    tiles = np.asarray(tiles, dtype=np.float64)
    if saved is None:
        t1 = zero_outside(conv_valid(tiles, w1, b1, relu=True), idx, g_in, H, W)
        t2 = conv_valid(t1, w2, b2, relu=True)
    else:
        t1, t2 = (np.asarray(t, dtype=np.float64) for t in saved)
    dt3 = np.asarray(dt3, dtype=np.float64)
    dw3 = conv_valid_backward_weights(t2, dt3, 1, 1)
    db3 = bias_backward(dt3)
    dt2 = relu_backward(t2, conv_valid_backward_data(dt3, w3, t2.shape[1], t2.shape[2]))
    dw2 = conv_valid_backward_weights(t1, dt2, 3, 3)
    db2 = bias_backward(dt2)
    dt1 = relu_backward(t1, conv_valid_backward_data(dt2, w2, t1.shape[1], t1.shape[2]))
    dw1 = conv_valid_backward_weights(tiles, dt1, 1, 1)
    db1 = bias_backward(dt1)
    dtiles = conv_valid_backward_data(dt1, w1, tiles.shape[1], tiles.shape[2])
    return dtiles, dw1, db1, dw2, db2, dw3, db3


def sparse_bottleneck_tiled(x, idx, g_in, g_out, w1, b1, w2, b2, w3, b3, pre=None):
    """One sparse residual unit: one gather, three convolutions, one scatter-add onto x."""
    x = np.asarray(x, dtype=np.float64)
    tiles = gather(x, idx, g_in)
    t3 = bottleneck_on_tiles(tiles, idx, g_in, x.shape[1], x.shape[2], w1, b1, w2, b2, w3, b3, pre=pre)
    return scatter(t3, idx, g_out, x, add=True)


def sparse_bottleneck_dense(x, idx, g_out, w1, b1, w2, b2, w3, b3, pre=None):
    """Dense residual unit, residual branch kept only on active blocks."""
    x = np.asarray(x, dtype=np.float64)
    t1 = conv_dense(_pre_activate(x, pre), w1, b1, relu=True)
    t2 = conv_dense(t1, w2, b2, relu=True)
    t3 = conv_dense(t2, w3, b3, relu=False)
    m = block_mask(idx, g_out, *x.shape[:3])[..., None]
    return x + np.where(m, t3, 0.0)


# ---------------------------------------------------------------------------------------
# residual units of any width, with a strided 3x3 and a projected shortcut (the backbone's
# downsampling units, Sec. 4 "Architecture"; geometry of the strided tile: Sec. 3.1, Fig. 3)
# ---------------------------------------------------------------------------------------
def unit_on_tiles(tiles, idx, g_in, H, W, w1, b1, w2, b2, w3, b3, stride=1, shortcut=None):
    """What a residual unit adds up on the output block of every gathered tile: the branch
    1x1 + ReLU (whole tile, zero outside the image) -> valid 3x3 with `stride` + ReLU -> 1x1, plus the shortcut:
    shortcut = (ws, bs): the 1x1 convolution with the same stride, i.e. of the tile pixels (i*stride + 1,
    j*stride + 1) that lie under the output pixels (the tile starts one pixel outside the block);
    shortcut = None: those pixels themselves (identity; needs equal channel counts).
    Returns [B, bo_h, bo_w, Cout]."""
    tiles = np.asarray(tiles, dtype=np.float64)
    t1 = zero_outside(conv_valid(tiles, w1, b1, relu=True), idx, g_in, H, W)
    t2 = conv_valid(t1, w2, b2, stride=stride, relu=True)
    t3 = conv_valid(t2, w3, b3, relu=False)
    oh, ow = t3.shape[1], t3.shape[2]
    centre = tiles[:, 1:1 + (oh - 1) * stride + 1:stride, 1:1 + (ow - 1) * stride + 1:stride, :]
    if shortcut is None:
        return centre + t3
    ws, bs = shortcut
    return conv_valid(centre, ws, bs, relu=False) + t3


def sparse_unit_tiled(x, idx, g_in, g_out, w1, b1, w2, b2, w3, b3, y, stride=1, shortcut=None):
    """One sparse residual unit, step by step: one gather, the unit on the tiles, one scatter (plain: the
    shortcut is part of what is scattered) into y, whose other pixels stay."""
    x = np.asarray(x, dtype=np.float64)
    tiles = gather(x, idx, g_in)
    out = unit_on_tiles(tiles, idx, g_in, x.shape[1], x.shape[2], w1, b1, w2, b2, w3, b3, stride=stride, shortcut=shortcut)
    return scatter(out, idx, g_out, y, add=False)


def sparse_unit_dense(x, idx, g_out, w1, b1, w2, b2, w3, b3, y, stride=1, shortcut=None):
    """What it must equal: the dense unit (zero-padded 3x3 with `stride`, shortcut a 1x1 convolution with the same
    stride or the identity) on the pixels of the active output blocks, y elsewhere."""
    x = np.asarray(x, dtype=np.float64)
    t1 = conv_dense(x, w1, b1, relu=True)
    t2 = conv_dense(t1, w2, b2, stride=stride, relu=True)
    t3 = conv_dense(t2, w3, b3, relu=False)
    sc = x[:, ::stride, ::stride, :] if shortcut is None else conv_dense(x, shortcut[0], shortcut[1], stride=stride)
    d = sc + t3
    m = block_mask(idx, g_out, *d.shape[:3])[..., None]
    return np.where(m, d, np.asarray(y, dtype=np.float64))
