"""Pins for the CPU oracle: every check here compares the oracle with something that does
not come from the oracle itself -- values printed in the paper (tests/golden), library
routines written by someone else (torch's CPU conv2d / pooling, numpy.pad), closed forms,
brute force on tiny inputs, and the method's own invariants (Sec. 3.1-3.4 of the paper).
"""
import itertools
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle as orc

GOLD = os.path.join(os.path.dirname(__file__), "golden")
rng0 = np.random.default_rng(20180102)


def _torch_conv(x, w, b, stride, pad, relu=False):
    """torch CPU conv2d in fp64: x NHWC, w HWIO."""
    xt = torch.from_numpy(np.ascontiguousarray(x)).permute(0, 3, 1, 2)
    wt = torch.from_numpy(np.ascontiguousarray(w)).permute(3, 2, 0, 1)
    bt = None if b is None else torch.from_numpy(np.ascontiguousarray(b))
    o = F.conv2d(xt, wt, bt, stride=stride, padding=pad)
    if relu:
        o = torch.relu(o)
    return o.permute(0, 2, 3, 1).contiguous().numpy()


# ------------------------------------------------------------------ geometry
def _read_golden(name):
    d = {}
    for line in open(os.path.join(GOLD, name)):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            d[k] = int(v)
    return d


def test_geometry_fig3_toy():
    t = _read_golden("fig3_toy_geometry.txt")
    g_in, g_out, H_out, _ = orc.geometry(17, 17, t["kernel"], t["kernel_stride"], t["outputs_per_block"])
    assert g_in.size_h == g_in.size_w == t["block"]
    assert g_in.stride_h == t["block_stride"]
    assert g_in.size_h - g_in.stride_h == t["overlap"] == t["kernel"] - t["kernel_stride"]
    assert orc.conv_out_size(t["block"], t["kernel"], t["kernel_stride"]) == t["outputs_per_block"]
    assert g_out.size_h == g_out.stride_h == t["outputs_per_block"]


@pytest.mark.parametrize("h,k", [(18, 3), (10, 3), (5, 1), (34, 3), (7, 5)])
def test_out_size_stride1_is_h_minus_k_plus_1(h, k):
    # Sec. 3.2: h' = (h - k + 1) / s; exact for s = 1
    assert orc.conv_out_size(h, k, 1) == h - k + 1


@pytest.mark.parametrize("H,W,k,s,bo", [(64, 64, 3, 1, 8), (13, 11, 3, 1, 4), (17, 9, 3, 2, 2),
                                        (12, 12, 1, 1, 3), (800, 704, 3, 1, 16)])
def test_geometry_output_blocks_partition_the_output(H, W, k, s, bo):
    g_in, g_out, Ho, Wo = orc.geometry(H, W, k, s, bo)
    cover = np.zeros((Ho, Wo), dtype=int)
    for by in range(g_out.count_h):
        for bx in range(g_out.count_w):
            cover[by * bo:(by + 1) * bo, bx * bo:(bx + 1) * bo] += 1
    assert (cover == 1).all()          # non-overlapping writes (Sec. 3.1)
    # the input tile of a block is exactly the receptive field of its output block
    assert g_in.size_h == (bo - 1) * s + k and g_in.stride_h == bo * s
    assert g_in.size_h - g_in.stride_h == k - s
    assert orc.conv_out_size(g_in.size_h, k, s) == bo


# ------------------------------------------------------------------ reduce_mask
def test_reduce_mask_all_ones_and_all_zeros():
    g_in, g_out, _, _ = orc.geometry(24, 16, 3, 1, 8)
    ones = np.ones((2, 24, 16))
    idx = orc.reduce_mask(ones, g_in, orc.POOL_AVG, 0.0)
    expect = np.array(list(itertools.product(range(2), range(3), range(2))), dtype=np.int32)
    assert idx.dtype == np.int32 and np.array_equal(idx, expect)      # lexicographic (n,by,bx)
    assert np.array_equal(orc.reduce_mask(ones, g_in, orc.POOL_MAX, 0.5), expect)
    for pool in (orc.POOL_MAX, orc.POOL_AVG):
        assert orc.reduce_mask(np.zeros((2, 24, 16)), g_in, pool, 0.0).shape == (0, 3)


@pytest.mark.parametrize("window", ["tile", "block"])
def test_reduce_mask_single_pixel_brute_force(window):
    H, W, bo = 12, 16, 4
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    g = g_in if window == "tile" else g_out
    seen_counts = set()
    for y in range(H):
        for x in range(W):
            m = np.zeros((1, H, W))
            m[0, y, x] = 1
            got = {tuple(r) for r in orc.reduce_mask(m, g, orc.POOL_MAX, 0.0)}
            want = set()
            for by in range(g.count_h):
                for bx in range(g.count_w):
                    y0, x0 = g.off_h + by * g.stride_h, g.off_w + bx * g.stride_w
                    if y0 <= y < y0 + g.size_h and x0 <= x < x0 + g.size_w:
                        want.add((0, by, bx))
            assert got == want
            seen_counts.add(len(got))
    # with the halo in the window a pixel can switch on 1, 2 or 4 blocks; without it exactly 1
    assert seen_counts == ({1, 2, 4} if window == "tile" else {1})


@pytest.mark.parametrize("a,b", [(1, 1), (8, 8), (7, 9), (16, 23), (17, 24), (32, 32)])
def test_reduce_mask_top_left_rectangle_closed_form(a, b):
    # the paper's synthetic masks: a top-left sub-region (Sec. 4.3).  A block whose window
    # starts at by*bo - 1 is active iff by*bo - 1 <= a - 1, i.e. by <= a/bo.
    H = W = 32
    bo = 8
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    m = np.zeros((1, H, W))
    m[0, :a, :b] = 1
    rows = min(a // bo + 1, H // bo)
    cols = min(b // bo + 1, W // bo)
    idx = orc.reduce_mask(m, g_in, orc.POOL_AVG, 0.0)
    assert len(idx) == rows * cols
    assert np.array_equal(idx, np.array([(0, r, c) for r in range(rows) for c in range(cols)], dtype=np.int32))
    # window = output block only: ceil(a/bo) * ceil(b/bo)
    idx2 = orc.reduce_mask(m, g_out, orc.POOL_AVG, 0.0)
    assert len(idx2) == -(-a // bo) * -(-b // bo)


def test_reduce_mask_matches_torch_pooling():
    # library special case: pooling with kernel=bsize, stride=bo, padding=1 (zeros)
    N, H, W, bo = 3, 40, 24, 8
    g_in, _, _, _ = orc.geometry(H, W, 3, 1, bo)
    m = (rng0.random((N, H, W)) < 0.02).astype(np.float64)
    real = rng0.random((N, H, W)) * m
    mt = torch.from_numpy(real)[:, None]
    avg = F.avg_pool2d(mt, g_in.size_h, stride=bo, padding=1, count_include_pad=True)[:, 0, :H // bo, :W // bo]
    mx = F.max_pool2d(mt, g_in.size_h, stride=bo, padding=1)[:, 0, :H // bo, :W // bo]
    for thr in (0.0, 0.001, 0.004, 0.3):
        want = np.argwhere(avg.numpy() > thr).astype(np.int32)
        assert np.array_equal(orc.reduce_mask(real, g_in, orc.POOL_AVG, thr), want)
        want = np.argwhere(mx.numpy() > thr).astype(np.int32)
        assert np.array_equal(orc.reduce_mask(real, g_in, orc.POOL_MAX, thr), want)


def test_reduce_mask_threshold_is_strict_and_avg_divides_by_full_window():
    g = orc.Geom(2, 2, 2, 2, 0, 0, 1, 2)
    m = np.zeros((1, 2, 4))
    m[0, 0, 0] = 1; m[0, 1, 1] = 1          # block 0: mean 0.5 ; block 1: mean 0
    assert len(orc.reduce_mask(m, g, orc.POOL_AVG, 0.5)) == 0          # 0.5 > 0.5 is false
    assert np.array_equal(orc.reduce_mask(m, g, orc.POOL_AVG, 0.49), [[0, 0, 0]])
    # window partly outside the image still divides by the full 3x3 area
    g = orc.Geom(3, 3, 2, 2, -1, -1, 1, 1)
    m = np.ones((1, 2, 2))                   # 4 ones in a 9-cell window: mean 4/9
    assert len(orc.reduce_mask(m, g, orc.POOL_AVG, 0.45)) == 0
    assert len(orc.reduce_mask(m, g, orc.POOL_AVG, 0.44)) == 1


def test_reduce_mask_max_equals_avg_at_zero_threshold_on_binary_masks():
    g_in, _, _, _ = orc.geometry(48, 40, 3, 1, 8)
    for seed in range(5):
        m = (np.random.default_rng(seed).random((2, 48, 40)) < 0.01).astype(np.float64)
        assert np.array_equal(orc.reduce_mask(m, g_in, orc.POOL_MAX, 0.0),
                              orc.reduce_mask(m, g_in, orc.POOL_AVG, 0.0))


def test_reduce_mask_sample_order_independence():
    g_in, _, _, _ = orc.geometry(32, 32, 3, 1, 8)
    m = (rng0.random((3, 32, 32)) < 0.01).astype(np.float64)
    full = orc.reduce_mask(m, g_in)
    for n in range(3):
        one = orc.reduce_mask(m[n:n + 1], g_in)
        assert np.array_equal(full[full[:, 0] == n][:, 1:], one[:, 1:])


# ------------------------------------------------------------------ gather / scatter
@pytest.mark.parametrize("H,W,C,k,s,bo", [(16, 24, 3, 3, 1, 8), (13, 10, 2, 3, 1, 4), (17, 17, 1, 3, 2, 2),
                                          (9, 9, 4, 5, 1, 3), (8, 8, 5, 1, 1, 4)])
def test_gather_equals_pad_and_slice(H, W, C, k, s, bo):
    g_in, g_out, Ho, Wo = orc.geometry(H, W, k, s, bo)
    x = rng0.standard_normal((2, H, W, C))
    idx = orc.reduce_mask(np.ones((2, H, W)), g_in)
    tiles = orc.gather(x, idx, g_in)
    P = g_in.size_h + max(g_in.stride_h * g_in.count_h, g_in.stride_w * g_in.count_w)
    xp = np.pad(x, ((0, 0), (P, P), (P, P), (0, 0)))
    for b, (n, by, bx) in enumerate(idx):
        y0 = g_in.off_h + by * g_in.stride_h + P
        x0 = g_in.off_w + bx * g_in.stride_w + P
        assert np.array_equal(tiles[b], xp[n, y0:y0 + g_in.size_h, x0:x0 + g_in.size_w])
    # first tile: its top row and left column lie outside the image for k = 3
    if k == 3:
        assert (tiles[0, 0] == 0).all() and (tiles[0, :, 0] == 0).all()
        assert np.array_equal(tiles[0, 1, 1], x[0, 0, 0])


def test_gather_delta_input_lands_where_predicted():
    H, W, bo = 12, 12, 4
    g_in, _, _, _ = orc.geometry(H, W, 3, 1, bo)
    idx = orc.reduce_mask(np.ones((1, H, W)), g_in)
    x = np.zeros((1, H, W, 2))
    x[0, 4, 7, 1] = 5.0        # row 4 is the first row of block-row 1 and the halo of block-row 0
    tiles = orc.gather(x, idx, g_in)
    hits = {(int(b), int(i), int(j), int(c)) for b, i, j, c in np.argwhere(tiles != 0)}
    # block (by,bx) has origin (4by-1, 4bx-1); pixel (4,7) sits at (4-4by+1, 7-4bx+1)
    want = set()
    for b, (n, by, bx) in enumerate(idx):
        i, j = 4 - (4 * by - 1), 7 - (4 * bx - 1)
        if 0 <= i < 6 and 0 <= j < 6:
            want.add((b, i, j, 1))
    assert hits == want and len(want) == 4


def test_transposing_gather_and_scatter_by_brute_force():
    """Channel-major tiles (Sec. 3.4, fused transpose): every element written out from the definition, loop by loop,
    and scatter as the inverse of gather on the blocks' own pixels."""
    H, W, C, bo = 10, 7, 3, 4                                   # ragged: the last blocks hang over the edge
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    x = rng0.standard_normal((2, H, W, C))
    mask = np.zeros((2, H, W))
    mask[0, 1, 1] = mask[1, 9, 6] = mask[1, 4, 3] = 1
    idx = orc.reduce_mask(mask, g_in)
    t = orc.gather_chw(x, idx, g_in)
    assert t.shape == (len(idx), C, bo + 2, bo + 2)
    for b, (n, by, bx) in enumerate(idx):
        for c in range(C):
            for i in range(bo + 2):
                for j in range(bo + 2):
                    yy, xx = by * bo - 1 + i, bx * bo - 1 + j
                    want = x[n, yy, xx, c] if 0 <= yy < H and 0 <= xx < W else 0.0
                    assert t[b, c, i, j] == want
    # scatter the interiors back: active blocks' pixels reproduce x, the rest keeps y0; add doubles them
    y0 = rng0.standard_normal((2, H, W, C))
    inner = t[:, :, 1:-1, 1:-1]
    y = orc.scatter_chw(inner, idx, g_out, y0)
    bm = orc.block_mask(idx, g_out, 2, H, W)
    assert np.array_equal(y[bm], x[bm]) and np.array_equal(y[~bm], y0[~bm])
    ya = orc.scatter_chw(inner, idx, g_out, x, add=True)
    assert np.array_equal(ya[bm], 2 * x[bm]) and np.array_equal(ya[~bm], x[~bm])


@pytest.mark.parametrize("H,W,C,k,s,bo", [(12, 9, 2, 3, 1, 4), (17, 17, 1, 3, 2, 2), (9, 9, 3, 5, 1, 3), (10, 14, 2, 7, 1, 2)])
def test_gather_backward_is_the_adjoint_of_gather(H, W, C, k, s, bo):
    """<gather(x), t> == <x, gather_backward(t)> for any x, t: the defining property of a gradient of a linear
    map; and with all-ones tile gradients dx counts the tiles covering each pixel (1 inside a block's own cells,
    2 on shared edges, 4 on shared corners for a one-pixel halo)."""
    g_in, _, _, _ = orc.geometry(H, W, k, s, bo)
    mask = rng0.random((2, H, W)) < 0.08
    mask[0, 0, 0] = mask[1, H - 1, W - 1] = True
    idx = orc.reduce_mask(mask.astype(np.float64), g_in)
    x = rng0.standard_normal((2, H, W, C))
    t = rng0.standard_normal((len(idx), g_in.size_h, g_in.size_w, C))
    lhs = float((orc.gather(x, idx, g_in) * t).sum())
    rhs = float((x * orc.gather_backward(t, idx, g_in, np.zeros_like(x))).sum())
    assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))
    # accumulation: dx is added to, not overwritten
    d0 = rng0.standard_normal(x.shape)
    assert np.allclose(orc.gather_backward(t, idx, g_in, d0), d0 + orc.gather_backward(t, idx, g_in, np.zeros_like(x)), atol=1e-12)
    # coverage counts by brute force
    cover = np.zeros((2, H, W))
    for n, by, bx in idx:
        y0, x0 = g_in.off_h + by * g_in.stride_h, g_in.off_w + bx * g_in.stride_w
        cover[n, max(y0, 0):max(min(y0 + g_in.size_h, H), 0), max(x0, 0):max(min(x0 + g_in.size_w, W), 0)] += 1
    ones = orc.gather_backward(np.ones_like(t), idx, g_in, np.zeros_like(x))
    assert np.array_equal(ones, np.repeat(cover[..., None], C, axis=3))


def test_bottleneck_backward_by_finite_differences():
    """Every gradient of the residual branch against central differences of L = sum(coef * bottleneck_on_tiles(...)),
    the forward oracle, which shares nothing with the backward composition but the two convolution gradients
    pinned above; a tile at the image corner is among the tiles, so the zeroing of t1 outside the image is on the
    path.  Inputs are kept away from the ReLU kinks by construction of the check (a difference across a kink would
    not match, and none does at this step size)."""
    H, W, C, Cm, bo = 9, 8, 3, 2, 4
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    idx = np.array([(0, 0, 0), (0, 1, 1), (0, 2, 1)], dtype=np.int32)
    x = rng0.standard_normal((1, H, W, C))
    tiles = orc.gather(x, idx, g_in)
    w1, b1 = rng0.standard_normal((1, 1, C, Cm)), rng0.standard_normal(Cm) * 0.5 + 0.3
    w2, b2 = rng0.standard_normal((3, 3, Cm, Cm)) * 0.5, rng0.standard_normal(Cm) * 0.5
    w3, b3 = rng0.standard_normal((1, 1, Cm, C)), rng0.standard_normal(C)
    coef = rng0.standard_normal((len(idx), bo, bo, C))

    def loss(t=tiles, a1=w1, c1=b1, a2=w2, c2=b2, a3=w3, c3=b3):
        return float((coef * orc.bottleneck_on_tiles(t, idx, g_in, H, W, a1, c1, a2, c2, a3, c3)).sum())
    grads = orc.bottleneck_backward_on_tiles(tiles, idx, g_in, H, W, w1, b1, w2, b2, w3, b3, coef)
    names = ["t", "a1", "c1", "a2", "c2", "a3", "c3"]
    args = [tiles, w1, b1, w2, b2, w3, b3]
    h = 1e-6
    checked = 0
    for name, arg, grad in zip(names, args, grads):
        assert grad.shape == arg.shape
        flat = list(np.ndindex(*arg.shape))
        for k in rng0.choice(len(flat), min(len(flat), 12), replace=False):
            e = np.zeros_like(arg)
            e[flat[k]] = h
            fd = (loss(**{name: arg + e}) - loss(**{name: arg - e})) / (2 * h)
            assert abs(grad[flat[k]] - fd) < 1e-6 * max(1.0, abs(fd)), (name, flat[k], grad[flat[k]], fd)
            checked += 1
    assert checked > 40
    # the corner tile's t1 is zeroed outside the image: the input gradient vanishes there
    dt = grads[0]
    assert np.all(dt[0, 0, :, :] == 0) and np.all(dt[0, :, 0, :] == 0) and np.any(dt[0, 1:, 1:, :] != 0)
    assert np.allclose(orc.relu_backward([-1.0, 0.0, 2.0], [5.0, 6.0, 7.0]), [0.0, 0.0, 7.0])
    assert np.allclose(orc.bias_backward(np.ones((2, 3, 4, 5))), 24.0)


def test_e4m3_against_the_format_and_the_library():
    """Decode: the values the OCP format fixes (1.0 = 0x38, 448 = 0x7e, 2^-9 = 0x01, 2^-6 = 0x08, 0x7f NaN) and all
    256 codes against torch's float8_e4m3fn.  Encode: every code decodes and encodes back to itself; exact midpoints
    go to the even mantissa; above 448 saturates; random values against torch's conversion (which saturates the same
    way for finite inputs within range)."""
    import torch
    assert orc.e4m3_decode([0x38, 0x7e, 0x01, 0x08, 0xb8, 0x00])[:5].tolist() == [1.0, 448.0, 2.0 ** -9, 2.0 ** -6, -1.0]
    assert np.isnan(orc.e4m3_decode([0x7f, 0xff])).all()
    codes = np.arange(256, dtype=np.uint8)
    lib_vals = torch.from_numpy(codes).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    ours = orc.e4m3_decode(codes)
    assert np.array_equal(np.isnan(ours), np.isnan(lib_vals)) and np.array_equal(ours[~np.isnan(ours)], lib_vals[~np.isnan(ours)])
    finite = codes[~np.isnan(ours)]
    back = orc.e4m3_encode(ours[~np.isnan(ours)])
    assert np.array_equal(back & 0x7f, finite & 0x7f)            # the sign of zero aside
    assert orc.e4m3_encode([1.0625, 1.1875, 17.0, 500.0, -1e9, 2.0 ** -10, 3 * 2.0 ** -10]).tolist() == \
        [0x38, 0x3a, 0x58, 0x7e, 0xfe, 0x00, 0x02]               # ties to even; 17 -> 16; saturation; subnormal ties
    x = (rng0.standard_normal(20000) * np.exp(rng0.uniform(-8, 5, 20000))).astype(np.float32)
    x = x[np.abs(x) <= 448.0]
    lib_codes = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    ours = orc.e4m3_encode(x.astype(np.float64))
    assert np.array_equal(ours, lib_codes), int((ours != lib_codes).sum())
    # the convolution on codes is the fp64 convolution of their values
    t = rng0.integers(0, 0x7f, (2, 4, 5, 3)).astype(np.uint8)
    w = rng0.integers(0, 0x7f, (3, 3, 3, 2)).astype(np.uint8)
    assert np.allclose(orc.conv_valid_f8(t, w, out_scale=0.5), 0.5 * orc.conv_valid(orc.e4m3_decode(t), orc.e4m3_decode(w)))


def test_bn_apply_and_backward():
    """All blocks active and no activation: the library's batch_norm in training mode and its autograd gradients
    (fp64).  Some blocks active, with and without ReLU: the forward value by brute force over pixels; the three
    gradients by central differences of L = sum(coef * bn_apply(x with statistics of the active pixels)), which
    knows nothing of the backward formulas; pixels outside the active blocks keep the caller's values."""
    import torch
    N, H, W, C, bo, eps = 2, 9, 7, 3, 4, 1e-3
    _, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    x = rng0.standard_normal((N, H, W, C)) * 2.0 + 0.5
    dy = rng0.standard_normal((N, H, W, C))
    gamma, beta = rng0.standard_normal(C) + 1.5, rng0.standard_normal(C) * 0.3
    full = np.array([(n, by, bx) for n in range(N) for by in range(g_out.count_h) for bx in range(g_out.count_w)], dtype=np.int32)
    mean, var = orc.bn_stats(x, full, g_out)
    xt = torch.tensor(x.transpose(0, 3, 1, 2), dtype=torch.float64, requires_grad=True)
    gt, bt = torch.tensor(gamma, requires_grad=True), torch.tensor(beta, requires_grad=True)
    out_t = torch.nn.functional.batch_norm(xt, None, None, gt, bt, training=True, eps=eps)
    out_t.backward(torch.tensor(dy.transpose(0, 3, 1, 2)))
    out = orc.bn_apply(x, full, g_out, mean, var, gamma, beta, eps, np.zeros_like(x))
    assert np.allclose(out, out_t.detach().numpy().transpose(0, 2, 3, 1), atol=1e-12)
    dx, dgam, dbet = orc.bn_backward(x, dy, full, g_out, gamma, beta, eps, np.zeros_like(x))
    assert np.allclose(dx, xt.grad.numpy().transpose(0, 2, 3, 1), atol=1e-11)
    assert np.allclose(dgam, gt.grad.numpy(), atol=1e-11) and np.allclose(dbet, bt.grad.numpy(), atol=1e-11)

    idx = full[[0, 3, 4, len(full) - 1]]                        # the last block hangs over both image edges
    inside = orc.block_mask(idx, g_out, N, H, W)
    y0 = rng0.standard_normal(x.shape)
    for relu in (False, True):
        mean, var = orc.bn_stats(x, idx, g_out)
        out = orc.bn_apply(x, idx, g_out, mean, var, gamma, beta, eps, y0, relu=relu)
        for n, yy, xx in [(0, 0, 0), (0, 3, 6), (1, 8, 6), (1, 4, 3), (0, 5, 1)]:
            z = gamma * (x[n, yy, xx] - mean) / np.sqrt(var + eps) + beta
            want = (np.maximum(z, 0) if relu else z) if inside[n, yy, xx] else y0[n, yy, xx]
            assert np.allclose(out[n, yy, xx], want, atol=1e-12)

        def loss(xv, gv, bv):
            mu, vv = orc.bn_stats(xv, idx, g_out)
            return float((dy * orc.bn_apply(xv, idx, g_out, mu, vv, gv, bv, eps, np.zeros_like(xv), relu=relu)).sum())
        d0 = rng0.standard_normal(x.shape)
        dx, dgam, dbet = orc.bn_backward(x, dy, idx, g_out, gamma, beta, eps, d0, relu=relu)
        assert np.array_equal(dx[~inside], d0[~inside])
        h = 1e-6
        for n, yy, xx, c in [(0, 0, 0, 0), (0, 5, 5, 1), (1, 8, 6, 2), (0, 3, 3, 1), (0, 8, 2, 0)]:
            assert inside[n, yy, xx]
            e = np.zeros_like(x)
            e[n, yy, xx, c] = h
            fd = (loss(x + e, gamma, beta) - loss(x - e, gamma, beta)) / (2 * h)
            assert abs(dx[n, yy, xx, c] - fd) < 1e-6 * max(1.0, abs(fd))
        for c in range(C):
            e = np.zeros(C)
            e[c] = h
            assert abs(dgam[c] - (loss(x, gamma + e, beta) - loss(x, gamma - e, beta)) / (2 * h)) < 1e-6 * max(1.0, abs(dgam[c]))
            assert abs(dbet[c] - (loss(x, gamma, beta + e) - loss(x, gamma, beta - e)) / (2 * h)) < 1e-6 * max(1.0, abs(dbet[c]))


@pytest.mark.parametrize("th,tw,Cin,Cout,k,s", [(5, 4, 2, 3, 3, 1), (7, 6, 2, 2, 3, 2), (6, 7, 1, 2, 3, 2), (4, 4, 3, 2, 1, 1),
                                                (5, 5, 2, 1, 1, 2), (6, 5, 1, 2, 5, 1)])
def test_conv_gradients_element_by_element(th, tw, Cin, Cout, k, s):
    """The convolution is linear in its input and in its weights, so its two gradients are fixed by the forward
    map alone: d out[q] / d x[p] and d out[q] / d w[p] are read off conv_valid (the C routine, separate code)
    applied to unit inputs, and every element of both gradients is rebuilt from them.  A mirrored tap, exchanged
    channel roles, a stride applied on the wrong side or a row a strided window never reaches (the (6, 7) and
    (7, 6) tiles at stride 2) each change some element."""
    B = 2
    ho, wo = orc.conv_out_size(th, k, s), orc.conv_out_size(tw, k, s)
    w = rng0.standard_normal((k, k, Cin, Cout))
    x = rng0.standard_normal((B, th, tw, Cin))
    g = rng0.standard_normal((B, ho, wo, Cout))
    # data gradient: din[p] = sum_q g[q] * d out[q] / d x[p]
    din = orc.conv_valid_backward_data(g, w, th, tw, stride=s)
    assert din.shape == x.shape
    want = np.zeros_like(x)
    for p in np.ndindex(1, th, tw, Cin):                          # tiles do not interact: unit inputs in tile 0
        e = np.zeros((1, th, tw, Cin))
        e[p] = 1.0
        col = orc.conv_valid(e, w, stride=s)[0]
        for b in range(B):
            want[(b,) + p[1:]] = float((col * g[b]).sum())
    assert np.allclose(din, want, rtol=0, atol=1e-12)
    # weight gradient: dw[p] = sum_q g[q] * d out[q] / d w[p]
    dw = orc.conv_valid_backward_weights(x, g, k, k, stride=s)
    want = np.zeros_like(w)
    for p in np.ndindex(*w.shape):
        e = np.zeros_like(w)
        e[p] = 1.0
        want[p] = float((orc.conv_valid(x, e, stride=s) * g).sum())
    assert np.allclose(dw, want, rtol=0, atol=1e-12)


def test_conv_gradients_special_cases():
    """1x1 at stride 1 is a matrix product per pixel, so the gradients are the textbook ones of y = x W; and the
    sparse convolution's input gradient, gather_backward of the tile gradient, satisfies the adjoint identity
    against the tiled forward path."""
    x = rng0.standard_normal((3, 4, 5, 6))
    w = rng0.standard_normal((1, 1, 6, 7))
    g = rng0.standard_normal((3, 4, 5, 7))
    assert np.allclose(orc.conv_valid_backward_data(g, w, 4, 5), g @ w[0, 0].T, atol=1e-12)
    assert np.allclose(orc.conv_valid_backward_weights(x, g, 1, 1)[0, 0], x.reshape(-1, 6).T @ g.reshape(-1, 7), atol=1e-12)
    H, W, Cin, Cout, bo = 13, 11, 2, 3, 4
    for s in (1, 2):
        g_in, g_out, Ho, Wo = orc.geometry(H, W, 3, s, bo)
        mask = rng0.random((1, H, W)) < 0.1
        idx = orc.reduce_mask(mask.astype(np.float64), g_in)
        x = rng0.standard_normal((1, H, W, Cin))
        w = rng0.standard_normal((3, 3, Cin, Cout))
        gy_tiles = rng0.standard_normal((len(idx), g_out.size_h, g_out.size_w, Cout))
        fwd = orc.conv_valid(orc.gather(x, idx, g_in), w, stride=s)
        dx = orc.gather_backward(orc.conv_valid_backward_data(gy_tiles, w, g_in.size_h, g_in.size_w, stride=s), idx, g_in,
                                 np.zeros_like(x))
        lhs, rhs = float((fwd * gy_tiles).sum()), float((x * dx).sum())
        assert abs(lhs - rhs) <= 1e-10 * max(1.0, abs(lhs))


def test_bn_stats_over_active_blocks():
    """Sparse batch-norm statistics (Sec. 3.3): all blocks active == the library's mean / variance over N, H, W;
    affine maps of x move the statistics as they must; a pixel counts once and only if it is inside the image and
    inside a listed block (brute force); the order of the list does not matter."""
    H, W, C, bo = 10, 7, 3, 4                                   # blocks hang over the right and lower edges
    _, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    x = rng0.standard_normal((2, H, W, C)) * np.array([1.0, 3.0, 0.1]) + np.array([0.0, 50.0, -2.0])
    all_idx = orc.reduce_mask(np.ones((2, H, W)), g_out)
    m, v = orc.bn_stats(x, all_idx, g_out)
    assert np.allclose(m, x.mean(axis=(0, 1, 2)), rtol=1e-12) and np.allclose(v, x.var(axis=(0, 1, 2)), rtol=1e-12)
    idx = all_idx[[1, 4, 5, 9]]
    m, v = orc.bn_stats(x, idx, g_out)
    rows = []
    for n, by, bx in idx:
        for i in range(bo):
            for j in range(bo):
                yy, xx = by * bo + i, bx * bo + j
                if yy < H and xx < W:
                    rows.append(x[n, yy, xx])
    rows = np.array(rows)
    assert np.allclose(m, rows.mean(axis=0), rtol=1e-12) and np.allclose(v, rows.var(axis=0), rtol=1e-12)
    m2, v2 = orc.bn_stats(2.0 * x - 3.0, idx, g_out)
    assert np.allclose(m2, 2.0 * m - 3.0, rtol=1e-12) and np.allclose(v2, 4.0 * v, rtol=1e-12)
    m3, v3 = orc.bn_stats(x, idx[::-1], g_out)
    assert np.allclose(m3, m, rtol=1e-13) and np.allclose(v3, v, rtol=1e-13)
    mc, vc = orc.bn_stats(np.full_like(x, 7.0), idx, g_out)
    assert np.array_equal(mc, np.full(C, 7.0)) and np.array_equal(vc, np.zeros(C))
    m0, v0 = orc.bn_stats(x, np.zeros((0, 3), dtype=np.int32), g_out)
    assert np.array_equal(m0, np.zeros(C)) and np.array_equal(v0, np.zeros(C))


def test_scatter_invariants():
    H, W, C, bo = 20, 12, 3, 4
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    x = rng0.standard_normal((2, H, W, C))
    y0 = rng0.standard_normal((2, H, W, C))
    all_idx = orc.reduce_mask(np.ones((2, H, W)), g_in)
    # (1) empty index list: y untouched
    assert np.array_equal(orc.scatter(np.zeros((0, bo, bo, C)), np.zeros((0, 3), np.int32), g_out, y0), y0)
    # (2) round trip with every block active: scatter(interior(gather(x))) == x
    tiles = orc.gather(x, all_idx, g_in)
    assert np.array_equal(orc.scatter(tiles[:, 1:-1, 1:-1], all_idx, g_out, np.zeros_like(x)), x)
    # (3) add onto zeros equals plain write; add onto y0 equals y0 + write-onto-zeros
    m = (rng0.random((2, H, W)) < 0.02).astype(float)
    idx = orc.reduce_mask(m, g_in)
    assert 0 < len(idx) < len(all_idx)
    t = rng0.standard_normal((len(idx), bo, bo, C))
    w0 = orc.scatter(t, idx, g_out, np.zeros_like(x))
    assert np.array_equal(orc.scatter(t, idx, g_out, np.zeros_like(x), add=True), w0)
    assert np.array_equal(orc.scatter(t, idx, g_out, y0, add=True), y0 + w0)
    # (4) written set == union of active blocks, each pixel written exactly once
    hits = orc.scatter(np.ones_like(t), idx, g_out, np.zeros_like(x), add=True)
    bm = orc.block_mask(idx, g_out, 2, H, W)
    assert np.array_equal(hits[..., 0], bm.astype(float)) and hits.max() == 1.0
    # (5) plain write leaves pixels of inactive blocks bit-identical
    out = orc.scatter(t, idx, g_out, y0)
    assert np.array_equal(out[~bm], y0[~bm])
    # (6) ragged edge: blocks hanging over the image are clipped
    g_in2, g_out2, _, _ = orc.geometry(10, 10, 3, 1, 4)
    idx2 = orc.reduce_mask(np.ones((1, 10, 10)), g_in2)
    assert len(idx2) == 9
    full = orc.scatter(np.ones((9, 4, 4, 1)), idx2, g_out2, np.zeros((1, 10, 10, 1)), add=True)
    assert (full == 1).all()


# ------------------------------------------------------------------ convolution
@pytest.mark.parametrize("k,s,Cin,Cout", [(3, 1, 4, 5), (1, 1, 6, 3), (3, 2, 3, 4), (5, 1, 2, 2)])
def test_conv_matches_torch_fp64(k, s, Cin, Cout):
    x = rng0.standard_normal((2, 11, 9, Cin))
    w = rng0.standard_normal((k, k, Cin, Cout))
    b = rng0.standard_normal(Cout)
    for relu in (False, True):
        np.testing.assert_allclose(orc.conv_valid(x, w, b, stride=s, relu=relu),
                                   _torch_conv(x, w, b, s, 0, relu), rtol=1e-12, atol=1e-12)
        np.testing.assert_allclose(orc.conv_dense(x, w, b, stride=s, relu=relu),
                                   _torch_conv(x, w, b, s, (k - 1) // 2, relu), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(orc.conv_dense(x, w, None, stride=s), _torch_conv(x, w, None, s, (k - 1) // 2),
                               rtol=1e-12, atol=1e-12)


def test_conv_ones_closed_form():
    # all-ones input and kernel: each output counts the taps that fall inside the image
    Cin = 3
    out = orc.conv_dense(np.ones((1, 5, 6, Cin)), np.ones((3, 3, Cin, 2)))
    assert out.shape == (1, 5, 6, 2)
    assert out[0, 0, 0, 0] == 4 * Cin and out[0, 0, 2, 1] == 6 * Cin and out[0, 2, 2, 0] == 9 * Cin
    assert out[0, 4, 5, 1] == 4 * Cin
    assert (orc.conv_valid(np.ones((1, 5, 6, Cin)), np.ones((3, 3, Cin, 2))) == 9 * Cin).all()


def test_conv_identity_and_shift_taps():
    x = rng0.standard_normal((1, 7, 8, 3))
    eye = np.eye(3)
    w = np.zeros((3, 3, 3, 3)); w[1, 1] = eye
    assert np.array_equal(orc.conv_dense(x, w), x)
    # tap (r,t) = (0,2): out[y,x] = in[y-1, x+1] (cross-correlation: no kernel flip)
    w = np.zeros((3, 3, 3, 3)); w[0, 2] = eye
    out = orc.conv_dense(x, w)
    assert np.array_equal(out[0, 1:, :-1], x[0, :-1, 1:])
    assert (out[0, 0] == 0).all() and (out[0, :, -1] == 0).all()
    # channel mixing orientation: w[r,t,c,o] maps input channel c to output channel o
    w = np.zeros((1, 1, 3, 2)); w[0, 0, 2, 1] = 1.0
    out = orc.conv_valid(x, w)
    assert np.array_equal(out[..., 1], x[..., 2]) and (out[..., 0] == 0).all()


def test_conv_linearity():
    x1, x2 = rng0.standard_normal((2, 1, 6, 6, 2))
    w1, w2 = rng0.standard_normal((2, 3, 3, 2, 3))
    np.testing.assert_allclose(orc.conv_valid(2 * x1 - x2, w1), 2 * orc.conv_valid(x1, w1) - orc.conv_valid(x2, w1),
                               atol=1e-12)
    np.testing.assert_allclose(orc.conv_valid(x1, w1 + 3 * w2), orc.conv_valid(x1, w1) + 3 * orc.conv_valid(x1, w2),
                               atol=1e-12)


# ------------------------------------------------------------------ the method == dense conv on active blocks
@pytest.mark.parametrize("H,W,C,K,k,s,bo", [(16, 16, 3, 4, 3, 1, 4), (13, 10, 2, 3, 3, 1, 4), (17, 17, 2, 2, 3, 2, 2),
                                            (12, 12, 3, 2, 1, 1, 3), (10, 12, 1, 1, 3, 1, 2), (11, 9, 2, 2, 5, 1, 3)])
def test_all_ones_mask_equals_dense_conv(H, W, C, K, k, s, bo):
    g_in, g_out, Ho, Wo = orc.geometry(H, W, k, s, bo)
    x = rng0.standard_normal((2, H, W, C))
    w = rng0.standard_normal((k, k, C, K))
    b = rng0.standard_normal(K)
    idx = orc.reduce_mask(np.ones((2, H, W)), g_in)
    y = orc.sparse_conv_tiled(x, idx, g_in, g_out, w, b, np.full((2, Ho, Wo, K), 7.0), stride=s)
    np.testing.assert_allclose(y, _torch_conv(x, w, b, s, (k - 1) // 2), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("seed", range(6))
def test_tiled_equals_dense_on_active_blocks_brute_force(seed):
    r = np.random.default_rng(seed)
    H, W = int(r.integers(6, 13)), int(r.integers(6, 13))
    C, K = int(r.integers(1, 4)), int(r.integers(1, 4))
    k = int(r.choice([1, 3])); s = int(r.choice([1, 2])); bo = int(r.choice([2, 3, 4]))
    g_in, g_out, Ho, Wo = orc.geometry(H, W, k, s, bo)
    x = r.standard_normal((2, H, W, C)); w = r.standard_normal((k, k, C, K)); b = r.standard_normal(K)
    m = (r.random((2, H, W)) < 0.05).astype(float)
    idx = orc.reduce_mask(m, g_in)
    y0 = r.standard_normal((2, Ho, Wo, K))
    for add in (False, True):
        tiled = orc.sparse_conv_tiled(x, idx, g_in, g_out, w, b, y0, stride=s, add=add)
        dense = orc.sparse_conv_dense(x, idx, g_out, w, b, y0, stride=s, add=add)
        np.testing.assert_allclose(tiled, dense, rtol=1e-12, atol=1e-12)
        bm = orc.block_mask(idx, g_out, 2, Ho, Wo)
        assert np.array_equal(tiled[~bm], y0[~bm])            # inactive pixels bit-identical
        ref = _torch_conv(x, w, b, s, (k - 1) // 2)
        np.testing.assert_allclose(tiled[bm], (y0 + ref if add else ref)[bm], rtol=1e-12, atol=1e-12)


def test_mask_off_leaves_y_untouched():
    g_in, g_out, Ho, Wo = orc.geometry(8, 8, 3, 1, 4)
    idx = orc.reduce_mask(np.zeros((1, 8, 8)), g_in)
    y0 = rng0.standard_normal((1, 8, 8, 2))
    y = orc.sparse_conv_tiled(rng0.standard_normal((1, 8, 8, 2)), idx, g_in, g_out,
                              rng0.standard_normal((3, 3, 2, 2)), None, y0)
    assert np.array_equal(y, y0)


# ------------------------------------------------------------------ residual unit
def _bneck_weights(r, C, Cm):
    return (r.standard_normal((1, 1, C, Cm)), r.standard_normal(Cm), r.standard_normal((3, 3, Cm, Cm)),
            r.standard_normal(Cm), r.standard_normal((1, 1, Cm, C)), r.standard_normal(C))


def _torch_bottleneck(x, w1, b1, w2, b2, w3, b3):
    t1 = _torch_conv(x, w1, b1, 1, 0, relu=True)
    t2 = _torch_conv(t1, w2, b2, 1, 1, relu=True)
    return x + _torch_conv(t2, w3, b3, 1, 0)


@pytest.mark.parametrize("H,W,bo", [(8, 8, 4), (10, 7, 3), (12, 12, 2)])
def test_bottleneck_all_ones_equals_dense_unit(H, W, bo):
    r = np.random.default_rng(H * 100 + W)
    C, Cm = 4, 3
    ws = _bneck_weights(r, C, Cm)
    x = r.standard_normal((2, H, W, C))
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    idx = orc.reduce_mask(np.ones((2, H, W)), g_in)
    y = orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, *ws)
    np.testing.assert_allclose(y, _torch_bottleneck(x, *ws), rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(orc.sparse_bottleneck_dense(x, idx, g_out, *ws), _torch_bottleneck(x, *ws),
                               rtol=1e-11, atol=1e-11)


@pytest.mark.parametrize("H,W,bo", [(8, 8, 4), (10, 7, 3)])
def test_preactivation_unit(H, W, bo):
    """Pre-activation form: with every block active it equals the library's dense pre-activation unit (batch norm
    folded to scale and shift, ReLU, then the three convolutions, residual = x itself); with scale 1, shift 0 and a
    non-negative x it is the plain unit; on a partial mask the tiled and the dense statement agree, and the
    border rule is unchanged although ReLU(shift) is not zero outside the image."""
    r = np.random.default_rng(H * 10 + bo)
    C, Cm = 4, 3
    ws = _bneck_weights(r, C, Cm)
    pre = (r.standard_normal(C), r.standard_normal(C) + 0.5)
    x = r.standard_normal((2, H, W, C))
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    idx = orc.reduce_mask(np.ones((2, H, W)), g_in)
    xa = np.maximum(x * pre[0] + pre[1], 0.0)
    want = x + (_torch_bottleneck(xa, *ws) - xa)                # the library unit's branch on the activated input
    np.testing.assert_allclose(orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, *ws, pre=pre), want, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(orc.sparse_bottleneck_dense(x, idx, g_out, *ws, pre=pre), want, rtol=1e-11, atol=1e-11)
    xp = np.abs(x)
    np.testing.assert_allclose(orc.sparse_bottleneck_tiled(xp, idx, g_in, g_out, *ws, pre=(np.ones(C), np.zeros(C))),
                               orc.sparse_bottleneck_tiled(xp, idx, g_in, g_out, *ws), rtol=1e-12, atol=1e-12)
    part = idx[::3]
    np.testing.assert_allclose(orc.sparse_bottleneck_tiled(x, part, g_in, g_out, *ws, pre=pre),
                               orc.sparse_bottleneck_dense(x, part, g_out, *ws, pre=pre), rtol=1e-11, atol=1e-11)
    # and it differs from the plain unit (the test would pass vacuously if pre were ignored)
    assert np.abs(orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, *ws, pre=pre) -
                  orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, *ws)).max() > 1e-3


def test_bottleneck_partial_mask_and_special_cases():
    r = np.random.default_rng(5)
    H, W, C, Cm, bo = 12, 16, 4, 3, 4
    w1, b1, w2, b2, w3, b3 = _bneck_weights(r, C, Cm)
    x = r.standard_normal((2, H, W, C))
    g_in, g_out, _, _ = orc.geometry(H, W, 3, 1, bo)
    m = (r.random((2, H, W)) < 0.02).astype(float)
    idx = orc.reduce_mask(m, g_in)
    bm = orc.block_mask(idx, g_out, 2, H, W)
    assert 0 < bm.mean() < 1
    y = orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, w1, b1, w2, b2, w3, b3)
    ref = _torch_bottleneck(x, w1, b1, w2, b2, w3, b3)
    np.testing.assert_allclose(y[bm], ref[bm], rtol=1e-11, atol=1e-11)
    assert np.array_equal(y[~bm], x[~bm])
    np.testing.assert_allclose(y, orc.sparse_bottleneck_dense(x, idx, g_out, w1, b1, w2, b2, w3, b3), atol=1e-11)
    # last conv zero: the unit is the identity
    y = orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, w1, b1, w2, b2, 0 * w3, 0 * b3)
    assert np.array_equal(y, x)
    # first conv output forced to zero (w1 = 0, b1 <= 0): away from the image border the
    # branch is the constant relu(b2) @ w3 + b3
    y = orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, 0 * w1, -np.abs(b1), w2, b2, w3, b3)
    const = np.maximum(b2, 0) @ w3[0, 0] + b3
    np.testing.assert_allclose((y - x)[bm], np.broadcast_to(const, x.shape)[bm], atol=1e-12)
    # two units sharing one index list == applying the unit twice
    ws2 = _bneck_weights(r, C, Cm)
    y1 = orc.sparse_bottleneck_tiled(x, idx, g_in, g_out, w1, b1, w2, b2, w3, b3)
    y2 = orc.sparse_bottleneck_tiled(y1, idx, g_in, g_out, *ws2)
    d1 = orc.sparse_bottleneck_dense(x, idx, g_out, w1, b1, w2, b2, w3, b3)
    d2 = orc.sparse_bottleneck_dense(d1, idx, g_out, *ws2)
    # (dense form of a stack differs from the tiled one on halo pixels of inactive blocks only
    #  through t1/t2 of inactive pixels, which the dense form also computes from the current map)
    np.testing.assert_allclose(y2, d2, atol=1e-10)


def _torch_unit(x, w1, b1, w2, b2, w3, b3, stride, shortcut):
    t1 = _torch_conv(x, w1, b1, 1, 0, relu=True)
    t2 = _torch_conv(t1, w2, b2, stride, 1, relu=True)
    sc = x[:, ::stride, ::stride, :] if shortcut is None else _torch_conv(x, shortcut[0], shortcut[1], stride, 0)
    return sc + _torch_conv(t2, w3, b3, 1, 0)


@pytest.mark.parametrize("H,W,bo,stride,C,Cm,Co", [(9, 9, 2, 2, 4, 3, 6), (12, 10, 3, 2, 3, 2, 5), (11, 8, 4, 2, 5, 3, 5),
                                                  (8, 8, 4, 1, 4, 3, 6), (10, 7, 3, 1, 4, 3, 4)])
def test_general_unit_strided_and_projected(H, W, bo, stride, C, Cm, Co):
    """Residual units with a strided 3x3 and a projected (1x1, same stride) shortcut, and stride-1 units whose
    shortcut is a projection: with every block active the tiled statement equals the library's dense unit
    (torch, fp64); on a partial mask tiled and dense agree, active pixels equal torch's, the others keep y; with the
    last convolution zero the unit is the shortcut alone; at stride 1 with the identity it is the unit pinned above."""
    r = np.random.default_rng(H * 100 + W * 10 + stride)
    w1, b1 = r.standard_normal((1, 1, C, Cm)), r.standard_normal(Cm)
    w2, b2 = r.standard_normal((3, 3, Cm, Cm)), r.standard_normal(Cm)
    w3, b3 = r.standard_normal((1, 1, Cm, Co)), r.standard_normal(Co)
    sc = (r.standard_normal((1, 1, C, Co)), r.standard_normal(Co))
    ws = (w1, b1, w2, b2, w3, b3)
    x = r.standard_normal((2, H, W, C))
    g_in, g_out, Ho, Wo = orc.geometry(H, W, 3, stride, bo)
    y0 = r.standard_normal((2, Ho, Wo, Co))
    ref = _torch_unit(x, *ws, stride, sc)
    assert ref.shape == y0.shape
    every = orc.reduce_mask(np.ones((2, Ho, Wo)), g_out)
    np.testing.assert_allclose(orc.sparse_unit_tiled(x, every, g_in, g_out, *ws, y0, stride=stride, shortcut=sc), ref,
                               rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(orc.sparse_unit_dense(x, every, g_out, *ws, y0, stride=stride, shortcut=sc), ref,
                               rtol=1e-11, atol=1e-11)
    part = every[1::3]
    bm = orc.block_mask(part, g_out, 2, Ho, Wo)
    assert 0 < bm.mean() < 1
    yt = orc.sparse_unit_tiled(x, part, g_in, g_out, *ws, y0, stride=stride, shortcut=sc)
    np.testing.assert_allclose(yt[bm], ref[bm], rtol=1e-11, atol=1e-11)
    assert np.array_equal(yt[~bm], y0[~bm])
    np.testing.assert_allclose(yt, orc.sparse_unit_dense(x, part, g_out, *ws, y0, stride=stride, shortcut=sc), atol=1e-11)
    # last convolution zero: what is left is the shortcut, a 1x1 convolution with the unit's stride
    only = orc.sparse_unit_tiled(x, every, g_in, g_out, w1, b1, w2, b2, 0 * w3, 0 * b3, y0, stride=stride, shortcut=sc)
    np.testing.assert_allclose(only, _torch_conv(x, sc[0], sc[1], stride, 0), rtol=1e-11, atol=1e-11)
    if stride == 1 and C == Co:
        # identity shortcut: the unit of Sec. 3.3 as pinned above (scatter-add onto x)
        same = orc.sparse_unit_tiled(x, part, g_in, g_out, *ws, x, stride=1, shortcut=None)
        np.testing.assert_allclose(same, orc.sparse_bottleneck_tiled(x, part, g_in, g_out, *ws), rtol=1e-12, atol=1e-12)
    if stride == 2:
        # the strided tile of Fig. 3: input side (bo - 1) * 2 + 3, neighbouring tiles share one pixel
        assert g_in.size_h == 2 * bo + 1 and g_in.stride_h == 2 * bo
        # identity shortcut at stride 2 (a subsampling shortcut) needs equal channel counts: take the projection away
        if C == Co:
            sub = orc.sparse_unit_tiled(x, every, g_in, g_out, *ws, y0, stride=2, shortcut=None)
            np.testing.assert_allclose(sub, _torch_unit(x, *ws, 2, None), rtol=1e-11, atol=1e-11)


def test_bottleneck_border_needs_zeroed_t1():
    # without zeroing t1 outside the image, relu(b1) leaks into the 3x3 at the border and the
    # all-ones result no longer equals the dense unit: shows the border rule is load-bearing
    r = np.random.default_rng(9)
    w1, b1, w2, b2, w3, b3 = _bneck_weights(r, 3, 2)
    b1 = np.abs(b1) + 0.5
    x = r.standard_normal((1, 8, 8, 3))
    g_in, g_out, _, _ = orc.geometry(8, 8, 3, 1, 4)
    idx = orc.reduce_mask(np.ones((1, 8, 8)), g_in)
    tiles = orc.gather(x, idx, g_in)
    t1 = orc.conv_valid(tiles, w1, b1, relu=True)          # NOT zeroed outside
    t3 = orc.conv_valid(orc.conv_valid(t1, w2, b2, relu=True), w3, b3)
    leaky = orc.scatter(t3, idx, g_out, x, add=True)
    ref = _torch_bottleneck(x, w1, b1, w2, b2, w3, b3)
    assert np.abs(leaky - ref)[0, 0].max() > 1e-3                  # border row differs
    np.testing.assert_allclose(leaky[0, 1:-1, 1:-1], ref[0, 1:-1, 1:-1], atol=1e-11)   # interior agrees
