"""GPU parity of the tile convolution's gradients against the fp64 oracle (training support for the
convolution of Sec. 3.2): element by element on seeded inputs, for every kernel the forward dispatch can
pick for the gradient's own shape (1x1 and 3x3 matrix-core kernels, the LDS-tiled one, the direct fp32 one)."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1801_02108_amd as sb
from paper_1801_02108_amd import inputs as gen
from util import CONV_TOL, TORCH_DT, assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def step(msg):
    print("[case] " + msg, flush=True)


DGRAD_CASES = [
    # B, th, tw, Cin, Cout, k, s, dtype
    (5, 18, 18, 64, 64, 3, 1, "bf16"),       # the headline layer's tiles
    (3, 18, 18, 64, 64, 3, 1, "f16"),
    (4, 33, 33, 64, 96, 3, 2, "bf16"),       # downsampling layer: the output gradient is spread by the stride
    (2, 18, 18, 96, 192, 3, 1, "bf16"),
    (3, 10, 10, 32, 40, 3, 1, "bf16"),
    (2, 17, 17, 256, 384, 3, 2, "bf16"),
    (3, 16, 16, 64, 256, 1, 1, "bf16"),      # 1x1: no frame, no mirror
    (3, 18, 18, 96, 24, 1, 1, "bf16"),       # 1x1 with channel counts of the 96-channel stage
    (2, 9, 9, 24, 40, 1, 2, "f16"),          # 1x1 at stride 2: the gradient is spread, every other pixel stays zero
    (2, 12, 20, 24, 16, 3, 1, "f32"),        # direct fp32 kernel
    (2, 12, 13, 8, 8, 3, 2, "f32"),          # the last input column is not reached by any window
    (2, 14, 12, 16, 8, 3, 2, "bf16"),        # the last input row is not reached by any window
    (2, 11, 9, 6, 5, 3, 1, "bf16"),          # channel counts the matrix-core kernels do not take
    (1, 9, 9, 3, 7, 5, 1, "f16"),
    (2, 9, 11, 16, 16, 3, 3, "bf16"),        # stride 3
]


@pytest.mark.parametrize("B,th,tw,Cin,Cout,k,s,dtype", DGRAD_CASES)
def test_conv_on_tiles_backward_data(B, th, tw, Cin, Cout, k, s, dtype):
    step("conv_on_tiles_backward_data %s" % ((B, th, tw, Cin, Cout, k, s, dtype),))
    r = gen.rng_for(21, th * 1000 + tw * 10 + Cin + Cout + s)
    oh, ow = (th - k) // s + 1, (tw - k) // s + 1
    g = gen.activations(r, (B + 1, oh, ow, Cout), dtype)
    w = gen.conv_weights(r, k, k, Cin, Cout, dtype, unit_variance=(dtype == "f32"))
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    wt = sb.pack_weights_transposed(to_dev(w, dtype))
    out = torch.full((B + 1, th, tw, Cin), 5.0, dtype=TORCH_DT[dtype]).cuda()
    sb.conv_on_tiles_backward_data(to_dev(g, dtype), cnt, wt, th, tw, stride=s, out=out)
    got = to_host(out)
    ref = orc.conv_valid_backward_data(g[:B], w, th, tw, stride=s)
    assert_close(got[:B], ref, CONV_TOL[dtype], "conv_on_tiles_backward_data")
    assert (got[B] == 5.0).all()                        # tiles beyond the count are not touched
    # input rows and columns that no window reaches get an exact zero
    rh, rw = (oh - 1) * s + k, (ow - 1) * s + k
    assert (got[:B, rh:] == 0).all() and (got[:B, :, rw:] == 0).all()


WGRAD_CASES = [
    # B, th, tw, Cin, Cout, k, s, dtype
    (5, 18, 18, 64, 64, 3, 1, "bf16"),       # the headline layer's tiles: one tile per split
    (300, 18, 18, 64, 64, 3, 1, "bf16"),     # more tiles than splits: several tiles per workgroup, ragged
    (7, 18, 18, 64, 64, 3, 1, "f16"),
    (20, 33, 33, 64, 96, 3, 2, "bf16"),      # downsampling layer; the second block of output channels is half empty
    (9, 34, 34, 32, 64, 3, 2, "bf16"),       # even tile at stride 2: the last row and column are never read
    (6, 18, 18, 96, 192, 3, 1, "bf16"),      # several channel blocks
    (11, 10, 10, 40, 24, 3, 1, "bf16"),      # 8x8 blocks: half-filled matrix rows, ragged channel counts
    (4, 12, 15, 8, 16, 3, 1, "f16"),         # ragged tile: 10 x 13 outputs
    (3, 34, 34, 16, 16, 3, 1, "bf16"),       # 32 x 32 outputs: two segments per row
    (3, 37, 41, 16, 8, 3, 2, "bf16"),        # stride 2 with two segments per row (18 x 20 outputs)
    (2, 21, 16, 8, 8, 3, 1, "bf16"),         # 19 output rows: the last stage is partly empty
    (3, 12, 20, 24, 16, 3, 1, "f32"),        # plain kernel
    (3, 11, 9, 6, 5, 3, 1, "bf16"),
    (4, 16, 16, 64, 32, 1, 1, "bf16"),       # 1x1: one accumulator per wave
    (40, 18, 18, 256, 64, 1, 1, "bf16"),     # first convolution of the residual unit on its input tile (two segments)
    (5, 16, 16, 64, 256, 1, 1, "f16"),       # its last convolution
    (300, 16, 16, 64, 64, 1, 1, "bf16"),     # 1x1 with more tiles than splits: two or three tiles per workgroup
    (3, 17, 17, 32, 48, 1, 2, "bf16"),       # 1x1 at stride 2: 9 x 9 outputs, odd phase never read
    (4, 10, 10, 40, 24, 1, 1, "bf16"),
    (6, 17, 17, 64, 64, 1, 1, "bf16"),       # 289 pixels: one pixel in the last row of 16
    (9, 7, 5, 8, 16, 1, 1, "f16"),           # 35 pixels: not a whole item of four at the end
    (2, 9, 9, 3, 7, 5, 2, "f16"),
    (2, 13, 11, 16, 16, 3, 3, "bf16"),
]


@pytest.mark.parametrize("B,th,tw,Cin,Cout,k,s,dtype", WGRAD_CASES)
def test_conv_on_tiles_backward_weights(B, th, tw, Cin, Cout, k, s, dtype):
    step("conv_on_tiles_backward_weights %s" % ((B, th, tw, Cin, Cout, k, s, dtype),))
    r = gen.rng_for(23, th * 1000 + tw * 10 + Cin + Cout + s)
    oh, ow = (th - k) // s + 1, (tw - k) // s + 1
    x = gen.activations(r, (B + 2, th, tw, Cin), dtype)
    g = gen.activations(r, (B + 2, oh, ow, Cout), dtype)
    xd, gd = to_dev(x, dtype), to_dev(g, dtype)
    ref = orc.conv_valid_backward_weights(x[:B], g[:B], k, k, stride=s)
    # fp32 accumulation of exact products over B * oh * ow terms in a tree of partial sums
    tol = 1e-4 if dtype == "f32" else 2e-5
    for n in (B, 1, 0):
        cnt = torch.tensor([n], dtype=torch.int32).cuda()
        dw = torch.full((k, k, Cin, Cout), 7.0, dtype=torch.float32).cuda()
        sb.conv_on_tiles_backward_weights(xd, gd, cnt, k, stride=s, out=dw)
        want = ref if n == B else orc.conv_valid_backward_weights(x[:n], g[:n], k, k, stride=s)
        if n == 0:
            assert (dw == 0).all()
        else:
            assert_close(to_host(dw), want, tol, "conv_on_tiles_backward_weights n=%d" % n)
        if n == B:
            dw2 = torch.empty_like(dw)
            sb.conv_on_tiles_backward_weights(xd, gd, cnt, k, stride=s, out=dw2)
            assert torch.equal(dw, dw2)                  # fixed summation order: the same bits again


def test_sparse_conv_gradients_end_to_end():
    """dL/dx and dL/dw of the whole sparse convolution from library calls only: gather of dL/dy with the output
    geometry, data gradient on tiles, gather_backward into the image; gather of x, weight gradient on the two tile
    stacks; against the oracle's composition of the same steps."""
    N, H, W, Cin, Cout, bo, dtype = 2, 70, 66, 64, 96, 16, "bf16"
    for s in (1, 2):
        step("sparse conv input gradient stride %d" % s)
        r = gen.rng_for(22, s)
        g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, s, bo)
        mask = (r.random((N, H, W)) < 0.002).astype(np.float64)
        og_in, og_out = orc.Geom(*g_in.astuple()), orc.Geom(*g_out.astuple())
        idx_np = orc.reduce_mask(mask, og_in)
        n, total = len(idx_np), N * g_in.bcount_h * g_in.bcount_w
        assert 0 < n < total
        buf = np.zeros((n + 2, 3), dtype=np.int32)
        buf[:n] = idx_np
        idx, cnt = torch.from_numpy(buf).cuda(), torch.tensor([n], dtype=torch.int32).cuda()
        dy = gen.activations(r, (N, Ho, Wo, Cout), dtype)
        w = gen.conv_weights(r, 3, 3, Cin, Cout, dtype)
        dy_tiles = sb.sparse_gather(to_dev(dy, dtype), idx, cnt, g_out)
        din_tiles = sb.conv_on_tiles_backward_data(dy_tiles, cnt, sb.pack_weights_transposed(to_dev(w, dtype)),
                                                   g_in.bsize_h, g_in.bsize_w, stride=s)
        dx = torch.zeros((N, H, W, Cin), dtype=TORCH_DT[dtype]).cuda()
        sb.sparse_gather_backward(din_tiles, idx, cnt, g_in, dx)
        ref_tiles = orc.conv_valid_backward_data(orc.gather(dy, idx_np, og_out), w, g_in.bsize_h, g_in.bsize_w, stride=s)
        # the library rounds the tile gradient to bf16 before the overlap sum; so does the reference
        ref_tiles_r = torch.from_numpy(ref_tiles).to(TORCH_DT[dtype]).to(torch.float64).numpy()
        ref = orc.gather_backward(ref_tiles_r, idx_np, og_in, np.zeros((N, H, W, Cin)))
        assert_close(to_host(dx), ref, CONV_TOL[dtype], "sparse conv dL/dx")
        # dL/dw of the same layer: the forward input gathered with the input geometry against the gathered dL/dy
        x = gen.activations(r, (N, H, W, Cin), dtype)
        x_tiles = sb.sparse_gather(to_dev(x, dtype), idx, cnt, g_in)
        dw = sb.conv_on_tiles_backward_weights(x_tiles, dy_tiles, cnt, 3, stride=s)
        ref_dw = orc.conv_valid_backward_weights(orc.gather(x, idx_np, og_in), orc.gather(dy, idx_np, og_out), 3, 3, stride=s)
        assert_close(to_host(dw), ref_dw, 2e-5, "sparse conv dL/dw")


@pytest.mark.parametrize("n,th,Cin,Cout,s", [(2200, 18, 64, 64, 1), (220, 18, 64, 64, 1), (550, 33, 64, 96, 2)])
def test_gradients_at_full_size_sampled(n, th, Cin, Cout, s):
    """The tile counts and shapes bench.py times (all 2200 blocks and 10 % of them for the headline layer, the dense
    downsampling layer), in its launch configuration.  The oracle computes what it can one by one: the data gradient
    of a seeded sample of tiles (the first and the last among them), and a seeded sample of weights, each of which is
    a sum over every pixel of every tile."""
    step("gradients at full size %s" % ((n, th, Cin, Cout, s),))
    dtype = "bf16"
    r = gen.rng_for(24, n + th + Cout)
    oh = (th - 3) // s + 1
    x = gen.activations(r, (n, th, th, Cin), dtype)
    g = gen.activations(r, (n, oh, oh, Cout), dtype)
    w = gen.conv_weights(r, 3, 3, Cin, Cout, dtype)
    xd, gd = to_dev(x, dtype), to_dev(g, dtype)
    cnt = torch.tensor([n], dtype=torch.int32).cuda()
    din = sb.conv_on_tiles_backward_data(gd, cnt, sb.pack_weights_transposed(to_dev(w, dtype)), th, th, stride=s)
    dw = sb.conv_on_tiles_backward_weights(xd, gd, cnt, 3, stride=s)
    pick = np.unique(np.concatenate([[0, n - 1], r.choice(n, 10, replace=False)]))
    ref = orc.conv_valid_backward_data(g[pick], w, th, th, stride=s)
    assert_close(to_host(din[torch.from_numpy(pick).cuda()]), ref, CONV_TOL[dtype], "data gradient, sampled tiles")
    got = to_host(dw)
    samples = [(int(r.integers(0, 3)), int(r.integers(0, 3)), int(r.integers(0, Cin)), int(r.integers(0, Cout))) for _ in range(48)]
    samples += [(0, 0, 0, 0), (2, 2, Cin - 1, Cout - 1), (1, 2, Cin - 1, 0), (2, 0, 0, Cout - 1)]
    want = np.array([float((x[:, kr:kr + s * (oh - 1) + 1:s, kt:kt + s * (oh - 1) + 1:s, c] * g[:, :, :, o]).sum())
                     for kr, kt, c, o in samples])
    have = np.array([got[kr, kt, c, o] for kr, kt, c, o in samples])
    # every weight's gradient is a sum of n * oh * oh products of independent unit-scale factors: scale sqrt(terms)
    scale = np.sqrt(n * oh * oh)
    assert np.abs(have - want).max() <= 2e-5 * scale + 2e-5 * np.abs(want).max()
    assert np.isfinite(got).all() and 0.3 < np.sqrt((got ** 2).mean()) / scale < 3.0


RELU_BIAS_CASES = [(7, 18, 18, 64, "bf16"), (3, 5, 7, 6, "f32"), (4, 3, 3, 10, "f16"), (2, 1, 3, 2, "bf16"), (5, 16, 16, 256, "bf16")]


@pytest.mark.parametrize("B,h,w,C,dtype", RELU_BIAS_CASES)
def test_relu_and_bias_backward_on_tiles(B, h, w, C, dtype):
    step("relu / bias backward %s" % ((B, h, w, C, dtype),))
    r = gen.rng_for(25, B * 100 + h * w + C)
    y = gen.activations(r, (B + 1, h, w, C), dtype)
    y[r.random(y.shape) < 0.3] = 0.0
    y = np.abs(y) * (r.random(y.shape) < 0.7)                       # a ReLU output: zeros and positive values
    y = gen.round_to(y.astype(np.float32), dtype)
    dy = gen.activations(r, (B + 1, h, w, C), dtype)
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    out = torch.full((B + 1, h, w, C), 3.0, dtype=TORCH_DT[dtype]).cuda()
    sb.relu_backward_on_tiles(to_dev(y, dtype), to_dev(dy, dtype), cnt, out=out)
    got = to_host(out)
    assert np.array_equal(got[:B], orc.relu_backward(y[:B], dy[:B])) and (got[B] == 3.0).all()
    inplace = to_dev(dy, dtype)
    sb.relu_backward_on_tiles(to_dev(y, dtype), inplace, cnt, out=inplace)
    assert torch.equal(inplace[:B], out[:B])
    db = sb.bias_backward_on_tiles(to_dev(dy, dtype), cnt)
    ref = orc.bias_backward(dy[:B])
    assert np.abs(db.cpu().numpy() - ref).max() <= 1e-5 * np.sqrt(B * h * w) + 1e-6
    db2 = sb.bias_backward_on_tiles(to_dev(dy, dtype), cnt)
    assert torch.equal(db, db2)
    assert (sb.bias_backward_on_tiles(to_dev(dy, dtype), torch.tensor([0], dtype=torch.int32).cuda()) == 0).all()
    # both in one pass: the masked gradient bit for bit, its sum against the oracle and, bit for bit, against the sum
    # the separate call makes of the masked stack
    out2 = torch.full((B + 1, h, w, C), 3.0, dtype=TORCH_DT[dtype]).cuda()
    _, dbm = sb.relu_bias_backward_on_tiles(to_dev(y, dtype), to_dev(dy, dtype), cnt, out=out2)
    assert torch.equal(out2, out)
    refm = orc.bias_backward(orc.relu_backward(y[:B], dy[:B]))
    assert np.abs(dbm.cpu().numpy() - refm).max() <= 1e-5 * np.sqrt(B * h * w) + 1e-6
    assert torch.equal(dbm, sb.bias_backward_on_tiles(out, cnt))
    inplace = to_dev(dy, dtype)
    _, dbi = sb.relu_bias_backward_on_tiles(to_dev(y, dtype), inplace, cnt, out=inplace)
    assert torch.equal(inplace[:B], out[:B]) and torch.equal(inplace[B], to_dev(dy, dtype)[B]) and torch.equal(dbi, dbm)
    _, db0 = sb.relu_bias_backward_on_tiles(to_dev(y, dtype), to_dev(dy, dtype), torch.tensor([0], dtype=torch.int32).cuda(), out=out2)
    assert (db0 == 0).all() and torch.equal(out2, out)             # no active tile: nothing written, zero sums


@pytest.mark.parametrize("C,Cm,dens", [(64, 64, 0.02), (256, 64, 0.004), (96, 24, 0.01)])
def test_residual_unit_backward_composed_from_single_calls(C, Cm, dens):
    """The residual branch of a unit (Sec. 3.3) forward with its activations kept, then every gradient from library
    calls alone: weight, bias and data gradients of the three convolutions, the two ReLU masks, and the gather's
    gradient into the image.  The oracle's chain rule runs on the same kept activations (the ReLU masks are
    decisions, taken on the stored bf16 values by both sides)."""
    step("residual unit backward C=%d Cm=%d" % (C, Cm))
    dtype, bo, N, H, W = "bf16", 16, 1, 70, 66
    r = gen.rng_for(26, C)
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    og_in = orc.Geom(*g_in.astuple())
    mask = (r.random((N, H, W)) < dens).astype(np.float64)
    mask[0, 0, 0] = mask[0, H - 1, W - 1] = 1.0                      # corner tiles: t1 is zeroed outside the image
    idx_np = orc.reduce_mask(mask, og_in)
    n = len(idx_np)
    buf = np.zeros((n + 1, 3), dtype=np.int32)
    buf[:n] = idx_np
    idx, cnt = torch.from_numpy(buf).cuda(), torch.tensor([n], dtype=torch.int32).cuda()
    x = gen.activations(r, (N, H, W, C), dtype)
    w1, b1, w2, b2, w3, b3 = gen.bottleneck_weights(r, C, Cm, dtype)
    dt3 = gen.activations(r, (n + 1, bo, bo, C), dtype)
    dev = lambda a: to_dev(a, dtype)
    fb = lambda b: torch.from_numpy(b).cuda()
    # forward, activations kept
    tiles = sb.sparse_gather(dev(x), idx, cnt, g_in)
    t1 = sb.conv_on_tiles(tiles, cnt, sb.pack_weights(dev(w1)), fb(b1), relu=True)
    sb.zero_outside(t1, idx, cnt, g_in, H, W)
    t2 = sb.conv_on_tiles(t1, cnt, sb.pack_weights(dev(w2)), fb(b2), relu=True)
    # backward
    d3 = dev(dt3)
    th = g_in.bsize_h
    dw3 = sb.conv_on_tiles_backward_weights(t2, d3, cnt, 1)
    db3 = sb.bias_backward_on_tiles(d3, cnt)
    d2 = sb.relu_backward_on_tiles(t2, sb.conv_on_tiles_backward_data(d3, cnt, sb.pack_weights_transposed(dev(w3)), bo, bo), cnt)
    dw2 = sb.conv_on_tiles_backward_weights(t1, d2, cnt, 3)
    db2 = sb.bias_backward_on_tiles(d2, cnt)
    d1 = sb.relu_backward_on_tiles(t1, sb.conv_on_tiles_backward_data(d2, cnt, sb.pack_weights_transposed(dev(w2)), th, th), cnt)
    dw1 = sb.conv_on_tiles_backward_weights(tiles, d1, cnt, 1)
    db1 = sb.bias_backward_on_tiles(d1, cnt)
    dtiles = sb.conv_on_tiles_backward_data(d1, cnt, sb.pack_weights_transposed(dev(w1)), th, th)
    dx = torch.zeros((N, H, W, C), dtype=TORCH_DT[dtype]).cuda()
    sb.sparse_gather_backward(dtiles, idx, cnt, g_in, dx)
    # oracle on the kept activations
    ref = orc.bottleneck_backward_on_tiles(orc.gather(x, idx_np, og_in), idx_np, og_in, H, W, w1, b1, w2, b2, w3, b3, dt3[:n],
                                           saved=(to_host(t1)[:n], to_host(t2)[:n]))
    tol = 3e-2                                                       # a chain of up to three bf16 roundings of the gradient
    assert_close(to_host(dtiles)[:n], ref[0], tol, "d tiles")
    for name, got, want in (("dw1", dw1, ref[1]), ("dw2", dw2, ref[3]), ("dw3", dw3, ref[5])):
        assert_close(to_host(got), want, tol, name)
    for name, got, want in (("db1", db1, ref[2]), ("db2", db2, ref[4]), ("db3", db3, ref[6])):
        assert_close(to_host(got), want, tol, name)
    ref_tiles_r = torch.from_numpy(ref[0]).to(TORCH_DT[dtype]).to(torch.float64).numpy()
    assert_close(to_host(dx), orc.gather_backward(ref_tiles_r, idx_np, og_in, np.zeros((N, H, W, C))), tol, "dx")
    # the forward pass that keeps its activations, as one call: the same t1 and t2, and t3 against the oracle's branch
    k1, k2, k3 = sb.bottleneck_forward_keep_on_tiles(tiles, idx, cnt, g_in, H, W, (sb.pack_weights(dev(w1)), fb(b1), sb.pack_weights(dev(w2)),
                                                                                     fb(b2), sb.pack_weights(dev(w3)), fb(b3)))
    assert torch.equal(k1[:n], t1[:n]) and torch.equal(k2[:n], t2[:n])
    assert_close(to_host(k3)[:n], orc.bottleneck_on_tiles(orc.gather(x, idx_np, og_in), idx_np, og_in, H, W, w1, b1, w2, b2, w3, b3),
                 tol, "t3 of the keeping forward pass")
    # the one-call form runs the same sequence: the same bits
    one = sb.bottleneck_backward_on_tiles(tiles, t1, t2, d3, cnt, (sb.pack_weights_transposed(dev(w1)),
                                                                    sb.pack_weights_transposed(dev(w2)),
                                                                    sb.pack_weights_transposed(dev(w3))))
    for got, want in zip(one, (dtiles, dw1, db1, dw2, db2, dw3, db3)):
        assert torch.equal(got[:n] if got.dim() == 4 and got.shape[0] == n + 1 else got, want[:n] if want.dim() == 4 and want.shape[0] == n + 1 else want)


def test_weight_gradient_of_a_stack_beyond_two_gib():
    """13 500 tiles of 18 x 18 x 256 (the residual unit's first convolution at the batched configurations' scale) are
    2.24 GB: byte offsets into the stack do not fit 31 bits, and the kernel addresses every tile through a descriptor
    of its own.  Inputs come from a seeded device generator (a host copy serves the oracle: sampled single weights, each a sum
    over every pixel of every tile, and the last tiles' whole contribution)."""
    step("weight gradient, stack beyond 2 GiB")
    n, th, C, K = 13500, 18, 256, 64
    gen_t = torch.Generator(device="cuda")
    gen_t.manual_seed(gen.BASE_SEED + 27)
    x = torch.randn((n, th, th, C), generator=gen_t, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    g = torch.randn((n, th, th, K), generator=gen_t, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    assert x.numel() * 2 > 2 ** 31
    cnt = torch.tensor([n], dtype=torch.int32).cuda()
    dw = sb.conv_on_tiles_backward_weights(x, g, cnt, 1)
    xc, gc = x.cpu(), g.cpu()
    got = dw.cpu().numpy()
    r = gen.rng_for(27)
    samples = [(int(r.integers(0, C)), int(r.integers(0, K))) for _ in range(10)] + [(0, 0), (C - 1, K - 1), (C - 1, 0), (0, K - 1)]
    scale = np.sqrt(n * th * th)
    # one weight of a 1x1 kernel depends on one input and one output channel only: the oracle's weight gradient on
    # those two channel planes of the WHOLE stack is that weight
    def plane(t, c):
        return t[..., c:c + 1].to(torch.float64).numpy()
    for c, o in samples:
        want = float(orc.conv_valid_backward_weights(plane(xc, c), plane(gc, o), 1, 1)[0, 0, 0, 0])
        assert abs(got[0, 0, c, o] - want) <= 2e-5 * scale + 2e-5 * abs(want), (c, o, got[0, 0, c, o], want)
    # the last tiles reach the sums: with three left out, every weight moves by the oracle's gradient of those three
    cnt2 = torch.tensor([n - 3], dtype=torch.int32).cuda()
    dw2 = sb.conv_on_tiles_backward_weights(x, g, cnt2, 1).cpu().numpy()
    tail = orc.conv_valid_backward_weights(xc[n - 3:].to(torch.float64).numpy(), gc[n - 3:].to(torch.float64).numpy(), 1, 1)
    assert np.abs(tail).max() > 10.0
    assert np.abs((got - dw2) - tail).max() <= 4e-5 * scale


def test_pointwise_forward_and_data_gradient_of_a_stack_beyond_two_gib():
    """The same 2.24 GB stack through the pointwise kernel, once as the input of the residual unit's first convolution
    (256 -> 64) and once as the result of that convolution's data gradient (64 -> 256): every tile is addressed from a
    64-bit base through a descriptor of its own.  Sampled tiles, the first and the last among them, against the oracle."""
    step("pointwise forward / data gradient, stack beyond 2 GiB")
    n, th, C, K = 13500, 18, 256, 64
    gen_t = torch.Generator(device="cuda")
    gen_t.manual_seed(gen.BASE_SEED + 29)
    x = torch.randn((n, th, th, C), generator=gen_t, device="cuda", dtype=torch.float32).to(torch.bfloat16)
    assert x.numel() * 2 > 2 ** 31
    r = gen.rng_for(29)
    w = gen.conv_weights(r, 1, 1, C, K, "bf16")
    wd = to_dev(w, "bf16")
    cnt = torch.tensor([n], dtype=torch.int32).cuda()
    y = sb.conv_on_tiles(x, cnt, sb.pack_weights(wd), None, relu=False)
    # whole sampled tiles, the first and the last of the stack among them, against the oracle's tile convolution
    pick = np.unique(np.concatenate([[0, n - 1, n // 2, 6472, 6473], r.integers(0, n, 8)]))   # 6473 * 165888 B > 2^30
    sel = torch.from_numpy(pick).cuda()
    assert_close(to_host(y[sel]), orc.conv_valid(to_host(x[sel]), w), CONV_TOL["bf16"], "pointwise forward, sampled tiles")
    # data gradient: dL/dx = dL/dy W^T, a stack of the size of x
    del x
    dx = sb.conv_on_tiles_backward_data(y, cnt, sb.pack_weights_transposed(wd), th, th)
    assert dx.numel() * 2 > 2 ** 31
    assert_close(to_host(dx[sel]), orc.conv_valid_backward_data(to_host(y[sel]), w, th, th), CONV_TOL["bf16"],
                 "pointwise data gradient, sampled tiles")


def _random_gradient_shapes(n, seed):
    """Seeded draws over what the matrix-core gradient kernels take: 1x1 and 3x3, stride 1 or 2, channels in multiples of 8."""
    r = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        k = (1, 3)[int(r.integers(0, 2))]
        s = int(r.integers(1, 3))
        th, tw = int(r.integers(k, 36)), int(r.integers(k, 36))
        out.append((int(r.integers(1, 7)), th, tw, 8 * int(r.integers(1, 25)), 8 * int(r.integers(1, 25)), k, s,
                    ("bf16", "f16")[int(r.integers(0, 2))]))
    return out


@pytest.mark.parametrize("B,th,tw,Cin,Cout,k,s,dtype", _random_gradient_shapes(24, 18010210))
def test_gradients_on_random_shapes(B, th, tw, Cin, Cout, k, s, dtype):
    """Both gradients on seeded random tiles: rows per stage, segments, stride phases, channel blocks and the choice
    between the pointwise, the 3x3 and the plain kernels all vary with the shape."""
    step("gradients random %s" % ((B, th, tw, Cin, Cout, k, s, dtype),))
    r = gen.rng_for(31, th * 1000 + tw * 10 + Cin + Cout + s + k)
    oh, ow = (th - k) // s + 1, (tw - k) // s + 1
    x = gen.activations(r, (B + 1, th, tw, Cin), dtype)
    g = gen.activations(r, (B + 1, oh, ow, Cout), dtype)
    w = gen.conv_weights(r, k, k, Cin, Cout, dtype)
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    dw = sb.conv_on_tiles_backward_weights(to_dev(x, dtype), to_dev(g, dtype), cnt, k, stride=s)
    assert_close(to_host(dw), orc.conv_valid_backward_weights(x[:B], g[:B], k, k, stride=s), 2e-5, "weights")
    dx = torch.full((B + 1, th, tw, Cin), 5.0, dtype=TORCH_DT[dtype]).cuda()
    sb.conv_on_tiles_backward_data(to_dev(g, dtype), cnt, sb.pack_weights_transposed(to_dev(w, dtype)), th, tw, stride=s, out=dx)
    got = to_host(dx)
    assert_close(got[:B], orc.conv_valid_backward_data(g[:B], w, th, tw, stride=s), CONV_TOL[dtype], "data")
    assert (got[B] == 5.0).all()
