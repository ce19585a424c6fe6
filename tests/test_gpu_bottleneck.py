"""GPU parity of the sparse residual (bottleneck) unit against the fp64 oracle: the branch on
gathered tiles, the fused one-kernel unit, stacks with two alternating buffers, and the unit
composed from single calls for block sizes the fused kernel does not take."""
import ctypes

import numpy as np
import pytest
import torch

import oracle as orc
import paper_1801_02108_amd as sb
from paper_1801_02108_amd import inputs as gen
from util import round_like, CONV_TOL, TORCH_DT, assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def step(msg):
    print("[case] " + msg, flush=True)


def ogeom(g):
    return orc.Geom(*g.astuple())


def dev_weights(ws, dtype):
    w1, b1, w2, b2, w3, b3 = ws
    return (sb.pack_weights(to_dev(w1, dtype)), torch.from_numpy(b1).cuda(), sb.pack_weights(to_dev(w2, dtype)),
            torch.from_numpy(b2).cuda(), sb.pack_weights(to_dev(w3, dtype)), torch.from_numpy(b3).cuda())


def block_aligned_mask(r, N, H, W, bo, dens):
    """Mask made of whole bo x bo blocks (ragged last blocks included) with the given block density."""
    bh, bw = -(-H // bo), -(-W // bo)
    blocks = (r.random((N, bh, bw)) < dens).astype(np.uint8)
    return np.repeat(np.repeat(blocks, bo, axis=1), bo, axis=2)[:, :H, :W].copy()


UNIT_CASES = [
    # N, H, W, C, bo, dtype
    (2, 48, 48, 256, 16, "bf16"),
    (1, 40, 56, 128, 16, "bf16"),     # ragged: 40 = 2*16 + 8
    (1, 64, 32, 64, 16, "f16"),
    (1, 64, 96, 256, 32, "bf16"),     # four 16x16 sub-tiles per block
    (1, 40, 40, 64, 32, "f16"),       # sub-tiles hanging over the image edge
    (2, 40, 24, 256, 8, "bf16"),      # 8 x 8 blocks: the 8-pixel sub-tile variant
    (1, 37, 29, 64, 8, "f16"),        # ... with ragged image edges
    (1, 48, 72, 128, 24, "bf16"),     # block side a multiple of 8 only: nine 8 x 8 sub-tiles per block
    (3, 160, 192, 64, 16, "bf16"),    # 360 blocks: at density 1.0 and 0.3 the device picks different variants
]


@pytest.mark.parametrize("N,H,W,C,bo,dtype", UNIT_CASES)
def test_bottleneck_on_tiles_and_fused(N, H, W, C, bo, dtype):
    _unit_case(N, H, W, C, 64, bo, dtype)


UNIT_WIDTH_CASES = [
    # N, H, W, C, Cm, bo, dtype: the unit widths of the detector backbone's stages (Sec. 4) and bottleneck widths around them
    (1, 48, 64, 96, 24, 16, "bf16"),      # second stage: 96 / 24; C = 96 fills one and a half 64-channel chunks
    (2, 40, 40, 192, 48, 16, "bf16"),     # third stage: 192 / 48, three chunks
    (1, 40, 24, 96, 24, 8, "f16"),        # 8 x 8 blocks
    (1, 64, 48, 128, 32, 16, "bf16"),     # bottleneck width exactly 32: two k-steps per tap in W2 / W3
    (1, 48, 48, 256, 56, 16, "bf16"),     # a width between 32 and 64
    (1, 37, 45, 192, 8, 8, "bf16"),       # the narrowest, ragged image edges
    (3, 160, 192, 96, 24, 16, "bf16"),    # 360 blocks: both sub-tile variants
]


@pytest.mark.parametrize("N,H,W,C,Cm,bo,dtype", UNIT_WIDTH_CASES)
def test_unit_widths_of_the_backbone(N, H, W, C, Cm, bo, dtype):
    _unit_case(N, H, W, C, Cm, bo, dtype)


def _unit_case(N, H, W, C, Cm, bo, dtype):
    step("bottleneck %s" % ((N, H, W, C, Cm, bo, dtype),))
    r = gen.rng_for(3, H * 100 + C + bo + (0 if Cm == 64 else Cm))
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, C), dtype)
    ws = gen.bottleneck_weights(r, C, Cm, dtype)
    dws = dev_weights(ws, dtype)
    dx = to_dev(x, dtype)
    for dens in (1.0, 0.3, 0.0):
        mask = block_aligned_mask(r, N, H, W, bo, dens)
        d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_out)
        idx = orc.reduce_mask(mask, ogeom(g_out))
        assert sb.read_count(d_cnt, d_idx.shape[0]) == len(idx)
        # --- branch on gathered tiles
        tiles = sb.sparse_gather(dx, d_idx, d_cnt, g_in)
        t3 = torch.full((d_idx.shape[0], bo, bo, C), 3.0, dtype=TORCH_DT[dtype]).cuda()
        sb.bottleneck_on_tiles(tiles, d_idx, d_cnt, g_in, g_out, H, W, dws, out=t3)
        ref_t3 = orc.bottleneck_on_tiles(orc.gather(x, idx, ogeom(g_in)), idx, ogeom(g_in), H, W, *ws)
        got = to_host(t3)
        assert_close(got[:len(idx)], ref_t3, CONV_TOL[dtype], "bottleneck_on_tiles")
        assert (got[len(idx):] == 3.0).all()
        # --- separate scatter-add onto a copy of x (the paper's in-place form)
        y = dx.clone()
        sb.sparse_scatter(t3, d_idx, d_cnt, g_out, y, add=True)
        ref = orc.sparse_bottleneck_tiled(x, idx, ogeom(g_in), ogeom(g_out), *ws)
        unfused = to_host(y)
        assert_close(unfused, ref, CONV_TOL[dtype], "unfused unit")
        # --- fused unit into a second buffer holding other values at inactive pixels
        y0 = gen.activations(r, (N, H, W, C), dtype)
        y = to_dev(y0, dtype)
        sb.sparse_bottleneck(dx, d_idx, d_cnt, g_in, g_out, dws, y)
        got = to_host(y)
        bm = orc.block_mask(idx, ogeom(g_out), N, H, W)
        assert np.array_equal(got[~bm], y0[~bm])                   # inactive pixels neither read nor written
        assert_close(got[bm], ref[bm], CONV_TOL[dtype], "fused unit")
        # the fused kernel forms x + t3 in fp32 and rounds once; the unfused path rounds t3 to the storage type (its
        # tile stack) and the sum again: half a unit in the last place of t3 plus one of the sum apart, at most
        eps = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11
        t3_img = orc.scatter(to_host(t3)[:len(idx)], idx, ogeom(g_out), np.zeros_like(x), add=False)
        apart = eps * np.abs(t3_img) + 2 * eps * np.maximum(np.abs(got), np.abs(unfused))
        assert (np.abs(got - unfused) <= apart)[bm].all()
        # A tighter, second check: the oracle with t1, t2 and t3 rounded to the storage type where the kernel rounds
        # them.  What is left is fp32 summation order and the rare value that lands on the other side of a rounding
        # boundary: every element within four units in the last place (bf16: 2^-8, f16: 2^-11) of the magnitude
        # of its terms, where the stated tolerance allows 2e-2 of the tensor's RMS.
        if len(idx):
            rl = lambda a: round_like(a, dtype)
            tiles_r = orc.gather(x, idx, ogeom(g_in))
            t1_r = rl(orc.zero_outside(orc.conv_valid(tiles_r, ws[0], ws[1], relu=True), idx, ogeom(g_in), H, W))
            t2_r = rl(orc.conv_valid(t1_r, ws[2], ws[3], relu=True))
            t3_r = rl(orc.conv_valid(t2_r, ws[4], ws[5]))
            y_r = rl(orc.scatter(t3_r, idx, ogeom(g_out), x, add=True))
            # magnitude an element's error scales with: |x| plus the sum of |t2| |w3| over the last layer's terms (t3
            # itself may be small by cancellation while a one-unit change of any t2 moves it by that unit's share)
            t3_mag = orc.conv_valid(np.abs(t2_r), np.abs(ws[4]), np.abs(ws[5]))
            mag = np.abs(x) + orc.scatter(t3_mag, idx, ogeom(g_out), np.zeros_like(x), add=False)
            ulp = 2.0 ** -8 if dtype == "bf16" else 2.0 ** -11
            worst = (np.abs(got - y_r) / (mag + 1e-30))[bm].max()
            print("rounded-intermediates check: worst %.2f units in the last place" % (worst / ulp), flush=True)
            assert worst <= 4 * ulp, "fused unit against the oracle with rounded intermediates: %.3g units in the last place" % (worst / ulp)
        if dens == 1.0:                                            # every block active: the dense unit
            assert_close(got, orc.sparse_bottleneck_dense(x, idx, ogeom(g_out), *ws), CONV_TOL[dtype], "dense unit")


@pytest.mark.parametrize("N,H,W,C,bo,dtype", [(2, 48, 48, 256, 16, "bf16"), (1, 40, 56, 128, 16, "f16"), (2, 40, 24, 256, 8, "bf16"),
                                              (1, 37, 29, 64, 8, "f16")])
def test_preactivation_unit(N, H, W, C, bo, dtype):
    """Pre-activation form of the unit: ReLU(scale * x + shift) feeds conv1, the residual stays x."""
    step("pre-activation bottleneck %s" % ((N, H, W, C, bo, dtype),))
    r = gen.rng_for(3, H * 100 + C + bo + 5)
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, C), dtype)
    ws = gen.bottleneck_weights(r, C, 64, dtype)
    scale = (1.0 + 0.3 * r.standard_normal(C)).astype(np.float32)
    shift = (0.5 * r.standard_normal(C)).astype(np.float32)
    pre = (scale.astype(np.float64), shift.astype(np.float64))
    dpre = (torch.from_numpy(scale).cuda(), torch.from_numpy(shift).cuda())
    dws = dev_weights(ws, dtype)
    dx = to_dev(x, dtype)
    for dens in (1.0, 0.3):
        mask = block_aligned_mask(r, N, H, W, bo, dens)
        d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_out)
        idx = orc.reduce_mask(mask, ogeom(g_out))
        ref = orc.sparse_bottleneck_tiled(x, idx, ogeom(g_in), ogeom(g_out), *ws, pre=pre)
        tiles = sb.sparse_gather(dx, d_idx, d_cnt, g_in)
        t3 = sb.bottleneck_on_tiles(tiles, d_idx, d_cnt, g_in, g_out, H, W, dws, pre=dpre)
        y = dx.clone()
        sb.sparse_scatter(t3, d_idx, d_cnt, g_out, y, add=True)
        unfused = to_host(y)
        assert_close(unfused, ref, CONV_TOL[dtype], "unfused pre-activation unit")
        y0 = gen.activations(r, (N, H, W, C), dtype)
        y = to_dev(y0, dtype)
        sb.sparse_bottleneck(dx, d_idx, d_cnt, g_in, g_out, dws, y, pre=dpre)
        got = to_host(y)
        bm = orc.block_mask(idx, ogeom(g_out), N, H, W)
        assert np.array_equal(got[~bm], y0[~bm])
        assert_close(got[bm], ref[bm], CONV_TOL[dtype], "fused pre-activation unit")
        assert np.array_equal(got[bm], unfused[bm])
        # it is not the plain unit
        plain = orc.sparse_bottleneck_tiled(x, idx, ogeom(g_in), ogeom(g_out), *ws)
        assert np.abs(plain - ref).max() > 0.05


def test_bottleneck_border_rule_matters_on_gpu_inputs():
    """With a large positive b1 the value ReLU(b1) would leak into the 3x3 at the image border if t1
    were not zeroed there; the GPU result must follow the dense unit (which pads t1 with zeros)."""
    step("bottleneck border rule")
    r = gen.rng_for(3, 4242)
    N, H, W, C, bo = 1, 32, 32, 64, 16
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, C), "bf16")
    w1, b1, w2, b2, w3, b3 = gen.bottleneck_weights(r, C, 64, "bf16")
    b1 = (np.abs(b1) + 2.0).astype(np.float32)
    ws = (w1, b1, w2, b2, w3, b3)
    d_idx, d_cnt = sb.reduce_mask(torch.ones((N, H, W), dtype=torch.uint8).cuda(), g_out)
    idx = orc.reduce_mask(np.ones((N, H, W)), ogeom(g_out))
    y = torch.zeros((N, H, W, C), dtype=torch.bfloat16).cuda()
    sb.sparse_bottleneck(to_dev(x, "bf16"), d_idx, d_cnt, g_in, g_out, dev_weights(ws, "bf16"), y)
    assert_close(to_host(y), orc.sparse_bottleneck_dense(x, idx, ogeom(g_out), *ws), CONV_TOL["bf16"], "border")


def test_stack_of_units_with_two_buffers():
    """Three units sharing one index list, alternating two buffers that both start as the input."""
    step("bottleneck stack")
    r = gen.rng_for(5, 31)
    N, H, W, C, bo = 2, 48, 64, 128, 16
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, C), "bf16")
    units = [gen.bottleneck_weights(r, C, 64, "bf16") for _ in range(3)]
    mask = block_aligned_mask(r, N, H, W, bo, 0.4)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_out)
    idx = orc.reduce_mask(mask, ogeom(g_out))
    a = to_dev(x, "bf16")
    b = a.clone()
    ref = x.astype(np.float64)
    for ws in units:
        sb.sparse_bottleneck(a, d_idx, d_cnt, g_in, g_out, dev_weights(ws, "bf16"), b)
        a, b = b, a
        # the oracle consumes what the GPU actually fed the next unit (bf16-rounded activations)
        ref = orc.sparse_bottleneck_tiled(ref, idx, ogeom(g_in), ogeom(g_out), *ws)
    # three units: rounding of the running sum to bf16 after each unit adds ~2^-9 relative per unit
    assert_close(to_host(a), ref, 3e-2, "stack of 3")
    bm = orc.block_mask(idx, ogeom(g_out), N, H, W)
    assert np.array_equal(to_host(a)[~bm], x[~bm])


def test_unit_composed_from_single_calls_for_small_blocks():
    """Blocks whose sides are no multiple of 8 are not taken by the fused kernel (SBNET_EUNSUPPORTED); the unit
    composed of gather, three conv_on_tiles calls, zero_outside and scatter-add gives the oracle's result."""
    step("bottleneck composed, bo=4")
    r = gen.rng_for(4, 8)
    N, H, W, C, bo = 1, 40, 24, 64, 4
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, C), "bf16")
    ws = gen.bottleneck_weights(r, C, 64, "bf16")
    w1p, b1, w2p, b2, w3p, b3 = dev_weights(ws, "bf16")
    mask = block_aligned_mask(r, N, H, W, bo, 0.6)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_out)
    idx = orc.reduce_mask(mask, ogeom(g_out))
    dx = to_dev(x, "bf16")
    with pytest.raises(sb.SbnetError) as e:
        sb.sparse_bottleneck(dx, d_idx, d_cnt, g_in, g_out, (w1p, b1, w2p, b2, w3p, b3), dx.clone())
    assert e.value.code == sb.EUNSUPPORTED
    tiles = sb.sparse_gather(dx, d_idx, d_cnt, g_in)
    t1 = sb.conv_on_tiles(tiles, d_cnt, w1p, b1, relu=True)
    sb.zero_outside(t1, d_idx, d_cnt, g_in, H, W)
    t2 = sb.conv_on_tiles(t1, d_cnt, w2p, b2, relu=True)
    t3 = sb.conv_on_tiles(t2, d_cnt, w3p, b3)
    y = dx.clone()
    sb.sparse_scatter(t3, d_idx, d_cnt, g_out, y, add=True)
    assert_close(to_host(y), orc.sparse_bottleneck_tiled(x, idx, ogeom(g_in), ogeom(g_out), *ws), CONV_TOL["bf16"],
                 "composed unit")


def test_zero_outside_bit_exact():
    step("zero_outside")
    r = gen.rng_for(4, 9)
    N, H, W, C, bo = 2, 21, 13, 6, 4
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    mask = (r.random((N, H, W)) < 0.2).astype(np.uint8)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in)
    idx = orc.reduce_mask(mask, ogeom(g_in))
    t = gen.activations(r, (d_idx.shape[0], g_in.bsize_h, g_in.bsize_w, C), "bf16")
    dt = to_dev(t, "bf16")
    sb.zero_outside(dt, d_idx, d_cnt, g_in, H, W)
    got = to_host(dt)
    assert np.array_equal(got[:len(idx)], orc.zero_outside(t[:len(idx)], idx, ogeom(g_in), H, W))
    assert np.array_equal(got[len(idx):], t[len(idx):])


GENERAL_UNIT_CASES = [
    # N, H, W, Cin, Cm, Cout, stride, bo, projection, dtype
    (1, 66, 50, 64, 24, 96, 2, 16, True, "bf16"),      # the downsampling units of the backbone's four stages (Sec. 4) ...
    (2, 49, 65, 96, 48, 192, 2, 8, True, "bf16"),      # ... odd extents: blocks hang over the edge of the halved map
    (1, 64, 48, 192, 64, 256, 2, 16, True, "bf16"),
    (1, 40, 40, 256, 96, 384, 2, 8, True, "f16"),
    (1, 48, 40, 384, 96, 384, 1, 8, False, "bf16"),    # fourth stage, stride 1, identity: wider than the one-kernel unit takes
    (2, 40, 56, 96, 24, 96, 1, 16, False, "bf16"),     # a shape the one-kernel unit takes: routed to it
    (1, 32, 48, 64, 16, 128, 1, 16, True, "bf16"),     # stride 1 with a projection (a change of width without downsampling)
    (1, 35, 29, 24, 8, 40, 2, 4, True, "bf16"),        # small channel counts, 4 x 4 blocks
    (2, 258, 250, 64, 24, 96, 2, 8, True, "bf16"),     # more 8 x 8 items than workgroups: every workgroup loops over tiles
    (1, 100, 90, 128, 64, 256, 2, 24, True, "f16"),    # 3 x 3 sub-tiles per block, blocks over the edge, f16
    (1, 70, 70, 64, 32, 128, 2, 16, True, "f16"),
    (2, 130, 130, 384, 96, 384, 1, 8, False, "bf16"),  # fourth stage as one launch (width above 64), more items than workgroups
    (1, 50, 44, 384, 80, 384, 1, 16, False, "f16"),    # width 80, 16 x 16 blocks (8 x 8 sub-tiles)
    (2, 260, 200, 256, 72, 384, 2, 8, True, "bf16"),   # its downsampling unit, width 72, every workgroup loops
]
# shapes the one-launch downsampling unit serves (it needs no workspace: called without one below)
ONE_LAUNCH_DOWN = {(64, 96), (96, 192), (192, 256), (64, 128), (128, 256)}


@pytest.mark.parametrize("N,H,W,Cin,Cm,Cout,stride,bo,proj,dtype", GENERAL_UNIT_CASES)
def test_sparse_unit_any_width_stride_and_shortcut(N, H, W, Cin, Cm, Cout, stride, bo, proj, dtype):
    """sbnet_sparse_unit against the oracle's step-by-step unit: strided 3x3, projected shortcut, every stage width."""
    step("sparse_unit %s" % ((N, H, W, Cin, Cm, Cout, stride, bo, proj, dtype),))
    r = gen.rng_for(3, 9000 + H + Cin + Cout + stride)
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, stride, bo)
    og_in, og_out = ogeom(g_in), ogeom(g_out)
    x = gen.activations(r, (N, H, W, Cin), dtype)
    w1, b1 = gen.conv_weights(r, 1, 1, Cin, Cm, dtype), gen.bias_vector(r, Cm)
    w2, b2 = gen.conv_weights(r, 3, 3, Cm, Cm, dtype), gen.bias_vector(r, Cm)
    w3, b3 = gen.conv_weights(r, 1, 1, Cm, Cout, dtype, scale=0.5), gen.bias_vector(r, Cout)
    sc = (gen.conv_weights(r, 1, 1, Cin, Cout, dtype), gen.bias_vector(r, Cout)) if proj else None
    fb = lambda b: torch.from_numpy(b).cuda()
    dws = (sb.pack_weights(to_dev(w1, dtype)), fb(b1), sb.pack_weights(to_dev(w2, dtype)), fb(b2), sb.pack_weights(to_dev(w3, dtype)), fb(b3))
    dsc = (sb.pack_weights(to_dev(sc[0], dtype)), fb(sc[1])) if proj else None
    dx = to_dev(x, dtype)
    for dens in (1.0, 0.3, 0.0):
        mask = (r.random((N, Ho, Wo)) < dens * (0.02 if dens < 1.0 else 1.0)).astype(np.uint8) if dens > 0 else np.zeros((N, Ho, Wo), np.uint8)
        d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_out)
        idx = orc.reduce_mask(mask, og_out)
        assert sb.read_count(d_cnt, d_idx.shape[0]) == len(idx)
        y0 = gen.activations(r, (N, Ho, Wo, Cout), dtype)
        y = to_dev(y0, dtype)
        one_launch = stride == 2 and proj and bo % 8 == 0 and (((Cin, Cout) in ONE_LAUNCH_DOWN and Cm <= 64) or
                                                               ((Cin, Cout) == (256, 384) and 64 < Cm <= 96))
        one_launch = one_launch or (stride == 1 and not proj and Cin == 384 and 64 < Cm <= 96 and bo % 8 == 0)
        none = torch.empty((0,), dtype=torch.uint8, device="cuda")
        sb.sparse_unit(dx, d_idx, d_cnt, g_in, g_out, dws, y, stride=stride, shortcut=dsc, workspace=none if one_launch else None)
        got = to_host(y)
        ref = orc.sparse_unit_tiled(x, idx, og_in, og_out, w1, b1, w2, b2, w3, b3, y0, stride=stride, shortcut=sc)
        bm = orc.block_mask(idx, og_out, N, Ho, Wo)
        assert np.array_equal(got[~bm], y0[~bm])
        assert_close(got[bm], ref[bm], CONV_TOL[dtype], "sparse_unit")
        if dens == 1.0:
            assert_close(got, orc.sparse_unit_dense(x, idx, og_out, w1, b1, w2, b2, w3, b3, y0, stride=stride, shortcut=sc),
                         CONV_TOL[dtype], "dense unit")
        if not proj and dens == 0.3:
            # the identity shortcut in place (the scatter-add of Sec. 3.4): y is x
            z = dx.clone()
            sb.sparse_unit(z, d_idx, d_cnt, g_in, g_out, dws, z, stride=1, shortcut=None)
            ref_in = orc.sparse_unit_tiled(x, idx, og_in, og_out, w1, b1, w2, b2, w3, b3, x, stride=1, shortcut=None)
            got_in = to_host(z)
            assert np.array_equal(got_in[~bm], x[~bm])
            assert_close(got_in[bm], ref_in[bm], CONV_TOL[dtype], "sparse_unit in place")


def test_sparse_unit_rejects_what_it_cannot_mean():
    g_in, g_out, Ho, Wo = sb.geometry(32, 32, 3, 2, 8)
    lib = sb.lib()
    d = torch.zeros(64, dtype=torch.int32).cuda()
    p = ctypes.c_void_p(d.data_ptr())
    # identity shortcut at stride 2
    rc = lib.sbnet_sparse_unit(p, sb.BF16, 1, 32, 32, 64, 16, 64, 2, p, p, 4, g_in, g_out, p, p, p, p, p, p, None, None, p, Ho, Wo,
                               None, 0, None)
    assert rc == sb.EINVAL and b"identity" in lib.sbnet_last_error()
    # geometry of another stride
    g1_in, g1_out, _, _ = sb.geometry(32, 32, 3, 1, 8)
    rc = lib.sbnet_sparse_unit(p, sb.BF16, 1, 32, 32, 64, 16, 96, 2, p, p, 4, g1_in, g1_out, p, p, p, p, p, p, p, p, p, Ho, Wo,
                               None, 0, None)
    assert rc == sb.EINVAL and b"geometries" in lib.sbnet_last_error()
