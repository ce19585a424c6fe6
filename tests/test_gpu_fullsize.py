"""Parity at the full sizes of the benchmark configurations, in the launch configuration bench.py
times (device-side count, cap = all blocks, fused kernels).  The oracle cannot run these sizes
whole in seconds, so it computes a seeded sample of active tiles one by one (every image-border
tile among the active ones is in the sample); properties that hold at any size cover the rest:
the index list is checked whole and pixels of inactive blocks must be bit-identical."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1801_02108_amd as sb
from paper_1801_02108_amd import inputs as gen
from util import CONV_TOL, assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def step(msg):
    print("[case] " + msg, flush=True)


def ogeom(g):
    return orc.Geom(*g.astuple())


def sample_tiles(idx, g, r, n_interior=12):
    """Rows of idx to check: all active tiles touching the image border plus a random few others."""
    border = (idx[:, 1] == 0) | (idx[:, 2] == 0) | (idx[:, 1] == g.bcount_h - 1) | (idx[:, 2] == g.bcount_w - 1)
    b = np.flatnonzero(border)
    if len(b) > 24:
        b = r.choice(b, 24, replace=False)
    rest = np.flatnonzero(~border)
    pick = r.choice(rest, min(n_interior, len(rest)), replace=False) if len(rest) else rest
    return np.sort(np.concatenate([b, pick]))


def blocks_of(y_np, idx_rows, g_out):
    """Stack the output blocks of the listed tiles out of a full [N,H,W,C] array (clipped blocks padded with 0)."""
    out = np.zeros((len(idx_rows), g_out.bsize_h, g_out.bsize_w, y_np.shape[-1]))
    for k, (n, by, bx) in enumerate(idx_rows):
        y0, x0 = by * g_out.bstride_h, bx * g_out.bstride_w
        blk = y_np[n, y0:y0 + g_out.bsize_h, x0:x0 + g_out.bsize_w]
        out[k, :blk.shape[0], :blk.shape[1]] = blk
    return out


def road_mask(r, H, W, g_in, N, target):
    fields = gen.road_band_fields(r, H, W, 3)
    og = ogeom(g_in)
    total = N * g_in.bcount_h * g_in.bcount_w
    m, _, frac = gen.calibrate(lambda s: np.repeat(gen.road_band_mask(fields, s), N, axis=0),
                               lambda mm: len(orc.reduce_mask(mm, og)), total, target, 0.0, 12.0)
    return m, frac


def test_config2_full_size_sampled():
    """800 x 704 x 64 -> 64, bf16, 16 x 16 blocks, road-band mask at 10 % active blocks."""
    step("config 2 full size")
    r = gen.rng_for(2)
    N, H, W, C, K, bo = 1, 800, 704, 64, 64, 16
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, C), "bf16")
    w = gen.conv_weights(r, 3, 3, C, K, "bf16")
    b = gen.bias_vector(r, K)
    mask, frac = road_mask(r, H, W, g_in, N, 0.10)
    assert abs(frac - 0.10) < 0.01
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in, sb.POOL_AVG, 0.0)
    idx = orc.reduce_mask(mask, ogeom(g_in), orc.POOL_AVG, 0.0)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert n == len(idx) and np.array_equal(d_idx[:n].cpu().numpy(), idx)          # whole index list
    y0 = gen.activations(r, (N, Ho, Wo, K), "bf16")
    y = to_dev(y0, "bf16")
    sb.sparse_conv(to_dev(x, "bf16"), d_idx, d_cnt, g_in, g_out, sb.pack_weights(to_dev(w, "bf16")),
                   torch.from_numpy(b).cuda(), y)
    got = to_host(y)
    bm = orc.block_mask(idx, ogeom(g_out), N, Ho, Wo)
    assert np.array_equal(got[~bm], y0[~bm])                                        # inactive pixels untouched
    rows = sample_tiles(idx, g_in, r)
    ref = orc.conv_valid(orc.gather(x, idx[rows], ogeom(g_in)), w, b)
    assert_close(blocks_of(got, idx[rows], g_out), ref, CONV_TOL["bf16"], "config 2 sampled tiles")


@pytest.mark.parametrize("target", [0.10, 0.30])
def test_config3_full_size_sampled(target):
    """Bottleneck 256 -> 64 -> 64 -> 256 on 400 x 352, bf16, 16 x 16 blocks, road-band mask."""
    step("config 3 full size target=%s" % target)
    r = gen.rng_for(3, int(target * 100))
    N, H, W, C, bo = 1, 400, 352, 256, 16
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, C), "bf16")
    ws = gen.bottleneck_weights(r, C, 64, "bf16")
    mask, frac = road_mask(r, H, W, g_in, N, target)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in, sb.POOL_AVG, 0.0)
    idx = orc.reduce_mask(mask, ogeom(g_in), orc.POOL_AVG, 0.0)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert n == len(idx) and np.array_equal(d_idx[:n].cpu().numpy(), idx)
    dws = (sb.pack_weights(to_dev(ws[0], "bf16")), torch.from_numpy(ws[1]).cuda(), sb.pack_weights(to_dev(ws[2], "bf16")),
           torch.from_numpy(ws[3]).cuda(), sb.pack_weights(to_dev(ws[4], "bf16")), torch.from_numpy(ws[5]).cuda())
    dx = to_dev(x, "bf16")
    y = dx.clone()
    sb.sparse_bottleneck(dx, d_idx, d_cnt, g_in, g_out, dws, y)
    got = to_host(y)
    bm = orc.block_mask(idx, ogeom(g_out), N, H, W)
    assert np.array_equal(got[~bm], x[~bm])
    rows = sample_tiles(idx, g_in, r, 6)
    t3 = orc.bottleneck_on_tiles(orc.gather(x, idx[rows], ogeom(g_in)), idx[rows], ogeom(g_in), H, W, *ws)
    ref = blocks_of(x.astype(np.float64), idx[rows], g_out) + t3
    assert_close(blocks_of(got, idx[rows], g_out), ref, CONV_TOL["bf16"], "config 3 sampled tiles")


@pytest.mark.parametrize("bo", [16, 8])
def test_stack_shape_batch_of_samples_sampled(bo):
    """The shape of the batched configurations at a size the test can hold: N = 4 samples of
    800 x 704 x 256 with a per-sample low-resolution mask (about 15 % active blocks), two units
    sharing one index list and alternating two buffers; 16 x 16 and 8 x 8 blocks."""
    step("batched stack, sampled, bo=%d" % bo)
    r = gen.rng_for(5, bo)
    N, H, W, C = 4, 800, 704, 256
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    dev = torch.device("cuda:0")
    tg = torch.Generator(device=dev)
    tg.manual_seed(1234)
    a = torch.randn((N, H, W, C), generator=tg, device=dev, dtype=torch.float32).to(torch.bfloat16)
    b = a.clone()
    x0 = a.clone()
    logits = gen.smooth_noise(r, N, H // 8, W // 8, 2.0)
    og = ogeom(g_in)
    total = N * g_in.bcount_h * g_in.bcount_w
    mask, thr, frac = gen.calibrate(lambda t: gen.lowres_mask(logits, t), lambda mm: len(orc.reduce_mask(mm, og)), total,
                                    0.15, -4.0, 4.0, increasing=False)
    assert abs(frac - 0.15) < 0.01
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).to(dev), g_in)
    idx = orc.reduce_mask(mask, og)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert n == len(idx) and np.array_equal(d_idx[:n].cpu().numpy(), idx)
    units = [gen.bottleneck_weights(r, C, 64, "bf16") for _ in range(2)]
    for ws in units:
        dws = (sb.pack_weights(to_dev(ws[0], "bf16")), torch.from_numpy(ws[1]).to(dev), sb.pack_weights(to_dev(ws[2], "bf16")),
               torch.from_numpy(ws[3]).to(dev), sb.pack_weights(to_dev(ws[4], "bf16")), torch.from_numpy(ws[5]).to(dev))
        sb.sparse_bottleneck(a, d_idx, d_cnt, g_in, g_out, dws, b)
        a, b = b, a
    # inactive pixels never change (checked on the device: the tensors are large)
    bm = torch.from_numpy(orc.block_mask(idx, ogeom(g_out), N, H, W)).to(dev)
    assert torch.equal(a[~bm], x0[~bm])
    # Sampled tiles.  The second unit reads the first unit's output on the tile's halo, so the oracle runs
    # both units on a window of 3 x 3 blocks around each sampled block (clipped at the image edge), treated
    # as an image of its own.  The window's artificial border is a whole block (16 px) away from the centre
    # block, while two stacked units only reach 2 px, so the centre block of the window result is exact.
    rows = r.choice(len(idx), 8, replace=False)
    for k in rows:
        n_, by, bx = (int(v) for v in idx[k])
        gy_lo, gx_lo = max(by - 1, 0) * bo, max(bx - 1, 0) * bo
        gy_hi, gx_hi = min((by + 2) * bo, H), min((bx + 2) * bo, W)
        win = x0[n_, gy_lo:gy_hi, gx_lo:gx_hi].to(torch.float64).cpu().numpy()[None]
        wg_in, wg_out, _, _ = orc.geometry(win.shape[1], win.shape[2], 3, 1, bo)
        sel = idx[(idx[:, 0] == n_) & (idx[:, 1] * bo >= gy_lo) & (idx[:, 1] * bo < gy_hi) &
                  (idx[:, 2] * bo >= gx_lo) & (idx[:, 2] * bo < gx_hi)].copy()
        sel[:, 0] = 0
        sel[:, 1] -= gy_lo // bo
        sel[:, 2] -= gx_lo // bo
        ref = win
        for ws in units:
            ref = orc.sparse_bottleneck_tiled(ref, sel, wg_in, wg_out, *ws)
        cy, cx = by * bo - gy_lo, bx * bo - gx_lo
        got = a[n_, by * bo:by * bo + bo, bx * bo:bx * bo + bo].to(torch.float64).cpu().numpy()
        assert_close(got, ref[0, cy:cy + bo, cx:cx + bo], 3e-2, "stack tile %d" % k)


def _window_reference(x0_dev, idx, n_, by, bx, bo, H, W, units):
    """Oracle result of a stack of residual units on the 3 x 3 block window around block (n_, by, bx), treated as an
    image of its own; returns the window result and the centre block's offset inside it."""
    gy_lo, gx_lo = max(by - 1, 0) * bo, max(bx - 1, 0) * bo
    gy_hi, gx_hi = min((by + 2) * bo, H), min((bx + 2) * bo, W)
    win = x0_dev[n_, gy_lo:gy_hi, gx_lo:gx_hi].to(torch.float64).cpu().numpy()[None]
    wg_in, wg_out, _, _ = orc.geometry(win.shape[1], win.shape[2], 3, 1, bo)
    sel = idx[(idx[:, 0] == n_) & (idx[:, 1] * bo >= gy_lo) & (idx[:, 1] * bo < gy_hi) &
              (idx[:, 2] * bo >= gx_lo) & (idx[:, 2] * bo < gx_hi)].copy()
    sel[:, 0] = 0
    sel[:, 1] -= gy_lo // bo
    sel[:, 2] -= gx_lo // bo
    ref = win
    for ws in units:
        ref = orc.sparse_bottleneck_tiled(ref, sel, wg_in, wg_out, *ws)
    return ref, by * bo - gy_lo, bx * bo - gx_lo


def test_config5_as_stated_sampled():
    """Config 5 at its stated size: N = 8 samples of 800 x 704 x 256, a per-sample low-resolution mask at 15 % active
    blocks, EIGHT residual units with distinct weights sharing one index list and alternating two buffers, 16 x 16
    blocks.  Eight stacked units reach 8 pixels; the oracle runs all eight on the 3 x 3 block window around each
    sampled block, whose artificial border is 16 pixels from the centre block, so the centre block is exact.
    Tolerance: each unit rounds the running sum once more to bf16 (2^-9) and the next unit's branch reads the rounded
    values; 3e-2 holds for 2-3 units, eight get 5e-2 (random-walk growth sqrt(8/3) of the per-unit share)."""
    step("config 5 as stated: N=8, 8 units")
    r = gen.rng_for(5, 88)
    N, H, W, C, bo, n_units = 8, 800, 704, 256, 16, 8
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    dev = torch.device("cuda:0")
    tg = torch.Generator(device=dev)
    tg.manual_seed(gen.BASE_SEED + 588)
    a = torch.empty((N, H, W, C), device=dev, dtype=torch.bfloat16)
    for n_ in range(N):      # sample by sample: the fp32 draw of the whole batch would be 4.6 GB
        a[n_] = torch.randn((H, W, C), generator=tg, device=dev, dtype=torch.float32).to(torch.bfloat16)
    b = a.clone()
    x0 = a.clone()
    logits = gen.smooth_noise(r, N, H // 8, W // 8, 2.0)
    og = ogeom(g_in)
    total = N * g_in.bcount_h * g_in.bcount_w
    assert total == 17600
    mask, thr, frac = gen.calibrate(lambda t: gen.lowres_mask(logits, t), lambda mm: len(orc.reduce_mask(mm, og)), total,
                                    0.15, -4.0, 4.0, increasing=False)
    assert abs(frac - 0.15) < 0.01
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).to(dev), g_in)
    idx = orc.reduce_mask(mask, og)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert n == len(idx) and np.array_equal(d_idx[:n].cpu().numpy(), idx)
    assert len(set(idx[:, 0].tolist())) == N                     # every sample has active blocks of its own
    units = [gen.bottleneck_weights(r, C, 64, "bf16") for _ in range(n_units)]
    for ws in units:
        dws = (sb.pack_weights(to_dev(ws[0], "bf16")), torch.from_numpy(ws[1]).to(dev), sb.pack_weights(to_dev(ws[2], "bf16")),
               torch.from_numpy(ws[3]).to(dev), sb.pack_weights(to_dev(ws[4], "bf16")), torch.from_numpy(ws[5]).to(dev))
        sb.sparse_bottleneck(a, d_idx, d_cnt, g_in, g_out, dws, b)
        a, b = b, a
    torch.cuda.synchronize()
    bm = torch.from_numpy(orc.block_mask(idx, ogeom(g_out), N, H, W)).to(dev)
    for n_ in range(N):                                          # inactive pixels never change, sample by sample
        assert torch.equal(a[n_][~bm[n_]], x0[n_][~bm[n_]])
    # sampled blocks: the first and the last of the list, one at an image corner or edge if active, a few random ones
    edge = np.flatnonzero((idx[:, 1] == 0) | (idx[:, 2] == 0) | (idx[:, 1] == g_in.bcount_h - 1) | (idx[:, 2] == g_in.bcount_w - 1))
    rows = [0, len(idx) - 1] + [int(v) for v in r.choice(len(idx), 4, replace=False)]
    if len(edge):
        rows += [int(v) for v in r.choice(edge, min(2, len(edge)), replace=False)]
    worst = 0.0
    for k in sorted(set(rows)):
        n_, by, bx = (int(v) for v in idx[k])
        ref, cy, cx = _window_reference(x0, idx, n_, by, bx, bo, H, W, units)
        got = a[n_, by * bo:by * bo + bo, bx * bo:bx * bo + bo].to(torch.float64).cpu().numpy()
        worst = max(worst, assert_close(got, ref[0, cy:cy + bo, cx:cx + bo], 5e-2, "config 5 tile %d" % k))
    print("config 5 sampled: worst max|err|/max|ref| = %.3g" % worst, flush=True)


def test_config4_block_32_batch_of_four_sampled():
    """Config 4's largest block size at its stated batch: N = 4 samples of 800 x 704 x 256, 32 x 32 blocks (2200
    blocks, 34 x 34 input tiles), blob mask at about 10 % active blocks, one residual unit; sampled tiles, every
    active image-border tile's candidates among them, against the oracle tile by tile."""
    step("config 4, bo=32, N=4")
    r = gen.rng_for(4, 32)
    N, H, W, C, bo = 4, 800, 704, 256, 32
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    assert N * g_in.bcount_h * g_in.bcount_w == 2200 and g_in.bsize_h == 34
    dev = torch.device("cuda:0")
    tg = torch.Generator(device=dev)
    tg.manual_seed(gen.BASE_SEED + 432)
    dx = torch.randn((N, H, W, C), generator=tg, device=dev, dtype=torch.float32).to(torch.bfloat16)
    field = gen.smooth_noise(r, N, H, W, 24.0)
    og = ogeom(g_in)
    mask, thr, frac = gen.calibrate(lambda t: gen.blob_mask(field, t), lambda mm: len(orc.reduce_mask(mm, og)),
                                    N * g_in.bcount_h * g_in.bcount_w, 0.10, -4.0, 4.0, increasing=False)
    assert abs(frac - 0.10) < 0.01
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).to(dev), g_in)
    idx = orc.reduce_mask(mask, og)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert n == len(idx) and np.array_equal(d_idx[:n].cpu().numpy(), idx)
    ws = gen.bottleneck_weights(r, C, 64, "bf16")
    dws = (sb.pack_weights(to_dev(ws[0], "bf16")), torch.from_numpy(ws[1]).to(dev), sb.pack_weights(to_dev(ws[2], "bf16")),
           torch.from_numpy(ws[3]).to(dev), sb.pack_weights(to_dev(ws[4], "bf16")), torch.from_numpy(ws[5]).to(dev))
    y = dx.clone()
    sb.sparse_bottleneck(dx, d_idx, d_cnt, g_in, g_out, dws, y)
    torch.cuda.synchronize()
    bm = torch.from_numpy(orc.block_mask(idx, ogeom(g_out), N, H, W)).to(dev)
    assert torch.equal(y[~bm], dx[~bm])
    rows = np.unique(np.concatenate([sample_tiles(idx, g_in, r, 5)[:12], [0, len(idx) - 1]]))
    host = {}
    for k in rows:
        n_, by, bx = (int(v) for v in idx[k])
        # the oracle gathers from the whole sample, so that zero padding at the image border is its own
        if n_ not in host:
            host = {n_: dx[n_].to(torch.float64).cpu().numpy()[None]}
        xs = host[n_]
        one = np.array([[0, by, bx]], dtype=np.int32)
        t3 = orc.bottleneck_on_tiles(orc.gather(xs, one, og), one, og, H, W, *ws)
        ref = xs[0, by * bo:(by + 1) * bo, bx * bo:(bx + 1) * bo] + t3[0]
        got = y[n_, by * bo:(by + 1) * bo, bx * bo:(bx + 1) * bo].to(torch.float64).cpu().numpy()
        assert_close(got, ref, CONV_TOL["bf16"], "config 4 bo=32 tile %d" % k)


def test_gather_scatter_of_stacks_beyond_two_gib():
    """Tile stacks whose byte offsets do not fit 31 bits: all 17 600 blocks of N = 8 samples of 800 x 704 x 256 bf16.
    The 18 x 18 input tiles are 2.92 GB: sampled tiles, the first and the last among them, bit-exact against the
    oracle's gather.  The 16 x 16 blocks are 2.31 GB: scattered into a cleared tensor they must give back the input
    bit for bit (every pixel belongs to exactly one block), and scatter-add onto the input must equal x + x."""
    step("gather / scatter, stacks beyond 2 GiB")
    r = gen.rng_for(5, 2)
    N, H, W, C, bo = 8, 800, 704, 256, 16
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    dev = torch.device("cuda:0")
    tg = torch.Generator(device=dev)
    tg.manual_seed(gen.BASE_SEED + 502)
    x = torch.empty((N, H, W, C), device=dev, dtype=torch.bfloat16)
    for n_ in range(N):
        x[n_] = torch.randn((H, W, C), generator=tg, device=dev, dtype=torch.float32).to(torch.bfloat16)
    og_in, og_out = ogeom(g_in), ogeom(g_out)
    ones = np.ones((N, H, W), np.uint8)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(ones).to(dev), g_out, sb.POOL_MAX, 0.0)
    idx = orc.reduce_mask(ones, og_out, orc.POOL_MAX, 0.0)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert n == 17600 == len(idx) and np.array_equal(d_idx.cpu().numpy(), idx)
    tiles = sb.sparse_gather(x, d_idx, d_cnt, g_in)
    assert tiles.numel() * 2 > 2 ** 31
    pick = np.unique(np.concatenate([[0, n - 1, n // 2, 43, 44, 2199, 2200], r.choice(n, 12, replace=False)]))
    host = {}
    for k in pick:
        n_ = int(idx[k, 0])
        one = idx[k:k + 1].copy()
        one[0, 0] = 0
        if n_ not in host:
            host = {n_: x[n_].to(torch.float64).cpu().numpy()[None]}
        ref = orc.gather(host[n_], one, og_in)
        assert np.array_equal(tiles[int(k)].to(torch.float64).cpu().numpy(), ref[0]), "gathered tile %d" % k
    del tiles
    blocks = sb.sparse_gather(x, d_idx, d_cnt, g_out)
    assert blocks.numel() * 2 > 2 ** 31
    y = torch.zeros_like(x)
    sb.sparse_scatter(blocks, d_idx, d_cnt, g_out, y)
    assert torch.equal(y, x)
    sb.sparse_scatter(blocks, d_idx, d_cnt, g_out, y, add=True)
    two = (x.to(torch.float32) * 2).to(torch.bfloat16)      # doubling is exact in bf16
    assert torch.equal(y, two)


STAGE_CASES = [
    # H, W, Cin, Cout, stride, bo: the other stage shapes of the detector backbone (Sec. 4), downsampling and not
    (800, 704, 64, 96, 2, 16),
    (400, 352, 96, 96, 1, 16),
    (400, 352, 96, 192, 2, 16),
    (200, 176, 192, 256, 2, 16),
    (100, 88, 256, 384, 2, 8),
]


@pytest.mark.parametrize("H,W,Cin,Cout,s,bo", STAGE_CASES)
def test_stage_shapes_sampled(H, W, Cin, Cout, s, bo):
    """Single sparse 3x3 convolutions at the backbone's other stage shapes, stride 1 and 2 (for stride 2 the
    input tile is (bo - 1) * 2 + 3 pixels wide and neighbouring tiles overlap by one pixel, Fig. 3), on a
    road-band mask at about 30 % active blocks; sampled tiles against the oracle."""
    step("stage shape %s" % ((H, W, Cin, Cout, s, bo),))
    r = gen.rng_for(6, H + Cin + s)
    N = 1
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, s, bo)
    x = gen.activations(r, (N, H, W, Cin), "bf16")
    w = gen.conv_weights(r, 3, 3, Cin, Cout, "bf16")
    b = gen.bias_vector(r, Cout)
    fields = gen.road_band_fields(r, Ho, Wo, 3)
    og = ogeom(g_out)
    total = N * g_out.bcount_h * g_out.bcount_w
    mask, _, frac = gen.calibrate(lambda sc: gen.road_band_mask(fields, sc), lambda mm: len(orc.reduce_mask(mm, og)), total,
                                  0.30, 0.0, 12.0, tol=0.03)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_out, sb.POOL_AVG, 0.0)
    idx = orc.reduce_mask(mask, og, orc.POOL_AVG, 0.0)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert n == len(idx) and n > 0 and np.array_equal(d_idx[:n].cpu().numpy(), idx)
    y0 = gen.activations(r, (N, Ho, Wo, Cout), "bf16")
    y = to_dev(y0, "bf16")
    sb.sparse_conv(to_dev(x, "bf16"), d_idx, d_cnt, g_in, g_out, sb.pack_weights(to_dev(w, "bf16")),
                   torch.from_numpy(b).cuda(), y, stride=s, relu=True)
    got = to_host(y)
    bm = orc.block_mask(idx, og, N, Ho, Wo)
    assert np.array_equal(got[~bm], y0[~bm])
    rows = sample_tiles(idx, g_out, r, 6)
    ref = np.maximum(orc.conv_valid(orc.gather(x, idx[rows], ogeom(g_in)), w, b, s), 0.0)
    # blocks hanging over the image edge: the part outside is never stored (blocks_of pads it with zeros)
    inside = blocks_of(np.ones((N, Ho, Wo, 1)), idx[rows], g_out) > 0
    assert_close(blocks_of(got, idx[rows], g_out), np.where(inside, ref, 0.0), CONV_TOL["bf16"], "stage shape sampled tiles")


def test_training_side_calls_at_the_headline_size():
    """The tile counts bench.py times for the headline layer (800 x 704 x 64, 16 x 16 blocks, all 2200 blocks): the
    FP8 tile convolution on a seeded sample of tiles, ReLU mask and bias gradient whole, and the normalisation over
    active blocks forward and backward on a road-band mask at 30 % (the oracle works on the gathered active pixels,
    which takes seconds)."""
    step("training-side calls, headline size")
    r = gen.rng_for(2, 91)
    n, th, bo, C = 2200, 18, 16, 64
    cnt = torch.tensor([n], dtype=torch.int32).cuda()
    t_codes = orc.quantize_f8(gen.activations(r, (n, th, th, C), "bf16"), 16.0)
    w_codes = orc.quantize_f8(gen.conv_weights(r, 3, 3, C, C, "bf16"), 64.0)
    out = sb.conv_on_tiles_f8(torch.from_numpy(t_codes).cuda(), cnt, sb.pack_weights_f8(torch.from_numpy(w_codes).cuda()),
                              relu=True, out_scale=1.0 / 1024.0)
    pick = np.unique(np.concatenate([[0, n - 1], r.choice(n, 10, replace=False)]))
    assert_close(to_host(out[torch.from_numpy(pick).cuda()]), orc.conv_valid_f8(t_codes[pick], w_codes, relu=True, out_scale=1.0 / 1024.0),
                 8e-3, "conv_on_tiles_f8, sampled tiles")
    y = to_host(out)
    dy = gen.activations(r, (n, bo, bo, C), "bf16")
    dyd = to_dev(dy, "bf16")
    assert np.array_equal(to_host(sb.relu_backward_on_tiles(out, dyd, cnt)), orc.relu_backward(y, dy))
    db = sb.bias_backward_on_tiles(dyd, cnt).cpu().numpy()
    assert np.abs(db - orc.bias_backward(dy)).max() <= 2e-5 * np.sqrt(n * bo * bo)

    N, H, W = 1, 800, 704
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    mask, frac = road_mask(r, H, W, g_out, N, 0.30)
    idx_np = orc.reduce_mask(mask, ogeom(g_out))
    nb = len(idx_np)
    assert 500 < nb < 800
    idx = torch.from_numpy(np.ascontiguousarray(idx_np)).cuda()
    cntb = torch.tensor([nb], dtype=torch.int32).cuda()
    x = gen.round_to((gen.activations(r, (N, H, W, C), "f32") * 1.5 + 0.25).astype(np.float32), "bf16")
    g = gen.activations(r, (N, H, W, C), "bf16")
    gamma = (r.standard_normal(C) * 0.3 + 1.0).astype(np.float32)
    beta = (r.standard_normal(C) * 0.3).astype(np.float32)
    xd, gd = to_dev(x, "bf16"), to_dev(g, "bf16")
    mean, var = sb.sparse_bn_stats(xd, idx, cntb, g_out)
    gm, bt = torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
    yb = sb.sparse_bn_apply(xd, idx, cntb, g_out, mean, var, gm, bt, eps=1e-3, relu=True, y=torch.zeros_like(xd))
    dx, dgam, dbet = sb.sparse_bn_backward(xd, gd, idx, cntb, g_out, mean, var, gm, bt, eps=1e-3, relu=True)
    inside = orc.block_mask(idx_np, ogeom(g_out), N, H, W)
    om, ov = orc.bn_stats(x, idx_np, ogeom(g_out))
    assert np.allclose(mean.cpu().numpy(), om, rtol=1e-5, atol=1e-5) and np.allclose(var.cpu().numpy(), ov, rtol=2e-4, atol=1e-6)
    ref_y = orc.bn_apply(x, idx_np, ogeom(g_out), om, ov, gamma, beta, 1e-3, np.zeros_like(x), relu=True)
    got_y = to_host(yb)
    assert not got_y[~inside].any()
    assert_close(got_y[inside], ref_y[inside], 8e-3, "bn_apply")
    rdx, rdg, rdb = orc.bn_backward(x, g, idx_np, ogeom(g_out), gamma, beta, 1e-3, np.zeros_like(x), relu=True)
    npx = int(inside.sum())
    assert np.abs(dgam.cpu().numpy() - rdg).max() <= 3e-5 * np.sqrt(npx) + 1e-4 * np.abs(rdg).max()
    assert np.abs(dbet.cpu().numpy() - rdb).max() <= 3e-5 * np.sqrt(npx) + 1e-4 * np.abs(rdb).max()
    got_dx = to_host(dx)
    assert not got_dx[~inside].any()
    assert_close(got_dx[inside], rdx[inside], 1.6e-2, "bn_backward dx")
