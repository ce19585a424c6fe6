"""GPU parity: every entry point of libsbnet_hip.so, called through the C ABI, against the
fp64 CPU oracle on the same seeded inputs.  Indices, gather and scatter must match bit for
bit; convolution outputs within the stated relative tolerance."""
import ctypes

import numpy as np
import pytest
import torch

import oracle as orc
import paper_1801_02108_amd as sb
from paper_1801_02108_amd import inputs as gen
from util import CONV_TOL, TORCH_DT, assert_close, round_like, to_dev, to_host

pytestmark = pytest.mark.gpu


def step(msg):
    print("[case] " + msg, flush=True)


def ogeom(g):
    """binding geometry -> oracle geometry (same eight integers, separately defined structs)."""
    return orc.Geom(*g.astuple())


def dev_indices(idx_np, cap=None):
    cap = max(len(idx_np), 1) if cap is None else cap
    buf = np.zeros((cap, 3), dtype=np.int32)
    buf[:len(idx_np)] = idx_np
    return torch.from_numpy(buf).cuda(), torch.tensor([len(idx_np)], dtype=torch.int32).cuda()


# --------------------------------------------------------------------------- geometry
@pytest.mark.parametrize("H,W,k,s,bo", [(64, 64, 3, 1, 8), (800, 704, 3, 1, 16), (13, 10, 3, 1, 4), (17, 17, 3, 2, 2),
                                        (12, 12, 1, 1, 3), (50, 88, 3, 1, 32)])
def test_geometry_matches_oracle(H, W, k, s, bo):
    g_in, g_out, ho, wo = sb.geometry(H, W, k, s, bo)
    og_in, og_out, oho, owo = orc.geometry(H, W, k, s, bo)
    assert g_in.astuple() == og_in.astuple() and g_out.astuple() == og_out.astuple() and (ho, wo) == (oho, owo)


# --------------------------------------------------------------------------- reduce_mask
def _reduce_case(mask_np, g, pool, thr, mdt):
    m = torch.from_numpy(mask_np.astype(np.uint8 if mdt == "u8" else np.float32)).cuda()
    idx, cnt = sb.reduce_mask(m, g, pool, thr)
    n = sb.read_count(cnt, idx.shape[0])
    want = orc.reduce_mask(mask_np, ogeom(g), pool, float(np.float32(thr)))
    assert n == len(want), (n, len(want))
    assert np.array_equal(idx[:n].cpu().numpy(), want)


@pytest.mark.parametrize("H,W,bo,N", [(64, 64, 8, 1), (48, 80, 16, 3), (37, 29, 4, 2), (100, 176, 32, 2), (33, 1000, 8, 1)])
@pytest.mark.parametrize("mdt", ["u8", "f32"])
def test_reduce_mask_binary(H, W, bo, N, mdt):
    step("reduce_mask binary H=%d W=%d bo=%d N=%d %s" % (H, W, bo, N, mdt))
    r = gen.rng_for(1, H * W + bo)
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    for dens in (0.0, 0.002, 0.05, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.float32)
        for g in (g_in, g_out):
            for pool in (sb.POOL_MAX, sb.POOL_AVG):
                _reduce_case(mask, g, pool, 0.0, mdt)
        _reduce_case(mask, g_in, sb.POOL_AVG, 0.01, mdt)


def test_reduce_mask_real_valued_max_and_avg():
    step("reduce_mask real-valued")
    r = gen.rng_for(1, 77)
    H, W, bo = 60, 44, 4
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    mask = (r.random((2, H, W)) * (r.random((2, H, W)) < 0.1)).astype(np.float32)
    for thr in (0.0, 0.25, 0.9):
        _reduce_case(mask, g_in, sb.POOL_MAX, thr, "f32")
    # average pooling on real values: summation order may flip a block sitting on the threshold,
    # so blocks whose pooled value is within 1e-6 of it are left out of the comparison
    for thr in (0.01, 0.03):
        m = torch.from_numpy(mask).cuda()
        idx, cnt = sb.reduce_mask(m, g_in, sb.POOL_AVG, thr)
        n = sb.read_count(cnt, idx.shape[0])
        got = {tuple(x) for x in idx[:n].cpu().numpy()}
        og = ogeom(g_in)
        t32 = float(np.float32(thr))
        sure_on = {tuple(x) for x in orc.reduce_mask(mask, og, orc.POOL_AVG, t32 + 1e-6)}
        maybe_on = {tuple(x) for x in orc.reduce_mask(mask, og, orc.POOL_AVG, t32 - 1e-6)}
        assert sure_on <= got <= maybe_on
        assert list(map(tuple, idx[:n].cpu().numpy())) == sorted(got)


@pytest.mark.parametrize("N,h,w,factor,bo,quant", [(2, 25, 22, 8, 16, 0.85), (1, 13, 9, 8, 8, 0.5), (3, 20, 12, 4, 16, 0.97), (1, 10, 11, 8, 16, 0.0)])
def test_reduce_mask_on_a_coarse_map_equals_reducing_its_upsampled_threshold(N, h, w, factor, bo, quant):
    """A mask predicted at 1/factor resolution (config 5: a logit map, thresholded and upsampled by pixel repetition):
    max-pooling the coarse map over sbnet_coarse_geometry's windows lists the blocks of the upsampled binary mask."""
    step("reduce_mask on a coarse map %s" % ((N, h, w, factor, bo, quant),))
    r = gen.rng_for(5, 40 + h + w + bo)
    logits = r.standard_normal((N, h, w)).astype(np.float32)
    thr = max(float(np.quantile(logits, quant)), 0.0) if quant > 0 else 0.0
    H, W = h * factor, w * factor
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    mask = np.repeat(np.repeat((logits > thr).astype(np.uint8), factor, axis=1), factor, axis=2)
    ref = orc.reduce_mask(mask, ogeom(g_in))
    i_up, c_up = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in)
    i_lo, c_lo = sb.reduce_mask(torch.from_numpy(logits).cuda(), sb.coarse_geometry(g_in, factor), sb.POOL_MAX, thr)
    n = sb.read_count(c_up, i_up.shape[0])
    assert n == len(ref) == sb.read_count(c_lo, i_lo.shape[0])
    assert np.array_equal(i_up.cpu().numpy()[:n], ref) and np.array_equal(i_lo.cpu().numpy()[:n], ref)


def test_reduce_mask_negative_values_max_pool_counts_outside_as_zero():
    step("reduce_mask negative values")
    H, W, bo = 16, 16, 4
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    mask = -np.ones((1, H, W), dtype=np.float32)
    _reduce_case(mask, g_in, sb.POOL_MAX, -0.5, "f32")     # only border windows see a 0 > -0.5


def test_reduce_mask_cap_smaller_than_count():
    step("reduce_mask cap")
    H, W, bo = 64, 64, 8
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    mask = np.ones((1, H, W), dtype=np.uint8)
    idx = torch.full((10, 3), -7, dtype=torch.int32).cuda()
    _, cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in, indices=idx)
    with pytest.raises(sb.SbnetError) as e:
        sb.read_count(cnt, 10)
    assert e.value.code == sb.ECAP
    assert int(cnt.item()) == 64
    assert np.array_equal(idx.cpu().numpy(), orc.reduce_mask(mask, ogeom(g_in))[:10])


def test_reduce_mask_repeatable_and_overwrites_count():
    step("reduce_mask repeat")
    r = gen.rng_for(1, 5)
    H, W, bo = 96, 128, 8
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    m = torch.from_numpy((r.random((2, H, W)) < 0.01).astype(np.uint8)).cuda()
    idx0, cnt0 = sb.reduce_mask(m, g_in)
    ref_i, ref_c = idx0.clone(), cnt0.clone()
    for _ in range(20):
        idx, cnt = sb.reduce_mask(m, g_in, indices=idx0, count=cnt0)
        assert torch.equal(cnt, ref_c) and torch.equal(idx[:int(ref_c)], ref_i[:int(ref_c)])


@pytest.mark.parametrize("fill", [0x00, 0xff, 0x5b])
def test_reduce_mask_reuses_one_workspace_whatever_it_held(fill):
    """The same scratch buffer serves a sequence of different problems; its first contents are arbitrary."""
    step("reduce_mask shared workspace fill=%#x" % fill)
    r = gen.rng_for(1, 9)
    cases = [(1, 64, 64, 8), (3, 48, 80, 4), (2, 100, 176, 16), (1, 64, 64, 8)]
    geoms = [sb.geometry(H, W, 3, 1, bo)[0] for (_, H, W, bo) in cases]
    need = max(sb.workspace_bytes(c[0], g) for c, g in zip(cases, geoms))
    ws = torch.full((need,), fill, dtype=torch.uint8).cuda()
    for rep in range(2):
        for (N, H, W, bo), g in zip(cases, geoms):
            mask = (r.random((N, H, W)) < 0.03).astype(np.uint8)
            idx, cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g, workspace=ws)
            want = orc.reduce_mask(mask, ogeom(g))
            n = sb.read_count(cnt, idx.shape[0])
            assert n == len(want) and np.array_equal(idx[:n].cpu().numpy(), want)


@pytest.mark.parametrize("N,H,W,bo,dens", [(4, 800, 704, 16, None),     # the batched configurations' block grid
                                           (2, 512, 512, 4, None),      # 256 block rows of 128 blocks
                                           (1, 4200, 40, 1, 0.3)])      # 4200 block rows: long prefix over row counts
def test_reduce_mask_many_blocks(N, H, W, bo, dens):
    step("reduce_mask many blocks N=%d H=%d W=%d bo=%d" % (N, H, W, bo))
    r = gen.rng_for(1, 11 + bo)
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    mask = gen.lowres_mask(gen.smooth_noise(r, N, H // 8, W // 8, 2.0), 1.0) if bo > 1 else r.random((N, H, W)) < dens
    for pool in (sb.POOL_MAX, sb.POOL_AVG):
        _reduce_case(np.asarray(mask, dtype=np.float32), g_in, pool, 0.0, "u8")
    _reduce_case(np.ones((N, H, W), dtype=np.float32), g_in, sb.POOL_AVG, 0.0, "f32")


# --------------------------------------------------------------------------- gather / scatter
GS_CASES = [
    # H, W, C, k, s, bo, N, dtype
    (64, 64, 16, 3, 1, 8, 1, "f32"),
    (48, 80, 64, 3, 1, 16, 2, "bf16"),
    (37, 29, 3, 3, 1, 4, 2, "bf16"),       # odd channel count: 2-byte vectors, ragged blocks
    (37, 29, 5, 3, 1, 4, 1, "f32"),
    (40, 40, 12, 5, 1, 8, 1, "f16"),       # 8-byte vectors, halo 2
    (33, 47, 256, 3, 1, 16, 1, "bf16"),
    (35, 35, 8, 3, 2, 4, 2, "f16"),        # strided geometry
    (24, 24, 6, 1, 1, 3, 1, "bf16"),       # 1x1: no halo
]


@pytest.mark.parametrize("H,W,C,k,s,bo,N,dtype", GS_CASES)
def test_gather_bit_exact(H, W, C, k, s, bo, N, dtype):
    step("gather %s" % ((H, W, C, k, s, bo, N, dtype),))
    r = gen.rng_for(2, H * 1000 + W + C)
    g_in, g_out, _, _ = sb.geometry(H, W, k, s, bo)
    x = gen.activations(r, (N, H, W, C), dtype)
    for dens in (0.004, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.float32)
        idx = orc.reduce_mask(mask, ogeom(g_in))
        cap = len(idx) + 3
        d_idx, d_cnt = dev_indices(idx, cap)
        tiles = torch.full((cap, g_in.bsize_h, g_in.bsize_w, C), 9.0, dtype=TORCH_DT[dtype]).cuda()
        sb.sparse_gather(to_dev(x, dtype), d_idx, d_cnt, g_in, tiles)
        got = to_host(tiles)
        assert np.array_equal(got[:len(idx)], orc.gather(x, idx, ogeom(g_in)))
        assert (got[len(idx):] == 9.0).all()          # rows beyond the count are not written


@pytest.mark.parametrize("H,W,C,k,s,bo,N,dtype", GS_CASES)
@pytest.mark.parametrize("add", [False, True])
def test_scatter_bit_exact(H, W, C, k, s, bo, N, dtype, add):
    step("scatter add=%s %s" % (add, (H, W, C, k, s, bo, N, dtype)))
    r = gen.rng_for(3, H * 1000 + W + C)
    g_in, g_out, Ho, Wo = sb.geometry(H, W, k, s, bo)
    y0 = gen.activations(r, (N, Ho, Wo, C), dtype)
    for dens in (0.0, 0.004, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.float32)
        idx = orc.reduce_mask(mask, ogeom(g_in))
        cap = len(idx) + 2
        d_idx, d_cnt = dev_indices(idx, cap)
        t = gen.activations(r, (cap, bo, bo, C), dtype)
        y = to_dev(y0, dtype)
        sb.sparse_scatter(to_dev(t, dtype), d_idx, d_cnt, g_out, y, add=add)
        want = round_like(orc.scatter(t[:len(idx)], idx, ogeom(g_out), y0, add=add), dtype)
        assert np.array_equal(to_host(y), want)


def test_gather_scatter_round_trip_all_blocks():
    step("gather/scatter round trip")
    r = gen.rng_for(3, 1)
    H, W, C, bo = 48, 32, 32, 8
    g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    x = to_dev(gen.activations(r, (2, H, W, C), "bf16"), "bf16")
    idx, cnt = sb.reduce_mask(torch.ones((2, H, W), dtype=torch.uint8).cuda(), g_in)
    tiles = sb.sparse_gather(x, idx, cnt, g_in)
    y = torch.zeros_like(x)
    sb.sparse_scatter(tiles[:, 1:-1, 1:-1].contiguous(), idx, cnt, g_out, y)
    assert torch.equal(x, y)


CHW_CASES = [
    # H, W, C, k, s, bo, N, dtype: C * element size must fill 16-byte vectors
    (48, 80, 64, 3, 1, 16, 2, "bf16"),     # one full slab of 64 channels
    (33, 47, 256, 3, 1, 16, 1, "bf16"),    # four slabs, ragged blocks
    (37, 29, 40, 3, 1, 4, 2, "f16"),       # a partial slab (5 vectors per pixel), tiny tiles
    (64, 64, 16, 3, 1, 8, 1, "f32"),       # four-byte elements: slabs of 32 channels, partial
    (40, 40, 72, 5, 1, 8, 1, "f32"),       # ... three slabs, halo 2
    (35, 35, 8, 3, 2, 4, 2, "f16"),        # strided geometry, a single vector per pixel
    (70, 70, 96, 3, 1, 32, 1, "bf16"),     # 34 x 34 tiles: the largest slab that fits in LDS
]


@pytest.mark.parametrize("H,W,C,k,s,bo,N,dtype", CHW_CASES)
def test_transposing_gather_and_scatter_bit_exact(H, W, C, k, s, bo, N, dtype):
    """Channel-major tile stack (Sec. 3.4, transpose fused into gather and scatter)."""
    step("gather/scatter chw %s" % ((H, W, C, k, s, bo, N, dtype),))
    r = gen.rng_for(2, H * 1000 + W + C + 7)
    g_in, g_out, Ho, Wo = sb.geometry(H, W, k, s, bo)
    x = gen.activations(r, (N, H, W, C), dtype)
    y0 = gen.activations(r, (N, Ho, Wo, C), dtype)
    for dens in (0.0, 0.004, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.float32)
        idx = orc.reduce_mask(mask, ogeom(g_in))
        cap = len(idx) + 2
        d_idx, d_cnt = dev_indices(idx, cap)
        tiles = torch.full((cap, C, g_in.bsize_h, g_in.bsize_w), 9.0, dtype=TORCH_DT[dtype]).cuda()
        sb.sparse_gather_chw(to_dev(x, dtype), d_idx, d_cnt, g_in, tiles)
        got = to_host(tiles)
        assert np.array_equal(got[:len(idx)], orc.gather_chw(x, idx, ogeom(g_in)))
        assert (got[len(idx):] == 9.0).all()          # rows beyond the count are not written
        t = gen.activations(r, (cap, C, bo, bo), dtype)
        for add in (False, True):
            y = to_dev(y0, dtype)
            sb.sparse_scatter_chw(to_dev(t, dtype), d_idx, d_cnt, g_out, y, add=add)
            want = round_like(orc.scatter_chw(t[:len(idx)], idx, ogeom(g_out), y0, add=add), dtype)
            assert np.array_equal(to_host(y), want)


def test_transposing_copies_refuse_what_they_do_not_take():
    g_in, g_out, _, _ = sb.geometry(160, 160, 3, 1, 40)           # 42 x 42 tiles: a slab would not fit in LDS
    x = torch.zeros((1, 160, 160, 64), dtype=torch.bfloat16).cuda()
    idx, cnt = sb.reduce_mask(torch.ones((1, 160, 160), dtype=torch.uint8).cuda(), g_in)
    with pytest.raises(sb.SbnetError) as e:
        sb.sparse_gather_chw(x, idx, cnt, g_in)
    assert e.value.code == sb.EUNSUPPORTED
    g_in, _, _, _ = sb.geometry(16, 16, 3, 1, 8)
    x = torch.zeros((1, 16, 16, 12), dtype=torch.bfloat16).cuda()  # 24 bytes per pixel
    idx, cnt = sb.reduce_mask(torch.ones((1, 16, 16), dtype=torch.uint8).cuda(), g_in)
    with pytest.raises(sb.SbnetError) as e:
        sb.sparse_gather_chw(x, idx, cnt, g_in)
    assert e.value.code == sb.EUNSUPPORTED


GB_CASES = [
    # H, W, C, k, s, bo, N, dtype
    (48, 80, 64, 3, 1, 16, 2, "bf16"),     # one-pixel halo: up to four tiles per pixel
    (37, 29, 6, 3, 1, 4, 2, "f16"),        # 4-byte vectors... 12 bytes per pixel, ragged blocks
    (64, 64, 16, 3, 1, 8, 1, "f32"),
    (40, 40, 12, 5, 1, 3, 1, "f32"),       # halo 2 on 3-pixel blocks: tiles reach over two following cells
    (30, 26, 8, 7, 1, 2, 1, "bf16"),       # halo 3 on 2-pixel blocks: three following cells, 16 tiles per pixel
    (35, 35, 8, 3, 2, 4, 2, "f16"),        # strided geometry: tile 9, stride 8
    (24, 24, 32, 1, 1, 3, 1, "bf16"),      # 1x1: no overlap at all
]


@pytest.mark.parametrize("H,W,C,k,s,bo,N,dtype", GB_CASES)
def test_gather_backward(H, W, C, k, s, bo, N, dtype):
    """Gradient of the gather (end of Sec. 3.3): overlapping tile gradients summed per pixel, deterministic order."""
    step("gather_backward %s" % ((H, W, C, k, s, bo, N, dtype),))
    r = gen.rng_for(8, H * 1000 + W + C)
    g_in, _, _, _ = sb.geometry(H, W, k, s, bo)
    dx0 = gen.activations(r, (N, H, W, C), dtype)
    for dens in (0.0, 0.01, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.float32)
        idx = orc.reduce_mask(mask, ogeom(g_in))
        cap = len(idx) + 2
        d_idx, d_cnt = dev_indices(idx, cap)
        t = gen.activations(r, (cap, g_in.bsize_h, g_in.bsize_w, C), dtype)
        dx = to_dev(dx0, dtype)
        sb.sparse_gather_backward(to_dev(t, dtype), d_idx, d_cnt, g_in, dx)
        got = to_host(dx)
        ref = orc.gather_backward(t[:len(idx)], idx, ogeom(g_in), dx0)
        if dtype == "f32":
            assert np.allclose(got, ref, rtol=2e-6, atol=2e-6)
        else:
            want = round_like(ref, dtype)
            # the fp32 sum of up to 17 terms is not always exact: allow the neighbouring representable value, rarely
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(want), 1e-30))) - (7 if dtype == "bf16" else 10))
            assert (np.abs(got - want) <= ulp).all()
            assert (got != want).mean() < 2e-3
        untouched = ref == dx0
        assert np.array_equal(got[untouched], dx0[untouched])
        # two runs give the same bits: no atomics
        dx2 = to_dev(dx0, dtype)
        sb.sparse_gather_backward(to_dev(t, dtype), d_idx, d_cnt, g_in, dx2)
        assert torch.equal(dx, dx2)


@pytest.mark.parametrize("H,W,C,bo,N,dtype", [(48, 80, 64, 16, 2, "bf16"), (37, 29, 40, 4, 2, "f16"), (64, 64, 16, 8, 1, "f32"),
                                              (33, 47, 256, 16, 1, "bf16"), (70, 70, 96, 32, 1, "f32")])
def test_sparse_bn_stats(H, W, C, bo, N, dtype):
    """Batch-norm statistics over the active blocks only (Sec. 3.3); channels with a mean far from zero included."""
    step("bn_stats %s" % ((H, W, C, bo, N, dtype),))
    r = gen.rng_for(9, H * 1000 + W + C)
    _, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    shift = np.where(np.arange(C) % 3 == 0, 20.0, 0.0)
    x = gen.round_to((gen.activations(r, (N, H, W, C), "f32") + shift).astype(np.float32), dtype)
    for dens in (0.0, 0.004, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.float32)
        idx = orc.reduce_mask(mask, ogeom(g_out))
        cap = len(idx) + 2
        d_idx, d_cnt = dev_indices(idx, cap)
        mean, var = sb.sparse_bn_stats(to_dev(x, dtype), d_idx, d_cnt, g_out)
        rm, rv = orc.bn_stats(x, idx, ogeom(g_out))
        assert np.allclose(mean.cpu().numpy(), rm, rtol=1e-5, atol=1e-5), np.abs(mean.cpu().numpy() - rm).max()
        assert np.allclose(var.cpu().numpy(), rv, rtol=2e-4, atol=1e-6), np.abs(var.cpu().numpy() - rv).max()
        mean2, var2 = sb.sparse_bn_stats(to_dev(x, dtype), d_idx, d_cnt, g_out)
        assert torch.equal(mean, mean2) and torch.equal(var, var2)        # fixed summation order


@pytest.mark.parametrize("H,W,C,bo,N,dtype", [(48, 80, 64, 16, 2, "bf16"), (37, 29, 40, 4, 2, "f16"), (64, 64, 16, 8, 1, "f32"),
                                              (33, 47, 256, 16, 1, "bf16")])
@pytest.mark.parametrize("relu", [False, True])
def test_sparse_bn_apply_and_backward(H, W, C, bo, N, dtype, relu):
    """Normalisation over the active blocks (Sec. 3.3), forward and training-mode backward, with the statistics the
    library itself computed; pixels outside the active blocks keep their bits."""
    step("bn apply/backward %s" % ((H, W, C, bo, N, dtype, relu),))
    r = gen.rng_for(10, H * 1000 + W + C + int(relu))
    _, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
    eps = 1e-3
    x = gen.round_to((gen.activations(r, (N, H, W, C), "f32") * 1.5 + 0.25).astype(np.float32), dtype)
    dy = gen.activations(r, (N, H, W, C), dtype)
    gamma = (r.standard_normal(C) * 0.3 + 1.0).astype(np.float32)
    beta = (r.standard_normal(C) * 0.3).astype(np.float32)
    y0 = gen.activations(r, (N, H, W, C), dtype)
    tol = {"f32": 2e-5, "bf16": 8e-3, "f16": 1e-3}[dtype]       # one rounding of the result to the storage type
    for dens in (0.0, 0.004, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.float32)
        idx = orc.reduce_mask(mask, ogeom(g_out))
        d_idx, d_cnt = dev_indices(idx, len(idx) + 2)
        xd, dyd = to_dev(x, dtype), to_dev(dy, dtype)
        mean, var = sb.sparse_bn_stats(xd, d_idx, d_cnt, g_out)
        gd, bd = torch.from_numpy(gamma).cuda(), torch.from_numpy(beta).cuda()
        y = sb.sparse_bn_apply(xd, d_idx, d_cnt, g_out, mean, var, gd, bd, eps=eps, relu=relu, y=to_dev(y0, dtype))
        om, ov = orc.bn_stats(x, idx, ogeom(g_out))
        ref = orc.bn_apply(x, idx, ogeom(g_out), om, ov, gamma, beta, eps, y0, relu=relu)
        inside = orc.block_mask(idx, ogeom(g_out), N, H, W)
        got = to_host(y)
        assert np.array_equal(got[~inside], y0[~inside])
        if inside.any():
            assert_close(got[inside], ref[inside], tol, "bn_apply")
        # in place gives the same bits
        x2 = to_dev(x, dtype)
        sb.sparse_bn_apply(x2, d_idx, d_cnt, g_out, mean, var, gd, bd, eps=eps, relu=relu)
        assert torch.equal(x2[torch.from_numpy(inside).cuda()], y[torch.from_numpy(inside).cuda()])
        # backward
        d0 = gen.activations(r, (N, H, W, C), dtype)
        dx, dgam, dbet = sb.sparse_bn_backward(xd, dyd, d_idx, d_cnt, g_out, mean, var, gd, bd, eps=eps, relu=relu,
                                               dx=to_dev(d0, dtype))
        rdx, rdg, rdb = orc.bn_backward(x, dy, idx, ogeom(g_out), gamma, beta, eps, d0, relu=relu)
        gotdx = to_host(dx)
        assert np.array_equal(gotdx[~inside], d0[~inside])
        npx = int(inside.sum())
        if npx:
            # sums of npx terms of unit scale in fp32, partial sums per block then a tree
            stol = 3e-5 * np.sqrt(npx) + 1e-4
            assert np.abs(dgam.cpu().numpy() - rdg).max() <= stol * max(1.0, np.abs(rdg).max() / np.sqrt(npx)), np.abs(dgam.cpu().numpy() - rdg).max()
            assert np.abs(dbet.cpu().numpy() - rdb).max() <= stol * max(1.0, np.abs(rdb).max() / np.sqrt(npx))
            assert_close(gotdx[inside], rdx[inside], tol * 2, "bn_backward dx")
        else:
            assert (dgam == 0).all() and (dbet == 0).all()
        dx2, dgam2, dbet2 = sb.sparse_bn_backward(xd, dyd, d_idx, d_cnt, g_out, mean, var, gd, bd, eps=eps, relu=relu,
                                                  dx=to_dev(d0, dtype))
        assert torch.equal(dx, dx2) and torch.equal(dgam, dgam2) and torch.equal(dbet, dbet2)


# --------------------------------------------------------------------------- convolution on tiles
CONV_CASES = [
    # B, th, tw, Cin, Cout, k, s, dtype, relu, bias
    (7, 10, 10, 16, 16, 3, 1, "f32", False, False),     # the small fp32 configuration
    (5, 18, 18, 64, 64, 3, 1, "bf16", False, True),     # headline tile shape
    (3, 18, 18, 64, 64, 3, 1, "f16", True, True),
    (3, 18, 18, 256, 64, 1, 1, "bf16", True, True),     # bottleneck conv1 shape: channel chunks in LDS
    (3, 16, 16, 64, 256, 1, 1, "bf16", False, True),    # bottleneck conv3 shape: four channel groups
    (2, 34, 34, 32, 64, 3, 1, "bf16", True, False),     # several 256-pixel passes per tile
    (4, 10, 10, 24, 40, 3, 1, "bf16", False, True),     # channel counts padded inside the MFMA path
    (4, 11, 9, 8, 8, 3, 2, "f16", True, True),          # strided, ragged pixel blocks
    (3, 7, 7, 5, 3, 3, 1, "bf16", False, True),         # odd channels: direct kernel in bf16
    (3, 9, 9, 4, 6, 5, 2, "f32", True, True),
    (2, 6, 12, 96, 96, 1, 1, "bf16", False, False),
    (3, 18, 18, 32, 128, 3, 1, "bf16", True, True),     # register-stationary 3x3 kernel: two channel groups
    (2, 34, 18, 64, 24, 3, 1, "f16", False, True),      # ... two sub-tiles per tile, partial channel group
    (2, 18, 50, 32, 64, 3, 1, "bf16", True, False),     # ... three sub-tiles side by side
    # LDS-tiled 3x3 kernel
    (3, 26, 26, 40, 96, 3, 1, "bf16", True, True),      # three passes, last one short; padded channel chunk; Cout % 64 == 32
    (2, 33, 33, 96, 64, 3, 2, "bf16", True, True),      # stride-2 tile of a 16x16 block: chunks of 16 channels
    (4, 17, 17, 64, 32, 3, 2, "f16", False, True),      # stride-2 tile of an 8x8 block: 64-pixel workgroup tile
    (2, 21, 19, 16, 8, 3, 1, "bf16", False, False),     # odd tile sides, one chunk per item
    (3, 12, 12, 8, 72, 3, 3, "f16", True, True),        # stride 3: three column phases; last group of 8 channels
    (2, 10, 70, 24, 16, 3, 1, "bf16", True, True),      # wide, flat tile: a pass covers part of a row
]


@pytest.mark.parametrize("B,th,tw,Cin,Cout,k,s,dtype,relu,bias", CONV_CASES)
def test_conv_on_tiles(B, th, tw, Cin, Cout, k, s, dtype, relu, bias):
    step("conv_on_tiles %s" % ((B, th, tw, Cin, Cout, k, s, dtype, relu, bias),))
    r = gen.rng_for(4, th * 100 + Cin + Cout)
    t = gen.activations(r, (B + 1, th, tw, Cin), dtype)
    w = gen.conv_weights(r, k, k, Cin, Cout, dtype, unit_variance=(dtype == "f32"))
    b = gen.bias_vector(r, Cout, 0.5) if bias else None
    wp = sb.pack_weights(to_dev(w, dtype))
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    oh, ow = (th - k) // s + 1, (tw - k) // s + 1
    out = torch.full((B + 1, oh, ow, Cout), 5.0, dtype=TORCH_DT[dtype]).cuda()
    sb.conv_on_tiles(to_dev(t, dtype), cnt, wp, None if b is None else torch.from_numpy(b).cuda(), stride=s, relu=relu,
                     out=out)
    ref = orc.conv_valid(t[:B], w, b, stride=s, relu=relu)
    got = to_host(out)
    assert_close(got[:B], ref, CONV_TOL[dtype], "conv_on_tiles")
    assert (got[B] == 5.0).all()


def _random_3x3_shapes(n, seed):
    """Seeded draws over what the 3x3 matrix-core kernels take: tile sides 3..40, strides 1..3, channels in multiples of 8."""
    r = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        s = int(r.integers(1, 4))
        th, tw = int(r.integers(3, 41)), int(r.integers(3, 41))
        cin, cout = 8 * int(r.integers(1, 13)), 8 * int(r.integers(1, 13))
        out.append((int(r.integers(1, 5)), th, tw, cin, cout, s, ("bf16", "f16")[int(r.integers(0, 2))],
                    bool(r.integers(0, 2)), bool(r.integers(0, 2))))
    return out


@pytest.mark.parametrize("B,th,tw,Cin,Cout,s,dtype,relu,bias", _random_3x3_shapes(40, 180102108))
def test_conv_on_tiles_random_3x3_shapes(B, th, tw, Cin, Cout, s, dtype, relu, bias):
    """Passes per tile, rows per pass, column phases, channel chunks and groups all vary with the shape."""
    step("conv_on_tiles random %s" % ((B, th, tw, Cin, Cout, s, dtype, relu, bias),))
    r = gen.rng_for(4, th * 1000 + tw * 10 + Cin + Cout + s)
    t = gen.activations(r, (B + 1, th, tw, Cin), dtype)
    w = gen.conv_weights(r, 3, 3, Cin, Cout, dtype)
    b = gen.bias_vector(r, Cout, 0.5) if bias else None
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    oh, ow = (th - 3) // s + 1, (tw - 3) // s + 1
    out = torch.full((B + 1, oh, ow, Cout), 5.0, dtype=TORCH_DT[dtype]).cuda()
    sb.conv_on_tiles(to_dev(t, dtype), cnt, sb.pack_weights(to_dev(w, dtype)), None if b is None else torch.from_numpy(b).cuda(),
                     stride=s, relu=relu, out=out)
    got = to_host(out)
    assert_close(got[:B], orc.conv_valid(t[:B], w, b, stride=s, relu=relu), CONV_TOL[dtype], "conv_on_tiles")
    assert (got[B] == 5.0).all()


def _random_pointwise_shapes(n, seed):
    """Seeded draws over what the pipelined pointwise path takes: input channels in multiples of 64, any tile and stride 1..2."""
    r = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        out.append((int(r.integers(1, 5)), int(r.integers(1, 36)), int(r.integers(1, 36)), 64 * int(r.integers(1, 6)),
                    8 * int(r.integers(1, 41)), int(r.integers(1, 3)), ("bf16", "f16")[int(r.integers(0, 2))],
                    bool(r.integers(0, 2)), bool(r.integers(0, 2))))
    return out


POINTWISE_PADDED_CASES = [
    # input channels that do not fill the last 64-channel chunk (40, 48, 104, 120 -> padded to 64 / 128)
    (3, 18, 18, 48, 192, 1, "bf16", True, True),
    (2, 11, 13, 40, 24, 1, "f16", False, True),
    (4, 9, 9, 104, 64, 1, "bf16", True, False),
    (2, 17, 17, 120, 40, 2, "bf16", False, True),
    # channel counts that are multiples of 32 only: chunks of 32 channels
    (3, 18, 18, 96, 24, 1, "bf16", True, True),
    (2, 16, 16, 24, 96, 1, "bf16", False, True),
    (2, 18, 18, 96, 96, 1, "f16", True, False),
    (2, 13, 11, 160, 48, 2, "bf16", False, True),
    (1, 34, 34, 32, 64, 1, "bf16", True, True),         # 1156 pixels: five passes of 256
    (5, 5, 7, 224, 8, 1, "f16", False, False),          # seven chunks, 35 pixels
]


@pytest.mark.parametrize("B,th,tw,Cin,Cout,s,dtype,relu,bias", POINTWISE_PADDED_CASES + _random_pointwise_shapes(24, 1801021081))
def test_conv_on_tiles_random_pointwise_shapes(B, th, tw, Cin, Cout, s, dtype, relu, bias):
    """1x1 convolutions on tiles from one pixel to several passes, one to five 64-channel chunks, up to five channel groups."""
    step("conv_on_tiles pointwise %s" % ((B, th, tw, Cin, Cout, s, dtype, relu, bias),))
    r = gen.rng_for(4, th * 1000 + tw * 10 + Cin + Cout + s)
    t = gen.activations(r, (B + 1, th, tw, Cin), dtype)
    w = gen.conv_weights(r, 1, 1, Cin, Cout, dtype)
    b = gen.bias_vector(r, Cout, 0.5) if bias else None
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    oh, ow = (th - 1) // s + 1, (tw - 1) // s + 1
    out = torch.full((B + 1, oh, ow, Cout), 5.0, dtype=TORCH_DT[dtype]).cuda()
    sb.conv_on_tiles(to_dev(t, dtype), cnt, sb.pack_weights(to_dev(w, dtype)), None if b is None else torch.from_numpy(b).cuda(),
                     stride=s, relu=relu, out=out)
    got = to_host(out)
    assert_close(got[:B], orc.conv_valid(t[:B], w, b, stride=s, relu=relu), CONV_TOL[dtype], "conv_on_tiles")
    assert (got[B] == 5.0).all()


# --------------------------------------------------------------------------- fused sparse conv
SPARSE_CASES = [
    # N, H, W, Cin, Cout, k, s, bo, dtype
    (1, 64, 64, 16, 16, 3, 1, 8, "f32"),
    (2, 48, 80, 64, 64, 3, 1, 16, "bf16"),
    (1, 37, 29, 32, 16, 3, 1, 4, "bf16"),      # ragged: blocks hang over the image edge
    (1, 40, 40, 64, 64, 3, 1, 32, "f16"),
    (2, 35, 35, 8, 8, 3, 2, 4, "bf16"),        # strided convolution
    (1, 24, 24, 6, 5, 3, 1, 8, "f32"),
    (1, 32, 32, 64, 256, 1, 1, 16, "bf16"),
    (2, 45, 39, 128, 72, 1, 1, 8, "f16"),      # pointwise, fused, blocks hang over the edge, two chunks
    (1, 50, 50, 64, 64, 1, 2, 8, "bf16"),      # pointwise stride 2: the shortcut of a downsampling unit
    (1, 40, 36, 96, 24, 1, 1, 8, "bf16"),      # pointwise with 32-channel chunks, fused, ragged blocks
    # LDS-tiled 3x3 kernel
    (2, 70, 66, 96, 96, 3, 2, 16, "bf16"),     # downsampling unit, blocks hang over the edge, Cout % 64 == 32
    (1, 96, 80, 192, 32, 3, 1, 16, "f16"),     # six channel chunks
    (3, 40, 40, 32, 64, 3, 1, 8, "bf16"),      # 8x8 blocks, one chunk per item: the chunk pipeline runs over items
    (1, 33, 49, 48, 40, 3, 2, 8, "bf16"),      # stride 2 with 8x8 blocks, ragged
]


@pytest.mark.parametrize("N,H,W,Cin,Cout,k,s,bo,dtype", SPARSE_CASES)
@pytest.mark.parametrize("add", [False, True])
def test_sparse_conv_fused_and_unfused(N, H, W, Cin, Cout, k, s, bo, dtype, add):
    step("sparse_conv add=%s %s" % (add, (N, H, W, Cin, Cout, k, s, bo, dtype)))
    r = gen.rng_for(5, H * 100 + Cin + bo)
    g_in, g_out, Ho, Wo = sb.geometry(H, W, k, s, bo)
    x = gen.activations(r, (N, H, W, Cin), dtype)
    w = gen.conv_weights(r, k, k, Cin, Cout, dtype, unit_variance=(dtype == "f32"))
    b = gen.bias_vector(r, Cout, 0.5)
    y0 = gen.activations(r, (N, Ho, Wo, Cout), dtype)
    wp = sb.pack_weights(to_dev(w, dtype))
    d_b = torch.from_numpy(b).cuda()
    for dens in (0.0, 0.003, 1.0):
        mask = (r.random((N, H, W)) < dens).astype(np.uint8)
        d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in)
        idx = orc.reduce_mask(mask, ogeom(g_in))
        ref = orc.sparse_conv_dense(x, idx, ogeom(g_out), w, b, y0, stride=s, relu=True, add=add)
        bm = orc.block_mask(idx, ogeom(g_out), N, Ho, Wo)
        # fused kernel
        y = to_dev(y0, dtype)
        sb.sparse_conv(to_dev(x, dtype), d_idx, d_cnt, g_in, g_out, wp, d_b, y, stride=s, relu=True, add=add)
        got = to_host(y)
        assert_close(got, ref, CONV_TOL[dtype], "fused")
        assert np.array_equal(got[~bm], y0[~bm])                  # inactive pixels bit-identical
        # four separate calls
        y = to_dev(y0, dtype)
        tiles = sb.sparse_gather(to_dev(x, dtype), d_idx, d_cnt, g_in)
        out = sb.conv_on_tiles(tiles, d_cnt, wp, d_b, stride=s, relu=True)
        sb.sparse_scatter(out, d_idx, d_cnt, g_out, y, add=add)
        got = to_host(y)
        assert_close(got, ref, CONV_TOL[dtype], "unfused")
        assert np.array_equal(got[~bm], y0[~bm])
        # mask in, result out in one call: the same bits as reduce_mask + the fused kernel, and the same list left behind
        y_fused = to_dev(y0, dtype)
        sb.sparse_conv(to_dev(x, dtype), d_idx, d_cnt, g_in, g_out, wp, d_b, y_fused, stride=s, relu=True, add=add)
        y = to_dev(y0, dtype)
        m_idx = torch.full_like(d_idx, -3)
        m_cnt = torch.full_like(d_cnt, -3)
        ws = torch.full((sb.workspace_bytes(N, g_in),), 0x5b, dtype=torch.uint8).cuda()
        sb.sparse_conv_from_mask(torch.from_numpy(mask).cuda(), g_in, to_dev(x, dtype), g_in, g_out, wp, d_b, y, m_idx, m_cnt, ws,
                                 stride=s, relu=True, add=add)
        assert torch.equal(y, y_fused)
        n = sb.read_count(m_cnt, m_idx.shape[0])
        assert n == len(idx) and np.array_equal(m_idx[:n].cpu().numpy(), idx) and bool((m_idx[n:] == -3).all())


FROM_MASK_CASES = [
    # N, H, W, Cin, Cout, bo, dtype, add, density, cap (None = all blocks): shapes the flag-fed kernel takes, and around them
    (1, 800, 704, 64, 64, 16, "bf16", False, 0.0008, None),   # the headline layer: 2200 flags, one round of the scan
    (4, 400, 352, 64, 64, 16, "bf16", True, 0.002, None),     # 2200 blocks over four samples
    (5, 800, 704, 32, 64, 16, "f16", False, 0.0005, None),    # 11 000 flags: three rounds of 4096, 32 input channels
    (1, 250, 170, 64, 128, 16, "bf16", False, 0.004, None),   # ragged edges, two groups of output channels
    (1, 800, 704, 64, 64, 16, "bf16", False, 1.0, None),      # every block active: 8-9 items per workgroup
    (2, 160, 160, 64, 64, 16, "bf16", True, 0.01, 7),         # fewer list rows than active blocks
    (1, 64, 48, 64, 64, 16, "bf16", False, 0.0, None),        # empty mask
    (1, 4112, 4112, 64, 8, 16, "bf16", False, 0.00002, None), # 66 049 blocks: beyond the flag path, the two calls in sequence
]


@pytest.mark.parametrize("N,H,W,Cin,Cout,bo,dtype,add,dens,cap", FROM_MASK_CASES)
def test_sparse_conv_from_mask(N, H, W, Cin, Cout, bo, dtype, add, dens, cap):
    """sbnet_sparse_conv_from_mask against the oracle: index list and count bit-exact, the convolved blocks within the
    convolution's tolerance on sampled tiles (whole tensor for the small cases), inactive pixels untouched."""
    step("sparse_conv_from_mask %s" % ((N, H, W, Cin, Cout, bo, dtype, add, dens, cap),))
    r = gen.rng_for(5, 7000 + H + W + Cin + N)
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, 1, bo)
    og_in, og_out = ogeom(g_in), ogeom(g_out)
    total = N * g_in.bcount_h * g_in.bcount_w
    mask = (r.random((N, H, W)) < dens).astype(np.uint8)
    tdt = {"bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    tg = torch.Generator(device="cuda")
    tg.manual_seed(gen.BASE_SEED + 7000 + H)
    xd = torch.randn((N, H, W, Cin), generator=tg, device="cuda", dtype=torch.float32).to(tdt)
    yd = torch.randn((N, Ho, Wo, Cout), generator=tg, device="cuda", dtype=torch.float32).to(tdt)
    y_before = yd.clone()
    w = gen.conv_weights(r, 3, 3, Cin, Cout, dtype)
    b = gen.bias_vector(r, Cout, 0.5)
    rows = total if cap is None else cap
    d_idx = torch.full((rows, 3), -3, dtype=torch.int32).cuda()
    d_cnt = torch.full((1,), -3, dtype=torch.int32).cuda()
    ws = torch.full((sb.workspace_bytes(N, g_in),), 0xa7, dtype=torch.uint8).cuda()
    sb.sparse_conv_from_mask(torch.from_numpy(mask).cuda(), g_in, xd, g_in, g_out, sb.pack_weights(to_dev(w, dtype)),
                             torch.from_numpy(b).cuda(), yd, d_idx, d_cnt, ws, relu=True, add=add)
    idx = orc.reduce_mask(mask, og_in)
    assert int(d_cnt.item()) == len(idx)
    if total <= 65536:
        # the two halves as calls of their own: flags = membership in the oracle's list; the same y, list and count
        flags = sb.block_flags(torch.from_numpy(mask).cuda(), g_in)
        want = np.zeros(total, np.uint8)
        want[(idx[:, 0] * g_in.bcount_h + idx[:, 1]) * g_in.bcount_w + idx[:, 2]] = 1
        assert np.array_equal(flags[:total].cpu().numpy(), want)
        y2, i2, c2 = y_before.clone(), torch.full_like(d_idx, -3), torch.full_like(d_cnt, -3)
        sb.sparse_conv_from_flags(flags, xd, g_in, g_out, sb.pack_weights(to_dev(w, dtype)), torch.from_numpy(b).cuda(), y2, i2, c2,
                                  relu=True, add=add)
        assert torch.equal(y2, yd) and torch.equal(i2, d_idx) and torch.equal(c2, d_cnt)
    used = min(len(idx), rows)
    got_idx = d_idx.cpu().numpy()
    assert np.array_equal(got_idx[:used], idx[:used]) and (got_idx[used:] == -3).all()
    idx = idx[:used]
    bm = torch.from_numpy(orc.block_mask(idx, og_out, N, Ho, Wo)).cuda()
    assert torch.equal(yd[~bm], y_before[~bm])
    if used == 0:
        return
    pick = np.unique(np.concatenate([[0, used - 1], r.integers(0, used, 10)]))
    for k in pick:
        n_, by, bx = (int(v) for v in idx[k])
        one = np.array([[0, by, bx]], dtype=np.int32)
        if H * W <= 800 * 704:
            tile = orc.gather(xd[n_].to(torch.float64).cpu().numpy()[None], one, og_in)
        else:
            # very large image: the oracle gets the 3 x 3 block window around the block as an image of its own (the
            # window ends a whole block beyond the tile, or at the image's edge, where its zero padding is the image's)
            y_lo, x_lo = max(by * bo - bo, 0), max(bx * bo - bo, 0)
            xs = xd[n_, y_lo:min(by * bo + 2 * bo, H), x_lo:min(bx * bo + 2 * bo, W)].to(torch.float64).cpu().numpy()[None]
            wg_in, _, _, _ = orc.geometry(xs.shape[1], xs.shape[2], 3, 1, bo)
            tile = orc.gather(xs, np.array([[0, (by * bo - y_lo) // bo, (bx * bo - x_lo) // bo]], dtype=np.int32), wg_in)
        hh, ww = min(bo, Ho - by * bo), min(bo, Wo - bx * bo)
        ref = np.maximum(orc.conv_valid(tile, w, b), 0.0)[0, :hh, :ww]
        if add:
            ref = ref + y_before[n_, by * bo:by * bo + hh, bx * bo:bx * bo + ww].to(torch.float64).cpu().numpy()
        blk = yd[n_, by * bo:by * bo + hh, bx * bo:bx * bo + ww].to(torch.float64).cpu().numpy()
        assert_close(blk, ref, CONV_TOL[dtype], "from mask, tile %d" % k)


def _random_fused_shapes(n, seed):
    r = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        out.append((int(r.integers(1, 3)), int(r.integers(20, 71)), int(r.integers(20, 71)), 8 * int(r.integers(1, 9)),
                    8 * int(r.integers(1, 9)), int(r.integers(1, 3)), (3, 4, 5, 8, 10, 16)[int(r.integers(0, 6))],
                    ("bf16", "f16")[int(r.integers(0, 2))], bool(r.integers(0, 2))))
    return out


@pytest.mark.parametrize("N,H,W,Cin,Cout,s,bo,dtype,add", _random_fused_shapes(16, 20180102))
def test_sparse_conv_random_shapes(N, H, W, Cin, Cout, s, bo, dtype, add):
    """Fused 3x3 on seeded random image sizes, block sizes and strides: blocks hang over every edge in some case."""
    step("sparse_conv random %s" % ((N, H, W, Cin, Cout, s, bo, dtype, add),))
    r = gen.rng_for(5, H * 1000 + W * 10 + Cin + bo + s)
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, s, bo)
    x = gen.activations(r, (N, H, W, Cin), dtype)
    w = gen.conv_weights(r, 3, 3, Cin, Cout, dtype)
    b = gen.bias_vector(r, Cout, 0.5)
    y0 = gen.activations(r, (N, Ho, Wo, Cout), dtype)
    mask = (r.random((N, H, W)) < 0.004).astype(np.uint8)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in)
    idx = orc.reduce_mask(mask, ogeom(g_in))
    assert np.array_equal(d_idx[:len(idx)].cpu().numpy(), idx)
    y = to_dev(y0, dtype)
    sb.sparse_conv(to_dev(x, dtype), d_idx, d_cnt, g_in, g_out, sb.pack_weights(to_dev(w, dtype)), torch.from_numpy(b).cuda(),
                   y, stride=s, relu=True, add=add)
    got = to_host(y)
    assert_close(got, orc.sparse_conv_dense(x, idx, ogeom(g_out), w, b, y0, stride=s, relu=True, add=add), CONV_TOL[dtype], "fused")
    bm = orc.block_mask(idx, ogeom(g_out), N, Ho, Wo)
    assert np.array_equal(got[~bm], y0[~bm])


@pytest.mark.parametrize("H,W,bh,bw,Cin,Cout,dtype", [
    # sizes at which the 128-pixel items of all blocks outnumber the workgroups: below that the host plans no second shape
    (110, 130, 18, 18, 96, 64, "bf16"),    # the 18x18 outputs of a data gradient on 16x16 blocks; blocks hang over the edge
    (80, 120, 13, 28, 40, 72, "f16"),      # 364 pixels whose input rows only fit in 16-channel chunks
    (120, 120, 19, 19, 32, 32, "bf16"),    # 361 pixels, one chunk
])
@pytest.mark.parametrize("choice", ["larger", "smaller", "by count"])
def test_sparse_conv_blocks_of_257_to_384_pixels(H, W, bh, bw, Cin, Cout, dtype, choice):
    """Blocks of 257 ... 384 output pixels have a tile shape of their own (one 384-pixel item per block) beside the
    128-pixel one; the count picks on the device.  Both forced, and the default rule, against the oracle."""
    step("sparse_conv 384-pixel shape %s %s" % (choice, (H, W, bh, bw, Cin, Cout, dtype)))
    r = gen.rng_for(5, H * 100 + Cin + bh)
    g_in, g_out = sb.Geom(), sb.Geom()
    ho, wo = ctypes.c_int(), ctypes.c_int()
    assert sb.lib().sbnet_geometry(H, W, 3, 3, 1, 1, bh, bw, g_in, g_out, ho, wo) == 0
    N = 2
    x = gen.activations(r, (N, H, W, Cin), dtype)
    w = gen.conv_weights(r, 3, 3, Cin, Cout, dtype)
    b = gen.bias_vector(r, Cout, 0.5)
    y0 = gen.activations(r, (N, H, W, Cout), dtype)
    wp = sb.pack_weights(to_dev(w, dtype))
    d_b = torch.from_numpy(b).cuda()
    try:
        if choice != "by count":
            sb.set_tuning(conv3_small_item_cost_eighths=100000 if choice == "larger" else 0)
        for dens in (0.002, 1.0):
            mask = (r.random((N, H, W)) < dens).astype(np.uint8)
            d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in)
            idx = orc.reduce_mask(mask, ogeom(g_in))
            ref = orc.sparse_conv_dense(x, idx, ogeom(g_out), w, b, y0, stride=1, relu=True, add=False)
            bm = orc.block_mask(idx, ogeom(g_out), N, H, W)
            y = to_dev(y0, dtype)
            sb.sparse_conv(to_dev(x, dtype), d_idx, d_cnt, g_in, g_out, wp, d_b, y, stride=1, relu=True, add=False)
            got = to_host(y)
            assert_close(got, ref, CONV_TOL[dtype], "fused, %s shape" % choice)
            assert np.array_equal(got[~bm], y0[~bm])
    finally:
        sb.set_tuning()


@pytest.mark.parametrize("H,W,Cin,Cout,dtype", [
    (224, 224, 16, 96, "bf16"),      # groups of 96 output channels
    (224, 200, 24, 128, "f16"),      # groups of 128; blocks hang over the right edge
    (224, 224, 32, 256, "bf16"),     # two groups of 128, two chunks
    (200, 224, 16, 384, "bf16"),     # three groups of 128
])
@pytest.mark.parametrize("add", [False, True])
def test_sparse_conv_strided_wide_channel_groups(H, W, Cin, Cout, dtype, add):
    """Stride-2 3x3 convolutions on 16x16 blocks whose output channels are a multiple of 96 or 128: one launch holds
    128-pixel work items with groups of 96 / 128 channels and with groups of 64, and the count picks (wide from 96 work
    items).  All 49 blocks active runs the wide items, a handful of blocks the 64-channel ones."""
    step("sparse_conv strided, wide groups add=%s %s" % (add, (H, W, Cin, Cout, dtype)))
    r = gen.rng_for(5, H * 100 + Cin + Cout)
    N, s, bo = 1, 2, 16
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, s, bo)
    assert g_out.bcount_h * g_out.bcount_w * 2 >= 96
    x = gen.activations(r, (N, H, W, Cin), dtype)
    w = gen.conv_weights(r, 3, 3, Cin, Cout, dtype)
    b = gen.bias_vector(r, Cout, 0.5)
    y0 = gen.activations(r, (N, Ho, Wo, Cout), dtype)
    wp = sb.pack_weights(to_dev(w, dtype))
    d_b = torch.from_numpy(b).cuda()
    for dens in (1.0, 0.0002):
        mask = (r.random((N, H, W)) < dens).astype(np.uint8)
        d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in)
        idx = orc.reduce_mask(mask, ogeom(g_in))
        assert len(idx) > 0
        ref = orc.sparse_conv_dense(x, idx, ogeom(g_out), w, b, y0, stride=s, relu=True, add=add)
        bm = orc.block_mask(idx, ogeom(g_out), N, Ho, Wo)
        y = to_dev(y0, dtype)
        sb.sparse_conv(to_dev(x, dtype), d_idx, d_cnt, g_in, g_out, wp, d_b, y, stride=s, relu=True, add=add)
        got = to_host(y)
        assert_close(got, ref, CONV_TOL[dtype], "fused, %d blocks" % len(idx))
        assert np.array_equal(got[~bm], y0[~bm])
        # the unfused call on the gathered tiles takes the same kernels
        tiles = sb.sparse_gather(to_dev(x, dtype), d_idx, d_cnt, g_in)
        out = sb.conv_on_tiles(tiles, d_cnt, wp, d_b, stride=s, relu=True)
        y = to_dev(y0, dtype)
        sb.sparse_scatter(out, d_idx, d_cnt, g_out, y, add=add)
        assert_close(to_host(y), ref, CONV_TOL[dtype], "unfused, %d blocks" % len(idx))


@pytest.mark.parametrize("dens", [1.0, 0.35])
@pytest.mark.parametrize("Cin", [32, 40])
def test_sparse_conv_more_tiles_than_workgroups(dens, Cin):
    """Persistent kernels: 342 tiles on at most 256 workgroups, so the double-buffered tile loop and its prefetch
    run several iterations per workgroup.  Cin = 32: register-stationary kernel; Cin = 40: LDS-tiled kernel, which
    launches its 256-pixel and its 128-pixel variant and lets the device-side count pick (above / below 256 items)."""
    step("sparse_conv persistent loop dens=%s Cin=%d" % (dens, Cin))
    r = gen.rng_for(5, 999)
    N, H, W, Cout, bo = 1, 288, 304, 64, 16
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, 1, bo)
    x = gen.activations(r, (N, H, W, Cin), "bf16")
    w = gen.conv_weights(r, 3, 3, Cin, Cout, "bf16")
    b = gen.bias_vector(r, Cout, 0.5)
    y0 = gen.activations(r, (N, Ho, Wo, Cout), "bf16")
    blocks = (r.random((N, H // bo, W // bo)) < dens).astype(np.uint8)
    mask = np.repeat(np.repeat(blocks, bo, axis=1), bo, axis=2)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_out)      # window = output block
    idx = orc.reduce_mask(mask, ogeom(g_out))
    assert len(idx) > 100 and sb.read_count(d_cnt, d_idx.shape[0]) == len(idx)
    y = to_dev(y0, "bf16")
    sb.sparse_conv(to_dev(x, "bf16"), d_idx, d_cnt, g_in, g_out, sb.pack_weights(to_dev(w, "bf16")),
                   torch.from_numpy(b).cuda(), y, relu=False, add=True)
    ref = orc.sparse_conv_tiled(x, idx, ogeom(g_in), ogeom(g_out), w, b, y0, add=True)
    got = to_host(y)
    assert_close(got, ref, CONV_TOL["bf16"], "persistent")
    bm = orc.block_mask(idx, ogeom(g_out), N, Ho, Wo)
    assert np.array_equal(got[~bm], y0[~bm])


def test_config1_end_to_end():
    """Small fp32 configuration: 64x64x16 -> 16, three-rectangle mask (~10 % ones), 8x8 blocks,
    average pooling with threshold 0, plain scatter into a zeroed output."""
    step("config 1 end to end")
    r = gen.rng_for(1)
    H = W = 64
    C = 16
    g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, 1, 8)
    mask = gen.rect_mask(r, H, W, 3, 0.10)
    x = gen.activations(r, (1, H, W, C), "f32")
    w = gen.conv_weights(r, 3, 3, C, C, "f32", unit_variance=True)
    d_idx, d_cnt = sb.reduce_mask(torch.from_numpy(mask).cuda(), g_in, sb.POOL_AVG, 0.0)
    idx = orc.reduce_mask(mask, ogeom(g_in), orc.POOL_AVG, 0.0)
    n = sb.read_count(d_cnt, d_idx.shape[0])
    assert 0 < n < 64 and np.array_equal(d_idx[:n].cpu().numpy(), idx)
    y = torch.zeros((1, Ho, Wo, C), dtype=torch.float32).cuda()
    sb.sparse_conv(to_dev(x, "f32"), d_idx, d_cnt, g_in, g_out, sb.pack_weights(to_dev(w, "f32")), None, y)
    ref = orc.sparse_conv_tiled(x, idx, ogeom(g_in), ogeom(g_out), w, None, np.zeros((1, Ho, Wo, C)))
    assert_close(to_host(y), ref, CONV_TOL["f32"], "config 1")
    np.testing.assert_allclose(ref, orc.sparse_conv_dense(x, idx, ogeom(g_out), w, None, np.zeros((1, Ho, Wo, C))),
                               atol=1e-10)


# --------------------------------------------------------------------------- error paths (host-side checks)
def test_bad_arguments_are_reported_not_launched():
    step("error paths")
    g_in, g_out, _, _ = sb.geometry(16, 16, 3, 1, 4)
    x = torch.zeros((1, 16, 16, 8), dtype=torch.bfloat16).cuda()
    idx, cnt = dev_indices(np.zeros((0, 3), np.int32), 4)
    with pytest.raises(sb.SbnetError) as e:          # overlapping blocks cannot be scattered
        sb.sparse_scatter(torch.zeros((4, 6, 6, 8), dtype=torch.bfloat16).cuda(), idx, cnt, g_in, x)
    assert e.value.code == sb.EINVAL
    with pytest.raises(sb.SbnetError) as e:          # integer feature maps are not supported
        sb.sparse_gather(torch.zeros((1, 16, 16, 8), dtype=torch.uint8).cuda(), idx, cnt, g_in,
                         torch.zeros((4, 6, 6, 8), dtype=torch.uint8).cuda())
    assert e.value.code == sb.EUNSUPPORTED
    with pytest.raises(sb.SbnetError) as e:          # bf16 masks are not supported
        sb.reduce_mask(torch.zeros((1, 16, 16), dtype=torch.bfloat16).cuda(), g_in)
    assert e.value.code == sb.EUNSUPPORTED
    wp = sb.pack_weights(torch.zeros((3, 3, 8, 8), dtype=torch.bfloat16).cuda())
    with pytest.raises(sb.SbnetError) as e:          # in-place fused convolution would race
        sb.sparse_conv(x, idx, cnt, g_in, g_out, wp, None, x)
    assert e.value.code == sb.EINVAL
