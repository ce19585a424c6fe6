"""GPU parity of the FP8 (E4M3) variant of the tile convolution: the quantiser bit for bit against the oracle's
encoder (both round the fp32 product x * scale to the nearest code, ties to even, saturating at 448), the
convolution on codes against the fp64 convolution of the decoded values."""
import numpy as np
import pytest
import torch

import oracle as orc
import paper_1801_02108_amd as sb
from paper_1801_02108_amd import inputs as gen
from util import TORCH_DT, assert_close, to_dev, to_host

pytestmark = pytest.mark.gpu


def step(msg):
    print("[case] " + msg, flush=True)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "f16"])
def test_quantize_f8_bit_exact(dtype):
    step("quantize_f8 " + dtype)
    r = gen.rng_for(30, len(dtype))
    x = (r.standard_normal(70001) * np.exp(r.uniform(-9, 7, 70001))).astype(np.float32)
    special = np.array([0.0, -0.0, 1.0, -1.0, 448.0, 449.0, 464.0, 480.0, 1e6, -1e6, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10,
                        2.0 ** -6, 0.9 * 2.0 ** -6, 1.0625, 1.1875, 17.0, 18.0, 19.0, 1e-30], dtype=np.float32)
    x = np.concatenate([special, x])
    if dtype == "f16":
        x = np.clip(x, -60000, 60000)
    x = gen.round_to(x, dtype)
    for scale in (1.0, 0.37, 12.5):
        got = sb.quantize_f8(to_dev(x, dtype), scale).cpu().numpy()
        want = orc.quantize_f8(x, scale)
        assert np.array_equal(got, want), (int((got != want).sum()), x[got != want][:5], got[got != want][:5], want[got != want][:5])


F8_CASES = [
    # B, th, tw, Cin, Cout, k, s, relu, bias
    (5, 18, 18, 64, 64, 3, 1, False, True),       # the headline tile shape
    (3, 18, 18, 64, 64, 3, 1, True, True),
    (2, 18, 18, 256, 64, 1, 1, True, True),       # residual unit's first convolution: channel chunks
    (3, 16, 16, 64, 256, 1, 1, False, False),     # ... and its last: four channel groups
    (4, 33, 33, 64, 96, 3, 2, True, True),        # stride 2, second channel group half empty
    (2, 34, 34, 32, 64, 3, 1, False, True),       # several passes per tile
    (4, 10, 10, 48, 40, 3, 1, True, False),       # Cin padded to 64 inside the kernel, ragged Cout
    (3, 11, 9, 16, 8, 3, 2, False, True),         # ragged pixel blocks
    (2, 9, 9, 16, 24, 5, 1, True, True),
    (300, 10, 10, 32, 32, 3, 1, True, True),      # many small tiles: more work items than workgroups
]


@pytest.mark.parametrize("B,th,tw,Cin,Cout,k,s,relu,bias", F8_CASES)
def test_conv_on_tiles_f8(B, th, tw, Cin, Cout, k, s, relu, bias):
    step("conv_on_tiles_f8 %s" % ((B, th, tw, Cin, Cout, k, s, relu, bias),))
    r = gen.rng_for(31, th * 1000 + tw * 10 + Cin + Cout + s)
    sx, sw = 16.0, 64.0                                          # activations O(1) and weights O(0.1) into the format's range
    t_codes = orc.quantize_f8(gen.activations(r, (B + 1, th, tw, Cin), "bf16"), sx)
    w_codes = orc.quantize_f8(gen.conv_weights(r, k, k, Cin, Cout, "bf16"), sw)
    b = gen.bias_vector(r, Cout, 0.5) if bias else None
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    oh, ow = (th - k) // s + 1, (tw - k) // s + 1
    out = torch.full((B + 1, oh, ow, Cout), 5.0, dtype=torch.bfloat16).cuda()
    wp = sb.pack_weights_f8(torch.from_numpy(w_codes).cuda())
    sb.conv_on_tiles_f8(torch.from_numpy(t_codes).cuda(), cnt, wp, None if b is None else torch.from_numpy(b).cuda(),
                        stride=s, relu=relu, out_scale=1.0 / (sx * sw), out=out)
    got = to_host(out)
    ref = orc.conv_valid_f8(t_codes[:B], w_codes, b, stride=s, relu=relu, out_scale=1.0 / (sx * sw))
    # exact products, fp32 sums, one rounding to bf16 (unit roundoff 2^-9 = 2e-3)
    assert_close(got[:B], ref, 8e-3, "conv_on_tiles_f8")
    assert (got[B] == 5.0).all()


def test_f8_pipeline_from_bf16_tiles_tracks_the_bf16_convolution():
    """Quantise gathered bf16 tiles and bf16 weights on the device, convolve in FP8, and compare with the oracle's
    convolution of the unquantised values: the difference is the quantisation error of two 3-bit mantissas averaged
    over 576 products, a few percent of the output's scale."""
    step("f8 pipeline")
    r = gen.rng_for(32)
    B, th, C, K = 6, 18, 64, 64
    t = gen.activations(r, (B, th, th, C), "bf16")
    w = gen.conv_weights(r, 3, 3, C, K, "bf16")
    cnt = torch.tensor([B], dtype=torch.int32).cuda()
    sx, sw = 16.0, 64.0
    tq = sb.quantize_f8(to_dev(t, "bf16"), sx)
    wq = sb.quantize_f8(to_dev(w, "bf16"), sw)
    out = sb.conv_on_tiles_f8(tq, cnt, sb.pack_weights_f8(wq), out_scale=1.0 / (sx * sw))
    ref = orc.conv_valid(t, w)
    err = to_host(out) - ref
    assert np.sqrt((err ** 2).mean()) < 0.05 * np.sqrt((ref ** 2).mean())
    # and exactly the oracle's FP8 convolution of the codes the device produced
    assert_close(to_host(out), orc.conv_valid_f8(tq.cpu().numpy(), wq.cpu().numpy(), out_scale=1.0 / (sx * sw)), 8e-3, "f8 on device codes")
