"""The C-ABI library loads and exports every symbol include/sbnet.h declares; host-only entry
points (geometry, size queries, argument checks that return before any launch) behave as the
header says.  No kernel is launched here."""
import ctypes
import os
import re

import pytest

import oracle as orc
import paper_1801_02108_amd as sb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "sbnet.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sbnet_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert len(names) >= 10
    raw = ctypes.CDLL(sb.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), "missing export " + n
    assert names == sb.exported_symbols()       # the binding wraps exactly the declared set


@pytest.mark.parametrize("H,W,k,s,bo", [(64, 64, 3, 1, 8), (800, 704, 3, 1, 16), (400, 352, 3, 1, 16), (13, 10, 3, 1, 4),
                                        (17, 17, 3, 2, 2), (12, 12, 1, 1, 3), (50, 88, 3, 1, 32), (9, 9, 5, 1, 3)])
def test_geometry_host_call_matches_oracle(H, W, k, s, bo):
    g_in, g_out, ho, wo = sb.geometry(H, W, k, s, bo)
    og_in, og_out, oho, owo = orc.geometry(H, W, k, s, bo)
    assert g_in.astuple() == og_in.astuple() and g_out.astuple() == og_out.astuple() and (ho, wo) == (oho, owo)


def test_geometry_rejects_bad_sizes():
    with pytest.raises(sb.SbnetError) as e:
        sb.geometry(0, 4, 3, 1, 2)
    assert e.value.code == sb.EINVAL and "positive" in str(e.value)


@pytest.mark.parametrize("k,s,bo,factor", [(3, 1, 16, 8), (3, 1, 8, 4), (3, 2, 8, 8), (5, 1, 16, 2), (3, 1, 24, 8), (1, 1, 8, 8)])
def test_coarse_geometry_covers_the_cells_each_window_touches(k, s, bo, factor):
    """sbnet_coarse_geometry against brute force: the cells a window's pixels fall into, block by block."""
    g_in, _, _, _ = sb.geometry(160, 96, k, s, bo)
    c = sb.coarse_geometry(g_in, factor)
    assert (c.bcount_h, c.bcount_w) == (g_in.bcount_h, g_in.bcount_w)
    for size, stride, off, csize, cstride, coff, cnt in (
            (g_in.bsize_h, g_in.bstride_h, g_in.boffset_h, c.bsize_h, c.bstride_h, c.boffset_h, g_in.bcount_h),
            (g_in.bsize_w, g_in.bstride_w, g_in.boffset_w, c.bsize_w, c.bstride_w, c.boffset_w, g_in.bcount_w)):
        for b in range(cnt):
            cells = sorted({(off + b * stride + i) // factor for i in range(size)})     # Python's // floors
            assert cells == list(range(coff + b * cstride, coff + b * cstride + csize)), (b, cells)
    # a block stride that is no multiple of the factor has no such geometry
    g3, _, _, _ = sb.geometry(160, 96, 3, 1, 12)
    with pytest.raises(sb.SbnetError):
        sb.coarse_geometry(g3, 8)


def test_size_queries():
    g_in, _, _, _ = sb.geometry(800, 704, 3, 1, 16)
    ws = sb.workspace_bytes(8, g_in)
    assert ws >= 8 * 50 * 44 + 4 * 8 * 50 and ws % 16 == 0
    nbytes = ctypes.c_size_t()
    lib = sb.lib()
    assert lib.sbnet_pack_weights(None, sb.BF16, 3, 3, 64, 64, None, nbytes, None) == sb.OK
    assert nbytes.value == 2 * 3 * 3 * 64 * 64 * 2         # two operand orders
    assert lib.sbnet_pack_weights(None, sb.BF16, 3, 3, 24, 40, None, nbytes, None) == sb.OK
    assert nbytes.value == 2 * 3 * 3 * 32 * 64 * 2      # channels padded to the MFMA tile
    assert lib.sbnet_pack_weights(None, sb.F32, 3, 3, 16, 16, None, nbytes, None) == sb.OK
    assert nbytes.value == 3 * 3 * 16 * 16 * 4


def test_null_pointers_are_rejected_before_any_launch():
    lib = sb.lib()
    g_in, g_out, _, _ = sb.geometry(16, 16, 3, 1, 4)
    assert lib.sbnet_reduce_mask(None, sb.U8, 1, 16, 16, g_in, 1, 0.0, None, None, 16, None, 0, None) == sb.EINVAL
    assert b"null" in lib.sbnet_last_error()
    assert lib.sbnet_sparse_gather(None, sb.BF16, 1, 16, 16, 8, None, None, 4, g_in, None, None) == sb.EINVAL
    assert lib.sbnet_sparse_scatter(None, sb.BF16, None, None, 4, g_out, None, 1, 16, 16, 8, 0, None) == sb.EINVAL
    assert lib.sbnet_conv_on_tiles(None, sb.BF16, None, 4, 6, 6, 8, None, None, 3, 3, 1, 1, 8, 0, None, None) == sb.EINVAL


def test_gradient_and_normalisation_calls_check_their_arguments_on_the_host():
    """Size queries and the argument checks of the training-side entry points, none of which reaches a launch."""
    lib = sb.lib()
    _, g_out, _, _ = sb.geometry(16, 16, 3, 1, 4)
    g_in = sb.geometry(16, 16, 3, 1, 4)[0]
    # data gradient: the framed copy at stride 2, one index triple per tile at stride 1
    assert lib.sbnet_conv_backward_data_workspace_bytes(sb.BF16, 10, 33, 33, 3, 3, 2, 2, 96) >= 10 * 35 * 35 * 96 * 2
    assert 2200 * 12 <= lib.sbnet_conv_backward_data_workspace_bytes(sb.BF16, 2200, 18, 18, 3, 3, 1, 1, 64) < 2200 * 12 + 256
    assert lib.sbnet_conv_backward_data_workspace_bytes(sb.U8, 7, 6, 6, 3, 3, 1, 1, 8) == 0
    nbytes = ctypes.c_size_t()
    assert lib.sbnet_pack_weights_transposed(None, sb.BF16, 3, 3, 64, 96, None, nbytes, None) == sb.OK
    fwd = ctypes.c_size_t()
    assert lib.sbnet_pack_weights(None, sb.BF16, 3, 3, 96, 64, None, fwd, None) == sb.OK
    assert nbytes.value == fwd.value                    # packed for a convolution with the channel roles exchanged
    assert lib.sbnet_conv_on_tiles_backward_data(None, sb.BF16, None, 4, 6, 6, 8, None, 3, 3, 1, 1, 8, None, None, 0,
                                                 None) == sb.EINVAL
    assert b"null" in lib.sbnet_last_error()
    # weight gradient: one partial result per split, a split for at most every tile
    one = lib.sbnet_conv_backward_weights_workspace_bytes(sb.BF16, 1, 18, 18, 64, 3, 3, 1, 1, 64)
    many = lib.sbnet_conv_backward_weights_workspace_bytes(sb.BF16, 5000, 18, 18, 64, 3, 3, 1, 1, 64)
    assert one >= 9 * 64 * 64 * 4 and one < 2 * 9 * 64 * 64 * 4 and many >= 256 * 9 * 64 * 64 * 4
    assert lib.sbnet_conv_backward_weights_workspace_bytes(sb.BF16, 4, 2, 2, 8, 3, 3, 1, 1, 8) == 0     # tile < kernel
    assert lib.sbnet_conv_on_tiles_backward_weights(None, None, sb.BF16, None, 4, 6, 6, 8, 3, 3, 1, 1, 8, None, None, 0,
                                                    None) == sb.EINVAL
    # ReLU mask and bias sum in one pass: refused without the activation or the place for the masked gradient,
    # and for pixels whose channels do not fill 4-byte words
    buf0 = (ctypes.c_char * 4096)()
    p0 = ctypes.cast(ctypes.byref(buf0, 16 - ctypes.addressof(buf0) % 16), ctypes.c_void_p)
    assert lib.sbnet_relu_bias_backward_on_tiles(None, p0, sb.BF16, p0, 4, 9, 8, p0, p0, p0, 4096, None) == sb.EINVAL
    assert lib.sbnet_relu_bias_backward_on_tiles(p0, p0, sb.BF16, p0, 4, 9, 8, None, p0, p0, 4096, None) == sb.EINVAL
    assert lib.sbnet_relu_bias_backward_on_tiles(p0, p0, sb.BF16, p0, 4, 9, 3, p0, p0, p0, 4096, None) == sb.EUNSUPPORTED
    assert lib.sbnet_relu_bias_backward_on_tiles(p0, p0, sb.BF16, p0, 4, 9, 8, p0, p0, p0, 8, None) == sb.EINVAL
    assert b"workspace" in lib.sbnet_last_error()
    # normalisation
    assert lib.sbnet_bn_backward_workspace_bytes(10, 64) == (10 * 64 * 2 + 10 + 1) * 4
    assert lib.sbnet_bn_backward_workspace_bytes(0, 64) == 4
    assert lib.sbnet_sparse_bn_apply(None, sb.BF16, 1, 16, 16, 8, None, None, 4, g_out, None, None, None, None, 1e-5, 0,
                                     None, None) == sb.EINVAL
    assert lib.sbnet_sparse_bn_backward(None, None, sb.BF16, 1, 16, 16, 8, None, None, 4, g_out, None, None, None, None,
                                        1e-5, 0, None, None, None, None, 0, None) == sb.EINVAL
    # overlapping blocks (an input-tile geometry) would count pixels twice: refused with valid pointers too
    buf = (ctypes.c_char * 4096)()
    ptr = ctypes.cast(ctypes.byref(buf, 16 - ctypes.addressof(buf) % 16), ctypes.c_void_p)
    assert lib.sbnet_sparse_bn_apply(ptr, sb.BF16, 1, 16, 16, 8, ptr, ptr, 4, g_in, ptr, ptr, None, None, 1e-5, 0, ptr,
                                     None) == sb.EINVAL
    assert b"overlap" in lib.sbnet_last_error()
    assert lib.sbnet_sparse_bn_apply(ptr, sb.BF16, 1, 16, 16, 8, ptr, ptr, 4, g_out, ptr, ptr, None, None, -1.0, 0, ptr,
                                     None) == sb.EINVAL


def test_f8_entry_points_check_their_arguments_on_the_host():
    lib = sb.lib()
    nbytes = ctypes.c_size_t()
    assert lib.sbnet_pack_weights_f8(None, 3, 3, 64, 64, None, nbytes, None) == sb.OK and nbytes.value == 9 * 64 * 64
    assert lib.sbnet_pack_weights_f8(None, 3, 3, 48, 40, None, nbytes, None) == sb.OK and nbytes.value == 9 * 64 * 64
    buf = (ctypes.c_char * 4096)()
    ptr = ctypes.cast(ctypes.byref(buf, 16 - ctypes.addressof(buf) % 16), ctypes.c_void_p)
    assert lib.sbnet_quantize_f8(None, sb.BF16, 16, 1.0, None, None) == sb.EINVAL
    assert lib.sbnet_quantize_f8(ptr, sb.BF16, 16, 0.0, ptr, None) == sb.EINVAL and b"scale" in lib.sbnet_last_error()
    assert lib.sbnet_quantize_f8(ptr, sb.U8, 16, 1.0, ptr, None) == sb.EUNSUPPORTED
    assert lib.sbnet_quantize_f8(ptr, sb.BF16, 0, 1.0, ptr, None) == sb.OK          # nothing to do, nothing launched
    assert lib.sbnet_conv_on_tiles_f8(ptr, ptr, 4, 6, 6, 24, ptr, None, 3, 3, 1, 1, 8, 0, 1.0, ptr, None) == sb.EUNSUPPORTED
    assert b"multiple of 16" in lib.sbnet_last_error()
    assert lib.sbnet_conv_on_tiles_f8(None, None, 4, 6, 6, 16, None, None, 3, 3, 1, 1, 8, 0, 1.0, None, None) == sb.EINVAL
    assert lib.sbnet_conv_on_tiles_f8(ptr, ptr, 4, 6, 6, 16, ptr, None, 3, 3, 1, 1, 8, 0, float("inf"), ptr, None) == sb.EINVAL


def test_bottleneck_backward_checks_its_arguments_on_the_host():
    lib = sb.lib()
    need = lib.sbnet_bottleneck_backward_workspace_bytes(sb.BF16, 100, 18, 18, 256, 64)
    # dL/dt2 and dL/dt1 of 100 tiles plus the largest scratch of the single calls (the 3x3 weight gradient's partial sums)
    assert need >= 100 * (16 * 16 + 18 * 18) * 64 * 2 + 100 * 9 * 64 * 64 * 4 // 2
    assert lib.sbnet_bottleneck_backward_workspace_bytes(sb.U8, 100, 18, 18, 256, 64) == 0
    assert lib.sbnet_bottleneck_backward_workspace_bytes(sb.BF16, 100, 2, 18, 256, 64) == 0
    n = None
    assert lib.sbnet_bottleneck_backward_on_tiles(n, n, n, n, sb.BF16, n, 4, 18, 18, 256, 64, n, n, n, n, n, n, n, n, n, n, n, 0,
                                                  n) == sb.EINVAL
    assert b"null" in lib.sbnet_last_error()


def test_overlapping_input_and_output_are_rejected_not_only_equal_pointers():
    """The fused calls read halo pixels of x that other workgroups may already have overwritten if y shared memory with
    x: any overlap of the two byte ranges is an argument error, found on the host (fake, aligned addresses; no launch)."""
    lib = sb.lib()
    g_in, g_out, _, _ = sb.geometry(32, 32, 3, 1, 16)
    base = 0x7f0000000000
    nbytes = 1 * 32 * 32 * 64 * 2
    P = ctypes.c_void_p
    for dy in (0, 16, nbytes // 2, nbytes - 16):
        rc = lib.sbnet_sparse_conv(P(base), sb.BF16, 1, 32, 32, 64, P(base), P(base), 4, g_in, g_out, P(base), None,
                                   3, 3, 1, 1, 64, 0, P(base + dy), 32, 32, 0, None)
        assert rc == sb.EINVAL and b"overlap" in lib.sbnet_last_error(), dy
        rc = lib.sbnet_sparse_bottleneck(P(base), sb.BF16, 1, 32, 32, 64, 64, P(base), P(base), 4, g_in, g_out, P(base), P(base),
                                         P(base), P(base), P(base), P(base), P(base + dy), None)
        assert rc == sb.EINVAL and b"overlap" in lib.sbnet_last_error(), dy
