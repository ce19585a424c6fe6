"""sbnet_reduce_mask_static (the entry point that allocates nothing) against sbnet_reduce_mask and the
oracle: bit-exact index lists and counts, on two calls in a row of which the second is smaller, so
that whatever the first call left in the built-in scratch buffer is shown not to matter."""
import ctypes

import numpy as np
import pytest
import torch

import oracle as orc
import paper_1801_02108_amd as sb
from paper_1801_02108_amd import inputs as gen

pytestmark = pytest.mark.gpu


def _one_call(lib, mask_np, N, H, W, bo, pool, thr, cap_extra=0):
    g_in, _, _, _ = sb.geometry(H, W, 3, 1, bo)
    cap = N * g_in.bcount_h * g_in.bcount_w + cap_extra
    mask = torch.from_numpy(mask_np).cuda()
    # every buffer exists before the call under test; the call itself gets raw pointers only
    idx_s = torch.full((cap, 3), -7, dtype=torch.int32, device="cuda")
    cnt_s = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    rc = lib.sbnet_reduce_mask_static(ctypes.c_void_p(mask.data_ptr()), sb.U8 if mask.dtype == torch.uint8 else sb.F32,
                                      N, H, W, g_in, pool, ctypes.c_float(thr), ctypes.c_void_p(idx_s.data_ptr()),
                                      ctypes.c_void_p(cnt_s.data_ptr()), cap, stream)
    assert rc == sb.OK, lib.sbnet_last_error()
    idx_w, cnt_w = sb.reduce_mask(mask, g_in, pool, thr)          # the existing entry point, with a workspace
    n_s, n_w = sb.read_count(cnt_s, cap), sb.read_count(cnt_w, cap)
    og = orc.Geom(*g_in.astuple())
    oidx = orc.reduce_mask(mask_np, og, pool, thr)
    assert n_s == n_w == len(oidx)
    got = idx_s.cpu().numpy()
    assert np.array_equal(got[:n_s], idx_w[:n_w].cpu().numpy())
    assert np.array_equal(got[:n_s], oidx)
    assert (got[n_s:] == -7).all()                                   # rows beyond the count stay untouched
    return n_s


def test_static_scratch_matches_workspace_call_twice_second_smaller():
    lib = sb.lib()
    r = gen.rng_for(7)
    # first call: 3 samples of 160 x 208, 8 x 8 blocks (1560 blocks, 60 block rows)
    m1 = (r.random((3, 160, 208)) < 0.004).astype(np.uint8)
    n1 = _one_call(lib, m1, 3, 160, 208, 8, sb.POOL_MAX, 0.0)
    assert 0 < n1 < 3 * 20 * 26
    # second call, smaller in every extent, other pooling and mask type: 1 sample of 50 x 37 (ragged), 16 x 16 blocks
    m2 = (r.random((1, 50, 37)) < 0.01).astype(np.float32)
    n2 = _one_call(lib, m2, 1, 50, 37, 16, sb.POOL_AVG, 0.0, cap_extra=5)
    assert 0 < n2 <= 4 * 3
    # and an empty mask after both: the count must be rewritten to 0, not left over
    n3 = _one_call(lib, np.zeros((1, 50, 37), np.uint8), 1, 50, 37, 16, sb.POOL_AVG, 0.0)
    assert n3 == 0


def test_static_scratch_rejects_problems_beyond_its_size():
    lib = sb.lib()
    g_in, _, _, _ = sb.geometry(4096, 4096, 3, 1, 2)      # 2048 x 2048 blocks: 4 MiB of flags per sample
    assert sb.workspace_bytes(1, g_in) > (1 << 20)
    d = torch.zeros(16, dtype=torch.int32, device="cuda")
    rc = lib.sbnet_reduce_mask_static(ctypes.c_void_p(d.data_ptr()), sb.U8, 1, 4096, 4096, g_in, sb.POOL_MAX,
                                      ctypes.c_float(0.0), ctypes.c_void_p(d.data_ptr()), ctypes.c_void_p(d.data_ptr()),
                                      4, None)
    assert rc == sb.EUNSUPPORTED and b"built-in buffer" in lib.sbnet_last_error()
