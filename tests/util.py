"""Helpers shared by the GPU parity tests: host<->device marshalling and the tolerance rule."""
import numpy as np
import torch

TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}
# relative tolerance of convolution outputs against the fp64 oracle: 1e-4 for fp32 and 2e-2 for
# bf16 are the stated targets; fp16 (11-bit significand, unit roundoff 2^-11 = 4.9e-4, one
# rounding of the output plus fp32 accumulation) gets 4e-3.
CONV_TOL = {"f32": 1e-4, "bf16": 2e-2, "f16": 4e-3}


def to_dev(a, dtype):
    """numpy float array holding values exact in `dtype` -> contiguous device tensor of that dtype."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(TORCH_DT[dtype])
    return t.cuda().contiguous()


def to_host(t):
    """device tensor -> float64 numpy (exact)."""
    return t.detach().to(torch.float64).cpu().numpy()


def round_like(a64, dtype):
    """Round an fp64 array to the storage type the way the GPU's final store does (nearest even)."""
    return torch.from_numpy(np.ascontiguousarray(a64)).to(TORCH_DT[dtype]).to(torch.float64).numpy()


def assert_close(got, ref, tol, what=""):
    """|got - ref| <= tol*|ref| + tol*RMS(ref), element by element."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    rms = float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0
    err = np.abs(got - ref)
    bound = tol * np.abs(ref) + tol * rms
    bad = err > bound
    if bad.any():
        k = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError("%s: %d of %d elements out of tolerance %g; worst at %s got %r ref %r (rms %g)" % (
            what, int(bad.sum()), err.size, tol, k, got[k], ref[k], rms))
    return float(err.max() / (np.abs(ref).max() + 1e-300)) if ref.size else 0.0
