"""Seeded synthetic inputs shaped like the paper's LiDAR bird's-eye-view workloads.

Serves the tests (oracle side and GPU side alike) and the benchmark.  It holds none of the
method's arithmetic: masks are drawn, tensors are sampled and rounded to the storage type,
nothing is pooled, gathered or convolved here.  Where a mask family has to hit a target
fraction of active *blocks*, the caller supplies the function that counts active blocks
(`count_active(mask) -> int`), so the count comes from whichever implementation is under test.

The paper's own masks (road maps of a private dataset, outputs of a trained segmentation
network; Sec. 4.1-4.3) are not available; these generators stand in for them:
  rect_mask       a few axis-aligned rectangles (small correctness case)
  topleft_mask    the paper's "synthetic" mask: a top-left sub-region (Sec. 4.3)
  road_band_mask  thick random polylines crossing the frame (road / sidewalk maps)
  blob_mask       thresholded low-pass noise (predicted foreground masks)
  lowres_mask     thresholded 1/8-resolution logits, nearest-upsampled (dynamic mask network)
"""
import numpy as np

BASE_SEED = 180102108


def rng_for(config, extra=0):
    return np.random.default_rng(BASE_SEED + 1000 * int(config) + int(extra))


# ----------------------------------------------------------------------------- storage rounding
def round_to_bf16(a):
    """float32 array rounded to the nearest bfloat16 (ties to even), returned as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def round_to(a, dtype):
    """Round a float array to storage type 'f32' | 'bf16' | 'f16'; result is float32 holding exact values."""
    if dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    if dtype == "bf16":
        return round_to_bf16(a)
    if dtype == "f16":
        return np.asarray(a, dtype=np.float32).astype(np.float16).astype(np.float32)
    raise ValueError(dtype)


def activations(rng, shape, dtype):
    """N(0,1) feature map, rounded to the storage type."""
    return round_to(rng.standard_normal(shape, dtype=np.float32), dtype)


def conv_weights(rng, kh, kw, cin, cout, dtype, unit_variance=False, scale=1.0):
    """HWIO weights: N(0,1) when unit_variance (the small fp32 case), else N(0, 2/fan_in)."""
    w = rng.standard_normal((kh, kw, cin, cout), dtype=np.float32)
    if not unit_variance:
        w *= np.float32(np.sqrt(2.0 / (kh * kw * cin)) * scale)
    return round_to(w, dtype)


def bias_vector(rng, cout, std=0.1):
    return (rng.standard_normal(cout, dtype=np.float32) * np.float32(std)).astype(np.float32)


def bottleneck_weights(rng, c, cm, dtype):
    """Folded-BN weights of a 1x1 -> 3x3 -> 1x1 unit; last conv halved so a stack of units stays O(1-10)."""
    w1 = conv_weights(rng, 1, 1, c, cm, dtype)
    w2 = conv_weights(rng, 3, 3, cm, cm, dtype)
    w3 = conv_weights(rng, 1, 1, cm, c, dtype, scale=0.5)
    return w1, bias_vector(rng, cm), w2, bias_vector(rng, cm), w3, bias_vector(rng, c)


# ----------------------------------------------------------------------------- masks
def rect_mask(rng, H, W, n_rects=3, target=0.10):
    """n_rects random axis-aligned rectangles whose areas sum to about `target` of the frame."""
    m = np.zeros((1, H, W), dtype=np.uint8)
    per = target / n_rects
    for _ in range(n_rects):
        aspect = rng.uniform(0.5, 2.0)
        h = int(np.clip(round(np.sqrt(per * H * W * aspect)), 1, H))
        w = int(np.clip(round(per * H * W / h), 1, W))
        y0 = int(rng.integers(0, H - h + 1))
        x0 = int(rng.integers(0, W - w + 1))
        m[0, y0:y0 + h, x0:x0 + w] = 1
    return m


def topleft_mask(N, H, W, rows, cols):
    m = np.zeros((N, H, W), dtype=np.uint8)
    m[:, :rows, :cols] = 1
    return m


def _polyline_distance(H, W, pts):
    """Distance of every pixel centre to a polyline given as [(y, x), ...]."""
    yy, xx = np.mgrid[0:H, 0:W].astype(np.float32)
    d = np.full((H, W), np.inf, dtype=np.float32)
    for (y0, x0), (y1, x1) in zip(pts[:-1], pts[1:]):
        vy, vx = y1 - y0, x1 - x0
        L2 = max(vy * vy + vx * vx, 1e-6)
        t = np.clip(((yy - y0) * vy + (xx - x0) * vx) / L2, 0.0, 1.0)
        d = np.minimum(d, np.hypot(yy - (y0 + t * vy), xx - (x0 + t * vx)))
    return d


def road_band_fields(rng, H, W, n_roads=3):
    """Per road: (distance field, base half-width in [10, 30] px, i.e. widths of 20-60 px)."""
    fields = []
    for _ in range(n_roads):
        horizontal = rng.random() < 0.5
        n_pts = int(rng.integers(3, 6))
        if horizontal:
            xs = np.linspace(-10, W + 10, n_pts)
            ys = rng.uniform(0.1 * H, 0.9 * H) + np.cumsum(rng.normal(0, 0.08 * H, n_pts))
        else:
            ys = np.linspace(-10, H + 10, n_pts)
            xs = rng.uniform(0.1 * W, 0.9 * W) + np.cumsum(rng.normal(0, 0.08 * W, n_pts))
        pts = [(float(y), float(x)) for y, x in zip(ys, xs)]
        fields.append((_polyline_distance(H, W, pts), float(rng.uniform(10.0, 30.0))))
    return fields


def road_band_mask(fields, width_scale):
    d0 = fields[0][0]
    m = np.zeros(d0.shape, dtype=bool)
    for d, half in fields:
        m |= d <= half * width_scale
    return m[None].astype(np.uint8)


def smooth_noise(rng, N, H, W, sigma):
    """White noise low-passed with a separable Gaussian of std `sigma` pixels (FFT, periodic)."""
    z = rng.standard_normal((N, H, W), dtype=np.float32)
    fy = np.fft.fftfreq(H)[:, None]
    fx = np.fft.rfftfreq(W)[None, :]
    g = np.exp(-2.0 * (np.pi * sigma) ** 2 * (fy * fy + fx * fx)).astype(np.float32)
    out = np.fft.irfft2(np.fft.rfft2(z, axes=(1, 2)) * g, s=(H, W), axes=(1, 2)).astype(np.float32)
    return out / out.std()


def blob_mask(field, thresh):
    return (field > thresh).astype(np.uint8)


def lowres_mask(logits, thresh, up=8):
    """Threshold a low-resolution logit map and nearest-upsample it by `up`."""
    m = (logits > thresh).astype(np.uint8)
    return np.repeat(np.repeat(m, up, axis=1), up, axis=2)


def calibrate(make_mask, count_active, total_blocks, target, lo, hi, increasing=True, iters=30, tol=0.005):
    """Bisect the free parameter of a mask family until the active-block fraction is within
    `tol` of `target`.  make_mask(param) -> mask; count_active(mask) -> int (caller's choice of
    implementation).  Returns (mask, param, achieved_fraction)."""
    best = None
    for _ in range(iters):
        mid = 0.5 * (lo + hi)
        m = make_mask(mid)
        frac = count_active(m) / float(total_blocks)
        if best is None or abs(frac - target) < abs(best[2] - target):
            best = (m, mid, frac)
        if abs(frac - target) <= tol:
            break
        if (frac < target) == increasing:
            lo = mid
        else:
            hi = mid
    return best
