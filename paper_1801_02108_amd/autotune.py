"""Block-size search (Sec. 4 of arXiv 1801.02108, "Choosing the optimal block sizes").

Small blocks follow the mask closely but read more overlap; large blocks read less overlap but
cover more inactive pixels.  The paper picks the block size of a layer by timing a sweep; this
module does the same on the device the library runs on: for every candidate it builds the
geometry, reduces the mask to its block list and times the fused sparse step (reduce_mask +
sparse_conv, or reduce_mask + sparse_bottleneck) from HIP-graph replays, then keeps the fastest.

Only host logic and calls of the binding live here; the sub-tile choices inside the kernels (16- or
8-pixel sub-tiles of the residual unit, 256- or 128-pixel workgroup tiles of the 3x3 kernels) are
made on the device from the active count and need no tuning.  Winners are cached under a key of the
layer shape and the mask's coarse density, and the cache can be stored as JSON.
"""
import json

import torch

from . import (POOL_AVG, geometry, pack_weights, read_count, reduce_mask, sparse_bottleneck, sparse_conv,
               workspace_bytes)


class TuneResult:
    """Outcome of one sweep: `best` block size and the `table` of per-candidate measurements."""

    def __init__(self, best, table):
        self.best = best
        self.table = table

    def as_dict(self):
        return {"best": self.best, "table": self.table}


def density_bucket(active_pixel_fraction):
    """Masks within the same factor-of-two band of pixel density share a cache entry (0: empty mask)."""
    f = float(active_pixel_fraction)
    if f <= 0.0:
        return 0
    b = 1
    while f < 1.0 and b < 16:
        f *= 2.0
        b += 1
    return b


def cache_key(kind, N, H, W, Cin, Cout, stride, dtype, bucket):
    return "%s:%dx%dx%dx%d->%d:s%d:%s:d%d" % (kind, N, H, W, Cin, Cout, stride, str(dtype).replace("torch.", ""), bucket)


def pick_best(table):
    """Fastest valid candidate of a sweep table ({block: {"ms": ...} or {"error": ...}}); ties go to the
    larger block (less overlap).  Raises if no candidate ran."""
    ok = [(row["ms"], -bo, bo) for bo, row in table.items() if "ms" in row]
    if not ok:
        raise ValueError("no block size could be run: %r" % (table,))
    return min(ok)[2]


def device_ms(fn, reps=10, replays=5):
    """Milliseconds of device time per call of fn(): HIP events around replays of a graph of `reps` calls."""
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(reps):
            fn()
    g.replay()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / (reps * replays)


class BlockSizeTuner:
    """Sweeps block sizes for one layer on one mask and remembers the winners.

    measure: callable(fn) -> milliseconds; the default times HIP-graph replays on the current device
    (tests of the host logic pass their own).
    """

    def __init__(self, candidates=(8, 16, 32), measure=device_ms):
        self.candidates = tuple(candidates)
        self.measure = measure
        self.cache = {}

    # ---- cache -------------------------------------------------------------------------------
    def save(self, path):
        with open(path, "w") as f:
            json.dump(self.cache, f, indent=1, sort_keys=True)

    def load(self, path):
        with open(path) as f:
            self.cache.update(json.load(f))

    def lookup(self, key):
        hit = self.cache.get(key)
        return None if hit is None else hit["best"]

    # ---- sweeps ------------------------------------------------------------------------------
    def _sweep(self, key, run_for_block):
        if key in self.cache:
            c = self.cache[key]
            return TuneResult(c["best"], c["table"])
        table = {}
        for bo in self.candidates:
            try:
                step, nact, total = run_for_block(bo)
                table[bo] = {"ms": self.measure(step), "active_blocks": nact, "total_blocks": total}
            except Exception as e:                       # a candidate the kernels do not take is skipped, not fatal
                table[bo] = {"error": str(e)}
        res = TuneResult(pick_best(table), table)
        # JSON keys are strings: store the table that way so that a reloaded cache looks the same
        self.cache[key] = {"best": res.best, "table": {str(bo): row for bo, row in table.items()}}
        return res

    def tune_conv(self, x, mask, w_hwio, bias=None, stride=1, relu=True):
        """Fastest block size for y = sparse 3x3 (or kxk) conv of x [N,H,W,Cin] under `mask` [N,H,W] (uint8)."""
        N, H, W, Cin = x.shape
        k, _, _, Cout = w_hwio.shape
        wp = pack_weights(w_hwio)
        bucket = density_bucket(float(mask.float().mean().item()))
        key = cache_key("conv%d" % k, N, H, W, Cin, Cout, stride, x.dtype, bucket)

        def run_for_block(bo):
            g_in, g_out, Ho, Wo = geometry(H, W, k, stride, bo)
            total = N * g_in.bcount_h * g_in.bcount_w
            idx = torch.empty((total, 3), dtype=torch.int32, device=x.device)
            cnt = torch.empty((1,), dtype=torch.int32, device=x.device)
            ws = torch.empty((workspace_bytes(N, g_in),), dtype=torch.uint8, device=x.device)
            y = torch.zeros((N, Ho, Wo, Cout), dtype=x.dtype, device=x.device)

            def step():
                reduce_mask(mask, g_in, POOL_AVG, 0.0, idx, cnt, ws)
                sparse_conv(x, idx, cnt, g_in, g_out, wp, bias, y, stride=stride, relu=relu)
            step()
            return step, read_count(cnt, total), total
        return self._sweep(key, run_for_block)

    def tune_bottleneck(self, x, mask, weights):
        """Fastest block size for the fused residual unit (Sec. 3.3) on x [N,H,W,C] under `mask`; `weights` as
        sparse_bottleneck takes them.  The unit writes x + t3 into a second buffer (ping-pong)."""
        N, H, W, C = x.shape
        bucket = density_bucket(float(mask.float().mean().item()))
        key = cache_key("bottleneck", N, H, W, C, C, 1, x.dtype, bucket)

        def run_for_block(bo):
            g_in, g_out, _, _ = geometry(H, W, 3, 1, bo)
            total = N * g_in.bcount_h * g_in.bcount_w
            idx = torch.empty((total, 3), dtype=torch.int32, device=x.device)
            cnt = torch.empty((1,), dtype=torch.int32, device=x.device)
            ws = torch.empty((workspace_bytes(N, g_in),), dtype=torch.uint8, device=x.device)
            y = x.clone()

            def step():
                reduce_mask(mask, g_in, POOL_AVG, 0.0, idx, cnt, ws)
                sparse_bottleneck(x, idx, cnt, g_in, g_out, weights, y)
            step()
            return step, read_count(cnt, total), total
        return self._sweep(key, run_for_block)
