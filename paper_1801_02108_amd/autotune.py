"""Block-size search (Sec. 4 of arXiv 1801.02108, "Choosing the optimal block sizes").

Small blocks follow the mask closely but read more overlap; large blocks read less overlap but
cover more inactive pixels.  The paper picks the block size of a layer by timing a sweep; this
module does the same on the device the library runs on: for every candidate it builds the
geometry, reduces the mask to its block list and times the fused sparse step (reduce_mask +
sparse_conv, or reduce_mask + sparse_bottleneck) from HIP-graph replays, then keeps the fastest.

Only host logic and calls of the binding live here.  Winners are cached under a key of the layer shape,
the mask's coarse density, the layer's options and the candidate set, and the cache can be stored as JSON.

The second half of the search are the compute-tile choices INSIDE the kernels, which the device makes from
its own count of active blocks against thresholds that come with the launch (sbnet_tuning): 16- or 8-pixel
sub-tiles of the residual unit, 256- or 128-pixel work items of the LDS-tiled 3x3 convolution, the number of
splits of the weight gradient.  KernelChoiceTuner measures each alternative forced, over a range of active
counts, reports where the faster one changes (the crossover the default threshold should sit at) and can put
the measured thresholds in force.
"""
import json

import torch

from . import (POOL_AVG, conv_backward_weights_workspace_bytes, conv_on_tiles_backward_weights, geometry, get_tuning,
               pack_weights, read_count, reduce_mask, set_tuning, sparse_bottleneck, sparse_conv, workspace_bytes)


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


def cache_key(kind, N, H, W, Cin, Cout, stride, dtype, bucket, options="", candidates=()):
    """Everything a sweep's outcome depends on: layer shape, density band, the layer's options (ReLU, bias, ...)
    and the block sizes that were tried."""
    return "%s:%dx%dx%dx%d->%d:s%d:%s:d%d:%s:c%s" % (kind, N, H, W, Cin, Cout, stride, str(dtype).replace("torch.", ""), bucket,
                                                   options, "-".join(str(c) for c in candidates))


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
        key = cache_key("conv%d" % k, N, H, W, Cin, Cout, stride, x.dtype, bucket,
                        "relu%d.bias%d" % (int(bool(relu)), int(bias is not None)), self.candidates)

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
        key = cache_key("bottleneck", N, H, W, C, C, 1, x.dtype, bucket, "cm%d" % weights[0].shape[3], self.candidates)

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


def crossover(counts, t_small_regime, t_large_regime):
    """Smallest count from which the large-regime alternative stays at least as fast, given the two alternatives'
    times at ascending `counts`; None when it never is.  (Host logic, separately testable.)"""
    first = None
    for n, a, b in zip(counts, t_small_regime, t_large_regime):
        if b <= a:
            if first is None:
                first = n
        else:
            first = None
    return first


def fit_cost_eighths(counts, ms_large, ms_small, per_large, per_small, floor_ms=0.004, workgroups=256):
    """Cost of a small work item in eighths of a large one, from the times of the two alternatives at `counts` active
    blocks: time above the launch floor divided by the rounds of work either needs, ratio small / large, median over
    the counts.  (Host logic, separately testable.)"""
    ratios = []
    for n, a, b in zip(counts, ms_large, ms_small):
        rl, rs = -(-n * per_large // workgroups), -(-n * per_small // workgroups)
        if a > floor_ms and b > floor_ms:
            ratios.append(((b - floor_ms) / rs) / ((a - floor_ms) / rl))
    if not ratios:
        return None
    ratios.sort()
    return round(8.0 * ratios[len(ratios) // 2], 2)


class KernelChoiceTuner:
    """Measures the device-side compute-tile choices with each alternative forced (through sbnet_tuning) and reports
    the measured crossovers beside the defaults.  `measure` as for BlockSizeTuner."""

    def __init__(self, measure=device_ms):
        self.measure = measure

    def _timed(self, fn, **forced):
        before = get_tuning()
        try:
            set_tuning(**forced)
            return self.measure(fn)
        finally:
            set_tuning(**before)

    def unit_subtiles(self, x, weights, block=16, counts=(8, 16, 32, 64, 96, 128, 160, 192, 256, 384, 512)):
        """Residual unit on x [N,H,W,C]: time with 16 x 16 and with 8 x 8 sub-tiles forced for the first n blocks of
        the grid active, n in `counts`.  Returns the two time rows, which was faster per count, and the cost of an
        8 x 8 item in eighths of a 16 x 16 one fitted to the full rounds of either (what unit_small_item_cost_eighths
        means): the median over counts of 8 * (ms8 / rounds8) / (ms16 / rounds16), launch floor taken off both."""
        N, H, W, C = x.shape
        g_in, g_out, _, _ = geometry(H, W, 3, 1, block)
        total = N * g_in.bcount_h * g_in.bcount_w
        per16, per8 = (block // 16) ** 2, (block // 8) ** 2
        idx_all = torch.tensor([(n, by, bx) for n in range(N) for by in range(g_in.bcount_h) for bx in range(g_in.bcount_w)],
                               dtype=torch.int32, device=x.device)
        y = x.clone()
        ms16, ms8, used = [], [], []
        for n in counts:
            if n > total:
                break
            cnt = torch.tensor([n], dtype=torch.int32, device=x.device)
            fn = lambda: sparse_bottleneck(x, idx_all, cnt, g_in, g_out, weights, y)
            ms16.append(self._timed(fn, unit_small_item_cost_eighths=1000))
            ms8.append(self._timed(fn, unit_small_item_cost_eighths=0))
            used.append(n)
        return {"counts": used, "ms16": ms16, "ms8": ms8, "faster": ["16" if a <= b else "8" for a, b in zip(ms16, ms8)],
                "cost_eighths": fit_cost_eighths(used, ms16, ms8, per16, per8)}

    def conv3_items(self, x, w_hwio, bias=None, stride=1, block=16, counts=(8, 16, 32, 64, 128, 192, 256, 384, 512, 1024)):
        """LDS-tiled 3x3 convolution: time with the larger and with the smaller work item forced (256 and 128 pixels;
        384 and 256 for blocks of 257 ... 384 output pixels, where the rows keep the names ms256 / ms128 for the larger /
        smaller item).  Returns the two time rows and, per count, which was faster."""
        N, H, W, Cin = x.shape
        k, _, _, Cout = w_hwio.shape
        wp = pack_weights(w_hwio)
        g_in, g_out, Ho, Wo = geometry(H, W, k, stride, block)
        total = N * g_in.bcount_h * g_in.bcount_w
        idx_all = torch.tensor([(n, by, bx) for n in range(N) for by in range(g_in.bcount_h) for bx in range(g_in.bcount_w)],
                               dtype=torch.int32, device=x.device)
        y = torch.zeros((N, Ho, Wo, Cout), dtype=x.dtype, device=x.device)
        big, small, used = [], [], []
        for n in counts:
            if n > total:
                break
            cnt = torch.tensor([n], dtype=torch.int32, device=x.device)
            fn = lambda: sparse_conv(x, idx_all, cnt, g_in, g_out, wp, bias, y, stride=stride, relu=True)
            big.append(self._timed(fn, conv3_small_item_cost_eighths=1000))
            small.append(self._timed(fn, conv3_small_item_cost_eighths=0))
            used.append(n)
        return {"counts": used, "ms256": big, "ms128": small,
                "faster": ["256" if b <= s_ else "128" for b, s_ in zip(big, small)]}

    def wgrad_splits(self, tiles, dout, k, stride=1, factors=(4, 8, 16, 32), counts=(32, 128, 512, 2048)):
        """Weight gradient on tile stacks: time per split factor and active-tile count; returns the table and the
        factor with the smallest total."""
        cap = tiles.shape[0]
        Cin, Cout = tiles.shape[3], dout.shape[3]
        ws = torch.empty((max(conv_backward_weights_workspace_bytes(tiles.dtype, cap, tiles.shape[1], tiles.shape[2], Cin, k, stride, Cout), 16),),
                         dtype=torch.uint8, device=tiles.device)
        dw = torch.empty((k, k, Cin, Cout), dtype=torch.float32, device=tiles.device)
        field = "wgrad_split_factor_1x1" if k == 1 else "wgrad_split_factor_3x3"
        table = {}
        for f in factors:
            row = []
            for n in counts:
                if n > cap:
                    break
                cnt = torch.tensor([n], dtype=torch.int32, device=tiles.device)
                row.append(self._timed(lambda: conv_on_tiles_backward_weights(tiles, dout, cnt, k, stride=stride, out=dw, workspace=ws),
                                       **{field: f}))
            table[f] = row
        best = min(table, key=lambda f: sum(table[f]))
        return {"counts": [n for n in counts if n <= cap], "ms": table, "best": best}
