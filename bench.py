#!/usr/bin/env python3
"""Benchmark of the tiled sparse convolution hot path on one MI355X.

Workload (headline): one sparse 3x3 convolution, stride 1, SAME padding, bf16 NHWC with fp32
accumulation, N=1, H=800, W=704, 64 -> 64 channels, 16x16 output blocks with a one-pixel halo,
synthetic road-band mask calibrated to 10 % active blocks.  One step = the whole path on inputs
already resident in HBM: reduce_mask (mask -> index list, count stays on the device) followed by
the fused gather -> MFMA convolution -> scatter kernel.  Steps are replayed from one HIP graph
so that host launch overhead does not hide the GPU time; the eager (Python-driven) figure is
reported next to it.

Prints ONE JSON line.  Extra keys: per-kernel times, the four-call (unfused) path, the same
path with every block active (the build's own dense baseline), MIOpen's dense convolution, the
density sweep 5/10/20/40 %, the roofline of the dominant kernel and the CPU oracle's time.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

H, W, C, K, BO, KS = 800, 704, 64, 64, 16, 3
TILE_FLOPS = 2 * BO * BO * KS * KS * C * K                       # 18 874 368 per active tile
TILE_BYTES = ((BO + 2) ** 2 * C + BO * BO * K) * 2               # read tile + write block, bf16
PEAK_BF16_TFLOPS = 2500.0                                        # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--density", type=float, default=0.10, help="target active-block fraction of the headline run")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip sweep, dense and MIOpen comparisons")
    ap.add_argument("--eager-kernel-timing", action="store_true",
                    help="time single kernels with eager launches instead of graph replays (use under rocprofv3, whose "
                         "per-node instrumentation inflates kernels replayed from a graph)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 256 MiB device copy: a known-size reference for scaling HBM byte counters")
    ap.add_argument("--stage", type=int, default=-1, help="stages workload: only this entry of its shape list")
    ap.add_argument("--conv-only", action="store_true",
                    help="stages workload: only the fused convolution with every block active (for counter runs)")
    ap.add_argument("--workload", default="cfg2", choices=["cfg2", "cfg3", "cfg4", "cfg5", "stages", "backward", "tune"],
                    help="cfg2 (default) is the headline single 3x3 conv; cfg3/4/5 are the residual-unit workloads; "
                         "stages = single 3x3 convs, stride 1 and 2, at the backbone's other stage shapes; "
                         "backward = the gradients of cfg2's convolution on its tile stacks; "
                         "tune = the compute-tile choices inside the kernels, each alternative forced, with the measured crossovers")
    return ap.parse_args()


# ---------------------------------------------------------------------------------------------------
# residual-unit workloads (configs 3-5): sparse bottleneck 256 -> 64 -> 64 -> 256, bf16
# ---------------------------------------------------------------------------------------------------
def unit_flops(bo, C=256, Cm=64):
    """FLOPs the method performs per active block, halo recompute of the first 1x1 included."""
    sub = (bo // 16) ** 2 if bo % 16 == 0 else None
    t = 18 if sub else bo + 2
    o = 16 if sub else bo
    per = 2 * (t * t * C * Cm + o * o * 9 * Cm * Cm + o * o * Cm * C)
    return per * (sub or 1)


def unit_bytes(bo, C=256):
    """Algorithmic HBM bytes per active block: input tile once, output block once (bf16)."""
    return ((bo + 2) ** 2 + bo * bo) * C * 2


def run_units(args):
    import numpy as np
    import torch
    import paper_1801_02108_amd as sb
    from paper_1801_02108_amd import inputs as gen
    from paper_1801_02108_amd.autotune import device_ms
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    cfg = args.workload
    C, Cm = 256, 64
    if cfg == "cfg3":
        N, H, W, bos, targets, n_units, kind = 1, 400, 352, [16], [0.10, 0.30, 1.0], 1, "road"
    elif cfg == "cfg4":
        N, H, W, bos, n_units, kind = 4, 800, 704, [8, 16, 32], 1, "blob"
        targets = [0.01, 0.02, 0.05, 0.10, 0.20, 0.30, 0.50, 0.70, 0.85, 1.0]
    else:
        N, H, W, bos, targets, n_units, kind = 8, 800, 704, [16], [0.15, 1.0], 8, "lowres"
    r = gen.rng_for(int(cfg[-1]))
    tg = torch.Generator(device=dev)
    tg.manual_seed(gen.BASE_SEED + int(cfg[-1]))
    x = torch.randn((N, H, W, C), generator=tg, device=dev, dtype=torch.float32).to(torch.bfloat16)
    bufs = [x.clone(), x.clone()]
    units = []
    for _ in range(n_units):
        w1, b1, w2, b2, w3, b3 = gen.bottleneck_weights(r, C, Cm, "bf16")
        units.append((sb.pack_weights(torch.from_numpy(w1).to(torch.bfloat16).to(dev)), torch.from_numpy(b1).to(dev),
                      sb.pack_weights(torch.from_numpy(w2).to(torch.bfloat16).to(dev)), torch.from_numpy(b2).to(dev),
                      sb.pack_weights(torch.from_numpy(w3).to(torch.bfloat16).to(dev)), torch.from_numpy(b3).to(dev)))
    if kind == "road":
        fields = gen.road_band_fields(r, H, W, 3)
    elif kind == "blob":
        field = gen.smooth_noise(r, N, H, W, 24.0)
    else:
        logits_np = gen.smooth_noise(r, N, H // 8, W // 8, 2.0)      # low-passed so 15 % of blocks is reachable
        logits = torch.from_numpy(logits_np).to(dev)

    rows = []
    for bo in bos:
        g_in, g_out, _, _ = sb.geometry(H, W, 3, 1, bo)
        total = N * g_in.bcount_h * g_in.bcount_w
        idx = torch.empty((total, 3), dtype=torch.int32, device=dev)
        cnt = torch.empty((1,), dtype=torch.int32, device=dev)
        ws = torch.empty((sb.workspace_bytes(N, g_in),), dtype=torch.uint8, device=dev)

        def count_active(m_np):
            sb.reduce_mask(torch.from_numpy(m_np).to(dev), g_in, sb.POOL_AVG, 0.0, idx, cnt, ws)
            return sb.read_count(cnt, total)

        dense_ms = None
        for target in sorted(targets, reverse=True):
            thr_t = None
            if target >= 1.0:
                m_np = np.ones((N, H, W), dtype=np.uint8)
            elif kind == "road":
                m_np = gen.calibrate(lambda s_: np.repeat(gen.road_band_mask(fields, s_), N, axis=0), count_active, total,
                                     target, 0.0, 12.0)[0]
            elif kind == "blob":
                m_np = gen.calibrate(lambda t_: gen.blob_mask(field, t_), count_active, total, target, -4.0, 4.0,
                                     increasing=False)[0]
            else:
                m_np, thr_t, _ = gen.calibrate(lambda t_: gen.lowres_mask(logits_np, t_), count_active, total, target, -4.0,
                                               4.0, increasing=False)
            m_d = torch.from_numpy(m_np).to(dev)
            n = count_active(m_np)

            # dynamic mask, two routes to the same block list: (a) threshold the low-resolution logits, upsample x8 by
            # pixel repetition (torch: the mask source), reduce the full-resolution mask; (b) reduce the logit map itself:
            # max-pool over the coarse cells each block window touches, against the same threshold (threshold >= 0)
            coarse = thr_t is not None and thr_t >= 0.0
            g_coarse = sb.coarse_geometry(g_in, 8) if coarse else None

            def step(lowres=False):
                if thr_t is not None and lowres:
                    sb.reduce_mask(logits, g_coarse, sb.POOL_MAX, thr_t, idx, cnt, ws)
                else:
                    if thr_t is not None:
                        md = (logits > thr_t).to(torch.uint8).repeat_interleave(8, 1).repeat_interleave(8, 2)
                    else:
                        md = m_d
                    sb.reduce_mask(md, g_in, sb.POOL_AVG, 0.0, idx, cnt, ws)
                a, b = bufs
                for u in units:
                    sb.sparse_bottleneck(a, idx, cnt, g_in, g_out, u, b)
                    a, b = b, a

            ms_coarse = None
            if coarse:
                step(False)
                ref_idx, ref_n = idx.clone(), sb.read_count(cnt, total)
                step(True)
                same = ref_n == sb.read_count(cnt, total) and bool((idx[:ref_n] == ref_idx[:ref_n]).all().item())
                if not same:
                    raise RuntimeError("coarse-map reduce_mask disagrees with the upsampled mask")
                bufs[1].copy_(bufs[0])

            for _ in range(3):
                step()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            iters = max(3, min(50, int(2000 / max(n * n_units, 1)) + 3))
            e0.record()
            for _ in range(iters):
                step()
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / iters
            if coarse:
                for _ in range(2):
                    step(True)
                e0.record()
                for _ in range(iters):
                    step(True)
                e1.record()
                torch.cuda.synchronize()
                ms_coarse = e0.elapsed_time(e1) / iters
            # the unit kernel alone, and in pre-activation form (ReLU(scale * x + shift) in front of conv1): device time
            # from graph replays (eager launches of a 10 us kernel would time the host), eager under the profiler
            u0 = units[0]
            pre = (torch.ones(C, device=dev), torch.zeros(C, device=dev))

            def unit_ms(fn):
                if not args.eager_kernel_timing:
                    return device_ms(fn, reps=5 if n * n_units > 2000 else 10, replays=5)
                for _ in range(2):
                    fn()
                e0.record()
                for _ in range(iters):
                    fn()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / iters
            k_ms = unit_ms(lambda: sb.sparse_bottleneck(bufs[0], idx, cnt, g_in, g_out, u0, bufs[1]))
            kp_ms = unit_ms(lambda: sb.sparse_bottleneck(bufs[0], idx, cnt, g_in, g_out, u0, bufs[1], pre=pre))
            if n * n_units <= 2000 and thr_t is None and not args.eager_kernel_timing:
                ms = device_ms(step)          # small problems: the step from graph replays too
            if target >= 1.0:
                dense_ms = ms
            rows.append({"block": bo, "target": target, "active_blocks": n, "total_blocks": total,
                         "step_ms": round(ms, 5), "unit_kernel_ms": round(k_ms, 5), "preact_unit_kernel_ms": round(kp_ms, 5),
                         "unit_tflops": round(unit_flops(bo) * n / k_ms / 1e9, 2),
                         "unit_hbm_GBps_algorithmic": round(unit_bytes(bo) * n / k_ms / 1e6, 1),
                         "speedup_vs_own_dense": round(dense_ms / ms, 3), "ideal_speedup": round(total / max(n, 1), 2)})
            if ms_coarse is not None:      # same block list from the 1/8-resolution logit map without the upsampled mask
                rows[-1]["step_ms_mask_reduced_at_logit_resolution"] = round(ms_coarse, 5)
            bufs[1].copy_(bufs[0])
    # MIOpen dense unit through torch, external baseline only (3 convs + ReLUs + add)
    miopen_ms = None
    try:
        xt = x.permute(0, 3, 1, 2)
        rr = gen.rng_for(int(cfg[-1]), 7)
        tw = [torch.from_numpy(w).to(torch.bfloat16).to(dev).permute(3, 2, 0, 1).contiguous(memory_format=torch.channels_last)
              for w in gen.bottleneck_weights(rr, C, Cm, "bf16")[0::2]]
        F = torch.nn.functional

        def dense_unit():
            t = F.relu(F.conv2d(xt, tw[0]))
            t = F.relu(F.conv2d(t, tw[1], padding=1))
            return xt + F.conv2d(t, tw[2])
        for _ in range(3):
            dense_unit()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dense_unit()
        e1.record()
        torch.cuda.synchronize()
        miopen_ms = e0.elapsed_time(e1) / 5 * n_units
    except Exception as e:                                         # pragma: no cover
        sys.stderr.write("MIOpen dense unit failed: %s\n" % e)
    head = rows[-1] if cfg != "cfg4" else [r_ for r_ in rows if r_["block"] == 16 and r_["target"] == 0.10][0]
    if cfg == "cfg5":
        head = [r_ for r_ in rows if r_["target"] == 0.15][0]
    elif cfg == "cfg3":
        head = [r_ for r_ in rows if r_["target"] == 0.10][0]
    traffic = None
    if cfg == "cfg5":
        try:
            traffic = json.load(open(os.path.join(ROOT, "profiles", "traffic.json"))).get("bottleneck16_kernel_fused/cfg5_15pct")
        except Exception:
            traffic = None
    # crossover against the dense path (all blocks active), per block size: the smallest density of the sweep at
    # which the sparse step is no faster than the dense one; null when it is faster at every density below 100 %
    crossover = {}
    for bo in bos:
        rb = [r_ for r_ in rows if r_["block"] == bo]
        dense_b = [r_["step_ms"] for r_ in rb if r_["target"] >= 1.0][0]
        slow = sorted(r_["target"] for r_ in rb if r_["target"] < 1.0 and r_["step_ms"] >= dense_b)
        crossover[str(bo)] = slow[0] if slow else None
    out = {"metric": "sparse_residual_unit_ms", "value": head["step_ms"], "unit": "ms", "n_gpus": 1,
           "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["step_ms"], "higher_is_better": False,
           "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
           "config": {"workload": "%s: %d sparse bottleneck unit(s) 256->64->64->256 bf16, N=%d H=%d W=%d, %s mask" % (
               cfg, n_units, N, H, W, kind), "headline_row": head},
           "rows": rows, "crossover": crossover, "miopen_dense_units_ms": None if miopen_ms is None else round(miopen_ms, 4),
           "roofline": {"bound": "hbm", "kernel": "bottleneck16_kernel<bf16,256,fused>",
                        "achieved": head["unit_hbm_GBps_algorithmic"], "peak": PEAK_HBM_GBS, "unit": "GB/s",
                        "frac": round(head["unit_hbm_GBps_algorithmic"] / PEAK_HBM_GBS, 4), "traffic": traffic}}
    print(json.dumps(out))


# ---------------------------------------------------------------------------------------------------
# single sparse 3x3 convolutions at the other stage shapes of the backbone (Sec. 4), stride 1 and 2
# ---------------------------------------------------------------------------------------------------
def run_stages(args):
    import numpy as np
    import torch
    import paper_1801_02108_amd as sb
    from paper_1801_02108_amd import inputs as gen
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    shapes = [(800, 704, 64, 96, 2, 16), (400, 352, 96, 96, 1, 16), (400, 352, 96, 192, 2, 16),
              (200, 176, 192, 192, 1, 16), (200, 176, 192, 256, 2, 16), (100, 88, 256, 384, 2, 8)]
    if args.stage >= 0:
        shapes = [shapes[args.stage]]
    F = torch.nn.functional
    rows = []
    for (H, W, Cin, Cout, s, bo) in shapes:
        r = gen.rng_for(6, H + Cin + s)
        g_in, g_out, Ho, Wo = sb.geometry(H, W, 3, s, bo)
        total = g_out.bcount_h * g_out.bcount_w
        x = torch.randn((1, H, W, Cin), device=dev).to(torch.bfloat16)
        y = torch.zeros((1, Ho, Wo, Cout), device=dev, dtype=torch.bfloat16)
        wp = sb.pack_weights(torch.from_numpy(gen.conv_weights(r, 3, 3, Cin, Cout, "bf16")).to(torch.bfloat16).to(dev))
        wp_t = sb.pack_weights_transposed(torch.from_numpy(gen.conv_weights(r, 3, 3, Cin, Cout, "bf16")).to(torch.bfloat16).to(dev))
        bias = torch.from_numpy(gen.bias_vector(r, Cout)).to(dev)
        idx = torch.empty((total, 3), dtype=torch.int32, device=dev)
        cnt = torch.empty((1,), dtype=torch.int32, device=dev)
        ws = torch.empty((sb.workspace_bytes(1, g_out),), dtype=torch.uint8, device=dev)
        fields = gen.road_band_fields(r, Ho, Wo, 3)

        def count_active(m_np):
            sb.reduce_mask(torch.from_numpy(m_np).to(dev), g_out, sb.POOL_AVG, 0.0, idx, cnt, ws)
            return sb.read_count(cnt, total)

        xt = x.permute(0, 3, 1, 2)
        wt = torch.randn((Cout, Cin, 3, 3), device=dev).to(torch.bfloat16).contiguous(memory_format=torch.channels_last)
        for _ in range(3):
            F.conv2d(xt, wt, stride=s, padding=1)
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(20):
            F.conv2d(xt, wt, stride=s, padding=1)
        e1.record()
        torch.cuda.synchronize()
        miopen_ms = e0.elapsed_time(e1) / 20
        dense_ms = None
        for target in ((1.0,) if args.conv_only else (1.0, 0.3, 0.1)):
            if target >= 1.0:
                m_np = np.ones((1, Ho, Wo), dtype=np.uint8)
            else:
                m_np = gen.calibrate(lambda sc: gen.road_band_mask(fields, sc), count_active, total, target, 0.0, 12.0, tol=0.03)[0]
            m_d = torch.from_numpy(m_np).to(dev)
            n = count_active(m_np)

            def step():
                sb.reduce_mask(m_d, g_out, sb.POOL_AVG, 0.0, idx, cnt, ws)
                sb.sparse_conv(x, idx, cnt, g_in, g_out, wp, bias, y, stride=s, relu=True)
            # device time per call: HIP events around replays of a graph of 20 back-to-back calls (eager launches of
            # kernels this short would measure the host's launch rate)
            def device_ms(fn, reps=20, replays=5):
                if args.eager_kernel_timing:                       # under rocprofv3: no graphs
                    for _ in range(3):
                        fn()
                    torch.cuda.synchronize()
                    e0.record()
                    for _ in range(50):
                        fn()
                    e1.record()
                    torch.cuda.synchronize()
                    return e0.elapsed_time(e1) / 50
                side = torch.cuda.Stream()
                side.wait_stream(torch.cuda.current_stream())
                with torch.cuda.stream(side):
                    fn()
                torch.cuda.current_stream().wait_stream(side)
                torch.cuda.synchronize()
                gr = torch.cuda.CUDAGraph()
                with torch.cuda.graph(gr):
                    for _ in range(reps):
                        fn()
                gr.replay()
                torch.cuda.synchronize()
                e0.record()
                for _ in range(replays):
                    gr.replay()
                e1.record()
                torch.cuda.synchronize()
                return e0.elapsed_time(e1) / (reps * replays)
            ms = device_ms(step)
            k_ms = device_ms(lambda: sb.sparse_conv(x, idx, cnt, g_in, g_out, wp, bias, y, stride=s, relu=True))
            if args.conv_only:
                rows.append({"H": H, "W": W, "Cin": Cin, "Cout": Cout, "stride": s, "block": bo, "target": target,
                             "active_blocks": n, "total_blocks": total, "step_ms": round(ms, 5), "conv_kernel_ms": round(k_ms, 5),
                             "conv_tflops": round(2.0 * n * bo * bo * 9 * Cin * Cout / k_ms / 1e9, 2)})
                continue
            # the two gradients of the same convolution on its tile stacks (unfused: tiles in, tiles out)
            th = g_in.bsize_h
            xt_tiles = torch.randn((max(n, 1), th, th, Cin), device=dev).to(torch.bfloat16)
            gt_tiles = torch.randn((max(n, 1), bo, bo, Cout), device=dev).to(torch.bfloat16)
            din_tiles = torch.empty_like(xt_tiles)
            dw = torch.empty((3, 3, Cin, Cout), dtype=torch.float32, device=dev)
            ws_d = torch.empty((max(sb.conv_backward_data_workspace_bytes(torch.bfloat16, max(n, 1), th, th, 3, 3, s, Cout), 16),),
                               dtype=torch.uint8, device=dev)
            ws_w = torch.empty((max(sb.conv_backward_weights_workspace_bytes(torch.bfloat16, max(n, 1), th, th, Cin, 3, s, Cout), 16),),
                               dtype=torch.uint8, device=dev)
            dgrad_ms = device_ms(lambda: sb.conv_on_tiles_backward_data(gt_tiles, cnt, wp_t, th, th, stride=s, out=din_tiles,
                                                                        workspace=ws_d))
            wgrad_ms = device_ms(lambda: sb.conv_on_tiles_backward_weights(xt_tiles, gt_tiles, cnt, 3, stride=s, out=dw,
                                                                           workspace=ws_w))
            # the 1x1 layers of a residual unit of the stage's width on the same tiles: Cin -> Cin / 4 on the input
            # tile, Cout / 4 -> Cout on the output block
            pw_ms = []
            for (pc, pk, side) in ((Cin, Cin // 4, th), (Cout // 4, Cout, bo)):
                pw_x = torch.randn((max(n, 1), side, side, pc), device=dev).to(torch.bfloat16)
                pw_y = torch.empty((max(n, 1), side, side, pk), device=dev, dtype=torch.bfloat16)
                pw_w = sb.pack_weights(torch.from_numpy(gen.conv_weights(r, 1, 1, pc, pk, "bf16")).to(torch.bfloat16).to(dev))
                pw_ms.append(device_ms(lambda: sb.conv_on_tiles(pw_x, cnt, pw_w, None, relu=True, out=pw_y)))
            # residual units of the stage (Sec. 4): the downsampling unit Cin -> Cout with a strided 3x3 and a projected
            # shortcut at stride 2 (sequence of calls on tile stacks), and the stage's stride-1 unit Cout / (Cout / 4)
            # with the identity shortcut on the same block grid (one kernel up to 256 / 64)
            Cm = Cout // 4

            def unit_weights(ci, cm, co, with_proj):
                ww = (gen.conv_weights(r, 1, 1, ci, cm, "bf16"), gen.bias_vector(r, cm), gen.conv_weights(r, 3, 3, cm, cm, "bf16"),
                      gen.bias_vector(r, cm), gen.conv_weights(r, 1, 1, cm, co, "bf16", scale=0.5), gen.bias_vector(r, co))
                dw_ = tuple(sb.pack_weights(torch.from_numpy(a).to(torch.bfloat16).to(dev)) if a.ndim == 4 else torch.from_numpy(a).to(dev)
                            for a in ww)
                pr = None
                if with_proj:
                    pr = (sb.pack_weights(torch.from_numpy(gen.conv_weights(r, 1, 1, ci, co, "bf16")).to(torch.bfloat16).to(dev)),
                          torch.from_numpy(gen.bias_vector(r, co)).to(dev))
                return dw_, pr
            unit_row = {}
            if s == 2:
                dwu, pru = unit_weights(Cin, Cm, Cout, True)
                wsu = torch.empty((max(sb.lib().sbnet_sparse_unit_workspace_bytes(sb.BF16, total, g_in, g_out, Cin, Cm, Cout), 256),),
                                  dtype=torch.uint8, device=dev)
                u_ms = device_ms(lambda: sb.sparse_unit(x, idx, cnt, g_in, g_out, dwu, y, stride=2, shortcut=pru, workspace=wsu))
                u_bytes = n * (g_in.bsize_h * g_in.bsize_w * Cin + bo * bo * Cout) * 2
                unit_row.update({"down_unit_ms": round(u_ms, 5), "down_unit_algorithmic_GBps": round(u_bytes / u_ms / 1e6, 1)})
            g1_in, g1_out, _, _ = sb.geometry(Ho, Wo, 3, 1, bo)
            dw1, _ = unit_weights(Cout, Cm, Cout, False)
            x1 = torch.randn((1, Ho, Wo, Cout), device=dev).to(torch.bfloat16)
            y1 = x1.clone()
            ws1 = torch.empty((max(sb.lib().sbnet_sparse_unit_workspace_bytes(sb.BF16, total, g1_in, g1_out, Cout, Cm, Cout), 256),),
                              dtype=torch.uint8, device=dev)
            u1_ms = device_ms(lambda: sb.sparse_unit(x1, idx, cnt, g1_in, g1_out, dw1, y1, stride=1, shortcut=None, workspace=ws1))
            u1_bytes = n * ((bo + 2) ** 2 + bo * bo) * Cout * 2
            unit_row.update({"unit_ms": round(u1_ms, 5), "unit_algorithmic_GBps": round(u1_bytes / u1_ms / 1e6, 1),
                             "unit_width": "%d/%d" % (Cout, Cm), "unit_path": "one kernel" if Cout <= 256 else "sequence of calls"})
            if target >= 1.0:
                dense_ms = ms
            rows.append({"H": H, "W": W, "Cin": Cin, "Cout": Cout, "stride": s, "block": bo, "target": target, **unit_row,
                         "pointwise_reduce_ms": round(pw_ms[0], 5), "pointwise_expand_ms": round(pw_ms[1], 5),
                         "backward_data_ms": round(dgrad_ms, 5), "backward_weights_ms": round(wgrad_ms, 5),
                         "backward_weights_tflops": round(2.0 * n * bo * bo * 9 * Cin * Cout / wgrad_ms / 1e9, 2),
                         "active_blocks": n, "total_blocks": total, "step_ms": round(ms, 5), "conv_kernel_ms": round(k_ms, 5),
                         "conv_tflops": round(2.0 * n * bo * bo * 9 * Cin * Cout / k_ms / 1e9, 2),
                         "speedup_vs_own_dense": round(dense_ms / ms, 3), "miopen_dense_ms": round(miopen_ms, 5)})
    head = ([r_ for r_ in rows if r_["H"] == 400 and r_["stride"] == 2 and r_["target"] == 0.3] or rows)[0]
    print(json.dumps({"metric": "sparse_conv_stage_shapes_ms", "value": head["step_ms"], "unit": "ms", "n_gpus": 1,
                      "steps": 50, "warmup": 3, "ms_per_step": head["step_ms"], "higher_is_better": False, "scaling": "weak",
                      "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "stages: single sparse 3x3 conv + ReLU, bf16, N=1, stride 1 and 2, road-band masks; "
                                             "HIP graph replays, step = reduce_mask + fused conv", "headline_row": head},
                      "rows": rows}))


def run_backward(args):
    """Gradients of cfg2's tile convolution (18x18x64 tiles -> 16x16x64, bf16) at 5 ... 100 % of its 2200 blocks:
    data gradient (frame + forward kernel), weight gradient (matrix-core kernel + sum of the partial results) and,
    beside them, the forward call on the same tiles."""
    import torch
    import paper_1801_02108_amd as sb
    from paper_1801_02108_amd import inputs as gen
    from paper_1801_02108_amd.autotune import device_ms
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    C = K = 64
    BO, TH, TOTAL = 16, 18, 2200
    r = gen.rng_for(2, 77)
    w = torch.from_numpy(gen.conv_weights(r, 3, 3, C, K, "bf16")).to(torch.bfloat16).to(dev)
    wp, wp_t = sb.pack_weights(w), sb.pack_weights_transposed(w)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def eager_ms(fn, reps=50):
        for _ in range(3):
            fn()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps
    tk = eager_ms if args.eager_kernel_timing else device_ms
    rows = []
    for frac in (0.05, 0.10, 0.20, 0.40, 1.0):
        n = max(1, int(round(frac * TOTAL)))
        x = torch.from_numpy(gen.activations(r, (n, TH, TH, C), "bf16")).to(torch.bfloat16).to(dev)
        g = torch.from_numpy(gen.activations(r, (n, BO, BO, K), "bf16")).to(torch.bfloat16).to(dev)
        cnt = torch.tensor([n], dtype=torch.int32, device=dev)
        y = torch.empty_like(g)
        din = torch.empty_like(x)
        dw = torch.empty((3, 3, C, K), dtype=torch.float32, device=dev)
        ws_d = torch.empty((sb.conv_backward_data_workspace_bytes(torch.bfloat16, n, TH, TH, 3, 3, 1, K),), dtype=torch.uint8, device=dev)
        ws_w = torch.empty((sb.conv_backward_weights_workspace_bytes(torch.bfloat16, n, TH, TH, C, 3, 1, K),), dtype=torch.uint8, device=dev)
        t_f = tk(lambda: sb.conv_on_tiles(x, cnt, wp, None, out=y))
        t_d = tk(lambda: sb.conv_on_tiles_backward_data(g, cnt, wp_t, TH, TH, out=din, workspace=ws_d))
        t_w = tk(lambda: sb.conv_on_tiles_backward_weights(x, g, cnt, 3, out=dw, workspace=ws_w))
        flops = 2.0 * n * BO * BO * 9 * C * K
        rows.append({"active_blocks": n, "forward_ms": round(t_f, 5), "forward_tflops": round(flops / t_f / 1e9, 2),
                     "backward_data_ms": round(t_d, 5),
                     "backward_data_tflops": round(flops * (TH * TH) / (BO * BO) / t_d / 1e9, 2),
                     "backward_weights_ms": round(t_w, 5), "backward_weights_tflops": round(flops / t_w / 1e9, 2)})
    # the residual unit 256 -> 64 -> 64 -> 256 composed from single calls, activations kept: forward (three
    # convolutions) and backward (three weight, three bias and three data gradients, two ReLU masks) on tile stacks
    unit_rows = []
    Cu, Cm = 256, 64
    w1, b1, w2, b2, w3, b3 = gen.bottleneck_weights(r, Cu, Cm, "bf16")
    tod = lambda a: torch.from_numpy(a).to(torch.bfloat16).to(dev)
    p1, p2, p3 = sb.pack_weights(tod(w1)), sb.pack_weights(tod(w2)), sb.pack_weights(tod(w3))
    q1, q2, q3 = sb.pack_weights_transposed(tod(w1)), sb.pack_weights_transposed(tod(w2)), sb.pack_weights_transposed(tod(w3))
    fb1, fb2, fb3 = (torch.from_numpy(b).to(dev) for b in (b1, b2, b3))
    for n in (330, 2200):
        xt = torch.from_numpy(gen.activations(r, (n, TH, TH, Cu), "bf16")).to(torch.bfloat16).to(dev)
        d3 = torch.from_numpy(gen.activations(r, (n, BO, BO, Cu), "bf16")).to(torch.bfloat16).to(dev)
        cnt = torch.tensor([n], dtype=torch.int32, device=dev)
        t1 = torch.empty((n, TH, TH, Cm), dtype=torch.bfloat16, device=dev)
        t2 = torch.empty((n, BO, BO, Cm), dtype=torch.bfloat16, device=dev)
        t3 = torch.empty((n, BO, BO, Cu), dtype=torch.bfloat16, device=dev)
        d2, d1, dxt = torch.empty_like(t2), torch.empty_like(t1), torch.empty_like(xt)
        dw1 = torch.empty((1, 1, Cu, Cm), dtype=torch.float32, device=dev)
        dw2 = torch.empty((3, 3, Cm, Cm), dtype=torch.float32, device=dev)
        dw3 = torch.empty((1, 1, Cm, Cu), dtype=torch.float32, device=dev)
        ws = torch.empty((64 << 20,), dtype=torch.uint8, device=dev)       # covers every workspace below

        def fwd():
            sb.conv_on_tiles(xt, cnt, p1, fb1, relu=True, out=t1)
            sb.conv_on_tiles(t1, cnt, p2, fb2, relu=True, out=t2)
            sb.conv_on_tiles(t2, cnt, p3, fb3, out=t3)

        ws_b = torch.empty((sb.lib().sbnet_bottleneck_backward_workspace_bytes(sb.BF16, n, TH, TH, Cu, Cm),), dtype=torch.uint8,
                           device=dev)

        def bwd():
            sb.bottleneck_backward_on_tiles(xt, t1, t2, d3, cnt, (q1, q2, q3), workspace=ws_b)
        fwd()
        unit_rows.append({"active_blocks": n, "unit_forward_composed_ms": round(tk(fwd), 5),
                          "unit_backward_composed_ms": round(tk(bwd), 5)})
    head = rows[1]
    print(json.dumps({"metric": "conv_on_tiles_backward_ms_at_10pct_active_blocks",
                      "value": round(head["backward_data_ms"] + head["backward_weights_ms"], 5), "unit": "ms", "n_gpus": 1,
                      "steps": 50, "warmup": 3, "ms_per_step": round(head["backward_data_ms"] + head["backward_weights_ms"], 5),
                      "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "backward: data and weight gradients of cfg2's 3x3 tile convolution "
                                             "(18x18x64 -> 16x16x64 tiles, bf16), value = both at 220 tiles",
                                 "timing": "eager launches" if args.eager_kernel_timing else "HIP graph replays"},
                      "rows": rows, "residual_unit_rows": unit_rows}))


def run_tune(args):
    """Compute-tile choices inside the kernels (the second half of Sec. 4's search): each alternative forced through
    sbnet_tuning over a range of active counts; reports the measured crossover beside the default in force."""
    import torch
    import paper_1801_02108_amd as sb
    from paper_1801_02108_amd import autotune as at
    from paper_1801_02108_amd import inputs as gen
    dev = torch.device("cuda:0")
    torch.cuda.set_device(0)
    r = gen.rng_for(9)
    kt = at.KernelChoiceTuner()
    out = {"defaults": sb.get_tuning(), "unit_subtiles": [], "conv3_items": [], "wgrad_splits": []}
    pk = lambda a: sb.pack_weights(torch.from_numpy(a).to(torch.bfloat16).to(dev)) if a.ndim == 4 else torch.from_numpy(a).to(dev)
    for (H, W, C, Cm) in ((400, 352, 256, 64), (400, 352, 96, 24), (200, 176, 192, 48)):
        x = torch.randn((1, H, W, C), device=dev).to(torch.bfloat16)
        ws = tuple(pk(a) for a in gen.bottleneck_weights(r, C, Cm, "bf16"))
        res = kt.unit_subtiles(x, ws, block=16, counts=(8, 16, 32, 48, 64, 80, 96, 112, 128, 144, 160, 192, 224, 256, 320, 384, 512))
        res.update({"shape": "%dx%dx%d/%d" % (H, W, C, Cm), "ms16": [round(v, 5) for v in res["ms16"]], "ms8": [round(v, 5) for v in res["ms8"]]})
        out["unit_subtiles"].append(res)
    # (strided layers with 96 / 256 ... output channels run 128-pixel items only and have no such choice)
    # the last entry has 18 x 18 blocks (324 output pixels, as in a data gradient on 16 x 16 blocks): its two items are
    # 384 and 256 pixels, one or two per block, and a 256-pixel item is taken as 6/5 of the ratio below
    for (H, W, Cin, Cout, s_, bo_) in ((400, 352, 96, 96, 1, 16), (400, 352, 96, 192, 2, 16), (200, 176, 192, 192, 1, 16),
                                       (396, 360, 64, 64, 1, 18)):
        x = torch.randn((1, H, W, Cin), device=dev).to(torch.bfloat16)
        w = torch.from_numpy(gen.conv_weights(r, 3, 3, Cin, Cout, "bf16")).to(torch.bfloat16).to(dev)
        res = kt.conv3_items(x, w, stride=s_, block=bo_, counts=(8, 16, 32, 64, 96, 128, 192, 256, 320, 384, 512))
        # what the default cost ratio would have picked at each count (rounds of work over 256 CUs)
        ngroups = (Cout + 63) // 64
        cost = out["defaults"]["conv3_small_item_cost_eighths"]
        if bo_ == 18:
            cost = (cost * 6 + 2) // 5
        picks = []
        for n in res["counts"]:
            rb, rs = (n * 1 * ngroups + 255) // 256, (n * 2 * ngroups + 255) // 256
            picks.append("larger" if rb * 8 <= rs * cost else "smaller")
        res["faster"] = ["larger" if f == "256" else "smaller" for f in res["faster"]]
        res.update({"shape": "%dx%dx%d->%d s%d, block %d" % (H, W, Cin, Cout, s_, bo_), "items": "384 / 256" if bo_ == 18 else "256 / 128",
                    "ms_larger": [round(v, 5) for v in res.pop("ms256")], "ms_smaller": [round(v, 5) for v in res.pop("ms128")],
                    "default_picks": picks})
        out["conv3_items"].append(res)
    for (k, th, oh, Cin, Cout) in ((3, 18, 16, 64, 64), (1, 18, 18, 256, 64), (3, 18, 16, 96, 96)):
        t = torch.randn((2200, th, th, Cin), device=dev).to(torch.bfloat16)
        g = torch.randn((2200, oh, oh, Cout), device=dev).to(torch.bfloat16)
        res = kt.wgrad_splits(t, g, k, factors=(2, 4, 8, 16, 32), counts=(30, 110, 220, 880, 2200))
        res.update({"shape": "%dx%d %d->%d on %dx%d tiles" % (k, k, Cin, Cout, th, th),
                    "ms": {str(f): [round(v, 5) for v in row] for f, row in res["ms"].items()}})
        out["wgrad_splits"].append(res)
    for res in out["unit_subtiles"]:      # what the rule in force picks at each count, beside what was faster
        cost = out["defaults"]["unit_small_item_cost_eighths"]
        res["default_picks"] = ["16" if -(-n // 256) * 8 <= -(-n * 4 // 256) * cost else "8" for n in res["counts"]]
    print(json.dumps({"metric": "kernel_choice_crossovers", "value": out["unit_subtiles"][0]["cost_eighths"], "unit": "eighths",
                      "n_gpus": 1, "steps": 50, "warmup": 1, "ms_per_step": None, "higher_is_better": False, "scaling": "weak",
                      "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "tune: compute-tile choices inside the kernels, each alternative forced; HIP graph replays"},
                      **out}))


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (--gpus 1); the path shards by blocks or samples "
                 "without collectives, each GPU running this same single-GPU path on its share")
    import numpy as np
    if not args.no_cpu_baseline:                                  # compile / load the CPU oracle before any GPU call
        import oracle as orc
        orc.build()
        orc._c()
    import torch
    import paper_1801_02108_amd as sb
    from paper_1801_02108_amd import inputs as gen

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    sb.lib()                                                      # fail loudly if the HIP library is missing
    if args.calibration_copy:
        src = torch.zeros(256 << 20, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.workload == "backward":
        return run_backward(args)
    if args.workload == "tune":
        return run_tune(args)
    if args.workload == "stages":
        return run_stages(args)
    if args.workload != "cfg2":
        return run_units(args)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    # ------------------------------------------------------------------ inputs (seeded, synthetic)
    r = gen.rng_for(2)
    g_in, g_out, Ho, Wo = sb.geometry(H, W, KS, 1, BO)
    total_blocks = g_in.bcount_h * g_in.bcount_w
    x_np = gen.activations(r, (1, H, W, C), "bf16")
    w_np = gen.conv_weights(r, KS, KS, C, K, "bf16")
    b_np = gen.bias_vector(r, K)
    x = torch.from_numpy(x_np).to(torch.bfloat16).to(dev)
    wp = sb.pack_weights(torch.from_numpy(w_np).to(torch.bfloat16).to(dev))
    bias = torch.from_numpy(b_np).to(dev)
    y = torch.zeros((1, Ho, Wo, K), dtype=torch.bfloat16, device=dev)
    fields = gen.road_band_fields(r, H, W, 3)

    idx = torch.empty((total_blocks, 3), dtype=torch.int32, device=dev)
    cnt = torch.empty((1,), dtype=torch.int32, device=dev)
    ws = torch.empty((sb.workspace_bytes(1, g_in),), dtype=torch.uint8, device=dev)

    def count_active(mask_np):
        sb.reduce_mask(torch.from_numpy(mask_np).to(dev), g_in, sb.POOL_AVG, 0.0, idx, cnt, ws)
        return sb.read_count(cnt, total_blocks)

    def mask_for(target):
        if target >= 1.0:
            m = np.ones((1, H, W), dtype=np.uint8)
            return m, 1.0
        m, _, frac = gen.calibrate(lambda s: gen.road_band_mask(fields, s), count_active, total_blocks, target, 0.0, 12.0)
        return m, frac

    flags = torch.empty((sb.lib().sbnet_block_flags_bytes(1, g_in),), dtype=torch.uint8, device=dev)

    def step_fused(mask_d):
        """the whole path, mask -> y (and the index list, for later consumers): two launches"""
        sb.block_flags(mask_d, g_in, sb.POOL_AVG, 0.0, flags)
        sb.sparse_conv_from_flags(flags, x, g_in, g_out, wp, bias, y, idx, cnt)

    def step_three_launches(mask_d):
        """the same through the four-call interface's first and fused last call: reduce_mask (2 launches) + sparse_conv"""
        sb.reduce_mask(mask_d, g_in, sb.POOL_AVG, 0.0, idx, cnt, ws)
        sb.sparse_conv(x, idx, cnt, g_in, g_out, wp, bias, y)

    tiles_buf = [None, None]

    def step_unfused(mask_d):
        sb.reduce_mask(mask_d, g_in, sb.POOL_AVG, 0.0, idx, cnt, ws)
        sb.sparse_gather(x, idx, cnt, g_in, tiles_buf[0])
        sb.conv_on_tiles(tiles_buf[0], cnt, wp, bias, out=tiles_buf[1])
        sb.sparse_scatter(tiles_buf[1], idx, cnt, g_out, y)

    def graph_of(fn, reps=1):
        """HIP graph holding `reps` back-to-back calls of fn() (captured on a side stream)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()                                                   # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for _ in range(reps):
                fn()
        return g

    def time_kernel(fn, reps=20, replays=10):
        """Average device milliseconds of one call of fn(): HIP events on the launch stream around
        `replays` replays of a graph of `reps` calls, so host launch cost is not in the figure."""
        g = graph_of(fn, reps)
        g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * replays)

    def time_events(fn, iters, warm=5):
        """average milliseconds per eager call of fn() (HIP events; includes host launch cost)"""
        for _ in range(warm):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(iters):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / iters

    def time_steps(fn, steps, warmup):
        """wall-clock ms per call over exactly `steps` calls bracketed by device synchronisation"""
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    INNER = 20      # steps captured per HIP graph: fixed, whatever --steps / --warmup say

    def time_step_graph(fn, steps, warmup):
        """Device milliseconds per step: HIP events on the launch stream around whole replays of a graph of INNER
        back-to-back steps.  At least 50 replays are timed (a step lasts ~10 us; fewer would time the clock), more
        if `steps` asks for more; warm-up runs as whole replays too.  Returns (ms per step, steps timed, wall-clock
        ms per step over the same region between two device synchronisations)."""
        g = graph_of(fn, INNER)
        replays = max(50, -(-steps // INNER))
        for _ in range(max(2, -(-warmup // INNER))):
            g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record()
        for _ in range(replays):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        return e0.elapsed_time(e1) / (replays * INNER), replays * INNER, wall / (replays * INNER)

    # ------------------------------------------------------------------ headline: 10 % active blocks
    mask_np, frac = mask_for(args.density)
    mask_d = torch.from_numpy(mask_np).to(dev)
    nact = count_active(mask_np)
    pix_density = float(mask_np.mean())

    eager_ms = time_steps(lambda: step_fused(mask_d), max(args.steps, 100), max(args.warmup, 10))
    graph_ok, steps_timed, wall_ms = True, args.steps, None
    try:
        if args.eager_kernel_timing:
            raise RuntimeError("eager timing requested")
        ms_per_step, steps_timed, wall_ms = time_step_graph(lambda: step_fused(mask_d), args.steps, args.warmup)
        single_graph_ms = time_steps(graph_of(lambda: step_fused(mask_d), 1).replay, 100, 10)
    except Exception as e:                                         # pragma: no cover
        graph_ok = False
        sys.stderr.write("graph capture failed (%s); reporting eager timing\n" % e)
        ms_per_step = single_graph_ms = eager_ms

    # per-kernel device time: graphs of 20 back-to-back launches of one entry point, HIP events
    tk = time_kernel if (graph_ok and not args.eager_kernel_timing) else (lambda fn: time_events(fn, 200))
    sb.block_flags(mask_d, g_in, sb.POOL_AVG, 0.0, flags)
    conv_ms = tk(lambda: sb.sparse_conv_from_flags(flags, x, g_in, g_out, wp, bias, y, idx, cnt))
    flags_ms = tk(lambda: sb.block_flags(mask_d, g_in, sb.POOL_AVG, 0.0, flags))
    conv_idx_ms = tk(lambda: sb.sparse_conv(x, idx, cnt, g_in, g_out, wp, bias, y))
    reduce_ms = tk(lambda: sb.reduce_mask(mask_d, g_in, sb.POOL_AVG, 0.0, idx, cnt, ws))
    three_ms = time_step_graph(lambda: step_three_launches(mask_d), args.steps, args.warmup)[0] if graph_ok else None
    count_active(mask_np)                                          # leave idx/cnt consistent

    flops = TILE_FLOPS * nact
    achieved_tflops = flops / (conv_ms * 1e-3) / 1e12
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("conv16_kernel_fused/cfg2_10pct")
        except Exception:
            traffic = None

    out = {
        "metric": "sparse_conv_ms_at_10pct_active_blocks",
        "value": round(ms_per_step, 6),
        "unit": "ms",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 6),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": "cfg2: sparse 3x3 conv bf16 NHWC, N=1 H=800 W=704 C=64->64, block 16x16 + halo 1, "
                               "road-band mask", "target_active_block_fraction": args.density,
                   "active_blocks": nact, "total_blocks": total_blocks, "active_block_fraction": round(frac, 4),
                   "mask_pixel_density": round(pix_density, 4),
                   "step": "block_flags (mask -> one flag per block) + sparse_conv_from_flags (compaction in the prologue, "
                           "gather / MFMA conv / scatter; also writes the index list and count)",
                   "timing": ("HIP events around %d steps replayed from HIP graphs of %d steps each (always at least "
                              "50 replays, warm-up in whole replays)" % (steps_timed, INNER)) if graph_ok
                   else "eager launches, wall clock between device syncs", "steps_timed": steps_timed},
        "ms_per_step_wall_clock_same_region": None if wall_ms is None else round(wall_ms, 6),
        "ms_per_step_eager": round(eager_ms, 6),
        "ms_per_step_one_graph_per_step": round(single_graph_ms, 6),
        "kernel_ms": {"block_flags(rm_pool_blocks)": round(flags_ms, 6),
                      "sparse_conv_from_flags(conv16_kernel, flag-fed)": round(conv_ms, 6)},
        "three_launch_path": {"ms_per_step": None if three_ms is None else round(three_ms, 6),
                              "reduce_mask(2 kernels)_ms": round(reduce_ms, 6),
                              "sparse_conv(conv16_kernel, index-fed)_ms": round(conv_idx_ms, 6)},
        "effective_tflops": round(flops / (ms_per_step * 1e-3) / 1e12, 3),
        # AI of the fused kernel = 18 874 368 FLOP / 74 240 B = 254 FLOP/B, below the ridge 2500 / 8 = 312: HBM-bound
        "roofline": {"bound": "hbm", "kernel": "conv16_kernel<bf16,64,fused,flag-fed>",
                     "achieved": round(TILE_BYTES * nact / (conv_ms * 1e-3) / 1e9, 2), "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": round(TILE_BYTES * nact / (conv_ms * 1e-3) / 1e9 / PEAK_HBM_GBS, 5),
                     "traffic": traffic, "algorithmic_bytes_per_launch": TILE_BYTES * nact,
                     "mfma_tflops": round(achieved_tflops, 3), "mfma_frac": round(achieved_tflops / PEAK_BF16_TFLOPS, 5)},
    }

    # ------------------------------------------------------------------ extras
    if not args.no_extras:
        sweep = []
        dense_ms = None
        wp_t = sb.pack_weights_transposed(torch.from_numpy(w_np).to(torch.bfloat16).to(dev))
        wp_f8 = sb.pack_weights_f8(sb.quantize_f8(torch.from_numpy(w_np).to(torch.bfloat16).to(dev), 64.0))
        for target in (0.05, 0.10, 0.20, 0.40, 1.0):
            m_np, fr = mask_for(target)
            m_d = torch.from_numpy(m_np).to(dev)
            n = count_active(m_np)
            t_step = time_step_graph(lambda: step_fused(m_d), args.steps, args.warmup)[0] if graph_ok else \
                time_steps(lambda: step_fused(m_d), 100, 10)
            sb.block_flags(m_d, g_in, sb.POOL_AVG, 0.0, flags)
            t_conv = tk(lambda: sb.sparse_conv_from_flags(flags, x, g_in, g_out, wp, bias, y, idx, cnt))
            tiles_buf[0] = torch.empty((n, BO + 2, BO + 2, C), dtype=torch.bfloat16, device=dev)
            tiles_buf[1] = torch.empty((n, BO, BO, K), dtype=torch.bfloat16, device=dev)
            idx_small = idx[:n]
            t_gather = tk(lambda: sb.sparse_gather(x, idx_small, cnt, g_in, tiles_buf[0]))
            t_tconv = tk(lambda: sb.conv_on_tiles(tiles_buf[0], cnt, wp, bias, out=tiles_buf[1]))
            t_scatter = tk(lambda: sb.sparse_scatter(tiles_buf[1], idx_small, cnt, g_out, y))
            # the same tile convolution with FP8 (E4M3) tiles and weights, BF16 results
            tiles_f8 = sb.quantize_f8(tiles_buf[0], 16.0)
            t_quant = tk(lambda: sb.quantize_f8(tiles_buf[0], 16.0, out=tiles_f8))
            t_f8 = tk(lambda: sb.conv_on_tiles_f8(tiles_f8, cnt, wp_f8, bias, out_scale=1.0 / (16.0 * 64.0), out=tiles_buf[1]))
            # the same copies with the transpose to channel-major tiles fused in (Sec. 3.4)
            chw_in = torch.empty((n, C, BO + 2, BO + 2), dtype=torch.bfloat16, device=dev)
            chw_out = torch.empty((n, K, BO, BO), dtype=torch.bfloat16, device=dev)
            t_gather_chw = tk(lambda: sb.sparse_gather_chw(x, idx_small, cnt, g_in, chw_in))
            t_scatter_chw = tk(lambda: sb.sparse_scatter_chw(chw_out, idx_small, cnt, g_out, y))
            # gradient of the gather: overlapping tile gradients summed onto dx (end of Sec. 3.3)
            dxg = torch.zeros_like(x)
            gb_ws = torch.empty((sb.lib().sbnet_gather_backward_workspace_bytes(1, g_in),), dtype=torch.uint8, device=dev)
            t_gb = tk(lambda: sb.sparse_gather_backward(tiles_buf[0], idx_small, cnt, g_in, dxg, gb_ws))
            # batch-norm statistics over the active blocks of the output (Sec. 3.3)
            bn_ws = torch.empty((sb.lib().sbnet_bn_stats_workspace_bytes(n, K),), dtype=torch.uint8, device=dev)
            t_bn = tk(lambda: sb.sparse_bn_stats(y, idx_small, cnt, g_out, bn_ws))
            # gradients of the tile convolution: with respect to its input tiles and to its weights
            dgrad_ws = torch.empty((max(sb.conv_backward_data_workspace_bytes(torch.bfloat16, n, BO + 2, BO + 2, 3, 3, 1, K), 16),),
                                   dtype=torch.uint8, device=dev)
            wgrad_ws = torch.empty((max(sb.conv_backward_weights_workspace_bytes(torch.bfloat16, n, BO + 2, BO + 2, C, 3, 1, K), 16),),
                                   dtype=torch.uint8, device=dev)
            din_buf = torch.empty_like(tiles_buf[0])
            dw_buf = torch.empty((3, 3, C, K), dtype=torch.float32, device=dev)
            t_dgrad = tk(lambda: sb.conv_on_tiles_backward_data(tiles_buf[1], cnt, wp_t, BO + 2, BO + 2, out=din_buf,
                                                                workspace=dgrad_ws))
            t_wgrad = tk(lambda: sb.conv_on_tiles_backward_weights(tiles_buf[0], tiles_buf[1], cnt, 3, out=dw_buf,
                                                                   workspace=wgrad_ws))
            # the data gradient contracts over the (BO+2)^2 input pixels of the framed tile
            dgrad_flops = 2 * 9 * C * K * (BO + 2) ** 2
            # normalisation over the active blocks of the output, forward (in place) and training-mode backward
            bn_mean, bn_var = sb.sparse_bn_stats(y, idx_small, cnt, g_out, bn_ws)
            bn_gamma = torch.ones((K,), dtype=torch.float32, device=dev)
            bn_beta = torch.zeros((K,), dtype=torch.float32, device=dev)
            y_bn, dy_bn, dx_bn = torch.empty_like(y), torch.ones_like(y), torch.empty_like(y)
            bnb_ws = torch.empty((sb.lib().sbnet_bn_backward_workspace_bytes(n, K),), dtype=torch.uint8, device=dev)
            t_bna = tk(lambda: sb.sparse_bn_apply(y, idx_small, cnt, g_out, bn_mean, bn_var, bn_gamma, bn_beta, relu=True, y=y_bn))
            t_bnb = tk(lambda: sb.sparse_bn_backward(y, dy_bn, idx_small, cnt, g_out, bn_mean, bn_var, bn_gamma, bn_beta,
                                                     relu=True, dx=dx_bn, workspace=bnb_ws))
            tile_in_b = (BO + 2) ** 2 * C * 2
            tile_out_b = BO * BO * K * 2
            row = {"target": target, "active_blocks": n, "step_ms": round(t_step, 5), "fused_conv_ms": round(t_conv, 5),
                   "fused_conv_tflops": round(TILE_FLOPS * n / t_conv / 1e9, 2),
                   "gather_ms": round(t_gather, 5), "gather_GBps": round(2 * tile_in_b * n / t_gather / 1e6, 1),
                   "conv_on_tiles_ms": round(t_tconv, 5), "conv_on_tiles_tflops": round(TILE_FLOPS * n / t_tconv / 1e9, 2),
                   "quantize_f8_ms": round(t_quant, 5), "conv_on_tiles_f8_ms": round(t_f8, 5),
                   "conv_on_tiles_f8_tflops": round(TILE_FLOPS * n / t_f8 / 1e9, 2),
                   "scatter_ms": round(t_scatter, 5), "scatter_GBps": round(2 * tile_out_b * n / t_scatter / 1e6, 1),
                   "gather_chw_ms": round(t_gather_chw, 5), "gather_chw_GBps": round(2 * tile_in_b * n / t_gather_chw / 1e6, 1),
                   "scatter_chw_ms": round(t_scatter_chw, 5), "scatter_chw_GBps": round(2 * tile_out_b * n / t_scatter_chw / 1e6, 1),
                   "gather_backward_ms": round(t_gb, 5),
                   "gather_backward_GBps": round((tile_in_b + 2 * BO * BO * C * 2) * n / t_gb / 1e6, 1),
                   "bn_stats_ms": round(t_bn, 5), "bn_stats_GBps": round(tile_out_b * n / t_bn / 1e6, 1),
                   "bn_apply_ms": round(t_bna, 5), "bn_apply_GBps": round(2 * tile_out_b * n / t_bna / 1e6, 1),
                   "bn_backward_ms": round(t_bnb, 5), "bn_backward_GBps": round(5 * tile_out_b * n / t_bnb / 1e6, 1),
                   "conv_backward_data_ms": round(t_dgrad, 5),
                   "conv_backward_data_tflops": round(dgrad_flops * n / t_dgrad / 1e9, 2),
                   "conv_backward_weights_ms": round(t_wgrad, 5),
                   "conv_backward_weights_tflops": round(TILE_FLOPS * n / t_wgrad / 1e9, 2),
                   "unfused_sum_ms": round(t_gather + t_tconv + t_scatter, 5)}
            if target >= 1.0:
                dense_ms = t_step
            sweep.append(row)
            tiles_buf[0] = tiles_buf[1] = None
        for row in sweep:
            row["speedup_vs_own_dense"] = round(dense_ms / row["step_ms"], 3)
            row["ideal_speedup"] = round(total_blocks / max(row["active_blocks"], 1), 3)
        out["sweep"] = sweep
        # both rooflines of the fused kernel at every density of the sweep (its arithmetic intensity, 254 FLOP/B, sits
        # just under the ridge of 312, so the HBM fraction is the binding one; the matrix-core fraction is quoted
        # against the published dense bf16 peak)
        out["roofline_by_density"] = [
            {"target": row["target"], "active_blocks": row["active_blocks"], "kernel_ms": row["fused_conv_ms"],
             "hbm_GBps": round(TILE_BYTES * row["active_blocks"] / row["fused_conv_ms"] / 1e6, 1),
             "hbm_frac": round(TILE_BYTES * row["active_blocks"] / row["fused_conv_ms"] / 1e6 / PEAK_HBM_GBS, 4),
             "mfma_tflops": row["fused_conv_tflops"], "mfma_frac": round(row["fused_conv_tflops"] / PEAK_BF16_TFLOPS, 4)}
            for row in sweep]
        out["own_dense_ms"] = round(dense_ms, 5)
        out["speedup_vs_own_dense"] = round(dense_ms / ms_per_step, 3)
        # MIOpen dense convolution through torch (channels-last bf16), an external baseline only
        try:
            xt = x.permute(0, 3, 1, 2)                              # NCHW view of NHWC memory = channels_last
            wt = torch.from_numpy(w_np).to(torch.bfloat16).to(dev).permute(3, 2, 0, 1).contiguous(
                memory_format=torch.channels_last)
            fn = lambda: torch.nn.functional.conv2d(xt, wt, bias.to(torch.bfloat16), padding=1)
            miopen_ms = time_events(fn, 30, warm=5)
            out["miopen_dense_ms"] = round(miopen_ms, 5)
            out["speedup_vs_miopen_dense"] = round(miopen_ms / ms_per_step, 3)
        except Exception as e:                                     # pragma: no cover
            out["miopen_dense_ms"] = None
            sys.stderr.write("MIOpen dense baseline failed: %s\n" % e)
        count_active(mask_np)

    # ------------------------------------------------------------------ CPU oracle on the same workload
    if not args.no_cpu_baseline:
        og_in, og_out = orc.Geom(*g_in.astuple()), orc.Geom(*g_out.astuple())
        wg_in, wg_out, _, _ = orc.geometry(8, 8, 3, 1, 4)           # one tiny warm call: the timer starts on loaded code
        orc.sparse_conv_tiled(np.zeros((1, 8, 8, 2)), orc.reduce_mask(np.ones((1, 8, 8)), wg_in), wg_in, wg_out,
                              np.zeros((3, 3, 2, 2)), np.zeros(2), np.zeros((1, 8, 8, 2)))
        x64 = x_np.astype(np.float64)
        w64 = w_np.astype(np.float64)
        b64 = b_np.astype(np.float64)
        m64 = mask_np.astype(np.float64)
        y64 = np.zeros((1, Ho, Wo, K))
        t0 = time.perf_counter()
        oidx = orc.reduce_mask(m64, og_in, orc.POOL_AVG, 0.0)
        yref = orc.sparse_conv_tiled(x64, oidx, og_in, og_out, w64, b64, y64)
        cpu_s = time.perf_counter() - t0
        out["cpu_baseline"] = {"value": round(cpu_s * 1e3, 3), "unit": "ms", "cores": 1, "kind": "oracle",
                               "sample": "the whole step (reduce_mask, gather, valid conv, scatter) on all %d active "
                                         "tiles of the headline mask, fp64 direct loops, single thread; host has %d "
                                         "cores" % (len(oidx), os.cpu_count() or 0),
                               "gflops": round(TILE_FLOPS * len(oidx) / cpu_s / 1e9, 3)}
        # while the reference is here: check the GPU result of the headline step against it
        y.zero_()
        step_fused(mask_d)
        torch.cuda.synchronize()
        got = y.to(torch.float64).cpu().numpy()
        rms = float(np.sqrt(np.mean(yref * yref)))
        bad = np.abs(got - yref) > 2e-2 * np.abs(yref) + 2e-2 * rms
        out["parity_vs_oracle"] = {"elements": int(got.size), "out_of_tolerance": int(bad.sum()),
                                   "indices_equal": bool(nact == len(oidx) and np.array_equal(idx[:nact].cpu().numpy(), oidx))}

    print(json.dumps(out))


if __name__ == "__main__":
    main()
