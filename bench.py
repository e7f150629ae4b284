#!/usr/bin/env python3
"""Benchmark of the Winograd F(m x m, 3 x 3) hot path on one MI355X.

A step is one nova_winograd_conv2d call (input transform -> n*n channel contractions -> output
transform), inputs resident in HBM; the filter transform is done once outside the timed region.
Default workload, the headline: the VGG-16 conv3 shape (N=32, C=K=256, 56x56, F(8,3), fp16 storage,
fp32 accumulation, NOVA points); --workload selects the other single-layer configurations (the small
fp32 F(4,3) layer, the F(6,3) layer, the ResNet-style shapes at batch 256).
Prints ONE JSON line: effective TFLOP/s counted in direct-convolution FLOPs, the roofline figure
of the dominant kernel, per-stage figures, the fp16 error against the fp64 definition, and the
CPU oracle's direct convolution timed on the host cores on a bounded sample of the same tensors.
"""
import argparse
import json
import os
import sys
import time
from fractions import Fraction

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16 MFMA

TRAFFIC_TABLE = os.path.join(ROOT, "profiles", "hbm_traffic_table.txt")


def measured_traffic(version, workload, points, products, images_per_slab, stage):
    """HBM bytes per launch of one stage kernel as measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (scaled by what the same counters read for a plain copy; the commands are in the table's header).
    The table is keyed by the library version the counters were collected with: a figure taken with
    other kernels than the ones loaded now is not reported (None)."""
    try:
        with open(TRAFFIC_TABLE) as fh:
            for line in fh:
                cells = [c.strip() for c in line.split("|")]
                if len(cells) == 7 and not line.startswith("#") and \
                        cells[:6] == [version, workload, points, products, str(images_per_slab), stage]:
                    return int(cells[6])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="vgg_conv3_f83_fp16",
                    help="one of paper_2512_18453_amd.synth.LAYER_CONFIGS; the default is the headline workload")
    ap.add_argument("--points", default=None, help="standard | nova | classic_half (F(6,3)) | dyadic (F(4,3))")
    ap.add_argument("--images-per-slab", type=int, default=0, help="0 = library default")
    ap.add_argument("--m-f16", action="store_true", help="keep the products M in fp16 (NOVA_FLAG_M_F16)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg (profiling runs)")
    ap.add_argument("--headline-only", action="store_true",
                    help="skip the graph-replay and binary16-products legs (profiling runs: one configuration per kernel)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy, the yardstick for rocprofv3's FETCH_SIZE / WRITE_SIZE")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the path would shard by batch, with no "
                 "exchange between GPUs) -- use --gpus 1")

    import numpy as np
    import torch

    from paper_2512_18453_amd import nova, synth

    cfg = synth.LAYER_CONFIGS[args.workload]
    if args.points is None:
        args.points = synth.DEFAULT_POINTS.get(args.workload, "nova")
    N, C, K, H, W, m = cfg["N"], cfg["C"], cfg["K"], cfg["H"], cfg["W"], cfg["m"]
    n = m + 2
    tdtype = torch.float16 if cfg["dtype"] == "f16" else torch.float32
    dt = nova.NOVA_F16 if cfg["dtype"] == "f16" else nova.NOVA_F32
    es = 2 if cfg["dtype"] == "f16" else 4
    flags = nova.NOVA_FLAG_M_F16 if args.m_f16 else 0
    m_es = 2 if (args.m_f16 and dt == nova.NOVA_F16) else 4
    points = synth.point_set(args.points, m)

    x, w = synth.make_layer(N, C, K, H, W, seed=cfg["seed"], dtype=cfg["dtype"], x_dist=cfg["x_dist"])
    dev = "cuda:0"
    xd, wd = torch.from_numpy(x).to(dev), torch.from_numpy(w).to(dev)
    t = nova.nova_make_transforms(points, m, 3)
    U = nova.nova_filter_transform(t, wd)
    ws_bytes = nova.nova_conv2d_workspace_bytes(N, C, H, W, K, m, dt, flags, args.images_per_slab)
    # the slabs nova_winograd_conv2d cuts the batch into with this workspace: as many images as fit (V and M of a
    # slab, or V alone where contraction and output transform run as one kernel), then slabs of equal size
    path = nova.nova_conv2d_path(t, C, H, W, K, dt, flags)
    fused = path == nova.NOVA_PATH_FUSED_OUTPUT      # contraction and output transform are one kernel, no M
    if fused:
        fits = next(s for s in range(N, 0, -1) if nova.nova_input_bytes(s, C, H, W, m, dt) <= ws_bytes)
    else:
        fits = next(s for s in range(N, 0, -1)
                    if nova.nova_conv2d_workspace_bytes(N, C, H, W, K, m, dt, flags, s) <= ws_bytes)
    n_slabs = -(-N // fits)
    slab_imgs = -(-N // n_slabs)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    y = torch.empty((N, K, H, W), dtype=tdtype, device=dev)

    def step():
        nova.nova_winograd_conv2d(t, xd, U, K, y=y, flags=flags, workspace=ws)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(args.steps):
        step()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = ev0.elapsed_time(ev1) / args.steps
    ms_per_step = max(ms_per_step, wall_ms) if wall_ms > 0 else ms_per_step
    direct_flop = 2.0 * N * K * C * H * W * 9
    value = direct_flop / (ms_per_step * 1e-3) / 1e12

    # ---- per-stage timing inside the pipeline, same launch configuration (one launch = one slab):
    # the three stage entry points are called in sequence, as nova_winograd_conv2d does, with an
    # event between them, so each kernel sees the cache state it sees in the timed region above
    tiles = -(-H // m) * (-(-W // m))
    T_slab = slab_imgs * tiles
    cb, kb = -(-C // 32) * 32, -(-K // 32) * 32
    V = torch.empty(nova.nova_input_bytes(slab_imgs, C, H, W, m, dt) // es, dtype=tdtype, device=dev)
    M = torch.empty(nova.nova_product_bytes(slab_imgs, K, H, W, m, dt, flags) // m_es,
                    dtype=torch.float16 if m_es == 2 else torch.float32, device=dev)
    slabs = [(i, min(slab_imgs, N - i)) for i in range(0, N, slab_imgs)]
    reps = max(10, args.steps)
    marks = []
    for rep in range(reps + 3):
        for (i0, cnt) in slabs:
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev[0].record()
            nova.nova_input_transform(t, xd[i0:i0 + cnt], V=V)
            ev[1].record()
            if fused:
                nova.nova_contract_output_fused(t, U, V, cnt, C, H, W, K, flags, y=y[i0:i0 + cnt])
                ev[2].record()
            else:
                nova.nova_contract(t, U, V, cnt, C, H, W, K, flags, M=M)
                ev[2].record()
                nova.nova_output_transform(t, M, cnt, K, H, W, tdtype, flags, y=y[i0:i0 + cnt])
            ev[3].record()
            if rep >= 3 and cnt == slab_imgs:
                marks.append(ev)
    torch.cuda.synchronize()
    s_in, s_c, s_out = [sum(e[i].elapsed_time(e[i + 1]) for e in marks) / len(marks) * 1e-3 for i in range(3)]
    x_b = slab_imgs * C * H * W * es
    y_b = slab_imgs * K * H * W * es
    V_b = n * n * T_slab * cb * es
    M_b = n * n * T_slab * kb * m_es
    U_b = n * n * kb * cb * es
    gemm_flop = 2.0 * n * n * T_slab * C * K
    stages = {"input_transform": dict(us=s_in * 1e6, bytes=x_b + V_b, gbs=(x_b + V_b) / s_in / 1e9)}
    if fused:
        stages["contract_output_fused"] = dict(us=s_c * 1e6, bytes=U_b + V_b + y_b, gbs=(U_b + V_b + y_b) / s_c / 1e9,
                                               tflops=gemm_flop / s_c / 1e12,
                                               mfma_frac=gemm_flop / s_c / 1e12 / MFMA_F16_PEAK_TFLOPS)
    else:
        stages["contract"] = dict(us=s_c * 1e6, bytes=U_b + V_b + M_b, gbs=(U_b + V_b + M_b) / s_c / 1e9,
                                  tflops=gemm_flop / s_c / 1e12, mfma_frac=gemm_flop / s_c / 1e12 / MFMA_F16_PEAK_TFLOPS)
        stages["output_transform"] = dict(us=s_out * 1e6, bytes=M_b + y_b, gbs=(M_b + y_b) / s_out / 1e9)
    for st in stages.values():
        st["hbm_frac"] = st["gbs"] / HBM_PEAK_GBS
    # context for the fractions above: what a plain device copy moving the same number of bytes (half read, half
    # written) takes on this machine; the 8 TB/s peak stays the roofline's peak
    if not args.headline_only:
        most = max(st["bytes"] for st in stages.values()) // 2
        c_src = torch.empty(most, dtype=torch.uint8, device=dev)
        c_dst = torch.empty(most, dtype=torch.uint8, device=dev)
        for st in stages.values():
            half = st["bytes"] // 2
            for _ in range(5):
                c_dst[:half].copy_(c_src[:half])
            c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            c0.record()
            for _ in range(20):
                c_dst[:half].copy_(c_src[:half])
            c1.record()
            torch.cuda.synchronize()
            st["copy_same_bytes_us"] = c0.elapsed_time(c1) / 20 * 1e3
        del c_src, c_dst
    dominant = max(stages, key=lambda k: stages[k]["us"])
    dom = stages[dominant]
    traffic = measured_traffic(nova.nova_version(), args.workload, args.points, "f16" if m_es == 2 else "f32",
                               int(slab_imgs), dominant)
    roofline = dict(kernel=dominant, bound="hbm", achieved=round(dom["gbs"], 1), peak=HBM_PEAK_GBS, unit="GB/s",
                    frac=round(dom["gbs"] / HBM_PEAK_GBS, 4), traffic=traffic,
                    launch_us=round(dom["us"], 2), algorithmic_bytes=dom["bytes"])
    # the contraction against both of its bounds: the matrix cores' peak, and what its operand and
    # result bytes allow at the HBM peak (the binding one at these shapes)
    c_st = stages["contract_output_fused" if fused else "contract"]
    c_floor_us = max(gemm_flop / (MFMA_F16_PEAK_TFLOPS * 1e12), c_st["bytes"] / (HBM_PEAK_GBS * 1e9)) * 1e6
    c_st["attainable_us"] = c_floor_us
    c_st["frac_of_attainable"] = c_floor_us / c_st["us"]
    c_st["binding"] = "hbm" if c_st["bytes"] / (HBM_PEAK_GBS * 1e9) > gemm_flop / (MFMA_F16_PEAK_TFLOPS * 1e12) else "mfma"

    # ---- the same K steps replayed from a HIP graph (10 steps per graph): what the step costs once the
    # host-side launch work is taken out; reported beside the headline, never as `value`
    graph_info = None
    try:
        if args.headline_only:
            raise StopIteration
        per_graph = 10
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(per_graph):
                step()
        replays = max(1, args.steps // per_graph)
        graph.replay()
        torch.cuda.synchronize()
        g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g0.record()
        for _ in range(replays):
            graph.replay()
        g1.record()
        torch.cuda.synchronize()
        g_ms = g0.elapsed_time(g1) / (replays * per_graph)
        graph_info = dict(steps_per_graph=per_graph, ms_per_step=round(g_ms, 4),
                          value=round(direct_flop / (g_ms * 1e-3) / 1e12, 2), unit="TFLOP/s")
        del graph
    except StopIteration:
        pass
    except RuntimeError as exc:                        # capture refused: report, do not hide
        graph_info = dict(error=str(exc)[:200])

    # ---- the same step with the products M kept in binary16 (half the M traffic, one more rounding):
    # reported beside the headline, never as `value`
    variant = None
    if dt == nova.NOVA_F16 and not args.m_f16 and not args.headline_only:
        vflags = flags | nova.NOVA_FLAG_M_F16
        ws2 = torch.empty(nova.nova_conv2d_workspace_bytes(N, C, H, W, K, m, dt, vflags, args.images_per_slab),
                          dtype=torch.uint8, device=dev)
        y2 = torch.empty_like(y)
        for _ in range(args.warmup):
            nova.nova_winograd_conv2d(t, xd, U, K, y=y2, flags=vflags, workspace=ws2)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.steps):
            nova.nova_winograd_conv2d(t, xd, U, K, y=y2, flags=vflags, workspace=ws2)
        e1.record()
        torch.cuda.synchronize()
        v_ms = e0.elapsed_time(e1) / args.steps
        variant = dict(flags="NOVA_FLAG_M_F16", ms_per_step=round(v_ms, 4),
                       value=round(direct_flop / (v_ms * 1e-3) / 1e12, 2), unit="TFLOP/s")
        del ws2

    if args.copy_calibration:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- accuracy on sampled images and the CPU oracle leg
    result_extra = {}
    cpu_baseline = None
    if not args.no_cpu:
        from oracle import conv as oracle_conv
        torch.cuda.synchronize()
        w64 = w.astype(np.float64)
        tic = time.perf_counter()
        ref1 = oracle_conv.direct_conv2d(x[:1].astype(np.float64), w64)
        per_img = time.perf_counter() - tic
        n_cpu = int(min(N, max(1, round(12.0 / max(per_img, 1e-3)))))
        tic = time.perf_counter()
        ref = oracle_conv.direct_conv2d(x[:n_cpu].astype(np.float64), w64)
        cpu_s = time.perf_counter() - tic
        cpu_flop = 2.0 * n_cpu * K * C * H * W * 9
        cpu_baseline = dict(value=round(cpu_flop / cpu_s / 1e12, 6), unit="TFLOP/s", cores=oracle_conv.threads(),
                            kind="oracle", sample=f"fp64 direct conv of images 0..{n_cpu - 1} of {N} "
                            f"({cpu_flop / 1e9:.1f} GFLOP in {cpu_s:.2f} s, OpenMP)")
        # the oracle's fp64 Winograd beside it, on as many images as take a few seconds (same FLOP count:
        # the direct convolution's, so the two figures compare as times)
        n_w = max(1, min(n_cpu, 2))
        tic = time.perf_counter()
        wino = oracle_conv.winograd_conv2d_f64(x[:n_w].astype(np.float64), w64, [Fraction(a, b) for a, b in points], m)
        w_s = time.perf_counter() - tic
        if w_s < 2.0 and n_w < n_cpu:
            n_w = int(min(n_cpu, max(n_w, round(n_w * 4.0 / max(w_s, 1e-3)))))
            tic = time.perf_counter()
            wino = oracle_conv.winograd_conv2d_f64(x[:n_w].astype(np.float64), w64, [Fraction(a, b) for a, b in points], m)
            w_s = time.perf_counter() - tic
        cpu_baseline["winograd_f64"] = dict(
            value=round(2.0 * n_w * K * C * H * W * 9 / w_s / 1e12, 6), unit="TFLOP/s (direct-conv FLOPs)",
            sample=f"fp64 Winograd F({m},3) of images 0..{n_w - 1} in {w_s:.2f} s",
            rel_l2_vs_direct=float(np.linalg.norm(wino - ref[:n_w]) / np.linalg.norm(ref[:n_w])))
        del wino
        got = y[:n_cpu].cpu().numpy().astype(np.float64)
        fin = np.isfinite(got)
        result_extra["nonfinite_frac"] = float(1.0 - fin.mean())
        if variant is not None:
            got2 = y2[:n_cpu].cpu().numpy().astype(np.float64)
            if np.isfinite(got2).all():
                variant["rel_l2_vs_fp64"] = float(np.linalg.norm(got2 - ref) / np.linalg.norm(ref))
        if fin.all():
            result_extra["rel_l2_vs_fp64"] = float(np.linalg.norm(got - ref) / np.linalg.norm(ref))
            emu = oracle_conv.winograd_conv2d_emulated(x[:2].astype(np.float64), w64,
                                                       [Fraction(a, b) for a, b in points], m,
                                                       storage=16 if dt == nova.NOVA_F16 else 32,
                                                       m_storage=16 if m_es == 2 else 32)
            result_extra["rel_l2_vs_emulation"] = float(np.linalg.norm(got[:2] - emu) / np.linalg.norm(emu))
        del ref1

    out = {
        "metric": "effective TFLOP/s (direct-conv FLOPs), F(8,3) VGG-16 3x3 layer" if args.workload == "vgg_conv3_f83_fp16"
                  else f"effective TFLOP/s (direct-conv FLOPs), {args.workload}",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16" if dt == nova.NOVA_F16 else "f32", "data": "synthetic",
        "config": {"workload": f"{args.workload}: 3x3 conv N={N} C={C} K={K} H=W={H}, F({m},3), {args.points} points",
                   "points": args.points, "images_per_slab": int(slab_imgs), "slabs": int(n_slabs),
                   "products_dtype": "f16" if m_es == 2 else "f32",
                   "kernels": ["stages", "few_channels", "fused_output"][path]},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "stages": {k: {kk: (round(vv, 4) if isinstance(vv, float) else vv) for kk, vv in v.items()}
                   for k, v in stages.items()},
    }
    if graph_info is not None:
        out["graph_replay"] = graph_info
    if variant is not None:
        out["variant_products_f16"] = variant
    out.update(result_extra)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
