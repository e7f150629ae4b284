#!/usr/bin/env python3
"""The 13-layer VGG-16 3x3 convolution stack through libnova on one GPU: random He-normal weights,
N(0,1) input, ReLU fused into every layer, 2x2 max-pool after layers 2, 4, 7, 10, 13 (fused into the
output transform, or as the separate kernel with --separate-pool).  Prints one JSON line with the
time of a forward pass and the per-layer times.

    python vgg16_stack.py [--m 8] [--batch 32] [--points nova] [--separate-pool] [--m-f16]

With --stages it times, layer by layer, the three stage entry points on the whole batch (no slabs, the
products in binary32 or binary16 as chosen) and prints one line per layer: time and algorithmic
bytes / time of the input transform (x + V), the contraction (U + V + M) and the output transform (M + y).
"""
import argparse
import json

import torch

import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2512_18453_amd import nova, synth  # noqa: E402


def stage_times(args):
    dev = "cuda:0"
    m, N, n = args.m, args.batch, args.m + 2
    t = nova.nova_make_transforms(synth.point_set(args.points, m), m, 3)
    flags = nova.NOVA_FLAG_RELU | (nova.NOVA_FLAG_M_F16 if args.m_f16 else 0)
    m_es = 2 if args.m_f16 else 4
    gen = torch.Generator(device=dev).manual_seed(16)
    H = args.size
    print(f"VGG-16 layers, batch {N}, F({m},3), {args.points} points, fp16, products {'f16' if args.m_f16 else 'f32'}: "
          "stage entry points on the whole batch")
    print("layer  C->K @ HxW        T      input us  TB/s | contract us  TB/s  MFMA TF | output us  TB/s")
    for idx, (cin, cout) in enumerate(synth.VGG16_LAYERS, start=1):
        x = torch.randn((N, cin, H, H), device=dev, generator=gen).abs().half()
        w = (torch.randn((cout, cin, 3, 3), device=dev, generator=gen) * (2.0 / (9.0 * cin)) ** 0.5).half()
        U = nova.nova_filter_transform(t, w)
        V = nova.nova_input_transform(t, x)
        M = nova.nova_contract(t, U, V, N, cin, H, H, cout, flags)
        y = nova.nova_output_transform(t, M, N, cout, H, H, torch.float16, flags)
        marks = []
        for rep in range(args.reps + 3):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(4)]
            ev[0].record(); nova.nova_input_transform(t, x, V=V)
            ev[1].record(); nova.nova_contract(t, U, V, N, cin, H, H, cout, flags, M=M)
            ev[2].record(); nova.nova_output_transform(t, M, N, cout, H, H, torch.float16, flags, y=y)
            ev[3].record()
            if rep >= 3:
                marks.append(ev)
        torch.cuda.synchronize()
        us = [sum(e[i].elapsed_time(e[i + 1]) for e in marks) / len(marks) * 1e3 for i in range(3)]
        T = N * (-(-H // m)) ** 2
        cp, kp = -(-cin // 32) * 32, -(-cout // 32) * 32
        xb, yb = x.numel() * 2, y.numel() * 2
        Vb, Ub, Mb = n * n * T * cp * 2, n * n * kp * cp * 2, n * n * T * kp * m_es
        print(f"L{idx:<2d}   {cin:3d}->{cout:3d} @ {H:3d}x{H:<3d} {T:6d}   {us[0]:8.1f} {(xb + Vb) / us[0] / 1e6:5.2f} | "
              f"{us[1]:9.1f} {(Ub + Vb + Mb) / us[1] / 1e6:5.2f} {2.0 * n * n * T * cin * cout / us[1] / 1e6:7.0f} | "
              f"{us[2]:8.1f} {(Mb + yb) / us[2] / 1e6:5.2f}", flush=True)
        del x, w, U, V, M, y
        if idx in synth.VGG16_POOL_AFTER:
            H //= 2


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, default=8, choices=(2, 4, 6, 8))
    ap.add_argument("--batch", type=int, default=32)
    ap.add_argument("--size", type=int, default=224)
    ap.add_argument("--points", default="nova")
    ap.add_argument("--separate-pool", action="store_true")
    ap.add_argument("--m-f16", action="store_true", help="keep the products M in binary16")
    ap.add_argument("--reps", type=int, default=10)
    ap.add_argument("--stages", action="store_true", help="per-layer times of the three stage entry points")
    args = ap.parse_args()
    if args.stages:
        return stage_times(args)

    dev = "cuda:0"
    m, N = args.m, args.batch
    t = nova.nova_make_transforms(synth.point_set(args.points, m), m, 3)
    base = nova.NOVA_FLAG_RELU | (nova.NOVA_FLAG_M_F16 if args.m_f16 else 0)
    gen = torch.Generator(device=dev).manual_seed(16)
    x0 = torch.randn((N, 3, args.size, args.size), device=dev, generator=gen).half()
    layers, H, ws_bytes = [], args.size, 0
    for idx, (cin, cout) in enumerate(synth.VGG16_LAYERS, start=1):
        w = (torch.randn((cout, cin, 3, 3), device=dev, generator=gen) * (2.0 / (9.0 * cin)) ** 0.5).half()
        pool = idx in synth.VGG16_POOL_AFTER
        full = torch.empty((N, cout, H, H), dtype=torch.float16, device=dev) if (not pool or args.separate_pool) else None
        pooled = torch.empty((N, cout, H // 2, H // 2), dtype=torch.float16, device=dev) if pool else None
        ws_bytes = max(ws_bytes, nova.nova_conv2d_workspace_bytes(N, cin, H, H, cout, m, nova.NOVA_F16, base))
        layers.append(dict(U=nova.nova_filter_transform(t, w), cout=cout, H=H, pool=pool, full=full, pooled=pooled,
                           flop=2.0 * N * cout * cin * H * H * 9))
        if pool:
            H //= 2
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    def forward(events=None):
        a = x0
        for i, L in enumerate(layers):
            if events is not None:
                events[i].record()
            if L["pool"] and not args.separate_pool:
                a = nova.nova_winograd_conv2d(t, a, L["U"], L["cout"], y=L["pooled"], flags=base | nova.NOVA_FLAG_POOL2,
                                              workspace=ws)
            else:
                a = nova.nova_winograd_conv2d(t, a, L["U"], L["cout"], y=L["full"], flags=base, workspace=ws)
                if L["pool"]:
                    a = nova.nova_relu_maxpool2x2(a, out=L["pooled"])
        if events is not None:
            events[len(layers)].record()
        return a

    for _ in range(3):
        forward()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(args.reps):
        forward()
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / args.reps
    per_layer = [0.0] * len(layers)
    for _ in range(args.reps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(layers) + 1)]
        out = forward(ev)
        torch.cuda.synchronize()
        for i in range(len(layers)):
            per_layer[i] += ev[i].elapsed_time(ev[i + 1]) / args.reps
    flop = sum(L["flop"] for L in layers)
    print(json.dumps({
        "workload": f"VGG-16 conv stack, batch {N}, {args.size}x{args.size}, F({m},3), {args.points} points, fp16",
        "pooling": "separate kernel" if args.separate_pool else "fused (NOVA_FLAG_POOL2)",
        "products_dtype": "f16" if args.m_f16 else "f32",
        "ms_per_forward": round(ms, 4), "effective_tflops": round(flop / (ms * 1e-3) / 1e12, 1),
        "finite_output": bool(torch.isfinite(out).all().item()),
        "layer_us": [round(v * 1e3, 1) for v in per_layer],
    }))


if __name__ == "__main__":
    main()
