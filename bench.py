#!/usr/bin/env python3
"""Benchmark of the SPARQ hot path on one MI355X.

One "step" is one pass of the fused path -- activation gather, vSPARQ/bSPARQ
trim, int8 contraction, offset correction and per-channel dequantisation to
fp32 -- over the workload's synthetic input, through the C ABI
(``sparq_conv_gemm`` with ``out``).  The default workload is the large GEMM of
the option sweep (M=65536, K=4608, N=512, 5opt, rounding, pairing on, 50 %
zeros), the shape the int8-MFMA target is stated on.  The standalone trim and
dequantisation kernels are timed next to it and reported in the same line.

Prints ONE JSON line on stdout.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, published
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg3",
                    help="cfg3 (default: explicit GEMM A[M,K]) | cfg3-conv (same M,K,N as a 3x3x512 conv) | "
                         "cfg0 | cfg1 | cfg2 | cfg4 | cfg4-2bit")
    ap.add_argument("--mask", type=lambda s: int(s, 0), default=None, help="cfg3 only: shift mask override")
    ap.add_argument("--round", type=int, default=None, help="cfg3 only: rounding override")
    ap.add_argument("--pair", type=int, default=None, help="cfg3 only: pairing override")
    ap.add_argument("--zf", type=float, default=None, help="cfg3 only: zero fraction override")
    ap.add_argument("--rows", type=int, default=65536, help="cfg3 only: M")
    ap.add_argument("--batch", type=int, default=None, help="cfg1/2/4: batch override")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-layer", action="store_true", help="print a per-layer table on stderr")
    return ap.parse_args()


def build_workload(args):
    import sparq_synth as S
    from dataclasses import replace
    wl = args.workload
    if wl in ("cfg3", "cfg3-conv"):
        layer = S.config3_layer(args.rows)
        if wl == "cfg3-conv":
            # the same GEMM seen as a convolution: 3x3, 512 -> 512 channels, 32x32 pixels, pad 1
            layer = replace(layer, name="conv3x3_512_512_32x32", B=args.rows // 1024, H=32, W=32, C=512, KH=3, KW=3,
                            pad=(1, 1))
        mode = layer.mode
        if args.mask is not None:
            mode = replace(mode, shift_mask=args.mask)
        if args.round is not None:
            mode = replace(mode, round_nearest=args.round)
        if args.pair is not None:
            mode = replace(mode, pair=args.pair)
        layer = replace(layer, mode=mode, zf=args.zf if args.zf is not None else layer.zf)
        form = "explicit A[M,K]" if wl == "cfg3" else f"implicit 3x3 conv B={layer.B} 32x32x512"
        name = f"config3: GEMM M={layer.M} K={layer.K} N={layer.N} ({form}), {mode.label}, zf={layer.zf}"
        return 3, [layer], name
    if wl == "cfg0":
        return 0, S.config0(), "config0: 3x3 conv 56x56x64->64, batch 1"
    if wl == "cfg1":
        b = args.batch or 32
        return 1, S.config1(b), f"config1: ResNet-18 conv layers, batch {b}"
    if wl == "cfg2":
        b = args.batch or 256
        return 2, S.config2(b), f"config2: ResNet-50 conv stack, batch {b}"
    if wl in ("cfg4", "cfg4-2bit"):
        b = args.batch or 128
        mode = S.Mode(2, S.OPT7_2B, 1, 1) if wl.endswith("2bit") else None
        return 4, S.config4(b, mode), f"config4: Inception-v3-shaped convs, batch {b}" + (", 2-bit 7opt" if mode else "")
    raise SystemExit(f"unknown workload {wl}")


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path shards over output rows without communication, see DESIGN.md).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2105_11010_amd as sq
    import sparq_synth as S

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg_id, layers, wl_name = build_workload(args)

    # ---- inputs resident in HBM before anything is timed ----
    t_gen = time.time()
    items = []
    for layer in layers:
        x, w, sc = S.gen_layer(cfg_id, layer)
        d = sq.conv_desc(layer.B, layer.H, layer.W, layer.C, layer.N, layer.KH, layer.KW, layer.stride, layer.pad)
        m = sq.mode(*layer.mode.astuple())
        xd = torch.from_numpy(x).to(dev)
        wd = torch.from_numpy(w).to(dev)
        sd = torch.from_numpy(sc).to(dev)
        packed = torch.empty(sq.sparq_packed_bytes(d), dtype=torch.uint8, device=dev)
        sq.sparq_pack_weights(wd, d, packed)
        wsb = sq.sparq_workspace_bytes(d, m)
        ws = torch.empty(wsb, dtype=torch.uint8, device=dev) if wsb else None
        out = torch.empty((layer.M, layer.N), dtype=torch.float32, device=dev)
        items.append(dict(layer=layer, d=d, m=m, x=xd, sc=sd, packed=packed, ws=ws, out=out,
                          host=(x, w, sc) if len(layers) == 1 else None))
        del wd
    torch.cuda.synchronize()
    print(f"[bench] inputs generated and uploaded in {time.time() - t_gen:.1f}s", file=sys.stderr, flush=True)

    def step():
        for it in items:
            for _ in range(it["layer"].repeat):
                sq.sparq_conv_gemm(it["x"], it["packed"], it["d"], it["m"], acc=None, scale=it["sc"], out=it["out"],
                                   workspace=it["ws"])

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        step()
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ms_per_step = e0.elapsed_time(e1) / args.steps
    total_ops = S.total_ops(layers)
    tops = total_ops / (ms_per_step * 1e-3) / 1e12

    # ---- dominant kernel: the fused conv-GEMM of the largest layer, timed on its own ----
    dom = max(items, key=lambda it: it["layer"].ops * it["layer"].repeat)
    reps = max(5, args.steps)
    for _ in range(2):
        sq.sparq_conv_gemm(dom["x"], dom["packed"], dom["d"], dom["m"], scale=dom["sc"], out=dom["out"], workspace=dom["ws"])
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        sq.sparq_conv_gemm(dom["x"], dom["packed"], dom["d"], dom["m"], scale=dom["sc"], out=dom["out"], workspace=dom["ws"])
    e1.record()
    torch.cuda.synchronize()
    dom_ms = e0.elapsed_time(e1) / reps
    dom_tops = dom["layer"].ops / (dom_ms * 1e-3) / 1e12
    roofline = {"bound": "mfma", "achieved": round(dom_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": round(dom_tops / PEAK_INT8_TOPS, 4), "traffic": None,
                "kernel": "conv_gemm_kernel", "layer": dom["layer"].name, "ms_per_launch": round(dom_ms, 4),
                "ops_per_launch": dom["layer"].ops}

    # ---- standalone trim and dequant kernels (HBM-bound), on the dominant layer's tensors ----
    xin = dom["x"]
    y = torch.empty_like(xin)
    for _ in range(2):
        sq.sparq_trim(xin, y, dom["m"])
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        sq.sparq_trim(xin, y, dom["m"])
    e1.record()
    torch.cuda.synchronize()
    trim_ms = e0.elapsed_time(e1) / reps
    trim_gbps = 2 * xin.numel() / (trim_ms * 1e-3) / 1e9
    del y
    acc = torch.randint(-2 ** 24, 2 ** 24, dom["out"].shape, dtype=torch.int32, device=dev)
    for _ in range(2):
        sq.sparq_dequant(acc, dom["sc"], dom["out"])
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        sq.sparq_dequant(acc, dom["sc"], dom["out"])
    e1.record()
    torch.cuda.synchronize()
    deq_ms = e0.elapsed_time(e1) / reps
    deq_gbps = 8 * acc.numel() / (deq_ms * 1e-3) / 1e9
    del acc

    if args.per_layer:
        print(f"{'layer':28s} {'M':>8s} {'K':>6s} {'N':>5s} {'rep':>3s} {'ms':>9s} {'TOPS':>8s}", file=sys.stderr)
        for it in items:
            L = it["layer"]
            sq.sparq_conv_gemm(it["x"], it["packed"], it["d"], it["m"], scale=it["sc"], out=it["out"], workspace=it["ws"])
            torch.cuda.synchronize()
            e0.record()
            for _ in range(10):
                sq.sparq_conv_gemm(it["x"], it["packed"], it["d"], it["m"], scale=it["sc"], out=it["out"], workspace=it["ws"])
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / 10
            print(f"{L.name:28s} {L.M:8d} {L.K:6d} {L.N:5d} {L.repeat:3d} {ms:9.4f} {L.ops / ms / 1e9:8.1f}",
                  file=sys.stderr)

    # ---- CPU baseline: the oracle as it stands, on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        threads = int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1))
        L = dom["layer"]
        if dom["host"] is not None:
            xh, wh, sch = dom["host"]
        else:
            xh, wh, sch = S.gen_layer(cfg_id, L)
        # pilot on a few rows, then a sample sized for roughly 15 s of oracle work
        pilot = np.linspace(0, L.M - 1, min(L.M, 64)).astype(np.int64)
        t0 = time.perf_counter()
        oracle.conv_gemm(xh, wh, L.stride, L.pad, scale=sch, rows=pilot, **L.mode.kwargs())
        t_pilot = time.perf_counter() - t0
        t0 = time.perf_counter()
        oracle.conv_gemm(xh, wh, L.stride, L.pad, scale=sch, rows=pilot[:1], **L.mode.kwargs())
        t_fixed = time.perf_counter() - t0                       # trimming the whole input dominates this
        per_row = max(1e-7, (t_pilot - t_fixed) / max(1, len(pilot) - 1))
        n_rows = int(max(64, min(L.M, (15.0 - t_fixed) / per_row)))
        rows = np.linspace(0, L.M - 1, n_rows).astype(np.int64)
        t0 = time.perf_counter()
        oracle.conv_gemm(xh, wh, L.stride, L.pad, scale=sch, rows=rows, **L.mode.kwargs())
        dt = time.perf_counter() - t0
        cpu_tops = 2.0 * n_rows * L.K * L.N / dt / 1e12
        cpu = {"value": round(cpu_tops, 6), "unit": "TOPS", "cores": threads, "kind": "oracle",
               "sample": f"{n_rows} of {L.M} output rows of {L.name} (all {L.N} channels, whole input trimmed), "
                         f"{dt:.1f} s wall"}

    line = {
        "metric": "SPARQ conv-GEMM TOPS (int8-equiv)",
        "value": round(tops, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8",
        "data": "synthetic",
        "config": {"workload": wl_name, "layers": sum(l.repeat for l in layers), "total_gop": round(total_ops / 1e9, 3),
                   "output": "fp32 (fused dequant)", "wall_ms_per_step": round(wall_ms, 4)},
        "pct_int8_mfma_peak": round(100 * tops / PEAK_INT8_TOPS, 2),
        "roofline": roofline,
        "trim": {"GBps": round(trim_gbps, 1), "frac_hbm_peak": round(trim_gbps / PEAK_HBM_GBPS, 4),
                 "bytes_per_launch": 2 * xin.numel(), "ms": round(trim_ms, 4)},
        "dequant": {"GBps": round(deq_gbps, 1), "frac_hbm_peak": round(deq_gbps / PEAK_HBM_GBPS, 4),
                    "ms": round(deq_ms, 4)},
        "cpu_baseline": cpu,
    }
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
