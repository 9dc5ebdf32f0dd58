#!/usr/bin/env python3
"""Benchmark of the SPARQ hot path on one MI355X.

One "step" is one pass of the fused path -- activation gather, vSPARQ/bSPARQ
trim, int8 contraction, offset correction and per-channel dequantisation to
fp32 -- over the workload's synthetic input, through the C ABI
(``sparq_conv_gemm`` with ``out``).  The default workload is the large GEMM of
the option sweep (M=65536, K=4608 = 3x3x512, N=512, 5opt, rounding, pairing on,
50 % zeros), the shape the int8-MFMA target is stated on, run as what it is: a
3x3 convolution over 512 channels (64 images of 32x32), gathered implicitly.  The standalone trim and
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

# HBM bytes per launch of the dominant kernel come from rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE runs of this
# script; their summary is committed as profiles/conv_cfg3_hbm_traffic.md and carries one machine-readable line per
# workload ("traffic <workload> fetch_bytes=<n> write_bytes=<n>", already scaled by the copy-kernel calibration).
TRAFFIC_PROFILE = os.path.join("profiles", "conv_cfg3_hbm_traffic.md")


def measured_traffic(workload):
    """{"fetch_bytes", "write_bytes"} of `workload` from the committed counter summary, or None."""
    import re
    try:
        text = open(os.path.join(ROOT, TRAFFIC_PROFILE)).read()
    except OSError:
        return None
    m = re.search(rf"^traffic {re.escape(workload)} fetch_bytes=(\d+) write_bytes=(\d+)\s*$", text, re.M)
    return {"fetch_bytes": int(m.group(1)), "write_bytes": int(m.group(2))} if m else None


def layer_bounds(layer, out_bytes=4):
    """Lower bounds of one launch of `layer` against the published peaks: (ms at the int8 matrix peak, ms at the
    HBM peak on the algorithmic bytes = input once + weights + results)."""
    x_b = layer.B * layer.H * layer.W * layer.C
    alg = x_b + layer.K * layer.N + out_bytes * layer.M * layer.N
    return layer.ops / (PEAK_INT8_TOPS * 1e12) * 1e3, alg / (PEAK_HBM_GBPS * 1e9) * 1e3


def table_bound_ms(layers, out_bytes=4):
    """Sum over a layer table of max(matrix bound, HBM bound): no schedule of these launches can be faster."""
    return sum(max(layer_bounds(l, out_bytes)) * l.repeat for l in layers)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=50)
    ap.add_argument("--workload", default="cfg3-conv",
                    help="cfg3-conv (default: M=65536, K=3x3x512, N=512 as an implicit-GEMM 3x3 convolution) | "
                         "cfg3 (the same M,K,N with a materialised A[M,K]) | "
                         "cfg0 | cfg1 | cfg2 | cfg4 | cfg4-2bit | cfg3-sweep (all 36 option points, table on stderr)")
    ap.add_argument("--mask", type=lambda s: int(s, 0), default=None, help="cfg3 only: shift mask override")
    ap.add_argument("--round", type=int, default=None, help="cfg3 only: rounding override")
    ap.add_argument("--pair", type=int, default=None, help="cfg3 only: pairing override")
    ap.add_argument("--zf", type=float, default=None, help="cfg3 only: zero fraction override")
    ap.add_argument("--rows", type=int, default=65536, help="cfg3 only: M")
    ap.add_argument("--batch", type=int, default=None, help="cfg1/2/4: batch override")
    ap.add_argument("--output", default="fp32", choices=["fp32", "u8", "u8-chain"],
                    help="fp32: fused per-channel dequantisation (the headline form); u8: results requantised to the next "
                         "layer's unsigned 8-bit activations (sparq_conv_gemm_u8); u8-chain: the steady state of a chained "
                         "network -- inputs arrive trimmed (the layer runs at plain 8 bits), outputs leave requantised and "
                         "trimmed for the next layer, so every activation is trimmed once")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--per-layer", action="store_true", help="print a per-layer table on stderr")
    ap.add_argument("--no-extra", action="store_true", help="skip the secondary figures of the default run")
    ap.add_argument("--no-probes", action="store_true", help="skip the machine-ceiling probes and the zero-operand run")
    ap.add_argument("--sweep-bits", default="4", choices=["4", "low"],
                    help="cfg3-sweep: the 36 points of the 4-bit option sets (default) or the 24 points of the 3-bit / 6-shift "
                         "and 2-bit / 7-shift variants")
    ap.add_argument("--sweep-form", default="conv", choices=["conv", "explicit"],
                    help="cfg3-sweep: run the points as the 3x3 convolution (default) or on a materialised A[M,K]")
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
    if wl == "cfg3-sweep":
        return 3, [], "config3 sweep"
    raise SystemExit(f"unknown workload {wl}")


def prepare(sq, S, torch, dev, cfg_id, layers, keep_host=False, outputs=("fp32",)):
    """Generate every layer's tensors, upload them and pack the weights (all before any timing)."""
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
        out = torch.empty((layer.M, layer.N), dtype=torch.float32, device=dev) if "fp32" in outputs else None
        y = rq = None
        xt = m_out = None
        if "u8" in outputs or "u8-chain" in outputs:
            y = torch.empty((layer.M, layer.N), dtype=torch.uint8, device=dev)
            rq = torch.from_numpy(S.gen_requant(layer, S.rng_for(cfg_id, 900 + layer.index))).to(dev)
        if "u8-chain" in outputs:
            # what the previous layer would have handed over: x already trimmed with this layer's mode; the output is
            # trimmed with the network's mode (a plain 8-bit first layer trims for the layers that follow it)
            net_mode = next((l.mode for l in layers if l.mode.window_bits != 8), layer.mode)
            xt = torch.empty_like(xd)
            sq.sparq_trim(xd, xt, m)
            m_out = sq.mode(*net_mode.astuple())
            wsb2 = sq.sparq_workspace_bytes(d, sq.mode(*S.PLAIN8.astuple()))
            if wsb2 > wsb:
                ws = torch.empty(wsb2, dtype=torch.uint8, device=dev)
        items.append(dict(layer=layer, d=d, m=m, x=xd, sc=sd, packed=packed, ws=ws, out=out, y=y, rq=rq, xt=xt, m_out=m_out,
                          m_plain=sq.mode(*S.PLAIN8.astuple()), host=(x, w, sc) if keep_host else None))
        del wd
    torch.cuda.synchronize()
    return items


def run_layer(sq, it, output="fp32"):
    if output == "u8-chain":
        sq.sparq_conv_gemm_u8(it["xt"], it["packed"], it["d"], it["m_plain"], it["rq"], it["y"], workspace=it["ws"],
                              out_mode=it["m_out"])
    elif output == "u8":
        sq.sparq_conv_gemm_u8(it["x"], it["packed"], it["d"], it["m"], it["rq"], it["y"], workspace=it["ws"])
    else:
        sq.sparq_conv_gemm(it["x"], it["packed"], it["d"], it["m"], acc=None, scale=it["sc"], out=it["out"],
                           workspace=it["ws"])


def run_step(sq, items, output="fp32"):
    for it in items:
        for _ in range(it["layer"].repeat):
            run_layer(sq, it, output)


def time_steps(sq, torch, items, warmup, steps, output="fp32"):
    """(device ms per step from HIP events on the launch stream, host wall ms per step)."""
    for _ in range(warmup):
        run_step(sq, items, output)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        run_step(sq, items, output)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / steps, (time.perf_counter() - t0) * 1e3 / steps


def sweep(args, sq, S, torch, dev):
    """The option sweep: {2opt,3opt,5opt} x {floor,round} x pairing {off,on} x zero fraction {.2,.5,.8}
    on M=65536, K=4608, N=512; fused conv-GEMM TOPS and standalone trim GB/s for each point."""
    from dataclasses import replace
    points, by_zf = [], {}
    for mode, zf in (S.config3_sweep_low() if args.sweep_bits == "low" else S.config3_sweep()):
        by_zf.setdefault(zf, []).append(mode)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    print(f"{'mode':24s} {'zf':>4s} {'gemm ms':>9s} {'TOPS':>8s} {'trim GB/s':>10s}", file=sys.stderr)
    tot_ops = tot_ms = 0.0
    for zf, modes in by_zf.items():
        base = replace(S.config3_layer(args.rows), zf=zf)
        if args.sweep_form == "conv":
            base = replace(base, name="conv3x3_512_512_32x32", B=args.rows // 1024, H=32, W=32, C=512, KH=3, KW=3, pad=(1, 1))
        items = prepare(sq, S, torch, dev, 3, [base])
        it = items[0]
        y = torch.empty_like(it["x"])
        time_steps(sq, torch, items, args.warmup, args.warmup)     # clocks settle after the idle upload phase
        for mode in modes:
            it["layer"] = replace(base, mode=mode)
            it["m"] = sq.mode(*mode.astuple())
            ms, _ = time_steps(sq, torch, items, max(5, args.warmup // 5), max(10, args.steps // 10))
            for _ in range(2):
                sq.sparq_trim(it["x"], y, it["m"])
            torch.cuda.synchronize()
            e0.record()
            for _ in range(10):
                sq.sparq_trim(it["x"], y, it["m"])
            e1.record()
            torch.cuda.synchronize()
            gbps = 2 * y.numel() / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9
            t = base.ops / ms / 1e9
            tot_ops += base.ops
            tot_ms += ms
            points.append({"mode": mode.label, "zf": zf, "ms": round(ms, 4), "TOPS": round(t, 1), "trim_GBps": round(gbps, 1)})
            print(f"{mode.label:24s} {zf:4.1f} {ms:9.4f} {t:8.1f} {gbps:10.1f}", file=sys.stderr, flush=True)
        del items, it, y
        torch.cuda.empty_cache()
    tops = tot_ops / (tot_ms * 1e-3) / 1e12
    print(json.dumps({
        "metric": "SPARQ conv-GEMM TOPS (int8-equiv)", "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1,
        "steps": max(10, args.steps // 10), "warmup": max(5, args.warmup // 5), "ms_per_step": round(tot_ms / len(points), 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"config3 sweep ({'3-bit and 2-bit windows' if args.sweep_bits == 'low' else '4-bit windows'}): {len(points)} option points on GEMM M={args.rows} K=4608 N=512, "
                               f"{args.sweep_form} form (value = total ops / total time over the points)"},
        "points": points, "roofline": None, "cpu_baseline": None}), flush=True)


def time_calls(torch, fn, warm, reps):
    """ms per call of fn(i), HIP events on the current (launch) stream."""
    for i in range(warm):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(reps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps


def machine_probes(torch, dev):
    """Ceilings measured on this device (include/sparq_probe.h): the int8 matrix instruction on register operands with
    all-zero and with random operand bytes, and a streaming copy over 1 GiB (far larger than the last-level cache)."""
    import numpy as np
    from paper_2105_11010_amd import probe as P
    iters = 4000
    sink = torch.empty(P.SINK_BYTES, dtype=torch.uint8, device=dev)
    rng = np.random.Generator(np.random.PCG64(7))
    res = {}
    for name, host in (("zero_operands", np.zeros(P.OPERAND_BYTES, dtype=np.uint8)),
                       ("random_operands", rng.integers(0, 256, P.OPERAND_BYTES, dtype=np.uint8))):
        ops = torch.from_numpy(host).to(dev)
        ms = time_calls(torch, lambda i: P.sparq_probe_mfma_i8(ops, sink, iters), 3, 10)
        res[name] = round(P.sparq_probe_mfma_i8_ops(iters) / ms / 1e9, 1)
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 256)
    dst = torch.empty(n, dtype=torch.uint8, device=dev)
    ms = time_calls(torch, lambda i: P.sparq_probe_copy(src, dst), 2, 10)
    del src, dst
    torch.cuda.empty_cache()
    return {"int8_mfma_TOPS": res, "copy_GBps": round(2 * n / ms / 1e6, 1),
            "note": "v_mfma_i32_32x32x32_i8 on register operands, one wavefront per SIMD (its rate depends on the operand "
                    "data: the chip lowers its clock under the power the multipliers draw); copy: 1 GiB read + 1 GiB written"}


def sclk_file(torch):
    """The sysfs file with the shader-clock levels of device 0 (the current one is starred), or None."""
    import glob
    files = sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk"))
    if len(files) > 1:
        # several cards in sysfs: take the one at the PCI address of the device the benchmark runs on
        p = torch.cuda.get_device_properties(0)
        want = "%04x:%02x:%02x" % (getattr(p, "pci_domain_id", 0), getattr(p, "pci_bus_id", -1), getattr(p, "pci_device_id", 0))
        for f in files:
            try:
                if want in open(os.path.join(os.path.dirname(f), "uevent")).read().lower():
                    return f
            except OSError:
                pass
        return None
    return files[0] if files else None


def sclk_during(torch, fn, seconds=1.5):
    """Median shader clock (MHz; the starred level of sysfs pp_dpm_sclk, the file rocm-smi prints) while fn() is
    launched back to back for `seconds`; None if there is no reading.  Plain file reads between batches of launches:
    no child process.  Shows the chip lowering its clock under load."""
    import re
    import statistics
    path = sclk_file(torch)
    if path is None:
        return None
    vals, t0 = [], time.time()
    while time.time() - t0 < seconds:
        for _ in range(100):
            fn()
        try:
            m = re.search(r"(\d+)Mhz \*", open(path).read())
        except OSError:
            return None
        if m and time.time() - t0 > 0.4:
            vals.append(int(m.group(1)))
        torch.cuda.synchronize()
    return int(statistics.median(vals)) if vals else None


def streaming_kernels(sq, S, torch, dev, dom, reps):
    """Standalone trim and dequantisation kernels, HBM-bound.  'cold': on config 3's materialised A (302 MB in, 302 MB
    out per call) / on three rotating 134 MB accumulator tensors -- more than the 256 MB last-level cache holds, so every
    byte comes from and goes to HBM; 'warm': on the dominant layer's own input (33.5 MB), which stays cache-resident."""
    import numpy as np
    out = {}
    xin = dom["x"]
    y = torch.empty_like(xin)
    ms = time_calls(torch, lambda i: sq.sparq_trim(xin, y, dom["m"]), 2, reps)
    warm = {"GBps": round(2 * xin.numel() / ms / 1e6, 1), "bytes_per_launch": 2 * xin.numel(), "ms": round(ms, 4)}
    del y
    big = S.config3_layer()                      # A[65536][4608]
    rng = S.rng_for(3, 77)
    block = S.gen_activations((1 << 24,), big.zf, rng)
    xa = torch.from_numpy(np.resize(block, (big.M, big.K))).to(dev)
    ya = torch.empty_like(xa)
    ms = time_calls(torch, lambda i: sq.sparq_trim(xa, ya, dom["m"]), 2, reps)
    cold = {"GBps": round(2 * xa.numel() / ms / 1e6, 1), "bytes_per_launch": 2 * xa.numel(), "ms": round(ms, 4)}
    # the packed storage codec (n-bit data + ShiftCtrl + MuxCtrl records) on the same cold tensor
    codec = []
    for label, mode, group in (("the workload's mode", dom["layer"].mode, 1), ("4b-3opt-floor-novS", S.Mode(4, S.OPT3, 0, 0), 1),
                               ("4b-5opt-round-novS, ShiftCtrl shared by 8", S.Mode(4, S.OPT5, 1, 0), 8)):
        if mode.window_bits == 8:
            continue
        pm = sq.mode(*mode.astuple())
        nb = sq.sparq_packed_act_bytes(big.M, big.K, pm, group)
        pk = torch.empty(nb, dtype=torch.uint8, device=dev)
        ms_p = time_calls(torch, lambda i: sq.sparq_pack_act(xa, pk, pm, group), 2, reps)
        ms_u = time_calls(torch, lambda i: sq.sparq_unpack_act(pk, ya, pm, group), 2, reps)
        codec.append({"mode": mode.label if label.startswith("the") else label, "group": group,
                      "bits_per_activation": round(8 * nb / xa.numel(), 3), "packed_bytes": nb,
                      "pack_GBps": round((xa.numel() + nb) / ms_p / 1e6, 1), "unpack_GBps": round((xa.numel() + nb) / ms_u / 1e6, 1)})
        del pk
    out["packed_act"] = {"tensor": "config 3 A[65536][4608] uint8 (cold)", "GBps_counts": "bytes read + bytes written", "points": codec}
    del xa, ya
    out["trim"] = {"GBps": cold["GBps"], "frac_hbm_peak": round(cold["GBps"] / PEAK_HBM_GBPS, 4), "state": "cold (HBM)",
                   "tensor": "config 3 A[65536][4608] uint8", "bytes_per_launch": cold["bytes_per_launch"], "ms": cold["ms"],
                   "warm_cache_resident": dict(warm, tensor="the dominant layer's input")}
    L = dom["layer"]
    accs = [torch.randint(-2 ** 24, 2 ** 24, (L.M, L.N), dtype=torch.int32, device=dev) for _ in range(3)]
    outs = [torch.empty((L.M, L.N), dtype=torch.float32, device=dev) for _ in range(3)]
    ms_cold = time_calls(torch, lambda i: sq.sparq_dequant(accs[i % 3], dom["sc"], outs[i % 3]), 3, reps)
    ms_warm = time_calls(torch, lambda i: sq.sparq_dequant(accs[0], dom["sc"], outs[0]), 2, reps)
    nbytes = 8 * accs[0].numel()
    out["dequant"] = {"GBps": round(nbytes / ms_cold / 1e6, 1), "frac_hbm_peak": round(nbytes / ms_cold / 1e6 / PEAK_HBM_GBPS, 4),
                      "state": "cold (HBM): three rotating tensor pairs, 805 MB", "bytes_per_launch": nbytes, "ms": round(ms_cold, 4),
                      "warm_one_pair": {"GBps": round(nbytes / ms_warm / 1e6, 1), "ms": round(ms_warm, 4)}}
    del accs, outs
    torch.cuda.empty_cache()
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(the path would shard over output rows / batch without any communication).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2105_11010_amd as sq
    import sparq_synth as S

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    cfg_id, layers, wl_name = build_workload(args)

    if args.workload == "cfg3-sweep":
        return sweep(args, sq, S, torch, dev)

    # ---- inputs resident in HBM before anything is timed ----
    t_gen = time.time()
    items = prepare(sq, S, torch, dev, cfg_id, layers, keep_host=len(layers) == 1, outputs=(args.output,))
    print(f"[bench] inputs generated and uploaded in {time.time() - t_gen:.1f}s", file=sys.stderr, flush=True)

    # ---- the machine's own ceilings, measured first (they also take the chip out of its idle clocks) ----
    probes = None if args.no_probes else machine_probes(torch, dev)

    # ---- W untimed steps, then exactly K timed steps ----
    ms_per_step, wall_ms = time_steps(sq, torch, items, args.warmup, args.steps, args.output)
    total_ops = S.total_ops(layers)
    tops = total_ops / (ms_per_step * 1e-3) / 1e12
    out_bytes = 4 if args.output == "fp32" else 1

    # ---- dominant kernel: the fused conv-GEMM of the largest layer, timed on its own ----
    dom = max(items, key=lambda it: it["layer"].ops * it["layer"].repeat)
    reps = max(5, args.steps)
    if len(items) == 1 and dom["layer"].repeat == 1:
        dom_ms = ms_per_step                     # a one-layer workload: the timed region is this kernel's launches
    else:
        dom_ms = time_calls(torch, lambda i: run_layer(sq, dom, args.output), 2, reps)
    dom_tops = dom["layer"].ops / (dom_ms * 1e-3) / 1e12
    default_point = (args.rows == 65536 and args.mask is None and args.round is None and args.pair is None
                     and args.zf is None and args.output == "fp32")
    tr = measured_traffic(args.workload) if default_point else None
    x_b, w_b = dom["x"].numel(), dom["layer"].K * dom["layer"].N
    b_mfma, b_hbm = layer_bounds(dom["layer"], out_bytes)
    roofline = {"bound": "mfma", "achieved": round(dom_tops, 2), "peak": PEAK_INT8_TOPS, "unit": "TOP/s",
                "frac": round(dom_tops / PEAK_INT8_TOPS, 4),
                "traffic": (tr["fetch_bytes"] + tr["write_bytes"]) if tr else None,
                "traffic_detail": tr, "traffic_source": TRAFFIC_PROFILE if tr else None,
                "algorithmic_bytes": x_b + w_b + out_bytes * dom["layer"].M * dom["layer"].N,
                "kernel": sq.sparq_conv_plan(dom["d"], dom["m"]), "layer": dom["layer"].name, "ms_per_launch": round(dom_ms, 4),
                "ops_per_launch": dom["layer"].ops,
                "bound_ms": {"mfma": round(b_mfma, 4), "hbm": round(b_hbm, 4), "min_time": round(max(b_mfma, b_hbm), 4)}}
    if probes:
        roofline["peak_measured"] = probes
        roofline["frac_of_measured_random_operand_peak"] = round(dom_tops / probes["int8_mfma_TOPS"]["random_operands"], 4)
    if len(layers) == 1 and args.output == "fp32" and not args.no_probes:
        # The same kernel, the same launch, all-zero activations and weights: the instruction stream is identical,
        # only the operand bytes differ -- what is left of the difference is the chip's data-dependent clock.
        L = dom["layer"]
        xz = torch.zeros_like(dom["x"])
        wz = torch.zeros(L.w_shape(), dtype=torch.int8, device=dev)
        pz = torch.empty_like(dom["packed"])
        sq.sparq_pack_weights(wz, dom["d"], pz)
        zero_it = dict(dom, x=xz, packed=pz)
        z_ms = time_calls(torch, lambda i: run_layer(sq, zero_it, args.output), max(2, args.warmup), reps)
        roofline["same_kernel_zero_operands"] = {"TOPS": round(L.ops / z_ms / 1e9, 2), "frac": round(L.ops / z_ms / 1e9 / PEAK_INT8_TOPS, 4),
                                                 "ms_per_launch": round(z_ms, 4)}
        # the shader clock the chip settles at while each of the two runs back to back (2400 MHz nominal)
        roofline["sclk_mhz"] = {"nominal": 2400, "kernel_on_the_workload": sclk_during(torch, lambda: run_layer(sq, dom, args.output)),
                                "same_kernel_zero_operands": sclk_during(torch, lambda: run_layer(sq, zero_it, args.output)),
                                "source": "sysfs pp_dpm_sclk (what rocm-smi --showclocks prints), median over 1.5 s of back-to-back launches"}
        if roofline["sclk_mhz"]["kernel_on_the_workload"]:
            # the published peak is 5.0 POP/s at 2400 MHz; at the clock the chip grants this kernel it is proportionally less
            roofline["frac_of_peak_at_the_measured_clock"] = round(dom_tops / (PEAK_INT8_TOPS * roofline["sclk_mhz"]["kernel_on_the_workload"] / 2400.0), 4)
        del xz, wz, pz, zero_it

    # ---- standalone trim and dequant kernels (HBM-bound) ----
    stream = streaming_kernels(sq, S, torch, dev, dom, reps)

    if args.per_layer:
        print(f"{'layer':28s} {'M':>8s} {'K':>6s} {'N':>5s} {'rep':>3s} {'ms':>9s} {'TOPS':>8s} {'mfma ms':>8s} {'hbm ms':>8s} "
              f"{'bound':>5s} {'frac':>6s}", file=sys.stderr)
        for it in items:
            L = it["layer"]
            ms = time_calls(torch, lambda i: run_layer(sq, it, args.output), 1, 10)
            bm, bh = layer_bounds(L, out_bytes)
            print(f"{L.name:28s} {L.M:8d} {L.K:6d} {L.N:5d} {L.repeat:3d} {ms:9.4f} {L.ops / ms / 1e9:8.1f} {bm:8.4f} {bh:8.4f} "
                  f"{'mfma' if bm >= bh else 'hbm':>5s} {max(bm, bh) / ms:6.3f}", file=sys.stderr)

    # ---- secondary figures of the default run: the same GEMM with a materialised A[M,K] (no reuse
    #      between filter taps), the ResNet-18 layer table (small layers that do not fill the chip)
    #      and the Inception-shaped table; each with the sum of its layers' lower bounds ----
    also = None
    if args.workload == "cfg3-conv" and not args.no_extra and args.rows == 65536:
        also = []

        def entry(name, layers_, ms, ob):
            bound = table_bound_ms(layers_, ob)
            return {"workload": name, "value": round(S.total_ops(layers_) / ms / 1e9, 2), "unit": "TOPS", "ms_per_step": round(ms, 4),
                    "total_gop": round(S.total_ops(layers_) / 1e9, 3),
                    "bound_ms": {"mfma": round(sum(layer_bounds(l, ob)[0] * l.repeat for l in layers_), 4),
                                 "hbm": round(sum(layer_bounds(l, ob)[1] * l.repeat for l in layers_), 4),
                                 "sum_of_per_layer_max": round(bound, 4)},
                    "frac_of_bound": round(bound / ms, 4)}

        for wl in ("cfg3", "cfg1", "cfg4"):
            a2 = argparse.Namespace(**{**vars(args), "workload": wl})
            c2, l2, n2 = build_workload(a2)
            it2 = prepare(sq, S, torch, dev, c2, l2, outputs=("fp32", "u8", "u8-chain") if wl != "cfg3" else ("fp32",))
            ms2, _ = time_steps(sq, torch, it2, args.warmup, args.steps)
            also.append(entry(n2, l2, ms2, 4))
            if wl != "cfg3":
                # the same table with every result requantised to uint8 (one byte per output instead of four)
                ms3, _ = time_steps(sq, torch, it2, args.warmup, args.steps, "u8")
                also.append(entry(n2 + ", uint8 requantised outputs", l2, ms3, 1))
                # and as the layers of a chained network: trimmed once, in the producer's epilogue
                ms4, _ = time_steps(sq, torch, it2, args.warmup, args.steps, "u8-chain")
                also.append(entry(n2 + ", chained (input arrives trimmed; uint8 output trimmed for the next layer)", l2, ms4, 1))
            del it2
            torch.cuda.empty_cache()

        # the default layer from packed storage (n-bit data + ShiftCtrl + MuxCtrl records) and with 2:4 pruned weights;
        # ops counted as the dense layer's 2*M*K*N in both cases (what the layer computes, zeros included)
        L = dom["layer"]
        pm = dom["m"]
        if L.mode.window_bits < 8 and dom["out"] is not None:
            nb = sq.sparq_packed_act_bytes(L.B * L.H * L.W, L.C, pm, 1)
            px = torch.empty(nb, dtype=torch.uint8, device=dev)
            sq.sparq_pack_act(dom["x"], px, pm, 1)
            wsb = sq.sparq_conv_packed_workspace_bytes(dom["d"], pm)
            ws = torch.empty(max(wsb, 1), dtype=torch.uint8, device=dev)
            ms5 = time_calls(torch, lambda i: sq.sparq_conv_gemm_packed(px, 1, dom["packed"], dom["d"], pm, scale=dom["sc"],
                                                                        out=dom["out"], workspace=ws), args.warmup, args.steps)
            e = entry(wl_name + ", input held in packed storage (unpack pass + the same kernel at plain 8 bits)", [L], ms5, 4)
            e["packed_input_bytes"] = nb
            also.append(e)
            del px, ws
        if L.C % 4 == 0 and dom["out"] is not None:
            wv, wi = S.gen_sparse24_weights(L.w_shape(), S.rng_for(cfg_id, 24))
            wvd, wid = torch.from_numpy(wv).to(dev), torch.from_numpy(wi).to(dev)
            sp = torch.empty(sq.sparq_sparse24_packed_bytes(dom["d"], pm), dtype=torch.uint8, device=dev)
            sq.sparq_pack_weights_sparse24(wvd, wid, dom["d"], pm, sp)
            ws = torch.empty(max(sq.sparq_sparse24_workspace_bytes(dom["d"], pm), 1), dtype=torch.uint8, device=dev)
            ms6 = time_calls(torch, lambda i: sq.sparq_conv_gemm_sparse24(dom["x"], sp, dom["d"], pm, scale=dom["sc"], out=dom["out"],
                                                                          workspace=ws), args.warmup, args.steps)
            e = entry(wl_name + ", 2:4 pruned weights (activations picked by the kept weights, then paired: an expanded problem "
                                "with 4x the channels whose weights are again 2:4 sparse)", [L], ms6, 4)
            e["plan"] = sq.sparq_sparse24_plan(dom["d"], pm)
            e["note"] = ("value counts the dense layer's operations; with pairing on the expanded problem holds 4x the channels, "
                         "on the sparse matrix instruction (plan ends in sparse_mfma) that is 2x the dense layer's matrix instructions")
            also.append(e)
            del sp, ws
            # the same pruned weights with vSPARQ off: no expansion, the layer itself on the sparse matrix instruction
            if L.mode.window_bits < 8 and L.mode.pair:
                m1 = sq.mode(L.mode.window_bits, L.mode.shift_mask, L.mode.round_nearest, 0)
                sp = torch.empty(sq.sparq_sparse24_packed_bytes(dom["d"], m1), dtype=torch.uint8, device=dev)
                sq.sparq_pack_weights_sparse24(wvd, wid, dom["d"], m1, sp)
                ws = torch.empty(max(sq.sparq_sparse24_workspace_bytes(dom["d"], m1), 1), dtype=torch.uint8, device=dev)
                ms7 = time_calls(torch, lambda i: sq.sparq_conv_gemm_sparse24(dom["x"], sp, dom["d"], m1, scale=dom["sc"], out=dom["out"],
                                                                              workspace=ws), args.warmup, args.steps)
                e = entry(wl_name + ", 2:4 pruned weights with vSPARQ off (each picked activation trimmed alone: the layer itself, "
                                    "half its weights)", [L], ms7, 4)
                e["plan"] = sq.sparq_sparse24_plan(dom["d"], m1)
                e["note"] = "value counts the dense layer's operations; the dense layer (all weights kept) is this run's headline figure"
                also.append(e)
                del sp, ws
            del wvd, wid
        torch.cuda.empty_cache()

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
                   "output": {"fp32": "fp32 (fused dequant)", "u8": "uint8 (fused requantisation)",
                              "u8-chain": "uint8 (fused requantisation + the next layer's trim; input arrives trimmed)"}[args.output],
                   "wall_ms_per_step": round(wall_ms, 4),
                   "bound_ms_per_step": round(table_bound_ms(layers, out_bytes), 4)},
        "pct_int8_mfma_peak": round(100 * tops / PEAK_INT8_TOPS, 2),
        "roofline": roofline,
        "trim": stream["trim"],
        "dequant": stream["dequant"],
        "packed_act": stream["packed_act"],
        "cpu_baseline": cpu,
    }
    if also:
        line["also"] = also
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
