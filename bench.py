#!/usr/bin/env python3
"""Benchmark of the zero-skipping convolution passes on one MI355X.

A step is one pass of the whole hot path -- st_conv_fwd, st_conv_bwi, st_conv_bww -- over one
batch of the VGG16 conv3_2-shaped layer (N=16, C=K=256, 56x56, 3x3, stride 1, pad 1) with
synthetic inputs: x = ReLU-shifted Gaussian with 60 % zeros, dy = Bernoulli-masked Gaussian with
50 % zeros, He-normal filters.  Inputs are resident in HBM before the timed region.

Prints ONE JSON line.  value = effective (dense-equivalent) TFLOP/s of the step,
3 * 2*N*K*C*OH*OW*R*S / step time.  Extra objects: per-pass timings of the sparse entry points and
of the dense controls, the sparse-over-dense speedup at 0/30/50/70/90 % zeros, the roofline of the
dominant kernel, and the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_FP32_VECTOR = 157.3      # TFLOP/s, published MI355X fp32 vector peak (needs packed fp32 math)
PEAK_FP32_FMA = 78.6          # TFLOP/s, 256 CU x 4 SIMD x 16 lanes x 2 flop x 2.4 GHz: one v_fma_f32 per lane-clock
PEAK_FP32_MFMA = 157.3        # TFLOP/s, published dense fp32 matrix peak

# HBM traffic per launch of the dominant kernel (fwd_sparse_kernel on this workload) from two
# rocprofv3 --pmc runs, FETCH_SIZE x 2.000 and WRITE_SIZE x 1.000 (factors from a 256 MiB copy of known
# size): 47712.9 KiB * 2 + 50176.0 KiB.  See profiles/bench_vgg3_2_hbm_traffic.md.
MEASURED_TRAFFIC_BYTES = int((47712.9 * 2.0 + 50176.0) * 1024)


def sustain(fn, ms, stream):
    """Keeps the GPU busy with fn for about ms milliseconds (untimed).  After an idle spell of 50 ms or
    more the chip needs some 30 ms of continuous work to return to its sustained clocks (the same launch
    reads 0.46 ms right after a pause and 0.40 ms from then on); every timing below starts from that state,
    which is the one a training run is in."""
    import torch
    t0 = time.perf_counter()
    while True:
        for _ in range(4):
            fn()
        torch.cuda.current_stream().synchronize()
        if (time.perf_counter() - t0) * 1e3 >= ms:
            return

def write_config_table(path, st, stgen, torch, dev, stream, sustain_ms=30.0):
    """Per (layer, zero fraction, pass): sparse and dense time, effective TFLOP/s, executed TFLOP/s as a
    fraction of the fp32 vector peak, dense fraction of the MFMA peak, speed-up.  Inputs are drawn on the
    device (torch generator, seed 0) with the same distributions as stgen: timing only, no parity."""
    import math

    torch.manual_seed(0)

    def relu_sparse(shape, p):
        z = torch.randn(shape, device=dev)
        if p <= 0:
            return z
        t = math.sqrt(2.0) * torch.erfinv(torch.tensor(2.0 * p - 1.0, dtype=torch.float64)).item()
        return torch.clamp(z - t, min=0)

    def masked(shape, q):
        g = torch.randn(shape, device=dev)
        return g if q <= 0 else g * (torch.rand(shape, device=dev) >= q)

    def timeit(fn, iters=7):
        sustain(fn, sustain_ms, stream)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for a, b in evs:
            a.record(stream)
            fn()
            b.record(stream)
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in evs)
        return ts[len(ts) // 2]

    rows = []
    totals = {}                     # cfg -> [sparse, dense, auto, best] summed over its rows (us)

    def run(cfg, L, px, pdy, group=None):
        d = st.ConvDesc(L.N, L.C, L.K, L.H, L.W, L.R, L.S, L.stride, L.stride, L.pad, L.pad)
        x = relu_sparse((L.N, L.C // 16, L.H, L.W, 16), px)
        dy = masked((L.N, L.K // 16, L.OH, L.OW, 16), pdy)
        w = torch.randn((L.K // 16, L.C // 16, L.S, L.R, 16, 16), device=dev) * math.sqrt(2.0 / (L.C * L.R * L.S))
        y, dx, dw = torch.empty_like(dy), torch.empty_like(x), torch.empty_like(w)
        zx = float((x == 0).float().mean())
        zdy = float((dy == 0).float().mean())

        def ws(p, dn):
            n = st.st_conv_workspace_bytes(d, p, dn)
            return torch.empty(max(n // 4, 1), device=dev) if n else None

        for name, fs, fd, fa, a, b, o, pi, pa, z in (
                ("FWD", st.st_conv_fwd, st.st_conv_fwd_dense, st.st_conv_fwd_auto, x, w, y, 0, st.ST_PASS_FWD_AUTO, zx),
                ("BWI", st.st_conv_bwi, st.st_conv_bwi_dense, st.st_conv_bwi_auto, dy, w, dx, 1, st.ST_PASS_BWI_AUTO, zdy),
                ("BWW", st.st_conv_bww, st.st_conv_bww_dense, st.st_conv_bww_auto, x, dy, dw, 2, st.ST_PASS_BWW_AUTO, zx)):
            wss, wsd, wsa = ws(pi, False), ws(pi, True), ws(pa, False)
            ts = timeit(lambda: fs(d, a, b, o, wss, stream))
            td = timeit(lambda: fd(d, a, b, o, wsd, stream))
            ta = timeit(lambda: fa(d, a, b, o, wsa, stream))
            best = min(ts, td)
            eff = d.flops / ts / 1e9
            label = f"{L.name} {L.C}->{L.K} @{L.H} {L.R}x{L.S}" + (f"/{L.stride}" if L.stride != 1 else "") + f" N={L.N}"
            rows.append(f"| {cfg} | {label} | {name} | {z:.2f} | {ts * 1e3:.0f} | "
                        f"{td * 1e3:.0f} | {eff:.1f} | {eff * (1 - z) / PEAK_FP32_VECTOR:.3f} | "
                        f"{d.flops / td / 1e9 / PEAK_FP32_MFMA:.3f} | {td / ts:.2f} | {ta * 1e3:.0f} |")
            if name == "BWW":       # the same tensor with the zero test on dy (st_conv_bww_dy); same dense control
                wsy = ws(st.ST_PASS_BWW_DY, False)
                ty = timeit(lambda: st.st_conv_bww_dy(d, a, b, o, wsy, stream))
                best = min(best, ty)
                effy = d.flops / ty / 1e9
                rows.append(f"| {cfg} | {label} | BWW(dy) | {zdy:.2f} | {ty * 1e3:.0f} | {td * 1e3:.0f} | {effy:.1f} | "
                            f"{effy * (1 - zdy) / PEAK_FP32_VECTOR:.3f} | {d.flops / td / 1e9 / PEAK_FP32_MFMA:.3f} | "
                            f"{td / ty:.2f} | |")
            t = totals.setdefault(group or str(cfg), [0.0, 0.0, 0.0, 0.0])
            for i, v in enumerate((ts, td, ta, best)):
                t[i] += v * 1e3
        del x, dy, w, y, dx, dw

    run(3, stgen.RESNET3_2, stgen.RESNET3_2.p_x, stgen.RESNET3_2.p_dy)
    for L in stgen.BOTTLENECK:
        run(4, L, L.p_x, L.p_dy)
    for p in (0.0, 0.3, 0.5, 0.7, 0.9):
        for L in stgen.vgg16_stack(p):
            if L.name in ("vgg3_3", "vgg4_3", "vgg5_2", "vgg5_3"):      # same shapes as 3_2, 4_2, 5_1
                continue
            run(5, L, p, p, group=f"5 at {p:.0%} zeros")
    # every row of the paper's Table 1 (stride-2 and the late 1x1 layers included) at 50 % zeros
    for L in stgen.table1_layers(32, 0.5, 0.5):
        if L.name == "vgg1_2":
            L = stgen.Layer(L.name, 16, L.C, L.K, L.H, L.W, L.R, L.S, L.pad, 0.5, 0.5, L.stride)
        run("T1", L, 0.5, 0.5)
    with open(path, "w") as f:
        f.write("# Per-workload timings: `python bench.py --no-cpu --no-sweep --table <this file>` on one MI355X\n\n"
                "Median of 7 launches (HIP events) per entry point; inputs drawn on the device with the benchmark's\n"
                "distributions. config 3 = ResNet-34 block, 4 = ResNet-50 bottleneck, 5 = VGG16 stack at 0-90 % zeros,\n"
                "T1 = every layer of the paper's Table 1 at 50 % zeros. BWW tests x, BWW(dy) tests dy; auto = the\n"
                "st_conv_*_auto entry point of the pass (form chosen on the device from sampled zero counts).\n\n")
        f.write("| config | layer | pass | zeros of tested operand | sparse us | dense us | effective TFLOP/s | "
                "executed / 157.3 (fp32 vector peak) | dense / 157.3 (MFMA peak) | speed-up | auto us |\n")
        f.write("|---|---|---|---|---|---|---|---|---|---|---|\n")
        f.write("\n".join(rows) + "\n")
        f.write("\nSums over the rows of a config (FWD + BWI + BWW of every layer, us): what always calling the\n"
                "zero-skipping entry points (st_conv_fwd/bwi/bww), always the dense ones, or the self-selecting ones\n"
                "costs, and the sum of the fastest form per row (BWW(dy) included) as the lower bound of any choice.\n\n")
        f.write("| config | zero-skipping | dense | auto | fastest form per row | dense / auto |\n|---|---|---|---|---|---|\n")
        for cfg, t in totals.items():
            f.write(f"| {cfg} | {t[0]:.0f} | {t[1]:.0f} | {t[2]:.0f} | {t[3]:.0f} | {t[1] / t[2]:.2f} |\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--sustain-ms", type=float, default=30.0,
                    help="untimed spell of the launch about to be timed, before every per-pass / table timing")
    ap.add_argument("--clock-warm-ms", type=float, default=200.0,
                    help="untimed spell of continuous steps before the warm-up steps (sustained clocks)")
    ap.add_argument("--no-sweep", action="store_true", help="skip the 0-90 %% zero-fraction sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--sweep-iters", type=int, default=5)
    ap.add_argument("--table", metavar="FILE", default=None,
                    help="also time every other workload of the benchmark definition (ResNet-34 block, ResNet-50 "
                         "bottleneck, VGG16 stack at 0-90 %% zeros) and write a markdown table to FILE")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy kernel (reference for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one MI355X per box); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_1911_10175_amd as st
    import stgen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    st.load_library()

    L = stgen.VGG3_2_N16
    d = st.ConvDesc(L.N, L.C, L.K, L.H, L.W, L.R, L.S, 1, 1, L.pad, L.pad)
    F = d.flops
    stream = torch.cuda.current_stream()

    def upload(x, w, dy):
        return (torch.from_numpy(st.pack_activations(x)).to(dev),
                torch.from_numpy(st.pack_filters(w)).to(dev),
                torch.from_numpy(st.pack_activations(dy)).to(dev))

    x_h, w_h, dy_h = stgen.make_layer_tensors(L, seed=0)
    px, pdy = stgen.zero_fraction(x_h), stgen.zero_fraction(dy_h)
    xd, wd, dyd = upload(x_h, w_h, dy_h)
    y = torch.empty((L.N, L.K // 16, L.OH, L.OW, 16), device=dev)
    dx = torch.empty((L.N, L.C // 16, L.H, L.W, 16), device=dev)
    dw = torch.empty((L.K // 16, L.C // 16, L.S, L.R, 16, 16), device=dev)

    def ws_for(p, dense):
        n = st.st_conv_workspace_bytes(d, p, dense)
        return torch.empty(max(n, 4) // 4, dtype=torch.float32, device=dev) if n else None

    ws = {(p, dn): ws_for(p, dn) for p in (0, 1, 2) for dn in (False, True)}
    ws_dy = ws_for(st.ST_PASS_BWW_DY, False)
    ws_auto = ws_for(st.ST_PASS_BWW_AUTO, False)
    ws_fauto, ws_bauto = ws_for(st.ST_PASS_FWD_AUTO, False), ws_for(st.ST_PASS_BWI_AUTO, False)

    def run_pass(name, dense, xin=None, dyin=None):
        xin = xd if xin is None else xin
        dyin = dyd if dyin is None else dyin
        if name == "fwd":
            (st.st_conv_fwd_dense if dense else st.st_conv_fwd)(d, xin, wd, y, ws[0, dense], stream)
        elif name == "bwi":
            (st.st_conv_bwi_dense if dense else st.st_conv_bwi)(d, dyin, wd, dx, ws[1, dense], stream)
        elif name == "bww_dy":          # side measurement: BWW with the zero test on dy (not part of the step)
            st.st_conv_bww_dy(d, xin, dyin, dw, ws_dy, stream)
        elif name == "bww_auto":        # side measurement: BWW that samples both operands and picks one
            st.st_conv_bww_auto(d, xin, dyin, dw, ws_auto, stream)
        elif name == "fwd_auto":        # side measurements: sparse/dense form picked on the device
            st.st_conv_fwd_auto(d, xin, wd, y, ws_fauto, stream)
        elif name == "bwi_auto":
            st.st_conv_bwi_auto(d, dyin, wd, dx, ws_bauto, stream)
        else:
            (st.st_conv_bww_dense if dense else st.st_conv_bww)(d, xin, dyin, dw, ws[2, dense], stream)

    def step():
        run_pass("fwd", False)
        run_pass("bwi", False)
        run_pass("bww", False)

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)              # one elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    # ---- the timed region: W warm-up steps, then exactly K steps ----
    sustain(step, args.clock_warm_ms, stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = 3 * F / (ms_per_step * 1e-3) / 1e12

    # ---- per-pass timing with events on the launch stream ----
    def time_pass(name, dense, iters, xin=None, dyin=None, warm=2):
        sustain(lambda: run_pass(name, dense, xin, dyin), args.sustain_ms, stream)
        for _ in range(warm):
            run_pass(name, dense, xin, dyin)
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
        for a, b in evs:
            a.record(stream)
            run_pass(name, dense, xin, dyin)
            b.record(stream)
        torch.cuda.synchronize()
        ts = sorted(a.elapsed_time(b) for a, b in evs)
        return ts[len(ts) // 2], sum(ts) / len(ts)

    tested_p = {"fwd": px, "bwi": pdy, "bww": px}
    passes = {}
    for name in ("fwd", "bwi", "bww"):
        s_med, s_avg = time_pass(name, False, args.steps)
        d_med, d_avg = time_pass(name, True, args.steps)
        passes[name] = {
            "sparse_ms": round(s_med, 4), "dense_ms": round(d_med, 4),
            "sparse_avg_ms": round(s_avg, 4),
            "speedup_vs_dense": round(d_med / s_med, 3),
            "effective_tflops": round(F / (s_med * 1e-3) / 1e12, 2),
            "executed_tflops": round(F * (1 - tested_p[name]) / (s_med * 1e-3) / 1e12, 2),
            "dense_tflops": round(F / (d_med * 1e-3) / 1e12, 2),
            "dense_frac_of_mfma_peak": round(F / (d_med * 1e-3) / 1e12 / PEAK_FP32_MFMA, 3),
            "tested_zero_fraction": round(tested_p[name], 4),
        }

    dy_med, _ = time_pass("bww_dy", False, args.steps)
    passes["bww"]["tests_dy_ms"] = round(dy_med, 4)
    passes["bww"]["tests_dy_zero_fraction"] = round(pdy, 4)
    passes["bww"]["auto_select_ms"] = round(time_pass("bww_auto", False, args.steps)[0], 4)
    passes["fwd"]["auto_select_ms"] = round(time_pass("fwd_auto", False, args.steps)[0], 4)
    passes["bwi"]["auto_select_ms"] = round(time_pass("bwi_auto", False, args.steps)[0], 4)

    # side measurement: the same zero fraction of x arranged as whole dead (image, channel) planes
    xdead_h = stgen.dead_channels(stgen.relu_sparse((L.N, L.C, L.H, L.W), 0.0, 200), px, 201)
    xdead = torch.from_numpy(st.pack_activations(xdead_h)).to(dev)
    passes["fwd"]["dead_channel_pattern"] = {
        "zero_fraction": round(stgen.zero_fraction(xdead_h), 4),
        "sparse_ms": round(time_pass("fwd", False, args.steps, xdead)[0], 4)}
    del xdead, xdead_h

    # ---- roofline of the dominant kernel ----
    # FWD is one launch of the zero-skipping tile kernel (BWI launches the same kernel on dy) behind a
    # filter-copy launch of about 5 us (1-2 % of the call), so the event time of st_conv_fwd is that
    # kernel's launch duration plus the copy: the fraction below is the slightly pessimistic one.
    # Algorithmic work per launch: F * (1 - realised zero fraction) flops on the vector ALUs.
    dom = max(passes, key=lambda k: passes[k]["sparse_avg_ms"])
    fwd_avg_ms = passes["fwd"]["sparse_avg_ms"]
    achieved = F * (1 - px) / (fwd_avg_ms * 1e-3) / 1e12
    roofline = {
        "kernel": "fwd_sparse_kernel<3,3,4,8,2,4,4,1,1,0> (st_conv_fwd incl. its 5 us filter copy; st_conv_bwi runs the same kernel on dy)",
        "bound": "alu", "achieved": round(achieved, 2), "peak": PEAK_FP32_VECTOR, "unit": "TFLOP/s",
        "frac": round(achieved / PEAK_FP32_VECTOR, 4),
        "peak_unpacked_fma": PEAK_FP32_FMA, "frac_of_unpacked_fma_peak": round(achieved / PEAK_FP32_FMA, 4),
        "avg_launch_ms": fwd_avg_ms, "algorithmic_flops_per_launch": F * (1 - px),
        "traffic": MEASURED_TRAFFIC_BYTES, "algorithmic_bytes_per_launch": 4 * (x_h.size + w_h.size + x_h.size * L.K // L.C),
        "slowest_pass": dom,
    }

    # ---- sparse-over-dense speedup at 0-90 % zeros ----
    sweep = []
    if not args.no_sweep:
        for p in (0.0, 0.3, 0.5, 0.7, 0.9):
            xs_h = stgen.relu_sparse((L.N, L.C, L.H, L.W), p, 100)
            dys_h = stgen.bernoulli_masked((L.N, L.K, L.OH, L.OW), p, 102, 103)
            xs = torch.from_numpy(st.pack_activations(xs_h)).to(dev)
            dys = torch.from_numpy(st.pack_activations(dys_h)).to(dev)
            row = {"zero_fraction": p}
            for name in ("fwd", "bwi", "bww"):
                s_med, _ = time_pass(name, False, args.sweep_iters, xs, dys, warm=1)
                d_med, _ = time_pass(name, True, args.sweep_iters, xs, dys, warm=1)
                row[name] = {"sparse_ms": round(s_med, 4), "dense_ms": round(d_med, 4),
                             "speedup": round(d_med / s_med, 3),
                             "effective_tflops": round(F / (s_med * 1e-3) / 1e12, 2)}
            row["bww"]["tests_dy_ms"] = round(time_pass("bww_dy", False, args.sweep_iters, xs, dys, warm=1)[0], 4)
            row["fwd"]["auto_select_ms"] = round(time_pass("fwd_auto", False, args.sweep_iters, xs, dys, warm=1)[0], 4)
            row["bwi"]["auto_select_ms"] = round(time_pass("bwi_auto", False, args.sweep_iters, xs, dys, warm=1)[0], 4)
            sweep.append(row)
            del xs, dys

    # ---- CPU oracle on a bounded sample of the same workload ----
    cpu = None
    if not args.no_cpu:
        from oracle import st_ref

        def oracle_step(n_img):
            g = st_ref.Geom(n_img, L.C, L.K, L.H, L.W, L.R, L.S, 1, 1, L.pad, L.pad)
            xs_, dys_ = x_h[:n_img], dy_h[:n_img]
            t = time.perf_counter()
            st_ref.conv_fwd(g, xs_, w_h)
            st_ref.conv_bwi(g, dys_, w_h)
            st_ref.conv_bww(g, xs_, dys_)
            return time.perf_counter() - t, 3 * g.flops

        t1img, f1 = oracle_step(1)
        n_img = int(max(1, min(L.N, 15.0 // max(t1img, 1e-3))))
        if n_img > 1:
            tt, ff = oracle_step(n_img)
        else:
            tt, ff = t1img, f1
        cpu = {"value": round(ff / tt / 1e12, 5), "unit": "TFLOP/s", "cores": st_ref.threads(), "kind": "oracle",
               "sample": f"FWD+BWI+BWW of the first {n_img} of {L.N} images of the same tensors, "
                         f"{tt:.2f} s of wall time; dense-equivalent flops / time"}

    if args.table:
        write_config_table(args.table, st, stgen, torch, dev, stream, args.sustain_ms)

    out = {
        "metric": "effective conv TFLOP/s (FWD+BWI+BWW, zero-skipping entry points)",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "clock_warm_ms": args.clock_warm_ms,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "vgg3_2-shaped 3x3 conv layer N=16 C=256 K=256 56x56 stride 1 pad 1; "
                               "x ReLU-shifted Gaussian, dy Bernoulli-masked Gaussian, He-normal filters, seed 0",
                   "zero_fraction_x": round(px, 4), "zero_fraction_dy": round(pdy, 4),
                   "flops_per_pass": F},
        "passes": passes,
        "roofline": roofline,
        "cpu_baseline": cpu,
        "sweep": sweep,
        "paper_context": "SparseTrain reports 2.19x/1.37x/1.31x/1.51x projected conv-training speedups for "
                         "VGG16/ResNet-34/ResNet-50/Fixup ResNet-50 on a 6-core Skylake-X CPU (Table 5); "
                         "other machine, not a target",
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
