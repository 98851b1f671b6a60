#!/usr/bin/env python3
"""Benchmark of the zero-skipping convolution passes on one MI355X.

Workload: the VGG16 non-initial convolution stack of the paper's Table 1 at minibatch 32 (twelve 3x3
layers, stride 1, pad 1: 64-64 @224, 64-128 @112, 128-128 @112, 128-256 @56, 256-256 @56 x2,
256-512 @28, 512-512 @28 x2, 512-512 @14 x3) with synthetic inputs: x = ReLU-shifted Gaussian,
dy = Bernoulli-masked Gaussian, He-normal filters, the zero fraction of x and of dy swept over
{0, 30, 50, 70, 90} % (the experiment of Sec. 5.1 / Table 3 of the paper, which used minibatch 16).

A step is one pass of the whole hot path -- st_conv_fwd, st_conv_bwi, st_conv_bww of every layer of the
stack -- at the headline zero fraction (--level, default 50 %), all tensors resident in HBM before the
timed region.  Prints ONE JSON line.  value = effective (dense-equivalent) TFLOP/s of the step,
3 * sum_layers 2*N*K*C*OH*OW*R*S / step time.  Extra objects: "sweep" (per zero fraction: time of the
zero-skipping entry points and of the dense controls per layer and pass, and the stack's speed-up),
"roofline" (the kernel that takes most of the step), "cpu_baseline" (the CPU oracle on one image of
every layer), "other_configs" (the single-layer workloads of the benchmark definition, the 1x1 layers
also with cold caches).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X peaks (TFLOP/s).  fp32 vector: 256 CU x 4 SIMD x 32 lanes/clk x 2 flop x 2.4 GHz; a stream of
# independent v_fmac_f32 from two or more wavefronts per SIMD measures 141 TFLOP/s (one wave-wide
# instruction every 2 cycles at the ~2.15 GHz the chip sustains under that load; see
# profiles/valu_fma_rate.md), so the published figure is the ceiling of plain, unpacked FMAs too.
PEAK_FP32_VECTOR = 157.3
PEAK_FP32_MFMA = 157.3
PEAK_HBM_TBS = 8.0
LEVELS = (0.0, 0.3, 0.5, 0.7, 0.9)
# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (not read in this
# run: the figure and how it was scaled are in the file named here); None until such a run exists for the kernel
TRAFFIC_SOURCE = "profiles/vgg16_stack_step_hbm_traffic.md"
TRAFFIC_BYTES_PER_LAUNCH = {
    "fwd_sparse_kernel<3, 3, 7, 7, 1, 4, 2, 1, 1, 0>": 656477168,
    "bww_sparse_kernel<3, 3, 7, 8, 0>": 343440616,
    "fwd_sparse_kernel<3, 3, 4, 7, 2, 4, 2, 1, 1, 0>": 332792674,
    "fwd_sparse_kernel<3, 3, 4, 7, 2, 4, 4, 1, 1, 0>": 215813771,
}
CPU_IMAGES = 4          # images per layer the CPU oracle is timed on (of the minibatch of 32): 10-20 s of work


def sustain(fn, ms):
    """Keeps the GPU busy with fn for about ms milliseconds (untimed).  After an idle spell of 50 ms or
    more the chip needs some 30 ms of continuous work to return to its sustained clocks; every timing
    below starts from that state, which is the one a training run is in."""
    import torch
    t0 = time.perf_counter()
    while True:
        for _ in range(2):
            fn()
        torch.cuda.current_stream().synchronize()
        if (time.perf_counter() - t0) * 1e3 >= ms:
            return


def time_call(fn, iters, sustain_ms, stream):
    """(median, mean) milliseconds of fn over iters launches, HIP events on the launch stream."""
    import torch
    sustain(fn, sustain_ms)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(iters)]
    for a, b in evs:
        a.record(stream)
        fn()
        b.record(stream)
    torch.cuda.synchronize()
    ts = sorted(a.elapsed_time(b) for a, b in evs)
    return ts[len(ts) // 2], sum(ts) / len(ts)


class LayerOnDevice:
    """One layer: the random draws behind x and dy (fp64, blocked layout) stay on the device, so that the
    tensors of any zero fraction are one elementwise pass away; outputs and workspaces are allocated once."""

    def __init__(self, layer, seed, st, stgen, torch, dev, keep_host_image=True):
        import numpy as np
        self.L, self.st, self.torch = layer, st, torch
        L = layer
        self.d = st.ConvDesc(L.N, L.C, L.K, L.H, L.W, L.R, L.S, L.stride, L.stride, L.pad, L.pad)
        self.F = self.d.flops
        xs, ys = (L.N, L.C, L.H, L.W), (L.N, L.K, L.OH, L.OW)
        z = stgen.normal(4 * seed, int(np.prod(xs))).reshape(xs)
        g = stgen.normal(4 * seed + 2, int(np.prod(ys))).reshape(ys)
        u = stgen.uniform(4 * seed + 3, int(np.prod(ys))).reshape(ys)
        self.w_host = stgen.he_normal((L.K, L.C, L.S, L.R), 4 * seed + 1)
        # first image of every tensor, for the CPU baseline and for the check of the on-device derivation
        self.host0 = (z[:CPU_IMAGES].copy(), g[:CPU_IMAGES].copy(), u[:CPU_IMAGES].copy()) if keep_host_image else None
        self.z = torch.from_numpy(st.pack_activations(z)).to(dev)
        self.g = torch.from_numpy(st.pack_activations(g)).to(dev)
        self.u = torch.from_numpy(st.pack_activations(u)).to(dev)
        del z, g, u
        self.w = torch.from_numpy(st.pack_filters(self.w_host)).to(dev)
        self.x = torch.empty(self.z.shape, dtype=torch.float32, device=dev)
        self.dy = torch.empty(self.g.shape, dtype=torch.float32, device=dev)
        self.y = torch.empty_like(self.dy)
        self.dx = torch.empty_like(self.x)
        self.dw = torch.empty_like(self.w)
        self.ws = {}
        for p in (st.ST_PASS_FWD, st.ST_PASS_BWI, st.ST_PASS_BWW):
            for dense in (False, True):
                n = st.st_conv_workspace_bytes(self.d, p, dense)
                self.ws[p, dense] = torch.empty(max(n, 4) // 4, dtype=torch.float32, device=dev) if n else None
        self.px = self.pdy = None

    def set_level(self, p, stgen):
        """x = max(0, z - t) and dy = g * (u >= p), computed in fp64 and rounded once to fp32: the same
        bits as stgen.relu_from_normal / stgen.mask_from_uniform give on the host."""
        torch = self.torch
        if p <= 0.0:
            self.x.copy_(self.z)
            self.dy.copy_(self.g)
        else:
            self.x.copy_(torch.clamp_min(self.z - stgen.relu_threshold(p), 0.0))
            self.dy.copy_(self.g.to(torch.float32) * (self.u >= p).to(torch.float32))
        self.px = float((self.x == 0).sum()) / self.x.numel()
        self.pdy = float((self.dy == 0).sum()) / self.dy.numel()

    def check_derivation(self, p, stgen):
        """The first image of x and dy on the device against the host generator (bit for bit)."""
        import numpy as np
        z0, g0, u0 = self.host0
        x0 = self.st.pack_activations(stgen.relu_from_normal(z0, p))
        dy0 = self.st.pack_activations(stgen.mask_from_uniform(g0, u0, p))
        n0 = x0.shape[0]
        ok = np.array_equal(self.x[:n0].cpu().numpy().view(np.uint32), x0.view(np.uint32)) and \
            np.array_equal(self.dy[:n0].cpu().numpy().view(np.uint32), dy0.view(np.uint32))
        assert ok, f"{self.L.name}: device-derived inputs differ from the host generator at p={p}"

    def run(self, name, dense, stream):
        st, d = self.st, self.d
        if name == "fwd":
            (st.st_conv_fwd_dense if dense else st.st_conv_fwd)(d, self.x, self.w, self.y, self.ws[0, dense], stream)
        elif name == "bwi":
            (st.st_conv_bwi_dense if dense else st.st_conv_bwi)(d, self.dy, self.w, self.dx, self.ws[1, dense], stream)
        else:
            (st.st_conv_bww_dense if dense else st.st_conv_bww)(d, self.x, self.dy, self.dw, self.ws[2, dense], stream)


def single_layer_config(label, layer, seed, st, stgen, torch, dev, stream, iters, sustain_ms, cold=False):
    """Sparse and dense time of the three passes of one layer on stgen inputs at the layer's own zero
    fractions; cold = True also times the 1x1 layers over rotating buffer sets larger than the 256 MB
    last-level cache."""
    Ld = LayerOnDevice(layer, seed, st, stgen, torch, dev, keep_host_image=False)
    L = layer
    # the layer's own zero fractions differ for x and dy
    t = stgen.relu_threshold(L.p_x) if L.p_x > 0 else None
    Ld.x.copy_(Ld.z if t is None else torch.clamp_min(Ld.z - t, 0.0))
    Ld.dy.copy_(Ld.g.to(torch.float32) * (Ld.u >= L.p_dy).to(torch.float32) if L.p_dy > 0 else Ld.g)
    px = float((Ld.x == 0).sum()) / Ld.x.numel()
    pdy = float((Ld.dy == 0).sum()) / Ld.dy.numel()
    out = {"layer": f"{L.name} {L.C}->{L.K} @{L.H} {L.R}x{L.S} N={L.N}", "zero_fraction_x": round(px, 4),
           "zero_fraction_dy": round(pdy, 4), "flops_per_pass": Ld.F}
    d = Ld.d
    autos = {"fwd": (st.st_conv_fwd_auto, st.ST_PASS_FWD_AUTO, lambda: (Ld.x, Ld.w, Ld.y)),
             "bwi": (st.st_conv_bwi_auto, st.ST_PASS_BWI_AUTO, lambda: (Ld.dy, Ld.w, Ld.dx)),
             "bww": (st.st_conv_bww_auto, st.ST_PASS_BWW_AUTO, lambda: (Ld.x, Ld.dy, Ld.dw))}
    for name, tested in (("fwd", px), ("bwi", pdy), ("bww", px)):
        s, _ = time_call(lambda: Ld.run(name, False, stream), iters, sustain_ms, stream)
        dn, _ = time_call(lambda: Ld.run(name, True, stream), iters, sustain_ms, stream)
        # the self-selecting entry point against the faster of the two direct calls
        fn, pa, ops = autos[name]
        nws = st.st_conv_workspace_bytes(d, pa, False)
        wsa = torch.empty(max(nws, 4) // 4, dtype=torch.float32, device=dev) if nws else None
        a, b, o = ops()
        au, _ = time_call(lambda: fn(d, a, b, o, wsa, stream), iters, sustain_ms, stream)
        out[name] = {"sparse_ms": round(s, 4), "dense_ms": round(dn, 4), "speedup": round(dn / s, 3),
                     "effective_tflops": round(Ld.F / s / 1e9, 2), "auto_ms": round(au, 4),
                     "auto_over_faster_form": round(au / min(s, dn), 3)}
        del wsa
    if cold:
        # rotate over enough copies of (input, output) that a launch never finds its tensors in the cache
        per_set = (Ld.x.numel() + Ld.y.numel()) * 4
        copies = max(2, int(768e6 // per_set) + 1)
        xs = [Ld.x.clone() for _ in range(copies)]
        dys = [Ld.dy.clone() for _ in range(copies)]
        ys = [torch.empty_like(Ld.y) for _ in range(copies)]
        dxs = [torch.empty_like(Ld.dx) for _ in range(copies)]
        d = Ld.d
        for name, dense, fn in (("fwd", False, st.st_conv_fwd), ("fwd", True, st.st_conv_fwd_dense),
                                ("bwi", False, st.st_conv_bwi), ("bwi", True, st.st_conv_bwi_dense)):
            state = {"i": 0}

            def call():
                i = state["i"] = (state["i"] + 1) % copies
                if name == "fwd":
                    fn(d, xs[i], Ld.w, ys[i], Ld.ws[0, dense], stream)
                else:
                    fn(d, dys[i], Ld.w, dxs[i], Ld.ws[1, dense], stream)

            m, _ = time_call(call, max(iters, 2 * copies), sustain_ms, stream)
            out[name]["cold_dense_ms" if dense else "cold_sparse_ms"] = round(m, 4)
        bytes_moved = {"fwd": (Ld.x.numel() + Ld.y.numel() + Ld.w.numel()) * 4,
                       "bwi": (Ld.dy.numel() + Ld.dx.numel() + Ld.w.numel()) * 4}
        for name in ("fwd", "bwi"):
            out[name]["cold_dense_hbm_frac"] = round(bytes_moved[name] / (out[name]["cold_dense_ms"] * 1e-3) / 1e12 / PEAK_HBM_TBS, 3)
            out[name]["cold_sparse_hbm_frac"] = round(bytes_moved[name] / (out[name]["cold_sparse_ms"] * 1e-3) / 1e12 / PEAK_HBM_TBS, 3)
        out["cold_buffer_sets"] = copies
    return out


def write_table1(path, st, stgen, torch, dev, stream, sustain_ms=30.0, iters=7):
    """Every row of the paper's Table 1 at 50 % zeros (N=32; vgg1_2 as in the stack): all entry points."""
    rows = []
    tot = [0.0, 0.0, 0.0, 0.0]
    for i, L in enumerate(stgen.table1_layers(32, 0.5, 0.5)):
        Ld = LayerOnDevice(L, 300 + i, st, stgen, torch, dev, keep_host_image=False)
        Ld.set_level(0.5, stgen)
        d = Ld.d
        wsa = {}
        for p in (st.ST_PASS_FWD_AUTO, st.ST_PASS_BWI_AUTO, st.ST_PASS_BWW_AUTO, st.ST_PASS_BWW_DY):
            n = st.st_conv_workspace_bytes(d, p, False)
            wsa[p] = torch.empty(max(n, 4) // 4, dtype=torch.float32, device=dev) if n else None
        label = f"{L.name} {L.C}->{L.K} @{L.H} {L.R}x{L.S}" + (f"/{L.stride}" if L.stride != 1 else "")
        for name, auto, a, b, o, pa, z in (("fwd", st.st_conv_fwd_auto, Ld.x, Ld.w, Ld.y, st.ST_PASS_FWD_AUTO, Ld.px),
                                           ("bwi", st.st_conv_bwi_auto, Ld.dy, Ld.w, Ld.dx, st.ST_PASS_BWI_AUTO, Ld.pdy),
                                           ("bww", st.st_conv_bww_auto, Ld.x, Ld.dy, Ld.dw, st.ST_PASS_BWW_AUTO, Ld.px)):
            ts, _ = time_call(lambda: Ld.run(name, False, stream), iters, sustain_ms, stream)
            td, _ = time_call(lambda: Ld.run(name, True, stream), iters, sustain_ms, stream)
            ta, _ = time_call(lambda: auto(d, a, b, o, wsa[pa], stream), iters, sustain_ms, stream)
            best = min(ts, td)
            extra = ""
            if name == "bww":
                ty, _ = time_call(lambda: st.st_conv_bww_dy(d, Ld.x, Ld.dy, Ld.dw, wsa[st.ST_PASS_BWW_DY], stream),
                                  iters, sustain_ms, stream)
                best = min(best, ty)
                extra = f"{ty * 1e3:.0f}"
            eff = Ld.F / ts / 1e9
            # every tensor of the pass once: the HBM roofline of the dense control (what bounds the 1x1 layers)
            nbytes = 4 * (Ld.x.numel() + Ld.dy.numel() + Ld.w.numel())
            rows.append(f"| {label} | {name.upper()} | {z:.2f} | {ts * 1e3:.0f} | {td * 1e3:.0f} | {ta * 1e3:.0f} | {extra} | "
                        f"{eff:.1f} | {eff * (1 - z) / PEAK_FP32_VECTOR:.3f} | {Ld.F / td / 1e9 / PEAK_FP32_MFMA:.3f} | "
                        f"{nbytes / td / 1e9 / PEAK_HBM_TBS:.3f} | {td / ts:.2f} | {ta / best:.2f} |")
            for k, v in enumerate((ts, td, ta, best)):
                tot[k] += v * 1e3
        del Ld
        torch.cuda.empty_cache()
    with open(path, "w") as f:
        f.write("# Every layer of the paper's Table 1 at 50 % zeros, N=32: `python bench.py --no-cpu --no-sweep --table1 <this file>` on one MI355X\n\n"
                "Median of 7 launches (HIP events) per entry point after 30 ms of the same launch; stgen inputs (x ReLU-shifted\n"
                "Gaussian, dy Bernoulli-masked Gaussian, both 50 % zeros). sparse = st_conv_fwd/bwi/bww (BWW tests x),\n"
                "auto = st_conv_*_auto, BWW(dy) = st_conv_bww_dy; dense HBM = bytes of every tensor of the pass once / dense time /\n"
                "8 TB/s; auto / fastest = the self-selecting entry point against the fastest direct call of the row.\n\n")
        f.write("| layer | pass | zeros of tested operand | sparse us | dense us | auto us | BWW(dy) us | effective TFLOP/s | "
                "executed / 157.3 | dense / 157.3 (MFMA peak) | dense HBM | speed-up | auto / fastest |\n"
                "|---|---|---|---|---|---|---|---|---|---|---|---|---|\n")
        f.write("\n".join(rows) + "\n")
        f.write(f"\nSums over all rows (us): zero-skipping {tot[0]:.0f}, dense {tot[1]:.0f}, auto {tot[2]:.0f}, "
                f"fastest form per row {tot[3]:.0f}; dense / auto = {tot[1] / tot[2]:.2f}.\n")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--level", type=float, default=0.5, help="zero fraction of x and dy in the timed step")
    ap.add_argument("--minibatch", type=int, default=32, help="N of the VGG16 stack (32 in the benchmark definition)")
    ap.add_argument("--sustain-ms", type=float, default=25.0,
                    help="untimed spell of the launch about to be timed, before every per-pass timing")
    ap.add_argument("--clock-warm-ms", type=float, default=200.0,
                    help="untimed spell of continuous steps before the warm-up steps (sustained clocks)")
    ap.add_argument("--no-sweep", action="store_true", help="only the headline zero fraction, no 0-90 %% sweep")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-other", action="store_true", help="skip the single-layer workloads")
    ap.add_argument("--sweep-iters", type=int, default=5)
    ap.add_argument("--only-step", action="store_true",
                    help="run only warm-up and timed steps (the command profiled for profiles/)")
    ap.add_argument("--profile-layer", metavar="NAME", default=None,
                    help="run only one layer of the stack (e.g. vgg3_2): --steps launches of the entry point named by "
                         "--profile-pass at --level; the command rocprofv3 counter runs are made with")
    ap.add_argument("--profile-pass", choices=("fwd", "bwi", "bww"), default="fwd")
    ap.add_argument("--profile-dense", action="store_true", help="with --profile-layer: the dense control instead")
    ap.add_argument("--probe-valu", action="store_true",
                    help="measure the issue rate of bare v_fmac_f32 / MFMA streams (st_probe_issue_rate) and exit")
    ap.add_argument("--table1", metavar="FILE", default=None,
                    help="also time every row of the paper's Table 1 at 50 %% zeros and write a markdown table to FILE")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device-to-device copy kernel (reference for rocprofv3 "
                         "FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (one MI355X per box); --gpus must be 1",
              file=sys.stderr)
        sys.exit(2)
    if args.only_step:
        args.no_sweep = args.no_cpu = args.no_other = True

    import numpy as np
    import torch

    import paper_1911_10175_amd as st
    import stgen

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    st.load_library()
    stream = torch.cuda.current_stream()
    t_start = time.perf_counter()

    if args.copy_calibration:
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)              # one elementwise copy kernel: reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    if args.probe_valu:
        out = torch.empty(256 * 16 * 256, dtype=torch.float32, device=dev)
        res = {}
        names = {0: "fmac_value_changes_every_instruction", 1: "fmac_same_value_first_source_x9",
                 2: "fmac_same_value_second_source_x9", 3: "mfma_f32_32x32x2",
                 4: "fmac_all_three_registers_even", 5: "fmac_second_factor_in_odd_registers"}
        iters = 16000
        for pattern in (0, 1, 2, 3, 4, 5):
            for wps in (1, 2, 4):
                wgs = 256 * wps
                it = iters if pattern != 3 else iters // 8
                call = lambda: st.st_probe_issue_rate(pattern, wgs, it, out, stream)
                med, _ = time_call(call, 7, 300.0 if (pattern, wps) == (0, 1) else 30.0, stream)
                fl = (2.0 * 64 * 63 if pattern != 3 else 4096.0 * 4) * it * 4 * wgs
                res[f"{names[pattern]}@{wps}_waves_per_simd"] = round(fl / med / 1e9, 1)
        print(json.dumps({"probe": "st_probe_issue_rate", "unit": "TFLOP/s", "results": res}))
        return

    if args.profile_layer:
        # a layer of the timed stack, or any other row of the paper's Table 1 (ResNet-50: 1x1 and stride-2 layers)
        pool = stgen.vgg16_stack(args.level, args.minibatch)
        pool += [l for l in stgen.table1_layers(args.minibatch, args.level, args.level) if l.name not in {q.name for q in pool}]
        names = [l.name for l in pool]
        if args.profile_layer not in names:
            sys.exit(f"--profile-layer: unknown layer {args.profile_layer!r}; one of {', '.join(names)}")
        idx = names.index(args.profile_layer)
        L = pool[idx]
        Ld = LayerOnDevice(L, 10 + idx, st, stgen, torch, dev, keep_host_image=False)
        Ld.set_level(args.level, stgen)
        call = lambda: Ld.run(args.profile_pass, args.profile_dense, stream)
        sustain(call, args.clock_warm_ms)
        for _ in range(args.warmup):
            call()
        med, avg = time_call(call, args.steps, 0.0, stream)
        tested = Ld.pdy if args.profile_pass == "bwi" else Ld.px
        print(json.dumps({"layer": L.name, "N": L.N, "pass": args.profile_pass, "dense": args.profile_dense,
                          "zero_fraction_tested": round(tested, 4), "median_ms": round(med, 4), "avg_ms": round(avg, 4),
                          "flops": Ld.F, "executed_tflops": round(Ld.F * (1 - (0 if args.profile_dense else tested)) / avg / 1e9, 2)}))
        return

    # ---- inputs: the twelve layers, draws resident on the device ----
    stack = [LayerOnDevice(L, 10 + i, st, stgen, torch, dev) for i, L in enumerate(stgen.vgg16_stack(args.level, args.minibatch))]
    F_stack = sum(Ld.F for Ld in stack)
    t_inputs = time.perf_counter() - t_start

    def set_level(p):
        for Ld in stack:
            Ld.set_level(p, stgen)
        torch.cuda.synchronize()

    set_level(args.level)
    for Ld in (stack[0], stack[4], stack[-1]):
        Ld.check_derivation(args.level, stgen)

    def step():
        for Ld in stack:
            Ld.run("fwd", False, stream)
            Ld.run("bwi", False, stream)
            Ld.run("bww", False, stream)

    # ---- the timed region: W warm-up steps, then exactly K steps ----
    sustain(step, args.clock_warm_ms)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    value = 3 * F_stack / (ms_per_step * 1e-3) / 1e12

    # ---- per layer and pass, at every swept zero fraction: zero-skipping entry point and dense control ----
    def measure_level(p, iters):
        set_level(p)
        rows = []
        for Ld in stack:
            row = {"layer": Ld.L.name, "zero_fraction_x": round(Ld.px, 4), "zero_fraction_dy": round(Ld.pdy, 4)}
            for name in ("fwd", "bwi", "bww"):
                s_med, s_avg = time_call(lambda: Ld.run(name, False, stream), iters, args.sustain_ms, stream)
                d_med, _ = time_call(lambda: Ld.run(name, True, stream), iters, args.sustain_ms, stream)
                row[name] = {"sparse_ms": round(s_med, 4), "dense_ms": round(d_med, 4), "sparse_avg_ms": round(s_avg, 4)}
            rows.append(row)
        tot = {}
        for name in ("fwd", "bwi", "bww"):
            s = sum(r[name]["sparse_ms"] for r in rows)
            dn = sum(r[name]["dense_ms"] for r in rows)
            tot[name] = {"sparse_ms": round(s, 3), "dense_ms": round(dn, 3), "speedup": round(dn / s, 3),
                         "effective_tflops": round(F_stack / s / 1e9, 1),
                         "dense_tflops": round(F_stack / dn / 1e9, 1),
                         "layers_where_sparse_wins": sum(1 for r in rows if r[name]["sparse_ms"] < r[name]["dense_ms"])}
        s_all = sum(tot[n]["sparse_ms"] for n in tot)
        d_all = sum(tot[n]["dense_ms"] for n in tot)
        return {"zero_fraction": p, "stack_sparse_ms": round(s_all, 3), "stack_dense_ms": round(d_all, 3),
                "stack_speedup": round(d_all / s_all, 3), "effective_tflops": round(3 * F_stack / s_all / 1e9, 1),
                "passes": tot, "layers": rows}

    sweep = []
    headline = None
    if not args.only_step:
        levels = (args.level,) if args.no_sweep else tuple(sorted(set(LEVELS) | {args.level}))
        for p in levels:
            rec = measure_level(p, args.steps if p == args.level else args.sweep_iters)
            sweep.append(rec)
            if p == args.level:
                headline = rec
        set_level(args.level)

    # ---- roofline of the kernel that takes most of the step ----
    # st_conv_fwd and st_conv_bwi both launch fwd_sparse_kernel (BWI on dy with the transposed filter copy), one
    # launch per call behind a filter-copy launch of 2-6 us that the event time includes (the fraction is that
    # much pessimistic).  The launches of the step are grouped by kernel instance (st_conv_kernel_name); the
    # instance with the most time is the dominant kernel.  Algorithmic work of a launch: F * (1 - realised zero
    # fraction of the tested operand) flops on the vector ALUs; bytes: every tensor element once.
    roofline = None
    if headline is not None:
        groups = {}
        for Ld, r in zip(stack, headline["layers"]):
            for n, pid, tested in (("fwd", st.ST_PASS_FWD, Ld.px), ("bwi", st.ST_PASS_BWI, Ld.pdy)):
                name = st.st_conv_kernel_name(Ld.d, pid) or "generic"
                g = groups.setdefault(name, {"ms": 0.0, "flops": 0.0, "bytes": 0, "launches": 0, "calls": []})
                g["ms"] += r[n]["sparse_avg_ms"]
                g["flops"] += Ld.F * (1 - tested)
                g["bytes"] += 4 * (Ld.x.numel() + Ld.y.numel() + Ld.w.numel())
                g["launches"] += 1
                g["calls"].append(f"{Ld.L.name}:{n}")
        t_fb = sum(g["ms"] for g in groups.values())          # FWD and BWI so far
        t_w = sum(r["bww"]["sparse_avg_ms"] for r in headline["layers"])
        fl_w = sum(Ld.F * (1 - Ld.px) for Ld in stack)
        # st_conv_bww: one launch of the zero-skipping kernel plus the final sum of its partial gradients
        # (about 16 us, 2-3 % of the event time: again the pessimistic side)
        for Ld, r in zip(stack, headline["layers"]):
            name = st.st_conv_kernel_name(Ld.d, st.ST_PASS_BWW) or "generic bww"
            g = groups.setdefault(name, {"ms": 0.0, "flops": 0.0, "bytes": 0, "launches": 0, "calls": []})
            g["ms"] += r["bww"]["sparse_avg_ms"]
            g["flops"] += Ld.F * (1 - Ld.px)
            g["bytes"] += 4 * (Ld.x.numel() + Ld.dy.numel() + Ld.w.numel())
            g["launches"] += 1
            g["calls"].append(f"{Ld.L.name}:bww")
        name, dom = max(groups.items(), key=lambda kv: kv[1]["ms"])
        fwd_groups = {k: v for k, v in groups.items() if k.startswith("fwd_sparse")}
        achieved = dom["flops"] / (dom["ms"] * 1e-3) / 1e12
        fam = sum(g["flops"] for g in fwd_groups.values()) / (t_fb * 1e-3) / 1e12
        roofline = {
            "kernel": name, "calls": dom["calls"],
            "bound": "alu", "achieved": round(achieved, 2), "peak": PEAK_FP32_VECTOR, "unit": "TFLOP/s",
            "frac": round(achieved / PEAK_FP32_VECTOR, 4),
            "launches_per_step": dom["launches"], "avg_launch_ms": round(dom["ms"] / dom["launches"], 4),
            "algorithmic_flops_per_launch": dom["flops"] / dom["launches"],
            "algorithmic_bytes_per_launch": dom["bytes"] // dom["launches"],
            "traffic": TRAFFIC_BYTES_PER_LAUNCH.get(name), "traffic_source": TRAFFIC_SOURCE if name in TRAFFIC_BYTES_PER_LAUNCH else None,
            "share_of_step": round(dom["ms"] / (t_fb + t_w), 3),
            "all_fwd_sparse_kernel_instances": {"achieved": round(fam, 2), "frac": round(fam / PEAK_FP32_VECTOR, 4),
                                                "share_of_step": round(t_fb / (t_fb + t_w), 3),
                                                "ms_by_instance": {k: round(v["ms"], 3) for k, v in fwd_groups.items()}},
            "bww_sparse_kernel": {"achieved": round(fl_w / (t_w * 1e-3) / 1e12, 2),
                                  "frac": round(fl_w / (t_w * 1e-3) / 1e12 / PEAK_FP32_VECTOR, 4),
                                  "avg_launch_ms": round(t_w / 12, 4), "share_of_step": round(t_w / (t_fb + t_w), 3)},
        }

    # ---- the single-layer workloads of the benchmark definition ----
    other = None
    if not args.no_other:
        for Ld in stack:
            Ld.z = Ld.g = Ld.u = None          # the draws are no longer needed
        torch.cuda.empty_cache()
        other = {"config2": single_layer_config("config2", stgen.VGG3_2_N16, 0, st, stgen, torch, dev, stream, args.sweep_iters, args.sustain_ms),
                 "config3": single_layer_config("config3", stgen.RESNET3_2, 0, st, stgen, torch, dev, stream, args.sweep_iters, args.sustain_ms),
                 "config4": [single_layer_config("config4", L, 0, st, stgen, torch, dev, stream, args.sweep_iters, args.sustain_ms, cold=L.R == 1)
                             for L in stgen.BOTTLENECK]}
        c4 = other["config4"]
        other["config4_sum"] = {n: {"sparse_ms": round(sum(r[n]["sparse_ms"] for r in c4), 4),
                                    "dense_ms": round(sum(r[n]["dense_ms"] for r in c4), 4)} for n in ("fwd", "bwi", "bww")}

    # ---- CPU oracle on a bounded sample: the first images of every layer, all three passes ----
    cpu = None
    if not args.no_cpu:
        from oracle import st_ref
        t_cpu, f_cpu, done = 0.0, 0, 0
        for Ld in stack:
            L = Ld.L
            z0, g0, u0 = Ld.host0
            n0 = z0.shape[0]
            x0 = stgen.relu_from_normal(z0, args.level)
            dy0 = stgen.mask_from_uniform(g0, u0, args.level)
            g = st_ref.Geom(n0, L.C, L.K, L.H, L.W, L.R, L.S, 1, 1, L.pad, L.pad)
            t = time.perf_counter()
            st_ref.conv_fwd(g, x0, Ld.w_host)
            st_ref.conv_bwi(g, dy0, Ld.w_host)
            st_ref.conv_bww(g, x0, dy0)
            t_cpu += time.perf_counter() - t
            f_cpu += 3 * g.flops
            done += 1
            if t_cpu > 45.0:
                break
        cpu = {"value": round(f_cpu / t_cpu / 1e12, 5), "unit": "TFLOP/s", "cores": st_ref.threads(), "kind": "oracle",
               "sample": f"FWD+BWI+BWW of the first {CPU_IMAGES} of {args.minibatch} images of the first {done} of 12 layers, "
                         f"same tensors as the timed step, {t_cpu:.2f} s of wall time; dense-equivalent flops / time.  "
                         f"Linear extrapolation to the whole step: {t_cpu * (3 * F_stack) / f_cpu:.0f} s",
               "extrapolated_step_s": round(t_cpu * (3 * F_stack) / f_cpu, 1)}

    if args.table1:
        for Ld in stack:
            Ld.z = Ld.g = Ld.u = None
        del stack
        torch.cuda.empty_cache()
        write_table1(args.table1, st, stgen, torch, dev, stream, args.sustain_ms)

    out = {
        "metric": "effective conv TFLOP/s (FWD+BWI+BWW, zero-skipping entry points) + speedup vs dense at 0-90% zeros",
        "value": round(value, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "clock_warm_ms": args.clock_warm_ms, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": f"VGG16 non-initial conv stack (12 layers of Table 1, 3x3 stride 1 pad 1), N={args.minibatch}, "
                               f"x and dy at {args.level:.0%} zeros (x ReLU-shifted Gaussian, dy Bernoulli-masked Gaussian, "
                               f"He-normal filters); step = st_conv_fwd + st_conv_bwi + st_conv_bww of every layer",
                   "zero_fraction": args.level, "flops_per_step": 3 * F_stack, "input_setup_s": round(t_inputs, 1)},
        "stack_speedup_vs_dense": {f"{r['zero_fraction']:.0%}": r["stack_speedup"] for r in sweep},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "sweep": sweep,
        "other_configs": other,
        "paper_context": "SparseTrain Table 3 (3x3 layers, 6-core Skylake-X, N=16): FWD/BWI/BWW 1.38/1.40/1.30x over dense "
                         "direct convolution at 50 % zeros, 2.48/2.45/3.15x at 90 %; projected conv-training speedups "
                         "2.19x/1.37x/1.31x/1.51x for VGG16/ResNet-34/ResNet-50/Fixup ResNet-50 (Table 5); other machine, "
                         "not a target",
        "wall_s": round(time.perf_counter() - t_start, 1),
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
