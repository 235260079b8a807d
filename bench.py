#!/usr/bin/env python3
"""Benchmark of the tc355 hot path on one MI355X.

One "step" = one pass over all four operators at the benchmark configurations
2-5 (tbmm B=500, 3-layer MLP batch 128, grouped convolution 32x512x58x58,
Kronecker layer B=256) with inputs resident in HBM.  Prints ONE JSON line:
whole-step throughput in GFLOP/s (algorithmic flops of the four comprehensions
per step / wall time per step), a per-operator table, the roofline of the
dominant kernel (grouped convolution), and the float64 CPU oracle timed on the
host cores on a bounded sample of the same workload.

Per-operator protocol (Section 7 of the paper times 1000 runs and reports
p0 / p50 / p90): the launches are replayed from HIP graphs, so the figures are
GPU time and not the host's launch rate.  "warm": 20 launches on one buffer set
per replay (the 8 MB working sets of tbmm, the MLP and the Kronecker layer then
sit in the 256 MB Infinity Cache); "cold": one launch on each of 40 rotating
buffer sets per replay (more than 256 MB between two uses of a set), which is
what the HBM fractions are computed from.  Every sample is one replay divided
by its launches; p0 / p50 / p90 are taken over the samples.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

`--sustain SECONDS` (supplementary) runs the grouped convolution, a plain copy
and the whole step back to back and prints the launch time beside the board's
power and clock sensors: the int8 grouped convolution runs at the board's
power limit, so its time depends on what ran in the tens of milliseconds
before it.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published peaks
PEAK_HBM_GBS = 8000.0
PEAK_F64_MFMA_TFLOPS = 78.6
PEAK_F32_MFMA_TFLOPS = 157.3
PEAK_I8_MFMA_TOPS = 5000.0
# The grouped convolution multiplies 4 x 4 signed 8-bit slices of its operands and keeps 10 of the 16 slice products:
# 10 int8 multiply-adds per multiply-add of the comprehension.
GCONV_I8_PRODUCTS = 10


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # The defaults run long enough for the board's power management to settle (the shader clock needs about 50 ms
    # of load to come up from idle and, under the grouped convolution, settles at the 1400 W power limit): the
    # warm-up is 80 ms and the timed region 0.3 s.
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=500)
    ap.add_argument("--op-samples", type=int, default=200,
                    help="graph replays per operator and variant in the per-operator timing (20 or 40 launches each)")
    ap.add_argument("--prewarm-ms", type=float, default=150.0,
                    help="the step is run for this long before the counted warm-up steps, so that the shader clock "
                         "has come up from idle whatever --warmup says")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--scaling", action="store_true",
                    help="supplementary: time tbmm, the MLP and the Kronecker layer at 1x, 8x and 64x the benchmark "
                         "batch (one JSON line per point), to separate launch/latency floors from kernel throughput")
    ap.add_argument("--sustain", type=float, default=0.0, metavar="SECONDS",
                    help="supplementary: run the grouped convolution (both arithmetic paths), a plain copy of its "
                         "input and the whole step back to back for SECONDS each and report the launch time next to "
                         "the board's power, power limit and shader clock (amdgpu sysfs sensors, read-only): one "
                         "JSON line per leg")
    ap.add_argument("--counter-probe", action="store_true",
                    help="for rocprofv3 --pmc: tbmm, MLP and kron on 40 cold buffer sets, tbmm at 64x batch, and a "
                         "calibration copy; no timing")
    ap.add_argument("--traffic-probe", action="store_true",
                    help="only launch the grouped convolution, the largest transposed matmul, the strided convolution and a plain 512 MiB device copy a few times (for "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs; the copy calibrates the counters)")
    return ap.parse_args()


def read_traffic(name):
    """HBM bytes per launch from a committed rocprofv3 --pmc summary, or None."""
    path = os.path.join(ROOT, "profiles", name)
    if not os.path.exists(path):
        return None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return float(m.group(1)) if m else None


def capture(calls):
    """The launches in `calls`, captured on a side stream into one HIP graph (the first two are also run eagerly
    first: one-time set-up such as LDS limits stays outside the capture)."""
    import torch

    st = torch.cuda.Stream()
    st.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(st):
        for c in calls[:2]:
            c()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=st):
            for c in calls:
                c()
    torch.cuda.synchronize()
    return g


def replay_samples(g, launches, samples):
    """`samples` replays of graph g, each timed between two events on the current stream; microseconds per launch."""
    import numpy as np
    import torch

    t_end = time.perf_counter() + 0.05  # 50 ms of the same launches first (shader clock)
    while time.perf_counter() < t_end:
        g.replay()
        torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(samples + 1)]
    ev[0].record()
    for k in range(samples):
        g.replay()
        ev[k + 1].record()
    torch.cuda.synchronize()
    return np.array([ev[k].elapsed_time(ev[k + 1]) * 1e3 / launches for k in range(samples)])


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_1802_04730_amd import inputs, tc355

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    tc355.lib()
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    cfg = {c: {k: v for k, v in inputs.CONFIGS[c].items() if k != "op"} for c in (2, 3, 4, 5)}

    # ---- inputs, resident in HBM before anything is timed
    X, Y = (dev(a) for a in inputs.make_config(2)[1])
    Z = torch.empty((500, 26, 72), device="cuda")
    Ih, Wsh, bsh = inputs.make_config(3)[1]
    I, Ws, bs = dev(Ih), [dev(w) for w in Wsh], [dev(b) for b in bsh]
    dims = cfg[3]["dims"]
    O = [torch.empty((128, d), device="cuda") for d in dims[1:]]
    ws = torch.empty(max(1, tc355.tc_mlp_fcrelu_workspace_bytes(128, dims)), dtype=torch.uint8, device="cuda")
    Ig, W1g, bg = (dev(a) for a in inputs.make_config(4)[1])
    Og = torch.empty((32, 32, 16, 56, 56), device="cuda")
    K1, K2, Xk = (dev(a) for a in inputs.make_config(5)[1])
    Yk = torch.empty((256, 64, 64), device="cuda")

    ops = {
        "tbmm": (lambda: tc355.tc_tbmm(X, Y, Z), inputs.flops_tbmm(**cfg[2]), inputs.bytes_tbmm(**cfg[2])),
        "mlp": (lambda: tc355.tc_mlp_fcrelu(I, Ws, bs, O, ws), inputs.flops_mlp(**cfg[3]), inputs.bytes_mlp(**cfg[3])),
        "gconv": (lambda: tc355.tc_group_conv(Ig, W1g, bg, Og), inputs.flops_gconv(**cfg[4]),
                  inputs.bytes_gconv(**cfg[4])),
        "kron": (lambda: tc355.tc_kron(K1, K2, Xk, Yk), inputs.flops_kron(**cfg[5]), inputs.bytes_kron(**cfg[5])),
    }
    step_flops = sum(v[1] for v in ops.values())

    COLD_SETS = 40

    def cold_calls(name):
        """One launch on each of COLD_SETS copies of the operator's tensors (more than 256 MB in all)."""
        if name == "tbmm":
            sets = [(X.clone(), Y.clone(), torch.empty_like(Z)) for _ in range(COLD_SETS)]
            return sets, [(lambda a=a: tc355.tc_tbmm(*a)) for a in sets]
        if name == "mlp":
            sets = [(I.clone(), [w.clone() for w in Ws], [b.clone() for b in bs], [torch.empty_like(o) for o in O],
                     torch.empty_like(ws)) for _ in range(COLD_SETS)]
            return sets, [(lambda a=a: tc355.tc_mlp_fcrelu(*a)) for a in sets]
        if name == "kron":
            sets = [(K1.clone(), K2.clone(), Xk.clone(), torch.empty_like(Yk)) for _ in range(COLD_SETS)]
            return sets, [(lambda a=a: tc355.tc_kron(*a)) for a in sets]
        return None, None  # gconv: one set is 426 MB already

    if args.scaling:
        scaling_study(torch, tc355, inputs)
        return

    if args.counter_probe:
        # for `rocprofv3 --pmc ... -- python3 bench.py --counter-probe`: every small operator of the step once on each
        # of COLD_SETS buffer sets that no launch has touched since they were written (inputs come from HBM), five
        # times over, the batched matmul at 64 times the benchmark batch, and a plain copy of known size (calibration)
        t_pre = time.perf_counter()
        while (time.perf_counter() - t_pre) < 0.15:   # settle the clock
            for name in ("tbmm", "mlp", "kron"):
                ops[name][0]()
            torch.cuda.synchronize()
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float32, device="cuda")  # 512 MiB read + 512 MiB written
        dst = torch.empty_like(src)
        X64, Y64 = X.repeat(64, 1, 1), Y.repeat(64, 1, 1)
        Z64 = torch.empty((64 * 500, 26, 72), device="cuda")
        out = {"counter_probe": True, "copy_bytes_each_way": src.numel() * 4, "cold_sets": COLD_SETS, "rounds": 5,
               "algorithmic_bytes": {k: ops[k][2] for k in ("tbmm", "mlp", "kron")},
               "tbmm_x64_algorithmic_bytes": 64 * ops["tbmm"][2]}
        for name in ("tbmm", "mlp", "kron"):
            sets, calls = cold_calls(name)
            for _ in range(5):
                dst.copy_(src)               # 1 GiB through the caches: nothing of the sets is left in them
                for c in calls:
                    c()
            torch.cuda.synchronize()
            out[name + "_path"] = tc355.last_path()
            del sets, calls
        for _ in range(5):
            dst.copy_(src)
            tc355.tc_tbmm(X64, Y64, Z64)
        torch.cuda.synchronize()
        print(json.dumps(out), flush=True)
        return

    if args.traffic_probe:
        src = torch.ones(128 * 1024 * 1024, dtype=torch.float32, device="cuda")  # 512 MiB read + 512 MiB written
        dst = torch.empty_like(src)
        # the paper's largest transposed matmul (Section 7, tmm (M,K,N) = (128,4096,16384)) rides along
        Xp = torch.rand((1, 128, 4096), device="cuda") * 2 - 1
        Yp = torch.rand((1, 16384, 4096), device="cuda") * 2 - 1
        Zp = torch.empty((1, 128, 16384), device="cuda")
        # and the strided convolution (Section 3, listing sconv2d) at the size that the full run times
        Isp = torch.randn((32, 64, 56, 56), device="cuda")
        Wsp = torch.randn((128, 64, 3, 3), device="cuda") * 0.05
        bsp = torch.randn((128,), device="cuda") * 0.05
        Osp = torch.empty((32, 128, 27, 27), device="cuda")
        for _ in range(5):
            ops["gconv"][0]()
            dst.copy_(src)
            tc355.tc_tbmm(Xp, Yp, Zp)
            tc355.tc_sconv2d(Isp, Wsp, bsp, Osp, 2, 2)
        torch.cuda.synchronize()
        print(json.dumps({"traffic_probe": True, "copy_bytes_each_way": src.numel() * 4,
                          "gconv_algorithmic_bytes": ops["gconv"][2],
                          "tmm_algorithmic_bytes": 4 * (128 * 4096 + 16384 * 4096 + 128 * 16384),
                          "sconv2d_algorithmic_bytes": inputs.bytes_sconv2d(32, 64, 128, 56, 56, 3, 3, 2, 2)}), flush=True)
        return

    if args.sustain > 0:
        sustained_study(torch, tc355, ops, Ig, (W1g, bg, Og), args.sustain)
        return

    def step(ev=None):
        ops["tbmm"][0]()
        ops["mlp"][0]()
        if ev is not None:
            ev[0].record()
        ops["gconv"][0]()
        if ev is not None:
            ev[1].record()
        ops["kron"][0]()

    # ---- whole-step throughput; the dominant kernel is bracketed by HIP events on the launch stream
    t_pre = time.perf_counter()
    while (time.perf_counter() - t_pre) * 1e3 < args.prewarm_ms:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    prewarm_ms = (time.perf_counter() - t_pre) * 1e3
    for _ in range(args.warmup):
        step()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(evs[k])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    gconv_ms = float(np.mean([a.elapsed_time(b) for a, b in evs]))

    # ---- per-operator GPU time, replayed from HIP graphs: warm (one buffer set) and cold (40 rotating sets)
    def pcts(x):
        return {"us": round(float(x.mean()), 3), "p0": round(float(x.min()), 3), "p50": round(float(np.median(x)), 3),
                "p90": round(float(np.percentile(x, 90)), 3)}

    # A replay of a graph costs about 10 us of its own between two graphs (measured: the 1 x 1 x 1 product below takes
    # 2.18 / 1.82 / 1.69 / 1.63 us per launch with 20 / 50 / 100 / 200 launches per graph), so the graphs of the short
    # operators hold 200 launches; the convolution's (95 us per launch) 20.
    WARM_LAUNCHES, WARM_LAUNCHES_GCONV, COLD_ROUNDS = 200, 20, 5
    # the smallest launch the library makes (one 1 x 1 x 1 product), replayed the same way: the launch floor
    x1, y1, z1 = (torch.zeros((1, 1, 1), device="cuda") for _ in range(3))
    floor = replay_samples(capture([lambda: tc355.tc_tbmm(x1, y1, z1)] * WARM_LAUNCHES), WARM_LAUNCHES, args.op_samples)

    per_op = {}
    for name, (fn, flops, nbytes) in ops.items():
        nl = WARM_LAUNCHES_GCONV if name == "gconv" else WARM_LAUNCHES
        warm = replay_samples(capture([fn] * nl), nl, args.op_samples if name == "gconv" else max(20, args.op_samples // 4))
        sets, calls = cold_calls(name)
        # every buffer set COLD_ROUNDS times per graph: between two launches on one set lie the 39 others (> 256 MB)
        cold = replay_samples(capture(calls * COLD_ROUNDS), COLD_SETS * COLD_ROUNDS, max(20, args.op_samples // 4)) if calls else warm
        del sets, calls
        if name == "gconv":  # int8 matrix pipe on operand slices
            arith, t_mfma = "i8x4", GCONV_I8_PRODUCTS * flops / (PEAK_I8_MFMA_TOPS * 1e12)
        else:
            arith, t_mfma = "f64", flops / (PEAK_F64_MFMA_TFLOPS * 1e12)
        t_hbm = nbytes / (PEAK_HBM_GBS * 1e9)
        bound = "mfma" if t_mfma >= t_hbm else "hbm"
        roof_us = max(t_mfma, t_hbm) * 1e6
        us, cold_us = float(warm.mean()), float(cold.mean())
        per_op[name] = {
            "arith": arith,
            **pcts(warm),
            "cold": pcts(cold),
            "gflops": round(flops / us * 1e-3, 1),
            "gbs_cold": round(nbytes / cold_us * 1e-3, 1),
            "bound": bound,
            "roofline_us": round(roof_us, 3),
            "frac": round(roof_us / cold_us, 4),       # against inputs that come from HBM
            "frac_warm": round(roof_us / us, 4),       # inputs in the Infinity Cache
            "frac_vs_f32_mfma_or_hbm": round(max(flops / (PEAK_F32_MFMA_TFLOPS * 1e12), t_hbm) * 1e6 / cold_us, 4),
            # (roofline time + the time of the smallest launch the library makes) / cold time: what the kernel itself
            # leaves on the table once the launch, which no kernel can shorten, is granted
            "frac_launch_floor_aware": round((roof_us + float(floor.mean())) / cold_us, 4),
        }
    launch_floor = pcts(floor)

    # ---- beyond the step: the paper's largest transposed matmul (Section 7, tmm (M,K,N) = (128,4096,16384)),
    # the one shape of the paper that is bound by the matrix pipe alone; runs through tc_tbmm with B = 1
    Xt = torch.randn((1, 128, 4096), device="cuda")
    Yt = torch.randn((1, 16384, 4096), device="cuda")
    Zt = torch.empty((1, 128, 16384), device="cuda")
    def timed(fn, launches=100):
        """Mean GPU time per launch, microseconds: `launches` launches captured in a HIP graph, replayed 20 times."""
        return float(replay_samples(capture([fn] * launches), launches, 20).mean())

    # the other workloads of the paper's Section 7 tables, through the same entry points
    def entry(us, flops, nbytes):  # fp64 matrix path
        t_mfma, t_hbm = flops / (PEAK_F64_MFMA_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
        return {"us": round(us, 1), "gflops": round(flops / us * 1e-3, 1), "bound": "mfma" if t_mfma >= t_hbm else "hbm",
                "frac": round(max(t_mfma, t_hbm) * 1e6 / us, 4)}

    def entry_i8(us, flops, nbytes, products=13):  # int8 matrix path: `products` int8 multiply-adds per fp32 one
        # (13 digit products in the transposed-matmul and small-image kernels; the benchmark's convolution takes 10
        # wherever its per-band statistic allows, which is everywhere on this data)
        t_mfma, t_hbm = products * flops / (PEAK_I8_MFMA_TOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
        return {"us": round(us, 1), "gflops": round(flops / us * 1e-3, 1), "bound": "mfma_int8" if t_mfma >= t_hbm else "hbm",
                "frac": round(max(t_mfma, t_hbm) * 1e6 / us, 4)}

    tmm_flops, tmm_bytes = inputs.flops_tbmm(1, 128, 16384, 4096), 4 * (128 * 4096 + 16384 * 4096 + 128 * 16384)
    extra = {"tmm_128x4096x16384": entry_i8(timed(lambda: tc355.tc_tbmm(Xt, Yt, Zt)), tmm_flops, tmm_bytes)}
    # the same with X sliced once into a workspace (tc_tbmm_ws: the slicing kernel's launch is part of the time)
    wst = torch.empty(tc355.tc_tbmm_workspace_bytes(1, 128, 16384, 4096), dtype=torch.uint8, device="cuda")
    extra["tmm_128x4096x16384_workspace"] = entry_i8(timed(lambda: tc355.tc_tbmm_ws(Xt, Yt, Zt, wst)), tmm_flops, tmm_bytes)
    with tc355.option(tc355.TC_OPT_INT8, tc355.TC_INT8_OFF):
        extra["tmm_128x4096x16384_fp64_path"] = entry(timed(lambda: tc355.tc_tbmm(Xt, Yt, Zt)), tmm_flops, tmm_bytes)
    for (M_, K_, N_) in [(128, 32, 256), (128, 1024, 1024)]:
        Xt = torch.randn((1, M_, K_), device="cuda")
        Yt = torch.randn((1, N_, K_), device="cuda")
        Zt = torch.empty((1, M_, N_), device="cuda")
        extra["tmm_%dx%dx%d" % (M_, K_, N_)] = entry(timed(lambda: tc355.tc_tbmm(Xt, Yt, Zt)), inputs.flops_tbmm(1, M_, N_, K_),
                                                     4 * (M_ * K_ + N_ * K_ + M_ * N_))
    for name, width in (("mlp1_128x1024x1024", 1024), ("c3_128x1024x1000", 1000)):
        Im = torch.randn((128, 1024), device="cuda")
        Wm = [torch.randn((width, 1024), device="cuda") * 0.02]
        bm = [torch.randn((width,), device="cuda") * 0.01]
        Om = [torch.empty((128, width), device="cuda")]
        extra[name] = entry(timed(lambda: tc355.tc_mlp_fcrelu(Im, Wm, bm, Om, None)), 2 * 128 * 1024 * width,
                            4 * (128 * 1024 + width * 1024 + width + 128 * width))
    for (C_, F_, HW) in [(16, 16, 14), (32, 32, 7), (4, 4, 56), (8, 8, 28)]:
        It = torch.randn((32, 32, C_, HW, HW), device="cuda")
        Wt = torch.randn((32, F_, C_, 3, 3), device="cuda") * 0.05
        bt = torch.randn((32 * F_,), device="cuda") * 0.05
        Ot = torch.empty((32, 32, F_, HW - 2, HW - 2), device="cuda")
        extra["gconv_32x32x%dx%dx%dx%d" % (F_, C_, HW, HW)] = (entry_i8 if C_ >= 16 else entry)(
            timed(lambda: tc355.tc_group_conv(It, Wt, bt, Ot)), inputs.flops_gconv(32, 32, C_, F_, HW, HW, 3, 3),
            4 * (It.numel() + Wt.numel() + bt.numel() + Ot.numel()))
    # strided convolution (Section 3, listing sconv2d; the paper states no size: a ResNeXt-like down-sampling layer)
    Is_ = torch.randn((32, 64, 56, 56), device="cuda")
    Ws_ = torch.randn((128, 64, 3, 3), device="cuda") * 0.05
    bs_ = torch.randn((128,), device="cuda") * 0.05
    Os_ = torch.empty((32, 128, 27, 27), device="cuda")
    sc_flops, sc_bytes = inputs.flops_sconv2d(32, 64, 128, 56, 56, 3, 3, 2, 2), inputs.bytes_sconv2d(32, 64, 128, 56, 56, 3, 3, 2, 2)
    # (128 filters of 576 taps: the int8 kernel with 13 digit products; then the fp64 kernel)
    extra["sconv2d_32x64x128x56x56_3x3_s2"] = entry_i8(timed(lambda: tc355.tc_sconv2d(Is_, Ws_, bs_, Os_, 2, 2)), sc_flops, sc_bytes)
    extra["sconv2d_32x64x128x56x56_3x3_s2"]["path"] = tc355.last_path()
    with tc355.option(tc355.TC_OPT_INT8, tc355.TC_INT8_OFF):
        extra["sconv2d_32x64x128x56x56_3x3_s2_fp64_path"] = entry(timed(lambda: tc355.tc_sconv2d(Is_, Ws_, bs_, Os_, 2, 2)), sc_flops, sc_bytes)
    # lookup-table sums at the paper's size (Section 7, production models: (E,D,L) = (10^7,64,50), batch 128);
    # fresh random indices every call, so that no gathered row is still in a cache from the call before
    E_, D_, B_, L_ = 10**7, 64, 128, 50
    T1 = torch.randn((E_, D_), device="cuda")
    T2 = torch.randn((E_, D_), device="cuda")
    idx = [torch.randint(0, E_, (B_, L_), device="cuda", dtype=torch.int32) for _ in range(46)]
    O1, O2 = torch.empty((B_, D_), device="cuda"), torch.empty((B_, D_), device="cuda")
    turn = [0]

    def lut_call(n_tables):
        turn[0] = (turn[0] + 1) % 23
        a, b = idx[turn[0]], idx[23 + turn[0]]
        if n_tables == 1:
            tc355.tc_lut([T1], [a], [O1])
        else:
            tc355.tc_lut([T1, T2], [a, b], [O1, O2])

    for n_tables in (1, 2):
        us = timed(lambda: lut_call(n_tables))
        nbytes = n_tables * inputs.bytes_lut(E_, D_, B_, L_)
        extra["%dlut_1e7x64_l50_b128" % n_tables] = {
            "us": round(us, 2), "gbs": round(nbytes / us * 1e-3, 1), "bound": "hbm",
            "frac": round(nbytes / (PEAK_HBM_GBS * 1e9) * 1e6 / us, 4)}
    del Xt, Yt, Zt, Im, Wm, bm, Om, It, Wt, bt, Ot, Is_, Ws_, bs_, Os_, T1, T2, idx, O1, O2

    # the grouped convolution on the fp64 matrix path (what every other shape of the operator takes), for comparison
    with tc355.option(tc355.TC_OPT_INT8, tc355.TC_INT8_OFF):
        g64_us = timed(ops["gconv"][0])
    extra["gconv_cfg4_fp64_path"] = {"us": round(g64_us, 1), "gflops": round(ops["gconv"][1] / g64_us * 1e-3, 1), "bound": "mfma",
                                     "frac": round(ops["gconv"][1] / (PEAK_F64_MFMA_TFLOPS * 1e12) * 1e6 / g64_us, 4)}

    # what the chip delivers for a plain read + write stream of the convolution's size (the runtime's copy of the
    # input buffer onto a buffer as large): the achievable counterpart of the published HBM peak
    cp_dst = torch.empty_like(Ig)
    copy_us = timed(lambda: cp_dst.copy_(Ig))
    copy_gbs = 2 * Ig.numel() * 4 / copy_us * 1e-3
    del cp_dst

    g_flops, g_bytes = ops["gconv"][1], ops["gconv"][2]
    achieved = g_bytes / (gconv_ms * 1e-3) / 1e9
    i8_tops = GCONV_I8_PRODUCTS * g_flops / (gconv_ms * 1e-3) / 1e12
    roofline = {
        "kernel": "grouped convolution (configuration 4), int8 matrix pipe on 4 x 4 operand slices",
        "bound": "hbm",
        "achieved": round(achieved, 1),
        "peak": PEAK_HBM_GBS,
        "unit": "GB/s",
        "frac": round(achieved / PEAK_HBM_GBS, 4),
        "achievable_peak": round(copy_gbs, 1),
        "frac_of_achievable": round(achieved / copy_gbs, 4),
        "traffic": read_traffic("gconv_cfg4_hbm_traffic.txt"),
        "avg_launch_us": round(gconv_ms * 1e3, 2),
        "bytes_per_launch": g_bytes,
        "flops_per_launch": g_flops,
        "mfma_int8_tops": round(i8_tops, 1),
        "mfma_int8_frac": round(i8_tops / PEAK_I8_MFMA_TOPS, 4),
        "note": "at the published peaks the algorithmic bytes take 53.3 us and the 10 int8 slice products 29.6 us: "
                "HBM is the binding roofline; mfma_int8_* give the other one; achievable_peak is a plain device-to-device "
                "copy of the same size measured in this run (read + write GB/s)",
    }

    out = {
        "metric": "GFLOP/s and % of fp32-MFMA/HBM roofline per op (TBMM, MLP, group conv)",
        "value": round(step_flops / (ms_per_step * 1e-3) / 1e9, 1),
        "unit": "GFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "prewarm_ms": round(prewarm_ms, 1),
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f64 (tbmm, mlp, kron) + i8x4 (gconv: int8 slices, exact int32 sums)",
        "data": "synthetic",
        "config": {"workload": "configs 2-5 per step: tbmm B=500 N=26 M=72 K=26; MLP 128x1024->1024->512->256; "
                               "gconv N=32 G=32 C=F=16 58x58 3x3; kron B=256 64^4",
                   "flops_per_step": step_flops},
        "ops": per_op,
        "ops_protocol": "HIP-graph replays; warm = %d launches on one buffer set per sample (gconv: %d), cold = %d launches on "
                        "each of %d rotating buffer sets per sample (gconv: one 426 MB set); us = mean, p0/p50/p90 over the "
                        "samples; frac = roofline_us / cold us" % (WARM_LAUNCHES, WARM_LAUNCHES_GCONV, COLD_ROUNDS, COLD_SETS),
        "launch_floor_us": launch_floor,
        "ops_beyond_step": extra,
        "roofline": roofline,
    }

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(inputs, Ih, Wsh, bsh)
    print(json.dumps(out), flush=True)


def board_sensors():
    """Power (W), power limit (W) and shader clock (MHz) of the first amdgpu card, from sysfs; missing ones are None.
    The driver's figures are moving averages: they settle about half a second after the load changes."""
    import glob
    out = {"power_w": None, "power_cap_w": None, "sclk_mhz": None}
    for hw in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*")):
        for key, name in (("power_w", "power1_input"), ("power_w", "power1_average"), ("power_cap_w", "power1_cap")):
            try:
                if out[key] is None:
                    out[key] = int(open(os.path.join(hw, name)).read()) / 1e6
            except (OSError, ValueError):
                pass
        break
    for dev in sorted(glob.glob("/sys/class/drm/card*/device/pp_dpm_sclk")):
        try:
            cur = [ln for ln in open(dev).read().splitlines() if ln.rstrip().endswith("*")]
            m = re.search(r"(\d+)\s*Mhz", cur[0]) if cur else None
            out["sclk_mhz"] = int(m.group(1)) if m else None
        except OSError:
            pass
        break
    return out


def sustained_study(torch, tc355, ops, Ig, gconv_tensors, seconds):
    """Launch time under sustained load next to the board's power and clock sensors."""
    Icopy = torch.empty_like(Ig)

    def gconv_fp64():
        with tc355.option(tc355.TC_OPT_INT8, tc355.TC_INT8_OFF):
            ops["gconv"][0]()

    def whole_step():
        for name in ("tbmm", "mlp", "gconv", "kron"):
            ops[name][0]()

    # the same launch with all-zero weights: same instructions, same memory traffic, but the multipliers see zeros
    # on one side, the board stays under its power limit and the clock at its nominal value
    W1g, bg, Og = gconv_tensors
    Wzero = torch.zeros_like(W1g)
    legs = [("gconv_int8_path", ops["gconv"][0]),
            ("gconv_int8_path_zero_weights", lambda: tc355.tc_group_conv(Ig, Wzero, bg, Og)),
            ("gconv_fp64_path", gconv_fp64),
            ("copy_of_gconv_input", lambda: Icopy.copy_(Ig)), ("whole_step", whole_step)]
    idle = board_sensors()
    for name, fn in legs:
        fn()
        torch.cuda.synchronize()
        t_end = time.time() + seconds
        windows = []
        while time.time() < t_end:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(200):
                fn()
            e1.record()
            torch.cuda.synchronize()
            windows.append(e0.elapsed_time(e1) * 1e3 / 200)
        sens = board_sensors()  # read while the last window's heat is still in the averages
        tail = windows[-max(1, len(windows) // 4):]
        print(json.dumps({"sustained": name, "seconds": seconds, "us_per_launch_first_window": round(windows[0], 1),
                          "us_per_launch_last_quarter": round(sum(tail) / len(tail), 1), "launches": 200 * len(windows),
                          **{k: (round(v, 0) if v is not None else None) for k, v in sens.items()},
                          "idle_power_w": idle["power_w"]}), flush=True)
        time.sleep(1.0)  # let the averages fall back before the next leg


def scaling_study(torch, tc355, inputs):
    """Batch-scaled versions of the three latency-bound operators (supplementary, not the headline metric)."""
    def timed(fn, reps):
        launches = reps if reps >= 100 else 4  # (a replay costs ~10 us of its own: many launches per graph where they are short)
        return float(replay_samples(capture([fn] * launches), launches, 30).mean())

    def copy_us(nbytes):
        """A plain device-to-device copy that moves nbytes in all (half read, half written), timed the same way."""
        src = torch.ones(max(1, nbytes // 8), dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        return timed(lambda: dst.copy_(src), 100 if nbytes < (1 << 28) else 30)

    def report(op, scale, us, flops, nbytes):
        t_mfma, t_hbm = flops / (PEAK_F64_MFMA_TFLOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
        line = {"op": op, "batch_scale": scale, "us": round(us, 2), "gflops": round(flops / us * 1e-3, 1),
                "gbs": round(nbytes / us * 1e-3, 1), "bound": "mfma" if t_mfma >= t_hbm else "hbm",
                "frac": round(max(t_mfma, t_hbm) * 1e6 / us, 4)}
        if t_hbm > t_mfma:  # what the runtime's copy kernel needs for the same number of bytes
            line["copy_same_bytes_us"] = round(copy_us(nbytes), 2)
        print(json.dumps(line), flush=True)

    for scale in (1, 8, 64):
        B = 500 * scale
        X = torch.rand((B, 26, 26), device="cuda") * 2 - 1
        Y = torch.rand((B, 72, 26), device="cuda") * 2 - 1
        Z = torch.empty((B, 26, 72), device="cuda")
        us = timed(lambda: tc355.tc_tbmm(X, Y, Z), 100 if scale < 64 else 30)
        report("tbmm", scale, us, inputs.flops_tbmm(B, 26, 72, 26), inputs.bytes_tbmm(B, 26, 72, 26))
        del X, Y, Z
    dims = inputs.CONFIGS[3]["dims"]
    Ws = [torch.randn((dims[l + 1], dims[l]), device="cuda") * 0.02 for l in range(3)]
    bs = [torch.randn((dims[l + 1],), device="cuda") * 0.01 for l in range(3)]
    for scale in (1, 8, 64):
        batch = 128 * scale
        I = torch.randn((batch, dims[0]), device="cuda")
        O = [torch.empty((batch, d), device="cuda") for d in dims[1:]]
        ws = torch.empty(tc355.tc_mlp_fcrelu_workspace_bytes(batch, dims), dtype=torch.uint8, device="cuda")
        us = timed(lambda: tc355.tc_mlp_fcrelu(I, Ws, bs, O, ws), 100 if scale < 64 else 20)
        report("mlp", scale, us, inputs.flops_mlp(batch, dims), inputs.bytes_mlp(batch, dims))
        del I, O, ws
    W1 = torch.randn((64, 64), device="cuda") / 8
    W2 = torch.randn((64, 64), device="cuda") / 8
    for scale in (1, 8, 64):
        B = 256 * scale
        X = torch.randn((B, 64, 64), device="cuda") / 8
        Y = torch.empty((B, 64, 64), device="cuda")
        us = timed(lambda: tc355.tc_kron(W1, W2, X, Y), 100 if scale < 64 else 30)
        report("kron", scale, us, inputs.flops_kron(B, 64, 64, 64, 64), inputs.bytes_kron(B, 64, 64, 64, 64))
        del X, Y


def cpu_baseline(inputs, Ih, Wsh, bsh):
    """The float64 oracle, as it stands, on the host cores, over three full steps of the workload (configurations 2-5)."""
    import oracle

    threads = oracle.max_threads()
    oracle.set_threads(threads)
    Xh, Yh = inputs.make_config(2)[1]
    Igh, W1h, bh = inputs.make_config(4)[1]
    K1h, K2h, Xkh = inputs.make_config(5)[1]
    cfg = {c: {k: v for k, v in inputs.CONFIGS[c].items() if k != "op"} for c in (2, 3, 4, 5)}
    flops = (inputs.flops_tbmm(**cfg[2]) + inputs.flops_mlp(**cfg[3]) + inputs.flops_gconv(**cfg[4])
             + inputs.flops_kron(**cfg[5]))
    reps = 3  # about 25 core-seconds on 16 cores
    t0 = time.perf_counter()
    for _ in range(reps):
        oracle.tbmm(Xh, Yh)
        oracle.mlp_fcrelu(Ih, Wsh, bsh)
        oracle.group_conv(Igh, W1h, bh)
        oracle.kron(K1h, K2h, Xkh)
    dt = time.perf_counter() - t0
    return {
        "value": round(reps * flops / dt / 1e9, 3),
        "unit": "GFLOP/s",
        "cores": threads,
        "kind": "oracle",
        "seconds": round(dt, 2),
        "sample": "three full steps (configurations 2-5, each once per step; the Kronecker layer as the single 5-index comprehension, "
                  "counted at the flops of the two-stage evaluation); algorithmic flops of the step / wall time",
    }


if __name__ == "__main__":
    main()
