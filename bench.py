#!/usr/bin/env python3
"""Benchmark of the quantized conv / GEMM hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

Primary workload (the one the headline metric is quoted on): the quantized GEMM sweep of
configuration 2 -- uint8 A with zero-point 128 times per-column int8 B, int32 accumulation,
zero-point correction, per-column fixed-point rescale to uint8 -- over all 64 triples of
{256,1024,4096,8192}^3 plus the skinny shapes M in {1..64}, N = K = 4096.  One step is one
pass over all 71 products; `value` is effective int8 TOPS = 2*sum(MNK) / time with all
operands resident in HBM.  The same run then times the conv stacks of configurations 3-5
(images/s, per-layer roofline fractions) and the streaming kernels, and the CPU oracle on a
bounded sample, and prints ONE JSON line.
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

PEAK_INT8_TOPS = 5033.0  # dense int8 MFMA, 256 CU x 2.4 GHz x 8192 ops/clk/CU
PEAK_HBM_GBS = 8000.0
# vector ALU: 256 CU x 4 SIMD x 16 lanes x 2.4 GHz full-rate 32-bit integer operations per second
PEAK_VALU_LANE_OPS = 256 * 64 * 2.4e9
# the exact fixed-point rescale + clamp + uint8 packing costs about 8 full-rate operations per output byte
EPILOGUE_OPS_PER_OUTPUT = 8.0
ADD_OPS_PER_OUTPUT = 10.0  # fused residual add: two table addresses, add, 7-operation rescale into a byte
# HBM bytes per launch of the dominant kernel, averaged over its launches in one pass of the sweep:
# rocprofv3 FETCH_SIZE / WRITE_SIZE counters scaled by what the same counters read for a plain 1 GiB
# copy (figures and commands: profiles/bench_gemm_sweep_and_stacks.md).  Not measured by this script.
MEASURED_TRAFFIC_BYTES = {"dma256x256": 283.8e6}


def _device_uint8(torch, shape, seed):
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    return torch.randint(0, 256, shape, dtype=torch.uint8, device="cuda:0", generator=g)


def _dev(torch, a):
    import numpy as np

    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


# ----------------------------------------------------------------------------- GEMM sweep

def build_gemm_sweep(torch, qnn, workloads, synth):
    full, skinny = workloads.gemm_sweep()
    shapes = full + skinny
    weights, acts, cases = {}, {}, []
    for i, (M, N, K) in enumerate(shapes):
        if (N, K) not in weights:
            c = synth.gemm_case(1, N, K, workloads.seed_for(2, len(weights)), qnn, with_a=False)
            weights[(N, K)] = dict(Bt=_dev(torch, c["Bt"]), mult=_dev(torch, c["mult"]), shift=_dev(torch, c["shift"]),
                                   z_a=c["z_a"], z_out=c["z_out"])
        if (M, K) not in acts:
            acts[(M, K)] = _device_uint8(torch, (M, K), workloads.seed_for(2, 500 + len(acts)))
        w = weights[(N, K)]
        C = torch.empty((M, N), dtype=torch.uint8, device="cuda:0")
        cases.append(dict(M=M, N=N, K=K, A=acts[(M, K)], w=w, C=C, plan=qnn.qgemm_plan(M, N, K), ops=2.0 * M * N * K,
                          launch=qnn.prepare_qgemm(acts[(M, K)], w["z_a"], w["Bt"], w["mult"], w["shift"], w["z_out"],
                                                   0, 255, C)))
    return cases


def run_gemm(qnn, c):
    c["launch"]()  # arguments marshalled once (binding.prepare_qgemm); same C-ABI call as qnn.qgemm


def time_gemm_sweep(torch, qnn, cases, steps, warmup, eager=False, streams=4):
    """Returns (seconds for `steps` passes, per-case milliseconds).

    Timed region: `steps` replays of one HIP graph that holds the 71 launches of a pass (the
    library calls are captured from the stream they run on), so that the short products are
    timed at GPU speed and not at the speed of the Python launch loop; with eager=True the
    launches are issued one by one instead.  The products of a pass are independent problems, so
    the graph spreads them round-robin over `streams` streams of equal (default) priority that fork
    from and join the capturing stream: short products then overlap with long ones instead of each
    paying a full launch-to-launch latency.  Products that use the library's scratch block (split-K)
    all stay on the capturing stream, in order, because captured launches are not ordered by the
    library itself.  The per-case durations come from a second, instrumented pass of the same
    launches, one by one on one stream, with one HIP event between consecutive launches.
    """
    for _ in range(warmup):
        for c in cases:
            run_gemm(qnn, c)
    torch.cuda.synchronize()
    if eager:
        t0 = time.perf_counter()
        for _ in range(steps):
            for c in cases:
                run_gemm(qnn, c)
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    else:
        side = [torch.cuda.Stream() for _ in range(max(streams, 1) - 1)]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            main = torch.cuda.current_stream()
            for st in side:
                st.wait_stream(main)
            lanes, k = [main] + side, 0
            for c in cases:
                if "/k" in c["plan"] or not side:
                    run_gemm(qnn, c)
                else:
                    with torch.cuda.stream(lanes[k % len(lanes)]):
                        run_gemm(qnn, c)
                    k += 1
            for st in side:
                main.wait_stream(st)
        graph.replay()  # untimed: first replay uploads the graph
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
    # instrumented pass: the time from event i to event i+1 is launch i's duration (events on the
    # stream the kernels run on)
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(cases) + 1)] for _ in range(steps)]
    torch.cuda.synchronize()
    for s in range(steps):
        for i, c in enumerate(cases):
            ev[s][i].record()
            run_gemm(qnn, c)
        ev[s][len(cases)].record()
    torch.cuda.synchronize()
    per_case_ms = [sum(ev[s][i].elapsed_time(ev[s][i + 1]) for s in range(steps)) / steps for i in range(len(cases))]
    return elapsed, per_case_ms


# ----------------------------------------------------------------------------- conv stacks

def time_kernel(torch, fn, reps=5, warm=2):
    """Seconds per launch.  The launches are captured into one HIP graph and the graph is replayed,
    so that short kernels are timed at GPU speed and not at the speed of the Python launch loop."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    n = max(reps, 10)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(n):
            fn()
    graph.replay()
    torch.cuda.synchronize()
    a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    a.record()
    graph.replay()
    b.record()
    torch.cuda.synchronize()
    return a.elapsed_time(b) / n * 1e-3


def time_stack(torch, qnn, workloads, synth, layers, batch, config_id, reps):
    from workloads import shapes as shp

    total_t = total_bound = 0.0
    total_macs = 0
    rows = []
    for idx, l in enumerate(shp.unique_shapes(layers)):
        seed = workloads.seed_for(config_id, idx)
        if l.kind == "qadd":
            n = batch * l.H * l.W * l.Cout
            c = synth.qadd_case((1,), seed, qnn, act=l.act)
            a = _device_uint8(torch, (n,), seed)
            b = _device_uint8(torch, (n,), seed + 1)
            y = torch.empty_like(a)
            fn = lambda: qnn.qadd(a, c["z_a"], b, c["z_b"], c["params"], c["z_out"], c["act_min"], c["act_max"], out=y)
        else:
            in_range = (-2.0, 2.2) if l.Cin == 3 and l.kind == "conv" else (0.0, 6.0)
            c = synth.conv_case(l, batch, seed, qnn, in_range=in_range, with_x=False)
            x = _device_uint8(torch, (batch, l.H, l.W, l.Cin), seed)
            w = _dev(torch, c.get("w_packed", c["w"]))
            mult, shift, bias = _dev(torch, c["mult"]), _dev(torch, c["shift"]), _dev(torch, c["bias"])
            y = torch.empty((batch, l.Ho, l.Wo, l.Cout), dtype=torch.uint8, device="cuda:0")
            if l.kind == "conv_add":  # the residual add of the block, fused behind its last 1x1
                ad = synth.qadd_case((1,), seed + 7, qnn, act=l.act)
                res = _device_uint8(torch, (batch, l.Ho, l.Wo, l.Cout), seed + 1)
                fn = lambda: qnn.qconv2d_add(x, c["z_x"], w, c["stride"], c["pad"], mult, shift, c["z_out"], 0, 255, res,
                                             ad["z_b"], ad["params"], ad["z_out"], ad["act_min"], ad["act_max"], bias=bias,
                                             weight_bits=l.weight_bits, out=y)
            elif l.kind == "dw":
                fn = lambda: qnn.qdwconv2d(x, c["z_x"], w, c["stride"], c["pad"], mult, shift, c["z_out"],
                                           c["act_min"], c["act_max"], bias=bias, out=y)
            else:
                fn = lambda: qnn.qconv2d(x, c["z_x"], w, c["stride"], c["pad"], mult, shift, c["z_out"],
                                         c["act_min"], c["act_max"], bias=bias, weight_bits=l.weight_bits, out=y)
        t = time_kernel(torch, fn, reps=reps)
        macs, nbytes = l.macs(batch), l.bytes(batch)
        t_mfma, t_hbm = 2.0 * macs / (PEAK_INT8_TOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
        outputs = batch * l.Ho * l.Wo * l.Cout if l.kind != "qadd" else batch * l.H * l.W * l.Cout
        alu_ops = EPILOGUE_OPS_PER_OUTPUT + (18.0 if l.kind == "dw" else 0.0)  # depthwise: + 9 MACs as unpack + mad
        if l.kind == "conv_add":
            alu_ops += ADD_OPS_PER_OUTPUT
        t_alu = outputs * alu_ops / PEAK_VALU_LANE_OPS
        bound = max(t_mfma, t_hbm)
        rows.append(dict(layer=l.name, kind=l.kind, count=l.count, us=round(t * 1e6, 2), tops=round(2e-12 * macs / t, 2),
                         gbs=round(nbytes / t * 1e-9, 1), bound="mfma" if t_mfma > t_hbm else "hbm",
                         frac=round(bound / t, 3), frac_alu=round(t_alu / t, 3)))
        total_t += t * l.count
        total_bound += bound * l.count
        total_macs += macs * l.count
        del fn
    return dict(batch=batch, images_per_s=round(batch / total_t, 1), ms=round(total_t * 1e3, 4),
                tops=round(2e-12 * total_macs / total_t, 2), frac_of_sum_of_bounds=round(total_bound / total_t, 3),
                layers=rows)


def time_asym(torch, qnn):
    """asymmetric per-channel weights (a zero-point per column) against the symmetric product, two shapes"""
    out = {}
    for (M, N, K) in [(4096, 4096, 4096), (50176, 256, 1024)]:
        A = _device_uint8(torch, (M, K), 11)
        Bt = _device_uint8(torch, (N, K), 12).view(torch.int8)
        z_w = (torch.arange(N, dtype=torch.int32, device="cuda:0") % 41) - 20
        mult = torch.full((N,), 1 << 30, dtype=torch.int32, device="cuda:0")
        shift = torch.full((N,), 16, dtype=torch.int32, device="cuda:0")
        Cm = torch.empty((M, N), dtype=torch.uint8, device="cuda:0")
        t_sym = time_kernel(torch, lambda: qnn.qgemm(A, 128, Bt, mult, shift, 128, 0, 255, out=Cm), reps=5)
        t_asym = time_kernel(torch, lambda: qnn.qgemm_asym(A, 128, Bt, z_w, mult, shift, 128, 0, 255, out=Cm), reps=5)
        out[f"{M}x{N}x{K}"] = dict(us=round(t_asym * 1e6, 1), tops=round(2e-12 * M * N * K / t_asym, 1),
                                  symmetric_us=round(t_sym * 1e6, 1))
    return out


def time_streaming(torch, qnn):
    """quantize / dequantize / requantize / qadd on configuration 5's 256x224x224x3 tensor size"""
    n = 256 * 224 * 224 * 3
    g = torch.Generator(device="cuda:0")
    g.manual_seed(5)
    x = torch.randn(n, dtype=torch.float32, device="cuda:0", generator=g)
    s, z = qnn.choose_qparams(float(x.min()), float(x.max()))
    q = torch.empty(n, dtype=torch.uint8, device="cuda:0")
    back = torch.empty_like(x)
    out = {}
    t = time_kernel(torch, lambda: qnn.quantize(x, s, z, out=q), reps=10)
    out["quantize"] = dict(us=round(t * 1e6, 1), gbs=round(5.0 * n / t * 1e-9, 1), frac=round(5.0 * n / t / 8e12, 3))
    t = time_kernel(torch, lambda: qnn.dequantize(q, s, z, out=back), reps=10)
    out["dequantize"] = dict(us=round(t * 1e6, 1), gbs=round(5.0 * n / t * 1e-9, 1), frac=round(5.0 * n / t / 8e12, 3))
    rows, ch = n // 256, 256
    acc = torch.randint(-200000, 200000, (rows, ch), dtype=torch.int32, device="cuda:0", generator=g)
    mult, shift = qnn.quantize_multipliers([0.0007 * (1 + 0.01 * i) for i in range(ch)])
    mult, shift = _dev(torch, mult), _dev(torch, shift)
    y = torch.empty((rows, ch), dtype=torch.uint8, device="cuda:0")
    t = time_kernel(torch, lambda: qnn.requantize(acc, mult, shift, True, 128, 0, 255, out=y), reps=10)
    out["requantize"] = dict(us=round(t * 1e6, 1), gbs=round(5.0 * n / t * 1e-9, 1), frac=round(5.0 * n / t / 8e12, 3))
    b = torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda:0", generator=g)
    p = qnn.qadd_params(0.02, 0.031, 0.04)
    t = time_kernel(torch, lambda: qnn.qadd(q, 120, b, 131, p, 0, 0, 255, out=y.view(-1)), reps=10)
    out["qadd"] = dict(us=round(t * 1e6, 1), gbs=round(3.0 * n / t * 1e-9, 1), frac=round(3.0 * n / t / 8e12, 3))
    st = qnn.new_range_state()
    t = time_kernel(torch, lambda: qnn.quantize_dynamic(x, st, out=q), reps=10)  # range pass (4 B) + quantize pass (5 B)
    out["quantize_dynamic"] = dict(us=round(t * 1e6, 1), gbs=round(9.0 * n / t * 1e-9, 1), frac=round(9.0 * n / t / 8e12, 3))
    return out


# ----------------------------------------------------------------------------- CPU baseline

def cpu_baseline():
    """The oracle as it stands, on the host cores, on a bounded sample of the sweep: the
    N = K = 4096 weight matrix times as many activation rows as take roughly 20 s of CPU work."""
    import numpy as np

    import oracle
    import workloads
    from workloads import synth

    N = K = 4096
    c = synth.gemm_case(256, N, K, workloads.seed_for(2, 999), oracle)
    t0 = time.perf_counter()
    oracle.qgemm(c["A"], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
    dt = time.perf_counter() - t0
    rate = 256.0 * N * K / dt
    rows = int(min(65536, max(256, (20.0 * rate / (N * K)) // 256 * 256)))
    A = np.random.Generator(np.random.PCG64(workloads.seed_for(2, 998))).integers(0, 256, (rows, K), dtype=np.uint8)
    t0 = time.perf_counter()
    oracle.qgemm(A, c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
    dt = time.perf_counter() - t0
    return dict(value=round(2e-12 * rows * N * K / dt, 5), unit="TOPS", cores=oracle.num_threads(), kind="oracle",
                sample=f"{rows} x 4096 x 4096 quantized GEMM, the N = K = 4096 weights of the sweep ({dt:.1f} s)")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-secondary", action="store_true", help="skip the conv stacks and streaming kernels")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="time the sweep as single launches instead of a graph replay")
    ap.add_argument("--streams", type=int, default=4,
                    help="streams the independent products of a sweep pass are spread over inside the graph (1: one after another)")
    ap.add_argument("--layers", action="store_true", help="include per-layer rows of the conv stacks in the JSON")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (reference point for the HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (every box has one; the path needs no exchange between GPUs); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_1806_08342_amd as qnn
    import workloads
    from workloads import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    qnn.load_library()  # fails loudly if the HIP library is not built
    torch.cuda.set_device(0)

    cases = build_gemm_sweep(torch, qnn, workloads, synth)
    elapsed, per_case_ms = time_gemm_sweep(torch, qnn, cases, args.steps, args.warmup, eager=args.eager,
                                           streams=args.streams)
    ops_per_step = sum(c["ops"] for c in cases)
    value = ops_per_step * args.steps / elapsed * 1e-12

    # dominant kernel = the tile configuration with the largest share of the step
    by_plan = {}
    for c, ms in zip(cases, per_case_ms):
        d = by_plan.setdefault(c["plan"], dict(ms=0.0, ops=0.0, launches=0, bytes=0.0))
        d["ms"] += ms
        d["ops"] += c["ops"]
        d["bytes"] += c["M"] * c["K"] + c["K"] * c["N"] + c["M"] * c["N"] + 12 * c["N"]
        d["launches"] += 1
    dom = max(by_plan, key=lambda k: by_plan[k]["ms"])
    d = by_plan[dom]
    achieved = d["ops"] / (d["ms"] * 1e-3) * 1e-12
    roofline = dict(bound="mfma", kernel=f"igemm_kernel<{dom}> (int8 32x32x32 MFMA)", achieved=round(achieved, 1),
                    peak=PEAK_INT8_TOPS, unit="TOP/s", frac=round(achieved / PEAK_INT8_TOPS, 4),
                    launches_per_step=d["launches"], avg_launch_us=round(d["ms"] * 1e3 / d["launches"], 2),
                    ops_per_launch=d["ops"] / d["launches"], traffic=MEASURED_TRAFFIC_BYTES.get(dom),
                    algorithmic_bytes_per_launch=d["bytes"] / d["launches"])
    big = {f"{c['M']}x{c['N']}x{c['K']}": round(c["ops"] / (ms * 1e-3) * 1e-12, 1)
           for c, ms in zip(cases, per_case_ms) if (c["M"], c["N"], c["K"]) in
           [(1024,) * 3, (4096,) * 3, (8192,) * 3, (256, 8192, 8192), (64, 4096, 4096), (1, 4096, 4096)]}

    os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
    with open(os.path.join(ROOT, "gpurun_out", "bench_gemm.json"), "w") as f:
        json.dump([dict(M=c["M"], N=c["N"], K=c["K"], plan=c["plan"], us=round(ms * 1e3, 2),
                        tops=round(c["ops"] / (ms * 1e-3) * 1e-12, 1)) for c, ms in zip(cases, per_case_ms)], f, indent=0)

    result = {
        "metric": "effective int8 TOPS (quantized GEMM sweep, uint8 x int8 -> int32 -> uint8)",
        "value": round(value, 2),
        "unit": "TOPS",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(elapsed / args.steps * 1e3, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "int8 (uint8 activations, int8 weights, int32 accumulate)",
        "data": "synthetic (seeded; shapes and value distributions of BASELINE configuration 2)",
        "config": {"workload": "config2 quantized GEMM sweep: 64 triples of {256,1024,4096,8192}^3 + M in {1..64} x 4096 x 4096",
                   "gemms_per_step": len(cases), "ops_per_step": ops_per_step,
                   "launch": "eager" if args.eager else
                   f"hip graph replay (one graph = one pass; independent products on {max(args.streams, 1)} streams)"},
        "frac_of_int8_peak": round(value / PEAK_INT8_TOPS, 4),
        "roofline": roofline,
        "tops_by_shape": big,
    }
    if not args.no_secondary:
        sec = {}
        sec["streaming"] = time_streaming(torch, qnn)
        sec["asymmetric_weights"] = time_asym(torch, qnn)
        sec["mobilenet_v1_b64"] = time_stack(torch, qnn, workloads, synth, workloads.mobilenet_v1(), 64, 3, 5)
        sec["mobilenet_v1_b1"] = time_stack(torch, qnn, workloads, synth, workloads.mobilenet_v1(), 1, 3, 5)
        # residual adds fused behind the last 1x1 of their block (qnn_qconv2d_add); the figure with
        # separate qnn_qadd launches is kept beside it
        fused = workloads.fuse_adds
        sec["resnet50_b256"] = time_stack(torch, qnn, workloads, synth, fused(workloads.resnet50()), 256, 4, 3)
        sec["mobilenet_v2_int4_b32"] = time_stack(torch, qnn, workloads, synth, fused(workloads.mobilenet_v2(4)), 32, 5, 5)
        for name, layers_, batch_, cfg_ in (("resnet50_b256", workloads.resnet50(), 256, 4),
                                            ("mobilenet_v2_int4_b32", workloads.mobilenet_v2(4), 32, 5)):
            plain = time_stack(torch, qnn, workloads, synth, layers_, batch_, cfg_, 3)
            sec[name]["separate_adds"] = dict(images_per_s=plain["images_per_s"], ms=plain["ms"],
                                              frac_of_sum_of_bounds=plain["frac_of_sum_of_bounds"])
        layer_dump = {}
        for k, v in sec.items():
            if isinstance(v, dict) and "layers" in v:
                layer_dump[k] = v.pop("layers")
        result["secondary"] = sec
        if args.layers:
            result["layers"] = layer_dump
        else:
            os.makedirs(os.path.join(ROOT, "gpurun_out"), exist_ok=True)
            with open(os.path.join(ROOT, "gpurun_out", "bench_layers.json"), "w") as f:
                json.dump(layer_dump, f, indent=1)
    if args.calibrate_copy:
        src = _device_uint8(torch, (1 << 30,), 12345)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        result["calibration_copy_bytes"] = 1 << 30
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
