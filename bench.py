#!/usr/bin/env python3
"""Benchmark of the quantized conv / GEMM hot path on one MI355X.

    python bench.py --gpus 1 --steps K --warmup W

Primary workload (the one the headline metric is quoted on): the quantized GEMM sweep of
configuration 2 -- uint8 A with zero-point 128 times per-column int8 B, int32 accumulation,
zero-point correction, per-column fixed-point rescale to uint8 -- over all 64 triples of
{256,1024,4096,8192}^3 plus the skinny shapes M in {1..64}, N = K = 4096.  One step is one
pass over all 71 products; `value` is effective int8 TOPS = 2*sum(MNK) / time with all
operands resident in HBM.

The same run then times, each from a replayed HIP graph with HIP events around the replay on the
stream the kernels run on:
  * every product of the sweep on its own (per-shape rows; operands rotated over enough copies
    that the working set of a row exceeds 512 MB, or the row is labelled cache-resident), the
    skinny rows with 8-bit and with packed 4-bit weights;
  * the conv stacks of configurations 3-5 layer by layer (rotated buffers again) and as one
    graph of the whole stack;
  * the streaming kernels on configuration 5's tensor;
  * two calibration kernels (register-only MFMA loop, 1 GiB copy) that say what this machine
    sustains;
and the CPU oracle on a bounded sample, and prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import re
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
ROTATE_BYTES = 512e6       # working set a timed row must exceed to count as served from HBM (2 x the 256 MB cache)
MAX_SETS = 48
TRAFFIC_PROFILE = os.path.join("profiles", "gemm_dma256x256_sweep.md")


def _device_uint8(torch, shape, seed):
    g = torch.Generator(device="cuda:0")
    g.manual_seed(seed)
    return torch.randint(0, 256, shape, dtype=torch.uint8, device="cuda:0", generator=g)


def _dev(torch, a):
    import numpy as np

    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def _sets_for(nbytes):
    """(number of buffer sets, label): enough distinct copies that the rotated working set exceeds
    ROTATE_BYTES; rows that would need more than MAX_SETS copies are timed cache-resident and say so."""
    need = int(math.ceil(ROTATE_BYTES / max(nbytes, 1))) + 1
    if need > MAX_SETS:
        return MAX_SETS, "cache-resident"
    return max(need, 2), "hbm"


def graph_time(torch, fns, min_launches=10, target_s=2e-3, est_s=None, repeats=3):
    """Seconds per launch.  `fns`: the launches of one rotation (one per buffer set).  They are captured
    into one HIP graph, repeated until the graph holds at least `min_launches` launches (and about
    target_s of work when an estimate is given); the graph is replayed between two HIP events on the
    current stream -- the stream the captured kernels run on -- and the best of `repeats` replays counts."""
    for f in fns:
        f()
    torch.cuda.synchronize()
    rounds = max(1, int(math.ceil(min_launches / len(fns))))
    if est_s:
        rounds = max(rounds, min(50, int(target_s / (est_s * len(fns))) or 1))
    n = rounds * len(fns)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        for _ in range(rounds):
            for f in fns:
                f()
    graph.replay()  # untimed: first replay uploads the graph
    torch.cuda.synchronize()
    best = float("inf")
    for _ in range(repeats):
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        graph.replay()
        b.record()
        torch.cuda.synchronize()
        best = min(best, a.elapsed_time(b) * 1e-3 / n)
    del graph
    return best


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
        # every product brings its own workspace (split-K partial sums), so all of them may overlap
        cases.append(dict(M=M, N=N, K=K, A=acts[(M, K)], w=w, C=C, plan=qnn.qgemm_plan(M, N, K), ops=2.0 * M * N * K,
                          bytes=M * K + K * N + M * N + 12 * N,
                          launch=qnn.prepare_qgemm(acts[(M, K)], w["z_a"], w["Bt"], w["mult"], w["shift"], w["z_out"],
                                                   0, 255, C)))
    return cases


def time_gemm_sweep(torch, cases, steps, warmup, eager=False, streams=4):
    """Seconds for `steps` passes.  Timed region: `steps` replays of one HIP graph that holds the 71
    launches of a pass (the library calls are captured from the stream they run on), so that the short
    products are timed at GPU speed and not at the speed of the Python launch loop; with eager=True the
    launches are issued one by one instead.  The products of a pass are independent problems, so the
    graph spreads the short ones round-robin over `streams` streams of equal (default) priority that fork from
    and join the capturing stream, so that they overlap instead of each paying a full launch-to-launch
    latency; the products whose kernels occupy the whole chip follow one after another."""
    for _ in range(warmup):
        for c in cases:
            c["launch"]()
    torch.cuda.synchronize()
    if eager:
        t0 = time.perf_counter()
        for _ in range(steps):
            for c in cases:
                c["launch"]()
        torch.cuda.synchronize()
        return time.perf_counter() - t0
    side = [torch.cuda.Stream() for _ in range(max(streams, 1) - 1)]
    # products whose kernel fills every CU with resident workgroups (the large pipelined tiles) gain nothing
    # from company: they run one after another.  The others -- launch-latency-bound or small -- overlap with
    # each other on all streams first.
    big = [c for c in cases if c["plan"] in ("dma256x256", "dma256x128")]
    small = [c for c in cases if c["plan"] not in ("dma256x256", "dma256x128")]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        main = torch.cuda.current_stream()
        for st in side:
            st.wait_stream(main)
        lanes = [main] + side
        for k, c in enumerate(small):
            with torch.cuda.stream(lanes[k % len(lanes)]):
                c["launch"]()
        for st in side:
            main.wait_stream(st)
        for c in big:
            c["launch"]()
    graph.replay()  # untimed: first replay uploads the graph
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        graph.replay()
    torch.cuda.synchronize()
    return time.perf_counter() - t0


def time_each_product(torch, qnn, cases):
    """Per-shape rows: every product alone, from a replayed graph of back-to-back launches over rotated
    copies of its operands and output (weights included: for the skinny shapes they are the traffic)."""
    rows = []
    for c in cases:
        sets, label = _sets_for(c["bytes"])
        w = c["w"]
        fns = [c["launch"]]
        keep = []
        for _ in range(sets - 1):
            A2, B2, C2 = c["A"].clone(), w["Bt"].clone(), torch.empty_like(c["C"])
            keep.append((A2, B2, C2))
            fns.append(qnn.prepare_qgemm(A2, w["z_a"], B2, w["mult"], w["shift"], w["z_out"], 0, 255, C2))
        est = max(c["ops"] / 2.0e15, c["bytes"] / 4e12, 4e-6)
        t = graph_time(torch, fns, est_s=est)
        t_mfma, t_hbm = c["ops"] / (PEAK_INT8_TOPS * 1e12), c["bytes"] / (PEAK_HBM_GBS * 1e9)
        rows.append(dict(M=c["M"], N=c["N"], K=c["K"], plan=c["plan"], us=round(t * 1e6, 2),
                         tops=round(c["ops"] / t * 1e-12, 1), gbs=round(c["bytes"] / t * 1e-9, 1),
                         bound="mfma" if t_mfma > t_hbm else "hbm", frac=round(max(t_mfma, t_hbm) / t, 3),
                         sets=sets, memory=label))
        del fns, keep
    return rows


def time_skinny_int4(torch, qnn, workloads, synth):
    """The M <= 64 rows with packed 4-bit weights (half the weight bytes to stream)."""
    rows = []
    _, skinny = workloads.gemm_sweep()
    c0 = synth.gemm_case(1, 4096, 4096, workloads.seed_for(2, 700), qnn, weight_bits=4, with_a=False)
    mult, shift = _dev(torch, c0["mult"]), _dev(torch, c0["shift"])
    for (M, N, K) in skinny:
        nbytes = M * K + K * N // 2 + M * N + 12 * N
        sets, label = _sets_for(nbytes)
        sets = min(sets, MAX_SETS)
        fns, keep = [], []
        base_b = _dev(torch, c0["Bt_packed"])
        for i in range(sets):
            A = _device_uint8(torch, (M, K), 7000 + i)
            B = base_b if i == 0 else base_b.clone()
            C = torch.empty((M, N), dtype=torch.uint8, device="cuda:0")
            keep.append((A, B, C))
            fns.append(qnn.prepare_qgemm(A, c0["z_a"], B, mult, shift, c0["z_out"], 0, 255, C, weight_bits=4))
        t = graph_time(torch, fns, est_s=4e-6)
        rows.append(dict(M=M, N=N, K=K, weight_bits=4, us=round(t * 1e6, 2), tops=round(2.0 * M * N * K / t * 1e-12, 2),
                         gbs=round(nbytes / t * 1e-9, 1), bound="hbm", frac=round(nbytes / (PEAK_HBM_GBS * 1e9) / t, 3),
                         sets=sets, memory=label))
        del fns, keep
    return rows


def time_skinny_large(torch, qnn):
    """Weight streaming where the bytes, not the launch, set the time: M = 1 and 16 rows against a 16384 x 16384
    weight matrix (268 MB as int8, 134 MB packed to 4 bits), timed like the other rows."""
    rows = []
    N = K = 16384
    mult = torch.full((N,), 1518500250, dtype=torch.int32, device="cuda:0")
    shift = torch.full((N,), 14, dtype=torch.int32, device="cuda:0")
    for bits in (8, 4):
        for M in (1, 16):
            nbytes = M * K + K * N * bits // 8 + M * N + 12 * N
            sets, label = _sets_for(nbytes)
            fns, keep = [], []
            for i in range(sets):
                A = _device_uint8(torch, (M, K), 7100 + i)
                if bits == 8:
                    B = _device_uint8(torch, (N, K), 7200 + i).view(torch.int8)
                else:
                    B = _device_uint8(torch, (N, K // 2), 7300 + i)
                C = torch.empty((M, N), dtype=torch.uint8, device="cuda:0")
                keep.append((A, B, C))
                fns.append(qnn.prepare_qgemm(A, 128, B, mult, shift, 128, 0, 255, C, weight_bits=bits))
            t = graph_time(torch, fns, est_s=5e-5)
            rows.append(dict(M=M, N=N, K=K, weight_bits=bits, us=round(t * 1e6, 2), tops=round(2.0 * M * N * K / t * 1e-12, 2),
                             gbs=round(nbytes / t * 1e-9, 1), bound="hbm", frac=round(nbytes / (PEAK_HBM_GBS * 1e9) / t, 3),
                             sets=sets, memory=label))
            del fns, keep
    return rows


# ----------------------------------------------------------------------------- conv stacks

def _layer_launches(torch, qnn, synth, workloads, l, batch, seed, sets):
    """`sets` launch closures of one layer, each on its own input / output (/ residual) tensors."""
    fns, keep = [], []
    if l.kind == "qadd":
        n = batch * l.H * l.W * l.Cout
        c = synth.qadd_case((1,), seed, qnn, act=l.act)
        for i in range(sets):
            a, b = _device_uint8(torch, (n,), seed + 17 * i), _device_uint8(torch, (n,), seed + 17 * i + 1)
            y = torch.empty_like(a)
            keep.append((a, b, y))
            fns.append(lambda a=a, b=b, y=y: qnn.qadd(a, c["z_a"], b, c["z_b"], c["params"], c["z_out"], c["act_min"],
                                                      c["act_max"], out=y))
        return fns, keep
    in_range = (-2.0, 2.2) if l.Cin == 3 and l.kind == "conv" else (0.0, 6.0)
    c = synth.conv_case(l, batch, seed, qnn, in_range=in_range, with_x=False)
    w = _dev(torch, c.get("w_packed", c["w"]))
    mult, shift, bias = _dev(torch, c["mult"]), _dev(torch, c["shift"]), _dev(torch, c["bias"])
    ad = synth.qadd_case((1,), seed + 7, qnn, act=l.act) if l.kind == "conv_add" else None
    ws_bytes = qnn.qconv2d_workspace_bytes(batch, l.H, l.W, l.Cin, l.Cout, l.k, l.k, c["stride"], c["pad"], l.weight_bits) \
        if l.kind != "dw" else 0
    for i in range(sets):
        x = _device_uint8(torch, (batch, l.H, l.W, l.Cin), seed + 17 * i)
        y = torch.empty((batch, l.Ho, l.Wo, l.Cout), dtype=torch.uint8, device="cuda:0")
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device="cuda:0") if ws_bytes else None
        if l.kind == "conv_add":  # the residual add of the block, fused behind its last 1x1
            res = _device_uint8(torch, (batch, l.Ho, l.Wo, l.Cout), seed + 17 * i + 1)
            keep.append((x, y, res, ws))
            fns.append(lambda x=x, y=y, res=res, ws=ws: qnn.qconv2d_add(
                x, c["z_x"], w, c["stride"], c["pad"], mult, shift, c["z_out"], 0, 255, res, ad["z_b"], ad["params"],
                ad["z_out"], ad["act_min"], ad["act_max"], bias=bias, weight_bits=l.weight_bits, out=y, workspace=ws))
        elif l.kind == "dw":
            keep.append((x, y))
            fns.append(lambda x=x, y=y: qnn.qdwconv2d(x, c["z_x"], w, c["stride"], c["pad"], mult, shift, c["z_out"],
                                                      c["act_min"], c["act_max"], bias=bias, out=y))
        else:
            keep.append((x, y, ws))
            fns.append(lambda x=x, y=y, ws=ws: qnn.qconv2d(x, c["z_x"], w, c["stride"], c["pad"], mult, shift, c["z_out"],
                                                           c["act_min"], c["act_max"], bias=bias,
                                                           weight_bits=l.weight_bits, out=y, workspace=ws))
    keep.append((w, mult, shift, bias))
    return fns, keep


def time_stack(torch, qnn, workloads, synth, layers, batch, config_id, whole_graph=True):
    """Per-layer rows (each layer alone, rotated buffers) and the stack as a whole: the layers of the
    network in order, each on buffers of its own, captured once into one HIP graph (`stack_graph`)."""
    from workloads import shapes as shp

    total_t = total_bound = 0.0
    total_macs = 0
    rows = []
    uniq = shp.unique_shapes(layers)
    for idx, l in enumerate(uniq):
        seed = workloads.seed_for(config_id, idx)
        sets, label = _sets_for(l.bytes(batch))
        fns, keep = _layer_launches(torch, qnn, synth, workloads, l, batch, seed, sets)
        macs, nbytes = l.macs(batch), l.bytes(batch)
        t_mfma, t_hbm = 2.0 * macs / (PEAK_INT8_TOPS * 1e12), nbytes / (PEAK_HBM_GBS * 1e9)
        t = graph_time(torch, fns, est_s=max(t_mfma, t_hbm) * 3)
        outputs = batch * l.Ho * l.Wo * l.Cout if l.kind != "qadd" else batch * l.H * l.W * l.Cout
        alu_ops = EPILOGUE_OPS_PER_OUTPUT + (18.0 if l.kind == "dw" else 0.0)  # depthwise: + 9 MACs as unpack + mad
        if l.kind == "conv_add":
            alu_ops += ADD_OPS_PER_OUTPUT
        t_alu = outputs * alu_ops / PEAK_VALU_LANE_OPS
        bound = max(t_mfma, t_hbm)
        rows.append(dict(layer=l.name, kind=l.kind, count=l.count, us=round(t * 1e6, 2), tops=round(2e-12 * macs / t, 2),
                         gbs=round(nbytes / t * 1e-9, 1), bound="mfma" if t_mfma > t_hbm else "hbm",
                         frac=round(bound / t, 3), frac_alu=round(t_alu / t, 3), sets=sets, memory=label))
        total_t += t * l.count
        total_bound += bound * l.count
        total_macs += macs * l.count
        del fns, keep
    out = dict(batch=batch, images_per_s=round(batch / total_t, 1), ms=round(total_t * 1e3, 4),
               tops=round(2e-12 * total_macs / total_t, 2), frac_of_sum_of_bounds=round(total_bound / total_t, 3),
               layers=rows)
    if whole_graph:
        # every layer of the network, in order, once; unique shapes share one pair of launch closures
        cache, seq, keep_all = {}, [], []
        for l in layers:
            key = shp.replace(l, name="", count=1)
            if key not in cache:
                fns, keep = _layer_launches(torch, qnn, synth, workloads, l, batch, workloads.seed_for(config_id, 800 + len(cache)), 2)
                cache[key] = fns
                keep_all.append(keep)
            fns = cache[key]
            seq.append(fns[len(seq) % 2])
        for f in seq:
            f()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for f in seq:
                f()
        graph.replay()
        torch.cuda.synchronize()
        best = float("inf")
        for _ in range(3):
            a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            a.record()
            for _ in range(5):
                graph.replay()
            b.record()
            torch.cuda.synchronize()
            best = min(best, a.elapsed_time(b) * 1e-3 / 5)
        out["stack_graph"] = dict(ms=round(best * 1e3, 4), images_per_s=round(batch / best, 1), launches=len(seq),
                                  frac_of_sum_of_bounds=round(total_bound / best, 3))
        del graph, cache, keep_all
    return out


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
        ws = torch.empty(qnn.qgemm_workspace_bytes(M, N, K, 8, True), dtype=torch.uint8, device="cuda:0")
        t_sym = graph_time(torch, [lambda: qnn.qgemm(A, 128, Bt, mult, shift, 128, 0, 255, out=Cm)])
        t_asym = graph_time(torch, [lambda: qnn.qgemm_asym(A, 128, Bt, z_w, mult, shift, 128, 0, 255, out=Cm, workspace=ws)])
        out[f"{M}x{N}x{K}"] = dict(us=round(t_asym * 1e6, 1), tops=round(2e-12 * M * N * K / t_asym, 1),
                                  symmetric_us=round(t_sym * 1e6, 1), memory="cache-resident")
    return out


def time_streaming(torch, qnn):
    """quantize / dequantize / requantize / qadd on configuration 5's 256x224x224x3 tensor size, rotated
    over 4 sets of buffers (0.46-0.77 GB of distinct data per rotation)."""
    n = 256 * 224 * 224 * 3
    sets = 4
    g = torch.Generator(device="cuda:0")
    g.manual_seed(5)
    xs = [torch.randn(n, dtype=torch.float32, device="cuda:0", generator=g) for _ in range(sets)]
    s, z = qnn.choose_qparams(float(xs[0].min()), float(xs[0].max()))
    qs = [torch.empty(n, dtype=torch.uint8, device="cuda:0") for _ in range(sets)]
    backs = [torch.empty(n, dtype=torch.float32, device="cuda:0") for _ in range(sets)]
    out = {}

    def row(name, t, bytes_per_elem):
        out[name] = dict(us=round(t * 1e6, 1), gbs=round(bytes_per_elem * n / t * 1e-9, 1),
                         frac=round(bytes_per_elem * n / t / (PEAK_HBM_GBS * 1e9), 3), sets=sets, memory="hbm")

    row("quantize", graph_time(torch, [lambda x=x, q=q: qnn.quantize(x, s, z, out=q) for x, q in zip(xs, qs)], 12), 5.0)
    row("dequantize", graph_time(torch, [lambda q=q, b=b: qnn.dequantize(q, s, z, out=b) for q, b in zip(qs, backs)], 12), 5.0)
    rows, ch = n // 256, 256
    accs = [torch.randint(-200000, 200000, (rows, ch), dtype=torch.int32, device="cuda:0", generator=g) for _ in range(sets)]
    mult, shift = qnn.quantize_multipliers([0.0007 * (1 + 0.01 * i) for i in range(ch)])
    mult, shift = _dev(torch, mult), _dev(torch, shift)
    ys = [torch.empty((rows, ch), dtype=torch.uint8, device="cuda:0") for _ in range(sets)]
    row("requantize", graph_time(torch, [lambda a=a, y=y: qnn.requantize(a, mult, shift, True, 128, 0, 255, out=y)
                                         for a, y in zip(accs, ys)], 12), 5.0)
    del accs
    bs = [torch.randint(0, 256, (n,), dtype=torch.uint8, device="cuda:0", generator=g) for _ in range(sets)]
    p = qnn.qadd_params(0.02, 0.031, 0.04)
    row("qadd", graph_time(torch, [lambda q=q, b=b, y=y: qnn.qadd(q, 120, b, 131, p, 0, 0, 255, out=y.view(-1))
                                   for q, b, y in zip(qs, bs, ys)], 12), 3.0)
    st = qnn.new_range_state()
    # range pass (4 B) + quantize pass (5 B); the second pass is meant to find the tensor in the cache
    row("quantize_dynamic", graph_time(torch, [lambda x=x, q=q: qnn.quantize_dynamic(x, st, out=q) for x, q in zip(xs, qs)], 12), 9.0)
    return out


def calibrate(torch, qnn):
    """What this machine sustains: the MFMA pipe from registers only, and a 1 GiB copy."""
    out = {}
    sink = torch.empty(1024 * 512, dtype=torch.int32, device="cuda:0")
    for name, rnd in (("mfma_loop_random_operands", 1), ("mfma_loop_constant_operands", 0)):
        ops = [0.0]

        def fn():
            ops[0] = qnn.calibrate_mfma(1024, 4096, rnd, sink)  # 4 workgroups of 8 waves per CU, 16384 MFMAs per wave
        t = graph_time(torch, [fn], min_launches=4)
        out[name] = dict(us=round(t * 1e6, 1), tops=round(ops[0] / t * 1e-12, 1), frac_of_peak=round(ops[0] / t / (PEAK_INT8_TOPS * 1e12), 3))
    # the vector ALU on the epilogue's own instruction sequence (registers only): accumulators turned into output
    # bytes per second, for 1, 2 and 4 waves per SIMD
    for w in (1, 2, 4):
        cnt = [0.0]

        def fn(w=w):
            cnt[0] = qnn.calibrate_rescale(256 * w, 2048, sink)
        t = graph_time(torch, [fn], min_launches=4)
        out[f"rescale_loop_{w}_waves_per_simd"] = dict(us=round(t * 1e6, 1), outputs_per_s=round(cnt[0] / t, -9),
                                                        lane_ops_per_output="5 + 1 (feedback)")
    n = 1 << 30
    srcs = [_device_uint8(torch, (n,), 12345 + i) for i in range(2)]
    dsts = [torch.empty_like(srcs[0]) for _ in range(2)]
    t = graph_time(torch, [lambda s=s, d=d: qnn.calibrate_copy(s, d) for s, d in zip(srcs, dsts)], min_launches=6)
    out["copy_1GiB_16B_per_lane"] = dict(us=round(t * 1e6, 1), gbs=round(2.0 * n / t * 1e-9, 1),
                                         frac_of_peak=round(2.0 * n / t / (PEAK_HBM_GBS * 1e9), 3))
    del srcs, dsts
    # The same copy kernel at the byte counts of two depthwise layers of MobileNetV1 at batch 64 (112 x 112 x 32
    # and 14 x 14 x 512, stride 1: as many bytes out as in), timed like the layer rows: what a launch that only
    # moves a layer's bytes costs on this machine, launch floor included.
    for name, nbytes in (("copy_25.7MB_each_way", 64 * 112 * 112 * 32), ("copy_6.4MB_each_way", 64 * 14 * 14 * 512)):
        sets, label = _sets_for(2 * nbytes)
        bufs = [(_device_uint8(torch, (nbytes,), 500 + i), torch.empty(nbytes, dtype=torch.uint8, device="cuda:0")) for i in range(sets)]
        t = graph_time(torch, [lambda s=s, d=d: qnn.calibrate_copy(s, d) for s, d in bufs], min_launches=10, est_s=1e-5)
        out[name] = dict(us=round(t * 1e6, 2), gbs=round(2.0 * nbytes / t * 1e-9, 1), frac_of_peak=round(2.0 * nbytes / t / (PEAK_HBM_GBS * 1e9), 3),
                         sets=sets, memory=label)
        del bufs
    # The dominant GEMM kernel itself on 8192^3 with the sweep's operands (uniform bytes, Gaussian weights) and
    # with operands that toggle no bits (all codes zero).  Same instructions, same memory traffic; what differs
    # is the power the data draws in the multipliers and on the wires, i.e. the clock the chip sustains.
    m = 8192
    mult = torch.full((m,), 1 << 30, dtype=torch.int32, device="cuda:0")
    shift = torch.full((m,), 12, dtype=torch.int32, device="cuda:0")
    for name in ("gemm_8192_sweep_operands", "gemm_8192_zero_operands"):
        if name.endswith("sweep_operands"):
            A = _device_uint8(torch, (m, m), 777)
            B = (torch.randn((m, m), device="cuda:0", generator=torch.Generator(device="cuda:0").manual_seed(778)) * (127 / 4.5))
            B = B.round().clamp(-127, 127).to(torch.int8)
        else:
            A = torch.zeros((m, m), dtype=torch.uint8, device="cuda:0")
            B = torch.zeros((m, m), dtype=torch.int8, device="cuda:0")
        Cm = torch.empty((m, m), dtype=torch.uint8, device="cuda:0")
        fn = qnn.prepare_qgemm(A, 128, B, mult, shift, 3, 0, 255, Cm)
        t = graph_time(torch, [fn], min_launches=10)
        ops = 2.0 * m * m * m
        out[name] = dict(us=round(t * 1e6, 1), tops=round(ops / t * 1e-12, 1), frac_of_peak=round(ops / t / (PEAK_INT8_TOPS * 1e12), 3),
                         plan=qnn.qgemm_plan(m, m, m))
        del A, B, Cm, fn
    return out


def traffic_from_profile(plan):
    """HBM bytes per launch of the dominant kernel as the committed rocprofv3 counter summary states
    them (a line `traffic_bytes_per_launch <plan> <bytes>`); None when the summary has no such line.
    The counters cannot be read from inside this process: the figure is quoted, with its source."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    try:
        text = open(path).read()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch\s+" + re.escape(plan) + r"\s+([0-9.eE+]+)", text)
    return float(m.group(1)) if m else None


# ----------------------------------------------------------------------------- CPU baseline

def cpu_baseline():
    """The oracle as it stands, on the host cores, on a bounded sample of the sweep: the
    N = K = 4096 weight matrix times as many activation rows as take roughly 15 s of CPU work; and
    configuration 1 (one 3x3 convolution) on one thread."""
    import ctypes

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
    rows = int(min(65536, max(256, (15.0 * rate / (N * K)) // 256 * 256)))
    A = np.random.Generator(np.random.PCG64(workloads.seed_for(2, 998))).integers(0, 256, (rows, K), dtype=np.uint8)
    t0 = time.perf_counter()
    oracle.qgemm(A, c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
    dt = time.perf_counter() - t0
    out = dict(value=round(2e-12 * rows * N * K / dt, 5), unit="TOPS", cores=oracle.num_threads(), kind="oracle",
               sample=f"{rows} x 4096 x 4096 quantized GEMM, the N = K = 4096 weights of the sweep ({dt:.1f} s)")
    try:  # configuration 1 on a single thread (the thread count is OpenMP's, set through its runtime)
        gomp = ctypes.CDLL("libgomp.so.1")
        layer = workloads.single_conv()[0]
        c1 = synth.single_conv_case(layer, workloads.seed_for(1, 0), oracle)
        gomp.omp_set_num_threads(1)
        best = float("inf")
        for _ in range(5):
            t0 = time.perf_counter()
            oracle.qconv2d(c1["x"], c1["z_x"], c1["w"], c1["stride"], c1["pad"], c1["mult"], c1["shift"], c1["z_out"],
                           c1["act_min"], c1["act_max"], bias=c1["bias"])
            best = min(best, time.perf_counter() - t0)
        gomp.omp_set_num_threads(oracle.num_threads())
        out["config1_single_thread"] = dict(ms=round(best * 1e3, 3), gops=round(2e-9 * layer.macs(1) / best, 3))
    except OSError:
        pass
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--no-secondary", action="store_true", help="skip the conv stacks, streaming kernels and calibration")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--eager", action="store_true", help="time the sweep as single launches instead of a graph replay")
    ap.add_argument("--streams", type=int, default=4,
                    help="streams the independent products of a sweep pass are spread over inside the graph (1: one after another)")
    ap.add_argument("--sweep-only", action="store_true",
                    help="only the timed sweep passes (the command the rocprofv3 summaries of the sweep are taken from); "
                         "the JSON line then lists the products in launch order")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="with --sweep-only: also one plain 1 GiB copy (reference point for the HBM byte counters)")
    ap.add_argument("--stack-only", default=None,
                    help="only the layer rows of one conv stack: mobilenet_v1_b64, mobilenet_v1_b1, resnet50_b256 or "
                         "mobilenet_v2_int4_b32 (the command the rocprofv3 summaries of the conv kernels are taken from)")
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

    if args.stack_only:
        stacks = {"mobilenet_v1_b64": (workloads.mobilenet_v1(), 64, 3), "mobilenet_v1_b1": (workloads.mobilenet_v1(), 1, 3),
                  "resnet50_b256": (workloads.fuse_adds(workloads.resnet50()), 256, 4),
                  "mobilenet_v2_int4_b32": (workloads.fuse_adds(workloads.mobilenet_v2(4)), 32, 5)}
        layers_, batch_, cfg_ = stacks[args.stack_only]
        print(json.dumps({args.stack_only: time_stack(torch, qnn, workloads, synth, layers_, batch_, cfg_, whole_graph=False)}))
        return

    cases = build_gemm_sweep(torch, qnn, workloads, synth)
    elapsed = time_gemm_sweep(torch, cases, args.steps, args.warmup, eager=args.eager, streams=args.streams)
    ops_per_step = sum(c["ops"] for c in cases)
    value = ops_per_step * args.steps / elapsed * 1e-12
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
    }
    if args.sweep_only:
        big = [c for c in cases if c["plan"] in ("dma256x256", "dma256x128")]
        small = [c for c in cases if c["plan"] not in ("dma256x256", "dma256x128")]
        result["launch_order"] = [[c["M"], c["N"], c["K"], c["plan"]] for c in (cases if args.eager else small + big)]
        if args.calibrate_copy:
            src = _device_uint8(torch, (1 << 30,), 12345)
            dst = torch.empty_like(src)
            qnn.calibrate_copy(src, dst)
            torch.cuda.synchronize()
            result["calibration_copy_bytes"] = 1 << 30
        print(json.dumps(result))
        return

    # per-shape rows; the dominant kernel = the tile configuration with the largest share of the rows' time
    rows = time_each_product(torch, qnn, cases)
    by_plan = {}
    for r in rows:
        d = by_plan.setdefault(r["plan"], dict(s=0.0, ops=0.0, launches=0, bytes=0.0))
        d["s"] += r["us"] * 1e-6
        d["ops"] += 2.0 * r["M"] * r["N"] * r["K"]
        d["bytes"] += r["M"] * r["K"] + r["K"] * r["N"] + r["M"] * r["N"] + 12 * r["N"]
        d["launches"] += 1
    dom = max(by_plan, key=lambda k: by_plan[k]["s"])
    d = by_plan[dom]
    achieved = d["ops"] / d["s"] * 1e-12
    result["roofline"] = dict(bound="mfma", kernel=f"igemm_dma_kernel<{dom}> (int8 32x32x32 MFMA)", achieved=round(achieved, 1),
                              peak=PEAK_INT8_TOPS, unit="TOP/s", frac=round(achieved / PEAK_INT8_TOPS, 4),
                              launches_per_step=d["launches"], avg_launch_us=round(d["s"] * 1e6 / d["launches"], 2),
                              ops_per_launch=d["ops"] / d["launches"], traffic=traffic_from_profile(dom),
                              traffic_source=TRAFFIC_PROFILE,
                              algorithmic_bytes_per_launch=d["bytes"] / d["launches"],
                              timing="HIP events around a replayed graph of back-to-back launches, per shape")
    result["gemm_rows"] = rows
    del cases

    if not args.no_secondary:
        result["gemm_rows_int4_skinny"] = time_skinny_int4(torch, qnn, workloads, synth)
        result["gemm_rows_skinny_16384"] = time_skinny_large(torch, qnn)
        result["calibration"] = calibrate(torch, qnn)
        sec = {}
        sec["streaming"] = time_streaming(torch, qnn)
        sec["asymmetric_weights"] = time_asym(torch, qnn)
        sec["mobilenet_v1_b64"] = time_stack(torch, qnn, workloads, synth, workloads.mobilenet_v1(), 64, 3)
        sec["mobilenet_v1_b1"] = time_stack(torch, qnn, workloads, synth, workloads.mobilenet_v1(), 1, 3)
        # residual adds fused behind the last 1x1 of their block (qnn_qconv2d_add); the figure with
        # separate qnn_qadd launches is kept beside it
        fused = workloads.fuse_adds
        sec["resnet50_b256"] = time_stack(torch, qnn, workloads, synth, fused(workloads.resnet50()), 256, 4)
        sec["mobilenet_v2_int4_b32"] = time_stack(torch, qnn, workloads, synth, fused(workloads.mobilenet_v2(4)), 32, 5)
        for name, layers_, batch_, cfg_ in (("resnet50_b256", workloads.resnet50(), 256, 4),
                                            ("mobilenet_v2_int4_b32", workloads.mobilenet_v2(4), 32, 5)):
            plain = time_stack(torch, qnn, workloads, synth, layers_, batch_, cfg_, whole_graph=False)
            sec[name]["separate_adds"] = dict(images_per_s=plain["images_per_s"], ms=plain["ms"],
                                              frac_of_sum_of_bounds=plain["frac_of_sum_of_bounds"])
        result["secondary"] = sec
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline()
    print(json.dumps(result))


if __name__ == "__main__":
    main()
