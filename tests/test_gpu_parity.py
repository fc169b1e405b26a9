"""GPU parity: every kernel of the library, called through the C ABI, against the CPU oracle
on the same seeded inputs.  Integer outputs must match bit for bit; fp32 quantize / dequantize
must match with 0 LSB difference (both sides perform the same binary32 operations, ties away
from zero)."""
import numpy as np
import pytest
import torch

import oracle
import paper_1806_08342_amd as qnn
import workloads
from workloads import synth

from gpu_util import assert_same, dev, host

pytestmark = pytest.mark.gpu


# ------------------------------------------------------------------ quantize / dequantize

@pytest.mark.parametrize("n", [0, 1, 3, 4, 1023, 4096, 1_000_003])
def test_quantize_matches_oracle(n):
    rng = np.random.default_rng(100 + n)
    x = rng.normal(0, 2, n).astype(np.float32)
    if n >= 1023:
        x[:8] = [np.nan, np.inf, -np.inf, 0.0, -0.0, 1e30, -1e30, 1e-40]
    for s, z in [(0.0213, 131), (2.0 ** -6, 128), (1 / 3, 0), (0.05, 255)]:
        got = host(qnn.quantize(dev(x), s, z)) if n else np.empty(0, np.uint8)
        assert_same(got, oracle.quantize(x, s, z), f"quantize n={n} s={s} z={z}")


def test_quantize_exact_ties_and_misaligned_views():
    k = np.arange(-200, 200)
    x = ((k + 0.5) * 2.0 ** -4).astype(np.float32)  # exact ties
    assert_same(host(qnn.quantize(dev(x), 2.0 ** -4, 100)), oracle.quantize(x, 2.0 ** -4, 100), "ties")
    rng = np.random.default_rng(7)
    big = rng.normal(0, 1, 10_001).astype(np.float32)
    t = dev(big)
    for off in (1, 2, 3):  # pointers that are not 16-byte aligned take the scalar path
        view = t[off:]
        out = torch.empty(view.numel() + 3, dtype=torch.uint8, device="cuda:0")[off % 3:][: view.numel()]
        qnn.quantize(view, 0.01, 128, out=out)
        assert_same(host(out), oracle.quantize(big[off:], 0.01, 128), f"offset {off}")
    assert_same(host(qnn.quantize(dev(big), 0.02, 10, qmin=5, qmax=14)), oracle.quantize(big, 0.02, 10, 5, 14),
                "restricted code range")


@pytest.mark.parametrize("n", [1, 5, 4096, 777_777])
def test_dequantize_matches_oracle(n):
    rng = np.random.default_rng(200 + n)
    q = rng.integers(0, 256, n).astype(np.uint8)
    for s, z in [(0.0213, 131), (2.0 ** -6, 0), (1 / 3, 255)]:
        got = host(qnn.dequantize(dev(q), s, z))
        want = oracle.dequantize(q, s, z)
        assert got.dtype == np.float32 and np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_quantize_large_tensor_config5_sample():
    # one image-batch slice of configuration 5's 256x224x224x3 tensor
    c = synth.quantize_case((8, 224, 224, 3), workloads.seed_for(5, 900), oracle)
    got = host(qnn.quantize(dev(c["x"]), c["scale"], c["zero_point"]))
    assert_same(got, oracle.quantize(c["x"], c["scale"], c["zero_point"]), "quantize cfg5 slice")
    back = host(qnn.dequantize(dev(got), c["scale"], c["zero_point"]))
    assert np.array_equal(back, oracle.dequantize(got, c["scale"], c["zero_point"]))


# ------------------------------------------------------------------------------ requantize

def _edge_acc(rng, rows, ch):
    acc = rng.integers(-2 ** 20, 2 ** 20, (rows, ch)).astype(np.int64)
    flat = acc.reshape(-1)
    edges = [2 ** 31 - 1, -2 ** 31, -2 ** 31 + 1, 0, 1, -1, 2 ** 30, -2 ** 30, 2 ** 30 - 1, 12345678, -12345678]
    n1 = min(len(edges), flat.size)
    flat[:n1] = edges[:n1]
    n2 = max(0, min(len(edges), flat.size - n1))
    flat[n1: n1 + n2] = edges[::-1][:n2]
    return acc.astype(np.int32)


@pytest.mark.parametrize("rows,ch", [(1, 1), (37, 13), (64, 64), (1000, 96), (5, 1024)])
def test_requantize_matches_oracle(rows, ch):
    rng = np.random.default_rng(300 + rows + ch)
    acc = _edge_acc(rng, rows, ch)
    mult = rng.integers(2 ** 30, 2 ** 31, ch).astype(np.int32)
    mult[0] = 2 ** 30
    mult[-1] = 2 ** 31 - 1
    shift = rng.integers(0, 32, ch).astype(np.int32)
    shift[: min(ch, 3)] = [0, 31, -3][: min(ch, 3)]
    mult[-1] = 2 ** 31 - 1
    if ch > 8:
        shift[5:8] = [-31, -1, 1]
        mult[8] = 0
    for z_out, lo, hi in [(0, 0, 255), (128, 0, 255), (3, 3, 120), (255, 7, 255)]:
        want = oracle.requantize(acc, mult, shift, True, z_out, lo, hi)
        got = host(qnn.requantize(dev(acc), dev(mult), dev(shift), True, z_out, lo, hi))
        assert_same(got, want, f"requantize per-channel {rows}x{ch} z={z_out}")
    for m0, s0 in [(int(mult[0]), 9), (2 ** 31 - 1, 0), (1518500250, -2)]:
        want = oracle.requantize(acc, np.array([m0]), np.array([s0]), False, 128, 0, 255)
        got = host(qnn.requantize(dev(acc), dev(np.array([m0], np.int32)), dev(np.array([s0], np.int32)), False, 128,
                                  0, 255))
        assert_same(got, want, f"requantize per-layer {rows}x{ch}")


# ------------------------------------------------------------------------------------ qadd

@pytest.mark.parametrize("n", [1, 17, 4096, 300_001])
def test_qadd_matches_oracle(n):
    for i, act in enumerate(["relu", "none"]):
        c = synth.qadd_case((n,), 400 + n + i, oracle, act=act)
        want = oracle.qadd(c["a"], c["z_a"], c["b"], c["z_b"], c["params"], c["z_out"], c["act_min"], c["act_max"])
        got = host(qnn.qadd(dev(c["a"]), c["z_a"], dev(c["b"]), c["z_b"], c["params"], c["z_out"], c["act_min"],
                            c["act_max"]))
        assert_same(got, want, f"qadd n={n} act={act}")


def test_qadd_all_code_pairs_and_odd_parameters():
    a = np.arange(256, dtype=np.uint8).repeat(256)
    b = np.tile(np.arange(256, dtype=np.uint8), 256)
    for s_a, s_b, s_o, z_a, z_b, z_o in [(0.1, 0.1, 0.1, 0, 0, 0), (0.02, 0.07, 0.05, 255, 0, 128),
                                         (1.0, 1e-3, 0.25, 17, 200, 3), (0.01, 0.01, 1e-4, 128, 128, 128)]:
        p = oracle.qadd_params(s_a, s_b, s_o)
        want = oracle.qadd(a, z_a, b, z_b, p, z_o, 0, 255)
        got = host(qnn.qadd(dev(a), z_a, dev(b), z_b, p, z_o, 0, 255))
        assert_same(got, want, f"qadd all pairs {s_a},{s_b},{s_o}")


# ----------------------------------------------------------------------------------- qgemm

def _gemm_params(rng, N, K, spread=True):
    real = 10 ** rng.uniform(-4.2, -3.2, N) / np.sqrt(K / 64.0)
    mult, shift = oracle.quantize_multipliers(real)
    bias = rng.integers(-20000, 20000, N).astype(np.int32)
    return bias, mult, shift


@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (5, 7, 3), (64, 64, 64), (100, 70, 200), (129, 257, 65), (300, 40, 1000),
                                   (256, 256, 256), (33, 500, 72), (70, 130, 24), (513, 129, 4104)])
@pytest.mark.parametrize("z_a", [0, 128, 255])
def test_qgemm_int8_matches_oracle(M, N, K, z_a):
    rng = np.random.default_rng(500 + M + N + K + z_a)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _gemm_params(rng, N, K)
    want = oracle.qgemm(A, z_a, Bt, mult, shift, 128, 0, 255, bias=bias)
    got = host(qnn.qgemm(dev(A), z_a, dev(Bt), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias)))
    assert_same(got, want, f"qgemm {M}x{N}x{K} z_a={z_a}")
    frac_clamped = np.mean((want == 0) | (want == 255))
    assert frac_clamped < 0.6, "parity would be vacuous"


def test_qgemm_rows_contiguous_b_and_pack_b():
    rng = np.random.default_rng(600)
    M, N, K = 77, 90, 150
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    B = rng.integers(-128, 128, (K, N)).astype(np.int8)  # [K, N], rows contiguous
    bias, mult, shift = _gemm_params(rng, N, K)
    want = oracle.qgemm(A, 99, np.ascontiguousarray(B.T), mult, shift, 100, 10, 240, bias=bias)
    got = host(qnn.qgemm(dev(A), 99, dev(B), dev(mult), dev(shift), 100, 10, 240, bias=dev(bias),
                         b_layout=qnn.binding.B_ROWS_CONTIGUOUS))
    assert_same(got, want, "qgemm rows-contiguous B")
    packed = qnn.pack_b(dev(B))
    assert_same(host(packed), B.T, "pack_b")
    got2 = host(qnn.qgemm(dev(A), 99, packed, dev(mult), dev(shift), 100, 10, 240, bias=dev(bias)))
    assert_same(got2, want, "qgemm after pack_b")


@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (50, 33, 24), (130, 200, 328), (9, 17, 6), (200, 96, 1040)])
def test_qgemm_int4_matches_oracle(M, N, K):
    rng = np.random.default_rng(700 + M + N + K)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-8, 8, (N, K)).astype(np.int8)
    Bt[0, :2] = (-8, 7)
    packed = oracle.pack_int4(Bt)
    bias, mult, shift = _gemm_params(rng, N, K)
    mult, shift = oracle.quantize_multipliers(10 ** rng.uniform(-3.0, -2.2, N) / np.sqrt(K / 64.0))
    want = oracle.qgemm(A, 131, packed, mult, shift, 128, 0, 255, bias=bias, weight_bits=4)
    assert_same(want, oracle.qgemm(A, 131, Bt, mult, shift, 128, 0, 255, bias=bias), "oracle int4 == int8 values")
    got = host(qnn.qgemm(dev(A), 131, dev(packed), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias), weight_bits=4))
    assert_same(got, want, f"qgemm int4 {M}x{N}x{K}")


@pytest.mark.parametrize("M,N,K", [(128, 128, 320), (300, 200, 576), (1000, 96, 960), (65, 33, 1024), (700, 520, 2048)])
def test_qgemm_int4_unpack_pass_then_pipelined_kernel(M, N, K):
    # aligned 4-bit products with M > 64 and K > 256: the nibbles are unpacked to scratch memory first
    rng = np.random.default_rng(720 + M + N + K)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-8, 8, (N, K)).astype(np.int8)
    Bt[0, :4] = (-8, 7, -1, 0)
    Bt[N - 1, K - 2:] = (-8, -8)
    packed = oracle.pack_int4(Bt)
    bias = rng.integers(-20000, 20000, N).astype(np.int32)
    mult, shift = oracle.quantize_multipliers(10 ** rng.uniform(-3.0, -2.2, N) / np.sqrt(K / 64.0))
    for z_a in (0, 131, 255):
        want = oracle.qgemm(A, z_a, packed, mult, shift, 128, 0, 255, bias=bias, weight_bits=4)
        got = host(qnn.qgemm(dev(A), z_a, dev(packed), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias), weight_bits=4))
        assert_same(got, want, f"qgemm int4 (unpack pass) {M}x{N}x{K} z_a={z_a}")


@pytest.mark.parametrize("shape", [(14, 14, 64, 96, 3, 1, 1), (7, 7, 960, 160, 1, 1, 0), (9, 9, 128, 40, 5, 2, 2), (7, 7, 576, 130, 1, 1, 0)],
                         ids=lambda s: "x".join(map(str, s)))
def test_qconv2d_int4_unpack_pass_matches_oracle(shape):
    H, W, Cin, Cout, k, s, p = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act="none", weight_bits=4)
    c = synth.conv_case(layer, 4, 740 + sum(shape), oracle)
    c["w"][0, 0, 0, :2] = (-8, 7)
    c["w_packed"] = oracle.pack_int4(c["w"])
    for z_x in (c["z_x"], 255):
        c["z_x"] = z_x
        _run_conv(c, f"conv int4 (unpack pass) {shape} z_x={z_x}")


def test_qgemm_extreme_accumulators_and_left_shift():
    # all-255 activations times all-(-128)/127 weights with z_a = 0 reach the largest |acc| for this K;
    # multipliers >= 1 (negative shift) and huge biases take the general rescale path
    M, N, K = 40, 48, 2048
    A = np.full((M, K), 255, np.uint8)
    Bt = np.where(np.arange(N)[:, None] % 2 == 0, 127, -128).astype(np.int8) * np.ones((1, K), np.int8)
    mult = np.full(N, 2 ** 30 + 12345, np.int32)
    shift = (np.arange(N) % 31 - 4).astype(np.int32)  # -4 .. 26
    bias = np.where(np.arange(N) % 3 == 0, 2 ** 30, -5).astype(np.int32)
    for z_a in (0, 255):
        want = oracle.qgemm(A, z_a, Bt, mult, shift, 17, 0, 255, bias=bias)
        got = host(qnn.qgemm(dev(A), z_a, dev(Bt), dev(mult), dev(shift), 17, 0, 255, bias=dev(bias)))
        assert_same(got, want, f"qgemm extremes z_a={z_a}")


@pytest.mark.parametrize("M,N", [(8, 48), (40, 33), (130, 70), (300, 256)])
@pytest.mark.parametrize("fill", ["max", "random"])
def test_qgemm_largest_k_every_kernel_family(M, N, fill):
    # K = 65536 is the largest reduction the int32 accumulator admits (255 * 128 * K < 2^31): few-row
    # kernel (M <= 64), split-K tiles (few output tiles) and plain tiles; all-255 x all-(-128) is the
    # accumulator of largest magnitude
    K = 65536
    rng = np.random.default_rng(2300 + M + N)
    if fill == "max":
        A = np.full((M, K), 255, np.uint8)
        Bt = np.where(np.arange(N)[:, None] % 2 == 0, -128, 127).astype(np.int8) * np.ones((1, K), np.int8)
    else:
        A = rng.integers(0, 256, (M, K)).astype(np.uint8)
        Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    mult, shift = oracle.quantize_multipliers(np.full(N, 2.0 ** -23 if fill == "max" else 2.0 ** -15))
    mult = (mult + np.arange(N)).astype(np.int32)
    for z_a in (0, 128, 255):
        want = oracle.qgemm(A, z_a, Bt, mult, shift, 128, 0, 255)
        got = host(qnn.qgemm(dev(A), z_a, dev(Bt), dev(mult), dev(shift), 128, 0, 255))
        assert_same(got, want, f"qgemm K=65536 {M}x{N} {fill} z_a={z_a}")
    if fill == "random":
        assert len(np.unique(want)) > 2


def test_qgemm_config2_small_shapes():
    for i, (M, N, K) in enumerate([(256, 256, 256), (1, 512, 512), (64, 256, 1024), (256, 1024, 256)]):
        c = synth.gemm_case(M, N, K, workloads.seed_for(2, i), oracle)
        want = oracle.qgemm(c["A"], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
        got = host(qnn.qgemm(dev(c["A"]), c["z_a"], dev(c["Bt"]), dev(c["mult"]), dev(c["shift"]), c["z_out"], 0, 255))
        assert_same(got, want, f"config 2 gemm {M}x{N}x{K}")
        assert np.mean((want == 0) | (want == 255)) < 0.05


# --------------------------------------------------------------------------------- qconv2d

def _run_conv(c, what):
    w_o = c.get("w_packed", c["w"])
    want = oracle.qconv2d(c["x"], c["z_x"], w_o, c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"],
                          c["act_min"], c["act_max"], bias=c["bias"], weight_bits=c["weight_bits"])
    got = host(qnn.qconv2d(dev(c["x"]), c["z_x"], dev(w_o), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]),
                           c["z_out"], c["act_min"], c["act_max"], bias=dev(c["bias"]), weight_bits=c["weight_bits"]))
    assert_same(got, want, what)
    return want


def test_config1_single_conv_exact():
    layer = workloads.single_conv()[0]
    c = synth.single_conv_case(layer, workloads.seed_for(1, 0), oracle)
    assert (c["z_x"], c["act_min"], c["act_max"]) == (128, 0, 120)
    want = _run_conv(c, "config 1")
    assert 0.05 < np.mean((want == 0) | (want == 120)) < 0.9


CONV_SHAPES = [
    # H, W, Cin, Cout, k, stride, pad, act, bits
    (9, 7, 16, 8, 3, 1, 1, "relu6", 8),
    (9, 7, 16, 8, 3, 2, 1, "relu", 8),
    (12, 12, 3, 32, 3, 2, 1, "relu6", 8),      # stem-like, Cin = 3 -> byte gather
    (20, 20, 3, 64, 7, 2, 3, "relu", 8),       # 7x7 stem
    (23, 301, 3, 64, 7, 2, 3, "relu", 8),      # stem wider than one 128-pixel strip, odd sizes
    (17, 40, 3, 20, 3, 2, 1, "relu6", 8),      # stem with a ragged channel count
    (9, 140, 3, 32, 3, 1, 1, "none", 8),       # stem-like, stride 1
    (30, 30, 1, 40, 7, 2, 3, "relu", 8),       # single input channel
    (14, 14, 32, 64, 1, 1, 0, "relu6", 8),     # pointwise
    (14, 14, 64, 96, 1, 2, 0, "none", 8),      # projection shortcut: 1x1 stride 2
    (8, 8, 24, 144, 1, 1, 0, "relu6", 8),      # Cin multiple of 8 only
    (8, 8, 20, 30, 3, 1, 1, "none", 8),        # nothing aligned
    (10, 10, 64, 64, 3, 1, 0, "relu", 8),      # no padding
    (11, 13, 48, 72, 5, 2, 2, "relu6", 8),
    (14, 14, 32, 192, 1, 1, 0, "relu6", 4),    # 4-bit expand
    (14, 14, 24, 144, 1, 1, 0, "relu6", 4),
    (9, 9, 16, 24, 3, 2, 1, "none", 4),
    (7, 7, 320, 1280, 1, 1, 0, "relu6", 4),
]


@pytest.mark.parametrize("shape", CONV_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("batch", [1, 3])
def test_qconv2d_matches_oracle(shape, batch):
    H, W, Cin, Cout, k, s, p, act, bits = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act=act, weight_bits=bits)
    rng_range = (0.0, 6.0) if Cin != 3 else (-2.0, 2.2)
    c = synth.conv_case(layer, batch, 800 + 10 * CONV_SHAPES.index(shape) + batch, oracle, in_range=rng_range)
    if bits == 4:
        c["w"][0, 0, 0, :2] = (-8, 7)  # the full 4-bit range must unpack correctly
        c["w_packed"] = oracle.pack_int4(c["w"])
    want = _run_conv(c, f"conv {shape} batch {batch}")
    assert np.mean((want == c["act_min"]) | (want == c["act_max"])) < 0.75


STEM_SHAPES = [(65, 70, 3, 64, 7, 2, 3), (50, 130, 3, 32, 3, 2, 1), (23, 301, 3, 64, 7, 2, 3), (17, 40, 3, 20, 3, 2, 1),
               (40, 36, 4, 48, 3, 1, 1), (30, 30, 1, 40, 7, 2, 3), (31, 64, 2, 16, 7, 3, 2)]


@pytest.mark.parametrize("kernel", ["wave", "block"])
@pytest.mark.parametrize("shape", STEM_SHAPES, ids=lambda s: "x".join(map(str, s)))
def test_qconv2d_stem_kernels_match_oracle(tuning, kernel, shape):
    # both stem kernels (one wave per strip walking row segments: the default; one workgroup per strip: on request),
    # images tall enough for several row segments, fused and general rescale, extreme fill codes
    if kernel == "block":
        tuning.setenv("QNN_STEM_BLOCK", "1")
    H, W, Cin, Cout, k, s, p = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act="relu")
    c = synth.conv_case(layer, 2, 3100 + sum(shape), oracle, in_range=(-2.0, 2.2))
    for z_x in (c["z_x"], 0, 255):
        c["z_x"] = z_x
        _run_conv(c, f"stem ({kernel}) {shape} z_x={z_x}")
    c["shift"][0] = 0  # one column off the fused path sends the whole launch down the general one
    c["mult"][Cout - 1], c["shift"][Cout - 1] = 2 ** 30, -1
    _run_conv(c, f"stem ({kernel}) {shape}, general rescale")


@pytest.mark.parametrize("z_x", [0, 255])
def test_qconv2d_padding_uses_zero_point(z_x):
    layer = workloads.Layer("t", "conv", 6, 6, 16, 16, k=3, stride=1, pad=1, act="none")
    c = synth.conv_case(layer, 2, 950 + z_x, oracle)
    c["z_x"] = z_x
    _run_conv(c, f"padding z_x={z_x}")


# ------------------------------------------------------------------------------- qdwconv2d

DW_SHAPES = [
    # H, W, C, k, stride, pad
    (12, 12, 32, 3, 1, 1), (12, 12, 32, 3, 2, 1), (7, 7, 64, 3, 1, 1), (15, 9, 8, 3, 2, 1), (9, 11, 4, 3, 1, 0),
    (10, 10, 6, 3, 1, 1), (8, 8, 5, 5, 1, 2), (9, 9, 16, 3, 3, 1), (14, 14, 144, 3, 2, 1), (5, 5, 960, 3, 1, 1),
]


@pytest.mark.parametrize("shape", DW_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("batch", [1, 2])
def test_qdwconv2d_matches_oracle(shape, batch):
    H, W, Cc, k, s, p = shape
    layer = workloads.Layer("t", "dw", H, W, Cc, Cc, k=k, stride=s, pad=p)
    c = synth.conv_case(layer, batch, 1100 + 10 * DW_SHAPES.index(shape) + batch, oracle)
    for z_x in (c["z_x"], 201):
        want = oracle.qdwconv2d(c["x"], z_x, c["w"], c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"],
                                c["act_min"], c["act_max"], bias=c["bias"])
        got = host(qnn.qdwconv2d(dev(c["x"]), z_x, dev(c["w"]), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]),
                                 c["z_out"], c["act_min"], c["act_max"], bias=dev(c["bias"])))
        assert_same(got, want, f"dwconv {shape} batch {batch} z_x={z_x}")


@pytest.mark.parametrize("variant", ["QNN_DW_RH=2", "QNN_DW_RH=4", "QNN_DW_MAD=1"])
@pytest.mark.parametrize("shape", [(12, 12, 32, 3, 1, 1), (12, 12, 32, 3, 2, 1), (7, 7, 64, 3, 1, 1), (15, 9, 8, 3, 2, 1),
                                   (9, 11, 4, 3, 1, 0), (30, 17, 24, 3, 1, 1), (29, 31, 96, 3, 2, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_qdwconv2d_every_3x3_variant_matches_oracle(tuning, variant, shape):
    # patch heights 2 and 4 of the dot-product kernel and the multiply-add kernel, forced by environment
    name, value = variant.split("=")
    tuning.setenv(name, value)
    tuning.setenv("QNN_DW_VARIANT", "0")  # the patch kernels (the rolling-window kernels have a test of their own)
    H, W, C, k, s, p = shape
    layer = workloads.Layer("t", "dw", H, W, C, C, k=k, stride=s, pad=p, act="relu6")
    c = synth.conv_case(layer, 3, 1250 + sum(shape), oracle)
    for z_x in (c["z_x"], 0, 255):
        want = oracle.qdwconv2d(c["x"], z_x, c["w"], c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"],
                                c["act_min"], c["act_max"], bias=c["bias"])
        got = host(qnn.qdwconv2d(dev(c["x"]), z_x, dev(c["w"]), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]),
                                 c["z_out"], c["act_min"], c["act_max"], bias=dev(c["bias"])))
        assert_same(got, want, f"dwconv {variant} {shape} z_x={z_x}")


@pytest.mark.parametrize("variant,seg_rows", [(0, 0), (3, 0), (3, 1), (3, 2), (3, 5), (3, 9)])
@pytest.mark.parametrize("shape", [(12, 12, 32, 1, 1), (12, 12, 32, 2, 1), (7, 7, 64, 1, 1), (30, 17, 16, 1, 1), (29, 31, 96, 2, 1),
                                   (23, 45, 144, 1, 1), (9, 140, 32, 1, 1), (10, 150, 32, 2, 1), (17, 6, 512, 1, 1), (16, 9, 1024, 2, 1),
                                   (8, 8, 48, 1, 0), (11, 13, 80, 2, 0), (5, 40, 64, 1, 2), (3, 3, 16, 1, 1), (28, 28, 576, 1, 1)],
                         ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("act", ["relu6", "none"])
def test_qdwconv2d_rolling_window_kernel_matches_oracle(tuning, variant, seg_rows, shape, act):
    # variant 0: patch kernel, 3: matrix-unit kernel with the window rolling down a segment of rows;
    # seg_rows forces short segments (many segment borders, rings that wrap, segments of one row)
    tuning.setenv("QNN_DW_VARIANT", str(variant))
    if seg_rows:
        tuning.setenv("QNN_DW_RH", str(seg_rows))
    H, W, C, s, p = shape
    layer = workloads.Layer("t", "dw", H, W, C, C, k=3, stride=s, pad=p, act=act)
    c = synth.conv_case(layer, 2, 1270 + sum(shape), oracle)
    for z_x in (c["z_x"], 255):
        want = oracle.qdwconv2d(c["x"], z_x, c["w"], c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"],
                                c["act_min"], c["act_max"], bias=c["bias"])
        got = host(qnn.qdwconv2d(dev(c["x"]), z_x, dev(c["w"]), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]),
                                 c["z_out"], c["act_min"], c["act_max"], bias=dev(c["bias"])))
        assert_same(got, want, f"dwconv variant {variant} seg {seg_rows} {shape} {act} z_x={z_x}")


@pytest.mark.parametrize("variant", [0, 3])
@pytest.mark.parametrize("xcd", [0, 1])
@pytest.mark.parametrize("shape,batch", [((12, 12, 32, 1, 1), 1), ((29, 31, 96, 2, 1), 3), ((23, 45, 144, 1, 1), 2),
                                         ((9, 140, 32, 1, 1), 5), ((56, 56, 128, 1, 1), 3), ((28, 28, 256, 2, 1), 7)],
                         ids=lambda s: "x".join(map(str, s)) if isinstance(s, tuple) else str(s))
def test_qdwconv2d_workgroup_numbering_per_xcd_is_a_permutation(tuning, variant, xcd, shape, batch):
    # the renumbering that hands each XCD a contiguous share of the patches must visit every patch once,
    # whatever the workgroup count modulo 8 (batches and shapes chosen to give remainders 0..7)
    tuning.setenv("QNN_DW_VARIANT", str(variant))
    tuning.setenv("QNN_DW_XCD", str(xcd))
    H, W, C, s_, p = shape
    layer = workloads.Layer("t", "dw", H, W, C, C, k=3, stride=s_, pad=p, act="relu6")
    c = synth.conv_case(layer, batch, 1390 + sum(shape) + batch, oracle)
    want = oracle.qdwconv2d(c["x"], c["z_x"], c["w"], c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"],
                            c["act_min"], c["act_max"], bias=c["bias"])
    got = host(qnn.qdwconv2d(dev(c["x"]), c["z_x"], dev(c["w"]), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]),
                             c["z_out"], c["act_min"], c["act_max"], bias=dev(c["bias"])))
    assert_same(got, want, f"dwconv variant {variant} xcd {xcd} {shape} batch {batch}")


# ------------------------------------------------ pipelined (LDS-DMA) tile configurations

@pytest.fixture
def force_tile(tuning):
    def _set(name):
        tuning.setenv("QNN_FORCE_TILE", name)
    return _set


@pytest.mark.parametrize("tile", ["dma128x128", "dma256x256", "dma256x64", "dma256x128", "dma128x128s3", "dma64x64", "dma256x64s3", "128x128", "64x64",
                                  "p128x256", "p256x128"])
@pytest.mark.parametrize("M,N,K", [(128, 128, 64), (256, 256, 256), (300, 270, 192), (1000, 520, 1088), (17, 33, 16),
                                   (515, 700, 64), (700, 64, 128), (300, 50, 320)])
def test_qgemm_forced_tiles_match_oracle(force_tile, tile, M, N, K):
    force_tile(tile)
    rng = np.random.default_rng(1300 + M + N + K)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _gemm_params(rng, N, K)
    for z_a in (77, 128):
        want = oracle.qgemm(A, z_a, Bt, mult, shift, 128, 0, 255, bias=bias)
        got = host(qnn.qgemm(dev(A), z_a, dev(Bt), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias)))
        assert_same(got, want, f"qgemm tile={tile} {M}x{N}x{K} z_a={z_a}")


@pytest.mark.parametrize("tile", ["dma128x128", "dma256x256", "dma256x64", "dma256x128", "dma128x128s3", "dma64x64", "dma256x64s3", "p128x256",
                                  "p256x128"])
@pytest.mark.parametrize("shape", [(14, 14, 64, 96, 3, 1, 1), (15, 13, 64, 160, 3, 2, 1), (9, 9, 128, 40, 5, 1, 2),
                                   (16, 16, 128, 256, 1, 2, 0), (12, 12, 192, 300, 3, 1, 0), (20, 20, 64, 64, 3, 1, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_qconv2d_forced_dma_tiles_match_oracle(force_tile, tile, shape):
    force_tile(tile)
    H, W, Cin, Cout, k, s, p = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act="relu")
    c = synth.conv_case(layer, 3, 1400 + sum(shape), oracle)
    for z_x in (c["z_x"], 255):
        c["z_x"] = z_x
        _run_conv(c, f"conv tile={tile} {shape} z_x={z_x}")


@pytest.mark.parametrize("tile,M,N,K", [("p128x256", 128 * 41 + 5, 256 * 14 + 9, 192), ("p256x128", 256 * 21 + 77, 128 * 27, 128),
                                        ("dma256x256", 256 * 19, 256 * 15 + 1, 128), ("dma64x64", 64 * 37, 64 * 31, 64)])
@pytest.mark.parametrize("prio", [0, 1, 2, 3])
def test_qgemm_persistent_workgroups_walk_several_tiles(force_tile, tuning, tile, M, N, K, prio):
    # more tiles than resident workgroups: with QNN_PERSIST every workgroup loops over several tiles
    # (the operand ring and the output staging area are reused from tile to tile); every issue-priority
    # scheme of the main loop must give the same bits
    force_tile(tile)
    tuning.setenv("QNN_PERSIST", "2" if tile.startswith("p") else "1")
    tuning.setenv("QNN_GEMM_PRIO", str(prio))
    rng = np.random.default_rng(1350 + M + N + K)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _gemm_params(rng, N, K)
    want = oracle.qgemm(A, 91, Bt, mult, shift, 128, 0, 255, bias=bias)
    got = host(qnn.qgemm(dev(A), 91, dev(Bt), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias)))
    assert_same(got, want, f"persistent qgemm tile={tile} {M}x{N}x{K} prio={prio}")


def test_qconv2d_persistent_workgroups(force_tile, tuning):
    force_tile("p256x128")
    tuning.setenv("QNN_PERSIST", "2")
    layer = workloads.Layer("t", "conv", 40, 40, 64, 128, k=3, stride=1, pad=1, act="relu")
    c = synth.conv_case(layer, 96, 1377, oracle)  # 153600 rows = 600 tiles of 256 rows
    _run_conv(c, "persistent conv p256x128")


@pytest.mark.parametrize("tile", ["dma64x64", "dma128x128", "dma256x256", None])
@pytest.mark.parametrize("M,N,K", [(128, 64, 64), (300, 270, 320), (1000, 520, 1088), (515, 96, 576), (2000, 40, 960)])
def test_qgemm_packed_4bit_weights_on_the_pipelined_tiles(tuning, tile, M, N, K):
    # nibble pairs go to LDS as they are and are expanded in registers after the fragment read;
    # -8 and 7 injected, zero-points away from 128 so that the column sums matter
    if tile:
        tuning.setenv("QNN_FORCE_TILE", tile)
    rng = np.random.default_rng(1360 + M + N + K)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-8, 8, (N, K)).astype(np.int8)
    Bt[0, :4] = (-8, 7, -8, 7)
    Bt[N - 1, K - 2:] = (-8, -8)
    B = oracle.pack_int4(Bt)
    bias, mult, shift = _gemm_params(rng, N, K)
    mult, shift = oracle.quantize_multipliers(10 ** rng.uniform(-3.2, -2.6, N) / np.sqrt(K / 64.0))
    for z_a in (0, 128, 255):
        want = oracle.qgemm(A, z_a, B, mult, shift, 128, 0, 255, bias=bias, weight_bits=4)
        got = host(qnn.qgemm(dev(A), z_a, dev(B), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias), weight_bits=4))
        assert_same(got, want, f"int4 qgemm tile={tile} {M}x{N}x{K} z_a={z_a}")
        assert len(np.unique(want)) > 32


@pytest.mark.parametrize("tile", ["dma64x64", "dma128x128", "dma256x256"])
@pytest.mark.parametrize("shape", [(14, 14, 64, 96, 3, 1, 1), (15, 13, 64, 160, 3, 2, 1), (12, 12, 192, 300, 3, 1, 0)],
                         ids=lambda s: "x".join(map(str, s)))
def test_qconv2d_packed_4bit_weights_on_the_pipelined_tiles(force_tile, tile, shape):
    force_tile(tile)
    H, W, Cin, Cout, k, s, p = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act="relu", weight_bits=4)
    c = synth.conv_case(layer, 3, 1460 + sum(shape), oracle)
    _run_conv(c, f"int4 conv tile={tile} {shape}")


# ------------------------------------------------------------ short reduction (K <= 256), weight-stationary kernel

def _short_k_params(rng, N, K, bits):
    real = 10 ** rng.uniform(-4.2, -3.2, N) / np.sqrt(K / 64.0) * (1.0 if bits == 8 else 14.0)
    mult, shift = oracle.quantize_multipliers(real)
    bias = rng.integers(-20000, 20000, N).astype(np.int32)
    return bias, mult, shift


@pytest.mark.parametrize("K", [8, 16, 24, 32, 40, 64, 96, 128, 136, 144, 192, 256])
@pytest.mark.parametrize("M,N", [(65, 1), (100, 16), (999, 33), (300, 96), (1000, 130), (4097, 256), (200, 300)])
@pytest.mark.parametrize("bits", [8, 4])
def test_qgemm_short_k_matches_oracle(M, N, K, bits):
    assert qnn.qgemm_plan(M, N, K) == "shortk"
    rng = np.random.default_rng(1800 + M + N + K + bits)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    if bits == 8:
        Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
        B = Bt
    else:
        Bt = rng.integers(-8, 8, (N, K)).astype(np.int8)
        B = oracle.pack_int4(Bt)
    bias, mult, shift = _short_k_params(rng, N, K, bits)
    for z_a in (0, 128, 255):
        want = oracle.qgemm(A, z_a, B, mult, shift, 120, 5, 250, bias=bias, weight_bits=bits)
        got = host(qnn.qgemm(dev(A), z_a, dev(B), dev(mult), dev(shift), 120, 5, 250, bias=dev(bias), weight_bits=bits))
        assert_same(got, want, f"short-K qgemm {M}x{N}x{K} bits={bits} z_a={z_a}")


@pytest.mark.parametrize("K,N", [(64, 70), (160, 40), (256, 129)])
def test_qgemm_short_k_general_rescale_columns(K, N):
    # columns whose multiplier / shift / bias fall outside the fast form: the whole wave takes the general path
    M = 500
    rng = np.random.default_rng(1900 + K + N)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _short_k_params(rng, N, K, 8)
    shift[0] = 0
    mult[1], shift[1] = 2 ** 30, -1          # multiplier 1: left shift
    mult[2], shift[2] = 2 ** 30 + 12345, -3
    shift[3] = 25
    shift[N - 1] = 31
    bias[5] = 2 ** 28
    bias[6] = -(2 ** 28)
    for z_a in (3, 128):
        want = oracle.qgemm(A, z_a, Bt, mult, shift, 7, 0, 255, bias=bias)
        got = host(qnn.qgemm(dev(A), z_a, dev(Bt), dev(mult), dev(shift), 7, 0, 255, bias=dev(bias)))
        assert_same(got, want, f"short-K general rescale {M}x{N}x{K} z_a={z_a}")


@pytest.mark.parametrize("K,pad_a,pad_c", [(256, 16, 16), (128, 48, 32), (256, 32, 0), (256, 8, 16)])
def test_qgemm_short_k_rows_through_lds_spaced_rows(K, pad_a, pad_c):
    # the staged form (A rows copied to LDS per workgroup) on column slices of wider matrices: lda > K, ldc > N;
    # pad 8 leaves the rows 8-byte aligned only, which takes the direct loads instead
    import torch
    M, N = 1333, 576
    rng = np.random.default_rng(2100 + K + pad_a + pad_c)
    wide_a = rng.integers(0, 256, (M, K + pad_a)).astype(np.uint8)
    A = wide_a[:, :K]
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _short_k_params(rng, N, K, 8)
    wide_c = torch.full((M, N + pad_c), 77, dtype=torch.uint8, device="cuda")
    want = oracle.qgemm(np.ascontiguousarray(A), 100, Bt, mult, shift, 128, 0, 255, bias=bias)
    qnn.qgemm(dev(wide_a)[:, :K], 100, dev(Bt), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias), out=wide_c[:, :N])
    got = host(wide_c)
    assert_same(got[:, :N], want, f"short-K through LDS, spaced rows K={K}")
    assert (got[:, N:] == 77).all(), "columns outside the output slice were written"


@pytest.mark.parametrize("K,pad_a,pad_c", [(64, 16, 16), (64, 8, 3), (96, 24, 0), (128, 0, 5), (40, 8, 1)])
def test_qgemm_short_k_spaced_rows(K, pad_a, pad_c):
    # A and C are column slices of wider matrices (lda > K, ldc > N); pad 8 leaves rows only 8-byte aligned
    import torch
    M, N = 333, 72
    rng = np.random.default_rng(2000 + K + pad_a + pad_c)
    wide_a = rng.integers(0, 256, (M, K + pad_a)).astype(np.uint8)
    A = wide_a[:, :K]
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _short_k_params(rng, N, K, 8)
    wide_c = torch.full((M, N + pad_c), 77, dtype=torch.uint8, device="cuda")
    want = oracle.qgemm(np.ascontiguousarray(A), 100, Bt, mult, shift, 128, 0, 255, bias=bias)
    qnn.qgemm(dev(wide_a)[:, :K], 100, dev(Bt), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias), out=wide_c[:, :N])
    got = host(wide_c)
    assert_same(got[:, :N], want, f"short-K spaced rows K={K}")
    assert (got[:, N:] == 77).all(), "columns outside the output slice were written"


@pytest.mark.parametrize("shape", [(28, 28, 64, 160, 1, 2, 0), (15, 13, 128, 96, 1, 2, 0), (9, 9, 256, 40, 1, 3, 0),
                                   (14, 14, 96, 24, 1, 1, 0), (14, 14, 144, 32, 1, 1, 0), (7, 7, 24, 144, 1, 1, 0)],
                         ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("bits", [8, 4])
def test_qconv2d_pointwise_short_k_matches_oracle(shape, bits):
    H, W, Cin, Cout, k, s, p = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act="relu6", weight_bits=bits)
    c = synth.conv_case(layer, 5, 2100 + sum(shape) + bits, oracle)
    for z_x in (c["z_x"], 0, 255):
        c["z_x"] = z_x
        _run_conv(c, f"pointwise short-K conv {shape} bits={bits} z_x={z_x}")


# ------------------------------------------------------------ medium reduction, weight-resident kernel

@pytest.mark.parametrize("M,N,K", [(4096, 128, 512), (5000, 200, 320), (4100, 64, 1024), (4096, 30, 288), (6000, 256, 1152),
                                   (4097, 97, 1280), (4500, 100, 352), (4300, 40, 736)])
@pytest.mark.parametrize("bits", [8, 4])
def test_qgemm_weight_resident_matches_oracle(tuning, M, N, K, bits):
    tuning.setenv("QNN_BRES", "1")  # shapes this small take the kernel only on request
    rng = np.random.default_rng(2400 + M + N + K + bits)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    if bits == 8:
        Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
        B = Bt
    else:
        Bt = rng.integers(-8, 8, (N, K)).astype(np.int8)
        B = oracle.pack_int4(Bt)
    bias, mult, shift = _short_k_params(rng, N, K, bits)
    for z_a in (0, 128, 255):
        want = oracle.qgemm(A, z_a, B, mult, shift, 120, 5, 250, bias=bias, weight_bits=bits)
        got = host(qnn.qgemm(dev(A), z_a, dev(B), dev(mult), dev(shift), 120, 5, 250, bias=dev(bias), weight_bits=bits))
        assert_same(got, want, f"weight-resident qgemm {M}x{N}x{K} bits={bits} z_a={z_a}")


def test_qgemm_weight_resident_default_plan():
    M, N, K = 40000, 128, 512
    assert qnn.qgemm_plan(M, N, K) == "bres"
    c = synth.gemm_case(M, N, K, workloads.seed_for(2, 90), oracle)
    got = host(qnn.qgemm(dev(c["A"]), c["z_a"], dev(c["Bt"]), dev(c["mult"]), dev(c["shift"]), c["z_out"], 0, 255))
    want = oracle.qgemm(c["A"], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
    assert_same(got, want, "weight-resident qgemm 40000x128x512, default plan")


def test_qgemm_weight_resident_general_rescale_and_many_column_groups(tuning):
    tuning.setenv("QNN_BRES", "1")  # also for N > 256 (several column groups)
    M, N, K = 4200, 600, 384
    rng = np.random.default_rng(2500)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _short_k_params(rng, N, K, 8)
    want = oracle.qgemm(A, 77, Bt, mult, shift, 128, 0, 255, bias=bias)
    got = host(qnn.qgemm(dev(A), 77, dev(Bt), dev(mult), dev(shift), 128, 0, 255, bias=dev(bias)))
    assert_same(got, want, "weight-resident qgemm, 5 column groups")
    shift[0] = 0
    mult[1], shift[1] = 2 ** 30, -1
    shift[N - 1] = 27
    bias[5] = 2 ** 28
    want = oracle.qgemm(A, 3, Bt, mult, shift, 7, 0, 255, bias=bias)
    got = host(qnn.qgemm(dev(A), 3, dev(Bt), dev(mult), dev(shift), 7, 0, 255, bias=dev(bias)))
    assert_same(got, want, "weight-resident qgemm, general rescale")


@pytest.mark.parametrize("shape,batch", [((40, 40, 64, 64, 3, 1, 1), 3), ((41, 37, 32, 96, 3, 2, 1), 12), ((30, 30, 32, 40, 5, 1, 2), 6),
                                         ((64, 64, 512, 128, 1, 2, 0), 4), ((36, 36, 128, 130, 3, 1, 0), 4)],
                         ids=lambda s: "x".join(map(str, s)) if isinstance(s, tuple) else str(s))
@pytest.mark.parametrize("bits", [8, 4])
def test_qconv2d_weight_resident_matches_oracle(tuning, shape, batch, bits):
    H, W, Cin, Cout, k, s, p = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act="relu", weight_bits=bits)
    tuning.setenv("QNN_BRES", "1")
    c = synth.conv_case(layer, batch, 2600 + sum(shape) + bits, oracle)
    for z_x in (c["z_x"], 255):
        c["z_x"] = z_x
        _run_conv(c, f"weight-resident conv {shape} bits={bits} z_x={z_x}")


# ------------------------------------------------------------ split-K (few output tiles, long K)

@pytest.mark.parametrize("tile", ["dma128x128", "dma64x64"])
@pytest.mark.parametrize("splits", [2, 3, 7])
@pytest.mark.parametrize("M,N,K", [(128, 128, 448), (300, 270, 640), (131, 66, 1088), (256, 63, 8192)])
def test_qgemm_split_k_matches_oracle(force_tile, tuning, tile, splits, M, N, K):
    force_tile(tile)
    tuning.setenv("QNN_FORCE_SPLIT", str(splits))
    rng = np.random.default_rng(1600 + M + N + K + splits)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
    bias, mult, shift = _gemm_params(rng, N, K)
    shift[0] = 0      # a column on the general rescale path
    mult[N // 2], shift[N // 2] = 2 ** 30, -1
    for z_a in (0, 128, 255):
        want = oracle.qgemm(A, z_a, Bt, mult, shift, 100, 3, 251, bias=bias)
        got = host(qnn.qgemm(dev(A), z_a, dev(Bt), dev(mult), dev(shift), 100, 3, 251, bias=dev(bias)))
        assert_same(got, want, f"split-K qgemm tile={tile} splits={splits} {M}x{N}x{K} z_a={z_a}")


def test_two_captured_split_k_graphs_replayed_concurrently_with_their_own_workspaces():
    # Scratch memory comes from the caller, so two products that both divide K over several workgroups can be
    # captured into graphs and replayed at the same time on two streams, each with its own workspace; replayed
    # several times with eager work in between, every replay is compared with the oracle
    import torch
    shapes = [(1024, 1024, 8192, 61), (256, 640, 4096, 62)]
    cases, graphs, streams = [], [], [torch.cuda.Stream(), torch.cuda.Stream()]
    for (M, N, K, seed), st in zip(shapes, streams):
        assert "/k" in qnn.qgemm_plan(M, N, K)
        c = synth.gemm_case(M, N, K, workloads.seed_for(2, seed), oracle)
        t = dict(A=dev(c["A"]), Bt=dev(c["Bt"]), mult=dev(c["mult"]), shift=dev(c["shift"]),
                 C=torch.zeros((M, N), dtype=torch.uint8, device="cuda:0"),
                 ws=torch.empty(qnn.qgemm_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda:0"))
        rows = np.r_[0:16, M - 16:M]
        want = oracle.qgemm(c["A"][rows], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
        cases.append((c, t, rows, want))
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.stream(st):
            qnn.qgemm(t["A"], c["z_a"], t["Bt"], t["mult"], t["shift"], c["z_out"], 0, 255, out=t["C"], workspace=t["ws"])  # warm-up
            st.synchronize()
            with torch.cuda.graph(g, stream=st):
                qnn.qgemm(t["A"], c["z_a"], t["Bt"], t["mult"], t["shift"], c["z_out"], 0, 255, out=t["C"], workspace=t["ws"])
        graphs.append(g)
    for rep in range(4):
        for (c, t, rows, want) in cases:
            t["C"].zero_()
            t["ws"].fill_(0xA5 + rep)  # whatever the workspace holds must not matter
        torch.cuda.synchronize()
        for g, st in zip(graphs, streams):
            with torch.cuda.stream(st):
                g.replay()
        torch.cuda.synchronize()
        for (c, t, rows, want) in cases:
            assert_same(host(t["C"])[rows], want, f"concurrent split-K graph replay {rep} {tuple(t['C'].shape)}")


@pytest.mark.parametrize("tile", ["dma128x128", "dma64x64"])
@pytest.mark.parametrize("shape", [(14, 14, 64, 96, 3, 1, 1), (9, 9, 128, 40, 5, 1, 2), (7, 7, 512, 130, 3, 1, 1)],
                         ids=lambda s: "x".join(map(str, s)))
def test_qconv2d_split_k_matches_oracle(force_tile, tuning, tile, shape):
    force_tile(tile)
    tuning.setenv("QNN_FORCE_SPLIT", "4")
    H, W, Cin, Cout, k, s, p = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p, act="relu6")
    c = synth.conv_case(layer, 3, 1700 + sum(shape), oracle)
    for z_x in (c["z_x"], 0):
        c["z_x"] = z_x
        _run_conv(c, f"split-K conv tile={tile} {shape} z_x={z_x}")


def test_qgemm_default_plan_splits_k_when_tiles_are_few():
    # 256 x 512 x 8192: 8 tiles of 128x128 would leave most of the chip idle; the plan divides K
    M, N, K = 256, 512, 8192
    plan = qnn.qgemm_plan(M, N, K)
    assert "/k" in plan, plan
    c = synth.gemm_case(M, N, K, workloads.seed_for(2, 78), oracle)
    for _ in range(2):  # the second call reuses the scratch block
        got = host(qnn.qgemm(dev(c["A"]), c["z_a"], dev(c["Bt"]), dev(c["mult"]), dev(c["shift"]), c["z_out"], 0, 255))
    want = oracle.qgemm(c["A"], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
    assert_same(got, want, "qgemm 256x512x8192 default split-K plan")


def test_qgemm_split_k_on_two_streams_shares_the_scratch_block():
    import torch
    M, N, K = 256, 256, 4096
    assert "/k" in qnn.qgemm_plan(M, N, K)
    cases = [synth.gemm_case(M, N, K, workloads.seed_for(2, 80 + i), oracle) for i in range(2)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    devs = [{k: dev(c[k]) for k in ("A", "Bt", "mult", "shift")} for c in cases]
    outs = [[], []]
    torch.cuda.synchronize()
    for rep in range(4):
        for i, st in enumerate(streams):
            with torch.cuda.stream(st):
                d, c = devs[i], cases[i]
                outs[i].append(qnn.qgemm(d["A"], c["z_a"], d["Bt"], d["mult"], d["shift"], c["z_out"], 0, 255))
    torch.cuda.synchronize()
    for i, c in enumerate(cases):
        want = oracle.qgemm(c["A"], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
        for rep, o in enumerate(outs[i]):
            assert_same(host(o), want, f"split-K on stream {i}, call {rep}")


def test_qgemm_default_plan_large_shape_sampled_rows():
    # 4096 x 4096 x 512 selects the 256x256 pipelined tile by itself (256 tiles); compare whole rows
    # at the top, in the middle and at the bottom of the matrix
    M, N, K = 4096, 4096, 512
    assert qnn.qgemm_plan(M, N, K) == "dma256x256"
    c = synth.gemm_case(M, N, K, workloads.seed_for(2, 77), oracle)
    got = host(qnn.qgemm(dev(c["A"]), c["z_a"], dev(c["Bt"]), dev(c["mult"]), dev(c["shift"]), c["z_out"], 0, 255))
    rows = np.r_[0:64, 2000:2064, 4032:4096]
    want = oracle.qgemm(c["A"][rows], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
    assert_same(got[rows], want, "qgemm 4096x4096x512 sampled rows")


@pytest.mark.parametrize("alds", [1, 0])
@pytest.mark.parametrize("M,N,K", [(1, 256, 256), (31, 300, 256), (100, 256, 256), (1000, 300, 256), (33, 512, 128), (5000, 1024, 128),
                                   (4097, 520, 256), (65, 8192, 256), (7000, 2100, 128)])
@pytest.mark.parametrize("bits", [8, 4])
def test_qgemm_short_k_rows_through_lds(tuning, alds, M, N, K, bits):
    # short-K kernel with the A rows copied to LDS once per workgroup (K = 128 / 256): ragged row blocks, column
    # counts that leave a workgroup with idle waves, one and many walkers; the switch off = direct fragment loads
    tuning.setenv("QNN_SHORTK_ALDS", str(alds))
    if M > 64:
        assert qnn.qgemm_plan(M, N, K) == "shortk"
    rng = np.random.default_rng(1600 + M + N + K + bits)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    A[0, :] = 255
    A[-1, :] = 0
    lim = 8 if bits == 4 else 128
    Bt = rng.integers(-lim, lim, (N, K)).astype(np.int8)
    Bt[0, :] = -lim
    B = oracle.pack_int4(Bt) if bits == 4 else Bt
    real = 10 ** rng.uniform(-4.2, -3.2, N) / np.sqrt(K / 64.0) * (16.0 if bits == 4 else 1.0)
    mult, shift = oracle.quantize_multipliers(real)
    bias = rng.integers(-20000, 20000, N).astype(np.int32)
    for z_a, lo in ((0, 0), (128, 120), (255, 0)):
        want = oracle.qgemm(A, z_a, B, mult, shift, 120, lo, 250, bias=bias, weight_bits=bits)
        got = host(qnn.qgemm(dev(A), z_a, dev(B), dev(mult), dev(shift), 120, lo, 250, bias=dev(bias), weight_bits=bits))
        assert_same(got, want, f"short-K through LDS={alds} {M}x{N}x{K} bits={bits} z_a={z_a}")


def test_empty_batches_are_no_ops():
    import torch
    z = lambda *shape, dt=torch.uint8: torch.empty(shape, dtype=dt, device="cuda:0")
    mult = torch.full((8,), 1 << 30, dtype=torch.int32, device="cuda:0")
    shift = torch.full((8,), 5, dtype=torch.int32, device="cuda:0")
    assert tuple(qnn.qgemm(z(0, 64), 128, z(8, 64, dt=torch.int8), mult, shift, 0, 0, 255).shape) == (0, 8)
    w = z(8, 3, 3, 16, dt=torch.int8)
    assert tuple(qnn.qconv2d(z(0, 9, 9, 16), 3, w, (1, 1), (1, 1), mult, shift, 0, 0, 255).shape) == (0, 9, 9, 8)
    wd = z(3, 3, 8, dt=torch.int8)
    assert tuple(qnn.qdwconv2d(z(0, 9, 9, 8), 3, wd, (2, 2), (1, 1), mult, shift, 0, 0, 255).shape) == (0, 5, 5, 8)
    assert qnn.quantize(z(0, dt=torch.float32), 0.1, 3).numel() == 0
    torch.cuda.synchronize()


# ------------------------------------------------------------ few-row (weight streaming) kernel

@pytest.mark.parametrize("M,N,K", [(1, 16, 64), (5, 50, 192), (16, 33, 64), (17, 100, 1024), (33, 257, 576), (64, 48, 4096),
                                   (48, 1000, 128), (1, 40, 128), (3, 64, 384), (32, 20, 2048), (64, 16, 256), (2, 7, 8192),
                                   (20, 130, 1152)])
@pytest.mark.parametrize("bits", [8, 4])
def test_qgemm_few_rows_matches_oracle(M, N, K, bits):
    assert qnn.qgemm_plan(M, N, K) == "skinny16"
    rng = np.random.default_rng(1500 + M + N + K + bits)
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    if bits == 8:
        Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
        B = Bt
        real = 10 ** rng.uniform(-4.2, -3.2, N) / np.sqrt(K / 64.0)
    else:
        Bt = rng.integers(-8, 8, (N, K)).astype(np.int8)
        B = oracle.pack_int4(Bt)
        real = 10 ** rng.uniform(-3.0, -2.2, N) / np.sqrt(K / 64.0)
    mult, shift = oracle.quantize_multipliers(real)
    shift[0] = 0
    bias = rng.integers(-20000, 20000, N).astype(np.int32)
    for z_a in (0, 128, 201):
        want = oracle.qgemm(A, z_a, B, mult, shift, 120, 5, 250, bias=bias, weight_bits=bits)
        got = host(qnn.qgemm(dev(A), z_a, dev(B), dev(mult), dev(shift), 120, 5, 250, bias=dev(bias), weight_bits=bits))
        assert_same(got, want, f"few-row qgemm {M}x{N}x{K} bits={bits} z_a={z_a}")


# ------------------------------------------------- rectangular kernels, strides and paddings

RECT_CASES = [
    # N, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw, bits
    (2, 17, 23, 16, 24, 1, 3, 1, 1, 0, 1, 8),
    (3, 20, 14, 32, 40, 3, 5, 2, 1, 1, 2, 8),
    (1, 31, 9, 64, 64, 7, 1, 3, 2, 3, 0, 8),
    (2, 12, 40, 3, 32, 3, 7, 1, 2, 1, 3, 8),      # few channels, kernel row of 21 bytes: stem kernels
    (2, 19, 19, 128, 96, 1, 1, 2, 3, 0, 0, 8),    # 1x1 with different strides: strided short-K rows
    (2, 16, 16, 64, 48, 3, 3, 1, 2, 2, 0, 4),
    (1, 9, 33, 20, 30, 5, 2, 2, 2, 4, 1, 8),      # padding larger than half the kernel
]


@pytest.mark.parametrize("case", RECT_CASES, ids=lambda c: "x".join(map(str, c)))
def test_qconv2d_rectangular_geometry_matches_oracle(case):
    N, H, W, Cin, Cout, kh, kw, sh, sw, ph, pw, bits = case
    rng = np.random.default_rng(8000 + sum(case))
    x = rng.integers(0, 256, (N, H, W, Cin)).astype(np.uint8)
    lim = 8 if bits == 4 else 128
    w = rng.integers(-lim, lim, (Cout, kh, kw, Cin)).astype(np.int8)
    K = kh * kw * Cin
    mult, shift = oracle.quantize_multipliers(10 ** rng.uniform(-4.2, -3.2, Cout) / np.sqrt(K / 64.0) * (16.0 if bits == 4 else 1.0))
    bias = rng.integers(-20000, 20000, Cout).astype(np.int32)
    w_o = oracle.pack_int4(w) if bits == 4 else w
    for z_x in (97, 0, 255):
        want = oracle.qconv2d(x, z_x, w_o, (sh, sw), (ph, pw), mult, shift, 110, 0, 255, bias=bias, weight_bits=bits)
        got = host(qnn.qconv2d(dev(x), z_x, dev(w_o), (sh, sw), (ph, pw), dev(mult), dev(shift), 110, 0, 255, bias=dev(bias),
                               weight_bits=bits))
        assert_same(got, want, f"qconv2d rectangular {case} z_x={z_x}")
    assert want.shape == (N, (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1, Cout)


@pytest.mark.parametrize("case", [(2, 15, 22, 16, 3, 5, 1, 2, 1, 2), (1, 30, 9, 7, 1, 3, 2, 1, 0, 1), (2, 12, 12, 32, 3, 3, 2, 1, 1, 1),
                                  (1, 20, 20, 8, 7, 7, 3, 3, 3, 3)], ids=lambda c: "x".join(map(str, c)))
def test_qdwconv2d_rectangular_geometry_matches_oracle(case):
    N, H, W, Cc, kh, kw, sh, sw, ph, pw = case
    rng = np.random.default_rng(8100 + sum(case))
    x = rng.integers(0, 256, (N, H, W, Cc)).astype(np.uint8)
    w = rng.integers(-128, 128, (kh, kw, Cc)).astype(np.int8)
    mult, shift = oracle.quantize_multipliers(10 ** rng.uniform(-3.6, -2.8, Cc) / np.sqrt(kh * kw / 9.0))
    bias = rng.integers(-5000, 5000, Cc).astype(np.int32)
    for z_x in (97, 0, 255):
        want = oracle.qdwconv2d(x, z_x, w, (sh, sw), (ph, pw), mult, shift, 110, 0, 255, bias=bias)
        got = host(qnn.qdwconv2d(dev(x), z_x, dev(w), (sh, sw), (ph, pw), dev(mult), dev(shift), 110, 0, 255, bias=dev(bias)))
        assert_same(got, want, f"qdwconv2d rectangular {case} z_x={z_x}")


# ------------------------------------------------------------------ exact ties below the lower clamp

@pytest.mark.parametrize("z_out,act_min,act_max", [(0, 0, 255), (7, 7, 130), (3, 10, 200), (40, 0, 255), (128, 5, 250)])
def test_rounding_ties_next_to_the_lower_clamp(tuning, z_out, act_min, act_max):
    """Small accumulators with multipliers 2^30 and 3 * 2^29 and shifts 1..4: every second or fourth
    sum is an exact tie, negative ones included.  With act_min >= z_out the kernels drop the
    ties-away term for negative values (the clamp decides there); the result must not change."""
    rng = np.random.default_rng(977 + z_out + act_min)
    z_a = 77
    for M, N, K, tile in [(200, 48, 16, None), (300, 130, 64, None), (256, 128, 64, "dma128x128"), (130, 70, 64, "64x64"),
                          (4096, 64, 288, None), (32768, 64, 288, None)]:
        A = (z_a + rng.integers(-1, 2, (M, K))).astype(np.uint8)
        Bt = rng.integers(-1, 2, (N, K)).astype(np.int8)
        bias = rng.integers(-24, 25, N).astype(np.int32)
        mult = np.where(rng.integers(0, 2, N) == 0, 1 << 30, 3 << 29).astype(np.int32)
        shift = rng.integers(1, 5, N).astype(np.int32)
        if tile:
            tuning.setenv("QNN_FORCE_TILE", tile)
        else:
            tuning.delenv("QNN_FORCE_TILE", raising=False)
        want = oracle.qgemm(A, z_a, Bt, mult, shift, z_out, act_min, act_max, bias=bias)
        got = host(qnn.qgemm(dev(A), z_a, dev(Bt), dev(mult), dev(shift), z_out, act_min, act_max, bias=dev(bias)))
        assert_same(got, want, f"ties {M}x{N}x{K} tile={tile} z_out={z_out} act=[{act_min},{act_max}] ({qnn.qgemm_plan(M, N, K)})")
    tuning.delenv("QNN_FORCE_TILE", raising=False)
    # depthwise 3x3 and a stem-shaped convolution
    C = 32
    x = (z_a + rng.integers(-1, 2, (2, 12, 12, C))).astype(np.uint8)
    w = rng.integers(-1, 2, (3, 3, C)).astype(np.int8)
    bias = rng.integers(-8, 9, C).astype(np.int32)
    mult = np.where(rng.integers(0, 2, C) == 0, 1 << 30, 3 << 29).astype(np.int32)
    shift = rng.integers(1, 4, C).astype(np.int32)
    want = oracle.qdwconv2d(x, z_a, w, (1, 1), (1, 1), mult, shift, z_out, act_min, act_max, bias=bias)
    got = host(qnn.qdwconv2d(dev(x), z_a, dev(w), (1, 1), (1, 1), dev(mult), dev(shift), z_out, act_min, act_max, bias=dev(bias)))
    assert_same(got, want, f"ties depthwise z_out={z_out} act=[{act_min},{act_max}]")
    xs = (z_a + rng.integers(-1, 2, (2, 20, 20, 3))).astype(np.uint8)
    ws = rng.integers(-1, 2, (32, 3, 3, 3)).astype(np.int8)
    bias = rng.integers(-12, 13, 32).astype(np.int32)
    mult = np.where(rng.integers(0, 2, 32) == 0, 1 << 30, 3 << 29).astype(np.int32)
    shift = rng.integers(1, 4, 32).astype(np.int32)
    want = oracle.qconv2d(xs, z_a, ws, (2, 2), (1, 1), mult, shift, z_out, act_min, act_max, bias=bias)
    got = host(qnn.qconv2d(dev(xs), z_a, dev(ws), (2, 2), (1, 1), dev(mult), dev(shift), z_out, act_min, act_max, bias=dev(bias)))
    assert_same(got, want, f"ties stem conv z_out={z_out} act=[{act_min},{act_max}]")
