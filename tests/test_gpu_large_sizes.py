"""Tensors whose byte offsets do not fit 32 bits: the kernels must index them with 64-bit arithmetic.
Inputs are generated on the device (seeded); the oracle checks slices that lie beyond the 4 GiB mark
(and the first ones), element by element."""
import numpy as np
import pytest
import torch

import oracle
import paper_1806_08342_amd as qnn

from gpu_util import assert_same, dev, host

pytestmark = pytest.mark.gpu

BIG = 2 ** 32 + 4099  # elements


def _slices(n, width=5000):
    return [(0, width), (2 ** 31 - 77, 2 ** 31 - 77 + width), (2 ** 32 - 100, 2 ** 32 + 150), (n - width, n)]


def test_streaming_kernels_beyond_4gi_elements():
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7001)
    x = torch.empty(BIG, dtype=torch.float32, device="cuda:0")
    x.normal_(0.0, 2.0, generator=g)
    q = qnn.quantize(x, 0.0213, 131)
    st = qnn.new_range_state()
    qnn.minmax(x, st)
    rng_state = qnn.read_range_state(st)
    assert rng_state["xmin"] == float(x.min()) and rng_state["xmax"] == float(x.max())
    for lo, hi in _slices(BIG):
        xs = host(x[lo:hi])
        assert_same(host(q[lo:hi]), oracle.quantize(xs, 0.0213, 131), f"quantize [{lo}:{hi}]")
    del x
    back = qnn.dequantize(q, 0.0213, 131)
    for lo, hi in _slices(BIG):
        want = oracle.dequantize(host(q[lo:hi]), 0.0213, 131)
        assert np.array_equal(host(back[lo:hi]).view(np.uint32), want.view(np.uint32)), f"dequantize [{lo}:{hi}]"
    del back
    b = torch.randint(0, 256, (BIG,), dtype=torch.uint8, device="cuda:0", generator=g)
    p = oracle.qadd_params(0.02, 0.031, 0.04)
    y = qnn.qadd(q, 120, b, 131, p, 3, 0, 255)
    for lo, hi in _slices(BIG):
        assert_same(host(y[lo:hi]), oracle.qadd(host(q[lo:hi]), 120, host(b[lo:hi]), 131, p, 3, 0, 255), f"qadd [{lo}:{hi}]")


def test_requantize_beyond_4gi_elements():
    ch = 256
    rows = BIG // ch + 3
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7002)
    acc = torch.randint(-300000, 300000, (rows, ch), dtype=torch.int32, device="cuda:0", generator=g)
    mult, shift = oracle.quantize_multipliers([0.0006 * (1 + 0.013 * i) for i in range(ch)])
    y = qnn.requantize(acc, dev(mult), dev(shift), True, 128, 0, 255)
    for r0 in (0, 2 ** 31 // ch - 3, 2 ** 32 // ch - 2, rows - 40):
        want = oracle.requantize(host(acc[r0:r0 + 40]), mult, shift, True, 128, 0, 255)
        assert_same(host(y[r0:r0 + 40]), want, f"requantize rows {r0}..")


def test_qgemm_with_operand_and_result_beyond_4gib():
    # A: 560000 x 8192 bytes = 4.6 GB; C: 560000 x 8192 = 4.6 GB through the tiled kernel,
    # then a few-column product on the same A through the weight-resident / tiled route
    M, K = 560_000, 8192
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7003)
    A = torch.randint(0, 256, (M, K), dtype=torch.uint8, device="cuda:0", generator=g)
    rng = np.random.default_rng(7004)
    for N in (8192, 64):
        Bt = rng.integers(-128, 128, (N, K)).astype(np.int8)
        mult, shift = oracle.quantize_multipliers(10 ** rng.uniform(-4.2, -3.2, N) / np.sqrt(K / 64.0))
        bias = rng.integers(-20000, 20000, N).astype(np.int32)
        Cm = qnn.qgemm(A, 131, dev(Bt), dev(mult), dev(shift), 120, 0, 255, bias=dev(bias))
        for r0 in (0, 2 ** 32 // K - 5, M - 300):  # rows around the 4 GiB mark of A (and of C when N = 8192), and the last ones
            rows = slice(r0, r0 + 300 if N == 64 else r0 + 12)
            want = oracle.qgemm(host(A[rows]), 131, Bt, mult, shift, 120, 0, 255, bias=bias)
            assert_same(host(Cm[rows]), want, f"qgemm {M}x{N}x{K} rows {r0}.. plan={qnn.qgemm_plan(M, N, K)}")
        del Cm


def test_qconv2d_with_tensors_beyond_4gib():
    # 140 images of 256 x 256 x 512: 4.7 GB in; 3x3 convolution to 128 channels and a 1x1 to 512 (4.7 GB out)
    import workloads
    from workloads import synth
    N, H, W, Cin = 140, 256, 256, 512
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7005)
    x = torch.randint(0, 256, (N, H, W, Cin), dtype=torch.uint8, device="cuda:0", generator=g)
    for Cout, k, pad in ((128, 3, 1), (512, 1, 0)):
        layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=1, pad=pad, act="relu")
        c = synth.conv_case(layer, 1, 7006 + k, oracle, with_x=False)
        y = qnn.qconv2d(x, c["z_x"], dev(c["w"]), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]), c["z_out"], c["act_min"],
                        c["act_max"], bias=dev(c["bias"]))
        assert 2 ** 32 // (H * W * Cin) + 1 < N
        for n in (0, 2 ** 32 // (H * W * Cin) - 1, 2 ** 32 // (H * W * Cin), N - 1):  # around the 4 GiB mark, the first and the last
            rows = slice(100, 104)  # a band of 4 output rows needs input rows 99..104
            xin = host(x[n:n + 1, 99:105]) if k == 3 else host(x[n:n + 1, 100:104])
            want = oracle.qconv2d(xin, c["z_x"], c["w"], c["stride"], (0, c["pad"][1]), c["mult"], c["shift"], c["z_out"],
                                  c["act_min"], c["act_max"], bias=c["bias"])
            assert_same(host(y[n:n + 1, rows]), want, f"qconv2d k={k} image {n} rows 100..103")
        del y


def test_qdwconv2d_with_tensors_beyond_4gib():
    import workloads
    from workloads import synth
    N, H, W, Cc = 140, 256, 256, 512
    g = torch.Generator(device="cuda:0")
    g.manual_seed(7007)
    x = torch.randint(0, 256, (N, H, W, Cc), dtype=torch.uint8, device="cuda:0", generator=g)
    for stride in (1, 2):
        layer = workloads.Layer("t", "dw", H, W, Cc, Cc, k=3, stride=stride, pad=1)
        c = synth.conv_case(layer, 1, 7008 + stride, oracle, with_x=False)
        y = qnn.qdwconv2d(x, c["z_x"], dev(c["w"]), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]), c["z_out"],
                          c["act_min"], c["act_max"], bias=dev(c["bias"]))
        for n in (0, 2 ** 32 // (H * W * Cc) - 1, 2 ** 32 // (H * W * Cc), N - 1):
            # output rows 50..53: input rows 49..54 (stride 1) or 99..107 (stride 2), no vertical padding inside the band
            lo, hi = (49, 55) if stride == 1 else (99, 108)
            want = oracle.qdwconv2d(host(x[n:n + 1, lo:hi]), c["z_x"], c["w"], c["stride"], (0, 1), c["mult"], c["shift"],
                                    c["z_out"], c["act_min"], c["act_max"], bias=c["bias"])
            assert_same(host(y[n:n + 1, 50:54]), want, f"qdwconv2d stride {stride} image {n} rows 50..53")
        del y
