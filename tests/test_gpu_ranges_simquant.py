"""GPU parity of the data-dependent quantizer (device-side min/max, moving average, dynamic
quantization; Sec. 2.5 + 2.1) and of simulated quantization with its straight-through backward
pass (Sec. 2.4) against the oracle's plain definitions.  fp32 results must agree bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_1806_08342_amd as qnn
import workloads
from workloads import synth

from gpu_util import assert_same, dev, host

pytestmark = pytest.mark.gpu


def _bits(a):
    return np.asarray(a, dtype=np.float32).view(np.uint32)


@pytest.mark.parametrize("n", [0, 1, 3, 1023, 4096, 1_000_003])
@pytest.mark.parametrize("bits", [8, 4])
def test_minmax_and_dynamic_qparams_match_oracle(n, bits):
    rng = np.random.default_rng(6000 + n)
    x = (rng.normal(0.3, 2, n) * rng.choice([1.0, 1.0, 5.0], n)).astype(np.float32)
    if n >= 1023:
        x[:6] = [np.nan, np.inf, -np.inf, -0.0, 1e-40, -1e-41]
    for shift in (0.0, 7.5, -9.0):  # ranges that straddle 0, lie above it, lie below it
        xs = (x + np.float32(shift)).astype(np.float32)
        st = qnn.new_range_state()
        qnn.minmax(dev(xs) if n else torch.empty(0, dtype=torch.float32, device="cuda:0"), st, bits=bits)
        got = qnn.read_range_state(st)
        s, z, lo, hi = oracle.dynamic_qparams(xs, bits=bits)
        assert (_bits(got["xmin"]), _bits(got["xmax"])) == (_bits(lo), _bits(hi)), (got, lo, hi)
        assert (_bits(got["scale"]), got["zero_point"]) == (_bits(s), z), (got, s, z)


def test_minmax_unaligned_and_all_non_finite():
    rng = np.random.default_rng(6100)
    big = rng.normal(0, 1, 10_001).astype(np.float32)
    t = dev(big)
    for off in (1, 2, 3):
        st = qnn.new_range_state()
        qnn.minmax(t[off:], st)
        got = qnn.read_range_state(st)
        lo, hi = oracle.finite_range(big[off:])
        assert (got["xmin"], got["xmax"]) == (float(lo), float(hi))
    st = qnn.new_range_state(3.0, 4.0)
    qnn.minmax(dev(np.array([np.nan, np.inf, -np.inf], np.float32)), st)
    assert qnn.read_range_state(st) == dict(scale=1.0, zero_point=0, xmin=0.0, xmax=0.0)


def test_moving_average_of_the_range_over_batches():
    rng = np.random.default_rng(6200)
    st = qnn.new_range_state(-1.0, 1.0)
    lo, hi = np.float32(-1.0), np.float32(1.0)
    for step in range(6):
        x = (rng.normal(0, 1 + step, 50_000)).astype(np.float32)
        qnn.minmax(dev(x), st, momentum=0.9)
        s, z, lo, hi = oracle.dynamic_qparams(x, state=(lo, hi), momentum=0.9)
        got = qnn.read_range_state(st)
        assert (_bits(got["xmin"]), _bits(got["xmax"])) == (_bits(lo), _bits(hi)), f"step {step}"
        assert (_bits(got["scale"]), got["zero_point"]) == (_bits(s), z), f"step {step}"


@pytest.mark.parametrize("n", [1, 4097, 777_777])
def test_quantize_dynamic_matches_oracle(n):
    c = synth.quantize_case((n,), workloads.seed_for(5, 950 + n % 7), oracle)
    x = c["x"] * np.float32(1.7) + np.float32(0.4)
    st = qnn.new_range_state()
    q = host(qnn.quantize_dynamic(dev(x), st))
    s, z, lo, hi = oracle.dynamic_qparams(x)
    assert_same(q, oracle.quantize(x, s, z), f"quantize_dynamic n={n}")
    got = qnn.read_range_state(st)
    assert (_bits(got["scale"]), got["zero_point"]) == (_bits(s), z)
    if n > 1000:
        assert q.min() == 0 and q.max() == 255  # the range of the tensor itself uses every code
    # the same state drives a later tensor (inference with a frozen range)
    x2 = (x[::-1] * np.float32(1.3)).astype(np.float32).copy()
    assert_same(host(qnn.quantize_with(dev(x2), st)), oracle.quantize(x2, s, z), "quantize_with")


@pytest.mark.parametrize("n", [1, 5, 4096, 300_001])
def test_simquant_forward_and_backward_match_oracle(n):
    rng = np.random.default_rng(6300 + n)
    x = rng.normal(0, 2, n).astype(np.float32)
    g = rng.normal(0, 1, n).astype(np.float32)
    if n >= 4096:
        x[:5] = [np.nan, np.inf, -np.inf, 1e30, -0.0]
    for scale, z, qmin, qmax in [(0.0213, 131, 0, 255), (2.0 ** -5, 102, 0, 255), (0.25, 8, 0, 15), (1 / 3, 0, 0, 255),
                                 (0.05, 255, 0, 255), (2.0 ** -14, 30000, 0, 65535), (1.7e-4, 21845, 0, 65535),
                                 (0.003, 2048, 0, 4095), (1e-3, 65535, 0, 65535)]:
        y = host(qnn.simquant(dev(x), scale, z, qmin, qmax))
        assert np.array_equal(_bits(y), _bits(oracle.simquant(x, scale, z, qmin, qmax))), (scale, z)
        gx = host(qnn.simquant_backward(dev(x), dev(g), scale, z, qmin, qmax))
        assert np.array_equal(_bits(gx), _bits(oracle.simquant_backward(x, g, scale, z, qmin, qmax))), (scale, z)
    # ends of the range are inside it (closed interval of eq. 15)
    ends = oracle.dequantize(np.array([0, 255], np.uint8), 2.0 ** -5, 102)
    gx = host(qnn.simquant_backward(dev(ends), dev(np.ones(2, np.float32)), 2.0 ** -5, 102))
    assert gx.tolist() == [1.0, 1.0]


@pytest.mark.parametrize("n,offset", [(0, 0), (1, 0), (5, 1), (4099, 0), (4099, 3), (1_000_003, 0)])
def test_quantize_and_dequantize_with_16_bit_codes_match_oracle(n, offset):
    """Sec. 3.3 activation precision of 16 bits: uint16 codes.  `offset` shifts both pointers off their
    vector alignment (the one-element-per-lane form of the kernels)."""
    import torch
    rng = np.random.default_rng(9100 + n + offset)
    x = rng.normal(0, 2, n + offset).astype(np.float32)
    if n >= 4096:
        x[offset:offset + 6] = [np.nan, np.inf, -np.inf, 1e30, -0.0, 1e-45]
    xd = dev(x)[offset:]
    x = x[offset:]
    for scale, z, qmin, qmax in [(2.0 ** -14, 30000, 0, 65535), (1.7e-4, 21845, 0, 65535), (0.003, 2048, 0, 4095),
                                 (0.0213, 131, 0, 255), (1e-3, 0, 0, 65535)]:
        qbuf = torch.zeros(n + offset, dtype=torch.uint16, device="cuda:0")[offset:]
        q = qnn.quantize_u16(xd, scale, z, qmin, qmax, out=qbuf)
        want = oracle.quantize_wide(x, scale, z, qmin, qmax)
        got = q.cpu().view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(got, want), (scale, z)
        back = host(qnn.dequantize_u16(q, scale, z))
        assert np.array_equal(_bits(back), _bits(oracle.dequantize_wide(want, scale, z))), (scale, z)
        if n:
            y = host(qnn.simquant(xd.contiguous(), scale, z, qmin, qmax))
            assert np.array_equal(_bits(y), _bits(back))  # SimQuant == de-quantize(quantize)


# ------------------------------------------------------------ rescale of uint8 codes (concat)

@pytest.mark.parametrize("rows,cols", [(1, 1), (7, 5), (100, 64), (333, 48), (4096, 130)])
def test_rescale_u8_matches_oracle_requantize(rows, cols):
    # the oracle side is its pinned requantize applied to (x - z_in): no arithmetic of its own
    rng = np.random.default_rng(6400 + rows + cols)
    x = rng.integers(0, 256, (rows, cols)).astype(np.uint8)
    for s_in, s_out, z_in, z_out, lo, hi in [(0.02, 0.05, 128, 100, 0, 255), (0.07, 0.03, 3, 0, 0, 255), (0.01, 0.01, 255, 255, 0, 255),
                                              (0.5, 0.001, 17, 128, 5, 250), (1e-3, 1.0, 200, 7, 0, 255)]:
        mult, shift = oracle.quantize_multiplier(s_in / s_out)
        want = oracle.requantize(x.astype(np.int32) - z_in, np.array([mult]), np.array([shift]), False, z_out, lo, hi)
        got = host(qnn.rescale_u8(dev(x), z_in, mult, shift, z_out, lo, hi))
        assert_same(got, want, f"rescale_u8 {rows}x{cols} s_in={s_in} s_out={s_out}")


def test_rescale_u8_writes_a_channel_slice_of_a_concatenation():
    rng = np.random.default_rng(6500)
    rows, c1, c2 = 500, 48, 80
    a = rng.integers(0, 256, (rows, c1)).astype(np.uint8)
    b = rng.integers(0, 256, (rows, c2)).astype(np.uint8)
    out = torch.full((rows, c1 + c2), 9, dtype=torch.uint8, device="cuda:0")
    want = np.empty((rows, c1 + c2), np.uint8)
    for src, z_in, s_in, off in [(a, 120, 0.031, 0), (b, 7, 0.012, c1)]:
        mult, shift = oracle.quantize_multiplier(s_in / 0.02)
        qnn.rescale_u8(dev(src), z_in, mult, shift, 64, 0, 255, out=out[:, off:off + src.shape[1]])
        want[:, off:off + src.shape[1]] = oracle.requantize(src.astype(np.int32) - z_in, np.array([mult]), np.array([shift]), False,
                                                           64, 0, 255)
    assert_same(host(out), want, "concat of two rescaled inputs")
    # a source that is itself a slice (odd byte offset: byte path)
    wide = rng.integers(0, 256, (rows, 100)).astype(np.uint8)
    mult, shift = oracle.quantize_multiplier(1.7)
    got = host(qnn.rescale_u8(dev(wide)[:, 3:70], 50, mult, shift, 60, 0, 255))
    assert_same(got, oracle.requantize(wide[:, 3:70].astype(np.int32) - 50, np.array([mult]), np.array([shift]), False, 60, 0, 255),
                "rescale_u8 from a slice")
