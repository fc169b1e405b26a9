"""GPU parity of the add fused behind a product (qnn_qgemm_add / qnn_qconv2d_add): the expected
value is the oracle's layer followed by the oracle's rescaling add -- no arithmetic of its own.
Every route of the dispatcher is forced once: kernels that apply the add on the way out of their
LDS tile (short-K, pipelined and staged tiles) and kernels followed by the in-place second pass."""
import numpy as np
import pytest
import torch

import oracle
import paper_1806_08342_amd as qnn
import workloads
from workloads import synth

from gpu_util import assert_same, dev, host

pytestmark = pytest.mark.gpu


def _add_setup(rng, shape, act="relu", odd=False):
    """Residual tensor + add parameters; `odd` picks scales that leave the fused 32-bit form."""
    R = rng.integers(0, 256, shape).astype(np.uint8)
    z_mid = int(rng.integers(90, 170))
    z_r = int(rng.integers(0, 256))
    if odd:
        s_mid, s_r, s_o = 0.03, 0.041, 0.3  # shift_o = 22: beyond the fused 32-bit form, the general output rescale
    else:
        s_mid = float(rng.uniform(0.02, 0.05))
        s_r = s_mid * float(rng.uniform(0.5, 2.0))
        s_o = float(rng.uniform(0.03, 0.08))
    z_o = 0 if act == "relu" else int(rng.integers(100, 150))
    lo, hi = (z_o, 255) if act == "relu" else (0, 255)
    return R, z_mid, z_r, oracle.qadd_params(s_mid, s_r, s_o), z_o, lo, hi


def _gemm_inputs(rng, M, N, K, bits=8):
    A = rng.integers(0, 256, (M, K)).astype(np.uint8)
    lim = 8 if bits == 4 else 128
    Bt = rng.integers(-lim, lim, (N, K)).astype(np.int8)
    real = 10 ** rng.uniform(-4.2, -3.2, N) / np.sqrt(K / 64.0) * (16.0 if bits == 4 else 1.0)
    mult, shift = oracle.quantize_multipliers(real)
    bias = rng.integers(-20000, 20000, N).astype(np.int32)
    return A, Bt, bias, mult, shift


def _check_gemm_add(M, N, K, seed, what, bits=8, odd=False, act="relu", mid=(0, 255), z_a=None):
    rng = np.random.default_rng(seed)
    A, Bt, bias, mult, shift = _gemm_inputs(rng, M, N, K, bits)
    R, z_mid, z_r, p, z_o, lo, hi = _add_setup(rng, (M, N), act, odd)
    z_a = int(rng.integers(0, 256)) if z_a is None else z_a
    Bo = oracle.pack_int4(Bt) if bits == 4 else Bt
    t = oracle.qgemm(A, z_a, Bo, mult, shift, z_mid, mid[0], mid[1], bias=bias, weight_bits=bits)
    want = oracle.qadd(t, z_mid, R, z_r, p, z_o, lo, hi)
    got = host(qnn.qgemm_add(dev(A), z_a, dev(Bo), dev(mult), dev(shift), z_mid, mid[0], mid[1], dev(R), z_r, p, z_o, lo, hi,
                             bias=dev(bias), weight_bits=bits))
    assert_same(got, want, what)
    assert len(np.unique(want)) > 8, "parity would be vacuous"
    return A, Bo, bias, mult, shift, R, z_a, z_mid, z_r, p, z_o, lo, hi, want


@pytest.mark.parametrize("M,N,K", [(300, 130, 64), (1000, 256, 128), (4099, 512, 256), (97, 48, 32), (2048, 64, 96),
                                   (500, 200, 72)])  # K = 72: no 16-byte rows, the add runs as a second pass
@pytest.mark.parametrize("bits", [8, 4])
def test_qgemm_add_short_k(M, N, K, bits):
    assert qnn.qgemm_plan(M, N, K) == "shortk"
    _check_gemm_add(M, N, K, 4000 + M + N + K + bits, f"qgemm_add short-K {M}x{N}x{K} bits={bits}", bits=bits)
    _check_gemm_add(M, N, K, 4100 + M + N + K + bits, f"qgemm_add short-K {M}x{N}x{K} bits={bits}, general add rescale",
                    bits=bits, odd=True, act="none")


@pytest.mark.parametrize("M,N,K,bits", [(70001, 256, 64, 8), (33000, 512, 160, 4)])
def test_qgemm_add_pair_table(M, N, K, bits):
    # from 2^24 outputs on, the short-K kernel combines the two codes through a 65536-entry table
    assert M * N >= 2 ** 24 and qnn.qgemm_plan(M, N, K) == "shortk"
    _check_gemm_add(M, N, K, 4150 + K, f"qgemm_add pair table {M}x{N}x{K} bits={bits}", bits=bits, mid=(2, 251))
    _check_gemm_add(M, N, K, 4160 + K, f"qgemm_add pair table {M}x{N}x{K} bits={bits}, general add rescale", bits=bits, odd=True,
                    act="none")


@pytest.mark.parametrize("alds", [1, 0])
@pytest.mark.parametrize("M,N,K,bits", [(1000, 512, 128, 8), (4099, 520, 256, 8), (133, 1030, 128, 4), (2500, 256, 256, 4),
                                         (16400, 1024, 256, 8),   # 2^24 outputs: 8-wave workgroups with the table of code pairs
                                         (33000, 1024, 128, 4)])
def test_qgemm_add_short_k_rows_through_lds(tuning, alds, M, N, K, bits):
    # K = 128 / 256 with at least one workgroup's worth of column groups: without an add these shapes stage the A
    # rows in LDS once per workgroup; with the add built in they keep the direct loads whatever the switch says,
    # and as a second pass behind the staged kernel when the operands are not made of whole aligned chunks
    tuning.setenv("QNN_SHORTK_ALDS", str(alds))
    assert qnn.qgemm_plan(M, N, K) == "shortk"
    _check_gemm_add(M, N, K, 4300 + M + N + K + bits, f"qgemm_add short-K through LDS={alds} {M}x{N}x{K} bits={bits}", bits=bits)
    _check_gemm_add(M, N, K, 4400 + M + N + K + bits, f"qgemm_add short-K through LDS={alds} {M}x{N}x{K} bits={bits}, general add rescale",
                    bits=bits, odd=True, act="none")


@pytest.mark.parametrize("tile", ["dma128x128", "dma256x256", "dma256x64", "dma256x128", "dma128x128s3", "dma64x64",
                                  "dma256x64s3", "128x128", "64x64"])
@pytest.mark.parametrize("M,N,K", [(300, 270, 512), (513, 130, 320)])
def test_qgemm_add_every_tile(tuning, tile, M, N, K):
    tuning.setenv("QNN_FORCE_TILE", tile)
    _check_gemm_add(M, N, K, 4200 + M + K, f"qgemm_add tile={tile} {M}x{N}x{K}", mid=(3, 250))
    _check_gemm_add(M, N, K, 4300 + M + K, f"qgemm_add tile={tile} {M}x{N}x{K}, general add rescale", odd=True, act="none")


def test_qgemm_add_default_routes():
    # tiles chosen by the cost model, split-K, few rows, 4-bit weights through the unpack pass
    for (M, N, K, bits) in [(2048, 2048, 512, 8), (256, 512, 8192, 8), (16, 256, 512, 8), (64, 4096, 1024, 8),
                            (1500, 384, 1024, 4), (12544, 2048, 512, 8)]:
        _check_gemm_add(M, N, K, 4400 + M + N, f"qgemm_add {M}x{N}x{K} bits={bits} plan={qnn.qgemm_plan(M, N, K)}", bits=bits)


def test_qgemm_add_weight_resident(tuning):
    tuning.setenv("QNN_BRES", "1")
    _check_gemm_add(4500, 64, 512, 4500, "qgemm_add weight-resident kernel + second pass")


def test_qgemm_add_spaced_rows_and_unaligned_residual():
    # output and residual are column slices of wider matrices; the residual starts at an odd byte
    rng = np.random.default_rng(4600)
    M, N, K = 700, 96, 128
    A, Bt, bias, mult, shift = _gemm_inputs(rng, M, N, K)
    Rw, z_mid, z_r, p, z_o, lo, hi = _add_setup(rng, (M, N + 37))
    R = Rw[:, 5:5 + N]
    t = oracle.qgemm(A, 77, Bt, mult, shift, z_mid, 0, 255, bias=bias)
    want = oracle.qadd(t, z_mid, np.ascontiguousarray(R), z_r, p, z_o, lo, hi)
    Cw = torch.zeros((M, N + 16), dtype=torch.uint8, device="cuda:0")
    for r_dev, what in [(dev(Rw)[:, 5:5 + N], "odd offset"), (dev(np.ascontiguousarray(R)), "dense")]:
        out = Cw[:, 16:]
        qnn.qgemm_add(dev(A), 77, dev(Bt), dev(mult), dev(shift), z_mid, 0, 255, r_dev, z_r, p, z_o, lo, hi, bias=dev(bias),
                      out=out)
        assert_same(host(out.contiguous()), want, f"qgemm_add spaced rows, residual {what}")
    assert int(Cw[:, :16].max()) == 0


CONV_ADD_SHAPES = [
    # H, W, Cin, Cout, k, stride, pad, bits
    (14, 14, 64, 256, 1, 1, 0, 8),     # last 1x1 of a bottleneck: short-K
    (14, 14, 512, 2048, 1, 1, 0, 8),   # K = 512: tiles
    (28, 28, 64, 96, 1, 2, 0, 8),      # strided 1x1
    (12, 12, 32, 64, 3, 1, 1, 8),      # 3x3 convolution through the tile kernel
    (14, 14, 96, 24, 1, 1, 0, 4),      # MobileNetV2-style linear bottleneck, 4-bit weights
    (20, 20, 3, 32, 3, 2, 1, 8),       # stem kernel + second pass
    (9, 9, 20, 30, 3, 1, 1, 8),        # nothing aligned
]


@pytest.mark.parametrize("shape", CONV_ADD_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("batch", [1, 5])
def test_qconv2d_add_matches_oracle(shape, batch):
    H, W, Cin, Cout, k, s, p_, bits = shape
    layer = workloads.Layer("t", "conv", H, W, Cin, Cout, k=k, stride=s, pad=p_, act="none", weight_bits=bits)
    c = synth.conv_case(layer, batch, 4700 + sum(shape) + batch, oracle)
    w_o = c.get("w_packed", c["w"])
    t = oracle.qconv2d(c["x"], c["z_x"], w_o, c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"], c["act_min"],
                       c["act_max"], bias=c["bias"], weight_bits=bits)
    rng = np.random.default_rng(4800 + sum(shape))
    R, _, z_r, p, z_o, lo, hi = _add_setup(rng, t.shape)
    want = oracle.qadd(t, c["z_out"], R, z_r, p, z_o, lo, hi)
    got = host(qnn.qconv2d_add(dev(c["x"]), c["z_x"], dev(w_o), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]),
                               c["z_out"], c["act_min"], c["act_max"], dev(R), z_r, p, z_o, lo, hi, bias=dev(c["bias"]),
                               weight_bits=bits))
    assert_same(got, want, f"qconv2d_add {shape} batch {batch}")
    assert len(np.unique(want)) > 8


def test_fused_add_equals_two_calls_on_the_gpu():
    # the documented identity, checked on the device side as well: layer into a temporary, then qnn_qadd
    A, Bo, bias, mult, shift, R, z_a, z_mid, z_r, p, z_o, lo, hi, want = _check_gemm_add(900, 256, 64, 4900, "identity case")
    t = qnn.qgemm(dev(A), z_a, dev(Bo), dev(mult), dev(shift), z_mid, 0, 255, bias=dev(bias))
    two = host(qnn.qadd(t, z_mid, dev(R), z_r, p, z_o, lo, hi))
    assert_same(two, want, "qgemm then qadd")
