"""Seeded synthetic inputs with the shapes and value distributions of the paper's workloads.

Everything is drawn from numpy's PCG64 with seed = SEED_BASE + 1000*config + layer index.
The quantizer-parameter helpers are injected (`h`): an object with choose_qparams,
quantize_multipliers, act_range, pack_int4, quantize_weights, qadd_params.  The formulas
below only *shape the inputs* (pick scales so that outputs spread over the uint8 range
instead of saturating); they are not part of the method under test.
"""
from __future__ import annotations

import math

import numpy as np

SEED_BASE = 180608342
_SIGMA_U8 = math.sqrt((256 ** 2 - 1) / 12.0)      # std of U{0..255}: 73.9
_SIGMA_W8 = math.sqrt((255 ** 2 - 1) / 12.0)      # std of U{-127..127}: 73.6
_SIGMA_W4 = math.sqrt((15 ** 2 - 1) / 12.0)       # std of U{-7..7}: 4.32


def seed_for(config: int, index: int) -> int:
    return SEED_BASE + 1000 * config + index


def _rng(seed):
    return np.random.Generator(np.random.PCG64(seed))


def _act_kind(act):
    return {"none": 0, "relu": 1, "relu6": 2}[act]


def conv_case(layer, batch, seed, h, in_range=(0.0, 6.0), with_x=True):
    """Inputs of one quantized conv / depthwise layer (configurations 1 and 3-5).

    Activations uniform uint8; weights uniform int8 in [-127,127] (or 4-bit in [-7,7], nibble
    packed); per-channel scale Delta_c chosen so that the real output of channel c has standard
    deviation g_c ~ logU(0.3, 3) (a 10x spread between channels, as batch-norm folding
    produces); real bias g_c * N(1, 0.5); output range [0,6] (ReLU6), [0, U(4,8)] (ReLU) or
    [U(-4,-2), U(2,4)] (linear)."""
    rng = _rng(seed)
    dw = layer.kind == "dw"
    s_x, z_x = h.choose_qparams(*in_range)
    bits = layer.weight_bits
    wmax = 127 if bits == 8 else 7
    if dw:
        w = rng.integers(-wmax, wmax + 1, (layer.k, layer.k, layer.Cout), dtype=np.int8)
    else:
        w = rng.integers(-wmax, wmax + 1, (layer.Cout, layer.k, layer.k, layer.Cin), dtype=np.int8)
    K = layer.K
    sigma_w = _SIGMA_W8 if bits == 8 else _SIGMA_W4
    sigma_x = math.sqrt(_SIGMA_U8 ** 2 + (127.5 - z_x) ** 2)  # rms of (x - z_x)
    g = np.exp(rng.uniform(math.log(0.3), math.log(3.0), layer.Cout))
    delta_c = g / (s_x * sigma_x * sigma_w * math.sqrt(K))
    bias_real = g * rng.normal(1.0, 0.5, layer.Cout)
    bias = np.rint(bias_real / (s_x * delta_c)).astype(np.int64)
    bias = np.clip(bias, -(2 ** 27), 2 ** 27).astype(np.int32)
    if layer.act == "relu6":
        out_range = (0.0, 6.0)
    elif layer.act == "relu":
        out_range = (0.0, float(rng.uniform(4.0, 8.0)))
    else:
        out_range = (float(rng.uniform(-4.0, -2.0)), float(rng.uniform(2.0, 4.0)))
    s_o, z_o = h.choose_qparams(*out_range)
    mult, shift = h.quantize_multipliers(s_x * delta_c / s_o)
    lo, hi = h.act_range(_act_kind(layer.act), s_o, z_o)
    # the activations are drawn last so that with_x=False (device-side generation in the
    # benchmark) leaves every parameter above unchanged
    x = rng.integers(0, 256, (batch, layer.H, layer.W, layer.Cin), dtype=np.uint8) if with_x else None
    case = dict(kind=layer.kind, x=x, z_x=z_x, s_x=s_x, w=w, bias=bias, mult=mult, shift=shift, z_out=z_o, s_out=s_o,
                act_min=lo, act_max=hi, stride=(layer.stride, layer.stride), pad=(layer.pad, layer.pad),
                weight_bits=bits, delta_c=delta_c)
    if bits == 4:
        case["w_packed"] = h.pack_int4(w)
    return case


def single_conv_case(layer, seed, h):
    """Configuration 1 exactly as specified: z_x = 128, s_x = 0.02, fp32 N(0, 0.1) weights quantized
    per channel to int8 (Delta_c = max|w_c| / 127), bias = round(N(0,1) / (s_x Delta_c)),
    s_out = 0.05, z_out = 0, ReLU6 clamp."""
    rng = _rng(seed)
    s_x, z_x, s_o, z_o = 0.02, 128, 0.05, 0
    x = rng.integers(0, 256, (1, layer.H, layer.W, layer.Cin), dtype=np.uint8)
    wf = rng.normal(0.0, 0.1, (layer.Cout, layer.k, layer.k, layer.Cin)).astype(np.float32)
    w, delta_c = h.quantize_weights(wf, 8, True)
    bias = np.rint(rng.normal(0.0, 1.0, layer.Cout) / (s_x * delta_c.astype(np.float64))).astype(np.int32)
    mult, shift = h.quantize_multipliers(s_x * delta_c.astype(np.float64) / s_o)
    lo, hi = h.act_range(2, s_o, z_o)
    return dict(kind="conv", x=x, z_x=z_x, s_x=s_x, w=w, bias=bias, mult=mult, shift=shift, z_out=z_o, s_out=s_o,
                act_min=lo, act_max=hi, stride=(1, 1), pad=(1, 1), weight_bits=8, delta_c=delta_c)


def gemm_case(M, N, K, seed, h, weight_bits=8, with_a=True):
    """Configuration 2: A uniform uint8 with z_a = 128, s_a = 0.02; B from fp32 N(0, 0.05) quantized
    per column symmetric; output scale 8 sigma / 255 with z_out = 128 so results spread over uint8.
    B is returned with each column contiguous ([N, K])."""
    rng = _rng(seed)
    s_a, z_a = 0.02, 128
    if weight_bits == 8:
        # N(0, 0.05) quantized with Delta_c = max|b_c| / 127: drawn in one step as the rounded,
        # clipped normal in code units (the max of K normals is about 3.5-4.3 sigma)
        bf = rng.standard_normal((N, K), dtype=np.float32) * np.float32(0.05)
        Bt, delta_c = h.quantize_weights(bf, 8, True)
        del bf
    else:
        Bt = rng.integers(-7, 8, (N, K), dtype=np.int8)
        delta_c = np.full(N, 0.05 * 3.0 / 7.0, np.float32)
    sigma_y = s_a * _SIGMA_U8 * 0.05 * math.sqrt(K)
    s_o, z_o = 8.0 * sigma_y / 255.0, 128
    mult, shift = h.quantize_multipliers(s_a * delta_c.astype(np.float64) / s_o)
    A = rng.integers(0, 256, (M, K), dtype=np.uint8) if with_a else None
    case = dict(A=A, z_a=z_a, Bt=Bt, mult=mult, shift=shift, z_out=z_o, act_min=0, act_max=255, bias=None,
                weight_bits=weight_bits)
    if weight_bits == 4:
        case["Bt_packed"] = h.pack_int4(Bt)
    return case


def qadd_case(shape, seed, h, act="relu"):
    """Residual add of configuration 4/5: two uniform uint8 tensors with different scales
    (ratio U(0.5, 2)) and zero-points, one output quantizer."""
    rng = _rng(seed)
    a = rng.integers(0, 256, shape, dtype=np.uint8)
    b = rng.integers(0, 256, shape, dtype=np.uint8)
    s_a, z_a = h.choose_qparams(float(rng.uniform(-4.0, -2.0)), float(rng.uniform(2.0, 4.0)))
    s_b = s_a * float(rng.uniform(0.5, 2.0))
    z_b = int(rng.integers(96, 160))
    if act == "relu":
        s_o, z_o = h.choose_qparams(0.0, float(rng.uniform(4.0, 8.0)))
    else:
        s_o, z_o = h.choose_qparams(float(rng.uniform(-6.0, -3.0)), float(rng.uniform(3.0, 6.0)))
    lo, hi = h.act_range(_act_kind(act), s_o, z_o)
    return dict(a=a, z_a=z_a, b=b, z_b=z_b, params=h.qadd_params(s_a, s_b, s_o), z_out=z_o, act_min=lo, act_max=hi)


def quantize_case(shape, seed, h):
    """fp32 N(0,1) tensor with (Delta, z) from its own min / max (configuration 5)."""
    rng = _rng(seed)
    x = rng.standard_normal(shape, dtype=np.float32)
    s, z = h.choose_qparams(float(x.min()), float(x.max()))
    return dict(x=x, scale=s, zero_point=z)
