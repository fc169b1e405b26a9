"""ctypes front-end of the CPU oracle (``qnn_oracle.c``).

TEST INFRASTRUCTURE.  Only the tests, the smoke check and the ``cpu_baseline`` leg of
the benchmark may import this package; the GPU library never does, and this package
imports nothing from the GPU library.  Arrays are numpy, on the host.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "qnn_oracle.c")
_LIB = os.path.join(_HERE, "libqnn_oracle.so")

OK, EINVAL, EOVERFLOW = 0, 1, 4


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP over independent outputs)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        )
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.oracle_rescale.restype = C.c_int32
        _lib.oracle_rescale.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    return _lib


class OracleError(RuntimeError):
    def __init__(self, code):
        super().__init__(f"oracle returned status {code}")
        self.code = code


def _check(rc):
    if rc != OK:
        raise OracleError(rc)


def _p(a, dtype):
    if a is None:
        return None
    assert isinstance(a, np.ndarray) and a.dtype == dtype and a.flags["C_CONTIGUOUS"], (a.dtype, dtype)
    return a.ctypes.data_as(C.c_void_p)


def _i32(a):
    return None if a is None else np.ascontiguousarray(a, dtype=np.int32)


def num_threads() -> int:
    """Threads the OpenMP loops of the oracle use in this process."""
    env = os.environ.get("OMP_NUM_THREADS")
    if env:
        try:
            return max(1, int(env.split(",")[0]))
        except ValueError:
            pass
    return len(os.sched_getaffinity(0))


# ---------------------------------------------------------------- parameters

def choose_qparams(xmin, xmax, bits=8):
    s, z = C.c_float(), C.c_int32()
    _check(lib().oracle_choose_qparams(C.c_double(xmin), C.c_double(xmax), int(bits), C.byref(s), C.byref(z)))
    return float(s.value), int(z.value)


def act_range(kind, s_out, z_out):
    lo, hi = C.c_int32(), C.c_int32()
    _check(lib().oracle_act_range(int(kind), C.c_float(s_out), int(z_out), C.byref(lo), C.byref(hi)))
    return int(lo.value), int(hi.value)


def quantize_multiplier(real_mult):
    m, s = C.c_int32(), C.c_int32()
    _check(lib().oracle_quantize_multiplier(C.c_double(real_mult), C.byref(m), C.byref(s)))
    return int(m.value), int(s.value)


def quantize_multipliers(real_mults):
    out = [quantize_multiplier(float(v)) for v in np.asarray(real_mults, dtype=np.float64).ravel()]
    return (np.array([o[0] for o in out], dtype=np.int32), np.array([o[1] for o in out], dtype=np.int32))


def rescale(a, mult, shift):
    return int(lib().oracle_rescale(int(a), int(mult), int(shift)))


def qadd_params(s_a, s_b, s_out):
    v = [C.c_int32() for _ in range(7)]
    _check(lib().oracle_qadd_params(C.c_double(s_a), C.c_double(s_b), C.c_double(s_out), *[C.byref(t) for t in v]))
    names = ["left_shift", "mult_a", "shift_a", "mult_b", "shift_b", "mult_o", "shift_o"]
    return {k: int(t.value) for k, t in zip(names, v)}


# ------------------------------------------------------- quantize / dequantize

def quantize(x, scale, zero_point, qmin=0, qmax=255):
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, dtype=np.uint8)
    _check(lib().oracle_quantize(_p(x, np.float32), _p(q, np.uint8), C.c_size_t(x.size), C.c_float(scale),
                                 int(zero_point), int(qmin), int(qmax)))
    return q


def dequantize(q, scale, zero_point):
    q = np.ascontiguousarray(q, dtype=np.uint8)
    x = np.empty(q.shape, dtype=np.float32)
    _check(lib().oracle_dequantize(_p(q, np.uint8), _p(x, np.float32), C.c_size_t(q.size), C.c_float(scale),
                                   int(zero_point)))
    return x


def quantize_wide(x, scale, zero_point, qmin=0, qmax=65535):
    """eq. 1-2 with codes of up to 16 bits (uint16 result)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, dtype=np.uint16)
    _check(lib().oracle_quantize_wide(_p(x, np.float32), _p(q, np.uint16), C.c_size_t(x.size), C.c_float(scale),
                                      int(zero_point), int(qmin), int(qmax)))
    return q


def dequantize_wide(q, scale, zero_point):
    """eq. 3 for uint16 codes."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    x = np.empty(q.shape, dtype=np.float32)
    _check(lib().oracle_dequantize_wide(_p(q, np.uint16), _p(x, np.float32), C.c_size_t(q.size), C.c_float(scale),
                                        int(zero_point)))
    return x


def quantize_weights(w, bits=8, restricted=True):
    """w: [channels, ...] fp32 -> (int8 array of the same shape, Delta_c[channels])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    ch = w.shape[0]
    per = w.size // ch
    wq = np.empty(w.shape, dtype=np.int8)
    d = np.empty(ch, dtype=np.float32)
    _check(lib().oracle_quantize_weights(_p(w, np.float32), C.c_size_t(ch), C.c_size_t(per), int(bits),
                                         int(bool(restricted)), _p(wq, np.int8), _p(d, np.float32)))
    return wq, d


def pack_int4(v):
    v = np.ascontiguousarray(v, dtype=np.int8)
    assert v.shape[-1] % 2 == 0
    out = np.empty(v.shape[:-1] + (v.shape[-1] // 2,), dtype=np.uint8)
    _check(lib().oracle_pack_int4(_p(v, np.int8), C.c_size_t(v.size), _p(out, np.uint8)))
    return out


def unpack_int4(packed):
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    out = np.empty(packed.shape[:-1] + (packed.shape[-1] * 2,), dtype=np.int8)
    _check(lib().oracle_unpack_int4(_p(packed, np.uint8), C.c_size_t(out.size), _p(out, np.int8)))
    return out


# ------------------------------------------------------------- integer layers

def requantize(acc, mult, shift, per_channel, z_out, act_min, act_max):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    rows, ch = acc.shape
    mult, shift = _i32(mult), _i32(shift)
    y = np.empty((rows, ch), dtype=np.uint8)
    _check(lib().oracle_requantize(_p(acc, np.int32), _p(y, np.uint8), C.c_size_t(rows), C.c_size_t(ch),
                                   _p(mult, np.int32), _p(shift, np.int32), int(bool(per_channel)), int(z_out),
                                   int(act_min), int(act_max)))
    return y


def qgemm(A, z_a, Bt, mult, shift, z_out, act_min, act_max, bias=None, weight_bits=8, z_w=None, K=None,
          allow_overflow=False):
    """A: uint8 [M,K].  Bt: the weights with each output column contiguous -- int8 [N,K], or
    uint8 [N,K/2] nibble-packed when weight_bits == 4."""
    A = np.ascontiguousarray(A, dtype=np.uint8)
    M, Ka = A.shape
    K = Ka if K is None else K
    if weight_bits == 8:
        Bt = np.ascontiguousarray(Bt, dtype=np.int8)
        N, ldb = Bt.shape
        bp = _p(Bt, np.int8)
    else:
        Bt = np.ascontiguousarray(Bt, dtype=np.uint8)
        N, ldb = Bt.shape[0], Bt.shape[1] * 2
        bp = _p(Bt, np.uint8)
    mult, shift, bias, z_w = _i32(mult), _i32(shift), _i32(bias), _i32(z_w)
    Cm = np.empty((M, N), dtype=np.uint8)
    rc = lib().oracle_qgemm(_p(A, np.uint8), C.c_int64(Ka), int(z_a), bp, C.c_int64(ldb), int(weight_bits),
                            _p(z_w, np.int32), C.c_int64(M), C.c_int64(N), C.c_int64(K), _p(bias, np.int32),
                            _p(mult, np.int32), _p(shift, np.int32), int(z_out), int(act_min), int(act_max),
                            _p(Cm, np.uint8), C.c_int64(N))
    if not (allow_overflow and rc == EOVERFLOW):
        _check(rc)
    return Cm


def _conv_out_hw(H, W, kh, kw, stride, pad):
    sh, sw = stride
    ph, pw = pad
    return (H + 2 * ph - kh) // sh + 1, (W + 2 * pw - kw) // sw + 1


def qconv2d(x, z_x, w, stride, pad, mult, shift, z_out, act_min, act_max, bias=None, weight_bits=8, z_w=None,
            sample=None):
    """x: uint8 NHWC.  w: int8 [Cout,kh,kw,Cin] (or uint8 [Cout,kh,kw,Cin/2] packed 4-bit).
    Returns uint8 NHWC output, or the 1-D values at the flat output indices in `sample`."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    N, H, W, Cin = x.shape
    if weight_bits == 8:
        w = np.ascontiguousarray(w, dtype=np.int8)
        wp = _p(w, np.int8)
        assert w.shape[3] == Cin
    else:
        w = np.ascontiguousarray(w, dtype=np.uint8)
        wp = _p(w, np.uint8)
        assert w.shape[3] * 2 == Cin
    Cout, kh, kw = w.shape[:3]
    Ho, Wo = _conv_out_hw(H, W, kh, kw, stride, pad)
    mult, shift, bias, z_w = _i32(mult), _i32(shift), _i32(bias), _i32(z_w)
    if sample is None:
        y = np.empty((N, Ho, Wo, Cout), dtype=np.uint8)
        sp, ns = None, 0
    else:
        sample = np.ascontiguousarray(sample, dtype=np.int64)
        y = np.empty(sample.shape, dtype=np.uint8)
        sp, ns = _p(sample, np.int64), sample.size
    _check(lib().oracle_qconv2d(_p(x, np.uint8), N, H, W, Cin, int(z_x), wp, Cout, kh, kw, int(weight_bits),
                                _p(z_w, np.int32), stride[0], stride[1], pad[0], pad[1], _p(bias, np.int32),
                                _p(mult, np.int32), _p(shift, np.int32), int(z_out), int(act_min), int(act_max),
                                _p(y, np.uint8), sp, C.c_int64(ns)))
    return y


def qconv2d_acc(x, z_x, w, stride, pad, weight_bits=8, z_w=None):
    """int64 accumulators sum (x - z_x)(w - z_w) of the convolution, no bias, no rescale."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    N, H, W, Cin = x.shape
    if weight_bits == 8:
        w = np.ascontiguousarray(w, dtype=np.int8)
        wp = _p(w, np.int8)
    else:
        w = np.ascontiguousarray(w, dtype=np.uint8)
        wp = _p(w, np.uint8)
    Cout, kh, kw = w.shape[:3]
    Ho, Wo = _conv_out_hw(H, W, kh, kw, stride, pad)
    z_w = _i32(z_w)
    acc = np.empty((N, Ho, Wo, Cout), dtype=np.int64)
    _check(lib().oracle_qconv2d_acc(_p(x, np.uint8), N, H, W, Cin, int(z_x), wp, Cout, kh, kw, int(weight_bits),
                                    _p(z_w, np.int32), stride[0], stride[1], pad[0], pad[1], _p(acc, np.int64)))
    return acc


def qdwconv2d(x, z_x, w, stride, pad, mult, shift, z_out, act_min, act_max, bias=None, z_w=None, sample=None):
    """x: uint8 NHWC.  w: int8 [kh,kw,C]."""
    x = np.ascontiguousarray(x, dtype=np.uint8)
    N, H, W, Cc = x.shape
    w = np.ascontiguousarray(w, dtype=np.int8)
    kh, kw, Cw = w.shape
    assert Cw == Cc
    Ho, Wo = _conv_out_hw(H, W, kh, kw, stride, pad)
    mult, shift, bias, z_w = _i32(mult), _i32(shift), _i32(bias), _i32(z_w)
    if sample is None:
        y = np.empty((N, Ho, Wo, Cc), dtype=np.uint8)
        sp, ns = None, 0
    else:
        sample = np.ascontiguousarray(sample, dtype=np.int64)
        y = np.empty(sample.shape, dtype=np.uint8)
        sp, ns = _p(sample, np.int64), sample.size
    _check(lib().oracle_qdwconv2d(_p(x, np.uint8), N, H, W, Cc, int(z_x), _p(w, np.int8), kh, kw, _p(z_w, np.int32),
                                  stride[0], stride[1], pad[0], pad[1], _p(bias, np.int32), _p(mult, np.int32),
                                  _p(shift, np.int32), int(z_out), int(act_min), int(act_max), _p(y, np.uint8), sp,
                                  C.c_int64(ns)))
    return y


def qadd(a, z_a, b, z_b, params, z_out, act_min, act_max):
    a = np.ascontiguousarray(a, dtype=np.uint8)
    b = np.ascontiguousarray(b, dtype=np.uint8)
    assert a.shape == b.shape
    y = np.empty(a.shape, dtype=np.uint8)
    p = params
    _check(lib().oracle_qadd(_p(a, np.uint8), int(z_a), p["mult_a"], p["shift_a"], _p(b, np.uint8), int(z_b),
                             p["mult_b"], p["shift_b"], p["left_shift"], p["mult_o"], p["shift_o"], int(z_out),
                             int(act_min), int(act_max), _p(y, np.uint8), C.c_size_t(a.size)))
    return y


# ------------------------------------------------ ranges from the data, simulated quantization
# Plain definitions written out with numpy and the pinned functions above (no new C code).

def finite_range(x):
    """(min, max) over the finite elements of x as binary32 (Sec. 2.5: the range of an activation tensor
    is its minimum and maximum); (0, 0) when there is none."""
    x = np.asarray(x, dtype=np.float32).reshape(-1)
    x = x[np.isfinite(x)]
    if x.size == 0:
        return np.float32(0.0), np.float32(0.0)
    return np.float32(x.min()), np.float32(x.max())


def moving_average(old, new, momentum):
    """momentum * old + (1 - momentum) * new (Sec. 2.5: moving average of the range across batches):
    the two products and the sum each rounded once in binary64, the result rounded to binary32."""
    m = np.float64(np.float32(momentum))
    return np.float32(m * np.float64(np.float32(old)) + (np.float64(1.0) - m) * np.float64(np.float32(new)))


def dynamic_qparams(x, bits=8, state=None, momentum=0.0):
    """(scale, zero_point, xmin, xmax) of the quantizer of x's own range, or of the moving average that
    starts from state = (xmin, xmax)."""
    lo, hi = finite_range(x)
    if momentum != 0.0:
        lo, hi = moving_average(state[0], lo, momentum), moving_average(state[1], hi, momentum)
    s, z = choose_qparams(float(lo), float(hi), bits)
    return s, z, lo, hi


def simquant(x, scale, zero_point, qmin=0, qmax=255):
    """Sec. 2.4 eq. 12-13: a quantizer followed by a de-quantizer (codes of up to 16 bits)."""
    if qmax > 255:
        return dequantize_wide(quantize_wide(x, scale, zero_point, qmin, qmax), scale, zero_point)
    return dequantize(quantize(x, scale, zero_point, qmin, qmax), scale, zero_point)


def simquant_backward(x, grad_y, scale, zero_point, qmin=0, qmax=255):
    """Sec. 2.4 eq. 14-15 (straight-through estimator): the gradient passes where x lies inside the
    representable range [x_min, x_max] = de-quantized extreme codes, and is zero elsewhere."""
    x = np.asarray(x, dtype=np.float32)
    if qmax > 255:
        ends = dequantize_wide(np.array([qmin, qmax], dtype=np.uint16), scale, zero_point)
    else:
        ends = dequantize(np.array([qmin, qmax], dtype=np.uint8), scale, zero_point)
    inside = (x >= ends[0]) & (x <= ends[1])
    return np.where(inside, np.asarray(grad_y, dtype=np.float32), np.float32(0.0)).astype(np.float32)
