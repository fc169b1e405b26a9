"""ctypes binding of libqnn.so: argument marshalling only.

Device tensors are torch tensors on a HIP device; the functions pass their ``data_ptr()`` and
the current torch stream to the C ABI (``include/qnn.h``) and allocate the output tensor.
No arithmetic of the method happens in Python.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libqnn.so")
_lib = None

STATUS = {0: "QNN_OK", 1: "QNN_EINVAL", 2: "QNN_EUNSUPPORTED", 3: "QNN_ELAUNCH"}
B_COLUMNS_CONTIGUOUS, B_ROWS_CONTIGUOUS = 0, 1

EXPORTS = [
    "qnn_last_error", "qnn_version", "qnn_qgemm_plan", "qnn_quantize", "qnn_dequantize", "qnn_requantize", "qnn_qgemm", "qnn_pack_b",
    "qnn_qconv2d", "qnn_qdwconv2d", "qnn_qadd", "qnn_qgemm_add", "qnn_qconv2d_add", "qnn_rescale_u8", "qnn_qgemm_asym", "qnn_qconv2d_asym", "qnn_qdwconv2d_asym", "qnn_minmax", "qnn_quantize_with",
    "qnn_quantize_dynamic", "qnn_simquant", "qnn_simquant_backward", "qnn_choose_qparams", "qnn_quantize_multiplier", "qnn_act_range",
    "qnn_qadd_params", "qnn_quantize_weights", "qnn_pack_int4", "qnn_qgemm_workspace_bytes", "qnn_qconv2d_workspace_bytes",
    "qnn_tuning_set", "qnn_calibrate_mfma", "qnn_calibrate_copy", "qnn_qgemm_noalloc", "qnn_quantize_u16", "qnn_dequantize_u16", "qnn_calibrate_rescale",
]


class QnnError(RuntimeError):
    def __init__(self, name, code, detail=""):
        super().__init__(f"{name} failed with {STATUS.get(code, code)}{(': ' + detail) if detail else ''}")
        self.code = code


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libqnn.so.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it first (python -m paper_1806_08342_amd._build, or "
            "__graft_entry__.build()); there is no CPU fallback")
    lib = C.CDLL(_LIB_PATH)
    lib.qnn_last_error.restype = C.c_char_p
    lib.qnn_version.restype = C.c_char_p
    lib.qnn_qgemm_plan.restype = C.c_char_p
    lib.qnn_qgemm_plan.argtypes = [C.c_int64, C.c_int64, C.c_int64]
    vp, i32, i64, sz, f32, f64 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float, C.c_double
    ci = C.c_int
    sigs = {
        "qnn_quantize": [vp, vp, sz, f32, i32, i32, i32, vp],
        "qnn_dequantize": [vp, vp, sz, f32, i32, vp],
        "qnn_quantize_u16": [vp, vp, sz, f32, i32, i32, i32, vp],
        "qnn_dequantize_u16": [vp, vp, sz, f32, i32, vp],
        "qnn_requantize": [vp, vp, sz, sz, vp, vp, ci, i32, i32, i32, vp],
        "qnn_qgemm": [vp, i64, i32, vp, i64, ci, ci, i64, i64, i64, vp, vp, vp, i32, i32, i32, vp, i64, vp, sz, vp],
        "qnn_qgemm_noalloc": [vp, i64, i32, vp, i64, ci, ci, i64, i64, i64, vp, vp, vp, i32, i32, i32, vp, i64, vp],
        "qnn_pack_b": [vp, i64, i64, i64, vp, i64, vp],
        "qnn_qconv2d": [vp, ci, ci, ci, ci, i32, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, vp, vp, i32, i32, i32, vp, vp, sz, vp],
        "qnn_tuning_set": [C.c_char_p, C.c_char_p],
        "qnn_calibrate_mfma": [ci, ci, ci, vp, C.POINTER(f64), vp],
        "qnn_calibrate_rescale": [ci, ci, vp, C.POINTER(f64), vp],
        "qnn_calibrate_copy": [vp, vp, sz, vp],
        "qnn_minmax": [vp, sz, f32, ci, vp, vp],
        "qnn_quantize_with": [vp, vp, sz, vp, vp],
        "qnn_quantize_dynamic": [vp, vp, sz, vp, vp],
        "qnn_simquant": [vp, vp, sz, f32, i32, i32, i32, vp],
        "qnn_simquant_backward": [vp, vp, vp, sz, f32, i32, i32, i32, vp],
        "qnn_qdwconv2d_asym": [vp, ci, ci, ci, ci, i32, vp, ci, ci, vp, ci, ci, ci, ci, vp, vp, vp, i32, i32, i32, vp, vp],
        "qnn_qgemm_asym": [vp, i64, i32, vp, i64, ci, ci, vp, i64, i64, i64, vp, vp, vp, i32, i32, i32, vp, i64, vp, sz, vp],
        "qnn_qconv2d_asym": [vp, ci, ci, ci, ci, i32, vp, ci, ci, ci, ci, vp, ci, ci, ci, ci, vp, vp, vp, i32, i32, i32, vp, vp,
                             sz, vp],
        "qnn_rescale_u8": [vp, i64, i32, i32, i32, i32, i32, i32, vp, i64, i64, i64, vp],
        "qnn_qgemm_add": [vp, i64, i32, vp, i64, ci, ci, i64, i64, i64, vp, vp, vp, i32, i32, i32, vp, i64, vp, vp, i64, vp,
                          sz, vp],
        "qnn_qconv2d_add": [vp, ci, ci, ci, ci, i32, vp, ci, ci, ci, ci, ci, ci, ci, ci, vp, vp, vp, i32, i32, i32, vp, vp,
                            vp, vp, sz, vp],
        "qnn_qdwconv2d": [vp, ci, ci, ci, ci, i32, vp, ci, ci, ci, ci, ci, ci, vp, vp, vp, i32, i32, i32, vp, vp],
        "qnn_qadd": [vp, i32, i32, i32, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp, sz, vp],
        "qnn_choose_qparams": [f64, f64, ci, C.POINTER(f32), C.POINTER(i32)],
        "qnn_quantize_multiplier": [f64, C.POINTER(i32), C.POINTER(i32)],
        "qnn_act_range": [ci, f32, i32, C.POINTER(i32), C.POINTER(i32)],
        "qnn_qadd_params": [f64, f64, f64] + [C.POINTER(i32)] * 7,
        "qnn_quantize_weights": [vp, sz, sz, ci, ci, vp, vp],
        "qnn_pack_int4": [vp, sz, vp],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.qnn_qgemm_workspace_bytes.restype = sz
    lib.qnn_qgemm_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    lib.qnn_qconv2d_workspace_bytes.restype = sz
    lib.qnn_qconv2d_workspace_bytes.argtypes = [ci] * 13
    _lib = lib
    return lib


def _check(name, rc):
    if rc != 0:
        detail = load_library().qnn_last_error().decode() if rc in (2, 3) else ""
        raise QnnError(name, rc, detail)


def _torch():
    import torch

    return torch


def _stream():
    return C.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dev(t, dtype, name):
    torch = _torch()
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: expected a contiguous device tensor of {dtype}, got "
                        f"{getattr(t, 'dtype', type(t))} on {getattr(t, 'device', '?')}")
    return C.c_void_p(t.data_ptr())


def _dev_rows(t, dtype, name):
    """Pointer and row pitch (in elements) of a 2-D device tensor whose rows are contiguous but may be
    spaced apart (a column slice of a wider matrix)."""
    torch = _torch()
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.dim() == 2 and
            (t.shape[1] == 1 or t.stride(1) == 1) and (t.shape[0] == 1 or t.stride(0) >= t.shape[1])):
        raise TypeError(f"{name}: expected a 2-D device tensor of {dtype} with contiguous rows")
    return C.c_void_p(t.data_ptr()), (t.stride(0) if t.shape[0] > 1 else t.shape[1])


def _out(out, shape, device, name="out"):
    """The output tensor: a new uint8 tensor of `shape`, or the caller's `out` after a shape check (the
    kernels write shape-many elements through its pointer)."""
    torch = _torch()
    if out is None:
        return torch.empty(shape, dtype=torch.uint8, device=device)
    if tuple(out.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(out.shape)}, expected {tuple(shape)}")
    return out


def _workspace(nbytes, device, workspace):
    """(pointer, size) of the scratch memory of a dense call: the caller's uint8 tensor, else a fresh
    one of the size the library asks for (none when that is 0).  The tensor is returned too, so that it
    stays referenced until the call has been enqueued (torch frees memory in stream order)."""
    torch = _torch()
    if workspace is not None:
        if not (isinstance(workspace, torch.Tensor) and workspace.is_cuda and workspace.dtype == torch.uint8 and
                workspace.is_contiguous()):
            raise TypeError("workspace: expected a contiguous uint8 device tensor")
        return C.c_void_p(workspace.data_ptr()), workspace.numel(), workspace
    if nbytes == 0:
        return None, 0, None
    ws = torch.empty(nbytes, dtype=torch.uint8, device=device)
    return C.c_void_p(ws.data_ptr()), nbytes, ws


def qgemm_workspace_bytes(M, N, K, weight_bits=8, asym=False):
    return int(load_library().qnn_qgemm_workspace_bytes(int(M), int(N), int(K), int(weight_bits), int(bool(asym))))


def qconv2d_workspace_bytes(N, H, W, Cin, Cout, kh, kw, stride, pad, weight_bits=8, asym=False):
    return int(load_library().qnn_qconv2d_workspace_bytes(int(N), int(H), int(W), int(Cin), int(Cout), int(kh), int(kw),
                                                          int(weight_bits), stride[0], stride[1], pad[0], pad[1],
                                                          int(bool(asym))))


def calibrate_mfma(workgroups, iters, random_operands, sink):
    """Enqueue the register-only MFMA loop; returns the integer operations of the launch."""
    torch = _torch()
    ops = C.c_double()
    _check("qnn_calibrate_mfma", load_library().qnn_calibrate_mfma(int(workgroups), int(iters), int(bool(random_operands)),
                                                                   _dev(sink, torch.int32, "sink"), C.byref(ops), _stream()))
    return float(ops.value)


def calibrate_rescale(workgroups, iters, sink):
    """Enqueue the register-only rescale loop; returns the number of accumulators it rescales."""
    torch = _torch()
    n = C.c_double()
    _check("qnn_calibrate_rescale", load_library().qnn_calibrate_rescale(int(workgroups), int(iters), _dev(sink, torch.int32, "sink"),
                                                                         C.byref(n), _stream()))
    return float(n.value)


def calibrate_copy(src, dst):
    torch = _torch()
    _check("qnn_calibrate_copy", load_library().qnn_calibrate_copy(_dev(src, torch.uint8, "src"), _dev(dst, torch.uint8, "dst"),
                                                                   src.numel(), _stream()))
    return dst


def tuning_set(name, value=None):
    """Set a tuning switch of the library (see qnn_tuning_set); value None restores the default."""
    v = None if value is None else str(value).encode()
    _check("qnn_tuning_set", load_library().qnn_tuning_set(name.encode(), v))


# ------------------------------------------------------------------ host helpers

def choose_qparams(xmin, xmax, bits=8):
    s, z = C.c_float(), C.c_int32()
    _check("qnn_choose_qparams", load_library().qnn_choose_qparams(xmin, xmax, bits, C.byref(s), C.byref(z)))
    return float(s.value), int(z.value)


def quantize_multiplier(real_mult):
    m, s = C.c_int32(), C.c_int32()
    _check("qnn_quantize_multiplier", load_library().qnn_quantize_multiplier(float(real_mult), C.byref(m), C.byref(s)))
    return int(m.value), int(s.value)


def quantize_multipliers(real_mults):
    """Vector form: returns (mult, shift) as int32 numpy arrays."""
    vals = np.asarray(real_mults, dtype=np.float64).ravel()
    out = [quantize_multiplier(v) for v in vals]
    return (np.array([o[0] for o in out], dtype=np.int32), np.array([o[1] for o in out], dtype=np.int32))


def act_range(kind, s_out, z_out):
    lo, hi = C.c_int32(), C.c_int32()
    _check("qnn_act_range", load_library().qnn_act_range(int(kind), float(s_out), int(z_out), C.byref(lo), C.byref(hi)))
    return int(lo.value), int(hi.value)


def qadd_params(s_a, s_b, s_out):
    v = [C.c_int32() for _ in range(7)]
    _check("qnn_qadd_params", load_library().qnn_qadd_params(float(s_a), float(s_b), float(s_out), *[C.byref(t) for t in v]))
    names = ["left_shift", "mult_a", "shift_a", "mult_b", "shift_b", "mult_o", "shift_o"]
    return {k: int(t.value) for k, t in zip(names, v)}


def quantize_weights(w, bits=8, restricted=True):
    """Host fp32 array [channels, ...] -> (int8 array of the same shape, Delta_c[channels])."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    ch = w.shape[0]
    wq = np.empty(w.shape, dtype=np.int8)
    d = np.empty(ch, dtype=np.float32)
    _check("qnn_quantize_weights", load_library().qnn_quantize_weights(
        w.ctypes.data, ch, w.size // ch, int(bits), int(bool(restricted)), wq.ctypes.data, d.ctypes.data))
    return wq, d


def pack_int4(v):
    v = np.ascontiguousarray(v, dtype=np.int8)
    out = np.empty(v.shape[:-1] + (v.shape[-1] // 2,), dtype=np.uint8)
    _check("qnn_pack_int4", load_library().qnn_pack_int4(v.ctypes.data, v.size, out.ctypes.data))
    return out


def qgemm_plan(M, N, K):
    """Tile configuration the dense kernels pick for an M x N x K product."""
    return load_library().qnn_qgemm_plan(int(M), int(N), int(K)).decode()


# ---------------------------------------------------------------- device kernels

def quantize(x, scale, zero_point, qmin=0, qmax=255, out=None):
    torch = _torch()
    q = _out(out, x.shape, x.device)
    _check("qnn_quantize", load_library().qnn_quantize(_dev(x, torch.float32, "x"), _dev(q, torch.uint8, "q"),
                                                      x.numel(), scale, zero_point, qmin, qmax, _stream()))
    return q


def dequantize(q, scale, zero_point, out=None):
    torch = _torch()
    x = torch.empty(q.shape, dtype=torch.float32, device=q.device) if out is None else out
    _check("qnn_dequantize", load_library().qnn_dequantize(_dev(q, torch.uint8, "q"), _dev(x, torch.float32, "x"),
                                                          q.numel(), scale, zero_point, _stream()))
    return x


def quantize_u16(x, scale, zero_point, qmin=0, qmax=65535, out=None):
    """Codes of up to 16 bits as a uint16 tensor."""
    torch = _torch()
    q = torch.empty(x.shape, dtype=torch.uint16, device=x.device) if out is None else out
    if tuple(q.shape) != tuple(x.shape):
        raise ValueError(f"out: shape {tuple(q.shape)}, expected {tuple(x.shape)}")
    _check("qnn_quantize_u16", load_library().qnn_quantize_u16(_dev(x, torch.float32, "x"), _dev(q, torch.uint16, "q"),
                                                              x.numel(), scale, zero_point, qmin, qmax, _stream()))
    return q


def dequantize_u16(q, scale, zero_point, out=None):
    torch = _torch()
    x = torch.empty(q.shape, dtype=torch.float32, device=q.device) if out is None else out
    if tuple(x.shape) != tuple(q.shape):
        raise ValueError(f"out: shape {tuple(x.shape)}, expected {tuple(q.shape)}")
    _check("qnn_dequantize_u16", load_library().qnn_dequantize_u16(_dev(q, torch.uint16, "q"), _dev(x, torch.float32, "x"),
                                                                  q.numel(), scale, zero_point, _stream()))
    return x


def requantize(acc, mult, shift, per_channel, z_out, act_min, act_max, out=None):
    torch = _torch()
    rows, ch = acc.shape
    y = _out(out, (rows, ch), acc.device)
    _check("qnn_requantize", load_library().qnn_requantize(
        _dev(acc, torch.int32, "acc"), _dev(y, torch.uint8, "y"), rows, ch, _dev(mult, torch.int32, "mult"),
        _dev(shift, torch.int32, "shift"), int(bool(per_channel)), z_out, act_min, act_max, _stream()))
    return y


def qgemm(A, z_a, B, mult, shift, z_out, act_min, act_max, bias=None, weight_bits=8,
          b_layout=B_COLUMNS_CONTIGUOUS, out=None, workspace=None):
    """A: uint8 [M,K] (rows may be spaced apart: a column slice of a wider matrix; same for `out`).  B: int8 [N,K] (columns contiguous), int8 [K,N] (rows contiguous), or uint8
    [N,K/2] nibble-packed when weight_bits == 4.  Returns uint8 [M,N]."""
    torch = _torch()
    M, K = A.shape
    if weight_bits == 4:
        N, ldb = B.shape[0], B.shape[1] * 2
        bp = _dev(B, torch.uint8, "B")
    elif b_layout == B_COLUMNS_CONTIGUOUS:
        N, ldb = B.shape
        bp = _dev(B, torch.int8, "B")
    else:
        ldb = N = B.shape[1]
        bp = _dev(B, torch.int8, "B")
    Cm = _out(out, (M, N), A.device)
    ap, lda = _dev_rows(A, torch.uint8, "A")
    cp, ldc = _dev_rows(Cm, torch.uint8, "C")
    wp, wbytes, _ws = _workspace(qgemm_workspace_bytes(M, N, K, weight_bits), A.device, workspace)
    _check("qnn_qgemm", load_library().qnn_qgemm(
        ap, lda, z_a, bp, ldb, b_layout, weight_bits, M, N, K, _dev(bias, torch.int32, "bias"),
        _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"), z_out, act_min, act_max,
        cp, ldc, wp, wbytes, _stream()))
    return Cm


def qgemm_noalloc(A, z_a, B, mult, shift, z_out, act_min, act_max, out, bias=None, weight_bits=8):
    """qnn_qgemm_noalloc: `qgemm` with columns-contiguous B into the caller's `out`, with the library's static
    scratch array; neither this wrapper nor the library allocates."""
    torch = _torch()
    M, K = A.shape
    if weight_bits == 4:
        N, ldb, bp = B.shape[0], B.shape[1] * 2, _dev(B, torch.uint8, "B")
    else:
        (N, ldb), bp = B.shape, _dev(B, torch.int8, "B")
    if tuple(out.shape) != (M, N):
        raise ValueError(f"out has shape {tuple(out.shape)}, expected {(M, N)}")
    ap, lda = _dev_rows(A, torch.uint8, "A")
    cp, ldc = _dev_rows(out, torch.uint8, "C")
    _check("qnn_qgemm_noalloc", load_library().qnn_qgemm_noalloc(
        ap, lda, z_a, bp, ldb, B_COLUMNS_CONTIGUOUS, weight_bits, M, N, K, _dev(bias, torch.int32, "bias"),
        _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"), z_out, act_min, act_max, cp, ldc, _stream()))
    return out


def prepare_qgemm(A, z_a, B, mult, shift, z_out, act_min, act_max, out, bias=None, weight_bits=8,
                  b_layout=B_COLUMNS_CONTIGUOUS, workspace=None):
    """Marshal the arguments of `qgemm` once and return a zero-argument callable that enqueues the
    product on the current stream.  For launch-bound loops: the per-call Python work shrinks to one
    foreign call.  The tensors must stay alive and unchanged in shape while the callable is used."""
    torch = _torch()
    M, K = A.shape
    if weight_bits == 4:
        N, ldb, bp = B.shape[0], B.shape[1] * 2, _dev(B, torch.uint8, "B")
    elif b_layout == B_COLUMNS_CONTIGUOUS:
        (N, ldb), bp = B.shape, _dev(B, torch.int8, "B")
    else:
        ldb = N = B.shape[1]
        bp = _dev(B, torch.int8, "B")
    fn = load_library().qnn_qgemm
    ap, lda = _dev_rows(A, torch.uint8, "A")
    cp, ldc = _dev_rows(out, torch.uint8, "C")
    wp, wbytes, ws = _workspace(qgemm_workspace_bytes(M, N, K, weight_bits), A.device, workspace)
    args = (ap, lda, z_a, bp, ldb, b_layout, weight_bits, M, N, K, _dev(bias, torch.int32, "bias"),
            _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"), z_out, act_min, act_max, cp, ldc,
            wp, wbytes)
    keep = (A, B, mult, shift, bias, out, ws)
    current_stream = torch.cuda.current_stream

    def launch(_keep=keep):
        rc = fn(*args, current_stream().cuda_stream)
        if rc != 0:
            _check("qnn_qgemm", rc)

    return launch


def pack_b(B_rows):
    """int8 [K,N] with contiguous rows -> int8 [N,K] (the layout qgemm runs fastest on)."""
    torch = _torch()
    K, N = B_rows.shape
    out = torch.empty((N, K), dtype=torch.int8, device=B_rows.device)
    _check("qnn_pack_b", load_library().qnn_pack_b(_dev(B_rows, torch.int8, "B"), N, K, N,
                                                  _dev(out, torch.int8, "out"), K, _stream()))
    return out


def _out_hw(H, W, kh, kw, stride, pad):
    return (H + 2 * pad[0] - kh) // stride[0] + 1, (W + 2 * pad[1] - kw) // stride[1] + 1


def qconv2d(x, z_x, w, stride, pad, mult, shift, z_out, act_min, act_max, bias=None, weight_bits=8, out=None,
            workspace=None):
    """x: uint8 NHWC.  w: int8 [Cout,kh,kw,Cin], or uint8 [Cout,kh,kw,Cin/2] packed 4-bit."""
    torch = _torch()
    N, H, W, Cin = x.shape
    Cout, kh, kw = w.shape[:3]
    wp = _dev(w, torch.uint8 if weight_bits == 4 else torch.int8, "w")
    Ho, Wo = _out_hw(H, W, kh, kw, stride, pad)
    y = _out(out, (N, Ho, Wo, Cout), x.device)
    sp, sbytes, _ws = _workspace(qconv2d_workspace_bytes(N, H, W, Cin, Cout, kh, kw, stride, pad, weight_bits), x.device,
                                 workspace)
    _check("qnn_qconv2d", load_library().qnn_qconv2d(
        _dev(x, torch.uint8, "x"), N, H, W, Cin, z_x, wp, Cout, kh, kw, weight_bits, stride[0], stride[1], pad[0],
        pad[1], _dev(bias, torch.int32, "bias"), _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"),
        z_out, act_min, act_max, _dev(y, torch.uint8, "y"), sp, sbytes, _stream()))
    return y


class _AddParams(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("mult_m", "shift_m", "z_r", "mult_r", "shift_r", "left_shift", "mult_o",
                                         "shift_o", "z_out", "act_min", "act_max")]


def _add_struct(z_r, params, z_out, act_min, act_max):
    """`params` is what qadd_params(s_mid, s_residual, s_out) returns (operand a = the layer's own result)."""
    p = params
    return _AddParams(p["mult_a"], p["shift_a"], z_r, p["mult_b"], p["shift_b"], p["left_shift"], p["mult_o"],
                      p["shift_o"], z_out, act_min, act_max)


def qgemm_add(A, z_a, B, mult, shift, z_mid, mid_min, mid_max, residual, z_r, params, z_out, act_min, act_max,
              bias=None, weight_bits=8, out=None, workspace=None):
    """qgemm (columns-contiguous B) whose uint8 result, quantized with (z_mid, mid_min, mid_max), is added to
    `residual` (uint8 [M,N], rows may be spaced apart) with the rescaling add of `params`; returns uint8 [M,N]."""
    torch = _torch()
    M, K = A.shape
    if weight_bits == 4:
        N, ldb, bp = B.shape[0], B.shape[1] * 2, _dev(B, torch.uint8, "B")
    else:
        (N, ldb), bp = B.shape, _dev(B, torch.int8, "B")
    Cm = _out(out, (M, N), A.device)
    ap, lda = _dev_rows(A, torch.uint8, "A")
    cp, ldc = _dev_rows(Cm, torch.uint8, "C")
    rp, ldr = _dev_rows(residual, torch.uint8, "residual")
    add = _add_struct(z_r, params, z_out, act_min, act_max)
    wp, wbytes, _ws = _workspace(qgemm_workspace_bytes(M, N, K, weight_bits), A.device, workspace)
    _check("qnn_qgemm_add", load_library().qnn_qgemm_add(
        ap, lda, z_a, bp, ldb, B_COLUMNS_CONTIGUOUS, weight_bits, M, N, K, _dev(bias, torch.int32, "bias"),
        _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"), z_mid, mid_min, mid_max, rp, ldr,
        C.addressof(add), cp, ldc, wp, wbytes, _stream()))
    return Cm


def qconv2d_add(x, z_x, w, stride, pad, mult, shift, z_mid, mid_min, mid_max, residual, z_r, params, z_out, act_min,
                act_max, bias=None, weight_bits=8, out=None, workspace=None):
    """qconv2d followed by the rescaling add with `residual` (uint8 NHWC, the shape of the output), fused."""
    torch = _torch()
    N, H, W, Cin = x.shape
    Cout, kh, kw = w.shape[:3]
    wp = _dev(w, torch.uint8 if weight_bits == 4 else torch.int8, "w")
    Ho, Wo = _out_hw(H, W, kh, kw, stride, pad)
    y = _out(out, (N, Ho, Wo, Cout), x.device)
    if tuple(residual.shape) != (N, Ho, Wo, Cout):
        raise ValueError(f"residual has shape {tuple(residual.shape)}, the output {(N, Ho, Wo, Cout)}")
    add = _add_struct(z_r, params, z_out, act_min, act_max)
    sp, sbytes, _ws = _workspace(qconv2d_workspace_bytes(N, H, W, Cin, Cout, kh, kw, stride, pad, weight_bits), x.device,
                                 workspace)
    _check("qnn_qconv2d_add", load_library().qnn_qconv2d_add(
        _dev(x, torch.uint8, "x"), N, H, W, Cin, z_x, wp, Cout, kh, kw, weight_bits, stride[0], stride[1], pad[0],
        pad[1], _dev(bias, torch.int32, "bias"), _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"),
        z_mid, mid_min, mid_max, _dev(residual, torch.uint8, "residual"), C.addressof(add),
        _dev(y, torch.uint8, "y"), sp, sbytes, _stream()))
    return y


def qgemm_asym(A, z_a, B, z_w, mult, shift, z_out, act_min, act_max, bias=None, weight_bits=8, out=None, workspace=None):
    """qgemm with a zero-point per weight column: z_w int32 [N] on the device.  B: int8 [N,K] (columns
    contiguous) or uint8 [N,K/2] nibble-packed."""
    torch = _torch()
    M, K = A.shape
    if weight_bits == 4:
        N, ldb, bp = B.shape[0], B.shape[1] * 2, _dev(B, torch.uint8, "B")
    else:
        (N, ldb), bp = B.shape, _dev(B, torch.int8, "B")
    Cm = _out(out, (M, N), A.device)
    ap, lda = _dev_rows(A, torch.uint8, "A")
    cp, ldc = _dev_rows(Cm, torch.uint8, "C")
    wp, wbytes, _ws = _workspace(qgemm_workspace_bytes(M, N, K, weight_bits, True), A.device, workspace)
    _check("qnn_qgemm_asym", load_library().qnn_qgemm_asym(
        ap, lda, z_a, bp, ldb, B_COLUMNS_CONTIGUOUS, weight_bits, _dev(z_w, torch.int32, "z_w"), M, N, K,
        _dev(bias, torch.int32, "bias"), _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"), z_out,
        act_min, act_max, cp, ldc, wp, wbytes, _stream()))
    return Cm


def qconv2d_asym(x, z_x, w, z_w, stride, pad, mult, shift, z_out, act_min, act_max, bias=None, weight_bits=8, out=None,
                 workspace=None):
    """qconv2d with a zero-point per output channel: z_w int32 [Cout] on the device."""
    torch = _torch()
    N, H, W, Cin = x.shape
    Cout, kh, kw = w.shape[:3]
    wp = _dev(w, torch.uint8 if weight_bits == 4 else torch.int8, "w")
    Ho, Wo = _out_hw(H, W, kh, kw, stride, pad)
    y = _out(out, (N, Ho, Wo, Cout), x.device)
    sp, sbytes, _ws = _workspace(qconv2d_workspace_bytes(N, H, W, Cin, Cout, kh, kw, stride, pad, weight_bits, True), x.device,
                                 workspace)
    _check("qnn_qconv2d_asym", load_library().qnn_qconv2d_asym(
        _dev(x, torch.uint8, "x"), N, H, W, Cin, z_x, wp, Cout, kh, kw, weight_bits, _dev(z_w, torch.int32, "z_w"),
        stride[0], stride[1], pad[0], pad[1], _dev(bias, torch.int32, "bias"), _dev(mult, torch.int32, "mult"),
        _dev(shift, torch.int32, "shift"), z_out, act_min, act_max, _dev(y, torch.uint8, "y"), sp, sbytes, _stream()))
    return y


def new_range_state(xmin=0.0, xmax=0.0):
    """Device-resident quantizer state (qnn_dyn_qparams: scale, zero_point, xmin, xmax, 2 work words) as
    an int32 tensor of 6 elements; `read_range_state` decodes it."""
    torch = _torch()
    host = np.zeros(6, dtype=np.int32)
    host[2:4] = np.array([xmin, xmax], dtype=np.float32).view(np.int32)
    return torch.from_numpy(host).to("cuda:0")


def read_range_state(state):
    h = state.cpu().numpy()
    f = h.view(np.float32)
    return dict(scale=float(f[0]), zero_point=int(h[1]), xmin=float(f[2]), xmax=float(f[3]))


def minmax(x, state, momentum=0.0, bits=8):
    """Range of the finite elements of x (or its moving average) and the quantizer parameters, into `state`."""
    torch = _torch()
    _check("qnn_minmax", load_library().qnn_minmax(_dev(x, torch.float32, "x"), x.numel(), float(momentum), int(bits),
                                                   _dev(state, torch.int32, "state"), _stream()))
    return state


def quantize_with(x, state, out=None):
    torch = _torch()
    q = _out(out, x.shape, x.device)
    _check("qnn_quantize_with", load_library().qnn_quantize_with(_dev(x, torch.float32, "x"), _dev(q, torch.uint8, "q"),
                                                                 x.numel(), _dev(state, torch.int32, "state"), _stream()))
    return q


def quantize_dynamic(x, state, out=None):
    """uint8 codes of x with the quantizer of its own range; the parameters are left in `state`."""
    torch = _torch()
    q = _out(out, x.shape, x.device)
    _check("qnn_quantize_dynamic", load_library().qnn_quantize_dynamic(
        _dev(x, torch.float32, "x"), _dev(q, torch.uint8, "q"), x.numel(), _dev(state, torch.int32, "state"), _stream()))
    return q


def simquant(x, scale, zero_point, qmin=0, qmax=255, out=None):
    torch = _torch()
    y = torch.empty(x.shape, dtype=torch.float32, device=x.device) if out is None else out
    _check("qnn_simquant", load_library().qnn_simquant(_dev(x, torch.float32, "x"), _dev(y, torch.float32, "y"), x.numel(),
                                                       float(scale), int(zero_point), int(qmin), int(qmax), _stream()))
    return y


def simquant_backward(x, grad_y, scale, zero_point, qmin=0, qmax=255, out=None):
    torch = _torch()
    gx = torch.empty(x.shape, dtype=torch.float32, device=x.device) if out is None else out
    _check("qnn_simquant_backward", load_library().qnn_simquant_backward(
        _dev(x, torch.float32, "x"), _dev(grad_y, torch.float32, "grad_y"), _dev(gx, torch.float32, "grad_x"), x.numel(),
        float(scale), int(zero_point), int(qmin), int(qmax), _stream()))
    return gx


def rescale_u8(x, z_in, mult, shift, z_out, act_min=0, act_max=255, out=None):
    """uint8 [rows, cols] (rows may be spaced apart) re-quantized to another quantizer; `out` may be a
    column slice of a wider tensor (the destination of a concatenation)."""
    torch = _torch()
    rows, cols = x.shape
    y = _out(out, (rows, cols), x.device)
    xp, ldx = _dev_rows(x, torch.uint8, "x")
    yp, ldy = _dev_rows(y, torch.uint8, "y")
    _check("qnn_rescale_u8", load_library().qnn_rescale_u8(xp, ldx, int(z_in), int(mult), int(shift), int(z_out), int(act_min),
                                                           int(act_max), yp, ldy, rows, cols, _stream()))
    return y


def qdwconv2d_asym(x, z_x, w, z_w, stride, pad, mult, shift, z_out, act_min, act_max, bias=None, out=None):
    """Depthwise layer with a weight zero-point per channel: z_w int32 [C] on the device."""
    torch = _torch()
    N, H, W, Cc = x.shape
    kh, kw = w.shape[:2]
    Ho, Wo = _out_hw(H, W, kh, kw, stride, pad)
    y = _out(out, (N, Ho, Wo, Cc), x.device)
    _check("qnn_qdwconv2d_asym", load_library().qnn_qdwconv2d_asym(
        _dev(x, torch.uint8, "x"), N, H, W, Cc, z_x, _dev(w, torch.int8, "w"), kh, kw, _dev(z_w, torch.int32, "z_w"), stride[0],
        stride[1], pad[0], pad[1], _dev(bias, torch.int32, "bias"), _dev(mult, torch.int32, "mult"),
        _dev(shift, torch.int32, "shift"), z_out, act_min, act_max, _dev(y, torch.uint8, "y"), _stream()))
    return y


def qdwconv2d(x, z_x, w, stride, pad, mult, shift, z_out, act_min, act_max, bias=None, out=None):
    """x: uint8 NHWC.  w: int8 [kh,kw,C]."""
    torch = _torch()
    N, H, W, Cc = x.shape
    kh, kw = w.shape[:2]
    Ho, Wo = _out_hw(H, W, kh, kw, stride, pad)
    y = _out(out, (N, Ho, Wo, Cc), x.device)
    _check("qnn_qdwconv2d", load_library().qnn_qdwconv2d(
        _dev(x, torch.uint8, "x"), N, H, W, Cc, z_x, _dev(w, torch.int8, "w"), kh, kw, stride[0], stride[1], pad[0],
        pad[1], _dev(bias, torch.int32, "bias"), _dev(mult, torch.int32, "mult"), _dev(shift, torch.int32, "shift"),
        z_out, act_min, act_max, _dev(y, torch.uint8, "y"), _stream()))
    return y


def qadd(a, z_a, b, z_b, params, z_out, act_min, act_max, out=None):
    torch = _torch()
    y = _out(out, a.shape, a.device)
    p = params
    _check("qnn_qadd", load_library().qnn_qadd(
        _dev(a, torch.uint8, "a"), z_a, p["mult_a"], p["shift_a"], _dev(b, torch.uint8, "b"), z_b, p["mult_b"],
        p["shift_b"], p["left_shift"], p["mult_o"], p["shift_o"], z_out, act_min, act_max, _dev(y, torch.uint8, "y"),
        a.numel(), _stream()))
    return y
