"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
its host helpers agree with the oracle's, and argument validation rejects bad calls before
anything is launched (so these run without a GPU)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_1806_08342_amd as qnn
from paper_1806_08342_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return qnn.load_library()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "qnn.h")).read()
    declared = sorted(set(re.findall(r"\b(qnn_[a-z0-9_]+)\s*\(", header)) - {"qnn_status"})
    assert len(declared) >= 15
    for name in declared:
        assert hasattr(lib, name), f"{name} declared in qnn.h but not exported"
    assert sorted(binding.EXPORTS) == declared
    assert lib.qnn_version().decode().count(".") == 1


def test_choose_qparams_matches_oracle_and_paper_example():
    rng = np.random.default_rng(0)
    assert qnn.choose_qparams(2.1, 3.5) == (float(np.float32(3.5 / 255)), 0)  # Sec. 2.1 worked example
    cases = [(0.0, 0.0), (-1.0, 1.0), (0.0, 6.0), (-6.0, 0.0), (-3.5, -2.1)]
    cases += [tuple(sorted(rng.normal(0, 5, 2))) for _ in range(500)]
    for lo, hi in cases:
        for bits in (8, 4):
            assert qnn.choose_qparams(lo, hi, bits) == oracle.choose_qparams(lo, hi, bits)


def test_quantize_multiplier_matches_oracle():
    rng = np.random.default_rng(1)
    vals = list(10 ** rng.uniform(-11, 2, 3000)) + [0.0, 0.5, 1.0, 1 - 2.0 ** -40, 2.0 ** -32, 2.0 ** -33, 2.0 ** 30]
    for v in vals:
        assert qnn.quantize_multiplier(v) == oracle.quantize_multiplier(v), v
    m, s = C.c_int32(), C.c_int32()
    assert qnn.load_library().qnn_quantize_multiplier(-1.0, C.byref(m), C.byref(s)) == 1
    assert qnn.load_library().qnn_quantize_multiplier(float("nan"), C.byref(m), C.byref(s)) == 1
    assert qnn.load_library().qnn_quantize_multiplier(2.0 ** 40, C.byref(m), C.byref(s)) == 1


def test_act_range_and_qadd_params_match_oracle():
    rng = np.random.default_rng(2)
    for _ in range(300):
        s, z = float(np.float32(10 ** rng.uniform(-3, 0))), int(rng.integers(0, 256))
        for kind in (0, 1, 2):
            assert qnn.act_range(kind, s, z) == oracle.act_range(kind, s, z)
        sa, sb, so = (10 ** rng.uniform(-3, 0, 3)).tolist()
        assert qnn.qadd_params(sa, sb, so) == oracle.qadd_params(sa, sb, so)
    assert qnn.act_range(2, 0.05, 0) == (0, 120)


def test_weight_quantizer_and_int4_pack_match_oracle():
    rng = np.random.default_rng(3)
    w = rng.normal(0, 0.1, (24, 3, 3, 16)).astype(np.float32)
    w[5] = 0
    for bits in (8, 4):
        for restricted in (True, False):
            a, da = qnn.quantize_weights(w, bits, restricted)
            b, db = oracle.quantize_weights(w, bits, restricted)
            assert (a == b).all() and (da == db).all()
    v = rng.integers(-8, 8, (7, 10)).astype(np.int8)
    assert (qnn.pack_int4(v) == oracle.pack_int4(v)).all()
    bad = v.copy()
    bad[0, 0] = 9
    with pytest.raises(qnn.QnnError):
        qnn.pack_int4(bad)


def test_device_entry_points_reject_bad_arguments_before_launching(lib):
    """Every path below returns from host-side validation; no HIP call is made."""
    p = C.c_void_p(4096)  # never dereferenced
    null = C.c_void_p(0)
    EINVAL = 1
    assert lib.qnn_quantize(p, p, 16, 0.0, 0, 0, 255, None) == EINVAL        # scale must be > 0
    assert lib.qnn_quantize(p, p, 16, 1.0, 300, 0, 255, None) == EINVAL      # zero-point outside range
    assert lib.qnn_quantize(null, p, 16, 1.0, 0, 0, 255, None) == EINVAL
    assert lib.qnn_quantize(null, null, 0, 1.0, 0, 0, 255, None) == 0        # empty input is a no-op
    assert lib.qnn_dequantize(p, p, 16, float("inf"), 0, None) == EINVAL
    assert lib.qnn_dequantize(null, null, 0, 1.0, 0, None) == 0
    assert lib.qnn_requantize(p, p, 4, 4, p, p, 1, 0, 10, 5, None) == EINVAL  # act_min > act_max
    assert lib.qnn_requantize(p, p, 0, 4, p, p, 1, 0, 0, 255, None) == EINVAL
    g = lambda **kw: lib.qnn_qgemm(*[kw.get(k, d) for k, d in [
        ("A", p), ("lda", 64), ("z_a", 128), ("B", p), ("ldb", 64), ("layout", 0), ("bits", 8), ("M", 8), ("N", 8),
        ("K", 64), ("bias", null), ("mult", p), ("shift", p), ("z_out", 0), ("lo", 0), ("hi", 255), ("C", p),
        ("ldc", 8), ("workspace", null), ("workspace_bytes", 0), ("stream", None)]])
    assert g(K=65537, lda=65537, ldb=65537) == EINVAL      # int32 accumulator bound
    assert g(bits=5) == EINVAL
    assert g(bits=4, K=63, lda=63) == EINVAL                # odd K with nibble pairs
    assert g(bits=4, layout=1) == EINVAL                    # 4-bit needs contiguous columns
    assert g(lda=8) == EINVAL
    assert g(z_a=256) == EINVAL
    assert g(M=0) == 0                                      # an empty batch is a no-op
    assert g(M=-1) == EINVAL
    assert g(mult=null) == EINVAL
    conv = lambda **kw: lib.qnn_qconv2d(*[kw.get(k, d) for k, d in [
        ("x", p), ("N", 1), ("H", 8), ("W", 8), ("Cin", 16), ("z_x", 0), ("w", p), ("Cout", 8), ("kh", 3), ("kw", 3),
        ("bits", 8), ("sh", 1), ("sw", 1), ("ph", 1), ("pw", 1), ("bias", null), ("mult", p), ("shift", p),
        ("z_out", 0), ("lo", 0), ("hi", 255), ("y", p), ("workspace", null), ("workspace_bytes", 0), ("stream", None)]])
    assert conv(kh=11, kw=11, ph=0, pw=0) == EINVAL          # kernel larger than the padded image
    assert conv(sh=0) == EINVAL
    assert conv(bits=4, Cin=15) == EINVAL
    assert conv(Cin=8192) == EINVAL                          # kh*kw*Cin > 65536
    assert conv(lo=-1) == EINVAL
    assert conv(N=0, x=null, y=null) == 0                    # an empty batch is a no-op
    assert conv(N=-1) == EINVAL
    dw = lambda **kw: lib.qnn_qdwconv2d(*[kw.get(k, d) for k, d in [
        ("x", p), ("N", 1), ("H", 8), ("W", 8), ("C", 16), ("z_x", 0), ("w", p), ("kh", 3), ("kw", 3), ("sh", 1),
        ("sw", 1), ("ph", 1), ("pw", 1), ("bias", null), ("mult", p), ("shift", p), ("z_out", 0), ("lo", 0),
        ("hi", 255), ("y", p), ("stream", None)]])
    assert dw(kh=9) == EINVAL
    assert dw(z_x=-1) == EINVAL
    assert dw(w=null) == EINVAL
    assert dw(N=0, x=null, y=null) == 0
    assert dw(N=-2) == EINVAL
    assert lib.qnn_qadd(p, 0, 1, 0, p, 0, 1, 0, 23, 1, 0, 0, 0, 255, p, 16, None) == EINVAL   # left_shift > 22
    assert lib.qnn_qadd(p, 0, 1, 40, p, 0, 1, 0, 20, 1, 0, 0, 0, 255, p, 16, None) == EINVAL  # shift out of range
    assert lib.qnn_qadd(null, 0, 1, 0, null, 0, 1, 0, 20, 1, 0, 0, 0, 255, null, 0, None) == 0
    assert lib.qnn_pack_b(p, 4, 8, 8, p, 8, None) == EINVAL  # ld_src < N
    # ranges on the device and simulated quantization
    assert lib.qnn_minmax(p, 16, C.c_float(0.0), 8, null, None) == EINVAL
    assert lib.qnn_minmax(p, 16, C.c_float(1.0), 8, p, None) == EINVAL      # momentum must stay below 1
    assert lib.qnn_minmax(p, 16, C.c_float(0.0), 1, p, None) == EINVAL      # 2..16 bits
    assert lib.qnn_quantize_with(p, p, 16, null, None) == EINVAL
    assert lib.qnn_quantize_dynamic(null, p, 16, p, None) == EINVAL
    assert lib.qnn_simquant(p, p, 16, C.c_float(0.0), 0, 0, 255, None) == EINVAL
    assert lib.qnn_simquant(p, p, 16, C.c_float(0.1), 300, 0, 255, None) == EINVAL
    assert lib.qnn_simquant(p, null, 16, C.c_float(0.1), 0, 0, 255, None) == EINVAL
    assert lib.qnn_simquant_backward(p, p, p, 16, C.c_float(0.1), 0, 9, 3, None) == EINVAL
    assert lib.qnn_simquant_backward(p, null, p, 16, C.c_float(0.1), 0, 0, 255, None) == EINVAL
    assert lib.qnn_simquant(null, null, 0, C.c_float(0.1), 0, 0, 255, None) == 0
    assert lib.qnn_simquant(p, p, 16, C.c_float(0.1), 0, 0, 65536, None) == EINVAL
    assert lib.qnn_quantize_u16(p, p, 16, C.c_float(0.1), 0, 0, 65536, None) == EINVAL
    assert lib.qnn_quantize_u16(p, p, 16, C.c_float(0.1), 70000, 0, 65535, None) == EINVAL
    assert lib.qnn_quantize_u16(p, null, 16, C.c_float(0.1), 0, 0, 65535, None) == EINVAL
    assert lib.qnn_quantize_u16(null, null, 0, C.c_float(0.1), 0, 0, 65535, None) == 0
    assert lib.qnn_dequantize_u16(p, p, 16, C.c_float(0.0), 0, None) == EINVAL
    assert lib.qnn_dequantize_u16(p, p, 16, C.c_float(0.1), 65536, None) == EINVAL
    assert lib.qnn_dequantize_u16(null, null, 0, C.c_float(0.1), 0, None) == 0
    assert lib.qnn_rescale_u8(p, 8, 0, 1 << 30, 1, 0, 0, 255, p, 4, 2, 8, None) == EINVAL   # ldy < cols
    assert lib.qnn_rescale_u8(p, 8, 300, 1 << 30, 1, 0, 0, 255, p, 8, 2, 8, None) == EINVAL
    assert lib.qnn_rescale_u8(null, 8, 0, 1 << 30, 1, 0, 0, 255, null, 8, 0, 8, None) == 0
    # asymmetric weights: the zero-point array is required, and K is limited to 32768
    asym = lambda z_w=p, K=64, ws=p, wsb=4096: lib.qnn_qgemm_asym(p, K, 0, p, K, 0, 8, z_w, 64, 64, K, null, p, p, 0, 0, 255,
                                                                   p, 64, ws, wsb, None)
    assert asym(z_w=null) == EINVAL
    assert asym(K=32768 + 64) == EINVAL
    assert asym(ws=null, wsb=0) == EINVAL                    # the row sums need the caller's workspace
    assert asym(wsb=64) == EINVAL                            # ... all of it
    assert asym(ws=C.c_void_p(4100)) == EINVAL               # ... 16-byte aligned
    assert lib.qnn_qgemm_workspace_bytes(64, 64, 64, 8, 1) == 256
    assert lib.qnn_qconv2d_asym(p, 1, 8, 8, 16, 0, p, 8, 3, 3, 8, null, 1, 1, 1, 1, null, p, p, 0, 0, 255, p, p, 4096,
                                None) == EINVAL
    assert lib.qnn_qconv2d_asym(p, 1, 64, 64, 4096, 0, p, 8, 3, 3, 8, p, 1, 1, 1, 1, null, p, p, 0, 0, 255, p, p, 1 << 20,
                                None) == EINVAL
    # the fused add: every field is checked on the host before anything is launched
    fields = dict(mult_m=1 << 30, shift_m=1, z_r=0, mult_r=1 << 30, shift_r=1, left_shift=20, mult_o=1 << 30, shift_o=10,
                  z_out=0, act_min=0, act_max=255)
    def gemm_add(residual=p, ldr=64, **kw):
        add = binding._AddParams(**{**fields, **kw})
        return lib.qnn_qgemm_add(p, 64, 0, p, 64, 0, 8, 64, 64, 64, null, p, p, 0, 0, 255, residual, ldr, C.addressof(add),
                                 p, 64, null, 0, None)
    assert gemm_add(residual=null) == EINVAL
    assert gemm_add(ldr=8) == EINVAL
    assert gemm_add(left_shift=23) == EINVAL
    assert gemm_add(shift_o=32) == EINVAL
    assert gemm_add(z_r=256) == EINVAL
    assert gemm_add(act_min=9, act_max=3) == EINVAL
    assert lib.qnn_qgemm_add(p, 64, 0, p, 64, 0, 8, 64, 64, 64, null, p, p, 0, 0, 255, p, 64, null, p, 64, null, 0,
                             None) == EINVAL
    add = binding._AddParams(**fields)
    assert lib.qnn_qconv2d_add(p, 1, 8, 8, 16, 0, p, 8, 3, 3, 8, 1, 1, 1, 1, null, p, p, 0, 0, 255, null, C.addressof(add),
                               p, null, 0, None) == EINVAL


def test_workspace_queries_and_tuning_switches(lib):
    # split-K shapes of the sweep ask for their partial sums; everything else for nothing
    assert qnn.qgemm_workspace_bytes(8192, 8192, 8192) == 0
    assert qnn.qgemm_workspace_bytes(1024, 1024, 8192) == 4 * 1024 * 1024 * 4 and qnn.qgemm_plan(1024, 1024, 8192).endswith("/k4")
    assert qnn.qgemm_workspace_bytes(256, 256, 4096) == 4 * 256 * 256 * 4
    assert qnn.qgemm_workspace_bytes(64, 4096, 4096) == 0 and qnn.qgemm_workspace_bytes(4096, 256, 256) == 0
    assert qnn.qgemm_workspace_bytes(1024, 1024, 8192, weight_bits=4) == 0      # 4-bit weights run unsplit
    assert qnn.qgemm_workspace_bytes(1000, 10, 100, asym=True) == 4096          # row sums, rounded up to 256 bytes
    assert qnn.qconv2d_workspace_bytes(2, 7, 7, 512, 512, 3, 3, (1, 1), (1, 1)) == qnn.qgemm_workspace_bytes(98, 512, 4608)
    assert qnn.qconv2d_workspace_bytes(0, 7, 7, 512, 512, 3, 3, (1, 1), (1, 1)) == 0
    # switches: unknown names are rejected, known ones change the plan and can be restored
    assert lib.qnn_tuning_set(b"QNN_NO_SUCH_SWITCH", b"1") == 1
    assert lib.qnn_tuning_set(None, b"1") == 1
    assert qnn.qgemm_plan(4096, 4096, 128) == "shortk"
    qnn.tuning_set("QNN_NO_SHORTK", 1)
    try:
        assert qnn.qgemm_plan(4096, 4096, 128) != "shortk"
        qnn.tuning_set("QNN_FORCE_TILE", "dma64x64")
        qnn.tuning_set("QNN_FORCE_SPLIT", 3)
        assert qnn.qgemm_plan(256, 256, 1024) == "dma64x64/k3"
        assert qnn.qgemm_workspace_bytes(256, 256, 1024) == 3 * 256 * 256 * 4
    finally:
        for name in ("QNN_NO_SHORTK", "QNN_FORCE_TILE", "QNN_FORCE_SPLIT"):
            qnn.tuning_set(name)
    assert qnn.qgemm_plan(4096, 4096, 128) == "shortk"


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", str(tmp_path / "libqnn.so"))
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load_library()


def test_workload_tables_match_the_networks():
    import workloads
    from workloads import shapes

    mb1 = workloads.mobilenet_v1()
    assert len(mb1) == 27 and sum(l.macs(1) for l in mb1) == 567_716_352
    rn = workloads.resnet50()
    assert sum(l.kind == "qadd" for l in rn) == 16 and sum(l.kind == "conv" for l in rn) == 53
    assert sum(l.macs(1) for l in rn) == 4_087_136_256
    mb2 = workloads.mobilenet_v2()
    assert sum(l.kind == "dw" for l in mb2) == 17 and mb2[-1].Cout == 1280
    assert workloads.single_conv()[0].macs(1) == 7_225_344
    full, skinny = workloads.gemm_sweep()
    assert len(full) == 64 and len(skinny) == 7
    assert len(shapes.unique_shapes(rn)) < len(rn)
