"""Parity at the full sizes of the five benchmark configurations, in the launch configuration
bench.py times.  Every output element is an independent dot product, so where the whole tensor
would take the oracle too long it evaluates a seeded sample of at least 10^6 outputs plus all
border pixels of the first and last image (where padding matters), and the same layer is
compared in full at batch 1 and 2; small cases are compared in full at their own batch."""
import numpy as np
import pytest

import oracle
import paper_1806_08342_amd as qnn
import workloads
from workloads import shapes as shp
from workloads import synth

from gpu_util import assert_same, dev, host

pytestmark = pytest.mark.gpu

N_SAMPLES = 1_000_000


def _sample_indices(rng, N, Ho, Wo, C):
    total = N * Ho * Wo * C
    if total <= 2_000_000:
        return None  # compare everything
    idx = [rng.integers(0, total, N_SAMPLES)]
    for n in {0, N - 1}:
        border = np.zeros((Ho, Wo), bool)
        border[[0, -1], :] = True
        border[:, [0, -1]] = True
        pix = np.flatnonzero(border.ravel())
        if pix.size * C > 400_000:
            pix = rng.choice(pix, 400_000 // C, replace=False)
        flat = ((n * Ho * Wo + pix)[:, None] * C + np.arange(C)[None, :]).ravel()
        idx.append(flat)
    return np.unique(np.concatenate(idx)).astype(np.int64)


def _check_layer(layer, batch, seed, what, whole=False):
    rng = np.random.default_rng(seed)
    if layer.kind == "qadd":
        n = batch * layer.H * layer.W * layer.Cout
        c = synth.qadd_case((n,), seed, oracle, act=layer.act)
        got = host(qnn.qadd(dev(c["a"]), c["z_a"], dev(c["b"]), c["z_b"], c["params"], c["z_out"], c["act_min"],
                            c["act_max"]))
        if n > 4_000_000 and not whole:
            idx = np.unique(np.r_[rng.integers(0, n, 2_000_000), np.arange(4096), np.arange(n - 4096, n)])
        else:
            idx = np.arange(n)
        want = oracle.qadd(c["a"][idx], c["z_a"], c["b"][idx], c["z_b"], c["params"], c["z_out"], c["act_min"],
                           c["act_max"])
        assert_same(got[idx], want, what)
        return
    in_range = (-2.0, 2.2) if (layer.kind == "conv" and layer.Cin == 3) else (0.0, 6.0)
    c = synth.conv_case(layer, batch, seed, oracle, in_range=in_range)
    w = c.get("w_packed", c["w"])
    args = (c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"], c["act_min"], c["act_max"])
    dargs = (c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]), c["z_out"], c["act_min"], c["act_max"])
    sample = None if whole else _sample_indices(rng, batch, layer.Ho, layer.Wo, layer.Cout)
    if layer.kind == "dw":
        got = host(qnn.qdwconv2d(dev(c["x"]), c["z_x"], dev(w), *dargs, bias=dev(c["bias"])))
        want = oracle.qdwconv2d(c["x"], c["z_x"], w, *args, bias=c["bias"], sample=sample)
    else:
        got = host(qnn.qconv2d(dev(c["x"]), c["z_x"], dev(w), *dargs, bias=dev(c["bias"]), weight_bits=layer.weight_bits))
        want = oracle.qconv2d(c["x"], c["z_x"], w, *args, bias=c["bias"], weight_bits=layer.weight_bits, sample=sample)
    if sample is None:
        assert_same(got, want, what)
    else:
        assert_same(got.ravel()[sample], want, what)
    clamped = np.mean((want == c["act_min"]) | (want == c["act_max"]))
    assert clamped < 0.8, f"{what}: {clamped:.0%} of the outputs sit on a clamp end, parity would be vacuous"


# ------------------------------------------------------------------ configuration 2

@pytest.mark.parametrize("M,N,K", workloads.gemm_sweep()[0], ids=lambda v: str(v))
def test_config2_gemm_sweep_shapes_sampled_rows(M, N, K):
    c = synth.gemm_case(M, N, K, workloads.seed_for(2, 100 + (M + 3 * N + 7 * K) % 97), oracle)
    got = host(qnn.qgemm(dev(c["A"]), c["z_a"], dev(c["Bt"]), dev(c["mult"]), dev(c["shift"]), c["z_out"], 0, 255))
    rng = np.random.default_rng(M + N + K)
    n_rows = max(8, min(M, int(2.5e9 // (N * K))))
    rows = np.unique(np.r_[0, M - 1, rng.integers(0, M, n_rows)])
    want = oracle.qgemm(c["A"][rows], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
    assert_same(got[rows], want, f"config 2 gemm {M}x{N}x{K} ({rows.size} rows)")
    assert np.mean((want == 0) | (want == 255)) < 0.05


@pytest.mark.parametrize("M", [1, 2, 4, 8, 16, 32, 64])
@pytest.mark.parametrize("bits", [8, 4])
def test_config2_skinny_gemm_full(M, bits):
    c = synth.gemm_case(M, 4096, 4096, workloads.seed_for(2, 200 + M + bits), oracle, weight_bits=bits)
    B = c["Bt_packed"] if bits == 4 else c["Bt"]
    got = host(qnn.qgemm(dev(c["A"]), c["z_a"], dev(B), dev(c["mult"]), dev(c["shift"]), c["z_out"], 0, 255,
                         weight_bits=bits))
    want = oracle.qgemm(c["A"], c["z_a"], B, c["mult"], c["shift"], c["z_out"], 0, 255, weight_bits=bits)
    assert_same(got, want, f"config 2 skinny M={M} bits={bits}")


# ------------------------------------------------------------------ configuration 3

MBV1 = workloads.mobilenet_v1()


@pytest.mark.parametrize("idx", range(len(MBV1)), ids=[l.name for l in MBV1])
@pytest.mark.parametrize("batch", [1, 64])
def test_config3_mobilenet_v1_layers(idx, batch):
    _check_layer(MBV1[idx], batch, workloads.seed_for(3, idx), f"config 3 {MBV1[idx].name} batch {batch}")


# ------------------------------------------------------------------ configuration 4

RN50 = shp.unique_shapes(workloads.resnet50())


@pytest.mark.parametrize("idx", range(len(RN50)), ids=[l.name for l in RN50])
def test_config4_resnet50_layers_batch256(idx):
    _check_layer(RN50[idx], 256, workloads.seed_for(4, idx), f"config 4 {RN50[idx].name} batch 256")


def _check_fused_add_layer(layer, batch, seed, what):
    """A convolution with the residual add of its block fused behind it, as bench.py times it: the
    oracle evaluates the sampled outputs of the convolution and adds the matching residual elements."""
    rng = np.random.default_rng(seed)
    conv = shp.replace(layer, kind="conv", act="none")
    c = synth.conv_case(conv, batch, seed, oracle)
    ad = synth.qadd_case((1,), seed + 7, oracle, act=layer.act)
    w = c.get("w_packed", c["w"])
    res = rng.integers(0, 256, (batch, layer.Ho, layer.Wo, layer.Cout)).astype(np.uint8)
    got = host(qnn.qconv2d_add(dev(c["x"]), c["z_x"], dev(w), c["stride"], c["pad"], dev(c["mult"]), dev(c["shift"]), c["z_out"], 0,
                               255, dev(res), ad["z_b"], ad["params"], ad["z_out"], ad["act_min"], ad["act_max"],
                               bias=dev(c["bias"]), weight_bits=layer.weight_bits))
    sample = _sample_indices(rng, batch, layer.Ho, layer.Wo, layer.Cout)
    mid = oracle.qconv2d(c["x"], c["z_x"], w, c["stride"], c["pad"], c["mult"], c["shift"], c["z_out"], 0, 255, bias=c["bias"],
                         weight_bits=layer.weight_bits, sample=sample)
    r = res.ravel() if sample is None else res.ravel()[sample]
    want = oracle.qadd(mid.ravel(), c["z_out"], r, ad["z_b"], ad["params"], ad["z_out"], ad["act_min"], ad["act_max"])
    assert_same(got.ravel() if sample is None else got.ravel()[sample], want, what)
    assert len(np.unique(want)) > 16, f"{what}: parity would be vacuous"


@pytest.mark.parametrize("idx", range(len(RN50)), ids=[l.name for l in RN50])
@pytest.mark.parametrize("batch", [1, 2])
def test_config4_resnet50_layers_whole_tensor_small_batch(idx, batch):
    _check_layer(RN50[idx], batch, workloads.seed_for(4, 600 + idx), f"config 4 {RN50[idx].name} batch {batch}", whole=True)


RN50_ADD = [l for l in shp.unique_shapes(workloads.fuse_adds(workloads.resnet50())) if l.kind == "conv_add"]


@pytest.mark.parametrize("idx", range(len(RN50_ADD)), ids=[l.name for l in RN50_ADD])
def test_config4_resnet50_fused_add_layers_batch256(idx):
    _check_fused_add_layer(RN50_ADD[idx], 256, workloads.seed_for(4, 300 + idx), f"config 4 {RN50_ADD[idx].name} batch 256")


# ------------------------------------------------------------------ configuration 5

MBV2 = shp.unique_shapes(workloads.mobilenet_v2(4))
MBV2_ADD = [l for l in shp.unique_shapes(workloads.fuse_adds(workloads.mobilenet_v2(4))) if l.kind == "conv_add"]


@pytest.mark.parametrize("idx", range(len(MBV2_ADD)), ids=[l.name for l in MBV2_ADD])
def test_config5_mobilenet_v2_fused_add_layers_batch32(idx):
    _check_fused_add_layer(MBV2_ADD[idx], 32, workloads.seed_for(5, 300 + idx), f"config 5 {MBV2_ADD[idx].name} batch 32")


@pytest.mark.parametrize("idx", range(len(MBV2)), ids=[l.name for l in MBV2])
def test_config5_mobilenet_v2_int4_layers_batch32(idx):
    _check_layer(MBV2[idx], 32, workloads.seed_for(5, idx), f"config 5 {MBV2[idx].name} batch 32")


@pytest.mark.parametrize("idx", range(len(MBV2)), ids=[l.name for l in MBV2])
@pytest.mark.parametrize("batch", [1, 2])
def test_config5_mobilenet_v2_int4_layers_whole_tensor_small_batch(idx, batch):
    _check_layer(MBV2[idx], batch, workloads.seed_for(5, 600 + idx), f"config 5 {MBV2[idx].name} batch {batch}", whole=True)


def test_config5_quantize_full_tensor():
    c = synth.quantize_case((256, 224, 224, 3), workloads.seed_for(5, 900), oracle)
    got = host(qnn.quantize(dev(c["x"]), c["scale"], c["zero_point"]))
    want = oracle.quantize(c["x"], c["scale"], c["zero_point"])
    assert_same(got, want, "config 5 quantize 256x224x224x3")
    back = host(qnn.dequantize(dev(want), c["scale"], c["zero_point"]))
    assert np.array_equal(back.view(np.uint32), oracle.dequantize(want, c["scale"], c["zero_point"]).view(np.uint32))
    # the quantizer's own guarantee (Sec. 2.1): error at most half a step inside the range
    assert np.abs(back.astype(np.float64) - c["x"]).max() <= 0.5 * c["scale"] * (1 + 2.0 ** -12)
