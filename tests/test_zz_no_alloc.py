"""qnn_qgemm_noalloc (the entry point that takes its scratch memory from a static device array instead
of a workspace argument) against qnn_qgemm, through the C ABI, bit for bit."""
import numpy as np
import pytest
import torch

import oracle
import paper_1806_08342_amd as qnn
import workloads
from workloads import synth

from gpu_util import assert_same, dev, host

pytestmark = pytest.mark.gpu


def _case(M, N, K, seed):
    c = synth.gemm_case(M, N, K, workloads.seed_for(2, seed), oracle)
    return c, [dev(c[k]) for k in ("A", "Bt", "mult", "shift")]


def test_noalloc_matches_qgemm_on_two_calls_in_a_row_the_second_smaller():
    # both shapes divide K over several workgroups per tile, i.e. they use the scratch array; the
    # second call leaves most of what the first one wrote there untouched
    for (M, N, K, seed) in [(1024, 1024, 8192, 41), (256, 320, 4096, 42)]:
        assert "/k" in qnn.qgemm_plan(M, N, K) and 0 < qnn.qgemm_workspace_bytes(M, N, K) <= 16 << 20
        c, (A, Bt, mult, shift) = _case(M, N, K, seed)
        want = qnn.qgemm(A, c["z_a"], Bt, mult, shift, c["z_out"], 0, 255)
        out = torch.full((M, N), 7, dtype=torch.uint8, device="cuda:0")
        got = qnn.qgemm_noalloc(A, c["z_a"], Bt, mult, shift, c["z_out"], 0, 255, out)
        assert_same(host(got), host(want), f"qgemm_noalloc {M}x{N}x{K}")
        rows = np.r_[0:8, M - 8:M]
        ref = oracle.qgemm(c["A"][rows], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255)
        assert_same(host(got)[rows], ref, f"qgemm_noalloc {M}x{N}x{K} against the oracle")


def test_noalloc_runs_products_that_need_no_scratch_and_rejects_oversized_plans(tuning):
    M, N, K = 300, 200, 128
    c, (A, Bt, mult, shift) = _case(M, N, K, 43)
    out = torch.empty((M, N), dtype=torch.uint8, device="cuda:0")
    qnn.qgemm_noalloc(A, c["z_a"], Bt, mult, shift, c["z_out"], 0, 255, out)
    assert_same(host(out), oracle.qgemm(c["A"], c["z_a"], c["Bt"], c["mult"], c["shift"], c["z_out"], 0, 255), "no scratch")
    # a forced split whose partial sums exceed the static array
    tuning.setenv("QNN_FORCE_TILE", "dma128x128")
    tuning.setenv("QNN_FORCE_SPLIT", "8")
    M, N, K = 1024, 1024, 8192
    assert qnn.qgemm_workspace_bytes(M, N, K) == 32 << 20
    c, (A, Bt, mult, shift) = _case(M, N, K, 44)
    out = torch.empty((M, N), dtype=torch.uint8, device="cuda:0")
    with pytest.raises(qnn.QnnError, match="static array"):
        qnn.qgemm_noalloc(A, c["z_a"], Bt, mult, shift, c["z_out"], 0, 255, out)
