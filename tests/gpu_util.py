"""Helpers shared by the GPU parity tests: host <-> device copies and comparison."""
import numpy as np
import torch


def dev(a):
    """numpy array (or None) -> contiguous tensor on cuda:0"""
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def assert_same(got, want, what=""):
    """Bit-exact comparison with a useful message (first mismatch and count)."""
    got = np.asarray(got)
    want = np.asarray(want)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got.ravel() != want.ravel())
        i = int(bad[0])
        idx = np.unravel_index(i, got.shape)
        raise AssertionError(f"{what}: {bad.size} of {got.size} differ; first at {idx}: "
                             f"gpu={got.ravel()[i]} oracle={want.ravel()[i]}")
