"""Helpers shared by the GPU parity tests (no arithmetic of the method lives here)."""
import numpy as np
import torch

from oracle import pipe_oracle as po

REL_TOL = 1e-3   # fp32 output: tolerance the benchmark's target states


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")


def oracle_expand(W, spec, min_gap=1e-9):
    """Oracle expansion; asserts no mask decision sits on a near-tie (where the order of an
    fp64 sum could decide it)."""
    gaps = []
    e = po.expand(W, spec.bits, spec.K, spec.gamma, spec.group, gaps=gaps)
    assert all(g > min_gap for g in gaps), "input has a near-tie in the group scores: %r" % (gaps,)
    return e


def assert_expansion_equal(gpu_exp, ora):
    """Bit-exact: kept groups, scales (fp32 bit patterns) and codes of every order."""
    assert gpu_exp.K == ora.K
    for k in range(1, ora.K + 1):
        gids, scales, codes = gpu_exp.order(k)
        o = ora.orders[k - 1]
        assert np.array_equal(gids, o.group_ids), "order %d: kept groups differ" % k
        assert np.array_equal(scales.view(np.uint32), o.scales.view(np.uint32)), "order %d: scales differ" % k
        assert np.array_equal(codes, o.codes), "order %d: codes differ (%d elements)" % (
            k, int((codes != o.codes).sum()))


def assert_close_fp32(y_gpu: np.ndarray, y_ref: np.ndarray, tol=REL_TOL, elementwise=True):
    """max|d| <= tol*max|ref| per tensor and |d| <= tol*|ref| + tol*rms(ref) per element."""
    assert y_gpu.shape == y_ref.shape
    d = np.abs(y_gpu.astype(np.float64) - y_ref.astype(np.float64))
    mx = float(np.abs(y_ref).max())
    rms = float(np.sqrt(np.mean(y_ref.astype(np.float64) ** 2)))
    assert d.max() <= tol * mx + 1e-30, "max error %g vs max|y| %g" % (d.max(), mx)
    if elementwise:
        assert np.all(d <= tol * np.abs(y_ref) + tol * rms + 1e-30)
    return d.max() / (mx + 1e-30)
