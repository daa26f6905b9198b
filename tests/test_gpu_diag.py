"""GPU parity of the data-free diagnostics (App. C) against the CPU checker."""
import math

import numpy as np
import pytest
import torch

from oracle import pipe_oracle as po
from paper_2311_15806_amd import workloads as wl

from _parity import assert_expansion_equal, dev, oracle_expand

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def pipe():
    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_2311_15806_amd.binding as b
    return b


@pytest.mark.parametrize("O,I", [(384, 1000), (1000, 130), (37, 53), (1, 7), (300, 1)])
def test_spectral_norm_parity(pipe, O, I):
    rng = np.random.default_rng(900 + O)
    W = (rng.standard_t(3, size=(O, I)) * 0.02).astype(f32)
    for iters in (1, 7, 60):
        ref = po.spectral_norm(W, iters)
        got = pipe.pipe_spectral_norm(dev(W), iters)
        assert math.isclose(got, ref, rel_tol=2e-6), (iters, got, ref)
    sv = np.linalg.svd(W.astype(np.float64), compute_uv=False)[0]
    assert pipe.pipe_spectral_norm(dev(W), 300) <= sv * (1 + 1e-6)
    assert pipe.pipe_spectral_norm(dev(np.zeros((8, 8), f32)), 3) == 0.0


@pytest.mark.parametrize("bits,K,gamma,group", [(4, 3, 0.5, 32), (2, 5, 0.25, 16), (8, 2, 1.0, 16), (3, 4, 0.5, 16)])
def test_reconstruction_and_bounds_parity(pipe, bits, K, gamma, group):
    O, I = 192, 328
    rng = np.random.default_rng(910 + bits)
    W = (rng.standard_t(3, size=(O, I)) * 0.015).astype(f32)
    spec = wl.LayerSpec(O, I, bits, K, gamma, group)
    ora = oracle_expand(W, spec)
    g = pipe.pipe_expand(dev(W), bits, K, gamma, group)
    assert_expansion_equal(g, ora)
    for upto in (1, K):
        R = pipe.pipe_expansion_reconstruct(g, upto).cpu().numpy()
        ref = ora.reconstruct(upto)
        assert np.abs(R - ref).max() <= 1e-6 * np.abs(ref).max()
    u_lemma, u_stored = pipe.pipe_expansion_error_bound(g)
    assert math.isclose(u_lemma, po.lemma_bound_u(ora), rel_tol=1e-12)
    assert math.isclose(u_stored, po.stored_bound_u(ora), rel_tol=1e-12)
    # the bound holds for what the GPU reconstructed
    err = np.abs(W.astype(np.float64) - pipe.pipe_expansion_reconstruct(g).cpu().numpy())
    assert err.max() <= u_stored + np.abs(W).max() * 2.0 ** -20
    # U of a two-layer stack of this layer, against the checker
    s = pipe.pipe_spectral_norm(dev(W), 40)
    assert math.isclose(pipe.pipe_error_bound_U([s, s], [u_stored, u_stored]),
                        po.error_bound_U([s, s], [u_stored, u_stored]), rel_tol=1e-12)
    g.free()


def test_spectral_norm_of_the_headline_layer(pipe):
    """Full-size C4 weight (11008 x 4096): same iterate as the checker after a few steps."""
    W = wl.make_weight(wl.C4, 0)
    ref = po.spectral_norm(W, 4)
    got = pipe.pipe_spectral_norm(dev(W), 4)
    assert math.isclose(got, ref, rel_tol=2e-6)


@pytest.mark.parametrize("bits,K,gamma,group", [(4, 3, 0.5, 32), (2, 5, 0.25, 16), (8, 2, 1.0, 16)])
def test_order_norms_and_U_ens_parity(pipe, bits, K, gamma, group):
    """||R^(k)|| of every order: the same power iteration on both sides, step for step; then
    U_ens and the predictor-size rule of a two-layer stack of this layer."""
    O, I = 192, 328
    rng = np.random.default_rng(940 + bits)
    W = (rng.standard_t(3, size=(O, I)) * 0.015).astype(f32)
    ora = oracle_expand(W, wl.LayerSpec(O, I, bits, K, gamma, group))
    g = pipe.pipe_expand(dev(W), bits, K, gamma, group)
    assert_expansion_equal(g, ora)
    for iters in (2, 30):
        ref = po.order_norms(ora, iters)
        got = pipe.pipe_expansion_order_norms(g, iters)
        assert len(got) == K
        for k in range(K):
            assert math.isclose(got[k], ref[k], rel_tol=2e-6), (iters, k, got[k], ref[k])
    # each norm is a lower bound of the order matrix's largest singular value
    for k in range(1, K + 1):
        Rk = ora.reconstruct(k) - (ora.reconstruct(k - 1) if k > 1 else 0.0)
        assert got[k - 1] <= np.linalg.svd(Rk, compute_uv=False)[0] * (1 + 1e-6)   # the GPU rounds s * code to fp32
    norms = [got, got]
    for split in ([K], [1, K - 1], [1] * K):
        assert math.isclose(pipe.pipe_error_bound_U_ens(norms, split), po.error_bound_U_ens(norms, split), rel_tol=1e-12)
    lam = [[0.5 + 0.1 * k for k in range(K)]]
    assert math.isclose(pipe.pipe_error_bound_U_ens(norms, [1, K - 1], lam), po.error_bound_U_ens(norms, [1, K - 1], lam),
                        rel_tol=1e-12)
    for ratio in (0.01, 0.5, 2.0):
        assert pipe.pipe_first_predictor_size(norms, got[0], ratio) == po.first_predictor_size(norms, got[0], ratio)
    g.free()
