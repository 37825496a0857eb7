"""GPU parity of the LayerNorm backward (chain rule through Eq. 12 / Eq. 15 of arXiv
2310.11453 under the straight-through estimator) against the fp64 CPU oracle.

Tolerance: the kernel keeps the statistics and the two row means in fp64 and evaluates
dx = rstd * ((gh - m1) - xn * m2) in fp32: a handful of fp32 roundings on O(1) quantities,
so |dX - oracle| <= 1e-5 * max(1, |dX|) elementwise (observed ~1e-6); column sums for
dgain/dbias are fp64 on both sides: 1e-5 relative.
"""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu
f32 = np.float32


@pytest.fixture(scope="module")
def bl():
    import paper_2310_11453_amd as lib
    lib.load_library()
    assert torch.cuda.is_available()
    return lib


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def close(a, b, tol):
    return np.all(np.abs(a - b) <= tol * np.maximum(1.0, np.abs(b)))


SHAPES = [(1, 32, 1), (5, 96, 1), (33, 256, 1), (100, 2048, 1), (17, 4096, 1), (9, 8192, 1),
          (6, 16384, 1), (40, 1024, 4), (12, 2048, 8), (3, 384, 4),
          # rows longer than the registers hold (the 30B down-projection's K and beyond), walked
          # from memory; also as K-groups
          (5, 28672, 1), (3, 36000, 1), (2, 65536, 1), (4, 57344, 2)]


@pytest.mark.parametrize("M,K,groups", SHAPES)
@pytest.mark.parametrize("affine", [False, True])
def test_ln_backward(bl, M, K, groups, affine):
    print(f"ln backward M={M} K={K} groups={groups} affine={affine}", flush=True)
    X = wl.make_activation(M, K, seed=wl.seed_for(4, K + M), outlier_p=0.01, outlier_mul=6.0)
    X += f32(0.7)
    g = wl.make_grad(M, K, seed=wl.seed_for(4, K + M + 1), std=1.0)
    gain = None
    if affine:
        gain = (1 + 0.1 * np.random.default_rng(K).standard_normal(K)).astype(f32)
    if affine:
        ref_dx, ref_dg, ref_db = oracle.layernorm_backward(g, X, gain=gain, groups=groups,
                                                           want_affine=True)
        dX, dgain, dbias = bl.bitlinear_layernorm_backward(dev(g), dev(X), ln_gain=dev(gain),
                                                           groups_k=groups, want_affine=True)
        scale = max(1.0, float(np.abs(ref_dg).max()))
        assert np.abs(host(dgain) - ref_dg).max() <= 1e-5 * scale
        assert np.abs(host(dbias) - ref_db).max() <= 1e-5 * max(1.0, float(np.abs(ref_db).max()))
    else:
        ref_dx = oracle.layernorm_backward(g, X, groups=groups)
        dX = bl.bitlinear_layernorm_backward(dev(g), dev(X), groups_k=groups)
    assert close(host(dX), ref_dx, 1e-5)


def test_ln_backward_in_place(bl):
    """dX may be written over dXhat, also when the gain/bias gradients are wanted."""
    M, K = 50, 1024
    X = wl.make_activation(M, K, seed=wl.seed_for(4, 900))
    g = wl.make_grad(M, K, seed=wl.seed_for(4, 901), std=1.0)
    gain = (1 + 0.1 * np.random.default_rng(3).standard_normal(K)).astype(f32)
    ref = oracle.layernorm_backward(g, X, gain=gain, want_affine=True)
    buf = dev(g)
    dX, dgain, dbias = bl.bitlinear_layernorm_backward(buf, dev(X), ln_gain=dev(gain),
                                                       want_affine=True, out=buf)
    assert dX.data_ptr() == buf.data_ptr()
    assert close(host(dX), ref[0], 1e-5)
    assert np.abs(host(dgain) - ref[1]).max() <= 1e-4 and np.abs(host(dbias) - ref[2]).max() <= 1e-4


def test_ln_backward_full_training_shape_sampled(bl):
    """M = 8192, K = 4096 (the training configuration): sampled rows against the oracle."""
    M, K = 8192, 4096
    print("ln backward training shape", flush=True)
    X = wl.make_activation(M, K, seed=wl.seed_for(4, 0))
    g = wl.make_grad(M, K, seed=wl.seed_for(4, 1), std=1.0)
    dX = host(bl.bitlinear_layernorm_backward(dev(g), dev(X)))
    rows = np.arange(0, M, 331)
    ref = oracle.layernorm_backward(g[rows], X[rows])
    assert close(dX[rows], ref, 1e-5)


def test_ln_backward_errors(bl):
    lib = bl.load_library()
    assert bl.workspace_bytes_grouped(bl.OP_LN_BACKWARD, 8, 16, 2048, 1, 1) > 0
    with pytest.raises(bl.BitLinearError):  # K/groups not a multiple of 32
        bl.bitlinear_layernorm_backward(dev(np.zeros((1, 48), f32)), dev(np.zeros((1, 48), f32)))
    assert lib.bitlinear_layernorm_backward(None, None, 0, 64, 1, None, 1e-5, None, None, None,
                                            None, 0, None) == 0
