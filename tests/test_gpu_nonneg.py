"""GPU parity for the non-negative quantiser (Eq. 6 of arXiv 2310.11453) against the CPU oracle:
eta, gamma, codes and row sums bit-exact given the normalised input the GPU dumped; wsum exact;
Y exact given the same codes (three fp32 operations in the same order on both sides) and within
1e-3 relative end to end."""
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


@pytest.mark.parametrize("M,K", [(1, 32), (7, 96), (33, 512), (100, 2048), (12, 4096), (5, 8192),
                                 (3, 16384), (2, 28672), (3, 36000), (2, 65536)])
@pytest.mark.parametrize("mode", ["ln", "noln", "affine"])
def test_quant_nonneg(bl, M, K, mode):
    print(f"quant nonneg M={M} K={K} {mode}", flush=True)
    X = wl.make_activation(M, K, seed=wl.seed_for(5, K + M), outlier_p=0.01, outlier_mul=6.0)
    X += f32(0.5)
    kw, okw = {}, {}
    if mode == "noln":
        kw["flags"] = bl.FLAG_SKIP_LN
    if mode == "affine":
        rng = np.random.default_rng(K)
        gain = (1 + 0.1 * rng.standard_normal(K)).astype(f32)
        bias = (0.1 * rng.standard_normal(K)).astype(f32)
        kw.update(ln_gain=dev(gain), ln_bias=dev(bias))
        okw.update(gain=gain, bias=bias)
    codes, gamma, eta, rowsum, xhat = bl.bitlinear_quant_act_nonneg(dev(X), want_xhat=True, **kw)
    xh = host(xhat)
    ref_xh = X if mode == "noln" else oracle.layernorm(X, **okw)
    assert np.abs(xh - ref_xh).max() <= 4e-6
    e_ref, g_ref = oracle.minmax_nonneg(xh)
    q_ref = oracle.quantize_nonneg(xh, e_ref, g_ref)
    assert np.array_equal(host(eta), e_ref) and np.array_equal(host(gamma), g_ref)
    assert np.array_equal(host(codes), q_ref)
    assert np.array_equal(host(rowsum), q_ref.astype(np.int32).sum(axis=1))


@pytest.mark.parametrize("N,K", [(512, 256), (17, 544), (2048, 2048), (240, 96)])
def test_weight_rowsums(bl, N, K):
    W = wl.make_weight(N, K, 0.02, seed=wl.seed_for(5, N + K), mean=0.003)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    sign = oracle.binarize(W, host(alpha)[0])
    assert np.array_equal(host(bl.bitlinear_weight_rowsums(packed, N, K)), oracle.weight_rowsum(sign))


@pytest.mark.parametrize("M,K,N", [(1, 256, 512), (8, 2048, 512), (16, 1056, 200), (40, 512, 384),
                                   (100, 2048, 512), (300, 4096, 1024), (70, 96, 240),
                                   (24, 2048, 512), (32, 1056, 201), (17, 8704, 384)])
def test_forward_nonneg(bl, M, K, N):
    print(f"forward nonneg M={M} K={K} N={N}", flush=True)
    X = wl.make_activation(M, K, seed=wl.seed_for(5, M + K + N), outlier_p=0.005, outlier_mul=8.0)
    X += f32(0.25)
    W = wl.make_weight(N, K, 0.02, seed=wl.seed_for(5, M + K + N + 1), mean=0.002)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    wsum = bl.bitlinear_weight_rowsums(packed, N, K)
    y = host(bl.bitlinear_forward_nonneg(dev(X), packed, N, beta, wsum))
    ref = oracle.forward_nonneg(X, W)
    err = np.linalg.norm(y.astype(np.float64) - ref["y"]) / np.linalg.norm(ref["y"])
    assert err <= 1e-3, err
    # given the oracle's own codes the epilogue must reproduce its y bit for bit
    y2 = host(bl.bitlinear_matmul_nonneg(dev(ref["codes"]), dev(ref["gamma"]), dev(ref["eta"]),
                                         dev(ref["codes"].astype(np.int32).sum(axis=1).astype(np.int32)),
                                         packed, N, beta, wsum))
    assert np.array_equal(y2, ref["y"])


def test_nonneg_errors(bl):
    lib = bl.load_library()
    import ctypes
    one = ctypes.c_void_p(256)
    # per-tensor statistics are not offered for Eq. 6
    assert lib.bitlinear_quant_act_nonneg(one, 4, 64, None, None, 1e-5, 1, 0, one, one, one, None,
                                          None, None, 0, None) == -3
    assert lib.bitlinear_quant_act_nonneg(one, 4, 64, None, None, 1e-5, 0, 0, one, one, None, None,
                                          None, None, 0, None) == -1
    assert lib.bitlinear_weight_rowsums(one, 16, 48, one, None) == -2
