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


# ---- per tensor (the training-time granularity) and per K-group (Eq. 14: eta_g beside gamma_g) ----
# one group per token is test_quant_nonneg above
@pytest.mark.parametrize("M,K,gk,per_tensor", [(7, 96, 1, True), (100, 2048, 1, True), (300, 512, 1, True),
                                               (5, 36000, 1, True), (37, 1024, 4, False), (37, 1024, 4, True),
                                               (9, 2048, 8, False), (9, 2048, 8, True), (3, 384, 4, False),
                                               (3, 384, 4, True)])
@pytest.mark.parametrize("mode", ["ln", "noln", "affine"])
def test_quant_nonneg_per_tensor_and_groups(bl, M, K, gk, mode, per_tensor):
    print(f"quant nonneg M={M} K={K} gk={gk} {mode} per_tensor={per_tensor}", flush=True)
    X = wl.make_activation(M, K, seed=wl.seed_for(5, K + M + gk), outlier_p=0.01, outlier_mul=6.0)
    X += f32(0.5)
    X[:, : K // 4] += f32(1.5)
    kw, okw = {}, {}
    if mode == "noln":
        kw["flags"] = bl.FLAG_SKIP_LN
    if mode == "affine":
        rng = np.random.default_rng(K)
        gain = (1 + 0.1 * rng.standard_normal(K)).astype(f32)
        bias = (0.1 * rng.standard_normal(K)).astype(f32)
        kw.update(ln_gain=dev(gain), ln_bias=dev(bias))
        okw.update(gain=gain, bias=bias)
    codes, gamma, eta, rowsum, xhat = bl.bitlinear_quant_act_nonneg(dev(X), want_xhat=True,
                                                                    per_tensor=per_tensor, groups_k=gk, **kw)
    xh = host(xhat)
    ref_xh = X if mode == "noln" else oracle.layernorm(X, groups=gk, **okw)
    assert np.abs(xh - ref_xh).max() <= 4e-6 * max(1.0, np.abs(ref_xh).max())
    Kg = K // gk
    g_gpu = host(gamma).reshape(-1, gk)
    e_gpu = host(eta).reshape(-1, gk)
    rs_gpu = host(rowsum).reshape(M, gk)
    for g in range(gk):  # each K-slice against the plain oracle functions on that slice
        xs = np.ascontiguousarray(xh[:, g * Kg:(g + 1) * Kg])
        e_ref, g_ref = oracle.minmax_nonneg(xs, per_tensor)
        q_ref = oracle.quantize_nonneg(xs, e_ref, g_ref, per_tensor)
        assert np.array_equal(e_gpu[:, g], e_ref) and np.array_equal(g_gpu[:, g], g_ref)
        assert np.array_equal(host(codes)[:, g * Kg:(g + 1) * Kg], q_ref)
        assert np.array_equal(rs_gpu[:, g], q_ref.astype(np.int32).sum(axis=1))


@pytest.mark.parametrize("M", [1, 8, 24, 48, 100])
@pytest.mark.parametrize("gn,gk,per_tensor", [(1, 1, True), (1, 4, False), (2, 2, True), (4, 4, False),
                                              (8, 1, True), (1, 8, True)])
def test_forward_nonneg_per_tensor_and_groups(bl, M, gn, gk, per_tensor):
    """Every GEMM kernel's epilogue (1, up to 16, 17-32, 33-64 tokens, large tiles) with a
    per-tensor eta and with eta_g per K-group."""
    K, N = 2048, 512
    print(f"forward nonneg M={M} gn={gn} gk={gk} per_tensor={per_tensor}", flush=True)
    X = wl.make_activation(M, K, seed=wl.seed_for(5, 700 + M + gn + gk), outlier_p=0.005, outlier_mul=8.0)
    X += f32(0.25)
    X[:, K // 2:] *= f32(1.7)
    W = wl.make_weight(N, K, 0.02, seed=wl.seed_for(5, 800 + gn + gk), mean=0.002)
    W[: N // 2] += f32(0.01)
    packed, alpha, beta = bl.bitlinear_pack_weights_grouped(dev(W), gn, gk)
    wsum = bl.bitlinear_weight_rowsums_grouped(packed, N, K, gk)
    y = host(bl.bitlinear_forward_nonneg(dev(X), packed, N, beta, wsum, per_tensor=per_tensor,
                                         groups_n=gn, groups_k=gk))
    ref = oracle.forward_grouped_nonneg(X, W, gn, gk, per_tensor=per_tensor)
    assert np.array_equal(host(wsum), ref["wsum"])
    assert np.array_equal(host(beta), ref["beta"])
    err = np.linalg.norm(y.astype(np.float64) - ref["y64"]) / np.linalg.norm(ref["y64"])
    assert err <= 1e-3, err
    # given the normalised input the GPU itself rounded: codes, eta_g, gamma_g exactly, and Y up to
    # the fp32 order of the group sums (exactly with one K-group)
    codes, gamma, eta, rowsum, xhat = bl.bitlinear_quant_act_nonneg(dev(X), want_xhat=True,
                                                                    per_tensor=per_tensor, groups_k=gk)
    given = oracle.forward_grouped_nonneg(X, W, gn, gk, per_tensor=per_tensor, xhat=host(xhat))
    assert np.array_equal(host(codes), given["codes"])
    assert np.array_equal(host(eta).reshape(-1, gk), given["eta"])
    assert np.array_equal(host(gamma).reshape(-1, gk), given["gamma"])
    err = np.linalg.norm(y.astype(np.float64) - given["y64"]) / np.linalg.norm(given["y64"])
    assert err <= 1e-5, err
    if gk == 1:
        assert np.array_equal(y, given["y"])


def test_nonneg_errors(bl):
    lib = bl.load_library()
    import ctypes
    one = ctypes.c_void_p(256)
    # a per-tensor eta needs the quantiser's workspace
    assert lib.bitlinear_quant_act_nonneg(one, 4, 64, None, None, 1e-5, 1, 0, one, one, one, None,
                                          None, None, 0, None) == -4
    assert lib.bitlinear_quant_act_nonneg(one, 4, 64, None, None, 1e-5, 7, 0, one, one, one, None,
                                          None, None, 0, None) == -3
    assert lib.bitlinear_quant_act_nonneg(one, 4, 64, None, None, 1e-5, 0, 0, one, one, None, None,
                                          None, None, 0, None) == -1
    assert lib.bitlinear_weight_rowsums(one, 16, 48, one, None) == -2
    assert lib.bitlinear_weight_rowsums_grouped(one, 16, 96, 2, one, None) == -2
    assert lib.bitlinear_forward_grouped_nonneg(one, 4, 2048, one, 512, 2, 4, one, None, None, None,
                                                1e-5, 0, 0, one, one, 1 << 20, None) == -1
