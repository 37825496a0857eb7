"""GPU parity for Group Quantization and Normalization (Eq. 13-15 of arXiv 2310.11453):
the grouped entry points of the C ABI against the grouped CPU oracle.

Bits, alpha_g and beta_g: exact.  Codes: bit-exact given the normalised input the GPU dumped;
x^ against the oracle's fp64 group LayerNorm.  Output: the oracle adds the K-group terms in
fp64, the GPU in fp32 in the order g = 0, 1, ...: relative Frobenius error <= 1e-5 (a few
fp32 roundings) given the normalised input the GPU dumped, far inside the 1e-3 of the plain
layer that also holds end to end; with groups_k = 1 it is exact.
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


def layer(M, K, N, seed):
    W = wl.make_weight(N, K, 0.02, seed=wl.seed_for(0, seed))
    W[: N // 2] += f32(0.01)          # row groups with different means
    W[:, K // 2:] *= f32(1.5)         # column groups with different scales
    X = wl.make_activation(M, K, seed=wl.seed_for(0, seed + 1), outlier_p=0.01, outlier_mul=8.0)
    X[:, : K // 4] += f32(2.0)        # K-slices of a token with different statistics
    return X, W


GROUPS = [(1, 1), (2, 1), (1, 2), (4, 4), (8, 8), (1, 8), (8, 1)]


@pytest.mark.parametrize("gn,gk", GROUPS)
def test_grouped_pack(bl, gn, gk):
    """Eq. 13: per-block alpha, beta and bits."""
    N, K = 512, 2048
    print(f"grouped pack N={N} K={K} gn={gn} gk={gk}", flush=True)
    _, W = layer(1, K, N, 100 + gn * 10 + gk)
    a, b = oracle.weight_stats_grouped(W, gn, gk)
    words = oracle.pack_canonical(oracle.binarize_grouped(W, a))
    packed, alpha, beta = bl.bitlinear_pack_weights_grouped(dev(W), gn, gk)
    assert np.array_equal(host(alpha), a) and np.array_equal(host(beta), b)
    canon = host(bl.bitlinear_packed_to_canonical_grouped(packed, N, K, gk)).view(np.uint32)
    assert np.array_equal(canon, words)


@pytest.mark.parametrize("per_tensor", [False, True])
@pytest.mark.parametrize("gk", [2, 4, 8])
def test_grouped_quant(bl, gk, per_tensor):
    """Eq. 14-15: group LayerNorm and gamma per slice of a token."""
    M, K = 37, 1024
    print(f"grouped quant M={M} K={K} gk={gk} per_tensor={per_tensor}", flush=True)
    X, _ = layer(M, K, 16, 200 + gk)
    codes, gamma, rowsum, xhat = bl.bitlinear_quant_act_grouped(dev(X), gk, per_tensor=per_tensor,
                                                                want_xhat=True)
    xh = host(xhat)
    ref_xh = oracle.layernorm(X, groups=gk)
    assert np.abs(xh - ref_xh).max() <= 2e-6
    g_ref = oracle.absmax(xh, per_tensor, groups=gk)
    q_ref = oracle.quantize(xh, g_ref, per_tensor, groups=gk)
    assert np.array_equal(host(gamma).reshape(-1), g_ref.reshape(-1))
    assert np.array_equal(host(codes), q_ref)
    rs_ref = q_ref.astype(np.int32).reshape(M, gk, K // gk).sum(axis=2)
    assert np.array_equal(host(rowsum), rs_ref)


def _check_forward(bl, M, K, N, gn, gk, per_tensor, seed):
    X, W = layer(M, K, N, seed)
    packed, alpha, beta = bl.bitlinear_pack_weights_grouped(dev(W), gn, gk)
    y = host(bl.bitlinear_forward_grouped(dev(X), packed, N, beta, gn, gk, per_tensor=per_tensor))
    ref = oracle.forward_grouped(X, W, gn, gk, per_tensor=per_tensor)
    assert np.array_equal(host(beta), ref["beta"])
    # end to end from raw X: the GPU's x^ may differ from the oracle's in the last bit of fp32
    # (fp64 statistics summed in another order), which moves a code only at an exact tie
    err = np.linalg.norm(y.astype(np.float64) - ref["y64"]) / np.linalg.norm(ref["y64"])
    assert err <= 1e-3, err
    # given the normalised input the GPU itself rounded: gamma_g, codes and row sums exactly, and
    # then the only difference left in Y is the fp32 order of the group sums (the oracle adds the
    # slices in fp64): 1e-5, and nothing at all with one K-group
    codes, gamma, rowsum, xhat = bl.bitlinear_quant_act_grouped(dev(X), gk, per_tensor=per_tensor,
                                                                want_xhat=True)
    given = oracle.forward_grouped(X, W, gn, gk, per_tensor=per_tensor, xhat=host(xhat))
    assert np.array_equal(host(codes), given["codes"])
    assert np.array_equal(host(gamma).reshape(-1), np.asarray(given["gamma"]).reshape(-1))
    err = np.linalg.norm(y.astype(np.float64) - given["y64"]) / np.linalg.norm(given["y64"])
    assert err <= 1e-5, err
    if gk == 1:
        assert np.array_equal(y, given["y"])
    return err


@pytest.mark.parametrize("gn,gk", GROUPS)
@pytest.mark.parametrize("M", [8, 24, 48, 100])
def test_grouped_forward(bl, M, gn, gk):
    """One batch size for each of the four GEMM kernels (up to 16, 17-32, 33-64 tokens, large
    tiles), per-token gamma."""
    K, N = 2048, 512
    print(f"grouped forward M={M} K={K} N={N} gn={gn} gk={gk}", flush=True)
    _check_forward(bl, M, K, N, gn, gk, False, 300 + gn * 10 + gk)


@pytest.mark.parametrize("M", [4, 300])
def test_grouped_forward_per_tensor(bl, M):
    print(f"grouped forward per-tensor M={M}", flush=True)
    _check_forward(bl, M, 1024, 256, 4, 4, True, 400 + M)


def test_grouped_forward_ragged(bl):
    """Shapes that are not multiples of the kernels' tiles: N = 3 * 80, K = 4 * 96."""
    print("grouped forward ragged", flush=True)
    _check_forward(bl, 70, 384, 240, 3, 4, False, 500)
    _check_forward(bl, 5, 384, 240, 3, 4, False, 501)
    _check_forward(bl, 19, 384, 240, 3, 4, False, 502)
    _check_forward(bl, 33, 384, 240, 3, 4, False, 503)


@pytest.mark.parametrize("M,K,N,gn,gk", [(5, 16384, 256, 1, 8),   # 16 waves of two chunks
                                         (9, 6144, 256, 2, 4),    # 12 waves of one chunk
                                         (3, 32768, 128, 1, 8),   # too many chunks for one workgroup
                                         (40, 8192, 384, 1, 2),   # 33-64 tokens, long K-groups
                                         (64, 3072, 256, 2, 6)])  # 33-64 tokens, six groups in two items
def test_grouped_forward_group_placement(bl, tuning, M, K, N, gn, gk):
    """Up to 64 tokens the K-groups share workgroups where they fit (waves dealt to the groups in
    the small-batch kernel, one K-group of the workgroup per layer group in the mid-batch one) and
    are work items of their own otherwise; both placements give the same bits."""
    print(f"grouped placement M={M} K={K} N={N} gn={gn} gk={gk}", flush=True)
    _check_forward(bl, M, K, N, gn, gk, False, 600 + M)
    X, W = layer(M, K, N, 600 + M)
    packed, alpha, beta = bl.bitlinear_pack_weights_grouped(dev(W), gn, gk)
    y0 = host(bl.bitlinear_forward_grouped(dev(X), packed, N, beta, gn, gk))
    tuning("group_slices=1")
    y1 = host(bl.bitlinear_forward_grouped(dev(X), packed, N, beta, gn, gk))
    assert np.array_equal(y0, y1)


def test_grouped_forward_full_size_30b(bl):
    """A 30B-shaped layer (7168 -> 28672) with eight groups on each axis, decode and prefill batch:
    alpha_g, beta_g and all bits; codes and gamma_g given the normalised input the GPU dumped;
    outputs on a stratified sample against the oracle's per-group sums."""
    K, N, G = 7168, 28672, 8
    W = wl.make_weight(N, K, 0.01, seed=wl.seed_for(3, 40))
    W[: N // 2] += f32(0.003)
    a, b = oracle.weight_stats_grouped(W, G, G)
    sign = oracle.binarize_grouped(W, a)
    packed, alpha, beta = bl.bitlinear_pack_weights_grouped(dev(W), G, G)
    del W
    assert np.array_equal(host(alpha), a) and np.array_equal(host(beta), b)
    canon = host(bl.bitlinear_packed_to_canonical_grouped(packed, N, K, G)).view(np.uint32)
    assert np.array_equal(canon, oracle.pack_canonical(sign))
    del canon
    Kg, Ng = K // G, N // G
    for M in (16, 300):
        print(f"grouped full size M={M}", flush=True)
        X = wl.make_activation(M, K, seed=wl.seed_for(3, 41 + M))
        X[:, : K // 4] += f32(1.0)
        y = host(bl.bitlinear_forward_grouped(dev(X), packed, N, beta, G, G))
        codes, gamma, rowsum, xhat = bl.bitlinear_quant_act_grouped(dev(X), G, want_xhat=True)
        xh = host(xhat)
        g_ref = oracle.absmax(xh, False, groups=G)
        q_ref = oracle.quantize(xh, g_ref, False, groups=G)
        assert np.array_equal(host(gamma).reshape(-1), g_ref) and np.array_equal(host(codes), q_ref)
        rng = np.random.default_rng(M)
        gm, gn = (M + 63) // 64, N // 64
        rows = np.minimum((np.arange(gm) * 64)[:, None] + rng.integers(0, 64, (gm, gn)), M - 1).ravel()
        cols = ((np.arange(gn) * 64)[None, :] + rng.integers(0, 64, (gm, gn))).ravel()
        gam = g_ref.reshape(M, G)
        ysum = np.zeros(rows.size)
        for g in range(G):  # each K-group dequantised with its own beta_g gamma_g, added in fp64
            acc = oracle.matmul_i32_sampled(np.ascontiguousarray(q_ref[:, g * Kg:(g + 1) * Kg]),
                                            np.ascontiguousarray(sign[:, g * Kg:(g + 1) * Kg]), rows, cols)
            sc = (b[cols // Ng, g] * gam[rows, g]) / f32(128.0)
            ysum += (acc.astype(f32) * sc).astype(np.float64)
        got = y[rows, cols].astype(np.float64)
        assert np.abs(got - ysum).max() <= 1e-5 * np.sqrt(np.mean(ysum ** 2))


def test_groups_of_one_match_the_plain_entry_points(bl):
    M, K, N = 50, 512, 256
    X, W = layer(M, K, N, 600)
    p0, a0, b0 = bl.bitlinear_pack_weights(dev(W))
    p1, a1, b1 = bl.bitlinear_pack_weights_grouped(dev(W), 1, 1)
    assert torch.equal(p0, p1) and torch.equal(a0, a1.reshape(-1)) and torch.equal(b0, b1.reshape(-1))
    y0 = bl.bitlinear_forward(dev(X), p0, N, b0)
    y1 = bl.bitlinear_forward_grouped(dev(X), p1, N, b1, 1, 1)
    assert torch.equal(y0, y1)


def test_grouped_argument_errors(bl):
    lib = bl.load_library()
    # groups that do not divide, or K-groups that are not multiples of 32: bad shape
    assert lib.bitlinear_packed_bytes_grouped(512, 2048, 3, 1) == 0
    assert lib.bitlinear_packed_bytes_grouped(512, 96, 1, 2) == 0
    # row groups that are not whole 16-row tiles: unsupported
    assert lib.bitlinear_packed_bytes_grouped(96, 64, 4, 1) == 0
    assert lib.bitlinear_packed_bytes_grouped(512, 2048, 8, 8) == 8 * (512 // 16) * 1024
    with pytest.raises(bl.BitLinearError):
        bl.bitlinear_pack_weights_grouped(dev(np.zeros((96, 64), f32)), 4, 1)
