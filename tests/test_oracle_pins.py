"""Pins the CPU oracle to things other than itself (no GPU needed).

Each test names the passage of the paper (arXiv 2310.11453) it checks against.
A plausible mistake in the oracle (dropped term, wrong sign or index, transposed
operand, wrong rounding mode) is meant to fail at least one test here.
"""
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

f32 = np.float32
GOLDEN = Path(__file__).parent / "golden" / "worked_example_n3k4m2.txt"


def _load_golden():
    d = {}
    for line in GOLDEN.read_text().splitlines():
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        d[key] = np.array([float(v) for v in vals])
    return d


# ---------------------------------------------------------------- worked example
@pytest.mark.parametrize("tag,skip_ln", [("noln", True), ("ln", False)])
def test_worked_example_eq1_to_eq12(tag, skip_ln):
    """Exact-rational derivation of Eq. 1-5, 7, 11, 12 on a 3x4 weight, 2 tokens."""
    g = _load_golden()
    W = g["W"].reshape(3, 4).astype(f32)
    X = g["X"].reshape(2, 4).astype(f32)
    r = oracle.forward(X, W, eps=float(g["eps"][0]), skip_ln=skip_ln)
    assert r["alpha"] == f32(g["alpha"][0])
    assert r["beta"] == f32(g["beta"][0])
    assert np.array_equal(r["sign"].ravel(), g["sign"].astype(np.int8))
    assert np.array_equal(r["words"].ravel(), g["words"].astype(np.uint32))
    assert np.array_equal(r["xhat"].ravel(), g[f"{tag}.xhat"].astype(f32))
    assert np.array_equal(r["gamma"], g[f"{tag}.gamma"].astype(f32))
    assert np.array_equal(r["codes"].ravel(), g[f"{tag}.codes"].astype(np.int8))
    assert np.array_equal(r["acc"].ravel(), g[f"{tag}.acc"].astype(np.int32))
    assert np.array_equal(r["y"].ravel(), g[f"{tag}.y"].astype(f32))


# ---------------------------------------------------------------- Eq. 4: rounding and clip
def test_quant_ties_and_clip_eq4():
    """gamma = 1 so t = 128 x exactly: ties go to even, +max clips to 127, -max hits -128."""
    row = np.array([[1, 1 / 256, 3 / 256, 5 / 256, -1 / 256, -3 / 256, -1, 127.5 / 128]], f32)
    gamma = oracle.absmax(row)
    assert gamma[0] == 1.0
    q = oracle.quantize(row, gamma)
    assert q.tolist() == [[127, 0, 2, 2, 0, -2, -128, 127]]


def test_quant_matches_python_rationals_eq4_eq5():
    """Independent re-derivation: fp32 division and multiply from numpy scalars, rounding
    with exact Fractions, on random rows including per-tensor granularity."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((5, 48)).astype(f32) * f32(3.0)
    for per_tensor in (False, True):
        gamma = oracle.absmax(x, per_tensor)
        q = oracle.quantize(x, gamma, per_tensor)
        for m in range(x.shape[0]):
            g = np.abs(x).max() if per_tensor else np.abs(x[m]).max()
            assert (gamma[0] if per_tensor else gamma[m]) == g
            scale = f32(128.0) / f32(g)
            for k in range(x.shape[1]):
                t = x[m, k] * scale
                e = max(-128, min(127, round(Fraction(float(t)))))
                assert q[m, k] == e


def test_code_range_and_argmax_code():
    """Codes lie in [-Q_b, Q_b-1]; the absmax element maps to 127 (positive) or -128."""
    x = wl.make_activation(64, 256, seed=3)
    xh = oracle.layernorm(x)
    gamma = oracle.absmax(xh)
    q = oracle.quantize(xh, gamma)
    assert q.min() >= -128 and q.max() <= 127
    for m in range(64):
        j = int(np.argmax(np.abs(xh[m])))
        assert q[m, j] == (127 if xh[m, j] > 0 else -128)


def test_power_of_two_equivariance():
    """Scaling by 2^j is exact in binary floating point: codes and bits do not change,
    gamma and beta scale by exactly 2^j."""
    x = wl.make_activation(4, 96, seed=11)
    W = wl.make_weight(8, 96, 0.02, seed=12)
    g1 = oracle.absmax(x)
    q1 = oracle.quantize(x, g1)
    a1, b1 = oracle.weight_stats(W)
    for j in (-3, 5):
        s = f32(2.0 ** j)
        g2 = oracle.absmax(x * s)
        assert np.array_equal(g2, g1 * s)
        assert np.array_equal(oracle.quantize(x * s, g2), q1)
        a2, b2 = oracle.weight_stats(W * s)
        assert a2 == a1 * s and b2 == b1 * s
        assert np.array_equal(oracle.binarize(W * s, a2), oracle.binarize(W, a1))


def test_zero_row_gamma_floor():
    """A constant input row normalises to zero: gamma is floored, codes and y are 0."""
    X = np.ones((2, 64), f32) * f32(3.25)
    X[1] = wl.make_activation(1, 64, seed=1)[0]
    W = wl.make_weight(16, 64, 0.02, seed=2)
    r = oracle.forward(X, W)
    assert r["gamma"][0] == f32(1e-5)
    assert not r["codes"][0].any() and not r["y"][0].any()
    assert np.isfinite(r["y"]).all()


# ---------------------------------------------------------------- Eq. 1-3, 12: weights
def test_sign_of_zero_is_minus_one_eq2():
    """W constant: W - alpha = 0 everywhere, Sign(0) = -1, so no bit is set and
    y[m,n] = -(beta gamma_m/128) sum_k q[m,k]."""
    W = np.full((8, 64), 0.03125, f32)
    X = wl.make_activation(3, 64, seed=4)
    r = oracle.forward(X, W)
    assert r["alpha"] == f32(0.03125) and r["beta"] == f32(0.03125)
    assert (r["sign"] == -1).all() and not r["words"].any()
    rowsum = r["codes"].astype(np.int64).sum(1)
    assert np.array_equal(r["acc"], np.repeat(-rowsum[:, None], 8, 1))


def test_alpha_beta_against_exact_rationals_eq3_eq12():
    rng = np.random.default_rng(9)
    W = (rng.standard_normal((7, 40)) * 0.02 + 0.04).astype(f32)
    fr = [Fraction(float(v)) for v in W.ravel()]
    alpha = f32(float(sum(fr) / len(fr)))
    beta = f32(float(sum(abs(v) for v in fr) / len(fr)))
    beta_c = f32(float(sum(abs(v - Fraction(float(alpha))) for v in fr) / len(fr)))
    a, b = oracle.weight_stats(W)
    assert a == alpha and b == beta
    a2, b2 = oracle.weight_stats(W, beta_centered=True)
    assert a2 == alpha and b2 == beta_c
    # with a mean of 2 sigma the two readings of beta are far apart
    assert abs(float(b) - float(b2)) > 0.3 * float(b2)


def test_centred_weights_have_zero_mean_and_beta_minimises_l2():
    """Pre-sign input W - alpha has zero mean; among all c, ||(W-a) - c sign(W-a)||_2 is
    least at c = mean|W - a| (the purpose the text above Eq. 1 gives for beta)."""
    W = wl.make_weight(64, 128, 0.02, seed=21, mean=0.01)
    a, bc = oracle.weight_stats(W, beta_centered=True)
    Wc = W.astype(np.float64) - float(a)
    assert abs(Wc.mean()) <= 4 * np.finfo(f32).eps * np.abs(W).max()
    s = oracle.binarize(W, a).astype(np.float64)
    assert np.array_equal(s, np.where(Wc > 0, 1.0, -1.0))
    err = lambda c: np.sum((Wc - c * s) ** 2)
    c0 = float(bc)
    assert err(c0) <= err(c0 * 1.01) and err(c0) <= err(c0 * 0.99)
    assert abs(c0 - np.sum(Wc * s) / s.size) < 1e-8  # closed-form least squares


def test_beta_closed_form_gaussian():
    """W ~ N(0, sigma^2): mean|W| -> sigma sqrt(2/pi); bits are balanced."""
    W = wl.make_weight(512, 1024, 0.02, seed=31)
    a, b = oracle.weight_stats(W)
    assert abs(float(b) / (0.02 * np.sqrt(2 / np.pi)) - 1) < 5e-3
    pop = int((oracle.binarize(W, a) > 0).sum())
    assert abs(pop - W.size / 2) < 3 * np.sqrt(W.size) / 2 + 1


def test_pack_canonical_bit_order_and_ragged_tail():
    sign = -np.ones((2, 40), np.int8)
    sign[0, 0] = 1
    sign[0, 33] = 1
    sign[1, 31] = 1
    sign[1, 39] = 1
    words = oracle.pack_canonical(sign)
    assert words.tolist() == [[1, 2], [1 << 31, 1 << 7]]
    assert np.array_equal(oracle.unpack_canonical(words, 40), sign)
    rng = np.random.default_rng(1)
    s = np.where(rng.random((5, 96)) < 0.5, 1, -1).astype(np.int8)
    w = oracle.pack_canonical(s)
    bits = np.unpackbits(w.view(np.uint8), axis=1, bitorder="little")[:, :96]
    assert np.array_equal(bits.astype(np.int8) * 2 - 1, s)


# ---------------------------------------------------------------- Eq. 12 / 15: LayerNorm
def test_layernorm_against_torch_and_moments():
    x = wl.make_activation(16, 320, seed=41) * f32(2.5) + f32(0.7)
    xh = oracle.layernorm(x, 1e-5)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (320,), eps=1e-5).numpy()
    assert np.abs(xh - ref).max() <= 1e-6
    x64 = x.astype(np.float64)
    var = x64.var(axis=1)
    assert np.abs(xh.astype(np.float64).mean(1)).max() < 1e-7
    assert np.allclose((xh.astype(np.float64) ** 2).mean(1), var / (var + 1e-5), atol=1e-6)
    gain = np.linspace(0.5, 1.5, 320).astype(f32)
    bias = np.linspace(-1, 1, 320).astype(f32)
    ref_aff = torch.nn.functional.layer_norm(torch.from_numpy(x).double(), (320,),
                                             torch.from_numpy(gain).double(),
                                             torch.from_numpy(bias).double(), 1e-5).numpy()
    assert np.abs(oracle.layernorm(x, 1e-5, gain, bias) - ref_aff).max() <= 2e-6


def test_group_layernorm_equals_groupnorm_eq15():
    """Group normalisation over G slices of the feature axis (Eq. 15)."""
    x = wl.make_activation(6, 256, seed=43) + f32(0.3)
    G = 4
    xh = oracle.layernorm(x, 1e-5, groups=G)
    ref = torch.nn.functional.group_norm(torch.from_numpy(x).double(), G, eps=1e-5).numpy()
    assert np.abs(xh - ref).max() <= 1e-6
    g = oracle.absmax(xh, groups=G)
    assert np.array_equal(g.reshape(6, G), np.abs(xh).reshape(6, G, 64).max(2))


# ---------------------------------------------------------------- Eq. 7: integer matmul
def test_matmul_against_numpy_int64_eq7():
    rng = np.random.default_rng(51)
    q = rng.integers(-128, 128, (9, 160), dtype=np.int8)
    s = np.where(rng.random((13, 160)) < 0.5, 1, -1).astype(np.int8)
    acc = oracle.matmul_i32(q, s)
    ref = q.astype(np.int64) @ s.astype(np.int64).T
    assert np.array_equal(acc, ref)
    # identities: parity, bit-count form, magnitude bound
    rs = q.astype(np.int64).sum(1, keepdims=True)
    assert np.array_equal((acc - rs) % 2, np.zeros_like(acc))
    pos = q.astype(np.int64) @ (s > 0).astype(np.int64).T
    assert np.array_equal(acc, 2 * pos - rs)
    assert np.abs(acc).max() <= 128 * 160
    rows = np.array([0, 8, 3]); cols = np.array([12, 0, 5])
    assert np.array_equal(oracle.matmul_i32_sampled(q, s, rows, cols), ref[rows, cols])
    assert np.array_equal(oracle.matmul_i32(q, s, 32, 96),
                          q[:, 32:96].astype(np.int64) @ s[:, 32:96].astype(np.int64).T)


def test_matmul_extreme_codes_no_overflow():
    K = 28672
    q = np.full((1, K), -128, np.int8)
    s = -np.ones((2, K), np.int8)
    s[1] = 1
    assert oracle.matmul_i32(q, s).tolist() == [[128 * K, -128 * K]]


# ---------------------------------------------------------------- Eq. 11: the whole layer
def test_dequant_counts_only_scale_multiplies_eq11_eq18():
    acc = np.array([[3, -5], [7, 11]], np.int32)
    gamma = np.array([2.0, 0.5], f32)
    y = oracle.dequant(acc, gamma, f32(0.25))
    assert np.array_equal(y, np.array([[3 * 0.25 * 2 / 128, -5 * 0.25 * 2 / 128],
                                       [7 * 0.25 * .5 / 128, 11 * 0.25 * .5 / 128]], f32))
    y_t = oracle.dequant(acc, gamma[:1], f32(0.25), per_tensor=True)
    assert np.array_equal(y_t, (acc * (0.25 * 2 / 128)).astype(f32))


@pytest.mark.parametrize("per_tensor", [False, True])
def test_forward_within_quantisation_bound_of_float_layer(per_tensor):
    """BitLinear output vs LN(x) @ (beta sign(W - alpha))^T in fp64: the only error is the
    activation rounding, |e_k| <= gamma/256 (gamma/128 for the clipped maximum)."""
    c = wl.CONFIGS[0]
    L = c.layers[0]
    W = wl.make_weight(L.N, L.K, c.w_std, wl.seed_for(0))
    X = wl.make_activation(8, L.K, wl.seed_for(0))
    r = oracle.forward(X, W, per_tensor=per_tensor)
    gamma = np.broadcast_to(r["gamma"].astype(np.float64), (8,)) if per_tensor else r["gamma"]
    y_fp = r["xhat"].astype(np.float64) @ (float(r["beta"]) * r["sign"].astype(np.float64)).T
    bound = float(r["beta"]) * np.asarray(gamma, np.float64)[:, None] * (L.K + 1) / 256.0
    assert (np.abs(r["y"] - y_fp) <= bound + 1e-6).all()
    # typical error is far below the worst case: rms ~ beta gamma/256 sqrt(K/3)
    rms = np.sqrt(np.mean((r["y"] - y_fp) ** 2))
    expect = float(r["beta"]) * float(np.mean(gamma)) / 256 * np.sqrt(L.K / 3)
    assert 0.5 * expect < rms < 2 * expect


def test_output_variance_eq8_to_eq10():
    """With LN the normalised input has unit variance, so Var(y) ~ K beta^2."""
    W = wl.make_weight(512, 1024, 0.02, seed=61)
    X = wl.make_activation(64, 1024, seed=62)
    r = oracle.forward(X, W)
    assert abs(r["y"].var() / (1024 * float(r["beta"]) ** 2) - 1) < 0.1


def test_transposed_or_swapped_operands_would_fail():
    """Non-square shapes with a planted asymmetric weight: only y = x~ W~^T fits."""
    W = np.full((4, 32), -0.01, f32)
    W[2, :] = 0.05                      # output column 2 is all +1
    X = np.zeros((2, 32), f32)
    X[0, :16] = 1.0
    X[1, 16:] = -2.0
    r = oracle.forward(X, W, skip_ln=True)
    assert r["acc"][0].tolist() == [-16 * 127, -16 * 127, 16 * 127, -16 * 127]
    assert r["acc"][1].tolist() == [16 * 128, 16 * 128, -16 * 128, 16 * 128]


# ---------------------------------------------------------------- Section 2.2: STE backward
def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(71)
    v = (rng.standard_normal(4096) * 1e-3).astype(f32)
    v[:4] = [1.00390625, 1.01171875, -1.00390625, 3.0e-41]  # two exact ties, a subnormal
    ref = torch.from_numpy(v).to(torch.bfloat16).float().numpy()
    assert np.array_equal(oracle.round_bf16(v), ref)


@pytest.mark.parametrize("per_tensor", [True, False])
def test_backward_ste_against_numpy_fp64(per_tensor):
    """dX^ = beta g S and dW = g^T (q gamma/128): plain fp64 matmuls of bf16-rounded dY."""
    M, N, K = 12, 20, 64
    W = wl.make_weight(N, K, 0.02, seed=81)
    X = wl.make_activation(M, K, seed=82)
    dY = wl.make_grad(M, N, seed=83)
    r = oracle.forward(X, W, per_tensor=per_tensor)
    dX, dW = oracle.backward_ste(dY, r["codes"], r["gamma"], r["sign"], r["beta"], per_tensor)
    S = r["sign"].astype(np.float64)
    q = r["codes"].astype(np.float64)
    if per_tensor:
        g = torch.from_numpy(dY).to(torch.bfloat16).double().numpy()
        dW_ref = (g.T @ q) * float(r["gamma"][0] / f32(128))
    else:
        sc = (r["gamma"] / f32(128)).astype(f32)
        g_w = torch.from_numpy(dY * sc[:, None]).to(torch.bfloat16).double().numpy()
        dW_ref = g_w.T @ q
        g = torch.from_numpy(dY).to(torch.bfloat16).double().numpy()
    dX_ref = float(r["beta"]) * (g @ S)
    assert np.allclose(dX, dX_ref, rtol=1e-6, atol=1e-12)
    assert np.allclose(dW, dW_ref, rtol=1e-6, atol=1e-12)
    rows = np.array([3, 0, 11])
    dXs, _ = oracle.backward_ste(dY, r["codes"], r["gamma"], r["sign"], r["beta"], per_tensor,
                                 rows_dx=rows, want_dw=False)
    assert np.array_equal(dXs, dX[rows])
    _, dWs = oracle.backward_ste(dY, r["codes"], r["gamma"], r["sign"], r["beta"], per_tensor,
                                 rows_dw=rows, want_dx=False)
    assert np.array_equal(dWs, dW[rows])


def test_backward_is_gradient_of_the_ste_surrogate():
    """Finite differences of the surrogate y = x^ (beta S)^T (Sign, Clip, rounding treated as
    identity): d<dY,y>/dx^ = dY beta S, d<dY,y>/dW~ = dY^T x^ with x^ ~ q gamma/128."""
    M, N, K = 3, 5, 32
    W = wl.make_weight(N, K, 0.02, seed=91)
    X = wl.make_activation(M, K, seed=92)
    r = oracle.forward(X, W, per_tensor=True)
    # choose dY exactly representable in bf16 so rounding plays no role
    dY = (np.round(wl.make_grad(M, N, seed=93) * 1e3 * 8) / 8).astype(f32)
    dX, dW = oracle.backward_ste(dY, r["codes"], r["gamma"], r["sign"], r["beta"], True)
    S = r["sign"].astype(np.float64)
    xq = r["codes"].astype(np.float64) * float(r["gamma"][0]) / 128.0
    loss = lambda xh, Wt: np.sum(dY.astype(np.float64) * (xh @ Wt.T))
    h = 1e-3
    for (m, k) in [(0, 0), (2, 17)]:
        e = np.zeros((M, K)); e[m, k] = h
        fd = (loss(xq + e, float(r["beta"]) * S) - loss(xq - e, float(r["beta"]) * S)) / (2 * h)
        assert abs(fd - dX[m, k]) <= 1e-6 * max(1, abs(fd))
    for (n, k) in [(1, 3), (4, 31)]:
        e = np.zeros((N, K)); e[n, k] = h
        fd = (loss(xq, S + e) - loss(xq, S - e)) / (2 * h)
        assert abs(fd - dW[n, k]) <= 1e-6 * max(1, abs(fd))


# ---------------------------------------------------------------- Eq. 13-15: groups
def _rand_layer(seed, M, K, N, w_mean=0.0):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(f32)
    X[:, : K // 2] += f32(1.5)  # the two halves of a token have different statistics
    W = (rng.standard_normal((N, K)) * 0.02 + w_mean).astype(f32)
    W[: N // 2] += f32(0.01)    # and so do the halves of W
    return X, W


def test_groups_of_one_are_the_plain_layer():
    """Eq. 13-15 with G = 1 are Eq. 3, 5, 12."""
    X, W = _rand_layer(11, 5, 128, 48)
    a, b = oracle.forward(X, W), oracle.forward_grouped(X, W, 1, 1)
    for key in ("codes", "sign", "y", "xhat"):
        assert np.array_equal(a[key], b[key]), key
    assert b["alpha"][0, 0] == a["alpha"] and b["beta"][0, 0] == a["beta"]


def test_group_parameters_eq13_are_block_means():
    """Eq. 13: alpha_g = (G/nm) sum W^(g), beta_g = (G/nm) ||W^(g)||_1, per block."""
    _, W = _rand_layer(12, 1, 96, 64)
    alpha, beta = oracle.weight_stats_grouped(W, 4, 3)
    for gn in range(4):
        for gk in range(3):
            blk = W[gn * 16:(gn + 1) * 16, gk * 32:(gk + 1) * 32].astype(np.float64)
            assert abs(float(alpha[gn, gk]) - blk.mean()) <= 1e-9
            assert abs(float(beta[gn, gk]) - np.abs(blk).mean()) <= 1e-9
    sign = oracle.binarize_grouped(W, alpha)
    for gn in range(4):
        for gk in range(3):
            blk = W[gn * 16:(gn + 1) * 16, gk * 32:(gk + 1) * 32]
            ref = np.where(blk > alpha[gn, gk], 1, -1)
            assert np.array_equal(sign[gn * 16:(gn + 1) * 16, gk * 32:(gk + 1) * 32], ref)


@pytest.mark.parametrize("per_tensor", [False, True])
def test_row_groups_are_independent_layers(per_tensor):
    """Column-parallel split (groups of output rows): each group's outputs are those of a
    BitLinear layer that holds only that group's rows - the point of Eq. 13."""
    X, W = _rand_layer(13, 6, 128, 64)
    r = oracle.forward_grouped(X, W, groups_n=4, groups_k=1, per_tensor=per_tensor)
    for g in range(4):
        solo = oracle.forward(X, W[g * 16:(g + 1) * 16], per_tensor=per_tensor)
        assert np.array_equal(r["y"][:, g * 16:(g + 1) * 16], solo["y"])
        assert r["beta"][g, 0] == solo["beta"]


@pytest.mark.parametrize("per_tensor", [False, True])
def test_column_groups_sum_independent_layers(per_tensor):
    """Row-parallel split (groups of input columns): group LayerNorm (Eq. 15), gamma_g (Eq. 14)
    and alpha_g, beta_g (Eq. 13) make each slice a BitLinear layer of its own; the output is
    the sum of their outputs."""
    X, W = _rand_layer(14, 6, 128, 32)
    r = oracle.forward_grouped(X, W, groups_n=1, groups_k=4, per_tensor=per_tensor)
    total = np.zeros((6, 32))
    for g in range(4):
        sl = slice(g * 32, (g + 1) * 32)
        solo = oracle.forward(np.ascontiguousarray(X[:, sl]), np.ascontiguousarray(W[:, sl]),
                              per_tensor=per_tensor)
        total += solo["y"].astype(np.float64)
        assert np.array_equal(r["codes"][:, sl], solo["codes"])
        assert np.array_equal(r["xhat"][:, sl], solo["xhat"])
    assert np.abs(r["y64"] - total).max() <= 1e-12
    # Eq. 15: every slice of a token is normalised on its own
    xh = r["xhat"].reshape(6, 4, 32).astype(np.float64)
    assert np.abs(xh.mean(axis=2)).max() < 1e-6
    assert np.abs(xh.var(axis=2) - 1.0).max() < 1e-4


def test_groups_brute_force_tiny():
    """Eq. 13-15 written out with Python loops on a 4x8 weight, 2 tokens, 2x2 groups."""
    rng = np.random.default_rng(15)
    M, K, N, GN, GK = 2, 8, 4, 2, 2
    X = rng.standard_normal((M, K)).astype(f32)
    W = (rng.standard_normal((N, K)) * 0.5).astype(f32)
    eps = 1e-5
    Ng, Kg = N // GN, K // GK
    y = np.zeros((M, N))
    for m in range(M):
        for gk in range(GK):
            xs = [float(X[m, gk * Kg + k]) for k in range(Kg)]
            mu = sum(xs) / Kg
            var = sum((v - mu) ** 2 for v in xs) / Kg
            xh = [f32((v - mu) / np.sqrt(var + eps)) for v in xs]
            gamma = max(abs(v) for v in xh)
            scale = f32(128.0) / f32(gamma)
            q = [int(np.clip(np.rint(f32(v) * scale), -128, 127)) for v in xh]
            for n in range(N):
                gn = n // Ng
                blk = [float(W[r, gk * Kg + k]) for r in range(gn * Ng, (gn + 1) * Ng) for k in range(Kg)]
                alpha = f32(sum(blk) / len(blk))
                beta = f32(sum(abs(v) for v in blk) / len(blk))
                acc = sum(q[k] * (1 if W[n, gk * Kg + k] > alpha else -1) for k in range(Kg))
                y[m, n] += float(f32(acc) * ((beta * f32(gamma)) / f32(128.0)))
    r = oracle.forward_grouped(X, W, GN, GK, eps=eps)
    # the fp64 sums of mu/var may differ in the last bit from Python's order: 1e-6 relative
    assert np.allclose(r["y64"], y, rtol=1e-6, atol=1e-7)


def test_groups_do_not_leak():
    """A change inside one block of W leaves every other block's bits and parameters alone."""
    X, W = _rand_layer(16, 3, 64, 32)
    r0 = oracle.forward_grouped(X, W, 2, 2)
    W2 = W.copy()
    W2[:16, :32] += f32(0.05)
    r1 = oracle.forward_grouped(X, W2, 2, 2)
    assert r0["alpha"][0, 0] != r1["alpha"][0, 0]
    for gn, gk in ((0, 1), (1, 0), (1, 1)):
        assert r0["alpha"][gn, gk] == r1["alpha"][gn, gk] and r0["beta"][gn, gk] == r1["beta"][gn, gk]
    assert np.array_equal(r0["sign"][16:], r1["sign"][16:])
    assert np.array_equal(r0["sign"][:16, 32:], r1["sign"][:16, 32:])
    assert np.array_equal(r0["y"][:, 16:], r1["y"][:, 16:])


# ---------------------------------------------------------------- backward of Eq. 12 / Eq. 15
@pytest.mark.parametrize("groups", [1, 4])
def test_layernorm_backward_matches_autograd(groups):
    """Chain rule through Eq. 12 (groups = 1: layer_norm; groups > 1: group_norm, Eq. 15),
    against torch's fp64 autograd of its own LayerNorm / GroupNorm."""
    rng = np.random.default_rng(21)
    M, K = 7, 96
    X = (rng.standard_normal((M, K)) * 2 + 0.5).astype(f32)
    g = rng.standard_normal((M, K)).astype(f32)
    gain = (1 + 0.2 * rng.standard_normal(K)).astype(f32)
    dX, dgain, dbias = oracle.layernorm_backward(g, X, gain=gain, groups=groups, want_affine=True)
    xt = torch.tensor(X, dtype=torch.float64, requires_grad=True)
    gt = torch.tensor(gain, dtype=torch.float64, requires_grad=True)
    bt = torch.zeros(K, dtype=torch.float64, requires_grad=True)
    if groups == 1:
        out = torch.nn.functional.layer_norm(xt, (K,), gt, bt, 1e-5)
    else:
        out = torch.nn.functional.group_norm(xt.reshape(M, groups, K // groups), groups, eps=1e-5)
        out = out.reshape(M, K) * gt + bt
    out.backward(torch.tensor(g, dtype=torch.float64))
    assert np.abs(dX - xt.grad.numpy()).max() <= 1e-6
    assert np.abs(dgain - gt.grad.numpy()).max() <= 2e-6
    assert np.abs(dbias - bt.grad.numpy()).max() <= 2e-6


def test_layernorm_backward_finite_differences_and_projections():
    """dX is the derivative of sum(g * LN(x)) (central differences on the oracle's forward in
    fp64-friendly sizes), and it is orthogonal to the two directions LN removes: the constant
    vector and the normalised row itself."""
    rng = np.random.default_rng(22)
    M, K = 3, 32
    X = rng.standard_normal((M, K)).astype(f32)
    g = rng.standard_normal((M, K)).astype(f32)
    dX = oracle.layernorm_backward(g, X).astype(np.float64)

    def loss(Xd):
        mu = Xd.mean(axis=1, keepdims=True)
        var = Xd.var(axis=1, keepdims=True)
        return float((g.astype(np.float64) * (Xd - mu) / np.sqrt(var + 1e-5)).sum())

    Xd = X.astype(np.float64)
    h = 1e-5
    for (m, k) in [(0, 0), (1, 7), (2, 31), (0, 16)]:
        e = np.zeros_like(Xd)
        e[m, k] = h
        fd = (loss(Xd + e) - loss(Xd - e)) / (2 * h)
        assert abs(fd - dX[m, k]) <= 1e-5 * max(1.0, abs(fd))
    xn = oracle.layernorm(X).astype(np.float64)
    assert np.abs(dX.sum(axis=1)).max() <= 1e-5
    # exact only for eps = 0: the residual is rstd * sum(g * xn) * eps / (var + eps) ~ 1e-4 here
    assert np.abs((dX * xn).sum(axis=1)).max() <= 1e-3


# ---------------------------------------------------------------- Eq. 6: non-negative quantiser
def test_eq6_range_and_reconstruction():
    """Eq. 6: the shifted activations fill [0, Q_b]; the minimum maps to code 0, the maximum to
    the top code, and q * gamma / 128 + eta reconstructs x to half a step."""
    rng = np.random.default_rng(31)
    x = (rng.standard_normal((6, 256)) * 1.7 + 0.4).astype(f32)
    eta, gamma = oracle.minmax_nonneg(x)
    assert np.array_equal(eta, x.min(axis=1)) and np.array_equal(gamma, (x.max(axis=1) - x.min(axis=1)))
    q = oracle.quantize_nonneg(x, eta, gamma)
    assert q.min() == 0 and q.max() == 127
    assert np.all(q[np.arange(6), x.argmin(axis=1)] == 0)
    assert np.all(q[np.arange(6), x.argmax(axis=1)] == 127)   # rne gives 128, the clamp 127
    rec = q.astype(np.float64) * gamma[:, None] / 128.0 + eta[:, None]
    step = gamma[:, None].astype(np.float64) / 128.0
    err = np.abs(rec - x)
    # half a step, plus the fp32 roundings of x - eta and of the scaling (a few ulps of |x|)
    assert np.all(err <= 0.5 * step + 4e-6 + (q == 127) * 0.5 * step)


def test_eq6_reduces_to_eq4_on_nonnegative_rows_with_a_zero():
    """With min x = 0 the shift vanishes and gamma = max x = ||x||_inf: Eq. 6 is Eq. 4."""
    rng = np.random.default_rng(32)
    x = np.abs(rng.standard_normal((5, 128))).astype(f32)
    x[:, 3] = 0.0
    eta, gamma = oracle.minmax_nonneg(x)
    assert np.all(eta == 0)
    assert np.array_equal(gamma, oracle.absmax(x))
    assert np.array_equal(oracle.quantize_nonneg(x, eta, gamma), oracle.quantize(x, gamma))


def test_eq6_shift_invariance():
    """eta absorbs a constant: x + c has the codes of x (integer-valued data, exact shift)."""
    rng = np.random.default_rng(33)
    x = rng.integers(-50, 50, (4, 64)).astype(f32)
    a = oracle.quantize_nonneg(x, *oracle.minmax_nonneg(x))
    b = oracle.quantize_nonneg(x + f32(1024), *oracle.minmax_nonneg(x + f32(1024)))
    assert np.array_equal(a, b)


def test_eq6_forward_matches_float_matmul_of_dequantised_activations():
    """The dequantisation proposed for Eq. 6: y = beta * W~ (x~ gamma / Q_b + eta), checked
    against numpy's fp64 matmul of the reconstructed activations."""
    rng = np.random.default_rng(34)
    X = (rng.standard_normal((9, 96)) + 0.3).astype(f32)
    W = (rng.standard_normal((40, 96)) * 0.02).astype(f32)
    r = oracle.forward_nonneg(X, W)
    assert np.array_equal(r["wsum"], r["sign"].astype(np.int64).sum(axis=1))
    rec = r["codes"].astype(np.float64) * r["gamma"][:, None] / 128.0 + r["eta"][:, None]
    y = float(r["beta"]) * rec @ r["sign"].astype(np.float64).T
    assert np.abs(r["y"] - y).max() <= 1e-5 * np.abs(y).max()
    # and the quantised layer stays close to the unquantised one (8-bit activations)
    yf = float(r["beta"]) * r["xhat"].astype(np.float64) @ r["sign"].astype(np.float64).T
    assert np.linalg.norm(r["y"] - yf) / np.linalg.norm(yf) < 0.05


def test_eq6_per_tensor_branches():
    """The paragraph after Eq. 6 makes per tensor the training-time granularity: one eta and one
    gamma for the whole tensor.  Pinned against numpy's min / max over the tensor, against the
    per-token functions applied to the tensor laid out as one long row (and on a one-row input,
    where the two granularities coincide), against hand values, and through the same fp64
    reconstruction as the per-token forward."""
    rng = np.random.default_rng(35)
    x = (rng.standard_normal((7, 160)) * 1.3 - 0.2).astype(f32)
    eta, gamma = oracle.minmax_nonneg(x, per_tensor=True)
    assert eta.shape == (1,) and gamma.shape == (1,)
    assert eta[0] == x.min() and gamma[0] == f32(x.max() - x.min())
    q = oracle.quantize_nonneg(x, eta, gamma, per_tensor=True)
    # one long row, per token: the same minimum, range and codes
    row = x.reshape(1, -1)
    e1, g1 = oracle.minmax_nonneg(row)
    assert e1[0] == eta[0] and g1[0] == gamma[0]
    assert np.array_equal(oracle.quantize_nonneg(row, e1, g1).reshape(x.shape), q)
    assert q.min() == 0 and q.max() == 127
    assert q.reshape(-1)[x.argmin()] == 0 and q.reshape(-1)[x.argmax()] == 127
    # a one-row tensor: both granularities are the same thing
    et, gt = oracle.minmax_nonneg(x[:1], per_tensor=True)
    ek, gk = oracle.minmax_nonneg(x[:1])
    assert et[0] == ek[0] and gt[0] == gk[0]
    assert np.array_equal(oracle.quantize_nonneg(x[:1], et, gt, per_tensor=True),
                          oracle.quantize_nonneg(x[:1], ek, gk))
    # hand values: rows [0, 1, 2, 4] and [-4, 0, 1, 3]: eta = -4, gamma = 8, scale 16
    h = np.array([[0, 1, 2, 4], [-4, 0, 1, 3]], f32)
    eh, gh = oracle.minmax_nonneg(h, per_tensor=True)
    assert eh[0] == -4 and gh[0] == 8
    assert oracle.quantize_nonneg(h, eh, gh, per_tensor=True).tolist() == [[64, 80, 96, 127], [0, 64, 80, 112]]
    # the per-tensor dequantisation is the per-token one with the two scalars repeated per row
    acc = rng.integers(-5000, 5000, (7, 12)).astype(np.int32)
    wsum = rng.integers(-160, 160, 12).astype(np.int32)
    y_t = oracle.dequant_nonneg(acc, gamma, eta, 0.017, wsum, per_tensor=True)
    y_k = oracle.dequant_nonneg(acc, np.repeat(gamma, 7), np.repeat(eta, 7), 0.017, wsum)
    assert np.array_equal(y_t, y_k)
    # end to end: y = beta * W~ (x~ gamma / Q_b + eta) with the tensor-wide scalars
    W = (rng.standard_normal((24, 160)) * 0.02).astype(f32)
    r = oracle.forward_nonneg(x, W, per_tensor=True)
    rec = r["codes"].astype(np.float64) * float(r["gamma"][0]) / 128.0 + float(r["eta"][0])
    y = float(r["beta"]) * rec @ r["sign"].astype(np.float64).T
    assert np.abs(r["y"] - y).max() <= 1e-5 * np.abs(y).max()


def test_eq6_grouped_forward_composition():
    """Eq. 14 gives every K-group its own eta_g and gamma_g.  One group is the plain Eq. 6 layer
    bit for bit; column groups equal the sum of independent Eq. 6 layers on the column slices;
    row groups equal independent layers on the row slices bit for bit; and the whole thing against
    a brute-force Python evaluation of y = sum_g beta_g W~_g (x~_g gamma_g / Q_b + eta_g)."""
    rng = np.random.default_rng(36)
    M, K, N = 5, 192, 48
    X = (rng.standard_normal((M, K)) * 1.2 + 0.3).astype(f32)
    X[:, :64] += 2.0
    W = (rng.standard_normal((N, K)) * 0.02).astype(f32)
    W[:24] += 0.01
    for pt in (False, True):
        one = oracle.forward_grouped_nonneg(X, W, 1, 1, per_tensor=pt)
        plain = oracle.forward_nonneg(X, W, per_tensor=pt)
        assert np.array_equal(one["y"], plain["y"]) and np.array_equal(one["codes"], plain["codes"])
        # three column groups: the sum of three independent layers, each on its slice of LN'd input
        r = oracle.forward_grouped_nonneg(X, W, 1, 3, per_tensor=pt)
        tot = np.zeros((M, N))
        for g in range(3):
            sl = slice(64 * g, 64 * (g + 1))
            part = oracle.forward_nonneg(X[:, sl], W[:, sl], per_tensor=pt)  # LN over the slice = group LN
            tot += part["y"].astype(np.float64)
            assert np.array_equal(r["codes"][:, sl], part["codes"])
            assert np.array_equal(r["eta"][:, g], part["eta"]) and np.array_equal(r["gamma"][:, g], part["gamma"])
        assert np.array_equal(r["y64"], tot)
        # two row groups: independent layers on the row slices
        r2 = oracle.forward_grouped_nonneg(X, W, 2, 1, per_tensor=pt)
        for g in range(2):
            rows = slice(24 * g, 24 * (g + 1))
            assert np.array_equal(r2["y"][:, rows], oracle.forward_nonneg(X, W[rows], per_tensor=pt)["y"])
        # brute force with Python floats on the 2 x 3 grouping
        r3 = oracle.forward_grouped_nonneg(X, W, 2, 3, per_tensor=pt)
        for m in (0, M - 1):
            for n in (0, 23, 24, N - 1):
                y = 0.0
                for g in range(3):
                    bg = float(r3["beta"][n // 24, g])
                    e = float(r3["eta"][0 if pt else m, g])
                    ga = float(r3["gamma"][0 if pt else m, g])
                    for k in range(64 * g, 64 * (g + 1)):
                        y += bg * int(r3["sign"][n, k]) * (int(r3["codes"][m, k]) * ga / 128.0 + e)
                assert abs(r3["y64"][m, n] - y) <= 1e-5 * max(1.0, abs(y))
