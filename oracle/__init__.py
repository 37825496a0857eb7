"""CPU oracle for BitLinear (BitNet, arXiv 2310.11453, Sections 2.1-2.2).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
bench.py's cpu_baseline leg.  The product package never imports this module and
this module never imports the product package.

The arithmetic lives in bitlinear_oracle.c (plain scalar C).  This file only
compiles that C file with gcc and marshals numpy arrays into it; `forward()` at
the bottom chains the steps in the order of Eq. 11.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "bitlinear_oracle.c"
_LIB = _HERE / "libbitlinear_oracle.so"

_CFLAGS = ["-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
           "-std=c99", "-Wall", "-Wextra"]


def build(force: bool = False) -> Path:
    """Compile the oracle with gcc (building the checker is not using it)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".tmp{os.getpid()}.so")
        subprocess.check_call(["gcc", *_CFLAGS, str(_SRC), "-o", str(tmp), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(str(_LIB))
        _lib.oracle_num_threads.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray | None):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


_i64 = ctypes.c_int64
_c_float = ctypes.c_float
_c_int = ctypes.c_int


def num_threads() -> int:
    return int(_load().oracle_num_threads())


def set_num_threads(n: int) -> None:
    _load().oracle_set_num_threads(_c_int(n))


# ---- Eq. 1-3, 12: weight side -------------------------------------------------
def weight_stats(W, beta_centered: bool = False):
    """alpha = mean(W) (Eq. 3), beta = mean(|W|) (Eq. 12); both np.float32."""
    W = _f32(W)
    N, K = W.shape
    a, b = _c_float(), _c_float()
    _load().oracle_weight_stats(_p(W), _i64(N), _i64(K), _c_int(int(beta_centered)),
                                ctypes.byref(a), ctypes.byref(b))
    return np.float32(a.value), np.float32(b.value)


def binarize(W, alpha):
    """Sign(W - alpha) with Sign(0) = -1 (Eq. 1-2) as int8 [N,K]."""
    W = _f32(W)
    N, K = W.shape
    s = np.empty((N, K), np.int8)
    _load().oracle_binarize(_p(W), _i64(N), _i64(K), _c_float(float(alpha)), _p(s))
    return s


def pack_canonical(sign):
    """int8 {-1,+1} [N,K] -> uint32 [N, ceil(K/32)], bit k%32 of word k//32 set iff +1."""
    sign = np.ascontiguousarray(sign, dtype=np.int8)
    N, K = sign.shape
    words = np.empty((N, (K + 31) // 32), np.uint32)
    _load().oracle_pack_canonical(_p(sign), _i64(N), _i64(K), _p(words))
    return words


def unpack_canonical(words, K):
    words = np.ascontiguousarray(words, dtype=np.uint32)
    N = words.shape[0]
    sign = np.empty((N, K), np.int8)
    _load().oracle_unpack_canonical(_p(words), _i64(N), _i64(K), _p(sign))
    return sign


# ---- Eq. 12, 4, 5: activation side ---------------------------------------------
def layernorm(X, eps=1e-5, gain=None, bias=None, groups: int = 1):
    X = _f32(X)
    M, K = X.shape
    assert K % groups == 0
    gain = None if gain is None else _f32(gain)
    bias = None if bias is None else _f32(bias)
    out = np.empty((M, K), np.float32)
    _load().oracle_layernorm(_p(X), _i64(M), _i64(K), _i64(groups), _p(gain), _p(bias),
                             _c_float(eps), _p(out))
    return out


def absmax(xhat, per_tensor: bool = False, groups: int = 1):
    """gamma (Eq. 5): [M*groups] per token or [groups] per tensor, floored at 1e-5."""
    xhat = _f32(xhat)
    M, K = xhat.shape
    g = np.empty(groups if per_tensor else M * groups, np.float32)
    _load().oracle_absmax(_p(xhat), _i64(M), _i64(K), _i64(groups), _c_int(int(per_tensor)), _p(g))
    return g


def quantize(xhat, gamma, per_tensor: bool = False, groups: int = 1):
    """Eq. 4 with round-half-even and clamp to [-128,127]; int8 [M,K]."""
    xhat = _f32(xhat)
    gamma = _f32(gamma)
    M, K = xhat.shape
    assert gamma.size == (groups if per_tensor else M * groups)
    q = np.empty((M, K), np.int8)
    _load().oracle_quantize(_p(xhat), _i64(M), _i64(K), _i64(groups), _c_int(int(per_tensor)),
                            _p(gamma), _p(q))
    return q


# ---- Eq. 7, 11 --------------------------------------------------------------------
def matmul_i32(codes, sign, k0: int = 0, k1: int | None = None):
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    sign = np.ascontiguousarray(sign, dtype=np.int8)
    M, K = codes.shape
    N, K2 = sign.shape
    assert K == K2
    k1 = K if k1 is None else k1
    acc = np.empty((M, N), np.int32)
    _load().oracle_matmul_i32(_p(codes), _p(sign), _i64(M), _i64(N), _i64(K), _i64(k0), _i64(k1),
                              _p(acc))
    return acc


def matmul_i32_sampled(codes, sign, rows, cols):
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    sign = np.ascontiguousarray(sign, dtype=np.int8)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    N, K = sign.shape
    assert codes.shape[1] == K and rows.size == cols.size
    acc = np.empty(rows.size, np.int32)
    _load().oracle_matmul_i32_sampled(_p(codes), _p(sign), _i64(N), _i64(K), _p(rows), _p(cols),
                                      _i64(rows.size), _p(acc))
    return acc


def dequant(acc, gamma, beta, per_tensor: bool = False, beta_rows_per_group: int | None = None):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    gamma = _f32(gamma)
    beta = _f32(np.atleast_1d(beta))
    M, N = acc.shape
    rpg = N if beta_rows_per_group is None else beta_rows_per_group
    assert beta.size * rpg >= N
    Y = np.empty((M, N), np.float32)
    _load().oracle_dequant(_p(acc), _i64(M), _i64(N), _p(gamma), _i64(0 if per_tensor else 1),
                           _p(beta), _i64(rpg), _p(Y))
    return Y


def round_bf16(a):
    a = _f32(a)
    out = np.empty_like(a)
    _load().oracle_round_bf16(_p(a), _i64(a.size), _p(out))
    return out


def backward_ste(dY, codes, gamma, sign, beta, per_tensor: bool, rows_dx=None, rows_dw=None,
                 want_dx=True, want_dw=True):
    """STE backward (Section 2.2).  Returns (dX, dW); sampled rows if rows_* given."""
    dY = _f32(dY)
    codes = np.ascontiguousarray(codes, dtype=np.int8)
    sign = np.ascontiguousarray(sign, dtype=np.int8)
    gamma = _f32(gamma)
    M, N = dY.shape
    K = codes.shape[1]
    assert codes.shape == (M, K) and sign.shape == (N, K)
    rdx = None if rows_dx is None else np.ascontiguousarray(rows_dx, dtype=np.int64)
    rdw = None if rows_dw is None else np.ascontiguousarray(rows_dw, dtype=np.int64)
    dX = np.empty((M if rdx is None else rdx.size, K), np.float32) if want_dx else None
    dW = np.empty((N if rdw is None else rdw.size, K), np.float32) if want_dw else None
    _load().oracle_backward_ste(_p(dY), _i64(M), _i64(N), _i64(K), _p(codes), _p(gamma),
                                _c_int(int(per_tensor)), _p(sign), _c_float(float(beta)),
                                _p(rdx), _i64(0 if rdx is None else rdx.size), _p(dX),
                                _p(rdw), _i64(0 if rdw is None else rdw.size), _p(dW))
    return dX, dW


def layernorm_backward(g, X, eps=1e-5, gain=None, groups: int = 1, want_affine: bool = False):
    """Backward of Eq. 12 / Eq. 15 (STE: g is the gradient w.r.t. the LayerNorm output).
    Returns dX, or (dX, dgain, dbias) with want_affine."""
    g = _f32(g)
    X = _f32(X)
    M, K = X.shape
    assert g.shape == (M, K) and K % groups == 0
    gain = None if gain is None else _f32(gain)
    dX = np.empty((M, K), np.float32)
    dgain = np.empty(K, np.float32) if want_affine else None
    dbias = np.empty(K, np.float32) if want_affine else None
    _load().oracle_layernorm_backward(_p(g), _p(X), _i64(M), _i64(K), _i64(groups), _p(gain),
                                      _c_float(eps), _p(dX), _p(dgain), _p(dbias))
    return (dX, dgain, dbias) if want_affine else dX

# ---- Eq. 11 end to end ----------------------------------------------------------------
def forward(X, W, eps=1e-5, per_tensor=False, skip_ln=False, beta_centered=False,
            gain=None, bias=None):
    """BitLinear forward, step by step in the order of Eq. 11.  Returns a dict with every
    intermediate: alpha, beta, sign, words, xhat, gamma, codes, acc, y."""
    alpha, beta = weight_stats(W, beta_centered)
    sign = binarize(W, alpha)
    words = pack_canonical(sign)
    xhat = _f32(X) if skip_ln else layernorm(X, eps, gain, bias)
    gamma = absmax(xhat, per_tensor)
    codes = quantize(xhat, gamma, per_tensor)
    acc = matmul_i32(codes, sign)
    y = dequant(acc, gamma, beta, per_tensor)
    return dict(alpha=alpha, beta=beta, sign=sign, words=words, xhat=xhat, gamma=gamma,
                codes=codes, acc=acc, y=y)


# ---- Eq. 13-15: Group Quantization and Normalization -----------------------------------
def weight_stats_grouped(W, groups_n: int = 1, groups_k: int = 1, beta_centered: bool = False):
    """Eq. 13: alpha_g, beta_g of each of the groups_n x groups_k blocks of W (rows split in
    groups_n equal parts, columns in groups_k).  Returns (alpha, beta), each [groups_n, groups_k]."""
    W = _f32(W)
    N, K = W.shape
    assert N % groups_n == 0 and K % groups_k == 0
    Ng, Kg = N // groups_n, K // groups_k
    alpha = np.empty((groups_n, groups_k), np.float32)
    beta = np.empty((groups_n, groups_k), np.float32)
    for gn in range(groups_n):
        for gk in range(groups_k):
            blk = np.ascontiguousarray(W[gn * Ng:(gn + 1) * Ng, gk * Kg:(gk + 1) * Kg])
            alpha[gn, gk], beta[gn, gk] = weight_stats(blk, beta_centered)
    return alpha, beta


def binarize_grouped(W, alpha):
    """Eq. 1-2 with the alpha of the block that holds each weight; sign int8 [N,K]."""
    W = _f32(W)
    N, K = W.shape
    groups_n, groups_k = alpha.shape
    Ng, Kg = N // groups_n, K // groups_k
    sign = np.empty((N, K), np.int8)
    for gn in range(groups_n):
        for gk in range(groups_k):
            blk = np.ascontiguousarray(W[gn * Ng:(gn + 1) * Ng, gk * Kg:(gk + 1) * Kg])
            sign[gn * Ng:(gn + 1) * Ng, gk * Kg:(gk + 1) * Kg] = binarize(blk, float(alpha[gn, gk]))
    return sign


def forward_grouped(X, W, groups_n: int = 1, groups_k: int = 1, eps=1e-5, per_tensor=False,
                    skip_ln=False, beta_centered=False, gain=None, bias=None, xhat=None):
    """BitLinear forward with the group parameters of Eq. 13-15.  The weights are split into
    groups_n row groups and groups_k column groups (alpha, beta per block); the activations into
    groups_k slices of each token (group LayerNorm, Eq. 15; gamma per slice, Eq. 14).  Each
    K-slice is contracted on its own and dequantised with its own beta_g * gamma_g / 128
    (fp32 product as in Eq. 11); the slices are added in fp64.  `xhat`, if given, replaces the
    group LayerNorm's output (a test passes the normalised input another implementation produced,
    to compare everything after it "given the same normalised input")."""
    X = _f32(X)
    W = _f32(W)
    M, K = X.shape
    N = W.shape[0]
    Ng, Kg = N // groups_n, K // groups_k
    alpha, beta = weight_stats_grouped(W, groups_n, groups_k, beta_centered)
    sign = binarize_grouped(W, alpha)
    if xhat is None:
        xhat = X if skip_ln else layernorm(X, eps, gain, bias, groups=groups_k)
    xhat = _f32(xhat)
    gamma = absmax(xhat, per_tensor, groups=groups_k)       # [M*groups_k] or [groups_k]
    codes = quantize(xhat, gamma, per_tensor, groups=groups_k)
    gam = gamma.reshape(-1, groups_k)                       # [M, groups_k] or [1, groups_k]
    ysum = np.zeros((M, N), np.float64)
    accs = []
    for gk in range(groups_k):
        acc = matmul_i32(codes, sign, gk * Kg, (gk + 1) * Kg)
        accs.append(acc)
        g_col = np.ascontiguousarray(gam[:, gk])
        part = dequant(acc, g_col, np.ascontiguousarray(beta[:, gk]), per_tensor,
                       beta_rows_per_group=Ng)
        ysum += part.astype(np.float64)
    return dict(alpha=alpha, beta=beta, sign=sign, words=pack_canonical(sign), xhat=xhat,
                gamma=gam if not per_tensor else gam.reshape(groups_k), codes=codes, acc=accs,
                y=ysum.astype(np.float32), y64=ysum)


# ---- Eq. 6: the non-negative quantiser ------------------------------------------------
def minmax_nonneg(xhat, per_tensor: bool = False):
    """eta = min, gamma = max(x - eta) floored at 1e-5; [M] each per token, [1] per tensor."""
    xhat = _f32(xhat)
    M, K = xhat.shape
    n = 1 if per_tensor else M
    eta = np.empty(n, np.float32)
    gamma = np.empty(n, np.float32)
    _load().oracle_minmax_nonneg(_p(xhat), _i64(M), _i64(K), _c_int(int(per_tensor)), _p(eta),
                                 _p(gamma))
    return eta, gamma


def quantize_nonneg(xhat, eta, gamma, per_tensor: bool = False):
    xhat = _f32(xhat)
    M, K = xhat.shape
    codes = np.empty((M, K), np.int8)
    _load().oracle_quantize_nonneg(_p(xhat), _i64(M), _i64(K), _c_int(int(per_tensor)),
                                   _p(_f32(eta)), _p(_f32(gamma)), _p(codes))
    return codes


def weight_rowsum(sign):
    sign = np.ascontiguousarray(sign, dtype=np.int8)
    N, K = sign.shape
    out = np.empty(N, np.int32)
    _load().oracle_weight_rowsum(_p(sign), _i64(N), _i64(K), _p(out))
    return out


def dequant_nonneg(acc, gamma, eta, beta, wsum, per_tensor: bool = False):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    M, N = acc.shape
    Y = np.empty((M, N), np.float32)
    _load().oracle_dequant_nonneg(_p(acc), _i64(M), _i64(N), _p(_f32(gamma)), _p(_f32(eta)),
                                  _i64(0 if per_tensor else 1), _c_float(float(beta)),
                                  _p(np.ascontiguousarray(wsum, dtype=np.int32)), _p(Y))
    return Y


def forward_nonneg(X, W, eps=1e-5, per_tensor=False, skip_ln=False, gain=None, bias=None):
    """BitLinear forward with the quantiser of Eq. 6 in place of Eq. 4."""
    alpha, beta = weight_stats(W)
    sign = binarize(W, alpha)
    xhat = _f32(X) if skip_ln else layernorm(X, eps, gain, bias)
    eta, gamma = minmax_nonneg(xhat, per_tensor)
    codes = quantize_nonneg(xhat, eta, gamma, per_tensor)
    acc = matmul_i32(codes, sign)
    wsum = weight_rowsum(sign)
    y = dequant_nonneg(acc, gamma, eta, beta, wsum, per_tensor)
    return dict(alpha=alpha, beta=beta, sign=sign, xhat=xhat, eta=eta, gamma=gamma, codes=codes,
                acc=acc, wsum=wsum, y=y)


def forward_grouped_nonneg(X, W, groups_n: int = 1, groups_k: int = 1, eps=1e-5, per_tensor=False,
                           skip_ln=False, gain=None, bias=None, xhat=None):
    """BitLinear forward with the group parameters of Eq. 13-15 and the quantiser of Eq. 6 per
    K-group (Eq. 14 defines eta_g beside gamma_g): each K-slice of a token is normalised (group
    LayerNorm), shifted by its own eta_g = min, scaled by its own gamma_g = max - min (per token,
    or over all tokens per tensor), contracted on its own, dequantised as
    acc_g * (beta_g gamma_g / 128) + (beta_g eta_g) * wsum_g[n] (the plain Eq. 6 layer's formula with
    the slice's own sums), and the slices are added in fp64.  `xhat` as in forward_grouped."""
    X = _f32(X)
    W = _f32(W)
    M, K = X.shape
    N = W.shape[0]
    Ng, Kg = N // groups_n, K // groups_k
    alpha, beta = weight_stats_grouped(W, groups_n, groups_k)
    sign = binarize_grouped(W, alpha)
    if xhat is None:
        xhat = X if skip_ln else layernorm(X, eps, gain, bias, groups=groups_k)
    xhat = _f32(xhat)
    n_par = 1 if per_tensor else M
    eta = np.empty((n_par, groups_k), np.float32)
    gamma = np.empty((n_par, groups_k), np.float32)
    codes = np.empty((M, K), np.int8)
    wsum = np.empty((groups_k, N), np.int32)
    ysum = np.zeros((M, N), np.float64)
    for gk in range(groups_k):
        sl = slice(gk * Kg, (gk + 1) * Kg)
        xs = np.ascontiguousarray(xhat[:, sl])
        e, g = minmax_nonneg(xs, per_tensor)
        q = quantize_nonneg(xs, e, g, per_tensor)
        eta[:, gk], gamma[:, gk], codes[:, sl] = e, g, q
        sg = np.ascontiguousarray(sign[:, sl])
        acc = matmul_i32(q, sg)
        wsum[gk] = weight_rowsum(sg)
        for gn in range(groups_n):   # beta of the block (row group gn, column group gk)
            rows = slice(gn * Ng, (gn + 1) * Ng)
            part = dequant_nonneg(np.ascontiguousarray(acc[:, rows]), g, e, float(beta[gn, gk]),
                                  np.ascontiguousarray(wsum[gk, rows]), per_tensor)
            ysum[:, rows] += part.astype(np.float64)
    return dict(alpha=alpha, beta=beta, sign=sign, xhat=xhat, eta=eta, gamma=gamma, codes=codes,
                wsum=wsum, y=ysum.astype(np.float32), y64=ysum)
