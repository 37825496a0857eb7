"""Thin ctypes binding of libbitlinear.so (see include/bitlinear.h).

Argument marshalling only: every step of BitLinear runs in the HIP kernels.
PyTorch supplies device memory and the current stream, nothing else.  There is
no CPU fallback: a missing library or a missing GPU raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_PKG = Path(__file__).resolve().parent
LIB_PATH = _PKG / "libbitlinear.so"

BL_OK = 0
GAMMA_PER_TOKEN, GAMMA_PER_TENSOR = 0, 1
FLAG_SKIP_LN, FLAG_OUT_ACC_I32, FLAG_BETA_CENTERED = 1, 2, 4
OP_PACK, OP_QUANT, OP_FORWARD, OP_BACKWARD, OP_LN_BACKWARD, OP_FORWARD_NONNEG = 0, 1, 2, 3, 4, 5
OP_MATMUL = 6

EXPORTS = (
    "bitlinear_packed_bytes", "bitlinear_workspace_bytes", "bitlinear_pack_weights",
    "bitlinear_packed_to_canonical", "bitlinear_quant_act", "bitlinear_matmul",
    "bitlinear_forward", "bitlinear_backward_ste", "bitlinear_status_string",
    "bitlinear_packed_bytes_grouped", "bitlinear_workspace_bytes_grouped",
    "bitlinear_pack_weights_grouped", "bitlinear_packed_to_canonical_grouped",
    "bitlinear_quant_act_grouped", "bitlinear_forward_grouped", "bitlinear_layernorm_backward",
    "bitlinear_weight_rowsums", "bitlinear_quant_act_nonneg", "bitlinear_matmul_nonneg",
    "bitlinear_forward_nonneg", "bitlinear_forward_workspace_layout", "bitlinear_set_tuning",
    "bitlinear_forward_static", "bitlinear_probe_read", "bitlinear_weight_rowsums_grouped",
    "bitlinear_quant_act_grouped_nonneg", "bitlinear_forward_grouped_nonneg",
)

_lib = None


class BitLinearError(RuntimeError):
    pass


def load_library() -> ctypes.CDLL:
    """Loads the in-tree library (build it first: python -m paper_2310_11453_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    if not LIB_PATH.exists():
        raise BitLinearError(f"{LIB_PATH} is missing: run `python -m paper_2310_11453_amd.build`")
    lib = ctypes.CDLL(str(LIB_PATH))
    i64, u32, vp, sz, ci, cf = (ctypes.c_int64, ctypes.c_uint, ctypes.c_void_p, ctypes.c_size_t,
                                ctypes.c_int, ctypes.c_float)
    lib.bitlinear_packed_bytes.restype = sz
    lib.bitlinear_packed_bytes.argtypes = [i64, i64, u32]
    lib.bitlinear_workspace_bytes.restype = sz
    lib.bitlinear_workspace_bytes.argtypes = [ci, i64, i64, i64, ci, u32]
    lib.bitlinear_pack_weights.restype = ci
    lib.bitlinear_pack_weights.argtypes = [vp, i64, i64, u32, vp, vp, vp, vp, sz, vp]
    lib.bitlinear_packed_to_canonical.restype = ci
    lib.bitlinear_packed_to_canonical.argtypes = [vp, i64, i64, vp, vp]
    lib.bitlinear_quant_act.restype = ci
    lib.bitlinear_quant_act.argtypes = [vp, i64, i64, vp, vp, cf, ci, u32, vp, vp, vp, vp, vp, sz, vp]
    lib.bitlinear_matmul.restype = ci
    lib.bitlinear_matmul.argtypes = [vp, vp, vp, i64, i64, vp, i64, vp, ci, u32, vp, vp, sz, vp]
    lib.bitlinear_forward.restype = ci
    lib.bitlinear_forward.argtypes = [vp, i64, i64, vp, i64, vp, vp, vp, cf, ci, u32, vp, vp, sz, vp]
    lib.bitlinear_backward_ste.restype = ci
    lib.bitlinear_backward_ste.argtypes = [vp, i64, i64, i64, vp, vp, ci, vp, vp, vp, vp, vp, sz, vp]
    lib.bitlinear_packed_bytes_grouped.restype = sz
    lib.bitlinear_packed_bytes_grouped.argtypes = [i64, i64, ci, ci]
    lib.bitlinear_workspace_bytes_grouped.restype = sz
    lib.bitlinear_workspace_bytes_grouped.argtypes = [ci, i64, i64, i64, ci, ci, ci]
    lib.bitlinear_pack_weights_grouped.restype = ci
    lib.bitlinear_pack_weights_grouped.argtypes = [vp, i64, i64, ci, ci, u32, vp, vp, vp, vp, sz, vp]
    lib.bitlinear_packed_to_canonical_grouped.restype = ci
    lib.bitlinear_packed_to_canonical_grouped.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.bitlinear_quant_act_grouped.restype = ci
    lib.bitlinear_quant_act_grouped.argtypes = [vp, i64, i64, ci, vp, vp, cf, ci, u32, vp, vp, vp, vp,
                                                vp, sz, vp]
    lib.bitlinear_forward_grouped.restype = ci
    lib.bitlinear_forward_grouped.argtypes = [vp, i64, i64, vp, i64, ci, ci, vp, vp, vp, cf, ci, u32,
                                              vp, vp, sz, vp]
    lib.bitlinear_layernorm_backward.restype = ci
    lib.bitlinear_layernorm_backward.argtypes = [vp, vp, i64, i64, ci, vp, cf, vp, vp, vp, vp, sz, vp]
    lib.bitlinear_weight_rowsums.restype = ci
    lib.bitlinear_weight_rowsums.argtypes = [vp, i64, i64, vp, vp]
    lib.bitlinear_quant_act_nonneg.restype = ci
    lib.bitlinear_quant_act_nonneg.argtypes = [vp, i64, i64, vp, vp, cf, ci, u32, vp, vp, vp, vp, vp,
                                               vp, sz, vp]
    lib.bitlinear_matmul_nonneg.restype = ci
    lib.bitlinear_matmul_nonneg.argtypes = [vp, vp, vp, vp, i64, i64, vp, i64, vp, vp, ci, u32, vp, vp]
    lib.bitlinear_forward_nonneg.restype = ci
    lib.bitlinear_forward_nonneg.argtypes = [vp, i64, i64, vp, i64, vp, vp, vp, vp, cf, ci, u32, vp,
                                             vp, sz, vp]
    lib.bitlinear_forward_static.restype = ci
    lib.bitlinear_forward_static.argtypes = [vp, i64, i64, vp, i64, vp, vp, vp, cf, ci, u32, vp, vp]
    lib.bitlinear_weight_rowsums_grouped.restype = ci
    lib.bitlinear_weight_rowsums_grouped.argtypes = [vp, i64, i64, ci, vp, vp]
    lib.bitlinear_quant_act_grouped_nonneg.restype = ci
    lib.bitlinear_quant_act_grouped_nonneg.argtypes = [vp, i64, i64, ci, vp, vp, cf, ci, u32, vp, vp, vp,
                                                       vp, vp, vp, sz, vp]
    lib.bitlinear_forward_grouped_nonneg.restype = ci
    lib.bitlinear_forward_grouped_nonneg.argtypes = [vp, i64, i64, vp, i64, ci, ci, vp, vp, vp, vp, cf,
                                                     ci, u32, vp, vp, sz, vp]
    lib.bitlinear_probe_read.restype = ci
    lib.bitlinear_probe_read.argtypes = [vp, sz, ci, ci, vp, vp]
    lib.bitlinear_forward_workspace_layout.restype = ci
    lib.bitlinear_forward_workspace_layout.argtypes = [i64, i64, i64, ci, ctypes.POINTER(sz)]
    lib.bitlinear_set_tuning.restype = ci
    lib.bitlinear_set_tuning.argtypes = [ctypes.c_char_p]
    lib.bitlinear_status_string.restype = ctypes.c_char_p
    lib.bitlinear_status_string.argtypes = [ci]
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load_library().bitlinear_status_string(code).decode()


def _check(code: int, what: str) -> None:
    if code != BL_OK:
        raise BitLinearError(f"{what}: {status_string(code)} ({code})")


def _ptr(t: torch.Tensor | None, dtype=None):
    if t is None:
        return None
    if not t.is_cuda:
        raise BitLinearError("tensor is not on the GPU")
    if not t.is_contiguous():
        raise BitLinearError("tensor is not contiguous")
    if dtype is not None and t.dtype != dtype:
        raise BitLinearError(f"expected {dtype}, got {t.dtype}")
    return t.data_ptr()


def _stream():
    return torch.cuda.current_stream().cuda_stream


def _gran(per_tensor: bool) -> int:
    return GAMMA_PER_TENSOR if per_tensor else GAMMA_PER_TOKEN


def packed_bytes(N: int, K: int, flags: int = 0) -> int:
    return int(load_library().bitlinear_packed_bytes(N, K, flags))


def workspace_bytes(op: int, M: int, N: int, K: int, per_tensor: bool = False, flags: int = 0) -> int:
    return int(load_library().bitlinear_workspace_bytes(op, M, N, K, _gran(per_tensor), flags))


def set_tuning(spec: str | None = None) -> None:
    """Launch-time switches for tests and benchmarks ("name=value,..."; None resets)."""
    _check(load_library().bitlinear_set_tuning(None if spec is None else spec.encode()),
           "bitlinear_set_tuning")


def forward_workspace_layout(M: int, N: int, K: int, per_tensor: bool = False) -> dict:
    """Byte offsets of what bitlinear_forward leaves in its workspace (xhat: M = 1 only)."""
    off = (ctypes.c_size_t * 4)()
    _check(load_library().bitlinear_forward_workspace_layout(M, N, K, _gran(per_tensor), off),
           "bitlinear_forward_workspace_layout")
    return dict(codes=off[0], gamma=off[1], rowsum=off[2],
                xhat=None if off[3] == ctypes.c_size_t(-1).value else off[3])


def _workspace(nbytes: int, device) -> torch.Tensor:
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


def bitlinear_pack_weights(W: torch.Tensor, flags: int = 0, workspace: torch.Tensor | None = None):
    """Eq. 1-3, 12.  Returns (packed uint8 blob, alpha [1], beta [1]) on W's device."""
    lib = load_library()
    N, K = W.shape
    nbytes = packed_bytes(N, K, flags)
    if nbytes == 0:
        _check(-2, "bitlinear_pack_weights")
    packed = torch.empty(nbytes, dtype=torch.uint8, device=W.device)
    alpha = torch.empty(1, dtype=torch.float32, device=W.device)
    beta = torch.empty(1, dtype=torch.float32, device=W.device)
    ws = workspace if workspace is not None else _workspace(workspace_bytes(OP_PACK, 0, N, K), W.device)
    _check(lib.bitlinear_pack_weights(_ptr(W, torch.float32), N, K, flags, _ptr(packed), _ptr(alpha),
                                      _ptr(beta), _ptr(ws), ws.numel(), _stream()),
           "bitlinear_pack_weights")
    return packed, alpha, beta


def bitlinear_packed_to_canonical(packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    """Blob -> int32 tensor [N, K/32] holding the canonical uint32 words."""
    out = torch.empty((N, K // 32), dtype=torch.int32, device=packed.device)
    _check(load_library().bitlinear_packed_to_canonical(_ptr(packed), N, K, _ptr(out), _stream()),
           "bitlinear_packed_to_canonical")
    return out


def bitlinear_quant_act(X: torch.Tensor, ln_eps: float = 1e-5, per_tensor: bool = False,
                        flags: int = 0, ln_gain=None, ln_bias=None, want_xhat: bool = False,
                        workspace: torch.Tensor | None = None):
    """Eq. 12 + Eq. 4-5.  Returns (codes int8 [M,K], gamma, rowsum int32 [M], xhat or None)."""
    M, K = X.shape
    dev = X.device
    codes = torch.empty((M, K), dtype=torch.int8, device=dev)
    gamma = torch.empty(1 if per_tensor else max(M, 1), dtype=torch.float32, device=dev)
    rowsum = torch.empty(max(M, 1), dtype=torch.int32, device=dev)
    xhat = torch.empty((M, K), dtype=torch.float32, device=dev) if want_xhat else None
    ws = workspace if workspace is not None else _workspace(
        workspace_bytes(OP_QUANT, M, 1, K, per_tensor), dev)
    _check(load_library().bitlinear_quant_act(
        _ptr(X, torch.float32), M, K, _ptr(ln_gain, torch.float32), _ptr(ln_bias, torch.float32),
        ln_eps, _gran(per_tensor), flags, _ptr(codes), _ptr(gamma), _ptr(rowsum), _ptr(xhat),
        _ptr(ws), ws.numel(), _stream()), "bitlinear_quant_act")
    return codes, gamma, rowsum, xhat


def bitlinear_matmul(codes: torch.Tensor, gamma: torch.Tensor, rowsum: torch.Tensor,
                     packed: torch.Tensor, N: int, beta: torch.Tensor, per_tensor: bool = False,
                     flags: int = 0, out: torch.Tensor | None = None,
                     workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Eq. 7 + Eq. 11 on quantised activations.  fp32 [M,N], or int32 with FLAG_OUT_ACC_I32.
    `workspace` (workspace_bytes(OP_MATMUL, ...) bytes) is optional: see include/bitlinear.h."""
    M, K = codes.shape
    want_int = bool(flags & FLAG_OUT_ACC_I32)
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32 if want_int else torch.float32,
                          device=codes.device)
    _check(load_library().bitlinear_matmul(
        _ptr(codes, torch.int8), _ptr(gamma, torch.float32), _ptr(rowsum, torch.int32), M, K,
        _ptr(packed), N, _ptr(beta, torch.float32), _gran(per_tensor), flags, _ptr(out),
        _ptr(workspace), 0 if workspace is None else workspace.numel(), _stream()),
        "bitlinear_matmul")
    return out


def bitlinear_forward(X: torch.Tensor, packed: torch.Tensor, N: int, beta: torch.Tensor,
                      ln_eps: float = 1e-5, per_tensor: bool = False, flags: int = 0,
                      ln_gain=None, ln_bias=None, out: torch.Tensor | None = None,
                      workspace: torch.Tensor | None = None) -> torch.Tensor:
    """Eq. 11, the whole layer, from fp32 X [M,K] to fp32 Y [M,N]."""
    M, K = X.shape
    want_int = bool(flags & FLAG_OUT_ACC_I32)
    if out is None:
        out = torch.empty((M, N), dtype=torch.int32 if want_int else torch.float32, device=X.device)
    ws = workspace if workspace is not None else _workspace(
        workspace_bytes(OP_FORWARD, M, N, K, per_tensor), X.device)
    _check(load_library().bitlinear_forward(
        _ptr(X, torch.float32), M, K, _ptr(packed), N, _ptr(beta, torch.float32),
        _ptr(ln_gain, torch.float32), _ptr(ln_bias, torch.float32), ln_eps, _gran(per_tensor),
        flags, _ptr(out), _ptr(ws), ws.numel(), _stream()), "bitlinear_forward")
    return out


def bitlinear_forward_static(X: torch.Tensor, packed: torch.Tensor, N: int, beta: torch.Tensor,
                             out: torch.Tensor, ln_eps: float = 1e-5, per_tensor: bool = False,
                             flags: int = 0, ln_gain=None, ln_bias=None) -> torch.Tensor:
    """bitlinear_forward with the library's own scratch array: nothing is allocated, here or in
    the library (the caller brings the output)."""
    M, K = X.shape
    _check(load_library().bitlinear_forward_static(
        _ptr(X, torch.float32), M, K, _ptr(packed), N, _ptr(beta, torch.float32),
        _ptr(ln_gain, torch.float32), _ptr(ln_bias, torch.float32), ln_eps, _gran(per_tensor),
        flags, _ptr(out), _stream()), "bitlinear_forward_static")
    return out


def probe_read(buf: torch.Tensor, workgroups: int = 256, threads: int = 448) -> None:
    """One launch that only reads `buf` (see bitlinear_probe_read): the floor a weight-streaming
    kernel is measured against."""
    _check(load_library().bitlinear_probe_read(_ptr(buf), buf.numel() * buf.element_size(), workgroups,
                                               threads, None, _stream()), "bitlinear_probe_read")


def bitlinear_backward_ste(dY: torch.Tensor, codes: torch.Tensor, gamma: torch.Tensor,
                           packed: torch.Tensor | None, beta: torch.Tensor, per_tensor: bool,
                           want_dx: bool = True, want_dw: bool = True,
                           workspace: torch.Tensor | None = None):
    """Section 2.2 (STE).  Returns (dX fp32 [M,K] or None, dW fp32 [N,K] or None)."""
    M, N = dY.shape
    K = codes.shape[1]
    dev = dY.device
    dX = torch.empty((M, K), dtype=torch.float32, device=dev) if want_dx else None
    dW = torch.empty((N, K), dtype=torch.float32, device=dev) if want_dw else None
    ws = workspace if workspace is not None else _workspace(
        workspace_bytes(OP_BACKWARD, M, N, K, per_tensor), dev)
    _check(load_library().bitlinear_backward_ste(
        _ptr(dY, torch.float32), M, N, K, _ptr(codes, torch.int8), _ptr(gamma, torch.float32),
        _gran(per_tensor), _ptr(packed), _ptr(beta, torch.float32), _ptr(dX), _ptr(dW), _ptr(ws),
        ws.numel(), _stream()), "bitlinear_backward_ste")
    return dX, dW


# ---- Group Quantization and Normalization (Eq. 13-15) ----------------------------------
def packed_bytes_grouped(N: int, K: int, groups_n: int, groups_k: int) -> int:
    return int(load_library().bitlinear_packed_bytes_grouped(N, K, groups_n, groups_k))


def workspace_bytes_grouped(op: int, M: int, N: int, K: int, groups_n: int, groups_k: int,
                            per_tensor: bool = False) -> int:
    return int(load_library().bitlinear_workspace_bytes_grouped(op, M, N, K, groups_n, groups_k,
                                                                _gran(per_tensor)))


def bitlinear_pack_weights_grouped(W: torch.Tensor, groups_n: int = 1, groups_k: int = 1,
                                   flags: int = 0):
    """Eq. 13.  Returns (packed blob, alpha [groups_n, groups_k], beta [groups_n, groups_k])."""
    N, K = W.shape
    nbytes = packed_bytes_grouped(N, K, groups_n, groups_k)
    packed = torch.empty(max(nbytes, 1), dtype=torch.uint8, device=W.device)
    alpha = torch.empty((groups_n, groups_k), dtype=torch.float32, device=W.device)
    beta = torch.empty((groups_n, groups_k), dtype=torch.float32, device=W.device)
    ws = _workspace(workspace_bytes_grouped(OP_PACK, 0, N, K, groups_n, groups_k), W.device)
    _check(load_library().bitlinear_pack_weights_grouped(
        _ptr(W, torch.float32), N, K, groups_n, groups_k, flags, _ptr(packed), _ptr(alpha),
        _ptr(beta), _ptr(ws), ws.numel(), _stream()), "bitlinear_pack_weights_grouped")
    return packed, alpha, beta


def bitlinear_packed_to_canonical_grouped(packed: torch.Tensor, N: int, K: int,
                                          groups_k: int) -> torch.Tensor:
    out = torch.empty((N, K // 32), dtype=torch.int32, device=packed.device)
    _check(load_library().bitlinear_packed_to_canonical_grouped(
        _ptr(packed), N, K, groups_k, _ptr(out), _stream()), "bitlinear_packed_to_canonical_grouped")
    return out


def bitlinear_quant_act_grouped(X: torch.Tensor, groups_k: int, ln_eps: float = 1e-5,
                                per_tensor: bool = False, flags: int = 0, ln_gain=None,
                                ln_bias=None, want_xhat: bool = False):
    """Eq. 14-15.  Returns (codes [M,K], gamma [M,groups_k] or [groups_k], rowsum [M,groups_k],
    xhat or None)."""
    M, K = X.shape
    dev = X.device
    codes = torch.empty((M, K), dtype=torch.int8, device=dev)
    gamma = torch.empty((groups_k,) if per_tensor else (max(M, 1), groups_k), dtype=torch.float32,
                        device=dev)
    rowsum = torch.empty((max(M, 1), groups_k), dtype=torch.int32, device=dev)
    xhat = torch.empty((M, K), dtype=torch.float32, device=dev) if want_xhat else None
    ws = _workspace(workspace_bytes_grouped(OP_QUANT, M, 16, K, 1, groups_k, per_tensor), dev)
    _check(load_library().bitlinear_quant_act_grouped(
        _ptr(X, torch.float32), M, K, groups_k, _ptr(ln_gain, torch.float32),
        _ptr(ln_bias, torch.float32), ln_eps, _gran(per_tensor), flags, _ptr(codes), _ptr(gamma),
        _ptr(rowsum), _ptr(xhat), _ptr(ws), ws.numel(), _stream()), "bitlinear_quant_act_grouped")
    return codes, gamma, rowsum, xhat


def bitlinear_forward_grouped(X: torch.Tensor, packed: torch.Tensor, N: int, beta: torch.Tensor,
                              groups_n: int = 1, groups_k: int = 1, ln_eps: float = 1e-5,
                              per_tensor: bool = False, flags: int = 0, ln_gain=None, ln_bias=None,
                              out: torch.Tensor | None = None) -> torch.Tensor:
    """Eq. 11 with the group parameters of Eq. 13-15."""
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=X.device)
    ws = _workspace(workspace_bytes_grouped(OP_FORWARD, M, N, K, groups_n, groups_k, per_tensor),
                    X.device)
    _check(load_library().bitlinear_forward_grouped(
        _ptr(X, torch.float32), M, K, _ptr(packed), N, groups_n, groups_k,
        _ptr(beta, torch.float32), _ptr(ln_gain, torch.float32), _ptr(ln_bias, torch.float32),
        ln_eps, _gran(per_tensor), flags, _ptr(out), _ptr(ws), ws.numel(), _stream()),
        "bitlinear_forward_grouped")
    return out


def bitlinear_layernorm_backward(dXhat: torch.Tensor, X: torch.Tensor, ln_eps: float = 1e-5,
                                 ln_gain=None, groups_k: int = 1, want_affine: bool = False,
                                 out: torch.Tensor | None = None):
    """Backward of Eq. 12 / Eq. 15.  Returns dX, or (dX, dgain, dbias) with want_affine."""
    M, K = X.shape
    dev = X.device
    dX = out if out is not None else torch.empty((M, K), dtype=torch.float32, device=dev)
    dgain = torch.empty(K, dtype=torch.float32, device=dev) if want_affine else None
    dbias = torch.empty(K, dtype=torch.float32, device=dev) if want_affine else None
    ws = _workspace(workspace_bytes_grouped(OP_LN_BACKWARD, M, 16, K, 1, groups_k), dev)
    _check(load_library().bitlinear_layernorm_backward(
        _ptr(dXhat, torch.float32), _ptr(X, torch.float32), M, K, groups_k,
        _ptr(ln_gain, torch.float32), ln_eps, _ptr(dX, torch.float32), _ptr(dgain), _ptr(dbias),
        _ptr(ws), ws.numel(), _stream()), "bitlinear_layernorm_backward")
    return (dX, dgain, dbias) if want_affine else dX


# ---- Eq. 6: the non-negative quantiser --------------------------------------------------
def bitlinear_weight_rowsums(packed: torch.Tensor, N: int, K: int) -> torch.Tensor:
    """wsum[n] = sum_k W~[n,k], int32 [N]."""
    out = torch.empty(N, dtype=torch.int32, device=packed.device)
    _check(load_library().bitlinear_weight_rowsums(_ptr(packed), N, K, _ptr(out), _stream()),
           "bitlinear_weight_rowsums")
    return out


def bitlinear_quant_act_nonneg(X: torch.Tensor, ln_eps: float = 1e-5, flags: int = 0, ln_gain=None,
                               ln_bias=None, want_xhat: bool = False, per_tensor: bool = False,
                               groups_k: int = 1):
    """Eq. 12 + Eq. 6 (per K-group: Eq. 14-15).  Returns (codes in 0..127, gamma, eta, rowsum, xhat or
    None); gamma and eta are [M, groups_k] per token, [groups_k] per tensor (flat for one group)."""
    M, K = X.shape
    dev = X.device
    codes = torch.empty((M, K), dtype=torch.int8, device=dev)
    n_par = groups_k if per_tensor else max(M, 1) * groups_k
    gamma = torch.empty(n_par, dtype=torch.float32, device=dev)
    eta = torch.empty(n_par, dtype=torch.float32, device=dev)
    rowsum = torch.empty(max(M, 1) * groups_k, dtype=torch.int32, device=dev)
    xhat = torch.empty((M, K), dtype=torch.float32, device=dev) if want_xhat else None
    ws = _workspace(workspace_bytes_grouped(OP_QUANT, M, 16, K, 1, groups_k, per_tensor), dev)
    lib = load_library()
    if groups_k == 1:
        _check(lib.bitlinear_quant_act_nonneg(
            _ptr(X, torch.float32), M, K, _ptr(ln_gain, torch.float32), _ptr(ln_bias, torch.float32),
            ln_eps, _gran(per_tensor), flags, _ptr(codes), _ptr(gamma), _ptr(eta), _ptr(rowsum),
            _ptr(xhat), _ptr(ws), ws.numel(), _stream()), "bitlinear_quant_act_nonneg")
    else:
        _check(lib.bitlinear_quant_act_grouped_nonneg(
            _ptr(X, torch.float32), M, K, groups_k, _ptr(ln_gain, torch.float32),
            _ptr(ln_bias, torch.float32), ln_eps, _gran(per_tensor), flags, _ptr(codes), _ptr(gamma),
            _ptr(eta), _ptr(rowsum), _ptr(xhat), _ptr(ws), ws.numel(), _stream()),
            "bitlinear_quant_act_grouped_nonneg")
    if groups_k > 1:
        shape = (groups_k,) if per_tensor else (max(M, 1), groups_k)
        gamma, eta, rowsum = gamma.view(shape), eta.view(shape), rowsum.view(max(M, 1), groups_k)
    return codes, gamma, eta, rowsum, xhat


def bitlinear_weight_rowsums_grouped(packed: torch.Tensor, N: int, K: int, groups_k: int) -> torch.Tensor:
    """wsum[g][n] = sum of W~[n, k] over the columns of K-group g, int32 [groups_k, N]."""
    out = torch.empty((groups_k, N), dtype=torch.int32, device=packed.device)
    _check(load_library().bitlinear_weight_rowsums_grouped(_ptr(packed), N, K, groups_k, _ptr(out),
                                                           _stream()), "bitlinear_weight_rowsums_grouped")
    return out


def bitlinear_matmul_nonneg(codes, gamma, eta, rowsum, packed, N: int, beta, wsum,
                            out: torch.Tensor | None = None, per_tensor: bool = False) -> torch.Tensor:
    M, K = codes.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=codes.device)
    _check(load_library().bitlinear_matmul_nonneg(
        _ptr(codes, torch.int8), _ptr(gamma, torch.float32), _ptr(eta, torch.float32),
        _ptr(rowsum, torch.int32), M, K, _ptr(packed), N, _ptr(beta, torch.float32),
        _ptr(wsum, torch.int32), _gran(per_tensor), 0, _ptr(out), _stream()),
        "bitlinear_matmul_nonneg")
    return out


def bitlinear_forward_nonneg(X: torch.Tensor, packed: torch.Tensor, N: int, beta: torch.Tensor,
                             wsum: torch.Tensor, ln_eps: float = 1e-5, flags: int = 0, ln_gain=None,
                             ln_bias=None, out: torch.Tensor | None = None, per_tensor: bool = False,
                             groups_n: int = 1, groups_k: int = 1) -> torch.Tensor:
    """Eq. 11 with the quantiser of Eq. 6 (with groups: Eq. 13-15, eta_g per K-group)."""
    M, K = X.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32, device=X.device)
    ws = _workspace(workspace_bytes_grouped(OP_FORWARD_NONNEG, M, N, K, groups_n, groups_k, per_tensor),
                    X.device)
    lib = load_library()
    if groups_n == 1 and groups_k == 1:
        _check(lib.bitlinear_forward_nonneg(
            _ptr(X, torch.float32), M, K, _ptr(packed), N, _ptr(beta, torch.float32),
            _ptr(wsum, torch.int32), _ptr(ln_gain, torch.float32), _ptr(ln_bias, torch.float32), ln_eps,
            _gran(per_tensor), flags, _ptr(out), _ptr(ws), ws.numel(), _stream()),
            "bitlinear_forward_nonneg")
    else:
        _check(lib.bitlinear_forward_grouped_nonneg(
            _ptr(X, torch.float32), M, K, _ptr(packed), N, groups_n, groups_k,
            _ptr(beta, torch.float32), _ptr(wsum, torch.int32), _ptr(ln_gain, torch.float32),
            _ptr(ln_bias, torch.float32), ln_eps, _gran(per_tensor), flags, _ptr(out), _ptr(ws),
            ws.numel(), _stream()), "bitlinear_forward_grouped_nonneg")
    return out
