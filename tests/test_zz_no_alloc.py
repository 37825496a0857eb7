"""The entry point that allocates nothing (bitlinear_forward_static: the library's own scratch
array in place of a workspace argument) against bitlinear_forward, through the C ABI: same
result bit for bit, on calls in a row that share the array, the later ones smaller."""
import ctypes

import numpy as np
import pytest
import torch

import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bl():
    import paper_2310_11453_amd as lib
    lib.load_library()
    assert torch.cuda.is_available()
    return lib


def _raw_static(bl, X, packed, N, beta, out, per_tensor=False, flags=0):
    """The raw C call: device pointers and sizes, no workspace, the current stream."""
    M, K = X.shape
    return bl.load_library().bitlinear_forward_static(
        ctypes.c_void_p(X.data_ptr()), M, K, ctypes.c_void_p(packed.data_ptr()), N,
        ctypes.c_void_p(beta.data_ptr()), None, None, 1e-5, int(per_tensor), flags,
        ctypes.c_void_p(out.data_ptr()), ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))


# in this order: a K split over workgroups (partial sums in the scratch array), then smaller
# inputs that reuse the array's front while its back still holds the earlier call's bytes
CALLS = [(64, 7168, 2048, False), (4, 2048, 512, False), (1, 2048, 512, False),
         (24, 1056, 300, True), (16, 28672, 520, False), (3, 96, 40, True)]


def test_static_scratch_matches_workspace_forward(bl):
    layers = []
    for i, (M, K, N, pt) in enumerate(CALLS):
        W = torch.from_numpy(wl.make_weight(N, K, 0.02, wl.seed_for(0, 900 + i))).cuda()
        X = torch.from_numpy(wl.make_activation(M, K, wl.seed_for(0, 950 + i))).cuda()
        packed, alpha, beta = bl.bitlinear_pack_weights(W)
        ref = bl.bitlinear_forward(X, packed, N, beta, per_tensor=pt)
        ref_acc = bl.bitlinear_forward(X, packed, N, beta, per_tensor=pt, flags=bl.FLAG_OUT_ACC_I32)
        layers.append((M, K, N, pt, X, packed, beta, ref, ref_acc))
    torch.cuda.synchronize()
    for rounds in range(2):  # the second round finds the array as the first left it
        for (M, K, N, pt, X, packed, beta, ref, ref_acc) in layers:
            print(f"static scratch M={M} K={K} N={N} per_tensor={pt}", flush=True)
            out = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            assert _raw_static(bl, X, packed, N, beta, out, pt) == 0
            assert torch.equal(out, ref)
            acc = torch.zeros((M, N), dtype=torch.int32, device="cuda")
            assert _raw_static(bl, X, packed, N, beta, acc, pt, bl.FLAG_OUT_ACC_I32) == 0
            assert torch.equal(acc, ref_acc)


def test_static_scratch_binding_and_limits(bl):
    M, K, N = 8, 256, 512
    W = torch.from_numpy(wl.make_weight(N, K, 0.02, 1)).cuda()
    X = torch.from_numpy(wl.make_activation(M, K, 2)).cuda()
    packed, alpha, beta = bl.bitlinear_pack_weights(W)
    out = torch.empty((M, N), dtype=torch.float32, device="cuda")
    assert torch.equal(bl.bitlinear_forward_static(X, packed, N, beta, out),
                       bl.bitlinear_forward(X, packed, N, beta))
    # M = 0 is a no-op; a workspace beyond 16 MiB is refused on the host, before any launch
    one = ctypes.c_void_p(256)
    lib = bl.load_library()
    assert lib.bitlinear_forward_static(one, 0, K, one, N, one, None, None, 1e-5, 0, 0, one, None) == 0
    assert bl.workspace_bytes(bl.OP_FORWARD, 4096, 7168, 7168) > (16 << 20)
    assert lib.bitlinear_forward_static(one, 4096, 7168, one, 7168, one, None, None, 1e-5, 0, 0, one,
                                        None) == -3
    assert lib.bitlinear_forward_static(one, 4, 48, one, N, one, None, None, 1e-5, 0, 0, one, None) == -2
    assert lib.bitlinear_forward_static(None, 4, 64, one, N, one, None, None, 1e-5, 0, 0, one, None) == -1
