"""GPU parity of the straight-through-estimator backward (Section 2.2 of arXiv 2310.11453)
against the CPU oracle: same bf16-rounded dY on both sides, fp32 accumulation on the GPU
against fp64 in the oracle.  Bar: relative Frobenius error <= 1e-3 (measured ~1e-6) and
max error <= 1e-3 of the rms."""
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


def close(a, ref):
    ref64 = ref.astype(np.float64)
    rms = np.sqrt(np.mean(ref64 ** 2)) + 1e-30
    assert np.linalg.norm(a - ref64) <= 1e-3 * np.linalg.norm(ref64) + 1e-30
    assert np.abs(a - ref64).max() <= 1e-3 * rms


# several tiles with ragged tails in every dimension, and both granularities of gamma
SHAPES = [(8, 512, 256), (12, 20, 64), (300, 200, 96), (64, 136, 1056), (257, 513, 544),
          (1024, 640, 512)]


# The library picks the GEMM kernel from the shape (the persistent 256 x 256 ring kernel needs
# many tiles); the bwd_ring switch forces either one so that both see the ragged shapes.
@pytest.mark.parametrize("M,N,K", SHAPES)
@pytest.mark.parametrize("per_tensor", [True, False])
@pytest.mark.parametrize("ring", ["2", "1"])
def test_backward_ste_matches_oracle(bl, tuning, M, N, K, per_tensor, ring):
    print(f"backward M={M} N={N} K={K} per_tensor={per_tensor} ring={ring}", flush=True)
    tuning(f"bwd_ring={ring}")
    sd = wl.seed_for(4, M + N + K)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    dY = wl.make_grad(M, N, sd)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X), per_tensor=per_tensor)
    dX, dW = bl.bitlinear_backward_ste(dev(dY), codes, gamma, packed, beta, per_tensor)
    sign = oracle.unpack_canonical(
        bl.bitlinear_packed_to_canonical(packed, N, K).cpu().numpy().view(np.uint32), K)
    dX_ref, dW_ref = oracle.backward_ste(dY, codes.cpu().numpy(), gamma.cpu().numpy(), sign,
                                         float(beta.cpu()[0]), per_tensor)
    close(dX.cpu().numpy(), dX_ref)
    close(dW.cpu().numpy(), dW_ref)
    # either output alone
    dX2, none = bl.bitlinear_backward_ste(dev(dY), codes, gamma, packed, beta, per_tensor,
                                          want_dw=False)
    assert none is None and torch.equal(dX2, dX)
    none, dW2 = bl.bitlinear_backward_ste(dev(dY), codes, gamma, None, beta, per_tensor,
                                          want_dx=False)
    assert none is None and torch.equal(dW2, dW)


def test_backward_ring_kernel_walks_several_tiles(bl, tuning):
    """The persistent kernel with fewer workgroups than tiles (the bwd_grid switch): dX has 16
    tiles on 8 workgroups (the tile order that groups tiles by L2 applies), dW 12 on 8."""
    tuning("bwd_ring=1,bwd_grid=8")
    M, N, K = 1024, 520, 1024
    sd = wl.seed_for(4, 77)
    print(f"backward ring grid=8 M={M} N={N} K={K}", flush=True)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    dY = wl.make_grad(M, N, sd)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X), per_tensor=False)
    dX, dW = bl.bitlinear_backward_ste(dev(dY), codes, gamma, packed, beta, False)
    sign = oracle.unpack_canonical(
        bl.bitlinear_packed_to_canonical(packed, N, K).cpu().numpy().view(np.uint32), K)
    dX_ref, dW_ref = oracle.backward_ste(dY, codes.cpu().numpy(), gamma.cpu().numpy(), sign,
                                         float(beta.cpu()[0]), False)
    close(dX.cpu().numpy(), dX_ref)
    close(dW.cpu().numpy(), dW_ref)


@pytest.mark.parametrize("ring", ["2", "1"])
def test_backward_exact_when_dy_is_bf16_representable(bl, tuning, ring):
    """Small integers in dY, codes and signs: every product and partial sum is exact in fp32,
    so the GPU must reproduce the integer result bit for bit (catches layout mistakes that a
    tolerance would hide)."""
    tuning(f"bwd_ring={ring}")
    M, N, K = 96, 80, 160
    rng = np.random.default_rng(3)
    W = wl.make_weight(N, K, 0.02, 5)
    X = wl.make_activation(M, K, 5)
    dY = rng.integers(-4, 5, (M, N)).astype(f32)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X), per_tensor=True)
    one = torch.ones(1, device="cuda")
    g128 = torch.full((1,), 128.0, device="cuda")
    dX, dW = bl.bitlinear_backward_ste(dev(dY), codes, g128, packed, one, True)
    sign = oracle.unpack_canonical(
        bl.bitlinear_packed_to_canonical(packed, N, K).cpu().numpy().view(np.uint32), K)
    q = codes.cpu().numpy().astype(np.int64)
    assert np.array_equal(dX.cpu().numpy(), (dY.astype(np.int64) @ sign.astype(np.int64)).astype(f32))
    assert np.array_equal(dW.cpu().numpy(), (dY.astype(np.int64).T @ q).astype(f32))


def test_backward_training_shape_sampled(bl):
    """Training-step shape (M=8192, 4096->16384, per-tensor gamma): sampled rows of dX and dW
    against the oracle."""
    M, K, N = 8192, 4096, 16384
    sd = wl.seed_for(4, 0)
    print(f"backward full M={M} N={N} K={K}", flush=True)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    dY = wl.make_grad(M, N, sd)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    a, b = oracle.weight_stats(W)
    sign = oracle.binarize(W, a)
    del W
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X), per_tensor=True)
    del X
    dX, dW = bl.bitlinear_backward_ste(dev(dY), codes, gamma, packed, beta, True)
    rng = np.random.default_rng(11)
    rows_dx = np.concatenate([[0, 1, 4097, 8191], rng.integers(0, M, 12)])
    rows_dw = np.concatenate([[0, 255, 256, 16383], rng.integers(0, N, 12)])
    dX_ref, dW_ref = oracle.backward_ste(dY, codes.cpu().numpy(), gamma.cpu().numpy(), sign,
                                         float(b), True, rows_dx=rows_dx, rows_dw=rows_dw)
    close(dX.cpu().numpy()[rows_dx], dX_ref)
    close(dW.cpu().numpy()[rows_dw], dW_ref)
