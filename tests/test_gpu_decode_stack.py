"""GPU parity of the one-launch layer chain (bitlinear_decode_stack) against the same chain run
layer by layer through bitlinear_forward, which the other parity tests tie to the CPU oracle
(Eq. 12, 4-5, 7, 11 of arXiv 2310.11453).  The chain kernel quantises with the reduction order of
the stand-alone quantiser at 4 waves per row (8 for K > 16384); BITLINEAR_QUANT_WPR pins the
stand-alone side to that order, so the comparison is exact: every output bit."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def bl():
    import paper_2310_11453_amd as lib
    lib.load_library()
    assert torch.cuda.is_available()
    return lib


def make_layers(bl, dims, seed):
    """dims: [(K, N), ...]; returns [(packed, beta, N, K)] and the fp32 weights."""
    layers, Ws = [], []
    for i, (K, N) in enumerate(dims):
        W = wl.make_weight(N, K, 0.02, wl.seed_for(7, seed + i))
        packed, alpha, beta = bl.bitlinear_pack_weights(torch.from_numpy(W).cuda())
        layers.append((packed, beta, N, K))
        Ws.append(W)
    return layers, Ws


def chain_reference(bl, X, layers):
    h = X
    outs = []
    for (packed, beta, N, K) in layers:
        x_in = h[:, :K].contiguous()
        h = bl.bitlinear_forward(x_in, packed, N, beta)
        outs.append(h)
    return outs


# (M, [(K, N), ...]): one chunk per wave and 8-way tile split (K=256); 4 chunks (K=2048); odd chunk
# count (K=2080 -> 5); two chunks per wave, 7 and 8 waves (K=7168, 8192); two rounds (K=16384);
# ragged N (520), N smaller than the grid (64), a layer narrower than its input (K < previous N)
CHAINS = [
    (1, [(256, 512), (512, 256)]),
    (4, [(2048, 6144), (2048, 2048), (2048, 8192), (8192, 2048)]),
    (2, [(2080, 520), (512, 64), (64, 1040)]),
    (1, [(7168, 21504), (7168, 7168), (7168, 28672)]),
    (3, [(16384, 4096), (4096, 16384)]),
    (16, [(2048, 2048), (2048, 4096), (4096, 1024)]),
]


@pytest.mark.parametrize("M,dims", CHAINS)
def test_stack_equals_layer_by_layer(bl, monkeypatch, M, dims):
    print(f"decode stack M={M} dims={dims}", flush=True)
    monkeypatch.setenv("BITLINEAR_QUANT_WPR", "4")
    layers, _ = make_layers(bl, dims, M)
    X = torch.from_numpy(wl.make_activation(M, dims[0][0], wl.seed_for(7, 99 + M))).cuda()
    ref = chain_reference(bl, X, layers)
    stack = bl.DecodeStack(layers, M)
    Y = bl.bitlinear_decode_stack(X, stack)
    assert not stack.barrier_failed()
    assert torch.equal(Y, ref[-1])
    # a second call on the same table and workspace gives the same bits
    Y2 = bl.bitlinear_decode_stack(X, stack)
    assert not stack.barrier_failed()
    assert torch.equal(Y2, Y)


def test_stack_long_k_eight_waves_per_row(bl, monkeypatch):
    """K = 28672 (the 30B down projection): 8 waves per row in both quantisers (a row of that
    length does not fit 4, so the override below does not apply to it), four rounds of K."""
    M, dims = 2, [(7168, 28672), (28672, 7168)]
    print(f"decode stack M={M} dims={dims}", flush=True)
    monkeypatch.setenv("BITLINEAR_QUANT_WPR", "4")
    layers, _ = make_layers(bl, dims, 40)
    X = torch.from_numpy(wl.make_activation(M, 7168, wl.seed_for(7, 41))).cuda()
    ref = chain_reference(bl, X, layers)
    stack = bl.DecodeStack(layers, M)
    Y = bl.bitlinear_decode_stack(X, stack)
    assert not stack.barrier_failed()
    assert torch.equal(Y, ref[-1])


def test_stack_single_layer_against_oracle(bl, monkeypatch):
    """One layer straight against the CPU oracle: codes from the oracle's quantiser applied to the
    GPU's normalised input, integer GEMM and dequantisation in the oracle."""
    M, K, N = 4, 2048, 1536
    print(f"decode stack vs oracle M={M} K={K} N={N}", flush=True)
    monkeypatch.setenv("BITLINEAR_QUANT_WPR", "4")
    layers, Ws = make_layers(bl, [(K, N)], 60)
    Xh = wl.make_activation(M, K, wl.seed_for(7, 61))
    X = torch.from_numpy(Xh).cuda()
    stack = bl.DecodeStack(layers, M)
    Y = bl.bitlinear_decode_stack(X, stack).cpu().numpy()
    assert not stack.barrier_failed()
    _, _, _, xhat = bl.bitlinear_quant_act(X, want_xhat=True)
    xh = xhat.cpu().numpy()
    g = oracle.absmax(xh)
    q = oracle.quantize(xh, g)
    a, b = oracle.weight_stats(Ws[0])
    acc = oracle.matmul_i32(q, oracle.binarize(Ws[0], a))
    y_ref = oracle.dequant(acc, g, b)
    assert np.array_equal(Y, y_ref)
