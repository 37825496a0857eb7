"""GPU parity: the HIP path, called through the C ABI binding, against the CPU oracle.

Integer results (packed bits, int8 codes, int32 accumulators) must be bit-exact; codes are
compared "given the same normalised input" (the oracle quantises the x^ the GPU dumped) and,
separately, x^ itself is compared with the oracle's fp64 LayerNorm.  fp32 outputs: exact
given shared codes/gamma/beta (the epilogue is one fp32 multiply on both sides), and
within 1e-3 relative (Frobenius, and max error against rms) end to end.
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


# ------------------------------------------------------------------ weights (Eq. 1-3, 12)
PACK_SHAPES = [(512, 256), (3, 32), (16, 512), (17, 544), (200, 96), (100, 1056), (2048, 2048)]


@pytest.mark.parametrize("N,K", PACK_SHAPES)
@pytest.mark.parametrize("mean", [0.0, 0.04])
def test_pack_bits_alpha_beta(bl, N, K, mean):
    print(f"pack N={N} K={K} mean={mean}", flush=True)
    W = wl.make_weight(N, K, 0.02, seed=wl.seed_for(0, N + K), mean=mean)
    a, b = oracle.weight_stats(W)
    words = oracle.pack_canonical(oracle.binarize(W, a))
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    canon = host(bl.bitlinear_packed_to_canonical(packed, N, K)).view(np.uint32)
    assert host(alpha)[0] == a and host(beta)[0] == b
    assert np.array_equal(canon, words)
    _, _, beta_c = bl.bitlinear_pack_weights(dev(W), flags=bl.FLAG_BETA_CENTERED)
    assert host(beta_c)[0] == oracle.weight_stats(W, beta_centered=True)[1]


def test_pack_constant_weight_sign_zero(bl):
    W = np.full((40, 64), 0.03125, f32)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    assert host(alpha)[0] == f32(0.03125) and host(beta)[0] == f32(0.03125)
    assert not host(bl.bitlinear_packed_to_canonical(packed, 40, 64)).any()


def test_pack_deterministic(bl):
    W = dev(wl.make_weight(1000, 2080, 0.02, seed=5))
    p1, a1, b1 = bl.bitlinear_pack_weights(W)
    p2, a2, b2 = bl.bitlinear_pack_weights(W)
    assert torch.equal(p1, p2) and torch.equal(a1, a2) and torch.equal(b1, b2)


# ------------------------------------------------------------------ activations (Eq. 12, 4, 5)
QUANT_SHAPES = [(8, 256), (1, 2048), (5, 96), (3, 544), (16, 8192), (33, 4096), (7, 7168),
                (2, 28672), (4, 16384), (64, 1024),
                # rows longer than the registers hold: walked from memory in passes
                (3, 36000), (2, 65536), (5, 32800)]


@pytest.mark.parametrize("M,K", QUANT_SHAPES)
@pytest.mark.parametrize("per_tensor", [False, True])
def test_quant_codes_bit_exact_given_xhat(bl, M, K, per_tensor):
    print(f"quant M={M} K={K} per_tensor={per_tensor}", flush=True)
    X = wl.make_activation(M, K, wl.seed_for(1, M + K), outlier_p=0.001, outlier_mul=20.0)
    X = X * f32(1.7) + f32(0.3)
    codes, gamma, rowsum, xhat = bl.bitlinear_quant_act(dev(X), 1e-5, per_tensor, want_xhat=True)
    xh_gpu = host(xhat)
    g_ref = oracle.absmax(xh_gpu, per_tensor)
    assert np.array_equal(host(gamma), g_ref)
    q_ref = oracle.quantize(xh_gpu, g_ref, per_tensor)
    assert np.array_equal(host(codes), q_ref)
    assert np.array_equal(host(rowsum)[:M], q_ref.astype(np.int64).sum(1))
    xh_ref = oracle.layernorm(X, 1e-5)
    assert np.abs(xh_gpu - xh_ref).max() <= 2e-6 * max(1.0, np.abs(xh_ref).max())
    # end to end from raw X: the fp64 LayerNorm on both sides rounds to the same fp32
    q_e2e = oracle.quantize(xh_ref, oracle.absmax(xh_ref, per_tensor), per_tensor)
    mism = int((host(codes) != q_e2e).sum())
    assert mism <= max(1, M * K // 100000), f"{mism} codes differ end to end"


def test_quant_skip_ln_ties_clip_zero_row_affine(bl):
    row = np.zeros((3, 32), f32)
    row[0, :8] = [1, 1 / 256, 3 / 256, 5 / 256, -1 / 256, -3 / 256, -1, 127.5 / 128]
    row[2] = wl.make_activation(1, 32, 3)[0]
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(row), flags=bl.FLAG_SKIP_LN)
    c = host(codes)
    assert c[0, :8].tolist() == [127, 0, 2, 2, 0, -2, -128, 127]
    assert not c[1].any() and host(gamma)[1] == f32(1e-5)
    g = oracle.absmax(row)
    assert np.array_equal(c, oracle.quantize(row, g)) and np.array_equal(host(gamma), g)
    # constant row through LN: normalises to zero
    X = np.full((2, 64), 3.25, f32)
    codes, gamma, _, _ = bl.bitlinear_quant_act(dev(X))
    assert not host(codes).any() and (host(gamma) == f32(1e-5)).all()
    # affine LN
    X = wl.make_activation(6, 320, 9)
    gain = np.linspace(0.5, 1.5, 320).astype(f32)
    bias = np.linspace(-1, 1, 320).astype(f32)
    codes, gamma, _, xhat = bl.bitlinear_quant_act(dev(X), ln_gain=dev(gain), ln_bias=dev(bias),
                                                   want_xhat=True)
    ref = oracle.layernorm(X, 1e-5, gain, bias)
    assert np.abs(host(xhat) - ref).max() <= 4e-6
    assert np.array_equal(host(codes), oracle.quantize(host(xhat), host(gamma)))
    # the same three variants on rows walked from memory (K > 32768)
    K = 36000
    X = wl.make_activation(3, K, 10)
    gain = np.linspace(0.5, 1.5, K).astype(f32)
    bias = np.linspace(-1, 1, K).astype(f32)
    for kw, ref in ((dict(ln_gain=dev(gain), ln_bias=dev(bias)), oracle.layernorm(X, 1e-5, gain, bias)),
                    (dict(flags=bl.FLAG_SKIP_LN), X), (dict(per_tensor=True), oracle.layernorm(X))):
        codes, gamma, rowsum, xhat = bl.bitlinear_quant_act(dev(X), want_xhat=True, **kw)
        pt = bool(kw.get("per_tensor"))
        assert np.abs(host(xhat) - ref).max() <= 4e-6 * max(1.0, np.abs(ref).max())
        g = oracle.absmax(host(xhat), pt)
        assert np.array_equal(host(gamma), g)
        q = oracle.quantize(host(xhat), g, pt)
        assert np.array_equal(host(codes), q)
        assert np.array_equal(host(rowsum)[:3], q.astype(np.int64).sum(1))


# ------------------------------------------------------------------ matmul (Eq. 7, 11)
# (M, K, N): decode path (M <= 16) and MFMA-tiled path (M > 16); several tiles + ragged tails
GEMM_SHAPES = [(8, 256, 512), (1, 2048, 2048), (4, 96, 40), (16, 544, 200), (13, 1056, 72),
               (3, 8192, 64), (16, 7168, 96), (2, 16384, 48), (5, 28672, 32), (1, 2048, 6144),
               (17, 256, 512), (70, 544, 200), (64, 1056, 136), (300, 96, 260), (256, 2048, 384),
               (513, 1024, 130),
               # 16 < M <= 64 (K split four ways inside the workgroup): fewer chunks than groups,
               # odd N, exact tiles, a long ragged K
               (33, 32, 20), (48, 3616, 257), (64, 2048, 128), (20, 7200, 264)]


@pytest.mark.parametrize("M,K,N", GEMM_SHAPES)
def test_matmul_acc_bit_exact_and_y(bl, M, K, N):
    print(f"matmul M={M} K={K} N={N}", flush=True)
    sd = wl.seed_for(2, M + K + N)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X))
    sign = oracle.unpack_canonical(host(bl.bitlinear_packed_to_canonical(packed, N, K)).view(np.uint32), K)
    acc_ref = oracle.matmul_i32(host(codes), sign)
    acc = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta, flags=bl.FLAG_OUT_ACC_I32)
    assert np.array_equal(host(acc), acc_ref)
    y = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta)
    y_ref = oracle.dequant(acc_ref, host(gamma), host(beta))
    assert np.array_equal(host(y), y_ref)  # one fp32 multiply per output on both sides
    # extreme codes: every product has the same sign, |acc| = 128 K
    q = torch.full((M, K), -128, dtype=torch.int8, device="cuda")
    rs = torch.full((M,), -128 * K, dtype=torch.int32, device="cuda")
    acc = bl.bitlinear_matmul(q, gamma, rs, packed, N, beta, flags=bl.FLAG_OUT_ACC_I32)
    assert np.array_equal(host(acc), np.repeat((-128 * sign.astype(np.int64).sum(1))[None], M, 0))


def _random_shapes(n, seed):
    """Seeded shapes across the three GEMM kernels' ranges of M, with K a multiple of 32 and any N."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        M = int(rng.choice([rng.integers(1, 17), rng.integers(17, 65), rng.integers(65, 400)]))
        K = 32 * int(rng.integers(1, 130))
        N = int(rng.integers(1, 700))
        out.append((M, K, N))
    return out


@pytest.mark.parametrize("M,K,N", _random_shapes(24, 20231011))
def test_matmul_random_shapes(bl, M, K, N):
    """Accumulators and outputs on seeded random shapes: whichever kernel the batch size selects
    (streaming, mid-batch, large tiles), with and without the workspace that allows a K split."""
    print(f"matmul random M={M} K={K} N={N}", flush=True)
    sd = wl.seed_for(2, 7 * M + 3 * K + N)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X))
    sign = oracle.unpack_canonical(host(bl.bitlinear_packed_to_canonical(packed, N, K)).view(np.uint32), K)
    acc_ref = oracle.matmul_i32(host(codes), sign)
    y_ref = oracle.dequant(acc_ref, host(gamma), host(beta))
    ws = torch.empty(max(256, bl.workspace_bytes(bl.OP_MATMUL, M, N, K)), dtype=torch.uint8, device="cuda")
    for workspace in (None, ws):
        acc = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta, flags=bl.FLAG_OUT_ACC_I32,
                                  workspace=workspace)
        assert np.array_equal(host(acc), acc_ref)
        y = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta, workspace=workspace)
        assert np.array_equal(host(y), y_ref)


# 17 to 32 tokens (weights streamed through registers): N not a multiple of 4 (element-wise
# stores), one to four pairs of tiles per workgroup, 1 / 5 / 7 / 8 waves, chunks spread unevenly
# over the waves, a K long enough for two slices, and a shape the kernel hands to the mid-batch one
STREAM_SHAPES = [(17, 512, 30), (32, 1056, 37), (25, 4608, 8200), (31, 1024, 32768), (24, 7168, 1536),
                 (32, 4096, 24000), (19, 8704, 520), (32, 16384, 1024), (18, 28672, 7168)]


@pytest.mark.parametrize("M,K,N", STREAM_SHAPES)
def test_matmul_17_to_32_tokens(bl, M, K, N):
    print(f"matmul stream M={M} K={K} N={N}", flush=True)
    sd = wl.seed_for(2, 11 * M + K + N)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X))
    sign = oracle.unpack_canonical(host(bl.bitlinear_packed_to_canonical(packed, N, K)).view(np.uint32), K)
    acc_ref = oracle.matmul_i32(host(codes), sign)
    y_ref = oracle.dequant(acc_ref, host(gamma), host(beta))
    ws = torch.empty(max(256, bl.workspace_bytes(bl.OP_MATMUL, M, N, K)), dtype=torch.uint8, device="cuda")
    for workspace in (None, ws):
        acc = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta, flags=bl.FLAG_OUT_ACC_I32,
                                  workspace=workspace)
        assert np.array_equal(host(acc), acc_ref)
        y = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta, workspace=workspace)
        assert np.array_equal(host(y), y_ref)


@pytest.mark.parametrize("M,K,N,per_tensor", [(8, 256, 512, False), (8, 256, 512, True),
                                              (16, 2048, 2048, False), (130, 512, 272, True),
                                              (24, 1056, 300, True), (48, 1056, 300, True),
                                              (40, 1024, 1000, False),
                                              # K beyond the register-resident quantiser
                                              (3, 36000, 48, False), (20, 40960, 130, True),
                                              (100, 33792, 96, False)])
def test_forward_end_to_end(bl, M, K, N, per_tensor):
    print(f"forward M={M} K={K} N={N} per_tensor={per_tensor}", flush=True)
    sd = wl.seed_for(0, M + K + N)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    r = oracle.forward(X, W, per_tensor=per_tensor)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    y = host(bl.bitlinear_forward(dev(X), packed, N, beta, per_tensor=per_tensor))
    rms = np.sqrt(np.mean(r["y"].astype(np.float64) ** 2))
    assert np.abs(y - r["y"]).max() <= 1e-3 * rms
    assert np.linalg.norm(y - r["y"]) <= 1e-3 * np.linalg.norm(r["y"])
    acc = host(bl.bitlinear_forward(dev(X), packed, N, beta, per_tensor=per_tensor,
                                    flags=bl.FLAG_OUT_ACC_I32))
    assert (acc != r["acc"]).mean() <= 1e-3  # differs only where an x^ sits on a rounding tie


# One token: the small-batch GEMM kernel normalises and quantises the row itself (one launch).
# K below one chunk, one chunk per wave, two per wave, the 16-wave kernels, a ragged last chunk,
# eight chunks per wave with operands from LDS (K > 16384; one to three tiles per workgroup);
# every variant of the quantiser the forward call offers.  The kernel leaves the normalised row
# it rounded in the workspace, so codes, row sum and accumulators are compared exactly "given
# the same normalised input", as for the stand-alone quantiser.
@pytest.mark.parametrize("K,N", [(96, 40), (2048, 6144), (3616, 257), (7168, 1000), (8192, 2048),
                                 (12320, 520), (16384, 300), (16896, 200), (28672, 7168), (32768, 1100),
                                 (20512, 12288)])
@pytest.mark.parametrize("variant", ["plain", "affine", "skip_ln", "per_tensor"])
def test_forward_single_token(bl, K, N, variant, tuning):
    print(f"forward single token K={K} N={N} {variant}", flush=True)
    sd = wl.seed_for(0, 5 * K + N)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(1, K, sd)
    rng = np.random.default_rng(sd)
    gain = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float32) if variant == "affine" else None
    bias = (0.05 * rng.standard_normal(K)).astype(np.float32) if variant == "affine" else None
    pt = variant == "per_tensor"
    kw = dict(per_tensor=pt, flags=bl.FLAG_SKIP_LN if variant == "skip_ln" else 0,
              ln_gain=None if gain is None else dev(gain), ln_bias=None if bias is None else dev(bias))
    kw_acc = dict(kw, flags=kw["flags"] | bl.FLAG_OUT_ACC_I32)
    r = oracle.forward(X, W, per_tensor=pt, skip_ln=variant == "skip_ln", gain=gain, bias=bias)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    lay = bl.forward_workspace_layout(1, N, K, pt)
    rms = np.sqrt(np.mean(r["y"].astype(np.float64) ** 2))
    for mode in ("one launch", "decode_nofuse=1"):
        tuning(None if mode == "one launch" else mode)
        ws = torch.zeros(bl.workspace_bytes(bl.OP_FORWARD, 1, N, K, pt), dtype=torch.uint8, device="cuda")
        y = host(bl.bitlinear_forward(dev(X), packed, N, beta, workspace=ws, **kw))
        held = host(ws)
        xh = held[lay["xhat"]:lay["xhat"] + 4 * K].view(f32).reshape(1, K)
        codes = held[:K].view(np.int8).reshape(1, K)
        gamma = held[lay["gamma"]:lay["gamma"] + 4].view(f32)
        rowsum = held[lay["rowsum"]:lay["rowsum"] + 4].view(np.int32)
        # integers, exactly, from the normalised row the kernel itself rounded
        g_ref = oracle.absmax(xh, pt)
        assert np.array_equal(gamma, g_ref), mode
        q_ref = oracle.quantize(xh, g_ref, pt)
        assert np.array_equal(codes, q_ref), mode
        assert rowsum[0] == int(q_ref.astype(np.int64).sum()), mode
        acc_ref = oracle.matmul_i32(q_ref, r["sign"])
        acc = host(bl.bitlinear_forward(dev(X), packed, N, beta, **kw_acc))
        assert np.array_equal(acc, acc_ref), mode
        assert np.array_equal(y, oracle.dequant(acc_ref, g_ref, r["beta"], pt)), mode
        # the normalised row itself, and the layer end to end from raw X
        assert np.abs(xh - r["xhat"]).max() <= 4e-6 * max(1.0, np.abs(r["xhat"]).max()), mode
        assert np.abs(y - r["y"]).max() <= 1e-3 * rms, mode


# Two to four tokens: the batch sizes next to the one-launch single-token path (they take the
# quantiser and the small-batch GEMM as two launches), in every variant of the quantiser.
@pytest.mark.parametrize("M,K,N", [(4, 2048, 6144), (2, 2048, 2048), (3, 8192, 2048), (4, 8192, 520),
                                   (2, 7168, 1000), (3, 7168, 21504), (4, 7168, 300), (2, 12320, 264),
                                   (2, 16384, 1000), (4, 512, 40), (3, 3616, 257)])
@pytest.mark.parametrize("variant", ["plain", "affine", "skip_ln", "per_tensor"])
def test_forward_few_tokens(bl, M, K, N, variant):
    print(f"forward few tokens M={M} K={K} N={N} {variant}", flush=True)
    sd = wl.seed_for(0, 9 * K + N + M)
    W = wl.make_weight(N, K, 0.02, sd)
    X = wl.make_activation(M, K, sd)
    X[M - 1] *= 3.0  # rows of different scale: a mixed-up gamma or row sum would show
    rng = np.random.default_rng(sd)
    gain = (1.0 + 0.1 * rng.standard_normal(K)).astype(np.float32) if variant == "affine" else None
    bias = (0.05 * rng.standard_normal(K)).astype(np.float32) if variant == "affine" else None
    pt = variant == "per_tensor"
    kw = dict(per_tensor=pt, flags=bl.FLAG_SKIP_LN if variant == "skip_ln" else 0,
              ln_gain=None if gain is None else dev(gain), ln_bias=None if bias is None else dev(bias))
    r = oracle.forward(X, W, per_tensor=pt, skip_ln=variant == "skip_ln", gain=gain, bias=bias)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    y = host(bl.bitlinear_forward(dev(X), packed, N, beta, **kw))
    rms = np.sqrt(np.mean(r["y"].astype(np.float64) ** 2))
    assert np.abs(y - r["y"]).max() <= 1e-3 * rms
    kw_acc = dict(kw, flags=kw["flags"] | bl.FLAG_OUT_ACC_I32)
    acc = host(bl.bitlinear_forward(dev(X), packed, N, beta, **kw_acc))
    assert (acc != r["acc"]).mean() <= 1e-3  # differs only where an x^ sits on a rounding tie
    # the workspace holds what the stand-alone quantiser would have put there
    ws = torch.zeros(bl.workspace_bytes(bl.OP_FORWARD, M, N, K, pt), dtype=torch.uint8, device="cuda")
    bl.bitlinear_forward(dev(X), packed, N, beta, workspace=ws, **kw)
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(dev(X), per_tensor=pt, flags=kw["flags"],
                                                     ln_gain=kw["ln_gain"], ln_bias=kw["ln_bias"])
    held = host(ws)
    assert np.array_equal(held[:M * K].view(np.int8).reshape(M, K), host(codes))
    # here the codes are the stand-alone quantiser's own, so the layer output follows from them
    y_ref = oracle.dequant(oracle.matmul_i32(host(codes), r["sign"]), host(gamma), host(beta), pt)
    assert np.array_equal(y, y_ref)


def test_empty_batch_and_errors(bl):
    W = dev(wl.make_weight(32, 64, 0.02, 1))
    packed, alpha, beta = bl.bitlinear_pack_weights(W)
    y = bl.bitlinear_forward(torch.empty((0, 64), device="cuda"), packed, 32, beta)
    assert y.shape == (0, 32)
    with pytest.raises(bl.BitLinearError):
        bl.bitlinear_forward(torch.empty((2, 48), device="cuda"), packed, 32, beta)  # K % 32
    with pytest.raises(bl.BitLinearError):
        bl.bitlinear_forward(torch.empty((2, 64), device="cuda"), packed, 32, beta,
                             workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))


def test_read_probe_reads_only(bl):
    """The measurement aid: any launch shape within its limits runs, leaves the buffer and a sink as
    they were (real data never trips its all-ones test), and bad shapes are host errors."""
    import ctypes
    lib = bl.load_library()
    rng = np.random.default_rng(7)
    words = rng.integers(0, 2**31, size=(1 << 20) + 12, dtype=np.int64).astype(np.uint32)
    buf = dev(words.view(np.int32))
    sink = torch.zeros(1024, dtype=torch.int32, device="cuda")
    for wgs, threads in [(1, 64), (256, 448), (1000, 1024), (37, 192)]:
        rc = lib.bitlinear_probe_read(ctypes.c_void_p(buf.data_ptr()), buf.numel() * 4, wgs, threads,
                                      ctypes.c_void_p(sink.data_ptr()), None)
        assert rc == 0
    torch.cuda.synchronize()
    assert np.array_equal(host(buf).view(np.uint32), words)
    assert int(sink.abs().sum()) == 0
    p = ctypes.c_void_p(buf.data_ptr())
    assert lib.bitlinear_probe_read(p, 24, 1, 64, None, None) == -2      # bytes % 16
    assert lib.bitlinear_probe_read(p, 1024, 1, 96, None, None) == -2    # threads % 64
    assert lib.bitlinear_probe_read(p, 1024, 0, 64, None, None) == -2
    assert lib.bitlinear_probe_read(None, 1024, 1, 64, None, None) == -1


# ------------------------------------------------------------------ full benchmark sizes
def _stratified_samples(M, N, seed, bm=64, bn=64, lines=3):
    """(rows, cols) of the outputs to check: one seeded position inside every bm x bn block of the
    output (every tile of every GEMM kernel is a union of such blocks: 16 weight rows x all tokens,
    64 x 128, 128 x 256, 256 x 256), the four corners, and `lines` whole rows and whole columns
    (first, last and seeded ones)."""
    rng = np.random.default_rng(seed)
    gm, gn = (M + bm - 1) // bm, (N + bn - 1) // bn
    r0 = (np.arange(gm) * bm)[:, None] + rng.integers(0, bm, (gm, gn))
    c0 = (np.arange(gn) * bn)[None, :] + rng.integers(0, bn, (gm, gn))
    rows = [np.minimum(r0, M - 1).ravel(), np.array([0, M - 1, 0, M - 1])]
    cols = [np.minimum(c0, N - 1).ravel(), np.array([0, N - 1, N - 1, 0])]
    for m in sorted({0, M - 1, *rng.integers(0, M, lines).tolist()}):
        rows.append(np.full(N, m))
        cols.append(np.arange(N))
    for n in sorted({0, N - 1, *rng.integers(0, N, lines).tolist()}):
        rows.append(np.arange(M))
        cols.append(np.full(M, n))
    return np.concatenate(rows).astype(np.int64), np.concatenate(cols).astype(np.int64)


_weight_cache = {}


def _weight(N, K, w_std, seed):
    """The seeded weight with the oracle's alpha, beta, signs and canonical words (kept for the
    next test of the same layer: a 30B-shaped matrix takes seconds to draw and binarise)."""
    key = (N, K, w_std, seed)
    if key not in _weight_cache:
        _weight_cache.clear()
        W = wl.make_weight(N, K, w_std, seed)
        a, b = oracle.weight_stats(W)
        sign = oracle.binarize(W, a)
        _weight_cache[key] = (W, a, b, sign, oracle.pack_canonical(sign))
    return _weight_cache[key]


def _sampled_check(bl, M, K, N, w_std, outlier_p, outlier_mul, seed, per_tensor=False):
    """Full-size run in the launch configuration the bench uses.  All bits, alpha, beta, gamma and
    codes are checked (codes given the normalised input the GPU dumped); accumulators and outputs
    on a stratified sample the oracle computes one by one: every 64 x 64 block of the output, the
    corners, and whole rows and columns."""
    W, a, b, sign, words = _weight(N, K, w_std, seed)
    X = wl.make_activation(M, K, seed, outlier_p, outlier_mul)
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    assert host(alpha)[0] == a and host(beta)[0] == b
    canon = host(bl.bitlinear_packed_to_canonical(packed, N, K)).view(np.uint32)
    assert np.array_equal(canon, words)
    del canon
    Xd = dev(X)
    codes, gamma, rowsum, xhat = bl.bitlinear_quant_act(Xd, per_tensor=per_tensor, want_xhat=True)
    xh = host(xhat)
    del xhat
    g_ref = oracle.absmax(xh, per_tensor)
    assert np.array_equal(host(gamma), g_ref)
    q_ref = oracle.quantize(xh, g_ref, per_tensor)
    assert np.array_equal(host(codes), q_ref)
    assert np.array_equal(host(rowsum)[:M], q_ref.astype(np.int32).sum(1, dtype=np.int64))
    xh_ref = oracle.layernorm(X[:64])
    assert np.abs(xh[:64] - xh_ref).max() <= 2e-6 * max(1.0, np.abs(xh_ref).max())
    del xh
    ws = torch.zeros(bl.workspace_bytes(bl.OP_FORWARD, M, N, K, per_tensor), dtype=torch.uint8,
                     device="cuda")
    y = host(bl.bitlinear_forward(Xd, packed, N, beta, per_tensor=per_tensor, workspace=ws))
    if M == 1:
        # one launch: the GEMM kernel quantises the row itself, with its own summation order; the
        # integers that follow are checked from the normalised row IT rounded (left in the workspace)
        lay = bl.forward_workspace_layout(1, N, K, per_tensor)
        held = host(ws)
        xh1 = held[lay["xhat"]:lay["xhat"] + 4 * K].view(f32).reshape(1, K)
        g_ref = oracle.absmax(xh1, per_tensor)
        q_ref = oracle.quantize(xh1, g_ref, per_tensor)
        assert np.array_equal(held[lay["gamma"]:lay["gamma"] + 4].view(f32), g_ref)
        assert np.array_equal(held[:K].view(np.int8).reshape(1, K), q_ref)
        assert np.abs(xh1 - xh_ref[:1]).max() <= 2e-6 * max(1.0, np.abs(xh_ref).max())
    del ws
    rows, cols = _stratified_samples(M, N, seed, bm=min(64, M), bn=64 if M > 16 else 16)
    acc_ref = oracle.matmul_i32_sampled(q_ref, sign, rows, cols)
    sc = (b * (g_ref[0] if per_tensor else g_ref[rows])) / f32(128.0)
    y_ref = acc_ref.astype(f32) * sc
    assert np.array_equal(y[rows, cols], y_ref)
    acc = host(bl.bitlinear_forward(Xd, packed, N, beta, per_tensor=per_tensor,
                                    flags=bl.FLAG_OUT_ACC_I32))
    assert np.array_equal(acc[rows, cols], acc_ref)
    return y


# every (layer, batch) cell of the 1.3B decode configuration
@pytest.mark.parametrize("M", [1, 4, 16])
@pytest.mark.parametrize("li", [0, 1, 2, 3])
def test_full_size_decode_1p3b(bl, li, M):
    L = wl.CONFIGS[1].layers[li]
    print(f"full decode {L} M={M}", flush=True)
    _sampled_check(bl, M, L.K, L.N, 0.02, 0, 1, wl.seed_for(1, li))


@pytest.mark.parametrize("li", [0, 1])
def test_full_size_prefill_6p7b(bl, li):
    L = wl.CONFIGS[2].layers[li]
    print(f"full prefill {L}", flush=True)
    y = _sampled_check(bl, 2048, L.K, L.N, 0.02, 0.001, 20.0, wl.seed_for(2, li))
    assert np.isfinite(y).all()


# Every (layer, batch) cell of the 30B configuration (M = 64: batched decode; 4096: prefill,
# the large-tile kernel, 5.25 to seven rounds of tiles per workgroup), and the batch sizes in
# between that select the other kernels: 16 small-batch; 32 and 24 the 17-32 token kernel (layer
# 2, K = 28672, goes on to the mid-batch one); 1 the quantiser inside the GEMM launch.
@pytest.mark.parametrize("li,M", [(0, 1), (0, 24), (0, 64), (0, 4096),
                                  (1, 1), (1, 16), (1, 32), (1, 64), (1, 4096),
                                  (2, 32), (2, 64), (2, 4096)])
def test_full_size_30b(bl, li, M):
    L = wl.CONFIGS[3].layers[li]
    print(f"full 30b {L} M={M}", flush=True)
    _sampled_check(bl, M, L.K, L.N, 0.01, 0, 1, wl.seed_for(3, li))


def test_full_size_training_forward_per_tensor(bl):
    """The training configuration's forward: M = 8192, 4096 -> 16384, one gamma for the tensor
    (the statistics pass with its grid-wide maximum, then the rounding pass)."""
    c = wl.CONFIGS[4]
    L, M = c.layers[0], c.Ms[0]
    print(f"full training forward {L} M={M} per-tensor", flush=True)
    _weight_cache.clear()
    y = _sampled_check(bl, M, L.K, L.N, c.w_std, 0, 1, wl.seed_for(4, 0), per_tensor=True)
    assert np.isfinite(y).all()
    _weight_cache.clear()


# ------------------------------------------------------------------ a chain of layers
def _glue(h, K):
    """What stands between two projections here: the next layer's input is the first K features of
    the previous output (the attention and the non-linearity are not part of the layer)."""
    return np.ascontiguousarray(h[:, :K])


@pytest.mark.parametrize("stack", ["1.3b", "6.7b"])
@pytest.mark.parametrize("M", [1, 4])
def test_decode_chain_of_layers(bl, stack, M):
    """One decoding step through QKV, O, up and down of two layers, each projection fed by the
    previous one's output, through bitlinear_forward (one launch per projection at one token),
    against the oracle chained the same way.  Outputs within 1e-3 of the oracle's rms at every
    link (a code may move by one where a normalised value sits on a rounding tie)."""
    d = 2048 if stack == "1.3b" else 4096
    shapes = [("qkv", d, 3 * d), ("o", d, d), ("up", d, 4 * d), ("down", 4 * d, d)] * 2
    print(f"chain {stack} M={M}", flush=True)
    h_ref = wl.make_activation(M, d, wl.seed_for(1, 500 + M))
    h_gpu = dev(h_ref)
    for i, (name, K, N) in enumerate(shapes):
        W = wl.make_weight(N, K, 0.02, wl.seed_for(1, 600 + i))
        packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
        x_ref = _glue(h_ref, K)
        x_gpu = h_gpu[:, :K].contiguous()
        h_ref = oracle.forward(x_ref, W)["y"]
        h_gpu = bl.bitlinear_forward(x_gpu, packed, N, beta)
        rms = np.sqrt(np.mean(h_ref.astype(np.float64) ** 2))
        err = np.abs(host(h_gpu) - h_ref).max()
        assert err <= 1e-3 * rms, (i, name, err, rms)


# ------------------------------------------------------------------ K split across workgroups
@pytest.mark.parametrize("M,K,N", [(1, 28672, 7168), (16, 28672, 7168), (5, 16896, 200),
                                   (16, 17920, 1040), (3, 32768, 64), (64, 7168, 2048),
                                   (40, 4096, 384), (64, 28672, 7168), (50, 3616, 130)])
def test_forward_long_k_split_matches_single_pass(bl, M, K, N):
    """Long K at small M (K > 16384 at M <= 16; 16 < M <= 64 when N alone leaves workgroup slots
    empty): bitlinear_forward splits K over workgroups and folds the slices in a second kernel;
    the result must equal the single-pass kernel's (bitlinear_matmul without a workspace never
    splits) bit for bit, and the oracle's on sampled outputs."""
    print(f"split-K forward M={M} K={K} N={N}", flush=True)
    X = wl.make_activation(M, K, seed=wl.seed_for(3, K + N + M))
    W = wl.make_weight(N, K, 0.01, seed=wl.seed_for(3, K + N))
    packed, alpha, beta = bl.bitlinear_pack_weights(dev(W))
    Xd = dev(X)
    y_split = bl.bitlinear_forward(Xd, packed, N, beta)
    codes, gamma, rowsum, _ = bl.bitlinear_quant_act(Xd)
    y_single = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta)
    assert torch.equal(y_split, y_single)
    acc_split = bl.bitlinear_forward(Xd, packed, N, beta, flags=bl.FLAG_OUT_ACC_I32)
    acc_single = bl.bitlinear_matmul(codes, gamma, rowsum, packed, N, beta, flags=bl.FLAG_OUT_ACC_I32)
    assert torch.equal(acc_split, acc_single)
    # sampled outputs against the oracle, from the GPU's own codes
    rng = np.random.default_rng(K)
    rows = rng.integers(0, M, 64)
    cols = rng.integers(0, N, 64)
    sign = oracle.binarize(W, host(alpha)[0])
    ref = oracle.matmul_i32_sampled(host(codes), sign, rows, cols)
    assert np.array_equal(host(acc_split)[rows, cols], ref)
