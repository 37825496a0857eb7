"""CPU-only checks of the C-ABI boundary: the library loads without a GPU, exports every
symbol include/bitlinear.h declares, and rejects bad arguments on the host (no launch)."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def lib():
    import paper_2310_11453_amd as bl
    if not bl.LIB_PATH.exists():
        from paper_2310_11453_amd.build import build
        build(verbose=False)
    return bl.load_library()


def declared_functions():
    text = (ROOT / "include" / "bitlinear.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(bitlinear_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    import paper_2310_11453_amd as bl
    names = declared_functions()
    assert set(names) == set(bl.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_host_size_queries(lib):
    import paper_2310_11453_amd as bl
    # 1 bit per weight, N padded to 16 and K to 512
    assert bl.packed_bytes(512, 256) == 512 * 512 // 8
    assert bl.packed_bytes(2048, 2048) == 2048 * 2048 // 8
    assert bl.packed_bytes(17, 544) == 32 * 1024 // 8
    assert bl.packed_bytes(16, 48) == 0 and bl.packed_bytes(0, 32) == 0
    assert bl.packed_bytes(512, 512, 8) == 0  # unknown flag
    for op in (bl.OP_PACK, bl.OP_QUANT, bl.OP_FORWARD, bl.OP_BACKWARD):
        assert bl.workspace_bytes(op, 8, 512, 256) > 0
    assert bl.workspace_bytes(bl.OP_FORWARD, 8, 512, 256) >= 8 * 256
    assert bl.workspace_bytes(bl.OP_BACKWARD, 64, 512, 256) >= 2 * (2 * 64 * 512 + 256 * 512 + 256 * 64)
    assert bl.workspace_bytes(99, 8, 512, 256) == 0


def test_argument_errors_are_found_on_the_host(lib):
    one = ctypes.c_void_p(256)  # never dereferenced: every call below fails before a launch
    assert lib.bitlinear_pack_weights(None, 8, 32, 0, one, one, one, one, 1 << 20, None) == -1
    assert lib.bitlinear_pack_weights(one, 8, 48, 0, one, one, one, one, 1 << 20, None) == -2
    assert lib.bitlinear_pack_weights(one, 8, 32, 1 << 10, one, one, one, one, 1 << 20, None) == -3
    assert lib.bitlinear_pack_weights(one, 8, 32, 0, one, one, one, one, 8, None) == -4
    assert lib.bitlinear_quant_act(one, 4, 64, None, None, 1e-5, 7, 0, one, one, None, None,
                                   one, 1 << 20, None) == -3
    assert lib.bitlinear_quant_act(one, 4, 64, None, None, 1e-5, 0, 0, None, one, None, None,
                                   one, 1 << 20, None) == -1
    assert lib.bitlinear_quant_act(one, -1, 64, None, None, 1e-5, 0, 0, one, one, None, None,
                                   one, 1 << 20, None) == -2
    assert lib.bitlinear_forward(one, 4, 64, one, 0, one, None, None, 1e-5, 0, 0, one, one,
                                 1 << 20, None) == -2
    assert lib.bitlinear_forward(one, 4, 64, one, 16, one, None, None, 1e-5, 0, 0, one, None,
                                 0, None) == -4
    assert lib.bitlinear_matmul(one, one, None, 4, 64, one, 16, one, 0, 0, one, None, 0, None) == -1
    assert lib.bitlinear_backward_ste(None, 4, 16, 64, one, one, 0, one, one, one, one, one,
                                      1 << 20, None) == -1
    # M == 0 is a successful no-op
    assert lib.bitlinear_forward(one, 0, 64, one, 16, one, None, None, 1e-5, 0, 0, one, one,
                                 1 << 20, None) == 0
    assert lib.bitlinear_status_string(-2).decode().startswith("bad shape")


def test_grouped_host_checks(lib):
    """Eq. 13-15 entry points: sizes and argument errors, all on the host."""
    import paper_2310_11453_amd as bl
    # K-groups are blobs of their own: 8 x [512, 256] slices, each padded to a 512-wide tile
    assert bl.packed_bytes_grouped(512, 2048, 1, 1) == bl.packed_bytes(512, 2048)
    assert bl.packed_bytes_grouped(512, 2048, 8, 8) == 8 * bl.packed_bytes(512, 256)
    assert bl.packed_bytes_grouped(512, 2048, 3, 1) == 0   # 3 does not divide N
    assert bl.packed_bytes_grouped(512, 96, 1, 2) == 0     # K/groups not a multiple of 32
    assert bl.packed_bytes_grouped(96, 64, 4, 1) == 0      # 24-row groups are not whole tiles
    assert bl.packed_bytes_grouped(512, 2048, 65, 1) == 0
    assert bl.workspace_bytes_grouped(bl.OP_FORWARD, 8, 512, 2048, 2, 4) >= 8 * 2048 + 2 * 8 * 4 * 4
    assert bl.workspace_bytes_grouped(bl.OP_BACKWARD, 8, 512, 2048, 2, 4) == 0
    one = ctypes.c_void_p(256)
    assert lib.bitlinear_pack_weights_grouped(one, 512, 2048, 3, 1, 0, one, one, one, one,
                                              1 << 20, None) == -2
    assert lib.bitlinear_pack_weights_grouped(one, 96, 64, 4, 1, 0, one, one, one, one,
                                              1 << 20, None) == -3
    assert lib.bitlinear_pack_weights_grouped(None, 512, 2048, 2, 2, 0, one, one, one, one,
                                              1 << 20, None) == -1
    assert lib.bitlinear_quant_act_grouped(one, 4, 96, 2, None, None, 1e-5, 0, 0, one, one, None,
                                           None, one, 1 << 20, None) == -2
    assert lib.bitlinear_forward_grouped(one, 4, 2048, one, 512, 2, 4, one, None, None, 1e-5, 0,
                                         2, one, one, 1 << 20, None) == -3  # OUT_ACC_I32 not offered
    assert lib.bitlinear_forward_grouped(one, 4, 2048, one, 512, 2, 4, one, None, None, 1e-5, 0,
                                         0, one, one, 8, None) == -4
    assert lib.bitlinear_forward_grouped(one, 0, 2048, one, 512, 2, 4, one, None, None, 1e-5, 0,
                                         0, one, one, 1 << 20, None) == 0


def test_tuning_switches_parse_on_the_host(lib):
    assert lib.bitlinear_set_tuning(b"decode_nofuse=1,bwd_grid=8") == 0
    assert lib.bitlinear_set_tuning(b"no_such_switch=1") == -3
    assert lib.bitlinear_set_tuning(b"decode_nofuse") == -3
    assert lib.bitlinear_set_tuning(b"decode_nofuse=x") == -3
    assert lib.bitlinear_set_tuning(b"") == 0
    assert lib.bitlinear_set_tuning(None) == 0


def test_size_limits_are_host_errors(lib):
    """K beyond what the GEMM kernels' int32 partial sums hold: refused before any launch."""
    one = ctypes.c_void_p(256)
    big = 65536 + 32
    assert lib.bitlinear_matmul(one, one, one, 4, big, one, 16, one, 0, 0, one, None, 0, None) == -3
    assert lib.bitlinear_forward(one, 4, big, one, 16, one, None, None, 1e-5, 0, 0, one, one,
                                 1 << 30, None) == -3
    assert lib.bitlinear_matmul_nonneg(one, one, one, one, 4, big, one, 16, one, one, 0, 0, one,
                                       None) == -3
    # a grouped layer is bounded per K-group
    assert lib.bitlinear_forward_grouped(one, 4, 2 * 65536, one, 16, 1, 2, one, None, None, 1e-5, 0,
                                         0, one, one, 8, None) == -4


def test_forward_workspace_layout(lib):
    import paper_2310_11453_amd as bl
    lay = bl.forward_workspace_layout(1, 512, 2048)
    assert lay["codes"] == 0 and lay["gamma"] >= 2048 and lay["rowsum"] > lay["gamma"]
    assert lay["xhat"] is not None and lay["xhat"] + 4 * 2048 <= bl.workspace_bytes(bl.OP_FORWARD, 1, 512, 2048)
    assert bl.forward_workspace_layout(4, 512, 2048)["xhat"] is None
    off = (ctypes.c_size_t * 4)()
    assert lib.bitlinear_forward_workspace_layout(1, 512, 48, 0, off) == -2
    assert lib.bitlinear_forward_workspace_layout(1, 512, 64, 0, None) == -1
