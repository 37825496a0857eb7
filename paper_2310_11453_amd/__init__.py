"""MI355X-native BitLinear (BitNet, arXiv 2310.11453): hand-written HIP kernels for gfx950
behind the C ABI of include/bitlinear.h, with a ctypes binding of the same names."""
from .binding import (  # noqa: F401
    BitLinearError, EXPORTS, LIB_PATH,
    FLAG_BETA_CENTERED, FLAG_OUT_ACC_I32, FLAG_SKIP_LN,
    OP_BACKWARD, OP_FORWARD, OP_FORWARD_NONNEG, OP_LN_BACKWARD, OP_MATMUL, OP_PACK, OP_QUANT,
    bitlinear_backward_ste, bitlinear_forward, bitlinear_matmul, bitlinear_pack_weights,
    bitlinear_packed_to_canonical, bitlinear_quant_act, load_library, packed_bytes,
    status_string, workspace_bytes,
    bitlinear_forward_grouped, bitlinear_pack_weights_grouped, bitlinear_packed_to_canonical_grouped,
    bitlinear_layernorm_backward, bitlinear_quant_act_grouped, packed_bytes_grouped,
    workspace_bytes_grouped,
    bitlinear_forward_nonneg, bitlinear_matmul_nonneg, bitlinear_quant_act_nonneg,
    bitlinear_weight_rowsums, bitlinear_weight_rowsums_grouped, forward_workspace_layout, set_tuning,
    bitlinear_forward_static, probe_read,
)
