"""Arithmetic-energy estimate of matrix multiplications (arXiv 2310.11453, Section 3, the two
equations for a vanilla Transformer and the one for BitNet, with the per-operation energies of
the table of ADD/MUL energies at 45 nm and 7 nm).  Host arithmetic for reports: nothing here
runs on the GPU or takes part in the layer's computation.

    vanilla  [m,n] x [n,p]:  E_add = m (n-1) p e_add,   E_mul = m n p e_mul
    BitNet   (W1A8)       :  E_add = m (n-1) p e_add(INT8),  E_mul = (m p + m n) e_mul
(the 1-bit weights leave only additions of 8-bit activations; multiplications remain for the
scaling by beta and gamma/Q_b, once per output and once per input element).
"""
from __future__ import annotations

# pJ per operation: {node: {format: (add, mul)}}
OP_ENERGY_PJ = {
    "45nm": {"fp32": (0.9, 3.7), "fp16": (0.4, 1.1), "int8": (0.03, 0.2)},
    "7nm": {"fp32": (0.38, 1.31), "fp16": (0.16, 0.34), "int8": (0.007, 0.07)},
}


def matmul_energy(m: int, n: int, p: int, fmt: str, node: str) -> tuple[float, float]:
    """(E_add, E_mul) in joules of a dense [m,n] x [n,p] product in `fmt`."""
    e_add, e_mul = OP_ENERGY_PJ[node][fmt]
    return m * (n - 1) * p * e_add * 1e-12, m * n * p * e_mul * 1e-12


def bitlinear_energy(m: int, n: int, p: int, node: str, scale_fmt: str = "fp16") -> tuple[float, float]:
    """(E_add, E_mul) in joules of a BitLinear product, m tokens, fan-in n, fan-out p: INT8
    additions, and m p + m n multiplications in `scale_fmt` for the two scalings."""
    e_add = OP_ENERGY_PJ[node]["int8"][0]
    e_mul = OP_ENERGY_PJ[node][scale_fmt][1]
    return m * (n - 1) * p * e_add * 1e-12, (m * p + m * n) * e_mul * 1e-12


def transformer_energy(d: int, layers: int, tokens: int, wbits: int, node: str) -> tuple[float, float]:
    """(E_add, E_mul) in joules of the matrix multiplications of a decoder with hidden size d
    and FFN size 4d over one sequence of `tokens` tokens: per layer the four d x d attention
    projections, the two d x 4d FFN matrices, and the two attention products (scores and the
    weighted sum, tokens x tokens x d each).  wbits = 32 or 16: everything in that format.
    wbits = 1: the six weight matrices are BitLinear, the attention products stay in fp16.
    With the paper's model sizes and 512 tokens this reproduces its energy table."""
    linear = [(d, d)] * 4 + [(d, 4 * d), (4 * d, d)]
    add = mul = 0.0
    for (n, p) in linear:
        a, b = (bitlinear_energy(tokens, n, p, node) if wbits == 1
                else matmul_energy(tokens, n, p, "fp32" if wbits == 32 else "fp16", node))
        add, mul = add + a, mul + b
    attn_fmt = "fp32" if wbits == 32 else "fp16"
    for (mm, nn, pp) in ((tokens, d, tokens), (tokens, tokens, d)):
        a, b = matmul_energy(mm, nn, pp, attn_fmt, node)
        add, mul = add + a, mul + b
    return add * layers, mul * layers
