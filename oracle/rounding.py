"""Operand rounding of the oracle (test infrastructure).

The bf16 configurations hold weights and matrix-multiply operands in bf16 and everything else
in wider precision ("bf16 weights and activations with fp32 accumulate" in the workload
statement; the paper itself fixes no precision). The oracle keeps all arithmetic in float64
and applies one round-to-nearest-even to bf16 at exactly the points where an operand of a
matrix product is formed: the normalised input of a projection, Q/K/V after the rotary
embedding, the un-normalised softmax weights before they multiply V, the attention output,
and the SwiGLU product. For the "f32" configuration nothing is rounded.
"""
import numpy as np


def round_bf16(x):
    """float64 -> nearest bf16 (ties to even), returned as float64. Normal range only."""
    a = np.ascontiguousarray(x, dtype=np.float64)
    b = a.view(np.uint64)
    drop = np.uint64(45)                      # 52 - 7 mantissa bits
    lsb = (b >> drop) & np.uint64(1)
    r = (b + ((np.uint64(1) << np.uint64(44)) - np.uint64(1)) + lsb) & ~((np.uint64(1) << drop) - np.uint64(1))
    return r.view(np.float64).reshape(a.shape)


def operand(x, dtype):
    if dtype == "f32":
        return np.asarray(x, dtype=np.float64)
    if dtype == "bf16":
        return round_bf16(x)
    raise ValueError(dtype)
