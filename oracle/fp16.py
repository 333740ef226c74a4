"""Half-precision storage model of the CPU oracle (TEST INFRASTRUCTURE ONLY; same import
rule as ``oracle/ref.py``; shares nothing with the HIP library).

The paper's GPU runs keep weights and intermediate results in 16-bit floating point
(section 2.2, section 6.1).  Reading taken here: IEEE binary16 *storage* - weights, input
and output tensors hold binary16 values (round to nearest, ties to even, on conversion from
wider types) - with the arithmetic in between exact: the oracle converts the stored values
to double, runs the plain definition (``ref.conv2d``) and rounds the result to binary16
once.  Bias stays fp32 (it is added before the final rounding).
"""

from __future__ import annotations

import numpy as np

from . import ref


def to_f16(x) -> np.ndarray:
    """Round to nearest even onto binary16 (overflow -> inf, tiny -> subnormal or zero)."""
    with np.errstate(over="ignore"):
        return np.asarray(x).astype(np.float16)


def conv2d_f16(weights, pattern_ids, kernel_mask, pattern_masks, x, bias=None, **kw):
    """-> (binary16 result, the exact fp64 result before the final rounding).  `weights`
    and `x` are rounded to binary16 first - pass values that already are to model a stored
    model and stored activations."""
    w16 = to_f16(weights).astype(np.float32)
    x16 = to_f16(x).astype(np.float32)
    exact = ref.conv2d(w16, pattern_ids, kernel_mask, pattern_masks, x16, bias, **kw)
    return to_f16(exact), exact
