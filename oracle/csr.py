"""CSR form of a pruned CONV layer, CPU oracle (TEST INFRASTRUCTURE ONLY; same import
rule as ``oracle/ref.py``; shares nothing with the library's implementation).

The paper compares its compact FKW storage with the conventional compressed sparse row
format (section 5.3, section 6.3) and runs a CSR-based sparse convolution as a negative
control (section 6.2).  The textbook definition written out: the layer's weight tensor,
with every pruned position zero, is the matrix A[c_out][c_in*9] (column = ci*9 + 3*kh + kw);
CSR stores, filter by filter, the column index and value of each structurally kept
position in ascending column order, and row_ptr[co] .. row_ptr[co+1] delimits filter co.
"Structurally kept" means a position of the kernel's pattern in a surviving kernel, also
when the stored value happens to be 0.0 (the format follows the pruning structure).
"""

from __future__ import annotations

import numpy as np


def build_csr(weights, pattern_ids, kernel_mask, pattern_masks):
    """-> (row_ptr int32 [c_out+1], col int32 [nnz], val float32 [nnz])"""
    w = np.asarray(weights, dtype=np.float32)
    c_out, c_in = w.shape[:2]
    row_ptr, col, val = [0], [], []
    for co in range(c_out):
        for ci in range(c_in):
            if kernel_mask is not None and not kernel_mask[co, ci]:
                continue
            m = int(pattern_masks[pattern_ids[co, ci]])
            for p in range(9):
                if (m >> p) & 1:
                    col.append(ci * 9 + p)
                    val.append(w[co, ci, p // 3, p % 3])
        row_ptr.append(len(col))
    return (np.array(row_ptr, dtype=np.int32), np.array(col, dtype=np.int32),
            np.array(val, dtype=np.float32))


def csr_conv2d(row_ptr, col, val, x, bias=None, *, stride=1, pad=1, relu=False):
    """Direct convolution that walks the CSR arrays (fp64).  Small inputs only."""
    x = np.asarray(x, dtype=np.float64)
    n, c_in, h, w = x.shape
    c_out = len(row_ptr) - 1
    ho, wo = (h + 2 * pad - 3) // stride + 1, (w + 2 * pad - 3) // stride + 1
    xp = np.zeros((n, c_in, h + 2 * pad, w + 2 * pad))
    xp[:, :, pad:pad + h, pad:pad + w] = x
    out = np.zeros((n, c_out, ho, wo))
    for co in range(c_out):
        for k in range(row_ptr[co], row_ptr[co + 1]):
            ci, p = divmod(int(col[k]), 9)
            kh, kw = divmod(p, 3)
            out[:, co] += float(val[k]) * xp[:, ci, kh:kh + stride * ho:stride, kw:kw + stride * wo:stride]
        if bias is not None:
            out[:, co] += float(bias[co])
    return np.maximum(out, 0.0) if relu else out
