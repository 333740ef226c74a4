"""Chained CONV stack of the CPU oracle (TEST INFRASTRUCTURE ONLY; same import rule as
``oracle/ref.py``; shares nothing with the HIP library).

The paper's headline scenario runs one image through all CONV layers of VGG-16 (section
6.2); a DNN is CONV layers each followed by ReLU, with pooling layers between the stages
(section 2.1).  Plain definitions written out:

* ``maxpool2x2``  2x2 max pooling with stride 2, no padding; an odd last row / column
  has no complete window and is dropped (floor).
* ``stack_forward``  every layer is the oracle's pruned convolution (``ref.conv2d``,
  fp64) with bias and ReLU, optionally followed by the pooling above.  Each layer's
  result is rounded to fp32 before it feeds the next one, because fp32 is the storage
  type of activations on the path under test (the value handed on is what an fp32
  tensor can hold); the fp64 result before that rounding is returned for comparison.
"""

from __future__ import annotations

import numpy as np

from . import ref


def maxpool2x2(x: np.ndarray) -> np.ndarray:
    """[n][c][h][w] -> [n][c][h//2][w//2], out[i][j] = max of x[2i..2i+1][2j..2j+1]."""
    n, c, h, w = x.shape
    ho, wo = h // 2, w // 2
    out = np.empty((n, c, ho, wo), dtype=x.dtype)
    for i in range(ho):
        for j in range(wo):
            win = x[:, :, 2 * i:2 * i + 2, 2 * j:2 * j + 2]
            out[:, :, i, j] = win.reshape(n, c, 4).max(axis=2)
    return out


def stack_forward(layers, x: np.ndarray, pool_after):
    """layers: dicts with weights / pattern_ids / kernel_mask / pattern_masks / bias / spec
    (as ``workloads.gen_layer`` builds them); pool_after[i] true = 2x2 max pooling after
    layer i.  Returns the list of per-layer fp64 outputs (after ReLU and pooling)."""
    outs = []
    cur = np.ascontiguousarray(x, dtype=np.float32)
    for d, pool in zip(layers, pool_after):
        spec = d["spec"]
        y = ref.conv2d(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], cur,
                       d["bias"], stride=spec.stride, pad=spec.pad, relu=True,
                       depthwise=spec.depthwise, dense=spec.dense, skip_removed=True)
        if pool:
            y = maxpool2x2(y)
        outs.append(y)
        cur = y.astype(np.float32)
    return outs
