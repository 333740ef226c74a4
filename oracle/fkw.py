"""Filter-kernel reorder and the FKW compact storage, as the paper states them
(TEST INFRASTRUCTURE ONLY; plain numpy / Python loops, small layers).

Followed passages:

* section 5.2 (FKR): filters are ordered by their number of non-empty kernels
  ("length"), filters of equal length by similarity of their pattern content;
  inside every filter the kernels are ordered by pattern id.
* section 5.3 (FKW): five arrays - ``offset`` (per filter, cumulative count of
  non-empty kernels), ``reorder`` (original output channel of each stored
  filter), ``index`` (input channel of each stored kernel), ``stride`` (per
  filter, cumulative kernel count per pattern) and ``weight`` (the four kept
  weights of each stored kernel).
* the execution order of the reordered layer (section 5.1 / 5.2): filter, then
  pattern, then the kernels of that pattern, four multiply-accumulates each,
  result written to the channel named by ``reorder``.

Readings taken where the text leaves a choice (none of them changes a result):
lengths ascend (the worked example of section 5.3 lists lengths 2,2,2,3 after
the reorder); equal-length filters are ordered by their per-pattern kernel-count
vector, then by original index; kernels of one pattern are ordered by input
channel; the four weights of a kernel are stored in ascending row-major
position; pattern ids are 0-based and ``stride`` has P+1 entries per filter.

``fkw_conv2d`` must give the same numbers as the plain definition in
``patdnn_ref.c`` - a test checks that - which ties this reading of the storage
format to the operation it encodes.
"""

from __future__ import annotations

from dataclasses import dataclass

import numpy as np


def _taps(mask: int):
    return [p for p in range(9) if (int(mask) >> p) & 1]


@dataclass
class FKW:
    offset: np.ndarray    # int64 [F+1]
    reorder: np.ndarray   # int64 [F]      stored filter -> original output channel
    index: np.ndarray     # int64 [kept]   input channel of each stored kernel
    stride: np.ndarray    # int64 [F][P+1] cumulative kernels per pattern, per filter
    weight: np.ndarray    # float32 [kept][4]
    pattern_masks: np.ndarray


def filter_order(pattern_ids, kernel_mask, num_patterns: int) -> np.ndarray:
    """Filter reorder: by length, then per-pattern count vector, then original index."""
    c_out = kernel_mask.shape[0]
    keys = []
    for f in range(c_out):
        kept = np.flatnonzero(kernel_mask[f])
        counts = np.bincount(pattern_ids[f, kept], minlength=num_patterns)
        keys.append((len(kept), tuple(int(c) for c in counts), f))
    return np.asarray([k[2] for k in sorted(keys)], dtype=np.int64)


def build_fkw(weights, pattern_ids, kernel_mask, pattern_masks) -> FKW:
    w = np.asarray(weights, dtype=np.float32)
    ids = np.asarray(pattern_ids)
    km = np.asarray(kernel_mask)
    P = len(pattern_masks)
    order = filter_order(ids, km, P)
    F = len(order)
    offset = np.zeros(F + 1, dtype=np.int64)
    stride = np.zeros((F, P + 1), dtype=np.int64)
    index, weight = [], []
    for pos, f in enumerate(order):
        kept = [int(c) for c in np.flatnonzero(km[f])]
        kept.sort(key=lambda c: (int(ids[f, c]), c))          # kernel reorder
        for c in kept:
            index.append(c)
            weight.append([w[f, c, p // 3, p % 3] for p in _taps(pattern_masks[ids[f, c]])])
            stride[pos, int(ids[f, c]) + 1] += 1
        stride[pos] = np.cumsum(stride[pos])
        offset[pos + 1] = offset[pos] + len(kept)
    return FKW(offset=offset, reorder=order, index=np.asarray(index, dtype=np.int64),
               stride=stride,
               weight=np.asarray(weight, dtype=np.float32).reshape(-1, 4),
               pattern_masks=np.asarray(pattern_masks, dtype=np.uint16))


def fkw_conv2d(fkw: FKW, x, bias=None, *, stride: int = 1, pad: int = 1,
               relu: bool = False) -> np.ndarray:
    """Run the reordered layer straight from the five arrays, float64."""
    x = np.asarray(x, dtype=np.float64)
    n, c_in, h, w = x.shape
    ho = (h + 2 * pad - 3) // stride + 1
    wo = (w + 2 * pad - 3) // stride + 1
    xp = np.zeros((n, c_in, h + 2 * pad, w + 2 * pad), dtype=np.float64)
    xp[:, :, pad:pad + h, pad:pad + w] = x
    F = len(fkw.reorder)
    out = np.zeros((n, F, ho, wo), dtype=np.float64)
    for f in range(F):
        co = int(fkw.reorder[f])
        acc = np.zeros((n, ho, wo), dtype=np.float64)
        if bias is not None:
            acc += float(bias[co])
        for p in range(len(fkw.pattern_masks)):
            taps = _taps(fkw.pattern_masks[p])
            lo = fkw.offset[f] + fkw.stride[f, p]
            hi = fkw.offset[f] + fkw.stride[f, p + 1]
            for k in range(int(lo), int(hi)):
                ci = int(fkw.index[k])
                for t, pos in enumerate(taps):
                    kh, kw = pos // 3, pos % 3
                    win = xp[:, ci, kh:kh + (ho - 1) * stride + 1:stride,
                             kw:kw + (wo - 1) * stride + 1:stride]
                    acc += float(fkw.weight[k, t]) * win
        out[:, co] = np.maximum(acc, 0.0) if relu else acc
    return out
