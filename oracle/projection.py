"""Projection operators of the pattern-based pruning stage, CPU oracle (TEST
INFRASTRUCTURE ONLY; same import rule as ``oracle/ref.py``; shares nothing with the
library's implementation).

Paper passages followed, each restated as the plain definition it amounts to:

* natural pattern (section 4.1): of a 3x3 kernel, the centre plus the three other
  positions whose weights have the largest magnitudes - a four-entry pattern that always
  keeps the centre, one of C(8,3) = 56.
* pattern candidate set (section 4.1): the k natural patterns that occur most often over
  all kernels.
* projection onto the pattern constraint (section 4.2, the second sub-problem: the
  Euclidean projection; "assign an appropriate pattern for each kernel based on the L2
  norm"): per kernel, the pattern of the set whose positions retain the largest sum of
  squares - equivalently the feasible kernel closest in Euclidean distance; weights
  outside the chosen pattern become zero.
* projection onto the connectivity constraint (section 4.2, the third sub-problem): keep
  the alpha kernels of the layer with the largest L2 norms, set the others to zero.

Readings where the paper is silent: magnitudes and norms are compared in IEEE double
computed from the fp32 weights; ties go to the lower position (natural pattern), the
lower mask value (pattern counts), the lower pattern id (pattern projection) and the
lower flat index co*c_in+ci (connectivity).  Pure Python / numpy loops, small inputs.
"""

from __future__ import annotations

import numpy as np


def natural_pattern(kernel: np.ndarray) -> int:
    """9-bit mask (bit 3*kh+kw) of the centre and the three largest-magnitude other weights."""
    k = np.asarray(kernel, dtype=np.float32).reshape(9).astype(np.float64)
    others = [p for p in range(9) if p != 4]
    # stable: larger magnitude first, then lower position
    others.sort(key=lambda p: (-abs(k[p]), p))
    mask = 1 << 4
    for p in others[:3]:
        mask |= 1 << p
    return mask


def mine_pattern_set(weights: np.ndarray, k: int) -> np.ndarray:
    """The k most frequent natural patterns over all kernels of [c_out][c_in][3][3],
    most frequent first (equal counts: lower mask first), as uint16 masks."""
    w = np.asarray(weights, dtype=np.float32)
    counts = {}
    for co in range(w.shape[0]):
        for ci in range(w.shape[1]):
            m = natural_pattern(w[co, ci])
            counts[m] = counts.get(m, 0) + 1
    order = sorted(counts, key=lambda m: (-counts[m], m))
    return np.array(order[:k], dtype=np.uint16)


def retained_energy(kernel: np.ndarray, mask: int) -> float:
    k = np.asarray(kernel, dtype=np.float32).reshape(9).astype(np.float64)
    e = 0.0
    for p in range(9):                       # fixed order: the library sums in the same one
        if (int(mask) >> p) & 1:
            e += k[p] * k[p]
    return e


def project_patterns(weights: np.ndarray, pattern_masks: np.ndarray):
    """-> (pattern_ids uint8 [c_out][c_in], projected fp32 weights): each kernel gets the
    pattern that retains the most energy; positions outside it are zeroed."""
    w = np.asarray(weights, dtype=np.float32)
    ids = np.zeros(w.shape[:2], dtype=np.uint8)
    out = np.zeros_like(w)
    for co in range(w.shape[0]):
        for ci in range(w.shape[1]):
            best, best_e = 0, -1.0
            for pid, m in enumerate(pattern_masks):
                e = retained_energy(w[co, ci], int(m))
                if e > best_e:
                    best, best_e = pid, e
            ids[co, ci] = best
            for p in range(9):
                if (int(pattern_masks[best]) >> p) & 1:
                    out[co, ci, p // 3, p % 3] = w[co, ci, p // 3, p % 3]
    return ids, out


def project_connectivity(weights: np.ndarray, alpha: int) -> np.ndarray:
    """-> kernel_mask uint8 [c_out][c_in] with exactly min(alpha, all) ones: the kernels of
    the largest L2 norms (squared norms compared, summed over positions 0..8 in order)."""
    w = np.asarray(weights, dtype=np.float32)
    c_out, c_in = w.shape[:2]
    norms = []
    for co in range(c_out):
        for ci in range(c_in):
            norms.append((-retained_energy(w[co, ci], 0x1FF), co * c_in + ci))
    norms.sort()
    mask = np.zeros((c_out, c_in), dtype=np.uint8)
    for _, flat in norms[:max(0, min(alpha, len(norms)))]:
        mask[flat // c_in, flat % c_in] = 1
    return mask
