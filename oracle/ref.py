"""Python face of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg may import this module.  It shares nothing with the HIP library: the C file
beside it is compiled with gcc into ``libpatdnn_ref.so`` and called through
ctypes; the two numpy helpers below are definitions written out.

Operation: paper section 2.1 (CONV layer followed by ReLU), with the weight
tensor constrained as in section 4.2 (each kernel keeps only the positions of
its pattern; kernels removed by connectivity pruning are zero).
"""

from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "patdnn_ref.c")
_LIB = os.path.join(_HERE, "libpatdnn_ref.so")
_lib = None


class _Desc(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int32) for k in (
        "c_out", "c_in", "depthwise", "dense", "stride", "pad",
        "num_patterns", "relu", "skip_removed", "nthreads")]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  Generic x86-64 code (the library is built in
    one container and may run on another host), no fast-math, no FMA contraction."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-ffp-contract=off", "-fPIC", "-shared",
               "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        vp = ctypes.c_void_p
        lib.patdnn_ref_conv2d.restype = ctypes.c_int
        lib.patdnn_ref_conv2d.argtypes = [ctypes.POINTER(_Desc), vp, vp, vp, vp, vp,
                                          ctypes.c_int, ctypes.c_int, ctypes.c_int, vp, vp]
        lib.patdnn_ref_conv2d_points.restype = ctypes.c_int
        lib.patdnn_ref_conv2d_points.argtypes = [ctypes.POINTER(_Desc), vp, vp, vp, vp, vp,
                                                 ctypes.c_int, ctypes.c_int, ctypes.c_int, vp,
                                                 vp, ctypes.c_long, vp]
        lib.patdnn_ref_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().patdnn_ref_num_threads())


def out_shape(h: int, w: int, stride: int, pad: int):
    return (h + 2 * pad - 3) // stride + 1, (w + 2 * pad - 3) // stride + 1


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _prep(weights, pattern_ids, kernel_mask, pattern_masks, x, bias, depthwise, dense):
    w = np.ascontiguousarray(weights, dtype=np.float32)
    assert w.ndim == 4 and w.shape[2:] == (3, 3)
    c_out, kpf = w.shape[0], w.shape[1]
    x = np.ascontiguousarray(x, dtype=np.float32)
    assert x.ndim == 4
    c_in = x.shape[1]
    if depthwise:
        assert kpf == 1 and c_in == c_out
    else:
        assert kpf == c_in
    ids = None if pattern_ids is None else np.ascontiguousarray(pattern_ids, dtype=np.uint8)
    km = None if kernel_mask is None else np.ascontiguousarray(kernel_mask, dtype=np.uint8)
    pm = None if pattern_masks is None else np.ascontiguousarray(pattern_masks, dtype=np.uint16)
    if ids is not None:
        assert ids.shape == (c_out, kpf)
    if km is not None:
        assert km.shape == (c_out, kpf)
    b = None if bias is None else np.ascontiguousarray(bias, dtype=np.float32)
    if b is not None:
        assert b.shape == (c_out,)
    return w, ids, km, pm, x, b, c_out, c_in


def conv2d(weights, pattern_ids, kernel_mask, pattern_masks, x, bias=None, *,
           stride: int = 1, pad: int = 1, relu: bool = False, depthwise: bool = False,
           dense: bool = False, skip_removed: bool = False, nthreads: int = 0) -> np.ndarray:
    """Full NCHW float64 output of the pruned convolution (definition in patdnn_ref.c)."""
    w, ids, km, pm, x, b, c_out, c_in = _prep(weights, pattern_ids, kernel_mask,
                                              pattern_masks, x, bias, depthwise, dense)
    n, _, h, wd = x.shape
    ho, wo = out_shape(h, wd, stride, pad)
    d = _Desc(c_out, c_in, int(depthwise), int(dense), stride, pad,
              0 if pm is None else len(pm), int(relu), int(skip_removed), nthreads)
    out = np.empty((n, c_out, max(ho, 0), max(wo, 0)), dtype=np.float64)
    rc = _load().patdnn_ref_conv2d(ctypes.byref(d), _ptr(w), _ptr(ids), _ptr(km), _ptr(pm),
                                   _ptr(x), n, h, wd, _ptr(b), _ptr(out))
    if rc:
        raise ValueError(f"patdnn_ref_conv2d rejected its arguments (code {rc})")
    return out


def conv2d_points(weights, pattern_ids, kernel_mask, pattern_masks, x, bias, coords, *,
                  stride: int = 1, pad: int = 1, relu: bool = False, depthwise: bool = False,
                  dense: bool = False, nthreads: int = 0) -> np.ndarray:
    """Output values at coords [npts][4] = (n, co, oh, ow) only."""
    w, ids, km, pm, x, b, c_out, c_in = _prep(weights, pattern_ids, kernel_mask,
                                              pattern_masks, x, bias, depthwise, dense)
    n, _, h, wd = x.shape
    c = np.ascontiguousarray(coords, dtype=np.int32).reshape(-1, 4)
    d = _Desc(c_out, c_in, int(depthwise), int(dense), stride, pad,
              0 if pm is None else len(pm), int(relu), 0, nthreads)
    out = np.empty((len(c),), dtype=np.float64)
    rc = _load().patdnn_ref_conv2d_points(ctypes.byref(d), _ptr(w), _ptr(ids), _ptr(km),
                                          _ptr(pm), _ptr(x), n, h, wd, _ptr(b), _ptr(c),
                                          len(c), _ptr(out))
    if rc:
        raise ValueError(f"patdnn_ref_conv2d_points rejected its arguments (code {rc})")
    return out


def tap_positions(mask: int) -> Sequence[int]:
    """Row-major positions 3*kh+kw kept by a pattern mask, ascending."""
    return [p for p in range(9) if (int(mask) >> p) & 1]


def masked_weights(weights, pattern_ids, kernel_mask, pattern_masks, dense: bool = False) -> np.ndarray:
    """The weight tensor the pruned layer actually holds (section 4.2): original fp32
    bits at the positions of each surviving kernel's pattern, +0.0 everywhere else.
    This is what a lossless compact storage must decode back to."""
    w = np.ascontiguousarray(weights, dtype=np.float32)
    out = np.zeros_like(w)
    c_out, kpf = w.shape[:2]
    for co in range(c_out):
        for k in range(kpf):
            if kernel_mask is not None and not kernel_mask[co, k]:
                continue
            m = 0x1FF if dense else int(pattern_masks[pattern_ids[co, k]])
            for p in tap_positions(m):
                out[co, k, p // 3, p % 3] = w[co, k, p // 3, p % 3]
    return out
