"""ctypes binding of ``libpatdnn.so`` - argument marshalling only.

Function names mirror the C ABI (``include/patdnn.h``).  Device buffers are passed
as ``torch`` CUDA/HIP tensors (or raw integer device pointers); every arithmetic
step runs inside the library.  There is no fallback: if the library is missing,
loading raises.
"""

from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpatdnn.so")

PATDNN_OK, PATDNN_EINVAL, PATDNN_EPATTERN, PATDNN_ENOMEM, PATDNN_EHIP, PATDNN_EUNSUPPORTED = range(6)
PATDNN_DENSE, PATDNN_STRICT, PATDNN_HOST_ONLY = 1, 2, 4
PATDNN_VARIANT_FKW = 0

EXPORTS = [
    "patdnn_mine_patterns", "patdnn_project_patterns", "patdnn_project_connectivity",
    "patdnn_encode", "patdnn_conv2d", "patdnn_conv2d_f16", "patdnn_conv2d_pool", "patdnn_conv2d_ws", "patdnn_workspace_floats",
    "patdnn_output_shape", "patdnn_decode",
    "patdnn_stack_create", "patdnn_stack_output_shape", "patdnn_stack_run", "patdnn_stack_run_static", "patdnn_stack_destroy",
    "patdnn_export_fkw", "patdnn_export_csr", "patdnn_layout_stats", "patdnn_num_variants", "patdnn_variant_name",
    "patdnn_set_config", "patdnn_get_config", "patdnn_tune", "patdnn_tune_ws", "patdnn_tiled_info",
    "patdnn_export_tiled", "patdnn_selftest", "patdnn_destroy",
    "patdnn_status_string", "patdnn_last_error",
]


class LayerDesc(ctypes.Structure):
    _fields_ = [("c_out", ctypes.c_int32), ("c_in", ctypes.c_int32), ("groups", ctypes.c_int32),
                ("stride", ctypes.c_int32), ("pad", ctypes.c_int32),
                ("num_patterns", ctypes.c_int32), ("pattern_masks", ctypes.c_void_p),
                ("flags", ctypes.c_uint32)]


class Stats(ctypes.Structure):
    _fields_ = [("kept_kernels", ctypes.c_int64), ("taps", ctypes.c_int32),
                ("num_patterns", ctypes.c_int32), ("fkw_weight_bytes", ctypes.c_int64),
                ("fkw_index_bytes", ctypes.c_int64), ("tiled_bytes", ctypes.c_int64),
                ("min_filter_length", ctypes.c_int32), ("max_filter_length", ctypes.c_int32),
                ("distinct_filter_lengths", ctypes.c_int32), ("filter_groups", ctypes.c_int32),
                ("group_size", ctypes.c_int32), ("max_group_kernels", ctypes.c_int64),
                ("min_group_kernels", ctypes.c_int64)]


class Config(ctypes.Structure):
    _fields_ = [("variant", ctypes.c_int32), ("ck", ctypes.c_int32), ("waves", ctypes.c_int32),
                ("ksplit", ctypes.c_int32)]


class TiledInfo(ctypes.Structure):
    _fields_ = [("G", ctypes.c_int32), ("num_groups", ctypes.c_int32), ("ck", ctypes.c_int32),
                ("num_chunks", ctypes.c_int32), ("num_steps", ctypes.c_int64),
                ("block_bytes", ctypes.c_uint32), ("table_off", ctypes.c_uint32),
                ("ctrl_bytes", ctypes.c_uint32), ("records", ctypes.c_uint32),
                ("double_window", ctypes.c_int32), ("lds_channel_bytes", ctypes.c_int32),
                ("threaded", ctypes.c_int32), ("patch_rows", ctypes.c_int32),
                ("patch_cols", ctypes.c_int32), ("conv_stride", ctypes.c_int32),
                ("lanes_x", ctypes.c_int32), ("experimental", ctypes.c_int32),
                ("mode", ctypes.c_int32)]


class StackLayer(ctypes.Structure):
    _fields_ = [("layer", ctypes.c_void_p), ("bias", ctypes.c_void_p), ("fuse_relu", ctypes.c_int32),
                ("pool2", ctypes.c_int32)]


class PatdnnError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"patdnn status {status}: {text}")
        self.status = status


_lib = None


def lib() -> ctypes.CDLL:
    """Load the shared library (built by ``buildlib.build()``); raises if absent."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2001_00138_amd.buildlib`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        L.patdnn_encode.argtypes = [ctypes.POINTER(LayerDesc), vp, vp, vp, ctypes.POINTER(vp)]
        L.patdnn_conv2d.argtypes = [vp, vp, i32, i32, i32, vp, vp, i32, vp]
        L.patdnn_mine_patterns.argtypes = [vp, i32, i32, i32, vp, ctypes.POINTER(i32)]
        L.patdnn_project_patterns.argtypes = [vp, i32, i32, vp, i32, vp, vp]
        L.patdnn_project_connectivity.argtypes = [vp, i32, i32, ctypes.c_int64, vp]
        L.patdnn_conv2d_f16.argtypes = [vp, vp, i32, i32, i32, vp, vp, i32, vp]
        L.patdnn_conv2d_pool.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp]
        L.patdnn_conv2d_ws.argtypes = [vp, vp, i32, i32, i32, vp, vp, i32, i32, vp, ctypes.c_size_t, vp]
        L.patdnn_workspace_floats.argtypes = [vp, i32, i32, i32]
        L.patdnn_workspace_floats.restype = ctypes.c_size_t
        L.patdnn_stack_create.argtypes = [ctypes.POINTER(StackLayer), i32, i32, i32, i32, ctypes.POINTER(vp)]
        L.patdnn_stack_output_shape.argtypes = [vp, ctypes.POINTER(i32 * 4)]
        L.patdnn_stack_run.argtypes = [vp, vp, vp, i32, vp]
        L.patdnn_stack_run_static.argtypes = [vp, vp, vp, vp]
        L.patdnn_stack_destroy.argtypes = [vp]
        L.patdnn_stack_destroy.restype = None
        L.patdnn_output_shape.argtypes = [vp, i32, i32, i32, ctypes.POINTER(i32 * 4)]
        L.patdnn_decode.argtypes = [vp, vp, vp, vp]
        L.patdnn_export_fkw.argtypes = [vp, vp, vp, vp, vp, vp]
        L.patdnn_layout_stats.argtypes = [vp, ctypes.POINTER(Stats)]
        L.patdnn_export_csr.argtypes = [vp, ctypes.POINTER(ctypes.c_int64), vp, vp, vp]
        L.patdnn_num_variants.argtypes = []
        L.patdnn_variant_name.argtypes = [i32]
        L.patdnn_variant_name.restype = ctypes.c_char_p
        L.patdnn_set_config.argtypes = [vp, ctypes.POINTER(Config)]
        L.patdnn_get_config.argtypes = [vp, ctypes.POINTER(Config)]
        L.patdnn_tune.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, ctypes.POINTER(ctypes.c_float)]
        L.patdnn_tune_ws.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, ctypes.c_size_t, vp,
                                     ctypes.POINTER(ctypes.c_float)]
        L.patdnn_tiled_info.argtypes = [vp, i32, i32, ctypes.POINTER(TiledInfo)]
        L.patdnn_export_tiled.argtypes = [vp, i32, i32, vp, vp, vp]
        L.patdnn_selftest.argtypes = []
        L.patdnn_destroy.argtypes = [vp]
        L.patdnn_destroy.restype = None
        L.patdnn_status_string.argtypes = [i32]
        L.patdnn_status_string.restype = ctypes.c_char_p
        L.patdnn_last_error.argtypes = []
        L.patdnn_last_error.restype = ctypes.c_char_p
        for name in EXPORTS:
            if getattr(L, name).restype is ctypes.c_int:
                getattr(L, name).restype = ctypes.c_int32
        _lib = L
    return _lib


def _check(status: int) -> None:
    if status != PATDNN_OK:
        raise PatdnnError(status, (lib().patdnn_last_error() or b"").decode() or
                          lib().patdnn_status_string(status).decode())


def _host(a: Optional[np.ndarray], dtype) -> Tuple[Optional[np.ndarray], Optional[int]]:
    if a is None:
        return None, None
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data


def _devptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    if not t.is_cuda:
        raise ValueError("device tensor expected")
    if not t.is_contiguous():
        raise ValueError("contiguous tensor expected")
    return t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream or None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None


# ---------------------------------------------------------------------------
# functions named after the C entry points
# ---------------------------------------------------------------------------

def patdnn_mine_patterns(dense_weights, k: int) -> np.ndarray:
    """The k most frequent natural patterns of [c_out][kpf][3][3] weights (uint16 masks)."""
    w, wp = _host(dense_weights, np.float32)
    masks = np.zeros(k, np.uint16)
    found = ctypes.c_int32()
    _check(lib().patdnn_mine_patterns(wp, w.shape[0], w.shape[1], k, masks.ctypes.data, ctypes.byref(found)))
    return masks[:found.value]


def patdnn_project_patterns(dense_weights, pattern_masks):
    """-> (pattern_ids uint8 [c_out][kpf], projected fp32 weights)"""
    w, wp = _host(dense_weights, np.float32)
    pm, pp = _host(pattern_masks, np.uint16)
    ids = np.zeros(w.shape[:2], np.uint8)
    proj = np.empty_like(w)
    _check(lib().patdnn_project_patterns(wp, w.shape[0], w.shape[1], pp, len(pm), ids.ctypes.data,
                                         proj.ctypes.data))
    return ids, proj


def patdnn_project_connectivity(dense_weights, alpha: int) -> np.ndarray:
    """-> kernel_mask uint8 [c_out][kpf] keeping the alpha kernels of largest L2 norm"""
    w, wp = _host(dense_weights, np.float32)
    mask = np.zeros(w.shape[:2], np.uint8)
    _check(lib().patdnn_project_connectivity(wp, w.shape[0], w.shape[1], int(alpha), mask.ctypes.data))
    return mask


def patdnn_encode(dense_weights, pattern_ids, kernel_mask, pattern_masks, *, stride=1, pad=1,
                  groups=1, flags=0) -> int:
    """-> handle (int).  Host arrays as in the header; ``dense_weights`` is OIHW."""
    w, wp = _host(dense_weights, np.float32)
    if w.ndim != 4 or w.shape[2:] != (3, 3):
        raise ValueError("dense_weights must be [c_out][c_in/groups][3][3]")
    c_out, kpf = int(w.shape[0]), int(w.shape[1])
    c_in = kpf * groups
    ids, ip = _host(pattern_ids, np.uint8)
    km, kp = _host(kernel_mask, np.uint8)
    pm, pp = _host(pattern_masks, np.uint16)
    for a in (ids, km):
        if a is not None and a.shape != (c_out, kpf):
            raise ValueError("pattern_ids / kernel_mask must be [c_out][c_in/groups]")
    d = LayerDesc(c_out, c_in, groups, stride, pad, 0 if pm is None else len(pm), pp, flags)
    h = ctypes.c_void_p()
    _check(lib().patdnn_encode(ctypes.byref(d), wp, ip, kp, ctypes.byref(h)))
    return h.value


def patdnn_output_shape(handle: int, n: int, h_in: int, w_in: int):
    out = (ctypes.c_int32 * 4)()
    _check(lib().patdnn_output_shape(handle, n, h_in, w_in, ctypes.byref(out)))
    return tuple(out)


def patdnn_conv2d(handle: int, x, bias=None, out=None, *, fuse_relu=False, stream=None):
    """x: device tensor NCHW fp32.  Returns ``out`` (allocated with torch if None)."""
    import torch
    if x.dtype != torch.float32 or x.dim() != 4:
        raise ValueError("input must be a 4-d float32 tensor")
    n, _, h_in, w_in = x.shape
    shape = patdnn_output_shape(handle, n, h_in, w_in)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    elif tuple(out.shape) != shape or out.dtype != torch.float32:
        raise ValueError(f"output must be float32 {shape}")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != shape[1]):
        raise ValueError("bias must be float32 [c_out]")
    _check(lib().patdnn_conv2d(handle, _devptr(x), n, h_in, w_in, _devptr(bias), _devptr(out),
                               int(bool(fuse_relu)), _stream_ptr(stream)))
    return out


def patdnn_workspace_floats(handle: int, n: int, h_in: int, w_in: int) -> int:
    return int(lib().patdnn_workspace_floats(handle, n, h_in, w_in))


def patdnn_conv2d_ws(handle: int, x, bias=None, out=None, *, workspace=None, fuse_relu=False, pool=False,
                     stream=None):
    """patdnn_conv2d / patdnn_conv2d_pool with a caller-owned workspace (a float32 device tensor)
    for the partial sums of a configuration that splits the input channels."""
    import torch
    if x.dtype != torch.float32 or x.dim() != 4:
        raise ValueError("input must be a 4-d float32 tensor")
    n, _, h_in, w_in = x.shape
    full = patdnn_output_shape(handle, n, h_in, w_in)
    shape = (full[0], full[1], full[2] // 2, full[3] // 2) if pool else full
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    elif tuple(out.shape) != shape or out.dtype != torch.float32:
        raise ValueError(f"output must be float32 {shape}")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != shape[1]):
        raise ValueError("bias must be float32 [c_out]")
    if workspace is not None and (workspace.dtype != torch.float32 or not workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous float32 tensor")
    _check(lib().patdnn_conv2d_ws(handle, _devptr(x), n, h_in, w_in, _devptr(bias), _devptr(out),
                                  int(bool(fuse_relu)), int(bool(pool)), _devptr(workspace),
                                  0 if workspace is None else workspace.numel(), _stream_ptr(stream)))
    return out


def patdnn_conv2d_f16(handle: int, x, bias=None, out=None, *, fuse_relu=False, stream=None):
    """x, out: float16 device tensors (half-precision storage); bias float32."""
    import torch
    if x.dtype != torch.float16 or x.dim() != 4:
        raise ValueError("input must be a 4-d float16 tensor")
    n, _, h_in, w_in = x.shape
    shape = patdnn_output_shape(handle, n, h_in, w_in)
    if out is None:
        out = torch.empty(shape, dtype=torch.float16, device=x.device)
    elif tuple(out.shape) != shape or out.dtype != torch.float16:
        raise ValueError(f"output must be float16 {shape}")
    if bias is not None and (bias.dtype != torch.float32 or bias.numel() != shape[1]):
        raise ValueError("bias must be float32 [c_out]")
    _check(lib().patdnn_conv2d_f16(handle, _devptr(x), n, h_in, w_in, _devptr(bias), _devptr(out),
                                   int(bool(fuse_relu)), _stream_ptr(stream)))
    return out


def patdnn_conv2d_pool(handle: int, x, bias=None, out=None, *, stream=None):
    """conv + bias + ReLU + 2x2 max pooling, fused.  Returns ``out`` [n][c_out][h_out/2][w_out/2]."""
    import torch
    if x.dtype != torch.float32 or x.dim() != 4:
        raise ValueError("input must be a 4-d float32 tensor")
    n, _, h_in, w_in = x.shape
    full = patdnn_output_shape(handle, n, h_in, w_in)
    shape = (full[0], full[1], full[2] // 2, full[3] // 2)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=x.device)
    elif tuple(out.shape) != shape or out.dtype != torch.float32:
        raise ValueError(f"output must be float32 {shape}")
    _check(lib().patdnn_conv2d_pool(handle, _devptr(x), n, h_in, w_in, _devptr(bias), _devptr(out),
                                    _stream_ptr(stream)))
    return out


class Stack:
    """patdnn_stack_*: layers run back to back; ``layers`` = [(Layer, bias tensor or None, relu, pool2)]."""

    def __init__(self, layers, n: int, h_in: int, w_in: int):
        self._keep = list(layers)               # handles and bias tensors must outlive the stack
        arr = (StackLayer * len(layers))()
        for i, (L, bias, relu, pool) in enumerate(layers):
            arr[i] = StackLayer(L.handle, _devptr(bias), int(bool(relu)), int(bool(pool)))
        h = ctypes.c_void_p()
        _check(lib().patdnn_stack_create(arr, len(layers), n, h_in, w_in, ctypes.byref(h)))
        self.handle = h.value

    def output_shape(self):
        out = (ctypes.c_int32 * 4)()
        _check(lib().patdnn_stack_output_shape(self.handle, ctypes.byref(out)))
        return tuple(out)

    def run(self, x, out=None, *, graph=False, stream=None):
        import torch
        if out is None:
            out = torch.empty(self.output_shape(), dtype=torch.float32, device=x.device)
        _check(lib().patdnn_stack_run(self.handle, _devptr(x), _devptr(out), int(bool(graph)),
                                      _stream_ptr(stream)))
        return out

    def run_static(self, x, out, *, stream=None):
        """patdnn_stack_run_static: the library's built-in buffer instead of the stack's own."""
        _check(lib().patdnn_stack_run_static(self.handle, _devptr(x), _devptr(out), _stream_ptr(stream)))
        return out

    def close(self):
        if self.handle:
            lib().patdnn_stack_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def patdnn_layout_stats(handle: int) -> dict:
    s = Stats()
    _check(lib().patdnn_layout_stats(handle, ctypes.byref(s)))
    return {k: getattr(s, k) for k, _ in Stats._fields_}


def patdnn_decode(handle: int, c_out: int, kernels_per_filter: int):
    w = np.empty((c_out, kernels_per_filter, 3, 3), dtype=np.float32)
    ids = np.empty((c_out, kernels_per_filter), dtype=np.uint8)
    km = np.empty((c_out, kernels_per_filter), dtype=np.uint8)
    _check(lib().patdnn_decode(handle, w.ctypes.data, ids.ctypes.data, km.ctypes.data))
    return w, ids, km


def patdnn_export_fkw(handle: int, c_out: int) -> dict:
    st = patdnn_layout_stats(handle)
    kept, taps, P = st["kept_kernels"], st["taps"], st["num_patterns"]
    out = {"offset": np.empty(c_out + 1, np.int32), "reorder": np.empty(c_out, np.int32),
           "index": np.empty(kept, np.int32), "stride": np.empty((c_out, P + 1), np.int32),
           "weight": np.empty((kept, taps), np.float32)}
    _check(lib().patdnn_export_fkw(handle, *(out[k].ctypes.data for k in
                                             ("offset", "reorder", "index", "stride", "weight"))))
    return out


def patdnn_export_csr(handle: int, c_out: int) -> dict:
    nnz = ctypes.c_int64()
    _check(lib().patdnn_export_csr(handle, ctypes.byref(nnz), None, None, None))
    out = {"row_ptr": np.empty(c_out + 1, np.int32), "col": np.empty(nnz.value, np.int32),
           "val": np.empty(nnz.value, np.float32)}
    _check(lib().patdnn_export_csr(handle, None, out["row_ptr"].ctypes.data, out["col"].ctypes.data,
                                   out["val"].ctypes.data))
    return out


def patdnn_num_variants() -> int:
    return int(lib().patdnn_num_variants())


def patdnn_variant_name(v: int) -> Optional[str]:
    s = lib().patdnn_variant_name(v)
    return None if s is None else s.decode()


def patdnn_set_config(handle: int, variant: int, ck: int = 0, waves: int = 0, ksplit: int = 0) -> None:
    c = Config(variant, ck, waves, ksplit)
    _check(lib().patdnn_set_config(handle, ctypes.byref(c)))


def patdnn_get_config(handle: int) -> dict:
    c = Config()
    _check(lib().patdnn_get_config(handle, ctypes.byref(c)))
    return {"variant": c.variant, "ck": c.ck, "waves": c.waves, "ksplit": c.ksplit}


def patdnn_tune(handle: int, x, bias, out, *, workspace=None, stream=None) -> float:
    """Times every applicable configuration on the given buffers (split configurations with the
    workspace, a float32 device tensor, if one is given); returns best microseconds."""
    n, _, h_in, w_in = x.shape
    best = ctypes.c_float()
    if workspace is None:
        _check(lib().patdnn_tune(handle, _devptr(x), n, h_in, w_in, _devptr(bias), _devptr(out),
                                 _stream_ptr(stream), ctypes.byref(best)))
    else:
        _check(lib().patdnn_tune_ws(handle, _devptr(x), n, h_in, w_in, _devptr(bias), _devptr(out),
                                    _devptr(workspace), workspace.numel(), _stream_ptr(stream), ctypes.byref(best)))
    return float(best.value)


def patdnn_tiled_info(handle: int, variant: int, ck: int = 0) -> dict:
    t = TiledInfo()
    _check(lib().patdnn_tiled_info(handle, variant, ck, ctypes.byref(t)))
    return {k: getattr(t, k) for k, _ in TiledInfo._fields_}


def patdnn_export_tiled(handle: int, variant: int, ck: int = 0) -> dict:
    """The filter-group layout of a tiled sparse variant: info fields plus the arrays."""
    info = patdnn_tiled_info(handle, variant, ck)
    out = dict(info)
    out["slot_channel"] = np.empty((info["num_groups"], info["G"]), np.int32)
    out["chunk_ptr"] = np.empty((info["num_groups"], info["num_chunks"]), np.uint32)
    out["steps"] = np.empty((info["num_steps"], 24), np.uint32)
    _check(lib().patdnn_export_tiled(handle, variant, ck, out["slot_channel"].ctypes.data,
                                     out["chunk_ptr"].ctypes.data, out["steps"].ctypes.data))
    return out


def patdnn_selftest() -> None:
    """Raises PatdnnError (EUNSUPPORTED) if the device fails the scalar-relative-move check."""
    _check(lib().patdnn_selftest())


def patdnn_destroy(handle: Optional[int]) -> None:
    if handle:
        lib().patdnn_destroy(handle)


# ---------------------------------------------------------------------------
# convenience wrapper owning one handle
# ---------------------------------------------------------------------------

class Layer:
    def __init__(self, dense_weights, pattern_ids, kernel_mask, pattern_masks, *, stride=1, pad=1,
                 depthwise=False, dense=False, strict=False, host_only=False):
        w = np.asarray(dense_weights)
        flags = (PATDNN_DENSE if dense else 0) | (PATDNN_STRICT if strict else 0) | \
                (PATDNN_HOST_ONLY if host_only else 0)
        self.c_out, self.kpf = int(w.shape[0]), int(w.shape[1])
        self.handle = patdnn_encode(w, pattern_ids, kernel_mask, pattern_masks, stride=stride,
                                    pad=pad, groups=self.c_out if depthwise else 1, flags=flags)

    @classmethod
    def from_workload(cls, layer: dict, **kw) -> "Layer":
        spec = layer["spec"]
        return cls(layer["weights"], layer["pattern_ids"], layer["kernel_mask"],
                   layer["pattern_masks"], stride=spec.stride, pad=spec.pad,
                   depthwise=spec.depthwise, dense=spec.dense, **kw)

    def conv2d(self, x, bias=None, out=None, *, relu=False, stream=None):
        return patdnn_conv2d(self.handle, x, bias, out, fuse_relu=relu, stream=stream)

    def conv2d_ws(self, x, bias=None, out=None, *, workspace=None, relu=False, pool=False, stream=None):
        return patdnn_conv2d_ws(self.handle, x, bias, out, workspace=workspace, fuse_relu=relu, pool=pool,
                                stream=stream)

    def workspace_floats(self, n, h, w):
        return patdnn_workspace_floats(self.handle, n, h, w)

    def conv2d_f16(self, x, bias=None, out=None, *, relu=False, stream=None):
        return patdnn_conv2d_f16(self.handle, x, bias, out, fuse_relu=relu, stream=stream)

    def conv2d_pool(self, x, bias=None, out=None, *, stream=None):
        return patdnn_conv2d_pool(self.handle, x, bias, out, stream=stream)

    def output_shape(self, n, h, w):
        return patdnn_output_shape(self.handle, n, h, w)

    def decode(self):
        return patdnn_decode(self.handle, self.c_out, self.kpf)

    def export_fkw(self):
        return patdnn_export_fkw(self.handle, self.c_out)

    def export_csr(self):
        return patdnn_export_csr(self.handle, self.c_out)

    def stats(self):
        return patdnn_layout_stats(self.handle)

    def set_config(self, variant, ck=0, waves=0, ksplit=0):
        patdnn_set_config(self.handle, variant, ck, waves, ksplit)

    def get_config(self):
        return patdnn_get_config(self.handle)

    def export_tiled(self, variant, ck=0):
        return patdnn_export_tiled(self.handle, variant, ck)

    def tune(self, x, bias, out, *, workspace=None, stream=None):
        return patdnn_tune(self.handle, x, bias, out, workspace=workspace, stream=stream)

    def close(self):
        patdnn_destroy(self.handle)
        self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
