"""Seeded synthetic workloads shaped like the paper's evaluation layers.

The paper evaluates pattern- and connectivity-pruned VGG-16, ResNet-50 and
MobileNet-V2 (section 6.1); the trained models are not available, so every
layer here is drawn from a seed with the same shapes, the same structure
(8 four-entry patterns that keep the centre weight, section 4.1; a uniform
3.6x connectivity pruning rate with the first layer left alone, section 4.2
and 4.3) and He-scale values.

This module contains data generation only: no convolution, no masking of
weights, no layout logic.  Both the HIP library and the CPU oracle receive the
arrays produced here; neither is imported from here.
"""

from __future__ import annotations

import itertools
from dataclasses import dataclass, replace
from typing import Dict, List, Optional

import numpy as np

# ---------------------------------------------------------------------------
# pattern library (section 4.1: 4-entry patterns that keep the centre weight,
# C(8,3) = 56 candidates)
# ---------------------------------------------------------------------------

CENTRE = 4  # row-major position 3*kh + kw of the centre tap


def pattern_universe() -> np.ndarray:
    """All 56 candidate masks as uint16, bit (3*kh+kw) set = weight kept.

    Enumerated as the lexicographic 3-combinations of the eight non-centre
    positions, plus the centre.
    """
    others = [p for p in range(9) if p != CENTRE]
    masks = []
    for combo in itertools.combinations(others, 3):
        m = 1 << CENTRE
        for p in combo:
            m |= 1 << p
        masks.append(m)
    return np.asarray(masks, dtype=np.uint16)


def pattern_library(seed: int, k: int = 8) -> np.ndarray:
    """k masks drawn without replacement from the 56, universe index ascending."""
    uni = pattern_universe()
    rng = np.random.default_rng(np.random.SeedSequence([int(seed), 0x9A77]))
    pick = np.sort(rng.choice(len(uni), size=k, replace=False))
    return uni[pick].copy()


# ---------------------------------------------------------------------------
# layer descriptions
# ---------------------------------------------------------------------------

@dataclass(frozen=True)
class LayerSpec:
    name: str
    c_in: int
    c_out: int
    h: int
    w: int
    stride: int = 1
    pad: int = 1
    depthwise: bool = False
    dense: bool = False          # first VGG layer: no pruning at all
    n: int = 1
    keep: str = "layer"          # "layer": round(C_in*C_out/3.6) over the whole grid
                                 # "half_per_filter": exactly C_in/2 per filter
                                 # "all": nothing removed
    input_dist: str = "normal"   # "normal", "relu_normal", "uniform"
    relu: bool = True

    @property
    def h_out(self) -> int:
        return (self.h + 2 * self.pad - 3) // self.stride + 1

    @property
    def w_out(self) -> int:
        return (self.w + 2 * self.pad - 3) // self.stride + 1

    @property
    def kernels_per_filter(self) -> int:
        return 1 if self.depthwise else self.c_in


def _vgg16(n: int, first_input: str = "normal") -> List[LayerSpec]:
    shapes = [
        (3, 64, 224), (64, 64, 224),
        (64, 128, 112), (128, 128, 112),
        (128, 256, 56), (256, 256, 56), (256, 256, 56),
        (256, 512, 28), (512, 512, 28), (512, 512, 28),
        (512, 512, 14), (512, 512, 14), (512, 512, 14),
    ]
    out = []
    for i, (ci, co, hw) in enumerate(shapes):
        out.append(LayerSpec(
            name=f"vgg16_L{i + 1}", c_in=ci, c_out=co, h=hw, w=hw, n=n,
            dense=(i == 0), keep="all" if i == 0 else "layer",
            input_dist="normal" if i == 0 else "relu_normal"))
    return out


def _resnet50() -> List[LayerSpec]:
    # the 3x3 convolution of each of the 16 bottleneck blocks; the first block
    # of stages 2-4 carries the stride
    plan = [(64, 56, 1)] * 3 + [(128, 56, 2)] + [(128, 28, 1)] * 3 + \
           [(256, 28, 2)] + [(256, 14, 1)] * 5 + [(512, 14, 2)] + [(512, 7, 1)] * 2
    return [LayerSpec(name=f"resnet50_R{i + 1}", c_in=c, c_out=c, h=hw, w=hw,
                      stride=s, input_dist="relu_normal")
            for i, (c, hw, s) in enumerate(plan)]


def _mobilenet_v2() -> List[LayerSpec]:
    plan = [(32, 112, 1), (96, 112, 2), (144, 56, 1), (144, 56, 2),
            (192, 28, 1), (192, 28, 1), (192, 28, 2),
            (384, 14, 1), (384, 14, 1), (384, 14, 1), (384, 14, 1),
            (576, 14, 1), (576, 14, 1), (576, 14, 2),
            (960, 7, 1), (960, 7, 1), (960, 7, 1)]
    return [LayerSpec(name=f"mbv2_D{i + 1}", c_in=c, c_out=c, h=hw, w=hw, stride=s,
                      depthwise=True, keep="all", input_dist="relu_normal")
            for i, (c, hw, s) in enumerate(plan)]


def config_layers(config: int) -> List[LayerSpec]:
    """The layer list of workload configuration 1..5."""
    if config == 1:
        return [LayerSpec(name="small_16x16x32", c_in=16, c_out=16, h=32, w=32,
                          keep="half_per_filter", input_dist="uniform")]
    if config == 2:
        return _vgg16(1)
    if config == 3:
        return _resnet50()
    if config == 4:
        return _mobilenet_v2()
    if config == 5:
        return _vgg16(64)
    raise ValueError(f"unknown workload configuration {config}")


CONFIG_NAMES = {
    1: "single 16->16 3x3 conv @32x32, N=1",
    2: "VGG-16 13-layer 3x3 stack, N=1",
    3: "ResNet-50 3x3 bottleneck convs (16 layers), N=1",
    4: "MobileNet-V2 depthwise 3x3 convs (17 layers), N=1",
    5: "VGG-16 13-layer 3x3 stack, N=64 (throughput case)",
}

PATTERN_SEED = 2001_00138   # one library for every configuration


# ---------------------------------------------------------------------------
# seeded tensors
# ---------------------------------------------------------------------------

_STREAMS = {"ids": 1, "mask": 2, "weights": 3, "bias": 4, "input": 5}


def _rng(config: int, layer: int, what: str, extra: int = 0) -> np.random.Generator:
    return np.random.default_rng(
        np.random.SeedSequence([1000 * int(config) + int(layer), _STREAMS[what], int(extra)]))


def round_half_even(x: float) -> int:
    return int(np.rint(x))


def kept_kernel_count(spec: LayerSpec) -> int:
    kpf = spec.kernels_per_filter
    if spec.keep == "all":
        return spec.c_out * kpf
    if spec.keep == "half_per_filter":
        return spec.c_out * (kpf // 2)
    return round_half_even(spec.c_out * kpf / 3.6)


def gen_structure(spec: LayerSpec, config: int, layer: int, num_patterns: int = 8):
    """(pattern_ids, kernel_mask), both uint8 [c_out][kernels_per_filter]."""
    kpf = spec.kernels_per_filter
    ids = _rng(config, layer, "ids").integers(
        0, num_patterns, size=(spec.c_out, kpf), dtype=np.uint8)
    r = _rng(config, layer, "mask")
    if spec.keep == "all":
        mask = np.ones((spec.c_out, kpf), dtype=np.uint8)
    elif spec.keep == "half_per_filter":
        mask = np.zeros((spec.c_out, kpf), dtype=np.uint8)
        for co in range(spec.c_out):
            mask[co, r.permutation(kpf)[: kpf // 2]] = 1
    else:
        kept = kept_kernel_count(spec)
        flat = np.zeros(spec.c_out * kpf, dtype=np.uint8)
        flat[r.permutation(spec.c_out * kpf)[:kept]] = 1
        mask = flat.reshape(spec.c_out, kpf)
    return ids, mask


def gen_weights(spec: LayerSpec, config: int, layer: int) -> np.ndarray:
    """He-normal OIHW float32 weights, std sqrt(2 / (9 * fan-in channels))."""
    kpf = spec.kernels_per_filter
    std = np.sqrt(2.0 / (9.0 * kpf))
    w = _rng(config, layer, "weights").standard_normal(
        size=(spec.c_out, kpf, 3, 3), dtype=np.float32)
    return (w * np.float32(std)).astype(np.float32)


def gen_bias(spec: LayerSpec, config: int, layer: int) -> np.ndarray:
    b = _rng(config, layer, "bias").standard_normal(size=(spec.c_out,), dtype=np.float32)
    return (b * np.float32(0.01)).astype(np.float32)


def gen_input_image(spec: LayerSpec, config: int, layer: int, image: int) -> np.ndarray:
    """One image [c_in][h][w] float32; each image has a seed of its own so that
    any subset of a large batch can be regenerated on its own."""
    r = _rng(config, layer, "input", image)
    shape = (spec.c_in, spec.h, spec.w)
    if spec.input_dist == "uniform":
        return r.random(size=shape, dtype=np.float32)
    x = r.standard_normal(size=shape, dtype=np.float32)
    if spec.input_dist == "relu_normal":
        np.maximum(x, np.float32(0), out=x)
    return x


def gen_input(spec: LayerSpec, config: int, layer: int, n: Optional[int] = None) -> np.ndarray:
    n = spec.n if n is None else n
    out = np.empty((n, spec.c_in, spec.h, spec.w), dtype=np.float32)
    for i in range(n):
        out[i] = gen_input_image(spec, config, layer, i)
    return out


def gen_layer(config: int, layer: int, n: Optional[int] = None,
              with_input: bool = True) -> Dict[str, object]:
    """Everything one layer needs: spec, pattern masks, ids, mask, weights, bias, input."""
    spec = config_layers(config)[layer]
    if n is not None:
        spec = replace(spec, n=n)
    lib = pattern_library(PATTERN_SEED)
    ids, mask = gen_structure(spec, config, layer, len(lib))
    out = {
        "spec": spec, "config": config, "layer": layer,
        "pattern_masks": lib, "pattern_ids": ids, "kernel_mask": mask,
        "weights": gen_weights(spec, config, layer),
        "bias": gen_bias(spec, config, layer),
    }
    if with_input:
        out["input"] = gen_input(spec, config, layer, spec.n)
    return out


# ---------------------------------------------------------------------------
# work counting (the paper reports "pure GFLOPS", section 6.3; both conventions)
# ---------------------------------------------------------------------------

def nz_flops(spec: LayerSpec, kept: int, n: Optional[int] = None) -> int:
    """2 flop x taps x kept kernels x output pixels (taps = 4, or 9 for a dense layer)."""
    n = spec.n if n is None else n
    taps = 9 if spec.dense else 4
    return 2 * taps * kept * spec.h_out * spec.w_out * n


def dense_flops(spec: LayerSpec, n: Optional[int] = None) -> int:
    n = spec.n if n is None else n
    return 2 * 9 * spec.c_out * spec.kernels_per_filter * spec.h_out * spec.w_out * n


def algorithmic_bytes(spec: LayerSpec, kept: int, n: Optional[int] = None) -> int:
    """Input once + output once + compressed weights (16 B + 2 B index per kept
    kernel; 36 B per kernel for a dense layer) + bias."""
    n = spec.n if n is None else n
    act = 4 * n * (spec.c_in * spec.h * spec.w + spec.c_out * spec.h_out * spec.w_out)
    per_kernel = 36 if spec.dense else 18
    return act + per_kernel * kept + 4 * spec.c_out


# ---------------------------------------------------------------------------
# launch configurations kept with the layer shapes (section 5.5: the tuner's result is
# written back into the layer's description).  Plain data: names and numbers.
# ---------------------------------------------------------------------------

def shape_key(spec: LayerSpec) -> str:
    kind = "dw" if spec.depthwise else ("dense" if spec.dense else "sparse")
    return f"{kind}:{spec.c_in}->{spec.c_out}@{spec.h}x{spec.w}:s{spec.stride}p{spec.pad}:n{spec.n}"


def load_tuned_configs(path: str) -> dict:
    """{shape_key: {"variant": name, "ck": .., "waves": .., "ksplit": ..}}; {} if the file is absent."""
    import json
    try:
        with open(path) as f:
            table = json.load(f)
    except OSError:
        return {}
    return {k: v for k, v in table.items()
            if isinstance(v, dict) and {"variant", "ck", "waves", "ksplit"} <= set(v)}
