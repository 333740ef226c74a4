"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by
element, on identical seeded inputs.  Bar: max|err| / max|ref| <= 1e-5 (fp32 FMA
accumulation in any order against an fp64 reference); exact where the result is
exactly representable (zeros, act(bias))."""

import os
import sys

import numpy as np
import pytest

from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.lib()     # the HIP library must be there; no fallback exists
    return torch


def _rel_err(got, ref):
    scale = float(np.abs(ref).max())
    err = float(np.abs(got.astype(np.float64) - ref).max())
    return err / scale if scale > 0 else err


def _gpu_conv(torch, L, x_np, bias_np, relu, canary=True):
    """Run the layer with the output carved out of a larger sentinel-filled buffer, so
    that any write outside the output tensor is seen."""
    x = torch.from_numpy(x_np).cuda()
    bias = None if bias_np is None else torch.from_numpy(bias_np).cuda()
    shape = L.output_shape(x_np.shape[0], x_np.shape[2], x_np.shape[3])
    numel = int(np.prod(shape))
    guard = 4096
    buf = torch.full((numel + 2 * guard,), 12345.0, dtype=torch.float32, device="cuda")
    out = buf[guard:guard + numel].view(shape)
    L.conv2d(x, bias, out, relu=relu)
    torch.cuda.synchronize()
    if canary:
        assert bool((buf[:guard] == 12345.0).all()) and bool((buf[guard + numel:] == 12345.0).all())
    return out.cpu().numpy()


def _check_layer(torch, oracle, d, x, relu=True, use_bias=True, configs=(None,)):
    spec = d["spec"]
    bias = d["bias"] if use_bias else None
    ref = oracle.conv2d(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], x,
                        bias, stride=spec.stride, pad=spec.pad, relu=relu,
                        depthwise=spec.depthwise, dense=spec.dense, skip_removed=True)
    L = B.Layer.from_workload(d)
    try:
        for cfg in configs:
            if cfg is not None:
                try:
                    L.set_config(*cfg)
                except B.PatdnnError as e:
                    assert e.status == B.PATDNN_EUNSUPPORTED
                    continue
            got = _gpu_conv(torch, L, x, bias, relu)
            assert got.shape == ref.shape
            err = _rel_err(got, ref)
            _say(f"    {spec.name} cfg={cfg} rel_err={err:.2e}")
            assert err <= TOL, (spec.name, cfg, err)
    finally:
        L.close()


def _all_configs():
    out = [(0, 0, 0)]
    for v in range(1, B.patdnn_num_variants()):
        out += [(v, 0, 0), (v, 3, 2), (v, 16, 4), (v, 5, 8)]
    return out


def test_config1_every_variant(torch, oracle):
    d = wl.gen_layer(1, 0)
    _check_layer(torch, oracle, d, d["input"], configs=[None] + _all_configs())
    _check_layer(torch, oracle, d, d["input"], relu=False, use_bias=False, configs=[None, (0, 0, 0)])


@pytest.mark.parametrize("config", [2, 3, 4])
def test_every_layer_of_config(torch, oracle, config):
    for li, spec in enumerate(wl.config_layers(config)):
        _say(f"  config {config} layer {li} {spec.name}")
        d = wl.gen_layer(config, li)
        _check_layer(torch, oracle, d, d["input"], configs=[None, (0, 0, 0)])


def _random_layer(rng, c_out, c_in, keep, dense=False, depthwise=False, stride=1, pad=1):
    lib = wl.pattern_library(wl.PATTERN_SEED)
    kpf = 1 if depthwise else c_in
    spec = wl.LayerSpec(name=f"rand_{c_in}x{c_out}_s{stride}p{pad}", c_in=c_in, c_out=c_out, h=0, w=0,
                        stride=stride, pad=pad, depthwise=depthwise, dense=dense)
    return {"spec": spec, "pattern_masks": lib,
            "pattern_ids": rng.integers(0, 8, (c_out, kpf), dtype=np.uint8),
            "kernel_mask": (rng.random((c_out, kpf)) < keep).astype(np.uint8),
            "weights": rng.standard_normal((c_out, kpf, 3, 3)).astype(np.float32),
            "bias": rng.standard_normal(c_out).astype(np.float32)}


@pytest.mark.parametrize("case", [
    dict(c_out=24, c_in=20, n=3, h=13, w=13, keep=0.3),           # ragged everywhere
    dict(c_out=40, c_in=7, n=2, h=29, w=17, keep=0.5),
    dict(c_out=16, c_in=33, n=5, h=7, w=50, keep=0.25),
    dict(c_out=70, c_in=64, n=1, h=15, w=16, keep=0.28),
    dict(c_out=8, c_in=8, n=2, h=3, w=3, keep=1.0),               # smallest image
    dict(c_out=32, c_in=16, n=2, h=20, w=20, keep=0.3, pad=0),
    dict(c_out=32, c_in=16, n=2, h=21, w=20, keep=0.3, stride=2),
    dict(c_out=32, c_in=16, n=2, h=20, w=21, keep=0.3, stride=2, pad=0),
    dict(c_out=48, c_in=5, n=2, h=18, w=33, keep=1.0, dense=True),
    dict(c_out=19, c_in=19, n=3, h=17, w=9, keep=1.0, depthwise=True, stride=2),
    dict(c_out=37, c_in=37, n=2, h=12, w=16, keep=1.0, depthwise=True),                 # vector loads and stores
    dict(c_out=37, c_in=37, n=2, h=12, w=16, keep=0.7, depthwise=True, stride=2),       # some kernels removed
    dict(c_out=21, c_in=21, n=3, h=9, w=20, keep=1.0, depthwise=True, pad=0),           # vector loads, ragged stores
    dict(c_out=21, c_in=21, n=3, h=11, w=24, keep=1.0, depthwise=True, pad=0, stride=2),
    dict(c_out=64, c_in=64, n=2, h=7, w=7, keep=1.0, depthwise=True),                   # scalar path, tiny planes
    dict(c_out=5, c_in=5, n=1, h=3, w=4, keep=1.0, depthwise=True),
    dict(c_out=33, c_in=33, n=2, h=30, w=130, keep=1.0, depthwise=True, stride=2),      # rows longer than a wavefront
])
def test_ragged_shapes_and_modes(torch, oracle, case):
    rng = np.random.default_rng(sum(int(v) for v in case.values() if not isinstance(v, bool)) + 77)
    d = _random_layer(rng, case["c_out"], case["c_in"], case["keep"], dense=case.get("dense", False),
                      depthwise=case.get("depthwise", False), stride=case.get("stride", 1),
                      pad=case.get("pad", 1))
    x = rng.standard_normal((case["n"], case["c_in"], case["h"], case["w"])).astype(np.float32)
    _say(f"  case {case}")
    _check_layer(torch, oracle, d, x, configs=[None] + _all_configs())
    _check_layer(torch, oracle, d, x, relu=False, use_bias=False, configs=[None])


def test_all_56_patterns_on_every_slot(torch, oracle):
    """The library may be any subset of the 56 centre-keeping patterns (section 4.1): every
    (filter slot, pattern) code block of the tiled kernels runs here."""
    uni = wl.pattern_universe()
    c_out, c_in = 32, 56
    rng = np.random.default_rng(5656)
    spec = wl.LayerSpec(name="all_patterns", c_in=c_in, c_out=c_out, h=0, w=0)
    d = {"spec": spec, "pattern_masks": uni,
         "pattern_ids": ((np.arange(c_in)[None, :] + np.arange(c_out)[:, None]) % 56).astype(np.uint8),
         "kernel_mask": np.ones((c_out, c_in), np.uint8),
         "weights": rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32),
         "bias": rng.standard_normal(c_out).astype(np.float32)}
    x = rng.standard_normal((2, c_in, 14, 17)).astype(np.float32)
    _check_layer(torch, oracle, d, x, configs=[None] + _all_configs())


def test_degenerate_layers(torch, oracle):
    rng = np.random.default_rng(99)
    d = _random_layer(rng, 20, 12, 0.3)
    x = rng.standard_normal((2, 12, 10, 10)).astype(np.float32)
    # a filter without any kernel: output = act(bias)
    d["kernel_mask"][3] = 0
    d["kernel_mask"][17] = 0
    _check_layer(torch, oracle, d, x, configs=[None] + _all_configs())
    # a channel no filter reads
    d["kernel_mask"][:, 5] = 0
    _check_layer(torch, oracle, d, x, configs=[None] + _all_configs())
    # every kernel removed: exactly act(bias), also without bias (exact zeros)
    d["kernel_mask"][:] = 0
    for cfg in [None] + _all_configs():
        L = B.Layer.from_workload(d)
        try:
            if cfg:
                L.set_config(*cfg)
        except B.PatdnnError:
            L.close()
            continue
        got = _gpu_conv(torch, L, x, d["bias"], True)
        want = np.maximum(d["bias"], 0)[None, :, None, None]
        np.testing.assert_array_equal(got, np.broadcast_to(want, got.shape))
        assert not _gpu_conv(torch, L, x, None, False).any()
        L.close()
    # n == 0 is a no-op
    L = B.Layer.from_workload(d)
    out = L.conv2d(torch.empty((0, 12, 10, 10), device="cuda"), None)
    assert tuple(out.shape) == (0, 20, 10, 10)
    # an output that overlaps the input is refused before anything is launched
    both = torch.zeros(2 * 12 * 10 * 10 + 2 * 20 * 10 * 10, device="cuda")
    xin = both[:2 * 12 * 10 * 10].view(2, 12, 10, 10)
    bad_out = both[100:100 + 2 * 20 * 10 * 10].view(2, 20, 10, 10)
    with pytest.raises(B.PatdnnError) as e:
        L.conv2d(xin, None, bad_out)
    assert e.value.status == B.PATDNN_EINVAL
    # so is a workspace that overlaps the input or the output, or is not 16-byte aligned
    good_out = torch.zeros((2, 20, 10, 10), device="cuda")
    spare = torch.zeros(4096, device="cuda")
    for ws in (both[2000:6000], good_out.view(-1)[400:2000], spare[1:1025]):
        with pytest.raises(B.PatdnnError) as e:
            L.conv2d_ws(xin, None, good_out, workspace=ws)
        assert e.value.status == B.PATDNN_EINVAL
    L.conv2d_ws(xin, None, good_out, workspace=spare)         # a fine one, unused by an unsplit layer
    L.close()


def test_decode_reads_back_the_device_layout(torch, oracle):
    d = wl.gen_layer(2, 4, with_input=False)
    L = B.Layer.from_workload(d)
    w, ids, km = L.decode()
    want = oracle.masked_weights(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"])
    assert w.view(np.uint32).tolist() == want.view(np.uint32).tolist()
    np.testing.assert_array_equal(km, d["kernel_mask"])
    np.testing.assert_array_equal(ids, d["pattern_ids"] * d["kernel_mask"])
    L.close()


def test_tune_keeps_a_correct_configuration(torch, oracle):
    d = wl.gen_layer(3, 5)             # 128 -> 128 @ 28
    spec = d["spec"]
    x = np.concatenate([d["input"]] * 4, axis=0)
    x[1:] *= np.float32(0.5)
    L = B.Layer.from_workload(d)
    xt = torch.from_numpy(x).cuda()
    bt = torch.from_numpy(d["bias"]).cuda()
    out = torch.empty(L.output_shape(4, spec.h, spec.w), device="cuda")
    us = L.tune(xt, bt, out)
    cfg = L.get_config()
    _say(f"    tuned: {cfg} {B.patdnn_variant_name(cfg['variant'])} {us:.1f} us")
    assert us > 0 and cfg["variant"] >= 0
    ref = oracle.conv2d(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], x,
                        d["bias"], skip_removed=True)
    # tune leaves a valid result (no ReLU) in the output buffer
    assert _rel_err(out.cpu().numpy(), ref) <= TOL
    got = _gpu_conv(torch, L, x, d["bias"], True)
    assert _rel_err(got, np.maximum(ref, 0)) <= TOL
    L.close()


@pytest.mark.parametrize("layer", list(range(13)))
def test_full_size_sampled(torch, oracle, layer):
    """Configuration 5 (VGG-16 stack, N=64) at full size, in the launch configuration
    the benchmark times (the committed table of tuned configurations): sampled outputs
    against the oracle one by one, plus two whole images."""
    d = wl.gen_layer(5, layer, with_input=False)
    spec = d["spec"]
    _say(f"  config 5 layer {layer} {spec.name}: generating {spec.n} images")
    x = wl.gen_input(spec, 5, layer)
    xt = torch.from_numpy(x).cuda()
    bt = torch.from_numpy(d["bias"]).cuda()
    L = B.Layer.from_workload(d)
    out = torch.empty(L.output_shape(spec.n, spec.h, spec.w), device="cuda")
    # the launch configuration bench.py times: the shape's entry of the committed table of
    # tuned configurations, else whatever the tuner picks now
    table = wl.load_tuned_configs(os.path.join(os.path.dirname(B.LIB_PATH), "tuned_configs.json"))
    c = table.get(wl.shape_key(spec))
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
    if c is not None and c["variant"] in names:
        L.set_config(names[c["variant"]], c["ck"], c["waves"], c["ksplit"])
    else:
        L.tune(xt, bt, out)
    _say(f"    configuration: {L.get_config()} {B.patdnn_variant_name(L.get_config()['variant'])}")
    # as bench.py launches it: with a workspace for the partial sums of a split configuration
    # (NaN beforehand and guarded: nothing may be read before it is written, or written outside)
    need, guard = L.workspace_floats(spec.n, spec.h, spec.w), 4096
    wbuf = torch.full((need + 2 * guard,), float("nan"), dtype=torch.float32, device="cuda")
    wbuf[:guard] = 4242.0
    wbuf[guard + need:] = 4242.0
    L.conv2d_ws(xt, bt, out, workspace=wbuf[guard:guard + need] if need else None, relu=True)
    torch.cuda.synchronize()
    assert bool((wbuf[:guard] == 4242.0).all()) and bool((wbuf[guard + need:] == 4242.0).all())
    got = out.cpu().numpy()
    rng = np.random.default_rng(500 + layer)
    coords = np.stack([rng.integers(0, s, 4096) for s in got.shape], axis=1).astype(np.int32)
    # corners and borders of the first and last image are always in the sample
    for n in (0, spec.n - 1):
        for oh in (0, spec.h_out - 1):
            for ow in (0, spec.w_out - 1):
                coords = np.vstack([coords, [[n, spec.c_out - 1, oh, ow]]]).astype(np.int32)
    ref = oracle.conv2d_points(d["weights"], d["pattern_ids"], d["kernel_mask"],
                               d["pattern_masks"], x, d["bias"], coords, relu=True, dense=spec.dense)
    scale = float(np.abs(ref).max())
    err = float(np.abs(got[tuple(coords.T)].astype(np.float64) - ref).max()) / scale
    _say(f"    sampled rel_err={err:.2e}")
    assert err <= TOL
    for n in (0, spec.n - 1):          # two complete images
        full = oracle.conv2d(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"],
                             x[n:n + 1], d["bias"], relu=True, dense=spec.dense, skip_removed=True)
        assert _rel_err(got[n:n + 1], full) <= TOL
    L.close()
