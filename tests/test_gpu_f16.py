"""GPU parity of the half-precision-storage entry point (binary16 weights, input and
output, fp32 arithmetic; the paper's GPU runs, section 6.1) against the oracle's storage
model.  Bar, derived from the arithmetic: the oracle rounds the exact result once to
binary16; the kernel rounds an fp32 sum that is within 1e-5 of the largest exact output,
so every element must lie within half a binary16 spacing of the exact value plus that
1e-5 (and therefore within one spacing, 2^-10 relative, of the oracle's rounded value)."""

import sys

import numpy as np
import pytest

from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl

pytestmark = pytest.mark.gpu


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.lib()
    return torch


def _check(torch, d, x, relu=True):
    from oracle import fp16
    spec = d["spec"]
    x16 = fp16.to_f16(x)
    want16, exact = fp16.conv2d_f16(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], x16,
                                    d["bias"], stride=spec.stride, pad=spec.pad, relu=relu,
                                    depthwise=spec.depthwise, dense=spec.dense, skip_removed=True)
    L = B.Layer.from_workload(d)
    xt = torch.from_numpy(x16).cuda()
    bt = torch.from_numpy(d["bias"]).cuda()
    guard, numel = 2048, int(np.prod(want16.shape))
    buf = torch.full((numel + 2 * guard,), 7.0, dtype=torch.float16, device="cuda")
    out = buf[guard:guard + numel].view(want16.shape)
    L.conv2d_f16(xt, bt, out, relu=relu)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == 7.0).all()) and bool((buf[guard + numel:] == 7.0).all())
    got = out.cpu().numpy().astype(np.float64)
    scale = float(np.abs(exact).max())
    bound = 2.0 ** -11 * np.maximum(np.abs(exact), 2.0 ** -14) + 1e-5 * scale
    worst = float((np.abs(got - exact) / bound).max())
    rel16 = float(np.abs(got - want16.astype(np.float64)).max() / scale)
    same = float((out.cpu().numpy().view(np.uint16) == want16.view(np.uint16)).mean())
    _say(f"    {spec.name}: worst error {worst:.3f} of the bound; vs the rounded oracle {rel16:.2e} of max; "
         f"{100 * same:.2f} % identical binary16 values")
    assert worst <= 1.0
    assert rel16 <= 2.0 ** -10
    L.close()


def _rand(rng, c_out, c_in, keep, **kw):
    lib = wl.pattern_library(wl.PATTERN_SEED)
    depthwise = kw.get("depthwise", False)
    kpf = 1 if depthwise else c_in
    spec = wl.LayerSpec(name=f"rand_{c_in}x{c_out}_{kw}", c_in=c_in, c_out=c_out, h=0, w=0, **kw)
    return {"spec": spec, "pattern_masks": lib,
            "pattern_ids": rng.integers(0, 8, (c_out, kpf), dtype=np.uint8),
            "kernel_mask": (rng.random((c_out, kpf)) < keep).astype(np.uint8),
            "weights": (rng.standard_normal((c_out, kpf, 3, 3)) * 0.3).astype(np.float32),
            "bias": rng.standard_normal(c_out).astype(np.float32)}


@pytest.mark.parametrize("case", [
    dict(c_out=37, c_in=37, n=2, h=12, w=16, keep=1.0, depthwise=True),
    dict(c_out=37, c_in=37, n=2, h=12, w=16, keep=0.7, depthwise=True, stride=2),
    dict(c_out=21, c_in=21, n=3, h=9, w=20, keep=1.0, depthwise=True, pad=0),
    dict(c_out=64, c_in=64, n=2, h=7, w=7, keep=1.0, depthwise=True),
    dict(c_out=29, c_in=29, n=2, h=9, w=32, keep=0.8, depthwise=True),               # eight outputs per lane
    dict(c_out=29, c_in=29, n=2, h=11, w=48, keep=1.0, depthwise=True, stride=2),    # ... stride 2
    dict(c_out=33, c_in=33, n=2, h=30, w=130, keep=1.0, depthwise=True, stride=2),
    dict(c_out=19, c_in=19, n=3, h=17, w=9, keep=1.0, depthwise=True, stride=2),
    dict(c_out=24, c_in=20, n=3, h=13, w=13, keep=0.3),
    dict(c_out=32, c_in=16, n=2, h=21, w=20, keep=0.3, stride=2),
    dict(c_out=48, c_in=5, n=2, h=18, w=33, keep=1.0, dense=True),
])
def test_f16_storage_matches_the_oracle(torch, case):
    rng = np.random.default_rng(1600 + case["c_out"] + case["h"])
    kw = {k: case[k] for k in ("depthwise", "stride", "pad", "dense") if k in case}
    d = _rand(rng, case["c_out"], case["c_in"], case["keep"], **kw)
    x = rng.standard_normal((case["n"], case["c_in"], case["h"], case["w"])).astype(np.float32)
    _check(torch, d, x)
    _check(torch, d, x, relu=False)


@pytest.mark.parametrize("layer", [0, 1, 3, 6, 13, 16])
def test_f16_on_the_depthwise_workload(torch, layer):
    d = wl.gen_layer(4, layer)
    _check(torch, d, np.concatenate([d["input"], d["input"] * np.float32(0.5)], axis=0))
