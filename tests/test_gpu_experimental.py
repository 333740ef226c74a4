"""GPU parity of the variants and launch options that are still experimental (threaded
dispatch, 7x2 patches, 7-lane bands, stride-2 tiles, input-channel slices).  They have
passed the host models (tests/test_interpreter_model.py, tests/test_host_model.py) but
not yet a hardware run, so the library only runs them with PATDNN_EXPERIMENTAL=1 in the
environment; without it this module is skipped.  Same bar as the other parity tests."""

import os
import sys

import numpy as np
import pytest

from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl

pytestmark = [pytest.mark.gpu,
              pytest.mark.skipif(os.environ.get("PATDNN_EXPERIMENTAL") != "1",
                                 reason="experimental variants run only with PATDNN_EXPERIMENTAL=1")]
TOL = 1e-5


@pytest.fixture(scope="module")
def torch():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    B.lib()
    return torch


def _say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


CASES = [
    dict(c_out=16, c_in=16, n=1, h=32, w=32, keep=0.5, ck=8, waves=4),
    dict(c_out=24, c_in=20, n=3, h=13, w=13, keep=0.3, ck=3, waves=2),
    dict(c_out=70, c_in=64, n=2, h=28, w=28, keep=0.28, ck=16, waves=4),
    dict(c_out=40, c_in=7, n=2, h=29, w=17, keep=0.5, ck=4, waves=8, pad=0),
    dict(c_out=32, c_in=16, n=2, h=21, w=20, keep=0.3, ck=8, waves=4, stride=2),
    dict(c_out=128, c_in=128, n=4, h=56, w=56, keep=0.278, ck=8, waves=4),
]


@pytest.mark.parametrize("case", CASES)
def test_experimental_variants_match_the_oracle(torch, oracle, case):
    rng = np.random.default_rng(9000 + case["c_out"] + case["h"])
    lib = wl.pattern_library(wl.PATTERN_SEED)
    stride, pad = case.get("stride", 1), case.get("pad", 1)
    ids = rng.integers(0, 8, (case["c_out"], case["c_in"]), dtype=np.uint8)
    mask = (rng.random((case["c_out"], case["c_in"])) < case["keep"]).astype(np.uint8)
    w = rng.standard_normal((case["c_out"], case["c_in"], 3, 3)).astype(np.float32)
    bias = rng.standard_normal(case["c_out"]).astype(np.float32)
    x = rng.standard_normal((case["n"], case["c_in"], case["h"], case["w"])).astype(np.float32)
    ref = oracle.conv2d(w, ids, mask, lib, x, bias, stride=stride, pad=pad, relu=True, skip_removed=True)
    L = B.Layer(w, ids, mask, lib, stride=stride, pad=pad)
    xt, bt = torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda()
    shape = L.output_shape(*x.shape[:1], x.shape[2], x.shape[3])
    numel, guard = int(np.prod(shape)), 4096
    seen = 0
    try:
        for v in range(1, B.patdnn_num_variants()):
            for ksplit in (1, 2, 3):
                try:
                    info = B.patdnn_tiled_info(L.handle, v, case["ck"])
                    if not info["experimental"] and ksplit == 1:
                        continue                      # covered by test_gpu_parity.py
                    L.set_config(v, case["ck"], case["waves"], ksplit)
                except B.PatdnnError as e:
                    assert e.status == B.PATDNN_EUNSUPPORTED
                    continue
                _say(f"  {case} variant {B.patdnn_variant_name(v)} ksplit={ksplit}")
                buf = torch.full((numel + 2 * guard,), 12345.0, dtype=torch.float32, device="cuda")
                out = buf[guard:guard + numel].view(shape)
                try:
                    L.conv2d(xt, bt, out, relu=True)
                except B.PatdnnError as e:
                    assert e.status == B.PATDNN_EUNSUPPORTED    # e.g. ksplit beyond the chunk count
                    continue
                torch.cuda.synchronize()
                assert bool((buf[:guard] == 12345.0).all()) and bool((buf[guard + numel:] == 12345.0).all())
                got = out.cpu().numpy()
                err = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
                _say(f"    rel_err={err:.2e}")
                assert err <= TOL, (B.patdnn_variant_name(v), ksplit, err)
                seen += 1
    finally:
        L.close()
    assert seen > 0
