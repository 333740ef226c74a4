"""GPU parity of every tiled variant (call and threaded dispatch, 7x2 patches, 7-lane
bands, band-major LDS layout, single staging buffer, stride-2 tiles) and of the split over
input channels (ksplit), on ragged layers, element by element against the oracle.  An
explicitly set configuration is taken as given or refused, never replaced, so each row
printed here is the variant that really ran.  Same bar as the other parity tests."""

import sys

import numpy as np
import pytest

from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl

pytestmark = pytest.mark.gpu
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
    dict(c_out=64, c_in=32, n=2, h=30, w=27, keep=0.3, ck=8, waves=4, stride=2, pad=0),
    dict(c_out=48, c_in=40, n=2, h=19, w=23, keep=0.3, ck=9, waves=3),       # the tuner's odd grid points
    dict(c_out=96, c_in=48, n=1, h=14, w=14, keep=0.3, ck=24, waves=6),
]


@pytest.mark.parametrize("case", CASES)
def test_every_variant_and_ksplit_matches_the_oracle(torch, oracle, case):
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
                    L.set_config(v, case["ck"], case["waves"], ksplit)
                except B.PatdnnError as e:
                    assert e.status == B.PATDNN_EUNSUPPORTED      # wrong stride, dense, ksplit > chunks
                    continue
                assert L.get_config()["variant"] == v
                _say(f"  {case} variant {B.patdnn_variant_name(v)} ksplit={ksplit}")
                buf = torch.full((numel + 2 * guard,), 12345.0, dtype=torch.float32, device="cuda")
                out = buf[guard:guard + numel].view(shape)
                L.conv2d(xt, bt, out, relu=True)      # an accepted explicit configuration must run
                torch.cuda.synchronize()
                assert bool((buf[:guard] == 12345.0).all()) and bool((buf[guard + numel:] == 12345.0).all())
                got = out.cpu().numpy()
                err = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
                _say(f"    rel_err={err:.2e}")
                assert err <= TOL, (B.patdnn_variant_name(v), ksplit, err)
                seen += 1
                need = L.workspace_floats(case["n"], case["h"], case["w"])
                assert (need > 0) == (L.get_config()["ksplit"] > 1)     # the comparison kernels never split
                if need:
                    # the same configuration with one partial-sum buffer per slice: the room is
                    # NaN beforehand and guarded, and two runs must agree bit for bit (no atomics)
                    wbuf = torch.full((need + 2 * guard,), float("nan"), dtype=torch.float32, device="cuda")
                    wbuf[:guard] = 4242.0
                    wbuf[guard + need:] = 4242.0
                    runs = []
                    for _ in range(2):
                        buf.fill_(12345.0)
                        L.conv2d_ws(xt, bt, out, workspace=wbuf[guard:guard + need], relu=True)
                        torch.cuda.synchronize()
                        assert bool((buf[:guard] == 12345.0).all()) and bool((buf[guard + numel:] == 12345.0).all())
                        assert bool((wbuf[:guard] == 4242.0).all()) and bool((wbuf[guard + need:] == 4242.0).all())
                        runs.append(out.clone())
                    assert bool((runs[0] == runs[1]).all()), "slice buffers must give repeatable bits"
                    err = float(np.abs(runs[0].cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max())
                    _say(f"    with a workspace: rel_err={err:.2e}")
                    assert err <= TOL, (B.patdnn_variant_name(v), ksplit, "workspace", err)
                    # a workspace that is too small is not used: the call runs as without one
                    buf.fill_(12345.0)
                    L.conv2d_ws(xt, bt, out, workspace=wbuf[guard:guard + need - 64], relu=True)
                    torch.cuda.synchronize()
                    err = float(np.abs(out.cpu().numpy().astype(np.float64) - ref).max() / np.abs(ref).max())
                    assert err <= TOL, (B.patdnn_variant_name(v), ksplit, "short workspace", err)
    finally:
        L.close()
    assert seen > 0


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_shapes_and_configurations(torch, oracle, seed):
    """Seeded random layers (channels that are no multiple of anything, tiny and ragged images,
    stride 1 and 2, pad 0 and 1, with and without bias and ReLU, sparse to fully connected) in the
    automatic configuration and in a random explicit configuration of every variant that accepts
    the layer: chunk sizes, workgroup sizes and channel slices off the tuner's grid included."""
    lib = wl.pattern_library(wl.PATTERN_SEED)
    runs = 0
    for case in range(8):
        rng = np.random.default_rng(1000 * seed + case)
        c_in = int(rng.choice([3, 5, 8, 16, 24, 33, 64, 96]))
        c_out = int(rng.choice([4, 8, 13, 16, 24, 40, 64, 72, 128]))
        h, w, n = int(rng.integers(5, 40)), int(rng.integers(5, 40)), int(rng.integers(1, 7))
        stride, pad, relu = int(rng.choice([1, 1, 1, 2])), int(rng.choice([0, 1, 1])), bool(rng.integers(0, 2))
        keep = float(rng.choice([0.1, 0.3, 0.6, 1.0]))
        ids = rng.integers(0, 8, (c_out, c_in), dtype=np.uint8)
        mask = (rng.random((c_out, c_in)) < keep).astype(np.uint8)
        wt = rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32)
        bias = rng.standard_normal(c_out).astype(np.float32) if rng.integers(0, 2) else None
        x = rng.standard_normal((n, c_in, h, w)).astype(np.float32)
        ref = oracle.conv2d(wt, ids, mask, lib, x, bias, stride=stride, pad=pad, relu=relu, skip_removed=True)
        scale = max(float(np.abs(ref).max()), 1e-30)
        L = B.Layer(wt, ids, mask, lib, stride=stride, pad=pad)
        xt = torch.from_numpy(x).cuda()
        bt = None if bias is None else torch.from_numpy(bias).cuda()
        shape = L.output_shape(n, h, w)
        numel, guard = int(np.prod(shape)), 2048
        cfgs = [(-1, 0, 0, 1)]
        for v in range(1, B.patdnn_num_variants()):
            cfgs.append((v, int(rng.choice([0, 2, 4, 8, 10, 16])), int(rng.choice([0, 3, 4, 8])),
                         int(rng.choice([1, 1, 2, 3, 5]))))
        try:
            for cfg in cfgs:
                try:
                    L.set_config(*cfg)
                except B.PatdnnError as e:
                    assert e.status in (B.PATDNN_EUNSUPPORTED, B.PATDNN_EINVAL)
                    continue
                _say(f"  seed {seed} case {case}: {c_in}->{c_out} @{h}x{w} n={n} s{stride} p{pad} relu={relu} "
                     f"keep={keep} bias={bias is not None} cfg={cfg}")
                buf = torch.full((numel + 2 * guard,), 4242.0, dtype=torch.float32, device="cuda")
                out = buf[guard:guard + numel].view(shape)
                L.conv2d(xt, bt, out, relu=relu)
                torch.cuda.synchronize()
                assert bool((buf[:guard] == 4242.0).all()) and bool((buf[guard + numel:] == 4242.0).all())
                err = float(np.abs(out.cpu().numpy().astype(np.float64) - ref).max() / scale)
                assert err <= TOL, (seed, case, cfg, err)
                runs += 1
        finally:
            L.close()
    assert runs >= 16


@pytest.mark.parametrize("kpat", [6, 12, 56])
def test_pattern_sets_of_other_sizes(torch, oracle, kpat):
    """Libraries of 6, 12 and all 56 patterns (the paper's study of the pattern count,
    section 6.6) on a 128 -> 128 layer at the paper's density, in the configuration the
    benchmark's sweep uses for that shape and in the library default."""
    import os
    rng = np.random.default_rng(6600 + kpat)
    lib = wl.pattern_library(wl.PATTERN_SEED, kpat)
    c = 128
    ids = rng.integers(0, kpat, (c, c), dtype=np.uint8)
    mask = (rng.random((c, c)) < 1 / 3.6).astype(np.uint8)
    w = (rng.standard_normal((c, c, 3, 3)) * np.sqrt(2 / (9 * c))).astype(np.float32)
    bias = (rng.standard_normal(c) * 0.01).astype(np.float32)
    x = np.maximum(rng.standard_normal((4, c, 56, 56)), 0).astype(np.float32)
    ref = oracle.conv2d(w, ids, mask, lib, x, bias, relu=True, skip_removed=True)
    L = B.Layer(w, ids, mask, lib)
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
    xt, bt = torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda()
    for cfg in (None, ("t_g8_p7x2_s1_x8_thw1b", 8, 4, 1), ("t_g12_p7x1_s1_x16_th", 8, 4, 2)):
        if cfg is not None:
            L.set_config(names[cfg[0]], *cfg[1:])
        got = L.conv2d(xt, bt, relu=True).cpu().numpy()
        err = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
        _say(f"    {kpat} patterns cfg={cfg}: rel_err={err:.2e}")
        assert err <= TOL
    L.close()


def test_layer_pruned_by_the_projection_operators(torch, oracle):
    """Magnitude-driven structure instead of random masks: patterns mined from the weights,
    every kernel projected onto its best pattern, the weakest kernels removed (section 4.1,
    4.2) - encoded and run, against the oracle on the oracle's own projection of the tensor."""
    from oracle import projection as proj
    rng = np.random.default_rng(4242)
    c_out, c_in = 48, 40
    w = (rng.standard_normal((c_out, c_in, 3, 3)) * rng.gamma(2.0, 0.1, (c_out, c_in, 1, 1))).astype(np.float32)
    lib = B.patdnn_mine_patterns(w, 8)
    ids, z = B.patdnn_project_patterns(w, lib)
    mask = B.patdnn_project_connectivity(z, wl.round_half_even(c_out * c_in / 3.6))
    lib_o = proj.mine_pattern_set(w, 8)
    ids_o, z_o = proj.project_patterns(w, lib_o)
    mask_o = proj.project_connectivity(z_o, wl.round_half_even(c_out * c_in / 3.6))
    bias = rng.standard_normal(c_out).astype(np.float32)
    x = rng.standard_normal((2, c_in, 20, 23)).astype(np.float32)
    ref = oracle.conv2d(w, ids_o, mask_o, lib_o, x, bias, relu=True)
    L = B.Layer(w, ids, mask, lib)               # weights outside the patterns are ignored by encode
    got = L.conv2d(torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda(), relu=True).cpu().numpy()
    err = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
    _say(f"    projected layer: rel_err={err:.2e}; filter lengths {L.stats()['min_filter_length']}..{L.stats()['max_filter_length']}")
    assert err <= TOL
    L.close()


@pytest.mark.parametrize("shape", [(12, 16), (9, 11)])     # planes of whole float4s, and not
def test_many_slices_with_a_workspace(torch, oracle, shape):
    """Up to 16 channel slices, each storing to its own buffer: the finishing kernel adds them
    in groups of eight, four and one (every tier of its loop), for planes it reads as float4
    and planes it reads float by float; atomics and buffers must both match the oracle."""
    h, w = shape
    rng = np.random.default_rng(31 + h)
    lib = wl.pattern_library(wl.PATTERN_SEED)
    c_out, c_in, n = 24, 64, 2
    ids = rng.integers(0, 8, (c_out, c_in), dtype=np.uint8)
    mask = (rng.random((c_out, c_in)) < 0.5).astype(np.uint8)
    wt = rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32)
    bias = rng.standard_normal(c_out).astype(np.float32)
    x = rng.standard_normal((n, c_in, h, w)).astype(np.float32)
    ref = oracle.conv2d(wt, ids, mask, lib, x, bias, relu=True, skip_removed=True)
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
    L = B.Layer(wt, ids, mask, lib)
    xt, bt = torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda()
    for vname in ("t_g8_p7x2_s1_x8_thw1b", "t_g8_p7x1_s1_x16_th"):
        for ksplit in (5, 9, 13, 16):
            L.set_config(names[vname], 4, 4, ksplit)
            need = L.workspace_floats(n, h, w)
            ws = torch.full((need,), float("nan"), dtype=torch.float32, device="cuda")
            got = L.conv2d_ws(xt, bt, workspace=ws, relu=True).cpu().numpy()
            plain = L.conv2d(xt, bt, relu=True).cpu().numpy()
            e1 = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
            e2 = float(np.abs(plain.astype(np.float64) - ref).max() / np.abs(ref).max())
            _say(f"    {vname} {h}x{w} ksplit {ksplit}: buffers {e1:.2e} atomics {e2:.2e}")
            assert e1 <= TOL and e2 <= TOL, (vname, ksplit, e1, e2)
    L.close()
