"""The generated step interpreter (csrc/gen_dispatch.py) executed on a functional model
of a wavefront (tests/gcn_model.py) against the encoder's step streams, for every sparse
tiled variant - including the ones not yet run on hardware.  The surrounding kernel is
modelled from its specification: band / patch geometry, the LDS layout of a staged
chunk (halo and zero fill), the lane's LDS address, the epilogue.  Outputs are compared
with the CPU oracle element by element (paper sections 2.1, 5.2-5.4)."""

import os
import sys

import numpy as np
import pytest

from conftest import ROOT
from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl

sys.path.insert(0, os.path.join(ROOT, "paper_2001_00138_amd", "csrc"))
import gen_dispatch  # noqa: E402
import gcn_model  # noqa: E402

TOL = 1e-5
_programs = {}


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(B.LIB_PATH):
        from paper_2001_00138_amd import buildlib
        buildlib.build()


def _program(t):
    key = (t["G"], t["patch_rows"], t["patch_cols"], t["conv_stride"], t["lanes_x"],
           t["mode"] & 15)               # bit 4 (one staging buffer) is the kernel's, not the interpreter's
    if key not in _programs:
        lines, geo = gen_dispatch.program(*key)
        assert geo["block_bytes"] == t["block_bytes"] and geo["table_off"] == t["table_off"]
        assert geo["ctrl_bytes"] == t["ctrl_bytes"] and geo["records"] == t["records"]
        # odd keys are laid out just below a 4 GiB boundary, so that the table straddles it and
        # the carry of every computed code address is exercised
        base = gcn_model.CODE_BASE if len(_programs) % 2 == 0 else 0x7F00_FFFF_0000
        _programs[key] = (gcn_model.Program(lines, base), geo)
    return _programs[key]


def _model_conv(t, x, bias, pad, relu, stats):
    """The tiled kernel around the interpreter, modelled: returns the output tensor."""
    prog, geo = _program(t)
    G, PR, PC, S, TGX = t["G"], t["patch_rows"], t["patch_cols"], t["conv_stride"], t["lanes_x"]
    NB, WR, WC = 64 // TGX, geo["WR"], geo["WC"]
    PITCH = (TGX * PC - 1) * S + 3
    assert geo["band_cols"] == PITCH
    RSTRIDE, BSTRIDE = geo["pitch"], geo["band_stride"]      # between window rows / between bands
    TILEP = t["lds_channel_bytes"] // 4
    assert TILEP >= (WR - 1) * RSTRIDE + (NB - 1) * BSTRIDE + PITCH and TILEP % 64 == 0
    n, c_in, h, w = x.shape
    ho, wo = (h + 2 * pad - 3) // S + 1, (w + 2 * pad - 3) // S + 1
    c_out = int(t["slot_channel"].max()) + 1
    out = np.full((n, c_out, ho, wo), np.nan, np.float32)
    bx, by = -(-wo // (TGX * PC)), -(-ho // PR)
    num_bands = n * bx * by
    ck = t["ck"]
    lds = np.zeros(2 * ck * TILEP, np.uint32)
    lane = np.arange(64)
    lb, gx = lane // TGX, lane % TGX
    lane_ok = lb < NB                      # TGX = 7: the 64th lane has no band
    lane_off = np.where(lane_ok, lb * BSTRIDE + gx * PC * S, 0)
    for tile in range(-(-num_bands // NB)):
        band0 = tile * NB
        for g in range(t["num_groups"]):
            acc = np.zeros((G, PR * PC, 64), np.float32)
            for chunk in range(t["num_chunks"]):
                c0 = chunk * ck
                cn = min(ck, c_in - c0)
                cur = 0 if t["mode"] & 16 else (chunk & 1) * ck * TILEP
                # the staged chunk: [channel][window row][band][column], zero outside the image
                lds[cur:cur + ck * TILEP] = 0xFFC00000           # NaN pattern where nothing is staged
                for c in range(cn):
                    ch = np.zeros((WR, NB, PITCH), np.float32)
                    img_of = np.full(TILEP, 0xFFC00000, np.uint32)   # the channel as it lies in LDS
                    for b in range(NB):
                        band = band0 + b
                        if band >= num_bands:
                            continue
                        bxi, byi, img = band % bx, (band // bx) % by, band // (bx * by)
                        for q in range(WR):
                            iy = byi * PR * S - pad + q
                            if not 0 <= iy < h:
                                continue
                            ix = bxi * TGX * PC * S - pad + np.arange(PITCH)
                            ok = (ix >= 0) & (ix < w)
                            ch[q, b, ok] = x[img, c0 + c, iy, ix[ok]]
                    for q in range(WR):
                        for b in range(NB):
                            o = q * RSTRIDE + b * BSTRIDE
                            img_of[o:o + PITCH] = ch[q, b].view(np.uint32)
                    at = cur + c * TILEP
                    lds[at:at + TILEP] = img_of
                cp = int(t["chunk_ptr"][g, chunk])
                wave = gcn_model.Wave(prog, t["steps"], lds)
                for s in range(G):
                    for i in range(PR * PC):
                        wave.v[f"a{s}_{i}"] = acc[s, i].view(np.uint32).copy()
                wave.v["lane"] = (4 * (cur + lane_off)).astype(np.uint32)
                wave.sop["sp"] = gcn_model.STREAM_BASE + 4 * 24 * (cp & 0x0FFFFFFF)
                wave.sop["entry"] = (cp >> 28) * t["ctrl_bytes"]
                wave.m0 = 0x12345
                wave.run()
                assert wave.m0 == 0x12345                     # M0 is handed back unchanged
                stats["instructions"] += wave.executed
                stats["jumps"] += wave.jumps
                for s in range(G):
                    for i in range(PR * PC):
                        acc[s, i] = wave.v[f"a{s}_{i}"].view(np.float32)
            # epilogue
            for ln in range(64):
                band = band0 + lb[ln]
                if not lane_ok[ln] or band >= num_bands:
                    continue
                bxi, byi, img = band % bx, (band // bx) % by, band // (bx * by)
                for s in range(G):
                    co = int(t["slot_channel"][g, s])
                    if co < 0:
                        continue
                    for r in range(PR):
                        for c in range(PC):
                            oy, ox = byi * PR + r, (bxi * TGX + gx[ln]) * PC + c
                            if oy < ho and ox < wo:
                                v = acc[s, r * PC + c, ln] + (bias[co] if bias is not None else np.float32(0))
                                out[img, co, oy, ox] = max(v, np.float32(0)) if relu else v
    return out


def _check(oracle, d, x, ck, pad=1, stride=1, only=None):
    ref = oracle.conv2d(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], x,
                        d["bias"], stride=stride, pad=pad, relu=True)
    L = B.Layer(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], pad=pad,
                stride=stride, host_only=True)
    seen = []
    for v in range(1, B.patdnn_num_variants()):
        if only is not None and B.patdnn_variant_name(v) not in only:
            continue
        try:
            t = L.export_tiled(v, ck)
        except B.PatdnnError as e:
            assert e.status == B.PATDNN_EUNSUPPORTED
            continue
        assert t["conv_stride"] == stride
        stats = {"instructions": 0, "jumps": 0}
        got = _model_conv(t, x, d["bias"], pad, True, stats)
        assert got.shape == ref.shape
        assert not np.isnan(got).any(), "an output element was never written"
        err = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
        kept = int(d["kernel_mask"].sum())
        print(f"  {B.patdnn_variant_name(v)} ck={t['ck']}: rel_err={err:.2e} "
              f"jumps per kernel-tile={stats['jumps'] / max(1, kept):.2f}")
        assert err <= TOL, (B.patdnn_variant_name(v), err)
        seen.append(B.patdnn_variant_name(v))
    L.close()
    return seen


def test_model_runs_config1_layer(oracle):
    d = wl.gen_layer(1, 0)
    seen = _check(oracle, d, d["input"], 8)
    assert len(seen) >= 7


@pytest.mark.parametrize("case", [
    dict(c_out=24, c_in=20, n=2, h=13, w=13, keep=0.3, ck=3, pad=1),     # ragged everywhere
    dict(c_out=10, c_in=5, n=1, h=9, w=20, keep=1.0, ck=16, pad=0),      # every kernel kept: full steps
    dict(c_out=40, c_in=9, n=3, h=8, w=5, keep=0.1, ck=4, pad=1),        # mostly empty chunks
    dict(c_out=20, c_in=12, n=2, h=15, w=18, keep=0.35, ck=5, pad=1, stride=2),
    dict(c_out=9, c_in=6, n=1, h=20, w=9, keep=0.5, ck=2, pad=0, stride=2),
])
def test_model_runs_ragged_layers(oracle, case):
    rng = np.random.default_rng(1234 + case["c_out"])
    lib = wl.pattern_library(wl.PATTERN_SEED)
    d = {"pattern_masks": lib,
         "pattern_ids": rng.integers(0, 8, (case["c_out"], case["c_in"]), dtype=np.uint8),
         "kernel_mask": (rng.random((case["c_out"], case["c_in"])) < case["keep"]).astype(np.uint8),
         "weights": rng.standard_normal((case["c_out"], case["c_in"], 3, 3)).astype(np.float32),
         "bias": rng.standard_normal(case["c_out"]).astype(np.float32)}
    x = rng.standard_normal((case["n"], case["c_in"], case["h"], case["w"])).astype(np.float32)
    stride = case.get("stride", 1)
    seen = _check(oracle, d, x, case["ck"], pad=case["pad"], stride=stride)
    assert len(seen) >= (7 if stride == 1 else 2)


def test_model_runs_long_streams(oracle):
    """A 128 -> 128 layer at the paper's density (hundreds of steps per group, sixteen
    chunks, both register-set parities many times over) on one variant of every
    interpreter mode."""
    d = wl.gen_layer(3, 4, with_input=False)           # 128 -> 128
    x = wl.gen_input(d["spec"], 3, 4, 1)[:, :, :7, :14]
    seen = _check(oracle, d, x, 8, only={
        "t_g16_p7x1_s1_x16", "t_g12_p7x1_s1_x16_th", "t_g8_p7x2_s1_x8_thw1b", "t_g16_p7x1_s1_x7_th",
        "t_g16_p7x1_s1_x16_thwb"})
    assert len(seen) == 5


def test_model_runs_every_block_of_the_table(oracle):
    """All 56 centre-keeping patterns on every filter slot: each (slot, pattern) code block of
    the table is executed at least once (section 4.1: the library may be any subset)."""
    uni = wl.pattern_universe()
    c_out, c_in = 16, 56
    rng = np.random.default_rng(56)
    d = {"pattern_masks": uni,
         "pattern_ids": ((np.arange(c_in)[None, :] + np.arange(c_out)[:, None]) % 56).astype(np.uint8),
         "kernel_mask": np.ones((c_out, c_in), np.uint8),
         "weights": rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32),
         "bias": rng.standard_normal(c_out).astype(np.float32)}
    x = rng.standard_normal((1, c_in, 7, 9)).astype(np.float32)
    seen = _check(oracle, d, x, 14, only={
        "t_g16_p7x1_s1_x16", "t_g16_p7x1_s1_x16_thwb", "t_g8_p7x2_s1_x8_thw1b", "t_g12_p7x1_s1_x16_th"})
    assert len(seen) == 4


def test_model_catches_planted_mistakes(oracle):
    """The model has teeth: a wait taken out of the program, or a corrupted code offset
    in the stream, fails instead of passing by luck."""
    d = wl.gen_layer(1, 0)
    L = B.Layer.from_workload(d, host_only=True)
    t = L.export_tiled(1, 8)                       # call dispatch, one window set
    L.close()
    key = (t["G"], t["patch_rows"], t["patch_cols"], t["conv_stride"], t["lanes_x"], t["mode"])
    assert t["mode"] == 0
    lines, _ = gen_dispatch.program(*key)
    stats = {"instructions": 0, "jumps": 0}
    # 1. the wait that ends the window load is removed
    waits = [i for i, l in enumerate(lines) if l.startswith("s_waitcnt")]
    broken = [l for i, l in enumerate(lines) if i != waits[2]]       # inside the first window block
    _programs[key] = (gcn_model.Program(broken), _program(t)[1])
    with pytest.raises(gcn_model.ModelError):
        _model_conv(t, d["input"], d["bias"], 1, True, stats)
    del _programs[key]
    # 2. a code offset that is not a block start
    t2 = dict(t)
    t2["steps"] = t["steps"].copy()
    first = int(t["chunk_ptr"][0, 0]) & 0x0FFFFFFF
    t2["steps"][first, 16] += 4
    with pytest.raises(gcn_model.ModelError):
        _model_conv(t2, d["input"], d["bias"], 1, True, stats)
