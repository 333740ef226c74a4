"""csrc/kernel_tiled.hip compiled as plain C++ for the host (tests/host_model/): one OS
thread per GPU thread, LDS as a poisoned array, buffer loads with the descriptor's range
check, every LDS / tensor access bounds-checked, the assembly interpreter replaced by a
C++ walk of the same streams.  Every tiled variant - also the ones not yet run on
hardware - computes small ragged layers here and is compared with the oracle, so that
an indexing mistake in a new tile geometry is found on the CPU."""

import ctypes
import os
import shutil
import subprocess
import sys

import numpy as np
import pytest

from conftest import ROOT
from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl

CSRC = os.path.join(ROOT, "paper_2001_00138_amd", "csrc")
sys.path.insert(0, CSRC)
import gen_dispatch  # noqa: E402

TOL = 1e-5


def _model_inc(geos):
    out = []
    for (G, PR, PC, S, TGX, MODE) in geos:
        g = gen_dispatch.geometry(G, PR, PC, S, TGX, MODE)
        out.append(f"""template <> struct StreamLoop<{G}, {PR}, {PC}, {S}, {TGX}, {MODE}> {{
    static constexpr unsigned kBlockBytes = {g['block_bytes']}u, kTableOff = {g['table_off']}u,
                              kCtrlBytes = {g['ctrl_bytes']}u, kRecords = {g['records']}u;
    static void run(float (&acc)[{G}][{g['nacc']}], unsigned lane_lds, const uint32_t* stream, unsigned entry)
    {{
        static const HostmodelGeo g{{{G}, {PR}, {PC}, {S}, {g['WR']}, {g['WC']}, {g['pitch']},
                                    {g['block_bytes']}u, {g['table_off']}u, {g['ctrl_bytes']}u, {g['records']}u,
                                    {g['sets']}, {int(g['threaded'])}}};
        hostmodel_walk(g, &acc[0][0], lane_lds, stream, entry);
    }}
}};
""")
    return "".join(out)


def _build_hostmodel(build, edit=None):
    """Compiles the host model in `build`; `edit(text) -> text` may plant a mistake in the
    copy of kernel_tiled.hip."""
    if not os.path.exists(B.LIB_PATH):
        from paper_2001_00138_amd import buildlib
        buildlib.build()
    from paper_2001_00138_amd import buildlib
    csrc = build / "pkg" / "csrc"
    (csrc / "gen").mkdir(parents=True)
    (build / "include").mkdir()
    for f in ("kernel_tiled.hip", "kernels.hpp", "layout.hpp", "variants.def"):
        shutil.copy(os.path.join(CSRC, f), csrc / f)
    if edit:
        text = (csrc / "kernel_tiled.hip").read_text()
        changed = edit(text)
        assert changed != text, "the planted edit did not apply"
        (csrc / "kernel_tiled.hip").write_text(changed)
    shutil.copy(os.path.join(ROOT, "include", "patdnn.h"), build / "include" / "patdnn.h")
    (csrc / "gen" / "dispatch_all.inc").write_text(_model_inc(buildlib.sparse_geometries()))
    lib = build / "libhostmodel.so"
    cmd = ["g++", "-O1", "-std=c++17", "-pthread", "-fPIC", "-shared", "-Wno-unknown-pragmas", "-Wno-attributes",
           "-I", os.path.join(ROOT, "tests", "host_model"), "-I", str(csrc),
           os.path.join(ROOT, "tests", "host_model", "hostmodel.cpp"), "-o", str(lib)]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-4000:]
    L = ctypes.CDLL(str(lib))
    L.hostmodel_run.restype = ctypes.c_long
    L.hostmodel_run.argtypes = [ctypes.c_int] * 5 + [ctypes.c_void_p] * 4 + [ctypes.c_int] * 10 + \
                               [ctypes.c_void_p] * 3 + [ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t,
                                                        ctypes.c_char_p, ctypes.c_int]
    return L


@pytest.fixture(scope="module")
def hostmodel(tmp_path_factory):
    return _build_hostmodel(tmp_path_factory.mktemp("hostmodel"))


def _run(hostmodel, v, t, x, bias, pad, stride, relu, waves, c_out, w9=None, ksplit=1, slice_buffers=False):
    """slice_buffers: the split launch gets room for one partial-sum buffer per channel slice
    (it then stores instead of adding with atomics); the room is guarded on both sides and starts
    as NaN, so a store outside it or an element that no slice wrote shows."""
    n, c_in, h, w = x.shape
    ho, wo = (h + 2 * pad - 3) // stride + 1, (w + 2 * pad - 3) // stride + 1
    guard = 1024
    buf = np.full(n * c_out * ho * wo + 2 * guard, 777.0, np.float32)
    out = buf[guard:-guard]
    out[:] = np.nan
    msg = ctypes.create_string_buffer(512)
    x = np.ascontiguousarray(x)
    ptr = lambda a: None if a is None else a.ctypes.data
    scratch, scratch_floats, sbuf = None, 0, None
    if slice_buffers:
        scratch_floats = ksplit * (-(-(n * c_out * ho * wo) // 64) * 64)
        sbuf = np.full(scratch_floats + 2 * guard, 555.0, np.float32)
        # 16-byte aligned start of the room, as the launcher demands
        skip = guard + (-(sbuf.ctypes.data + 4 * guard) % 16) // 4
        sbuf[skip:skip + scratch_floats] = np.nan
        scratch = sbuf.ctypes.data + 4 * skip
    errs = hostmodel.hostmodel_run(v - 1, t["G"], t["num_groups"], t["ck"], t["num_chunks"],
                                   ptr(t["slot_channel"]), ptr(t.get("chunk_ptr")), ptr(t.get("steps")), ptr(w9),
                                   n, c_in, c_out, h, w, ho, wo, stride, pad, int(relu), ptr(x), ptr(bias),
                                   out.ctypes.data, waves, ksplit, scratch, scratch_floats, msg, 512)
    assert errs == 0, msg.value.decode()
    assert (buf[:guard] == 777.0).all() and (buf[-guard:] == 777.0).all(), "write outside the output tensor"
    if sbuf is not None:
        assert (sbuf[:skip] == 555.0).all() and (sbuf[skip + scratch_floats:] == 555.0).all(), \
            "write outside the partial-sum buffers"
    return out.reshape(n, c_out, ho, wo)


CASES = [
    dict(c_out=24, c_in=20, n=2, h=13, w=13, keep=0.3, ck=3, waves=2, pad=1),
    dict(c_out=40, c_in=9, n=3, h=8, w=21, keep=0.25, ck=16, waves=4, pad=1),
    dict(c_out=16, c_in=6, n=1, h=30, w=37, keep=0.6, ck=4, waves=3, pad=0),
    dict(c_out=20, c_in=12, n=2, h=15, w=18, keep=0.35, ck=5, waves=2, pad=1, stride=2),
    dict(c_out=9, c_in=6, n=1, h=20, w=9, keep=0.5, ck=2, waves=4, pad=0, stride=2),
    dict(c_out=24, c_in=10, n=2, h=12, w=22, keep=0.4, ck=4, waves=4, pad=1),     # even rows: paired stores
]


@pytest.mark.parametrize("case", CASES)
def test_every_sparse_variant_on_the_host_model(hostmodel, oracle, case):
    rng = np.random.default_rng(4321 + case["c_out"] + case["h"])
    lib = wl.pattern_library(wl.PATTERN_SEED)
    stride = case.get("stride", 1)
    ids = rng.integers(0, 8, (case["c_out"], case["c_in"]), dtype=np.uint8)
    mask = (rng.random((case["c_out"], case["c_in"])) < case["keep"]).astype(np.uint8)
    w = rng.standard_normal((case["c_out"], case["c_in"], 3, 3)).astype(np.float32)
    bias = rng.standard_normal(case["c_out"]).astype(np.float32)
    x = rng.standard_normal((case["n"], case["c_in"], case["h"], case["w"])).astype(np.float32)
    ref = oracle.conv2d(w, ids, mask, lib, x, bias, stride=stride, pad=case["pad"], relu=True)
    L = B.Layer(w, ids, mask, lib, stride=stride, pad=case["pad"], host_only=True)
    seen = 0
    for v in range(1, B.patdnn_num_variants()):
        try:
            t = L.export_tiled(v, case["ck"])
        except B.PatdnnError as e:
            assert e.status == B.PATDNN_EUNSUPPORTED
            continue
        lds_per_channel = hostmodel.hostmodel_variant_lds_floats(v - 1)
        min_waves = -(-lds_per_channel // (64 * hostmodel.hostmodel_variant_max_slots(v - 1)))   # staging slots
        ks = min(3, t["num_chunks"])
        for ksplit, slice_buffers in ((1, False), (ks, False), (ks, True)):
            if slice_buffers and ksplit == 1:
                continue
            got = _run(hostmodel, v, t, x, bias, case["pad"], stride, True, max(case["waves"], min_waves, 3),
                       case["c_out"], ksplit=ksplit, slice_buffers=slice_buffers)
            assert not np.isnan(got).any(), (B.patdnn_variant_name(v), "output element never written or unstaged LDS read")
            err = float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max())
            print(f"  {B.patdnn_variant_name(v)} ksplit={ksplit} buffers={slice_buffers}: rel_err={err:.2e}")
            assert err <= TOL, (B.patdnn_variant_name(v), ksplit, slice_buffers, err)
        seen += 1
    L.close()
    assert seen >= 2


def test_division_by_launch_constants(hostmodel):
    """The multiply-and-shift that replaces the kernel's divisions by the bands per row and
    column: exact for every dividend below 2^31, checked at the edges of each quotient step
    and on random values, for small, large, power-of-two and odd divisors."""
    f = hostmodel.hostmodel_fast_div
    f.restype, f.argtypes = ctypes.c_uint, [ctypes.c_uint, ctypes.c_uint]
    rng = np.random.default_rng(5)
    top = 2 ** 31 - 1
    divisors = [1, 2, 3, 4, 5, 7, 8, 9, 14, 16, 28, 32, 33, 100, 255, 256, 257, 1000, 65535, 65536, 65537,
                10 ** 6, 2 ** 30 - 1, 2 ** 30, 2 ** 30 + 1, top] + [int(v) for v in rng.integers(1, top, 40)]
    for d in divisors:
        ns = {0, 1, d - 1, d, d + 1, top, top - 1, top - d if top > d else 0}
        for q in [int(v) for v in rng.integers(0, top // d + 1, 30)] + [top // d]:
            ns.update({q * d - 1, q * d, q * d + d - 1})
        ns.update(int(v) for v in rng.integers(0, top, 200))
        for n in ns:
            if 0 <= n <= top:
                assert f(n, d) == n // d, (n, d)


@pytest.mark.parametrize("plant", ["staging column", "epilogue guard", "lane offset"])
def test_host_model_catches_planted_mistakes(tmp_path, oracle, plant):
    edits = {
        "staging column": lambda t: t.replace("const int ix = bxi * TGX * PC * S - a.pad + x;",
                                              "const int ix = bxi * TGX * PC * S - a.pad + x + 1;"),
        "epilogue guard": lambda t: t.replace("if (oy < a.ho && ox < a.wo) dst", "if (ox < a.wo) dst"),
        "lane offset": lambda t: t.replace("+ gx * PC * S : 0;", "+ gx * PC * S + GEO::ROWP * 3 : 0;"),
    }
    broken = _build_hostmodel(tmp_path, edits[plant])
    with pytest.raises(AssertionError):
        test_every_sparse_variant_on_the_host_model(broken, oracle, CASES[0])


@pytest.mark.parametrize("ck,waves", [(6, 3), (9, 6), (12, 3), (24, 6), (1, 2), (28, 8)])
def test_default_variant_over_the_tuner_grid(hostmodel, oracle, ck, waves):
    """The launch parameters the tuner tries beyond the ones the GPU tests name: chunk sizes
    that do not divide c_in, three and six wavefronts, more wavefronts than filter groups."""
    rng = np.random.default_rng(77)
    lib = wl.pattern_library(wl.PATTERN_SEED)
    c_out, c_in = 64, 40
    ids = rng.integers(0, 8, (c_out, c_in), dtype=np.uint8)
    mask = (rng.random((c_out, c_in)) < 0.28).astype(np.uint8)
    w = rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32)
    bias = rng.standard_normal(c_out).astype(np.float32)
    x = rng.standard_normal((2, c_in, 21, 30)).astype(np.float32)
    ref = oracle.conv2d(w, ids, mask, lib, x, bias, stride=1, pad=1, relu=True)
    L = B.Layer(w, ids, mask, lib, host_only=True)
    names = {B.patdnn_variant_name(v): v for v in range(1, B.patdnn_num_variants())}
    for v in (names["t_g16_p7x1_s1_x16"], names["t_g8_p7x2_s1_x8_thw1b"]):   # call and threaded dispatch
        t = L.export_tiled(v, ck)
        min_waves = -(-hostmodel.hostmodel_variant_lds_floats(v - 1) // (64 * hostmodel.hostmodel_variant_max_slots(v - 1)))
        got = _run(hostmodel, v, t, x, bias, 1, 1, True, max(waves, min_waves), c_out)
        assert not np.isnan(got).any()
        assert float(np.abs(got.astype(np.float64) - ref).max() / np.abs(ref).max()) <= TOL
    L.close()
