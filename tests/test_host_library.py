"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every
symbol the header declares, and its offline stage (filter-kernel reorder + FKW
storage, paper section 5.2 / 5.3) round-trips exactly.  Handles are encoded with
PATDNN_HOST_ONLY, so no HIP call is made."""

import os
import re

import numpy as np
import pytest

from conftest import ROOT, read_golden_kv
from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl


@pytest.fixture(scope="module", autouse=True)
def _built():
    if not os.path.exists(B.LIB_PATH):
        from paper_2001_00138_amd import buildlib
        buildlib.build()


def _header_functions(header="patdnn.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(patdnn_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _header_functions()
    assert len(names) >= 12
    L = B.lib()
    for n in names:
        assert hasattr(L, n), f"{n} declared in patdnn.h but not exported"
    assert sorted(B.EXPORTS) == names
    assert B.patdnn_num_variants() >= 2
    assert B.patdnn_variant_name(0) == "fkw"
    assert B.patdnn_variant_name(B.patdnn_num_variants()) is None


def test_probe_library_exports_every_declared_symbol():
    """The bench-side probes live in a library of their own with a header of their own."""
    import ctypes
    from paper_2001_00138_amd import buildlib
    names = _header_functions("patdnn_probes.h")
    assert names == ["patdnn_probe_copy", "patdnn_probe_fma"]
    L = ctypes.CDLL(buildlib.PROBES_LIB)
    for n in names:
        assert hasattr(L, n), f"{n} declared in patdnn_probes.h but not exported"


def _host_layer(layer, **kw):
    return B.Layer.from_workload(layer, host_only=True, **kw)


@pytest.mark.parametrize("config,layer", [(1, 0), (2, 0), (2, 1), (2, 7), (3, 3), (4, 1), (4, 16)])
def test_encode_decode_roundtrip(oracle, config, layer):
    d = wl.gen_layer(config, layer, with_input=False)
    spec = d["spec"]
    L = _host_layer(d)
    w, ids, km = L.decode()
    want_w = oracle.masked_weights(d["weights"], d["pattern_ids"], d["kernel_mask"],
                                   d["pattern_masks"], dense=spec.dense)
    assert w.view(np.uint32).tolist() == want_w.view(np.uint32).tolist()   # exact bits
    if spec.dense:
        assert km.all() and not ids.any()
    else:
        np.testing.assert_array_equal(km, d["kernel_mask"])
        np.testing.assert_array_equal(ids, d["pattern_ids"] * d["kernel_mask"])
    st = L.stats()
    assert st["kept_kernels"] == int(km.sum()) == wl.kept_kernel_count(spec)
    assert st["taps"] == (9 if spec.dense else 4)
    assert st["fkw_weight_bytes"] == 4 * st["taps"] * st["kept_kernels"]
    L.close()


def test_fkw_arrays_follow_the_paper(oracle):
    """The exported arrays obey section 5.3, and coincide with the oracle's own
    construction (same stated reading of the tie-breaks)."""
    from oracle import fkw
    d = wl.gen_layer(3, 0, with_input=False)            # 64 -> 64
    L = _host_layer(d)
    f = L.export_fkw()
    ref = fkw.build_fkw(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"])
    c_out = d["spec"].c_out
    lengths = np.diff(f["offset"])
    assert (np.diff(lengths) >= 0).all()                        # grouped by length
    assert sorted(f["reorder"]) == list(range(c_out))           # a permutation
    for s, co in enumerate(f["reorder"]):
        ch = f["index"][f["offset"][s]:f["offset"][s + 1]]
        assert sorted(ch) == list(np.flatnonzero(d["kernel_mask"][co]))
        assert (np.diff(d["pattern_ids"][co, ch].astype(int)) >= 0).all()   # grouped by pattern
        assert f["stride"][s, 0] == 0 and f["stride"][s, -1] == len(ch)
    np.testing.assert_array_equal(f["offset"], ref.offset)
    np.testing.assert_array_equal(f["reorder"], ref.reorder)
    np.testing.assert_array_equal(f["index"], ref.index)
    np.testing.assert_array_equal(f["stride"], ref.stride)
    assert f["weight"].view(np.uint32).tolist() == ref.weight.view(np.uint32).tolist()
    # the exported arrays, walked as the paper describes, compute the layer
    x = wl.gen_input(d["spec"], 3, 0, 1)[:, :, :12, :12]
    got = fkw.fkw_conv2d(fkw.FKW(f["offset"], f["reorder"], f["index"], f["stride"], f["weight"],
                                 d["pattern_masks"]), x, d["bias"], relu=True)
    want = oracle.conv2d(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"], x,
                         d["bias"], relu=True)
    np.testing.assert_allclose(got, want, atol=1e-12)
    L.close()


def test_worked_example_through_the_library():
    g = read_golden_kv("fkw_worked_example.txt")
    ids = np.zeros((4, 4), np.uint8)
    mask = np.zeros((4, 4), np.uint8)
    mask[0, [1, 3]] = 1; ids[0, 3] = 0; ids[0, 1] = 1
    mask[1, [0, 2]] = 1; ids[1, 0] = 1; ids[1, 2] = 0
    mask[2, [0, 1, 2]] = 1; ids[2, 0] = 0; ids[2, 1] = 1; ids[2, 2] = 0
    mask[3, [2, 3]] = 1; ids[3, 2] = 0; ids[3, 3] = 0
    lib = wl.pattern_universe()[[3, 40]]
    w = np.random.default_rng(0).standard_normal((4, 4, 3, 3)).astype(np.float32)
    L = B.Layer(w, ids, mask, lib, host_only=True)
    f = L.export_fkw()
    assert [str(v) for v in np.diff(f["offset"])] == g["filter_lengths_after_reorder"]
    assert [str(v) for v in f["offset"][:4]] == g["offset"]
    assert [str(v) for v in f["index"][:2]] == g["filter0_index"]
    assert [str(v) for v in f["stride"][0]] == g["filter0_stride"]
    a, b = (int(v) for v in g["swapped_filters"])
    assert f["reorder"][a] == b and f["reorder"][b] == a
    assert [str(4 * v) for v in np.diff(f["offset"])] == g["weights_per_filter"]
    L.close()


def test_degenerate_layers_roundtrip(oracle):
    rng = np.random.default_rng(5)
    lib = wl.pattern_library(3)
    w = rng.standard_normal((5, 7, 3, 3)).astype(np.float32)
    ids = rng.integers(0, 8, (5, 7), dtype=np.uint8)
    for mask in (np.zeros((5, 7), np.uint8), np.ones((5, 7), np.uint8),
                 np.eye(5, 7, dtype=np.uint8)):
        L = B.Layer(w, ids, mask, lib, host_only=True)
        dw, dids, dm = L.decode()
        np.testing.assert_array_equal(dm, mask)
        np.testing.assert_array_equal(dw, oracle.masked_weights(w, ids, mask, lib))
        assert L.stats()["kept_kernels"] == mask.sum()
        L.close()
    # kernel_mask == NULL means every kernel kept
    L = B.Layer(w, ids, None, lib, host_only=True)
    assert L.decode()[2].all()
    L.close()
    # the id of a removed kernel is not read
    ids2 = ids.copy(); ids2[1, 1] = 250
    m = np.ones((5, 7), np.uint8); m[1, 1] = 0
    B.Layer(w, ids2, m, lib, host_only=True).close()


def test_error_reporting():
    rng = np.random.default_rng(6)
    lib = wl.pattern_library(3)
    w = rng.standard_normal((4, 4, 3, 3)).astype(np.float32)
    ids = rng.integers(0, 8, (4, 4), dtype=np.uint8)

    def status(**kw):
        args = dict(dense_weights=w, pattern_ids=ids, kernel_mask=None, pattern_masks=lib,
                    flags=B.PATDNN_HOST_ONLY)
        args.update(kw)
        with pytest.raises(B.PatdnnError) as e:
            B.patdnn_encode(**args)
        return e.value.status

    assert status(stride=3) == B.PATDNN_EINVAL
    assert status(pad=2) == B.PATDNN_EINVAL
    assert status(groups=2) == B.PATDNN_EINVAL
    bad = lib.copy(); bad[2] = 0b111110000          # five positions
    assert status(pattern_masks=bad) == B.PATDNN_EPATTERN
    ids2 = ids.copy(); ids2[0, 0] = 8
    assert status(pattern_ids=ids2) == B.PATDNN_EPATTERN
    assert status(flags=B.PATDNN_HOST_ONLY | B.PATDNN_STRICT) == B.PATDNN_EPATTERN
    # STRICT accepts a tensor that already obeys the constraints
    from oracle import ref
    h = B.patdnn_encode(ref.masked_weights(w, ids, None, lib), ids, None, lib,
                        flags=B.PATDNN_HOST_ONLY | B.PATDNN_STRICT)
    # a host-only handle cannot run
    L = B.lib()
    assert L.patdnn_conv2d(h, 1, 1, 8, 8, None, 1, 0, None) == B.PATDNN_EHIP
    assert b"HOST_ONLY" in L.patdnn_last_error()
    assert B.patdnn_output_shape(h, 2, 9, 10) == (2, 4, 9, 10)
    with pytest.raises(B.PatdnnError):
        B.patdnn_output_shape(h, 1, 0, 5)
    B.patdnn_destroy(h)
    B.patdnn_destroy(None)
    assert L.patdnn_status_string(B.PATDNN_EPATTERN) == b"pattern constraint violated"


def test_filter_groups_balance_after_reorder():
    """Grouping filters by length (section 5.2) leaves the filter groups of the tiled
    layout with nearly equal work: the spread inside the layer is a few percent."""
    d = wl.gen_layer(2, 8, with_input=False)           # 512 -> 512
    L = _host_layer(d)
    st = L.stats()
    assert st["group_size"] == 8 and st["filter_groups"] == 64     # the default variant: groups of 8
    assert st["distinct_filter_lengths"] > 10                     # lengths do vary ...
    mean = st["kept_kernels"] / st["filter_groups"]
    assert st["max_group_kernels"] < 1.25 * mean                  # ... groups follow the sort
    assert st["min_group_kernels"] > 0.75 * mean
    L.close()


def _walk_steps(t, lib_masks, c_out, c_in):
    """Executes the step streams of a tiled layout the way the kernel's interpreter does
    (two alternating scalar register sets, window register sets, one channel per
    window, call or threaded dispatch) and returns the dense weights / ids / mask they
    describe, plus the number of steps walked.  Raises on anything the interpreter
    could not execute."""
    uni_masks = wl.pattern_universe()
    G, R = t["G"], t["records"]
    cb, tab, bb = t["ctrl_bytes"], t["table_off"], t["block_bytes"]
    sets = 2 if t["double_window"] else 1
    threaded = bool(t["threaded"])
    w = np.zeros((c_out, c_in, 3, 3), np.float32)
    ids = np.full((c_out, c_in), 255, np.int32)
    km = np.zeros((c_out, c_in), np.uint8)
    steps = t["steps"]
    walked = 0

    def load_window(window, which, off, chunk):
        assert which < sets
        assert off % t["lds_channel_bytes"] == 0
        ch = chunk * t["ck"] + off // t["lds_channel_bytes"]
        assert ch < min(c_in, (chunk + 1) * t["ck"])
        window[which] = ch

    def run_kernel(g, window, tg, weights, loading):
        assert tg >= tab and (tg - tab) % bb == 0, tg
        ws, rest = divmod((tg - tab) // bb, G * 56)
        slot, u = divmod(rest, 56)
        assert ws < sets and window[ws] is not None
        # with two window sets, the set being loaded is not the one the kernels read
        if t["double_window"] and loading is not None:
            assert ws != loading
        co, ci = int(t["slot_channel"][g, slot]), window[ws]
        assert co >= 0 and km[co, ci] == 0
        km[co, ci] = 1
        m = int(uni_masks[u])
        w[co, ci].reshape(9)[[p for p in range(9) if (m >> p) & 1]] = weights.view(np.float32)
        ids[co, ci] = [i for i, lm in enumerate(lib_masks) if int(lm) == m][0]

    for g in range(t["num_groups"]):
        for chunk in range(t["num_chunks"]):
            cp = int(t["chunk_ptr"][g, chunk])
            pos, entry = cp & 0x0FFFFFFF, cp >> 28
            window = [None] * sets          # channel held by each window register set
            if not threaded:
                assert entry == 0
                for k in range(1 << 20):
                    st = steps[pos + k]
                    assert pos + k + 1 < len(steps)         # the step fetched ahead exists
                    walked += 1
                    blk = int(st[20])
                    assert blk % cb == 0 and blk // cb in (0, 1, 2, 5), blk
                    if blk // cb == 5:
                        break
                    loading = blk // cb if blk // cb in (0, 1) else None
                    if loading is not None:
                        load_window(window, loading, int(st[21]), chunk)
                    done = (4 if k & 1 else 3) * cb
                    for q in range(R):
                        if int(st[16 + q]) == done:
                            break
                        run_kernel(g, window, int(st[16 + q]), st[4 * q:4 * q + 4], loading)
                else:
                    raise AssertionError("stream does not end")
            else:
                k = 0
                while True:
                    assert entry <= 6 and k < (1 << 20)
                    if entry == 6:
                        break
                    st = steps[pos + k]
                    assert pos + k + 1 < len(steps)
                    walked += 1
                    assert entry // 3 == (k & 1)            # the register set the step was fetched into
                    loading = entry % 3 - 1 if entry % 3 else None
                    if loading is not None:
                        load_window(window, loading, int(st[23]), chunk)
                    q = 0
                    while True:
                        tg = int(st[6 * q + 4]) if q < R else int(st[22])
                        if tg < tab:                        # a control block: the step is over
                            assert tg % cb == 0
                            entry = tg // cb
                            break
                        assert q < R
                        run_kernel(g, window, tg, st[6 * q:6 * q + 4], loading)
                        q += 1
                    k += 1
    return w, ids, km, walked


@pytest.mark.parametrize("config,layer,ck", [(1, 0, 0), (1, 0, 3), (2, 3, 8), (3, 8, 16), (3, 15, 5)])
def test_tiled_step_streams_decode_to_the_layer(oracle, config, layer, ck):
    """Every sparse tiled variant's step stream, interpreted as the kernel does, is exactly
    the pruned layer: masks, pattern per kernel and weight bits (sections 5.2-5.4)."""
    d = wl.gen_layer(config, layer, with_input=False)
    spec = d["spec"]
    L = _host_layer(d)
    want = oracle.masked_weights(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"])
    seen = 0
    for v in range(1, B.patdnn_num_variants()):
        try:
            t = L.export_tiled(v, ck)
        except B.PatdnnError as e:
            assert e.status == B.PATDNN_EUNSUPPORTED
            continue
        seen += 1
        w, ids, km, walked = _walk_steps(t, d["pattern_masks"], spec.c_out, spec.c_in)
        assert w.view(np.uint32).tolist() == want.view(np.uint32).tolist()
        np.testing.assert_array_equal(km, d["kernel_mask"])
        np.testing.assert_array_equal(ids[km == 1], d["pattern_ids"][km == 1])
        assert walked == t["num_steps"] - 1            # every step is reached exactly once (+1 pad)
        assert t["threaded"] in (0, 1) and t["records"] == (3 if t["threaded"] else 4)
        assert sorted(c for c in t["slot_channel"].ravel() if c >= 0) == list(range(spec.c_out))
    assert seen >= 4          # call / threaded dispatch x one / two window register sets
    L.close()


def test_step_streams_of_random_layers_decode_exactly():
    """Random shapes, densities and chunk sizes (including filters without kernels, channels
    nobody reads, group sizes that do not divide c_out, chunk sizes that do not divide
    c_in): every sparse variant's stream rebuilds the layer bit for bit."""
    from hypothesis import given, settings, strategies as st

    lib = wl.pattern_library(wl.PATTERN_SEED)

    @settings(max_examples=30, deadline=None, derandomize=True)
    @given(c_out=st.integers(1, 70), c_in=st.integers(1, 40), keep=st.sampled_from([0.0, 0.1, 0.3, 0.6, 1.0]),
           ck=st.integers(1, 19), stride=st.sampled_from([1, 2]), seed=st.integers(0, 10_000))
    def run(c_out, c_in, keep, ck, stride, seed):
        rng = np.random.default_rng(seed)
        w = rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32)
        ids = rng.integers(0, 8, (c_out, c_in), dtype=np.uint8)
        mask = (rng.random((c_out, c_in)) < keep).astype(np.uint8)
        L = B.Layer(w, ids, mask, lib, stride=stride, host_only=True)
        bits = np.array([[(int(m) >> p) & 1 for p in range(9)] for m in lib], np.uint8).reshape(8, 3, 3)
        want = np.where((mask[:, :, None, None] == 1) & (bits[ids] == 1), w, np.float32(0)).astype(np.float32)
        try:
            for v in range(1, B.patdnn_num_variants()):
                try:
                    t = L.export_tiled(v, ck)
                except B.PatdnnError as e:
                    assert e.status == B.PATDNN_EUNSUPPORTED
                    continue
                got_w, got_ids, km, walked = _walk_steps(t, lib, c_out, c_in)
                assert got_w.view(np.uint32).tolist() == want.view(np.uint32).tolist()
                np.testing.assert_array_equal(km, mask)
                np.testing.assert_array_equal(got_ids[km == 1], ids[km == 1])
                assert walked == t["num_steps"] - 1
        finally:
            L.close()

    run()


def test_fkw_index_overhead_against_csr_matches_the_paper():
    """Section 6.3 quotes what FKW saves against CSR at the 8x rate on VGG-16's unique CONV
    layers: 87.9 % of the index overhead, 43.9 % of the total storage.  The exported arrays
    of the synthetic VGG-shaped layers (same 4-of-9 patterns, same 3.6x connectivity rate),
    stored in the narrowest integer type that holds each array, against CSR with one 32-bit
    column index per non-zero weight and one row pointer per filter, give the same figures."""
    g = read_golden_kv("paper_constants.txt")
    fkw_bytes = csr_bytes = weight_bytes = 0
    for li in (1, 2, 3, 4, 5, 7, 8, 10):                      # one layer of each distinct shape
        d = wl.gen_layer(2, li, with_input=False)
        L = _host_layer(d)
        f = L.export_fkw()
        L.close()

        def width(a):
            m = int(a.max()) if a.size else 0
            return 1 if m < 256 else 2 if m < 65536 else 4

        kept = f["index"].size
        fkw_bytes += sum(f[k].size * width(f[k]) for k in ("offset", "reorder", "index", "stride"))
        csr_bytes += 4 * 4 * kept + 4 * (d["spec"].c_out + 1)
        weight_bytes += 16 * kept
    index_saving = 1 - fkw_bytes / csr_bytes
    total_saving = (csr_bytes - fkw_bytes) / (csr_bytes + weight_bytes)
    assert abs(index_saving - float(g["fkw_vs_csr_index_saving_8x"][0])) < 0.02
    assert abs(total_saving - float(g["fkw_vs_csr_total_saving_8x"][0])) < 0.01


def test_an_explicit_configuration_is_strict():
    """A configuration the caller sets is accepted or refused, never replaced by another:
    more input-channel slices than the layer has chunks is an error at set_config time."""
    rng = np.random.default_rng(3)
    lib = wl.pattern_library(wl.PATTERN_SEED)
    c_out, c_in = 16, 7
    L = B.Layer(rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32),
                rng.integers(0, 8, (c_out, c_in), dtype=np.uint8),
                (rng.random((c_out, c_in)) < 0.5).astype(np.uint8), lib, host_only=True)
    L.set_config(1, 4, 4, 2)                       # 7 channels in chunks of 4: two chunks
    assert L.get_config() == {"variant": 1, "ck": 4, "waves": 4, "ksplit": 2}
    with pytest.raises(B.PatdnnError) as e:
        L.set_config(1, 4, 4, 3)
    assert e.value.status == B.PATDNN_EUNSUPPORTED
    assert L.get_config()["ksplit"] == 2           # the refused configuration replaced nothing
    L.close()


def test_workspace_size_follows_the_configuration():
    """patdnn_workspace_floats: one buffer of the un-pooled output, rounded up to 64 floats, per
    channel slice of the present configuration; nothing for a configuration that does not split,
    for the default configuration, or for arguments the convolution would reject."""
    rng = np.random.default_rng(4)
    lib = wl.pattern_library(wl.PATTERN_SEED)
    c_out, c_in = 24, 40
    L = B.Layer(rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32),
                rng.integers(0, 8, (c_out, c_in), dtype=np.uint8),
                (rng.random((c_out, c_in)) < 0.5).astype(np.uint8), lib, pad=0, host_only=True)
    assert L.workspace_floats(2, 13, 17) == 0                      # default configuration
    for ksplit in (1, 2, 5):
        L.set_config(1, 8, 4, ksplit)
        for n, h, w in ((2, 13, 17), (1, 8, 8), (3, 30, 5)):
            full = n * c_out * (h - 2) * (w - 2)
            want = 0 if ksplit == 1 else ksplit * (-(-full // 64) * 64)
            assert L.workspace_floats(n, h, w) == want, (ksplit, n, h, w)
    assert L.workspace_floats(1, 2, 9) == 0                        # smaller than the kernel: rejected
    assert L.workspace_floats(1, 0, 9) == 0
    L.close()


@pytest.mark.parametrize("config,layer", [(1, 0), (2, 3), (3, 3)])
def test_exported_csr_is_the_textbook_csr_of_the_pruned_layer(config, layer):
    """The CSR arrays the comparison kernel reads, against the oracle's CSR (itself pinned to
    scipy's): same row pointers, columns and weight bits."""
    from oracle import csr as ocsr
    d = wl.gen_layer(config, layer, with_input=False)
    L = _host_layer(d)
    got = L.export_csr()
    row_ptr, col, val = ocsr.build_csr(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"])
    np.testing.assert_array_equal(got["row_ptr"], row_ptr)
    np.testing.assert_array_equal(got["col"], col)
    assert got["val"].view(np.uint32).tolist() == val.view(np.uint32).tolist()
    L.close()
    # dense and depthwise layers have no such form here
    for cfg, li in ((2, 0), (4, 0)):
        Ld = _host_layer(wl.gen_layer(cfg, li, with_input=False))
        with pytest.raises(B.PatdnnError) as e:
            Ld.export_csr()
        assert e.value.status == B.PATDNN_EUNSUPPORTED
        Ld.close()
