"""Pins of the oracle modules behind the rows beyond single layers: the chained stack
with pooling (oracle/stack.py), the pruning projections (oracle/projection.py) and the
CSR form (oracle/csr.py).  Each is checked against something other than itself: values
worked by hand, library routines (torch, scipy), brute force on tiny inputs, closed forms."""

import itertools

import numpy as np
import pytest

from conftest import read_golden_rows
from oracle import csr as ocsr
from oracle import projection as proj
from oracle import ref
from oracle import stack as ostack
from paper_2001_00138_amd import workloads as wl


# ---------------------------------------------------------------------------- stack
def test_maxpool_hand_example():
    rows = read_golden_rows("maxpool_hand.txt")
    x = np.array([[float(v) for v in r[1:]] for r in rows if r[0] == "in:"])
    want = np.array([[float(v) for v in r[1:]] for r in rows if r[0] == "out:"])
    got = ostack.maxpool2x2(x[None, None])
    np.testing.assert_array_equal(got[0, 0], want)


@pytest.mark.parametrize("shape", [(2, 3, 8, 8), (1, 2, 7, 9), (3, 1, 2, 2), (1, 1, 5, 4)])
def test_maxpool_equals_the_library_routine(shape):
    import torch
    rng = np.random.default_rng(sum(shape))
    x = rng.standard_normal(shape)
    want = torch.nn.functional.max_pool2d(torch.from_numpy(x), 2, 2).numpy()
    np.testing.assert_array_equal(ostack.maxpool2x2(x), want)
    # ReLU is monotone, so it commutes with max pooling
    np.testing.assert_array_equal(ostack.maxpool2x2(np.maximum(x, 0)), np.maximum(ostack.maxpool2x2(x), 0))


def test_stack_forward_equals_a_torch_chain():
    import torch
    rng = np.random.default_rng(11)
    lib = wl.pattern_library(wl.PATTERN_SEED)
    chans = [3, 5, 4, 6]
    layers = []
    for i in range(3):
        c_in, c_out = chans[i], chans[i + 1]
        layers.append({"spec": wl.LayerSpec(name=f"l{i}", c_in=c_in, c_out=c_out, h=0, w=0),
                       "pattern_masks": lib,
                       "pattern_ids": rng.integers(0, 8, (c_out, c_in), dtype=np.uint8),
                       "kernel_mask": (rng.random((c_out, c_in)) < 0.6).astype(np.uint8),
                       "weights": rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32),
                       "bias": rng.standard_normal(c_out).astype(np.float32)})
    x = rng.standard_normal((2, 3, 11, 10)).astype(np.float32)
    pool = [True, False, True]
    got = ostack.stack_forward(layers, x, pool)
    cur = torch.from_numpy(x).double()
    for d, p, g in zip(layers, pool, got):
        wm = ref.masked_weights(d["weights"], d["pattern_ids"], d["kernel_mask"], d["pattern_masks"])
        y = torch.relu(torch.nn.functional.conv2d(cur, torch.from_numpy(wm).double(),
                                                  torch.from_numpy(d["bias"]).double(), padding=1))
        if p:
            y = torch.nn.functional.max_pool2d(y, 2, 2)
        assert np.abs(g - y.numpy()).max() <= 1e-12 * max(1.0, float(y.abs().max()))
        cur = y.float().double()          # the next layer sees what an fp32 tensor holds
    assert got[0].shape == (2, 5, 5, 5) and got[2].shape == (2, 6, 2, 2)


# ---------------------------------------------------------------------------- projections
def _universe_set():
    return {int(m) for m in wl.pattern_universe()}


def test_natural_pattern_hand_cases_and_invariants():
    # centre small, still kept; the three largest others are positions 0, 2, 7
    k = np.array([[9, 1, -8], [0.5, 0.01, 0.2], [0.3, 7, -0.1]], np.float32)
    assert proj.natural_pattern(k) == (1 << 4) | (1 << 0) | (1 << 2) | (1 << 7)
    # ties go to the lower position
    k = np.ones((3, 3), np.float32)
    assert proj.natural_pattern(k) == (1 << 4) | 0b111
    rng = np.random.default_rng(5)
    uni = _universe_set()
    assert len(uni) == 56                      # section 4.1: C(8,3) natural patterns
    seen = set()
    for _ in range(3000):
        k = rng.standard_normal((3, 3)).astype(np.float32)
        m = proj.natural_pattern(k)
        assert m in uni
        # brute force: the centre-keeping 4-entry mask with the largest sum of magnitudes
        best = max(uni, key=lambda u: sum(abs(float(k.reshape(9)[p])) for p in range(9) if (u >> p) & 1))
        assert m == best
        seen.add(m)
    assert len(seen) == 56                     # every one of the 56 occurs


def test_mine_pattern_set_counts_and_order():
    uni = sorted(_universe_set())
    freq = {uni[3]: 5, uni[40]: 9, uni[17]: 5, uni[8]: 2}
    kernels = []
    for m, c in freq.items():
        for j in range(c):
            k = np.full(9, 0.01 * (j + 1), np.float32)
            for p in range(9):
                if (m >> p) & 1 and p != 4:
                    k[p] = 1.0 + 0.1 * p
            kernels.append(k.reshape(3, 3))
    w = np.array(kernels, np.float32).reshape(3, 7, 3, 3)
    got = proj.mine_pattern_set(w, 3)
    assert got.tolist() == [uni[40], min(uni[3], uni[17]), max(uni[3], uni[17])]
    assert proj.mine_pattern_set(w, 10).tolist()[3] == uni[8]      # fewer patterns than asked


def test_pattern_projection_is_the_nearest_feasible_kernel():
    rng = np.random.default_rng(8)
    lib = wl.pattern_library(wl.PATTERN_SEED)
    w = rng.standard_normal((4, 5, 3, 3)).astype(np.float32)
    ids, z = proj.project_patterns(w, lib)
    for co in range(4):
        for ci in range(5):
            k = w[co, ci].astype(np.float64)
            # brute force: distance to the closest kernel that satisfies each pattern
            dist = []
            for m in lib:
                keep = np.array([(int(m) >> p) & 1 for p in range(9)], bool).reshape(3, 3)
                dist.append(float(((k * ~keep) ** 2).sum()))
            assert ids[co, ci] == int(np.argmin(dist))
            keep = np.array([(int(lib[ids[co, ci]]) >> p) & 1 for p in range(9)], bool).reshape(3, 3)
            np.testing.assert_array_equal(z[co, ci], np.where(keep, w[co, ci], np.float32(0)))
    ids2, z2 = proj.project_patterns(z, lib)      # a feasible tensor is its own projection
    np.testing.assert_array_equal(z2, z)
    np.testing.assert_array_equal(ids2, ids)


def test_connectivity_projection_is_the_nearest_feasible_tensor():
    rng = np.random.default_rng(13)
    w = rng.standard_normal((2, 3, 3, 3)).astype(np.float32)
    flat = w.reshape(6, 9).astype(np.float64)
    for alpha in range(0, 8):
        mask = proj.project_connectivity(w, alpha)
        assert int(mask.sum()) == min(alpha, 6)
        best = min(itertools.combinations(range(6), min(alpha, 6)),
                   key=lambda keep: sum((flat[i] ** 2).sum() for i in range(6) if i not in keep))
        assert sorted(np.flatnonzero(mask.reshape(-1)).tolist()) == sorted(best)
    # ties: equal norms keep the lower flat index
    w[:] = 1.0
    assert proj.project_connectivity(w, 2).reshape(-1).tolist() == [1, 1, 0, 0, 0, 0]


def test_joint_projection_reaches_the_papers_rates():
    """Pattern projection keeps 4 of 9 weights and connectivity projection 1/3.6 of the
    kernels: (9/4)*3.6 = 8.1, the roughly eightfold figure the paper gives for an all-3x3 network (section 4.3)."""
    rng = np.random.default_rng(21)
    w = rng.standard_normal((12, 15, 3, 3)).astype(np.float32)
    lib = proj.mine_pattern_set(w, 8)
    assert len(lib) == 8
    ids, z = proj.project_patterns(w, lib)
    alpha = wl.round_half_even(12 * 15 / 3.6)
    mask = proj.project_connectivity(z, alpha)
    kept_weights = int((z != 0).reshape(12, 15, 9).sum(axis=2)[mask.astype(bool)].sum())
    assert kept_weights == 4 * alpha
    assert abs(w.size / kept_weights - 8.1) < 1e-9


# ---------------------------------------------------------------------------- CSR
def _layer(rng, c_out, c_in, keep):
    lib = wl.pattern_library(wl.PATTERN_SEED)
    return (rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32),
            rng.integers(0, 8, (c_out, c_in), dtype=np.uint8),
            (rng.random((c_out, c_in)) < keep).astype(np.uint8), lib)


def test_csr_is_the_textbook_format():
    import scipy.sparse as sp
    rng = np.random.default_rng(31)
    w, ids, km, lib = _layer(rng, 7, 5, 0.5)
    row_ptr, col, val = ocsr.build_csr(w, ids, km, lib)
    wm = ref.masked_weights(w, ids, km, lib)
    a = sp.csr_matrix(wm.reshape(7, 45))           # scipy drops nothing here: no stored zero
    a.sort_indices()
    np.testing.assert_array_equal(row_ptr, a.indptr)
    np.testing.assert_array_equal(col, a.indices)
    np.testing.assert_array_equal(val.view(np.uint32), a.data.view(np.uint32))
    assert len(val) == 4 * int(km.sum())
    # an empty filter has an empty row
    km[3] = 0
    row_ptr, col, val = ocsr.build_csr(w, ids, km, lib)
    assert row_ptr[3] == row_ptr[4]


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 1), (1, 0), (2, 0)])
def test_csr_walk_equals_the_definition(stride, pad):
    rng = np.random.default_rng(37 + stride + pad)
    w, ids, km, lib = _layer(rng, 6, 4, 0.6)
    x = rng.standard_normal((2, 4, 9, 8)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    want = ref.conv2d(w, ids, km, lib, x, b, stride=stride, pad=pad, relu=True)
    got = ocsr.csr_conv2d(*ocsr.build_csr(w, ids, km, lib), x, b, stride=stride, pad=pad, relu=True)
    assert np.abs(got - want).max() <= 1e-12 * max(1.0, float(np.abs(want).max()))


# ---------------------------------------------------------------------------- fp16 storage
def test_binary16_rounding_hand_values_and_library():
    """The storage rounding the fp16 oracle relies on, against values fixed by the format
    (10 fraction bits: spacing 2 above 2048, ties to even; largest finite 65504; smallest
    subnormal 2^-24) and against torch's conversion."""
    import torch
    from oracle import fp16
    cases = [(2049.0, 2048.0), (2051.0, 2052.0), (2050.0, 2050.0), (1.0 + 2.0 ** -11, 1.0),
             (1.0 + 3 * 2.0 ** -11, 1.0 + 2.0 ** -9), (65504.0, 65504.0), (65519.9, 65504.0), (65520.0, np.inf),
             (2.0 ** -24, 2.0 ** -24), (2.0 ** -25, 0.0), (1.5 * 2.0 ** -24, 2.0 ** -23), (-0.1, -0.0999755859375)]
    for x, want in cases:
        got = float(fp16.to_f16(np.float64(x)))
        assert got == want, (x, got, want)
    rng = np.random.default_rng(16)
    x = (rng.standard_normal(20000) * 10.0 ** rng.integers(-6, 5, 20000)).astype(np.float32)
    np.testing.assert_array_equal(fp16.to_f16(x).view(np.uint16),
                                  torch.from_numpy(x).half().numpy().view(np.uint16))


def test_fp16_conv_is_the_definition_on_stored_values():
    """Independent route: torch conv2d in float64 on the binary16-rounded tensors (torch's
    own rounding), rounded once at the end."""
    import torch
    from oracle import fp16
    rng = np.random.default_rng(17)
    w, ids, km, lib = _layer(rng, 6, 5, 0.6)
    x = rng.standard_normal((2, 5, 9, 8)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    got16, exact = fp16.conv2d_f16(w, ids, km, lib, x, b, relu=True)
    wm = ref.masked_weights(torch.from_numpy(w).half().float().numpy(), ids, km, lib)
    y = torch.relu(torch.nn.functional.conv2d(torch.from_numpy(x).half().double(), torch.from_numpy(wm).double(),
                                              torch.from_numpy(b).double(), padding=1))
    assert float((torch.from_numpy(exact) - y).abs().max()) <= 1e-12 * float(y.abs().max())
    # rounding once at the end: within half a binary16 spacing of the exact value
    assert np.all(np.abs(got16.astype(np.float64) - exact) <= 2.0 ** -11 * np.maximum(np.abs(exact), 2.0 ** -14))
