"""GPU parity of the fused ReLU + 2x2 max-pool epilogue and of whole stacks run back to
back, plain and as a HIP graph (the paper's headline scenario, section 6.2: one image
through all CONV layers), against the oracle's chained stack layer by layer."""

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
    B.lib()
    return torch


def _rel(got, ref):
    scale = float(np.abs(ref).max())
    err = float(np.abs(got.astype(np.float64) - ref).max())
    return err / scale if scale > 0 else err


@pytest.mark.parametrize("case", [
    dict(c_out=24, c_in=20, n=3, h=13, w=13, keep=0.3),           # odd size: last row and column dropped
    dict(c_out=40, c_in=7, n=2, h=28, w=18, keep=0.5),
    dict(c_out=16, c_in=33, n=2, h=8, w=50, keep=0.25, pad=0),
    dict(c_out=32, c_in=16, n=2, h=21, w=20, keep=0.3, stride=2),
    dict(c_out=48, c_in=5, n=2, h=18, w=33, keep=1.0, dense=True),
])
def test_fused_pool_on_every_variant(torch, oracle, case):
    from oracle import stack as ostack
    rng = np.random.default_rng(4000 + case["c_out"] + case["h"])
    lib = wl.pattern_library(wl.PATTERN_SEED)
    stride, pad, dense = case.get("stride", 1), case.get("pad", 1), case.get("dense", False)
    ids = rng.integers(0, 8, (case["c_out"], case["c_in"]), dtype=np.uint8)
    mask = (rng.random((case["c_out"], case["c_in"])) < case["keep"]).astype(np.uint8)
    w = rng.standard_normal((case["c_out"], case["c_in"], 3, 3)).astype(np.float32)
    bias = rng.standard_normal(case["c_out"]).astype(np.float32)
    x = rng.standard_normal((case["n"], case["c_in"], case["h"], case["w"])).astype(np.float32)
    ref = ostack.maxpool2x2(oracle.conv2d(w, ids, mask, lib, x, bias, stride=stride, pad=pad, relu=True,
                                          dense=dense, skip_removed=True))
    L = B.Layer(w, ids, mask, lib, stride=stride, pad=pad, dense=dense)
    xt, bt = torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda()
    seen = 0
    for v in [-1] + list(range(B.patdnn_num_variants())):
        try:
            L.set_config(v, 4 if v > 0 else 0, 4 if v > 0 else 0, 1)
        except B.PatdnnError as e:
            assert e.status == B.PATDNN_EUNSUPPORTED
            continue
        guard = 1024
        numel = int(np.prod(ref.shape))
        buf = torch.full((numel + 2 * guard,), 777.0, dtype=torch.float32, device="cuda")
        out = buf[guard:guard + numel].view(ref.shape)
        try:
            L.conv2d_pool(xt, bt, out)
        except B.PatdnnError as e:
            # the comparison kernels (no-opt, CSR) have no pooled epilogue and say so
            assert e.status == B.PATDNN_EUNSUPPORTED and B.patdnn_variant_name(v) in ("noopt", "csr")
            continue
        full = L.conv2d(xt, bt, relu=True)
        torch.cuda.synchronize()
        assert bool((buf[:guard] == 777.0).all()) and bool((buf[guard + numel:] == 777.0).all())
        got = out.cpu().numpy()
        err = _rel(got, ref)
        _say(f"    {case} variant {B.patdnn_variant_name(v) if v >= 0 else 'auto'}: rel_err={err:.2e}")
        assert err <= TOL
        # and exactly the pooling of what the same configuration writes without the fusion
        want = torch.nn.functional.max_pool2d(full, 2, 2)
        assert bool((out == want).all())
        seen += 1
    L.close()
    assert seen >= 3


def _vgg_prefix(depth):
    """The first `depth` layers of the VGG-16 shaped stack (N = 1) with its pooling plan."""
    pool_after = {1, 3, 6, 9, 12}              # after conv 2, 4, 7, 10, 13
    layers = [wl.gen_layer(2, li, with_input=(li == 0)) for li in range(depth)]
    return layers, [li in pool_after for li in range(depth)]


def _apply_tuned(L, spec):
    """The launch configuration bench.py uses for this shape, if the committed table has one."""
    import os
    table = wl.load_tuned_configs(os.path.join(os.path.dirname(B.LIB_PATH), "tuned_configs.json"))
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
    c = table.get(wl.shape_key(spec))
    if c is not None and c["variant"] in names:
        L.set_config(names[c["variant"]], c["ck"], c["waves"], c["ksplit"])
    return L.get_config()


@pytest.mark.parametrize("depth,tuned", [(2, False), (4, False), (7, False), (13, False), (7, True), (13, True)])
def test_vgg_stack_matches_the_oracle_chain(torch, oracle, depth, tuned):
    """tuned: the batch-1 configurations of the committed table, most of which split the
    input channels (partial sums added with atomics, so the last bits vary from run to run
    and the graph replays are compared within the tolerance instead of bit for bit)."""
    from oracle import stack as ostack
    layers, pool = _vgg_prefix(depth)
    x = layers[0]["input"]
    ref = ostack.stack_forward(layers, x, pool)
    Ls = [B.Layer.from_workload(d) for d in layers]
    split = False
    if tuned:
        for L, d in zip(Ls, layers):
            cfg = _apply_tuned(L, d["spec"])
            split |= cfg["ksplit"] > 1
        _say(f"    tuned configurations: {[L.get_config() for L in Ls]}")
    biases = [torch.from_numpy(d["bias"]).cuda() for d in layers]
    st = B.Stack([(L, b, True, p) for L, b, p in zip(Ls, biases, pool)], 1, x.shape[2], x.shape[3])
    assert st.output_shape() == ref[-1].shape
    xt = torch.from_numpy(x).cuda()
    side = torch.cuda.Stream()
    plain = st.run(xt)
    torch.cuda.synchronize()
    err = _rel(plain.cpu().numpy(), ref[-1])
    _say(f"    depth {depth}: plain rel_err={err:.2e}")
    assert err <= TOL
    out = torch.empty_like(plain)
    with torch.cuda.stream(side):
        for rep in range(4):                   # capture, then replays, with eager work between
            out.fill_(-1.0)
            st.run(xt, out, graph=True, stream=side)
            side.synchronize()
            if split:
                assert _rel(out.cpu().numpy(), ref[-1]) <= TOL, f"graph run {rep} is off"
            else:
                assert bool((out == plain).all()), f"graph run {rep} differs from the plain run"
            _ = (xt * 2).sum().item()
    st.close()
    for L in Ls:
        L.close()


@pytest.mark.parametrize("ksplits", [
    (2, 2, 2, 2, 2, 2, 2),        # every layer hands the next one its zeroed target
    (1, 2, 1, 2, 2, 1, 2),        # unsplit layers have no finishing kernel: the next one fills for itself
    (2, 1, 2, 1, 1, 2, 1),        # ... and unsplit pooled layers after split ones get their output zeroed
])
@pytest.mark.parametrize("configured", ["before", "after"])
def test_neighbouring_layers_share_zero_fills(torch, oracle, ksplits, configured):
    """Every pairing of split / unsplit and pooled / plain neighbours in a stack must match the
    oracle's chain, also on later runs, when the buffers between the layers hold old values.
    Configured before the stack is created, the split layers find one partial-sum buffer per
    slice in it and store; configured afterwards they find room for one buffer at most and add
    their slices up with atomics - then a split layer clears, in its finishing kernel, what
    the next layer accumulates into (its output, its pooled output or the partial-sum buffer)."""
    from oracle import stack as ostack
    layers, pool = _vgg_prefix(len(ksplits))
    x = layers[0]["input"]
    ref = ostack.stack_forward(layers, x, pool)
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
    Ls = [B.Layer.from_workload(d) for d in layers]
    biases = [torch.from_numpy(d["bias"]).cuda() for d in layers]

    def configure():
        for L, d, k in zip(Ls, layers, ksplits):
            if d["spec"].c_in >= 16:             # the first layer (3 channels) has a single chunk to split
                L.set_config(names["t_g8_p7x2_s1_x8_thw1b"], 8, 4, k)

    if configured == "before":
        configure()
    st = B.Stack([(L, b, True, p) for L, b, p in zip(Ls, biases, pool)], 1, x.shape[2], x.shape[3])
    if configured == "after":
        configure()
    xt = torch.from_numpy(x).cuda()
    for rep in range(3):
        out = st.run(xt)
        torch.cuda.synchronize()
        err = _rel(out.cpu().numpy(), ref[-1])
        _say(f"    ksplits {ksplits} configured {configured} run {rep}: rel_err={err:.2e}")
        assert err <= TOL
    st.close()
    for L in Ls:
        L.close()


@pytest.mark.parametrize("ksplit", [2, 3])
def test_pooled_split_layer_with_a_workspace(torch, oracle, ksplit):
    """patdnn_conv2d_ws with fused pooling on a configuration that splits the input channels:
    with room for one buffer per slice (stores, summed in slice order: repeatable bits), with
    room for a single buffer (the slices add into it with atomics), and with none (the call
    falls back to the layer's default configuration) - all three against the oracle."""
    from oracle import stack as ostack
    rng = np.random.default_rng(77 + ksplit)
    lib = wl.pattern_library(wl.PATTERN_SEED)
    c_out, c_in, n, h, w = 40, 36, 3, 17, 22
    ids = rng.integers(0, 8, (c_out, c_in), dtype=np.uint8)
    mask = (rng.random((c_out, c_in)) < 0.4).astype(np.uint8)
    wt = rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32)
    bias = rng.standard_normal(c_out).astype(np.float32)
    x = rng.standard_normal((n, c_in, h, w)).astype(np.float32)
    ref = ostack.maxpool2x2(oracle.conv2d(wt, ids, mask, lib, x, bias, relu=True, skip_removed=True))
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
    L = B.Layer(wt, ids, mask, lib)
    xt, bt = torch.from_numpy(x).cuda(), torch.from_numpy(bias).cuda()
    for vname in ("t_g8_p7x2_s1_x8_thw1b", "t_g16_p7x1_s1_x16"):
        L.set_config(names[vname], 8, 4, ksplit)
        need = L.workspace_floats(n, h, w)
        full = n * c_out * h * w
        assert need >= ksplit * full
        guard = 1024
        for room, what in ((need, "one buffer per slice"), (full, "one buffer"), (0, "no workspace")):
            wbuf = torch.full((room + 2 * guard,), float("nan"), dtype=torch.float32, device="cuda")
            wbuf[:guard] = 4242.0
            wbuf[guard + room:] = 4242.0
            outs = []
            for _ in range(2):
                out = L.conv2d_ws(xt, bt, workspace=wbuf[guard:guard + room] if room else None, pool=True)
                torch.cuda.synchronize()
                assert bool((wbuf[:guard] == 4242.0).all()) and bool((wbuf[guard + room:] == 4242.0).all())
                err = _rel(out.cpu().numpy(), ref)
                assert err <= TOL, (vname, what, err)
                outs.append(out)
            _say(f"    {vname} ksplit {ksplit}, {what}: rel_err={err:.2e}")
            if room == need:
                assert bool((outs[0] == outs[1]).all()), "slice buffers must give repeatable bits"
    L.close()
