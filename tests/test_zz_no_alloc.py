"""The entry point that allocates nothing (patdnn_stack_run_static) against the entry point
it is a variant of (patdnn_stack_run): same results, on two calls in a row, the second on a
smaller stack - the built-in buffer keeps the first call's contents, which must not matter."""

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


def _layers(rng, chans, keep=0.4):
    lib = wl.pattern_library(wl.PATTERN_SEED)
    out = []
    for c_in, c_out in zip(chans[:-1], chans[1:]):
        out.append(dict(w=rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32) * np.float32(0.3),
                        ids=rng.integers(0, 8, (c_out, c_in), dtype=np.uint8),
                        mask=(rng.random((c_out, c_in)) < keep).astype(np.uint8), lib=lib,
                        bias=rng.standard_normal(c_out).astype(np.float32)))
    return out


def _run_both(torch, oracle, rng, chans, pool, n, h, w, split_layer):
    from oracle import stack as ostack
    specs = _layers(rng, chans)
    Ls = [B.Layer(d["w"], d["ids"], d["mask"], d["lib"]) for d in specs]
    names = {B.patdnn_variant_name(v): v for v in range(B.patdnn_num_variants())}
    if split_layer is not None:
        # a pooled layer that splits its input channels: its partial sums go through the buffer
        Ls[split_layer].set_config(names["t_g16_p7x1_s1_x16"], 4, 4, 2)
    biases = [torch.from_numpy(d["bias"]).cuda() for d in specs]
    st = B.Stack([(L, b, True, p) for L, b, p in zip(Ls, biases, pool)], n, h, w)
    x = rng.standard_normal((n, chans[0], h, w)).astype(np.float32)
    xt = torch.from_numpy(x).cuda()
    want = st.run(xt)
    torch.cuda.synchronize()
    guard, numel = 2048, int(np.prod(st.output_shape()))
    buf = torch.full((numel + 2 * guard,), 555.0, dtype=torch.float32, device="cuda")
    got = buf[guard:guard + numel].view(st.output_shape())
    st.run_static(xt, got)
    torch.cuda.synchronize()
    assert bool((buf[:guard] == 555.0).all()) and bool((buf[guard + numel:] == 555.0).all())
    a, b = got.cpu().numpy(), want.cpu().numpy()
    scale = float(np.abs(b).max())
    err = float(np.abs(a.astype(np.float64) - b).max()) / scale
    _say(f"    chans={chans} n={n} {h}x{w}: static vs own buffers rel_err={err:.2e}")
    if split_layer is None:
        assert bool((got == want).all())                 # same kernels, same order: the same bits
    else:
        assert err <= TOL                                # atomically added slices: any order
    # and both are the oracle's chain
    class _S:                                            # what stack_forward reads of a layer spec
        stride, pad, depthwise, dense = 1, 1, False, False
    chain = ostack.stack_forward([dict(weights=d["w"], pattern_ids=d["ids"], kernel_mask=d["mask"],
                                       pattern_masks=d["lib"], bias=d["bias"], spec=_S) for d in specs], x, pool)
    assert float(np.abs(a.astype(np.float64) - chain[-1]).max()) / float(np.abs(chain[-1]).max()) <= TOL
    st.close()
    for L in Ls:
        L.close()


def test_static_buffer_entry_point_matches_the_allocating_one():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from oracle import ref as oracle
    oracle.build()
    rng = np.random.default_rng(777)
    # first call: four layers, two pooled (one of them split), batch 3
    _run_both(torch, oracle, rng, [6, 24, 32, 20, 12], [False, True, False, True], 3, 29, 34, 1)
    # second call, smaller: the buffer still holds the first call's tensors
    _run_both(torch, oracle, rng, [5, 16, 9], [True, False], 1, 12, 11, None)
    # and the first size again after the small one
    _run_both(torch, oracle, rng, [6, 24, 32, 20, 12], [False, True, False, True], 2, 29, 34, 3)


def test_static_buffer_entry_point_rejects_what_does_not_fit():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    rng = np.random.default_rng(778)
    specs = _layers(rng, [8, 64, 64])
    Ls = [B.Layer(d["w"], d["ids"], d["mask"], d["lib"]) for d in specs]
    n, h, w = 8, 160, 160                                # 8 x 64 x 160 x 160 floats = 50 MiB between the layers
    st = B.Stack([(L, None, True, False) for L in Ls], n, h, w)
    x = torch.zeros((n, 8, h, w), device="cuda")
    out = torch.empty(st.output_shape(), device="cuda")
    with pytest.raises(B.PatdnnError) as e:
        st.run_static(x, out)
    assert e.value.status == B.PATDNN_EUNSUPPORTED and "holds" in str(e.value)
    st.run(x, out)                                       # the allocating entry point still takes it
    torch.cuda.synchronize()
    st.close()
    for L in Ls:
        L.close()
