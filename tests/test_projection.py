"""The library's projection operators (natural-pattern mining, projection onto the pattern
and connectivity constraints; paper section 4.1 / 4.2) against the oracle's, bit for bit:
integer outputs exactly, projected weights as fp32 bits.  Host code only."""

import numpy as np
import pytest

from oracle import projection as proj
from paper_2001_00138_amd import binding as B
from paper_2001_00138_amd import workloads as wl


def _weights(rng, c_out, c_in, ties):
    w = rng.standard_normal((c_out, c_in, 3, 3)).astype(np.float32)
    if ties:
        w = np.round(w * 2) / np.float32(2)        # few distinct magnitudes: every tie rule is exercised
    return w.astype(np.float32)


@pytest.mark.parametrize("c_out,c_in,ties,seed", [(6, 7, False, 1), (9, 5, True, 2), (16, 16, True, 3), (1, 1, False, 4)])
def test_projections_equal_the_oracle(c_out, c_in, ties, seed):
    rng = np.random.default_rng(seed)
    w = _weights(rng, c_out, c_in, ties)
    for k in (1, 6, 8, 56, 70):
        want = proj.mine_pattern_set(w, k)
        got = B.patdnn_mine_patterns(w, k)
        assert got.tolist() == want.tolist()
    lib = B.patdnn_mine_patterns(w, 8)
    ids, z = B.patdnn_project_patterns(w, lib)
    ids_o, z_o = proj.project_patterns(w, lib)
    np.testing.assert_array_equal(ids, ids_o)
    assert z.view(np.uint32).tolist() == z_o.view(np.uint32).tolist()
    for alpha in (0, 1, c_out * c_in // 3, c_out * c_in, c_out * c_in + 5):
        np.testing.assert_array_equal(B.patdnn_project_connectivity(z, alpha), proj.project_connectivity(z_o, alpha))


def test_projected_layer_satisfies_strict_encoding():
    """mine -> project -> encode with PATDNN_STRICT: the projected tensor obeys both
    constraints of section 4.2 exactly, and decodes back to itself."""
    rng = np.random.default_rng(9)
    w = _weights(rng, 24, 20, False)
    lib = B.patdnn_mine_patterns(w, 8)
    assert len(lib) == 8
    ids, z = B.patdnn_project_patterns(w, lib)
    alpha = wl.round_half_even(24 * 20 / 3.6)
    mask = B.patdnn_project_connectivity(z, alpha)
    assert int(mask.sum()) == alpha
    z = z * mask[:, :, None, None].astype(np.float32)
    L = B.Layer(z, ids, mask, lib, strict=True, host_only=True)
    w2, ids2, mask2 = L.decode()
    assert w2.view(np.uint32).tolist() == (z + np.float32(0)).view(np.uint32).tolist()
    np.testing.assert_array_equal(mask2, mask)
    np.testing.assert_array_equal(ids2, ids * mask)
    L.close()


def test_projection_argument_checks():
    w = np.zeros((2, 2, 3, 3), np.float32)
    with pytest.raises(B.PatdnnError) as e:
        B.patdnn_project_patterns(w, np.array([0], np.uint16))
    assert e.value.status == B.PATDNN_EPATTERN
    with pytest.raises(B.PatdnnError) as e:
        B.patdnn_project_connectivity(w, -1)
    assert e.value.status == B.PATDNN_EINVAL
