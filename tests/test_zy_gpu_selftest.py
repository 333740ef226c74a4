"""The device self-test behind the threaded-dispatch variants.  A device that fails it is
not an error of the library (the variants are then refused), so a failure is reported as
a skip that carries the reason."""

import pytest

from paper_2001_00138_amd import binding as B

pytestmark = pytest.mark.gpu


def test_scalar_relative_moves_behave_as_assumed():
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    try:
        B.patdnn_selftest()
    except B.PatdnnError as e:
        assert e.status == B.PATDNN_EUNSUPPORTED
        pytest.skip(f"threaded variants are off on this device: {e}")
    B.patdnn_selftest()          # the remembered result
