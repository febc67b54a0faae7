"""Host-side check of the stream allocator (no GPU needed): the tensors it
returns start at the requested offset past a 1 KiB boundary and are ordinary
contiguous tensors otherwise."""
import pytest
import torch

from paper_2601_05732_amd.layer import PHASE_G_X, PHASE_G_XOUT, PHASE_X, empty_stream, place_stream


@pytest.mark.parametrize("phase", [0, 16, 256, 512, 1008])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_empty_stream_phase_and_shape(phase, dtype):
    t = empty_stream((7, 3, 64), dtype, "cpu", phase)
    assert t.data_ptr() % 1024 == phase
    assert t.shape == (7, 3, 64) and t.dtype == dtype and t.is_contiguous()
    t.fill_(1.0)                      # the whole view is writable memory
    assert float(t.sum()) == 7 * 3 * 64


def test_place_stream_copies():
    x = torch.randn(5, 2, 32)
    y = place_stream(x, 512)
    assert torch.equal(x, y) and y.data_ptr() % 1024 == 512 and y.data_ptr() != x.data_ptr()


def test_roles_differ():
    assert len({PHASE_X, PHASE_G_XOUT, PHASE_G_X}) == 3
    assert all(p % 256 == 0 and 0 <= p < 1024 for p in (PHASE_X, PHASE_G_XOUT, PHASE_G_X))


@pytest.mark.parametrize("phase", [-16, 8, 1024])
def test_bad_phase(phase):
    with pytest.raises(ValueError):
        empty_stream((4,), torch.float32, "cpu", phase)
