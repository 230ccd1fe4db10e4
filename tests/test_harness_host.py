"""Host checks of the test harness itself: the guard-band checker must notice every kind of stray
write it is there to catch (planted here on CPU tensors) and accept writes to the payload."""
import pytest
import torch

from tests.gpu_harness import GUARD, Guarded


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.uint8, torch.int32])
def test_guard_checker_catches_planted_writes(dtype):
    g = Guarded(5, 24, dtype, pad_cols=8, device="cpu")
    assert g.intact_outside_payload()
    g.t.fill_(3)                                     # the payload may hold anything
    assert g.intact_outside_payload()
    for where in (GUARD - 1, GUARD + g.nbytes, 0, g.raw.numel() - 1,          # around the payload
                  GUARD + 24 * g.es, GUARD + (g.pitch * 3 - 1) * g.es + g.es - 1):   # padding columns of rows 0 and 2
        h = Guarded(5, 24, dtype, pad_cols=8, device="cpu")
        h.t.fill_(3)
        h.raw[where] = 0
        assert not h.intact_outside_payload(), where
    v = Guarded(1, 7, dtype, device="cpu")
    v.vec().fill_(1)
    assert v.intact_outside_payload() and v.vec().shape == (7,)
