"""The CPU oracle against closed forms, exact arithmetic and library routines (no GPU)."""
import pytest

import pins


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(pin):
    pin()


@pytest.mark.parametrize("clip,W,kind", [(False, 1, "f32"), (True, 4, "f32"), (False, 5, "bf16")])
def test_whole_step_variants(clip, W, kind):
    pins.pin_whole_step_vs_torch(clip=clip, W=W, steps=4, grad_kind=kind)
