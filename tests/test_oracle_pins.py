"""CPU-only: the oracle against its pins (closed forms, special inputs, invariants, library
routines, a hand-worked example).  See tests/pins.py for what each pin fixes."""
import pytest

import pins


@pytest.mark.parametrize("pin", pins.ALL_PINS, ids=lambda f: f.__name__)
def test_pin(orc, pin):
    out = pin(orc)
    if isinstance(out, dict):          # pin_sort_comparator reports EWMA-vs-sort overlap
        for ratio, (la, achieved, overlap) in out.items():
            print(f"table ratio {ratio:.1f} la {la:+.1f}: achieved sparsity {achieved:.3f}, "
                  f"overlap with the k smallest scores {overlap:.3f}")
