"""The CPU oracle against what the paper and the mathematics fix (no GPU needed)."""
import pytest

import oracle.hcache_oracle as oracle
import oracle_pins as pins


@pytest.mark.parametrize("check", pins.ALL_CHECKS, ids=lambda c: c.__name__)
def test_pin(check):
    check(oracle)


def test_lossless_interleaved_rope():
    pins.check_restore_equals_prefill(oracle, rope_style=1)
