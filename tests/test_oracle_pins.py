"""The CPU oracle against what the paper and the mathematics fix (no GPU)."""
import pytest

from oracle import probsparse_oracle as O
from tests import oracle_pins


@pytest.mark.parametrize("check", oracle_pins.ALL_CHECKS, ids=lambda f: f.__name__)
def test_pin(check):
    check(O)
