"""CPU tests: the oracle against what the paper prints, closed forms, numpy routines and brute force."""
import pytest

import oracle_checks as oc


@pytest.mark.parametrize("check", oc.ALL_CHECKS + [oc.check_errors], ids=lambda f: f.__name__)
def test_oracle_pin(orc, check):
    check(orc)
