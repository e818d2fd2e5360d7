"""Host logic of the library without a GPU: qrm_key_threshold against the exact oracle."""
from fractions import Fraction

import pytest

from oracle import keycheck


@pytest.fixture(scope="module")
def binding():
    from paper_2509_02447_amd import binding as b
    b.load_library()
    return b


def test_threshold_equals_the_oracle_including_exact_ties(binding):
    for K in list(range(1, 70, 2)) + [96, 128, 255]:
        rates = [0.0, 1e-300, 1e-12, 1e-9, 1e-6, 1e-4, 1e-2, 0.3, 0.5, 0.75, 1.0, 2.0,
                 2.0 ** -K, 2.0 ** -K * (1 + K)]          # the last two are tails hit exactly
        for fpr in rates:
            assert binding.qrm_key_threshold(K, fpr) == keycheck.key_threshold(K, Fraction(fpr)), (K, fpr)


def test_threshold_values_and_errors(binding):
    assert binding.qrm_key_threshold(48, 1e-6) == 41
    assert binding.qrm_key_threshold(32, 1e-6) == 30
    assert binding.qrm_key_threshold(64, 1e-6) == keycheck.key_threshold(64, Fraction(1e-6))
    assert binding.qrm_key_threshold(0, 0.1) == -1
    assert binding.qrm_key_threshold(2041, 0.1) == -1
    assert binding.qrm_key_threshold(8, -1e-3) == -1
    assert binding.qrm_key_threshold(8, float("nan")) == -1
    assert binding.qrm_key_threshold(2040, 1e-6) > 1020   # large sizes work (exact arithmetic)
