"""The CPU oracle against what the paper and the mathematics fix (no GPU, no oracle-vs-oracle)."""
import pytest

import oracle.gsi_oracle as O
from conftest import read_golden
from oracle_pins import FP8_PINS, PINS, pin_fp8_code_values, pin_paper_closed_forms, pin_paper_speedups


@pytest.mark.parametrize("pin", PINS + FP8_PINS, ids=lambda p: p.__name__)
def test_pin(pin):
    pin(O)


def test_paper_speedup_tables():
    pin_paper_speedups(O, read_golden("paper_speedup_tables.txt"))


def test_paper_closed_forms():
    pin_paper_closed_forms(O, read_golden("paper_closed_forms.txt"))


def test_fp8_code_values():
    pin_fp8_code_values(O, read_golden("fp8_e4m3_values.txt"))
