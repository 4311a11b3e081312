"""Each deliberate mistake that can be planted in the oracle (`-DSIG_ORACLE_MUTANT=n`, CPU only)
must be noticed by at least one pin of tests/test_oracle_pins.py or tests/test_oracle_backward_pins.py; the unmodified oracle by none."""
import inspect

import pytest

from oracle import sig_oracle as orc
from tests import test_oracle_backward_pins as backward_pins
from tests import test_oracle_log_pins as log_pins
from tests import test_oracle_pins as pins

MUTANTS = {
    1: "exp divides by 2 instead of k",
    2: "A_k (x) B_0 dropped from the group product",
    3: "the j = 1 cross term dropped from the group product",
    4: "cross terms written transposed",
    5: "increment sign flipped",
    6: "basepoint ignored",
    7: "stream mode writes only the last prefix",
    8: "level 3 stored one scalar too early",
    9: "gradient: the A_0 (x) B_k term of the product forgotten",
    10: "gradient: the 1/k of the exponential recurrence forgotten",
    11: "gradient: stream-mode output gradients shifted by one entry",
    12: "gradient: wrong sign at the lower end point of an increment",
    13: "logarithm: every term after the first subtracted",
    14: "logarithm: the cube divided by 2 instead of 3",
    15: "logarithm gradient: cotangent of a product read with the word split the other way round, for the first factor only",
    16: "logarithm gradient: the 1/m of the series left out",
}


def _pin_calls():
    """(name, callable) for every pin, with its parametrisations expanded."""
    calls = []
    members = (inspect.getmembers(pins, inspect.isfunction) + inspect.getmembers(backward_pins, inspect.isfunction) +
               [m for m in inspect.getmembers(log_pins, inspect.isfunction) if m[1].__module__ == log_pins.__name__])
    for name, fn in members:
        if not name.startswith("test_"):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, fn, {}))
            continue
        assert len(marks) == 1, name
        argnames, values = marks[0].args
        argnames = [a.strip() for a in argnames.split(",")]
        for v in values:
            v = v if isinstance(v, (tuple, list)) else (v,)
            calls.append((f"{name}[{v}]", fn, dict(zip(argnames, v))))
    return calls


def _failing_pins():
    failed = []
    for name, fn, kwargs in _pin_calls():
        try:
            fn(**kwargs)
        except Exception:  # an assertion, or an exception the pin does not expect
            failed.append(name)
    return failed


def test_the_unmodified_oracle_passes_every_pin():
    assert _failing_pins() == []


@pytest.mark.parametrize("number", sorted(MUTANTS), ids=lambda n: f"mutant{n}")
def test_every_planted_mistake_is_caught(number, tmp_path):
    with orc.use_mutant(number, str(tmp_path)):
        failed = _failing_pins()
    assert failed, f"no pin notices: {MUTANTS[number]}"
