"""Each deliberate mistake planted in a copy of the oracle's source (CPU only) must be noticed by at least one pin
of tests/test_oracle_pins.py, tests/test_oracle_backward_pins.py or tests/test_oracle_log_pins.py; the unmodified
oracle by none.  The mistakes live here, as textual replacements, so that the oracle's own source stays plain."""
import inspect

import pytest

from oracle import sig_oracle as orc
from tests import test_oracle_backward_pins as backward_pins
from tests import test_oracle_log_pins as log_pins
from tests import test_oracle_pins as pins

# number: (what goes wrong, text of sig_oracle.c, its replacement[, which of two occurrences (0-based): the anchor
# occurs exactly once otherwise])
MUTANTS = {
    1: ("exp divides by 2 instead of k",
        "cur[w * d + j] = prev[w] * z[j] / (double)k;", "cur[w * d + j] = prev[w] * z[j] / 2.0;"),
    2: ("A_k (x) B_0 dropped from the group product",
        "Ck[w] = B[off_k + w] + A[off_k + w];", "Ck[w] = B[off_k + w];"),
    3: ("the j = 1 cross term dropped from the group product",
        "for (int j = 1; j <= k - 1; ++j) {\n            const int m = k - j;\n            const double *Aj = A + level_offset(d, j);",
        "for (int j = 2; j <= k - 1; ++j) {\n            const int m = k - j;\n            const double *Aj = A + level_offset(d, j);",
        0),   # the first is sig_oracle_mul, the second the product without constant terms
    4: ("cross terms written transposed",
        "Ck[u * n_m + v] += Aj[u] * Bm[v];", "Ck[v * n_j + u] += Aj[u] * Bm[v];", 0),
    5: ("increment sign flipped", "z[c] = hi - lo;", "z[c] = lo - hi;"),
    6: ("basepoint ignored", "z[c] = hi - lo;", "z[c] = (basepoint && s == 0) ? 0.0 : hi - lo;"),
    7: ("stream mode writes only the last prefix",
        "if (stream) memcpy(out + s * S, cur, sizeof(double) * (size_t)S);",
        "if (stream && s + 1 == n_inc) memcpy(out + s * S, cur, sizeof(double) * (size_t)S);\n"
        "        else if (stream) memset(out + s * S, 0, sizeof(double) * (size_t)S);"),
    8: ("level 3 stored one scalar too early",
        "for (int j = 1; j < k; ++j) off += ipow64(d, j);\n    return off;",
        "for (int j = 1; j < k; ++j) off += ipow64(d, j);\n    if (k == 3) off -= 1;\n    return off;"),
    9: ("gradient: the A_0 (x) B_k term of the product forgotten",
        "            gB[off_k + w] += gk[w];\n            gA[off_k + w] += gk[w];", "            gA[off_k + w] += gk[w];"),
    10: ("gradient: the 1/k of the exponential recurrence forgotten",
         "const double div = (double)k;", "const double div = 1.0;"),
    11: ("gradient: stream-mode output gradients shifted by one entry",
         "const double *g = gout + s * S;", "const double *g = gout + (s > 0 ? s - 1 : s) * S;"),
    12: ("gradient: wrong sign at the lower end point of an increment",
         "gx[s * d + c] -= gz[c];", "gx[s * d + c] += gz[c];"),
    13: ("logarithm: every term after the first subtracted",
         "const double sign = (m % 2 == 0) ? -1.0 : 1.0;\n        const double div = (double)m;\n        for (int64_t i = 0; i < S; ++i) out[i] +=",
         "const double sign = -1.0;\n        const double div = (double)m;\n        for (int64_t i = 0; i < S; ++i) out[i] +="),
    14: ("logarithm: the cube divided by 2 instead of 3",
         "const double div = (double)m;\n        for (int64_t i = 0; i < S; ++i) out[i] +=",
         "const double div = (double)(m == 3 ? 2 : m);\n        for (int64_t i = 0; i < S; ++i) out[i] +="),
    15: ("logarithm gradient: cotangent of a product read with the word split the other way round, for the first "
         "factor only (for both factors at once that would be the mirrored, equally valid, chain rule)",
         "gA[off_j + u] += g * B[off_m + v];", "gA[off_j + u] += gk[v * n_j + u] * B[off_m + v];",
         1),   # the second occurrence: the adjoint of the product without constant terms
    16: ("logarithm gradient: the 1/m of the series left out",
         "const double div = (double)m;\n        for (int64_t i = 0; i < S; ++i) g_pow[i] +=",
         "const double div = 1.0;\n        for (int64_t i = 0; i < S; ++i) g_pow[i] +="),
}


def mutated_source(number):
    _, old, new, *which = MUTANTS[number]
    text = orc.source_text()
    assert text.count(old) == (2 if which else 1), f"mutant {number}: its anchor moved in sig_oracle.c"
    at = text.index(old) if not which or which[0] == 0 else text.index(old, text.index(old) + 1)
    return text[:at] + new + text[at + len(old):]


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
    with orc.use_source(mutated_source(number), str(tmp_path), tag=f"mutant{number}"):
        failed = _failing_pins()
    assert failed, f"no pin notices: {MUTANTS[number][0]}"
