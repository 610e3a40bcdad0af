import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as _oracle
    _oracle.build()
    return _oracle


@pytest.fixture
def tune():
    """Setter for the library's tuning knobs (snn_set_tuning); every knob is back to its automatic value after the test.
    tune("MFMA_TILE", "4,2") / tune("MFMA_KS", 2) / tune("SUBBIT_MFMA", "0")."""
    from paper_2110_09195_amd import binding as B
    touched = []

    def set_knob(name, value):
        knob = getattr(B, "SNN_TUNE_" + name)
        if isinstance(value, str) and "," in value:
            a, b = value.split(",")
            value = 10 * int(a) + int(b)
        B.snn_set_tuning(knob, int(value))
        touched.append(knob)

    yield set_knob
    for knob in touched:
        B.snn_set_tuning(knob, B.SNN_TUNE_AUTO)
