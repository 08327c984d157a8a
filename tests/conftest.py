import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

GOLDEN = os.path.join(ROOT, "tests", "golden")


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def golden():
    from klay_synth import parse_text_circuit

    def load(name):
        with open(os.path.join(GOLDEN, name)) as f:
            return parse_text_circuit(f.read())
    return load


def pytest_terminal_summary(terminalreporter):
    try:
        from tests import gpu_util
    except Exception:
        return
    if gpu_util.WORST_PLAIN_RATIO[0] > 0:
        terminalreporter.write_line("gradients under random dout: worst error / (1e-4 max(1, |ref|)) = %.3g "
                                    "(the cancellation-aware bound is what those tests assert)" % gpu_util.WORST_PLAIN_RATIO[0])
