import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session", autouse=True)
def _oracle_built():
    from oracle import lola_oracle
    lola_oracle.build()


def pytest_terminal_summary(terminalreporter):
    """After a GPU run: the largest error each compared quantity reached, beside its bounds."""
    parity = sys.modules.get("parity")
    if parity is None or not getattr(parity, "WORST", None):
        return
    terminalreporter.write_line("largest relative errors against the oracle in this session "
                                "(contract bf16 2e-3 / f32 1e-5; regression bounds bf16 1e-4 / f32 5e-6):")
    for (dtype, what), err in sorted(parity.WORST.items()):
        terminalreporter.write_line(f"  {dtype:5s} {what:28s} {err:.3e}")
