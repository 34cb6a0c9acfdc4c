import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


import pytest


class _Knobs:
    """Tuning knobs of the library (glowmi_tuning_set): force a tile variant or lower a kernel's size
    threshold so that a small test shape reaches it.  Results never depend on them."""

    def set(self, name, value):
        import paper_1805_00907_amd as glowmi
        glowmi.tuning_set(name, int(value))


@pytest.fixture
def knobs():
    import paper_1805_00907_amd as glowmi
    glowmi.tuning_reset()
    yield _Knobs()
    glowmi.tuning_reset()
