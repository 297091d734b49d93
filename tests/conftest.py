import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


class _Options:
    """Sets the library's process-wide switches (sd2_set_option) for one test and puts the defaults back afterwards."""

    def __init__(self):
        import paper_2504_08838_amd as sd2
        self.sd2 = sd2
        self.names = {"forward_multi": sd2.OPT_FORWARD_MULTI, "linear_partials": sd2.OPT_LINEAR_PARTIALS,
                      "spin_limit": sd2.OPT_SPIN_LIMIT, "mega_timing": sd2.OPT_MEGA_TIMING, "fixed_bits": sd2.OPT_FIXED_BITS}
        self.defaults = {"forward_multi": 0, "linear_partials": 0, "spin_limit": -1, "mega_timing": 0, "fixed_bits": 17}

    def set(self, name, value):
        self.sd2.set_option(self.names[name], value)

    def reset(self):
        for name, value in self.defaults.items():
            self.set(name, value)


@pytest.fixture
def sd2_options():
    o = _Options()
    o.reset()
    yield o
    o.reset()
