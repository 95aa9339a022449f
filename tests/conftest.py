import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


import pytest


@pytest.fixture
def knobs():
    """Developer options of the library (launch geometry only), restored to their defaults after
    the test: knobs.set("slab", 0) etc."""
    from paper_2506_04165_amd import binding

    class Knobs:
        def __init__(self):
            self.touched = set()

        def set(self, name, value):
            self.touched.add(name)
            binding.set_option(name, value)

    k = Knobs()
    yield k
    for name in k.touched:
        binding.set_option(name, -1)
