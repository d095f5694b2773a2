import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """GPU tests must fail loudly, not skip, when selected on a box without a GPU
    or without the built library; they are simply deselected by -m 'not gpu'."""
    return


@pytest.fixture(params=["groups-auto", "groups-32"])
def both_groupings(request):
    """Runs a test twice: with the library's own choice of query heads per attention workgroup (small launches, as the
    tests run them, get a group per KV head) and with up to 32 heads per workgroup, the form large launches take."""
    from paper_2512_06727_amd import harness
    old = harness.default_group_slots
    harness.default_group_slots = 32 if request.param == "groups-32" else 0
    yield request.param
    harness.default_group_slots = old
