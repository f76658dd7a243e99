import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs through the HIP library)")


def pytest_collection_modifyitems(config, items):
    import torch
    if torch.cuda.is_available():
        return
    skip = pytest.mark.skip(reason="no GPU in this process")
    for item in items:
        if "gpu" in item.keywords:
            item.add_marker(skip)


@pytest.fixture()
def wrong_oracle(tmp_path):
    """plant(find, replace): puts a copy of the oracle with one planted mistake behind its
    Python front end until the test ends.  The mistake is always planted on the CPU side,
    in the oracle; the HIP library is untouched."""
    from oracle import e3_oracle as o
    from tests import test_oracle_mutants as mut
    real = o.lib()
    source = open(mut.SRC).read()

    def plant(find, replace):
        assert source.count(find) == 1
        o._lib = mut._build(tmp_path, "wrong", source.replace(find, replace))
    yield plant
    o._lib = real
