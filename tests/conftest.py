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
    from oracle import lot_oracle
    lot_oracle.build()
    return lot_oracle


@pytest.fixture
def knobs():
    """The library's testing aids (lot_debug_set), restored to their defaults afterwards."""
    from paper_2509_23436_amd import lot
    yield lot
    for k in (lot.KNOB_SPIN_LIMIT, lot.KNOB_RESHIFT_BITS, lot.KNOB_BWD_ASSEMBLE_BY_ITERATION,
              lot.KNOB_BWD_SWEEP_LAUNCHES, lot.KNOB_FWD_STREAMING, lot.KNOB_FWD_DRIFT_LIMIT,
              lot.KNOB_GROUPED_ONE_LAUNCH_TILES, lot.KNOB_BWD_SWEEP_RECOMPUTE):
        lot.lot_debug_set(k, -1)
