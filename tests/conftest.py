import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu on the GPU box)")


@pytest.fixture(scope="session")
def oracle():
    from oracle import sla_oracle
    sla_oracle.lib()
    return sla_oracle


@pytest.fixture
def say(capsys):
    """Progress lines of the long tests: printed past pytest's capture, so that a run that is
    merely busy on the CPU (the oracle at full size takes minutes) is seen to be alive."""
    def _say(msg):
        with capsys.disabled():
            print(f"\n[{msg}]", end="", flush=True)
    return _say


@pytest.fixture(params=[False, True], ids=["four_wave_kernels", "eight_wave_kernels"])
def wide_tiles(request):
    """Both kernel choices for query blocks of an even number of tiles: two four-wave workgroups
    per pair of tiles (the default) and one eight-wave workgroup that loads K_j, V_j once."""
    from paper_2509_24006_amd import binding as sla
    sla.sla_wide_query_tiles(request.param)
    yield request.param
    sla.sla_wide_query_tiles(False)

