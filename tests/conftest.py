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
    from oracle import cpu_oracle
    cpu_oracle.build()
    return cpu_oracle


@pytest.fixture(autouse=True)
def _tuning_overrides_follow_the_environment():
    """The library reads its FG_FORCE_* tuning variables once, at load.  Tests that change them go
    through fg_reload_tuning(); after each test (monkeypatch has restored the environment by then:
    this fixture is set up first, so it is torn down last) the library reads them once more."""
    yield
    from paper_2009_12263_amd import binding
    if binding._lib is not None:
        binding.fg_reload_tuning()
