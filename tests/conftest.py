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
    from oracle import disco_oracle
    disco_oracle.lib()      # compiles with gcc when the shared object is missing or stale
    return disco_oracle


def load_build_module():
    """The build script, loaded by path so that it works before the package can be imported."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("disco_build", os.path.join(ROOT, "paper_2502_11417_amd", "build.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


@pytest.fixture(scope="session")
def B():
    """The binding of the HIP library (built first if no shared object is there)."""
    build = load_build_module()
    if not os.path.exists(build.LIB):
        build.build_library()
    from paper_2502_11417_amd import binding
    return binding
