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
    """The CPU oracle.  With BTC_ORACLE_SOURCE_UNDER_TEST set (tests/test_oracle_mutants.py does that in a
    child pytest), a second copy of the oracle's Python front end is bound to a build of THAT source file
    instead, so the pins can be run against a deliberately broken oracle without touching the real one."""
    alt = os.environ.get("BTC_ORACLE_SOURCE_UNDER_TEST")
    if alt:
        import importlib.util
        spec = importlib.util.spec_from_file_location("oracle_under_test", os.path.join(ROOT, "oracle", "__init__.py"))
        mod = importlib.util.module_from_spec(spec)
        spec.loader.exec_module(mod)
        mod._SRC = alt
        mod._LIB = os.path.splitext(alt)[0] + ".so"
        mod.build(force=True)
        return mod
    import oracle as _oracle
    _oracle.build()
    return _oracle
