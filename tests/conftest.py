import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


# tests/test_oracle_pin_sensitivity.py runs the pins in a child process against a copy of the checker with one
# deliberate mistake; the copy's path arrives here and takes the checker's place before any test imports it.
_ALT_CHECKER = os.environ.get("PCM_CHECKER_SOURCE")
if _ALT_CHECKER:
    import importlib.util

    import oracle

    _spec = importlib.util.spec_from_file_location("oracle.pcm_oracle", _ALT_CHECKER)
    _mod = importlib.util.module_from_spec(_spec)
    _spec.loader.exec_module(_mod)
    sys.modules["oracle.pcm_oracle"] = _mod
    oracle.pcm_oracle = _mod


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
