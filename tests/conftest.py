import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


def pytest_collection_modifyitems(config, items):
    """A test module may define ``combination_applies(test_name, params) -> bool``.  Parameter combinations it turns down
    (a model index the config does not have, a kernel variant a test is not meant for) are deselected at collection:
    they would only ever report "skipped", and a skip is kept for cases that are switched off for a stated reason."""
    kept, dropped = [], []
    for item in items:
        rule = getattr(item.module, "combination_applies", None)
        callspec = getattr(item, "callspec", None)
        if rule is not None and callspec is not None and not rule(item.originalname, callspec.params):
            dropped.append(item)
        else:
            kept.append(item)
    if dropped:
        config.hook.pytest_deselected(items=dropped)
        items[:] = kept


@pytest.fixture(scope="session")
def golden_dir():
    return os.path.join(ROOT, "tests", "golden")
