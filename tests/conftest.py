import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_addoption(parser):
    parser.addoption("--dump-case", default=None, metavar="DIR",
                     help="write the inputs of the last decode call of every failing test to DIR (.bin + .json)")
    parser.addoption("--load-case", default=None, metavar="PREFIX",
                     help="case written by --dump-case, replayed by tests/test_replay_case.py")


@pytest.hookimpl(hookwrapper=True)
def pytest_runtest_makereport(item, call):
    outcome = yield
    rep = outcome.get_result()
    folder = item.config.getoption("--dump-case")
    if folder and rep.when == "call" and rep.failed:
        import helpers
        if helpers.last_case is not None:
            name = "".join(c if c.isalnum() or c in "-_." else "_" for c in item.nodeid.split("::", 1)[-1])
            helpers.dump_case(os.path.join(folder, name), *helpers.last_case)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (run with -m gpu)")


@pytest.fixture(scope="session")
def oracle():
    import oracle as o
    o.build()
    return o
